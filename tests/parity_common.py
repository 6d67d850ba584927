"""Shared pieces of the GPU parity tests: the bar, the configs of both sides, the comparisons.

Both sides receive the same seeded inputs.  The bar, per step:
  * block scales Delta_m, Delta_v and bases alpha: bit-exact;
  * 1st-moment code words: bit-exact;
  * 2nd-moment codes: equal, except +-1 flips where the oracle's own binary64 margin to the
    rounding boundary is below FLIP_MARGIN = 1e-5 code units (the two sides use different log2
    routines); at most FLIP_RATE = 1e-5 of the elements.  Measured over 1.2e8 compared codes:
    one flip in 3e6 codes, largest margin 1.6e-6.
    In a block whose base alpha lies within a few thousand ulps of 1 (a nearly constant block)
    log_alpha amplifies the last bit of v^/Delta itself: one unit in the last place of the ratio
    moves the rounded quantity by 2^-23 / |ln alpha| code units, and the two sides form the
    ratio differently (a division on the CPU, a product with the correctly rounded reciprocal
    on the GPU, up to one unit apart).  There the margin a flip may have grows by
    FLIP_ILL * 2^-23 / |log2 alpha| (flip_allowance; measured: below 0.84 of that unit), and
    flips whose allowance exceeds twice FLIP_MARGIN are not counted against the rate;
  * parameters: |dp| <= 1e-6 |p| + 2e-6 lr + 4e-7 |update| after one step from equal states, and
    <= 1e-5 |p| + 1e-5 lr after ten free-running steps (a parameter can be arbitrarily close
    to zero while every step moves it by O(lr); the kernel's sqrt and reciprocal are good to
    1 ulp, so one step is off by ~1e-7 of its own size plus the rounding of p).
"""
import os

import numpy as np

TILE = 5120          # elements one wavefront of the step kernel owns
FLIP_MARGIN = 1e-5
FLIP_ILL = 2.0
FLIP_RATE = 1e-5

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# every 2nd-moment code on which the two sides disagreed, over the whole session:
# (oracle margin in code units, |log2 alpha| of the block, counted against the rate or not)
FLIP_LOG = []
CODES_COMPARED = [0]
NOTES = []           # per-config lines (flip counts, 10-step parameter error), printed at the end


def note(line):
    NOTES.append(line)
    print(line, flush=True)
    progress(line)


_progress_started = []


def progress(line):
    """A line into parity_progress.txt of the run's output folder: long tests show that they are alive."""
    out = os.path.join(ROOT, "gpurun_out")
    os.makedirs(out, exist_ok=True)
    mode = "a" if _progress_started else "w"
    _progress_started.append(1)
    with open(os.path.join(out, "parity_progress.txt"), mode) as f:
        f.write(line + "\n")


def write_flip_report():
    out = os.path.join(ROOT, "gpurun_out")
    os.makedirs(out, exist_ok=True)
    counted = [m for m, l, c in FLIP_LOG if c]
    with open(os.path.join(out, "flip_margins.txt"), "w") as f:
        f.write(f"# codes compared: {CODES_COMPARED[0]}, flips: {len(FLIP_LOG)}, of them in "
                f"well-conditioned blocks: {len(counted)} (largest margin {max(counted) if counted else 0:.3g})\n")
        for line in NOTES:
            f.write("# " + line + "\n")
        f.write("# margin  |log2 alpha|  margin*|log2 alpha|*2^23\n")
        for m, l, c in sorted(FLIP_LOG, key=lambda t: -t[0]):
            f.write(f"{m:.4g} {l:.4g} {m * l * 2 ** 23:.3g}\n")
    return len(counted), (max(counted) if counted else 0.0)


def flip_budget(codes):
    """Well-conditioned flips tolerated among `codes` compared codes of one case: the 1e-5 rate
    as a mean with room for its Poisson scatter (mean + 4 sqrt(mean)), but never less than one,
    and two from 1e4 codes on: every single flip has had its margin checked, and at the measured
    rate of 3e-7 ... 1e-6 per code a second flip in a case of 5e4 codes is a 1e-3 event, which
    over the few hundred cases of a session would fail a correct build every few runs.  The
    rate itself is asserted over all codes of the session by the last test."""
    mean = FLIP_RATE * codes
    return max(int(mean + 4.0 * np.sqrt(mean)), 2 if codes >= 10000 else 1)


def flip_allowance(alpha):
    """Largest oracle margin (code units) at which a +-1 disagreement of a 2nd-moment code is
    legitimate, per element, from the element's block base."""
    l2a = np.abs(np.log2(np.minimum(alpha.astype(np.float64), 1.0 - 2.0 ** -25)))
    return FLIP_MARGIN + FLIP_ILL * 2.0 ** -23 / l2a


def check_flips(margin, alpha, d, where):
    """Judge disagreeing 2nd-moment codes: `margin` the oracle's margins, `alpha` the bases of
    their blocks, `d` the code differences.  Returns the number counted against the rate and
    the number in nearly constant blocks."""
    assert np.abs(d).max() == 1, f"2nd-moment code off by {np.abs(d).max()} at {where[np.argmax(np.abs(d))]}"
    allow = flip_allowance(alpha)
    over = margin - allow
    assert over.max() < 0, \
        f"2nd-moment flip away from a tie: margin {margin[np.argmax(over)]:.3g} at {where[np.argmax(over)]}"
    well = allow < 2 * FLIP_MARGIN
    l2a = np.abs(np.log2(np.minimum(alpha.astype(np.float64), 1.0 - 2.0 ** -25)))
    FLIP_LOG.extend(zip(margin.tolist(), l2a.tolist(), well.tolist()))
    return int(well.sum()), int((~well).sum())


def dev(x):
    import torch
    if x.dtype == np.uint32:
        return torch.from_numpy(x.view(np.int32)).cuda()
    if x.dtype == np.uint16:        # bf16 bit patterns
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(x).cuda()


def host_words(t):
    return t.cpu().numpy().view(np.uint32)


def make_cfgs(so, solo, bm, bv, B, bf16=False, stochastic=1, beta1=None, p=0.1, seed=42, off=0,
              lr=1e-3, wd=0.01, eps=1e-8, beta2=0.999, de=False, optimizer="adamw", grad_scale=None):
    beta1 = {2: 0.5, 3: 0.6, 4: 0.8}[bm] if beta1 is None else beta1
    oc = so.make_config(bits_m=bm, bits_v=bv, block_size=B, stochastic=stochastic, lr=lr, beta1=beta1,
                        beta2=beta2, eps=eps, weight_decay=wd, quantile_p=p, seed=seed, index_offset=off,
                        m_codebook=1 if de else 0,
                        optimizer={"adamw": so.ADAMW, "adam_l2": so.ADAM_L2, "adabelief": so.ADABELIEF}[optimizer],
                        grad_scale=1.0 if grad_scale is None else grad_scale)
    gc = solo.make_config(bits_m=bm, bits_v=bv, block_size=B, grad_dtype=1 if bf16 else 0, lr=lr,
                          beta1=beta1, beta2=beta2, eps=eps, weight_decay=wd, quantile_p=p,
                          flags=(1 if stochastic else 0) | (2 if de else 0) |
                          {"adamw": 0, "adam_l2": 8, "adabelief": 4}[optimizer], seed=seed, index_offset=off)
    return oc, gc


def bits_equal(a, b):
    return np.array_equal(a.view(np.uint32), b.view(np.uint32))


def compare_step(so, oc, n, want_p, want_st, margin, got, p_rtol, p_atol, tainted=None, p_before=None):
    """Compare one step's results on the host; returns the number of v-code flips counted against
    the rate.  `tainted` (bool per block, updated in place) marks blocks whose state already
    differs legitimately."""
    B = oc.block_size
    gp, gm, gms, gv, gvs, gva = got
    nblk = want_st.m_scale.size
    clean = np.ones(nblk, bool) if tainted is None else ~tainted
    eclean = np.repeat(clean, B)[:n]
    assert bits_equal(gms[clean], want_st.m_scale[clean]), "Delta_m differs"
    assert bits_equal(gvs[clean], want_st.v_scale[clean]), "Delta_v differs"
    assert bits_equal(gva[clean], want_st.v_base[clean]), "alpha differs"
    wm, wv = so.unpack(want_st.m_words, n, oc.bits_m), so.unpack(want_st.v_words, n, oc.bits_v)
    hm, hv = so.unpack(gm, n, oc.bits_m), so.unpack(gv, n, oc.bits_v)
    assert np.array_equal(hm[eclean], wm[eclean]), "1st-moment codes differ"
    if tainted is None:
        assert np.array_equal(gm, want_st.m_words), "1st-moment words differ (pad bits?)"
    diff = np.nonzero((hv != wv) & eclean)[0]
    n_flips = 0
    CODES_COMPARED[0] += int(eclean.sum())
    if diff.size:
        alpha = np.repeat(want_st.v_base, B)[:n]
        n_flips, ill = check_flips(margin[diff], alpha[diff], hv[diff].astype(int) - wv[diff].astype(int), diff)
        # in nearly constant blocks a flip has probability ~2 x allowance per element, which bounds their number
        allow = flip_allowance(alpha[eclean])
        assert ill <= 10 + 4 * float(allow[allow >= 2 * FLIP_MARGIN].clip(max=0.5).sum()), \
            "too many flips in nearly constant blocks"
        if tainted is not None:
            tainted[np.unique(diff // B)] = True
    elif tainted is None:
        assert np.array_equal(gv, want_st.v_words), "2nd-moment words differ (pad bits?)"
    err = np.abs(gp.astype(np.float64) - want_p)
    tol = p_rtol * np.abs(want_p) + p_atol
    if p_before is not None:
        # the binary32 update (hardware sqrt and reciprocal, 1 ulp each) is off by a few 1e-7 of its
        # own size; p_atol covers that for updates of O(10 lr), this term for the settings in which
        # an update is orders of magnitude larger (a vanishing v^ under an eps of 1e-12, say)
        tol = tol + 4e-7 * np.abs(want_p.astype(np.float64) - p_before)
    bad = (err > tol) & eclean
    assert not bad.any(), f"parameter error {err[bad].max():.3g} at {np.nonzero(bad)[0][0]}"
    return n_flips


class DeviceView:
    """The device buffers of one piece of work (a whole buffer, a tensor, or a slice of a large
    flat buffer that starts on a block and code-word boundary): parameters and the five state
    arrays as torch tensors (views are fine)."""

    def __init__(self, p, m_codes, m_scale, v_codes, v_scale, v_base):
        self.p, self.m_codes, self.m_scale = p, m_codes, m_scale
        self.v_codes, self.v_scale, self.v_base = v_codes, v_scale, v_base

    @staticmethod
    def of(p, state, a=0, n=None):
        """Elements [a, a + n) of a flat parameter buffer and its SoloState."""
        cfg = state.cfg
        n = state.n - a if n is None else n
        cm, cv, B = 32 // cfg.bits_m, 32 // cfg.bits_v, cfg.block_size
        assert a % B == 0 and a % cm == 0 and a % cv == 0
        wm, wv, nb = -(-n // cm), -(-n // cv), -(-n // B)
        return DeviceView(p[a:a + n], state.m_codes[a // cm:a // cm + wm], state.m_scale[a // B:a // B + nb],
                          state.v_codes[a // cv:a // cv + wv], state.v_scale[a // B:a // B + nb],
                          state.v_base[a // B:a // B + nb])

    def to_host_state(self, so, oc):
        st = so.State(int(self.p.numel()), oc)
        st.m_words[:] = host_words(self.m_codes); st.v_words[:] = host_words(self.v_codes)
        st.m_scale[:] = self.m_scale.cpu().numpy(); st.v_scale[:] = self.v_scale.cpu().numpy()
        st.v_base[:] = self.v_base.cpu().numpy()
        return st

    def load(self, p, st):
        self.p.copy_(dev(p))
        self.m_codes.copy_(dev(st.m_words)); self.v_codes.copy_(dev(st.v_words))
        self.m_scale.copy_(dev(st.m_scale)); self.v_scale.copy_(dev(st.v_scale)); self.v_base.copy_(dev(st.v_base))


def compare_on_device(so, oc, view, want_p, want_st, margin, p_rtol, p_atol, tainted=None, p_before=None,
                      label=""):
    """The comparison of compare_step for a large piece: the oracle's results are uploaded and
    compared on the device, word by word and element by element; only the words that differ come
    back to the host, where every differing code is judged against its margin.  `tainted`: a bool
    tensor per block on the device, updated in place (free-running runs).  Returns
    (flips counted against the rate, largest parameter error relative to its tolerance)."""
    import torch
    n = int(view.p.numel())
    B, bm, bv = oc.block_size, oc.bits_m, oc.bits_v
    cm, cv = 32 // bm, 32 // bv
    nblk = want_st.m_scale.size
    clean = torch.ones(nblk, dtype=torch.bool, device="cuda") if tainted is None else ~tainted

    def as_i32(t):
        return t.view(torch.int32)

    for name, g, w in (("Delta_m", view.m_scale, want_st.m_scale), ("Delta_v", view.v_scale, want_st.v_scale),
                       ("alpha", view.v_base, want_st.v_base)):
        bad = (as_i32(g) != dev(w.view(np.uint32))) & clean
        assert not bool(bad.any()), f"{label}: {name} differs in block {int(bad.nonzero()[0])}"

    def blocks_of_words(widx, c):
        first = (widx * c) // B
        last = torch.clamp((widx * c + (c - 1)), max=n - 1) // B
        return first, last

    mbad = (view.m_codes != dev(want_st.m_words)).nonzero().flatten()
    if mbad.numel():
        first, last = blocks_of_words(mbad, cm)
        # a differing word must lie in blocks that have diverged before (free-running runs only)
        ok = (~clean[first]) | (~clean[last])
        assert bool(ok.all()), f"{label}: 1st-moment word {int(mbad[~ok][0])} differs"

    vbad = (view.v_codes != dev(want_st.v_words)).nonzero().flatten()
    n_flips = 0
    CODES_COMPARED[0] += int(clean.sum()) * B
    if vbad.numel():
        widx = vbad.cpu().numpy()
        gw = view.v_codes[vbad].cpu().numpy().view(np.uint32)
        ww = want_st.v_words[widx]
        shifts = (bv * np.arange(cv)).astype(np.uint32)
        mask = np.uint32((1 << bv) - 1)
        gf = (gw[:, None] >> shifts[None, :]) & mask
        wf = (ww[:, None] >> shifts[None, :]) & mask
        elem = widx[:, None] * cv + np.arange(cv)[None, :]
        if bv * cv < 32:
            assert np.array_equal(gw >> np.uint32(bv * cv), ww >> np.uint32(bv * cv)), f"{label}: pad bits differ"
        differs = (gf != wf)
        assert not differs[elem >= n].any(), f"{label}: fields behind the last element differ"
        e = elem[differs]
        d = gf[differs].astype(int) - wf[differs].astype(int)
        clean_h = clean.cpu().numpy()
        live = clean_h[e // B]
        if live.any():
            e, d = e[live], d[live]
            alpha = want_st.v_base[e // B]
            n_flips, ill = check_flips(margin[e], alpha, d, e)
            # in nearly constant blocks a flip has probability ~2 x allowance per element
            allow_blk = flip_allowance(want_st.v_base)
            ill_blk = (allow_blk >= 2 * FLIP_MARGIN) & clean_h
            assert ill <= 10 + 4 * B * float(allow_blk[ill_blk].clip(max=0.5).sum()), \
                f"{label}: too many flips in nearly constant blocks"
            if tainted is not None:
                tainted[torch.from_numpy(np.unique(e // B)).cuda()] = True
                clean = ~tainted

    wp = dev(want_p).double()
    err = (view.p.double() - wp).abs()
    tol = p_rtol * wp.abs() + p_atol
    if p_before is not None:
        tol = tol + 4e-7 * (wp - dev(p_before).double()).abs()
    ratio = err / tol
    if n % B:
        pad = torch.zeros(nblk * B - n, dtype=ratio.dtype, device="cuda")
        ratio = torch.cat([ratio, pad])
    ratio = ratio.view(nblk, B) * clean[:, None]
    worst = float(ratio.max())
    assert worst <= 1.0, f"{label}: parameter error {worst:.3g} of its tolerance at element {int(ratio.argmax())}"
    return n_flips, worst
