"""Pins of the oracle's whole optimizer step (no GPU).

The step is checked against closed forms (constant and zero gradients), a
textbook AdamW in binary64 (the limit of wide codes), an independent brute-force
step written from the definitions, the swamping thresholds the paper prints,
and the degenerate blocks the method has.
"""
import math

import numpy as np
import pytest

from conftest import read_golden

BITS = (2, 3, 4)

# Signed dynamic-exponent level sets (App. A), written out: sign bit, one fraction cell per
# exponent step 10^-i represented by the mean of its boundaries on [0.1, 1], plus 0 and 1.
DE_LEVELS = {2: [-0.55, 0.0, 0.55, 1.0],
             3: [-0.775, -0.325, -0.055, 0.0, 0.055, 0.325, 0.775, 1.0],
             4: [-0.8875, -0.6625, -0.4375, -0.2125, -0.0775, -0.0325, -0.0055, 0.0,
                 0.0055, 0.0325, 0.0775, 0.2125, 0.4375, 0.6625, 0.8875, 1.0]}


def fresh_unpacked(so, n, cfg):
    nblk = -(-n // cfg.block_size)
    return (np.full(n, so.L_of(cfg.bits_m), np.uint16), np.zeros(nblk, np.float32),
            np.zeros(n, np.uint16), np.zeros(nblk, np.float32), np.ones(nblk, np.float32))


# -------------------------------------------------- brute force from definitions

def brute_step(so, p, g, mc, ms, vc, vs, va, step, cfg):
    """One step in binary64 from the plain definitions: explicit level tables, argmin,
    full sort for the quantile, np.power for the levels and the root.  xi is taken from
    the oracle's stream (random numbers are inputs of the method, not its arithmetic).
    Returns new params, codes, scales, bases and a per-element flag 'decision is clear'."""
    B, bm, bv = cfg.block_size, cfg.bits_m, cfg.bits_v
    L, K = 2 ** (bm - 1) - 1, 2 ** bv - 1
    n = p.size
    b1, b2 = float(np.float32(cfg.beta1)), float(np.float32(cfg.beta2))
    lr, wd, eps = (float(np.float32(x)) for x in (cfg.lr, cfg.weight_decay, cfg.eps))
    mlevels = np.array(DE_LEVELS[bm]) if cfg.m_codebook else np.array([k / L for k in range(-L, L + 1)])
    out_p = np.empty(n)
    out_mc, out_vc = np.empty(n, int), np.empty(n, int)
    clear = np.ones(n, bool)
    out_ms, out_vs, out_va = (np.empty(ms.size) for _ in range(3))
    for blk in range(ms.size):
        sl = slice(blk * B, min(n, (blk + 1) * B))
        nb = sl.stop - sl.start
        gg = g[sl].astype(np.float64) * float(np.float32(cfg.grad_scale))
        if cfg.optimizer == so.ADAM_L2:
            gg = gg + wd * p[sl]
        mt = mlevels[mc[sl]] * float(ms[blk])
        vt = np.power(float(va[blk]), vc[sl].astype(np.float64)) * float(vs[blk])
        mh = b1 * mt + (1 - b1) * gg
        if cfg.optimizer == so.ADABELIEF:
            vh = b2 * vt + (1 - b2) * (gg - mh) ** 2 + eps
        else:
            vh = b2 * vt + (1 - b2) * gg * gg
        bc1, bc2 = 1 - b1 ** step, 1 - b2 ** step
        keep = 1.0 if cfg.optimizer == so.ADAM_L2 else 1 - lr * wd
        out_p[sl] = p[sl] * keep - lr * (mh / bc1) / (np.sqrt(vh / bc2) + eps)
        dm, dv = np.max(np.abs(mh)), np.max(vh)
        out_ms[blk], out_vs[blk] = dm, dv
        if dm < 2.0 ** -100:
            out_ms[blk] = 0
            out_mc[sl] = L
        else:
            dist = np.abs((mh / dm)[:, None] - mlevels[None, :])
            out_mc[sl] = np.argmin(dist, axis=1)
            srt = np.sort(dist, axis=1)
            clear[sl] &= (srt[:, 1] - srt[:, 0]) > 2e-5 * np.maximum(srt[:, 0] + srt[:, 1], 1e-3)
        if dv < 2.0 ** -100:
            out_vs[blk], out_va[blk] = 0, 1
            out_vc[sl] = 0
            continue
        r = max(1, math.ceil(float(np.float32(cfg.quantile_p) * np.float32(nb))))   # product in binary32
        rho = max(np.sort(vh)[r - 1] / dv, 2.0 ** -64)
        alpha = rho ** (1.0 / K)
        out_va[blk] = alpha
        if alpha == 1.0:
            out_vc[sl] = 0
            continue
        xi = so.xi_array(cfg.seed, step, cfg.index_offset + sl.start, nb).astype(np.float64) \
            if cfg.stochastic else np.zeros(nb)
        with np.errstate(divide="ignore"):
            t = np.log(vh / dv) / math.log(alpha) + xi
        code = np.clip(np.rint(t), 0, K)
        code[vh == 0] = K
        out_vc[sl] = code
        tt = np.clip(t, -1, K + 1)
        clear[sl] &= np.abs(np.abs(tt - np.floor(tt)) - 0.5) > 2e-5
    return out_p, out_mc, out_ms, out_vc, out_vs, out_va, clear


@pytest.mark.parametrize("bm,bv,B", [(2, 2, 64), (2, 3, 128), (3, 3, 128), (4, 4, 128),
                                     (4, 2, 64), (3, 4, 64), (2, 4, 128), (4, 3, 128), (3, 2, 64),
                                     (4, 2, 2048), (2, 2, 2048)])       # 2048: the large block of Sec. 4.2
@pytest.mark.parametrize("codebook", (0, 1))
def test_step_against_brute_force_on_tiny_tensors(so, bm, bv, B, codebook):
    rng = np.random.default_rng(1000 + 16 * bm + bv)
    for n in ((B, 2 * B + 17, 256, 5) if B < 2048 else (B + 300,)):
        cfg = so.make_config(bits_m=bm, bits_v=bv, block_size=B, beta1=0.5 if bm == 2 else 0.8,
                             seed=9, index_offset=8 * 123456789, m_codebook=codebook)
        p = (rng.standard_normal(n) * 0.02).astype(np.float32)
        mc, ms, vc, vs, va = fresh_unpacked(so, n, cfg)
        unclear = 0
        for step in range(1, 7):
            g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
            if step == 4:
                g[: n // 2] = 0                                    # a run of zero gradients
            want = brute_step(so, p, g, mc.astype(int), ms, vc.astype(int), vs, va, step, cfg)
            so.step_unpacked(p, g, mc, ms, vc, vs, va, step, cfg)
            wp, wmc, wms, wvc, wvs, wva, clear = want
            assert np.allclose(p, wp, rtol=2e-6, atol=1e-9)
            assert np.allclose(ms, wms, rtol=1e-6) and np.allclose(vs, wvs, rtol=1e-6)
            assert np.allclose(va, wva, rtol=1e-6)
            assert np.array_equal(mc[clear], wmc[clear]) and np.array_equal(vc[clear], wvc[clear])
            assert np.all(np.abs(mc.astype(int) - wmc) <= 1) and np.all(np.abs(vc.astype(int) - wvc) <= 1)
            unclear += int(np.sum(~clear))
        assert unclear <= max(2, n // 50)


@pytest.mark.parametrize("optimizer", ("ADAM_L2", "ADABELIEF"))
@pytest.mark.parametrize("bm,bv,B,codebook", [(2, 3, 128, 0), (4, 2, 128, 1), (3, 3, 64, 0)])
def test_other_optimizers_against_brute_force(so, optimizer, bm, bv, B, codebook):
    """Adam with the decay inside the gradient and AdaBelief, with a gradient scale, against
    the same brute-force step (Sec. 4.2 applies the quantizers to AdaBelief unchanged)."""
    rng = np.random.default_rng(77 + bm + 8 * bv)
    n = 2 * B + 17
    cfg = so.make_config(bits_m=bm, bits_v=bv, block_size=B, beta1=0.5 if bm == 2 else 0.8, seed=5,
                         m_codebook=codebook, optimizer=getattr(so, optimizer), grad_scale=1 / 1024,
                         weight_decay=0.1, eps=1e-8 if optimizer == "ADAM_L2" else 1e-12)
    p = (rng.standard_normal(n) * 0.02).astype(np.float32)
    mc, ms, vc, vs, va = fresh_unpacked(so, n, cfg)
    unclear = 0
    for step in range(1, 7):
        g = (rng.standard_normal(n) * 1.024).astype(np.float32)
        want = brute_step(so, p, g, mc.astype(int), ms, vc.astype(int), vs, va, step, cfg)
        so.step_unpacked(p, g, mc, ms, vc, vs, va, step, cfg)
        wp, wmc, wms, wvc, wvs, wva, clear = want
        assert np.allclose(p, wp, rtol=2e-6, atol=1e-9)
        assert np.allclose(ms, wms, rtol=1e-6) and np.allclose(vs, wvs, rtol=1e-6)
        assert np.allclose(va, wva, rtol=1e-6)
        assert np.array_equal(mc[clear], wmc[clear]) and np.array_equal(vc[clear], wvc[clear])
        unclear += int(np.sum(~clear))
    assert unclear <= max(2, n // 50)


# --------------------------------------------------------------- closed forms

@pytest.mark.parametrize("bm,bv", [(2, 2), (3, 3), (4, 4), (2, 3)])
def test_constant_gradient_closed_form(so, bm, bv):
    """g == c on every element: m^_t = (1-beta1^t) c sits on the top level, v^_t =
    (1-beta2^t) c^2 is a constant block (alpha = 1, code 0), nothing is lost to rounding and
    the parameters follow bias-corrected AdamW exactly; beta2 = 0.999 is above every linear
    swamping threshold of Cor. 3.2 and the state still moves."""
    n, c, T = 256, -3e-3, 12
    cfg = so.make_config(bits_m=bm, bits_v=bv, block_size=128, beta1=0.8, beta2=0.999,
                         lr=1e-3, weight_decay=0.01, eps=1e-8)
    rng = np.random.default_rng(0)
    p = (rng.standard_normal(n) * 0.02).astype(np.float32)
    p64 = p.astype(np.float64)
    mc, ms, vc, vs, va = fresh_unpacked(so, n, cfg)
    g = np.full(n, c, np.float32)
    b1, b2 = float(np.float32(0.8)), float(np.float32(0.999))
    c32 = float(np.float32(c))
    for t in range(1, T + 1):
        so.step_unpacked(p, g, mc, ms, vc, vs, va, t, cfg)
        mh, vh = (1 - b1 ** t) * c32, (1 - b2 ** t) * c32 * c32
        assert np.all(mc == 0) and np.all(vc == 0) and np.all(va == 1)          # c < 0: level -1
        assert np.allclose(ms, abs(mh), rtol=1e-6) and np.allclose(vs, vh, rtol=1e-5)
        lr, wd, eps = float(np.float32(1e-3)), float(np.float32(0.01)), float(np.float32(1e-8))
        p64 = p64 * (1 - lr * wd) - lr * (mh / (1 - b1 ** t)) / (math.sqrt(vh / (1 - b2 ** t)) + eps)
        assert np.allclose(p, p64, rtol=1e-6, atol=1e-9)


@pytest.mark.parametrize("bits_v", BITS)
def test_zero_gradient_keeps_codes_and_decays_scales(so, bits_v):
    """g == 0: every level is multiplied by beta, so codes stay and only the scales decay
    (the exact-decay property of Prop. 3.4 carried by Delta); xi is off and the quantile
    element already sits on the last level, so the base is reproduced too."""
    B, K = 128, 2 ** bits_v - 1
    cfg = so.make_config(bits_m=4, bits_v=bits_v, block_size=B, stochastic=0, beta1=0.8)
    rng = np.random.default_rng(3)
    n = 4 * B
    mc = rng.integers(0, 15, n).astype(np.uint16)
    mc[::B] = 14                                                   # the block maximum exists
    vc = rng.integers(0, K + 1, n).astype(np.uint16)
    vc[::B] = 0
    vc[1:: 4] = K                                                  # >= 13 elements on the last level
    ms = np.float32(10.0) ** rng.uniform(-6, 0, 4).astype(np.float32)
    vs = np.float32(10.0) ** rng.uniform(-9, 0, 4).astype(np.float32)
    va = np.array([0.31, 0.5, 0.77, 0.93], np.float32)
    p = np.ones(n, np.float32)
    g = np.zeros(n, np.float32)
    mc0, vc0, ms0, vs0, va0 = mc.copy(), vc.copy(), ms.copy(), vs.copy(), va.copy()
    so.step_unpacked(p, g, mc, ms, vc, vs, va, 5, cfg)
    assert np.array_equal(mc, mc0) and np.array_equal(vc, vc0)
    assert np.array_equal(vs, np.float32(0.999) * vs0)             # one rounding: fl(beta2*Delta)
    assert np.allclose(ms, np.float32(0.8) * ms0, rtol=3e-7)
    assert np.all(np.abs(va.astype(np.float64) / va0 - 1) <= 2.0 ** -21)


def test_reduces_to_adamw_as_codes_widen(so):
    """16-bit codes, p = 0 (base from the block minimum), xi off: the quantized step equals
    textbook AdamW (decoupled decay, bias correction, eps outside the root) in binary64 to
    the resolution of the codes; narrower codes move away from it monotonically."""
    n, T = 1024, 25
    rng = np.random.default_rng(21)
    p0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    grads = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(T)]
    # eps is made comparable to sqrt(v) (about 1e-3) so that its placement matters
    b1, b2, lr, wd, eps = (float(np.float32(x)) for x in (0.9, 0.999, 1e-3, 0.01, 3e-4))
    p64, m, v = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t, g in enumerate(grads, 1):
        g = g.astype(np.float64)
        m = b1 * m + (1 - b1) * g
        v = b2 * v + (1 - b2) * g * g
        p64 = p64 * (1 - lr * wd) - lr * (m / (1 - b1 ** t)) / (np.sqrt(v / (1 - b2 ** t)) + eps)
    err = {}
    for bits in (16, 8, 4):
        cfg = so.make_config(bits_m=bits, bits_v=bits, block_size=128, stochastic=0, beta1=0.9,
                             quantile_p=0.0, eps=3e-4)
        p = p0.copy()
        st = fresh_unpacked(so, n, cfg)
        for t, g in enumerate(grads, 1):
            so.step_unpacked(p, g, *st, t, cfg)
        err[bits] = np.max(np.abs(p - p64))
    total_move = np.max(np.abs(p64 - p0))
    # 65536 log levels between the block minimum and maximum leave a relative step of about
    # ln(max/min)/65535 ~ 3e-4 in v; the rounding errors ride along with beta2 = 0.999
    assert err[16] < 1e-3 * total_move and err[16] < 1e-5
    assert err[8] < 0.1 * total_move
    assert err[16] < err[8] < err[4]


def _wide_code_run(so, optimizer, p0, grads, eps, wd, beta1=0.9):
    cfg = so.make_config(bits_m=16, bits_v=16, block_size=128, stochastic=0, beta1=beta1,
                         quantile_p=0.0, eps=eps, weight_decay=wd, optimizer=optimizer)
    p = p0.copy()
    st = fresh_unpacked(so, p.size, cfg)
    for t, g in enumerate(grads, 1):
        so.step_unpacked(p, g, *st, t, cfg)
    return p


@pytest.mark.parametrize("which", ("AdamW", "Adam"))
def test_wide_codes_follow_the_library_optimizers(so, which):
    """16-bit codes against torch.optim.AdamW (decoupled decay) and torch.optim.Adam (decay added
    to the gradient) run in binary64: the two differ visibly at this decay, and the oracle's
    two modes follow the matching one."""
    import torch
    n, T, eps, wd = 1024, 25, 3e-4, 0.5
    rng = np.random.default_rng(33)
    p0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    grads = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(T)]
    ref = {}
    for name, cls in (("AdamW", torch.optim.AdamW), ("Adam", torch.optim.Adam)):
        w = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
        opt = cls([w], lr=float(np.float32(1e-3)), betas=(float(np.float32(0.9)), float(np.float32(0.999))),
                  eps=float(np.float32(eps)), weight_decay=float(np.float32(wd)))
        for g in grads:
            w.grad = torch.tensor(g, dtype=torch.float64)
            opt.step()
        ref[name] = w.detach().numpy()
    got = _wide_code_run(so, so.ADAMW if which == "AdamW" else so.ADAM_L2, p0, grads, eps, wd)
    other = "Adam" if which == "AdamW" else "AdamW"
    move = np.max(np.abs(ref[which] - p0))
    assert np.max(np.abs(got - ref[which])) < 2e-3 * move
    assert np.max(np.abs(got - ref[other])) > 20 * np.max(np.abs(got - ref[which]))


def test_adabelief_closed_forms(so):
    """AdaBelief (the unsigned EMA follows (g - m^)^2 and gains eps at every step) in two cases
    that have closed forms.  beta1 = 0: m^ = g, so s_t = eps (1 - beta2^t) / (1 - beta2) whatever
    the gradients, every block is constant, and the update is lr g / (sqrt(eps / (1 - beta2)) + eps).
    Constant gradient c: g - m^_t = c beta1^t, so s_t is a sum of two geometric series."""
    n, T = 256, 10
    rng = np.random.default_rng(8)
    b2, lr, eps = float(np.float32(0.999)), float(np.float32(1e-3)), float(np.float32(1e-8))
    # (1) beta1 = 0
    cfg = so.make_config(bits_m=4, bits_v=3, block_size=128, beta1=0.0, weight_decay=0.0, eps=1e-8,
                         optimizer=so.ADABELIEF)
    p = (rng.standard_normal(n) * 0.02).astype(np.float32)
    p64 = p.astype(np.float64)
    mc, ms, vc, vs, va = fresh_unpacked(so, n, cfg)
    for t in range(1, T + 1):
        g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        so.step_unpacked(p, g, mc, ms, vc, vs, va, t, cfg)
        s_t = eps * (1 - b2 ** t) / (1 - b2)
        assert np.allclose(vs, s_t, rtol=1e-5) and np.all(va == 1) and np.all(vc == 0)
        p64 = p64 - lr * g.astype(np.float64) / (math.sqrt(eps / (1 - b2)) + eps)
        assert np.allclose(p, p64, rtol=2e-6, atol=1e-9)
    # (2) constant gradient, beta1 = 0.8: m^ sits on the top level, s is a constant block
    b1, c = float(np.float32(0.8)), float(np.float32(2e-3))
    cfg = so.make_config(bits_m=4, bits_v=3, block_size=128, beta1=0.8, weight_decay=0.0, eps=1e-8,
                         optimizer=so.ADABELIEF)
    p = (rng.standard_normal(n) * 0.02).astype(np.float32)
    p64 = p.astype(np.float64)
    mc, ms, vc, vs, va = fresh_unpacked(so, n, cfg)
    g = np.full(n, c, np.float32)
    s = 0.0
    for t in range(1, T + 1):
        so.step_unpacked(p, g, mc, ms, vc, vs, va, t, cfg)
        s = sum(b2 ** (t - k) * ((1 - b2) * (c * b1 ** k) ** 2 + eps) for k in range(1, t + 1))
        assert np.allclose(vs, s, rtol=1e-5) and np.all(vc == 0)
        assert np.allclose(ms, c * (1 - b1 ** t), rtol=1e-6)
        p64 = p64 - lr * c / (math.sqrt(s / (1 - b2 ** t)) + eps)
        assert np.allclose(p, p64, rtol=2e-6, atol=1e-9)


def test_adabelief_follows_a_binary64_run_as_codes_widen(so):
    """16-bit codes against AdaBelief with decoupled decay written out in binary64."""
    n, T = 1024, 25
    rng = np.random.default_rng(34)
    p0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    grads = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(T)]
    b1, b2, lr, wd, eps = (float(np.float32(x)) for x in (0.9, 0.999, 1e-3, 0.01, 1e-8))
    p64, m, s = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t, g in enumerate(grads, 1):
        g = g.astype(np.float64)
        m = b1 * m + (1 - b1) * g
        s = b2 * s + (1 - b2) * (g - m) ** 2 + eps
        p64 = p64 * (1 - lr * wd) - lr * (m / (1 - b1 ** t)) / (np.sqrt(s / (1 - b2 ** t)) + eps)
    got = _wide_code_run(so, so.ADABELIEF, p0, grads, 1e-8, 0.01)
    adam = _wide_code_run(so, so.ADAMW, p0, grads, 1e-8, 0.01)
    move = np.max(np.abs(p64 - p0))
    assert np.max(np.abs(got - p64)) < 2e-3 * move
    assert np.max(np.abs(adam - p64)) > 20 * np.max(np.abs(got - p64))


def test_gradient_scale_is_one_multiplication_in_binary32(so):
    """scale s on g equals scale 1 on fl(g * s), bit for bit; a power of two undoes exactly."""
    n = 300
    rng = np.random.default_rng(4)
    g = (rng.standard_normal(n) * 3.0).astype(np.float32)
    p0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    outs = []
    for gg, s in ((g, 1 / 3), ((g * np.float32(1 / 3)).astype(np.float32), 1.0),
                  (g * np.float32(4096), 1 / 3 / 4096)):
        cfg = so.make_config(bits_m=2, bits_v=3, block_size=128, beta1=0.5, grad_scale=s)
        p = p0.copy()
        st = fresh_unpacked(so, n, cfg)
        for t in (1, 2, 3):
            so.step_unpacked(p, np.ascontiguousarray(gg, np.float32), *st, t, cfg)
        outs.append((p, *st))
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert np.array_equal(a, b)


def test_bf16_rounding_matches_the_library_conversion(so):
    import torch
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(200000) * 10.0 ** rng.integers(-30, 30, 200000)).astype(np.float32)
    x[:8] = [0.0, -0.0, 1.0, 3.39e38, 3.3895e38, -3.4e38, 1e-45, np.float32(1.00390625)]   # last: a tie
    ties = (rng.integers(0, 0x7F7F, 1000).astype(np.uint32) << 16 | 0x8000).view(np.float32)
    x = np.concatenate([x, ties, -ties])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(so.round_bf16(x), want)


def test_swamping_thresholds_match_paper(so):
    """Thm 3.1 / generalized Cor. 3.2: with the scale held fixed, a nearest-rounded signed
    linear code cannot change for any |z| <= Delta once beta >= 1 - r/2; below that
    threshold it can.  The thresholds are the ones the paper prints."""
    rng = np.random.default_rng(8)
    for bits, beta in read_golden("swamping_thresholds_signed_linear.txt"):
        bits, beta = int(bits), float(beta)
        if bits > 4:
            continue
        L = so.L_of(bits)
        assert abs((1 - 1 / (4 * L)) - beta) < 1.1e-3              # 1 - r/2 with r = 1/(2L)
        delta = np.float32(0.73)
        for b_test, must_hold in ((beta + 2e-3, True), (beta - 0.06, False)):
            changed = False
            for c in range(2 * L + 1):
                state = so.dequant_m(c, delta, bits)
                z = rng.uniform(-1, 1, 500).astype(np.float32) * delta
                z[:2] = (delta, -delta)
                xh = (np.float32(b_test) * state + np.float32(1 - b_test) * z).astype(np.float32)
                xh = np.clip(xh, -delta, delta)                    # rounding may add an ulp
                blk = np.concatenate([xh, [delta]]).astype(np.float32)   # keeps Delta fixed
                codes, scale = so.quant_m_block(blk, bits)
                assert scale == delta
                changed |= bool(np.any(codes[:-1] != c))
            assert changed != must_hold


# ------------------------------------------------------ degenerate inputs

def test_first_step_from_the_zero_state_and_zero_blocks(so):
    for bm in BITS:
        for bv in BITS:
            cfg = so.make_config(bits_m=bm, bits_v=bv, block_size=64, beta1=0.5)
            n = 64 * 3 + 10
            rng = np.random.default_rng(bm * 8 + bv)
            p = (rng.standard_normal(n) * 0.02).astype(np.float32)
            g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
            g[64:128] = 0                                          # an all-zero block
            g[128:192] = 2e-3                                      # a constant block
            st = so.State(n, cfg)
            p_before = p.copy()
            so.step_packed(p, g, st, 1, cfg)
            assert np.all(np.isfinite(p))
            assert st.m_scale[1] == 0 and st.v_scale[1] == 0 and st.v_base[1] == 1
            assert np.allclose(p[64:128], p_before[64:128] * (1 - 1e-3 * 0.01), rtol=1e-6)
            mc, vc = so.unpack(st.m_words, n, bm), so.unpack(st.v_words, n, bv)
            assert np.all(mc[64:128] == so.L_of(bm)) and np.all(vc[64:128] == 0)
            assert st.v_base[2] == 1 and np.all(vc[128:192] == 0) and np.all(mc[128:192] == 2 * so.L_of(bm))
            assert 0 < st.v_base[0] < 1 and 0 < st.v_base[3] < 1
            assert st.m_scale[3] == np.max(np.abs(np.float32(0.5) * g[192:]))   # tail block of 10


def test_sparse_block_clamps_the_base_and_zero_takes_last_code(so):
    """Most of a block has zero gradient (sparse embedding rows, Sec. 3.2.2): x_p = 0, the
    ratio is clamped at 2^-64 and zeros take the last code."""
    cfg = so.make_config(bits_m=2, bits_v=3, block_size=128, beta1=0.5)
    n = 128
    g = np.zeros(n, np.float32)
    g[:5] = [1e-3, -2e-3, 5e-4, 1e-4, 3e-3]
    p = np.zeros(n, np.float32)
    st = so.State(n, cfg)
    so.step_packed(p, g, st, 1, cfg)
    vc = so.unpack(st.v_words, n, 3)
    assert np.all(vc[5:] == 7) and vc[4] == 0
    assert abs(float(st.v_base[0]) / 2.0 ** (-64 / 7) - 1) < 1e-6
    assert np.all(np.isfinite(p))
    so.step_packed(p, np.zeros(n, np.float32), st, 2, cfg)          # and it stays finite
    assert np.all(np.isfinite(p)) and np.isfinite(st.v_base[0]) and st.v_scale[0] > 0


def test_underflowing_block_is_flushed_to_the_zero_block(so):
    cfg = so.make_config(bits_m=4, bits_v=4, block_size=64, beta1=0.8)
    g = np.full(64, 1e-17, np.float32)                              # v^ = 1e-37 < 2^-100
    p = np.zeros(64, np.float32)
    st = so.State(64, cfg)
    so.step_packed(p, g, st, 1, cfg)
    assert st.v_scale[0] == 0 and st.v_base[0] == 1 and st.m_scale[0] > 0
    assert np.all(np.isfinite(p))


@pytest.mark.parametrize("bm,bv,B", [(2, 3, 128), (3, 3, 64), (4, 2, 128)])
def test_packed_step_equals_unpacked_step(so, bm, bv, B):
    rng = np.random.default_rng(77)
    n = 5 * B + 37
    cfg = so.make_config(bits_m=bm, bits_v=bv, block_size=B, beta1=0.6)
    p1 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    p2 = p1.copy()
    st = so.State(n, cfg)
    un = fresh_unpacked(so, n, cfg)
    for step in range(1, 5):
        g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        so.step_packed(p1, g, st, step, cfg, threads=2)
        so.step_unpacked(p2, g, *un, step, cfg)
        assert np.array_equal(p1, p2)
        assert np.array_equal(so.unpack(st.m_words, n, bm), un[0])
        assert np.array_equal(so.unpack(st.v_words, n, bv), un[2])
        assert np.array_equal(st.m_scale, un[1]) and np.array_equal(st.v_scale, un[3])
        assert np.array_equal(st.v_base, un[4])


def test_index_offset_shifts_the_xi_stream(so):
    """A shard that starts at global element k sees the same xi as the full buffer."""
    rng = np.random.default_rng(4)
    n, B, off = 1024, 128, 512
    cfg = so.make_config(bits_m=3, bits_v=3, block_size=B, beta1=0.6)
    p = (rng.standard_normal(n) * 0.02).astype(np.float32)
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    full = fresh_unpacked(so, n, cfg)
    pf = p.copy()
    so.step_unpacked(pf, g, *full, 3, cfg)
    cfg2 = so.make_config(bits_m=3, bits_v=3, block_size=B, beta1=0.6, index_offset=off)
    part = fresh_unpacked(so, n - off, cfg2)
    pp = p[off:].copy()
    so.step_unpacked(pp, g[off:].copy(), *part, 3, cfg2)
    assert np.array_equal(pp, pf[off:]) and np.array_equal(part[2], full[2][off:])
    assert np.array_equal(part[4], full[4][off // B:])
