"""GPU parity on the named configurations at their real sizes (the bar is in parity_common.py).

  * Config 3 (GPT-2-125M shapes, 2-bit states, block 64) as its whole tensor set, every element:
    as one flat buffer and as its 99 tensors in one multi-tensor launch; ten teacher-forced steps
    (both sides start every step from the oracle's state) and ten free-running steps.
  * Configs 4 and 5 (1.3B and LLaMA-7B shapes) at full size in the launch configuration the
    benchmark times: ten free-running steps of the whole flat buffer on the GPU; the oracle
    follows a slice of up to 2^26 elements of every tensor class on its own trajectory
    (free-running) and, every step, recomputes from the GPU's own state those slices plus the
    first and last 1024 blocks of every tensor (equal starting states: teacher-forced by the
    state that is there).  Every byte of the slices is compared.
  * Exactly-once at full size (properties that need no oracle at that size): the step of the
    whole buffer equals, bit for bit, the same step made in unequal pieces with other launch
    shapes; it is reproducible; it changes every 5120-element tile; and from the zero state
    under a constant gradient every block of the buffer lands on the one closed-form state.
  * The sparse-embedding stress of Sec. 3.2.2 on an embedding-shaped slice.
"""
import types

import numpy as np
import pytest

from parity_common import (TILE, dev, make_cfgs, compare_step, compare_on_device, DeviceView, flip_budget,
                           note, progress)

pytestmark = pytest.mark.gpu

THREADS = 16


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2505_00347_amd import solo
    solo.lib()
    return solo


def workload_cfgs(so, solo, w, **kw):
    return make_cfgs(so, solo, w.bits_m, w.bits_v, w.block_size, bf16=(w.grad_dtype == "bf16"), beta1=w.beta1,
                     lr=w.lr, wd=w.weight_decay, eps=w.eps, beta2=w.beta2, p=w.quantile_p,
                     de=(w.m_codebook == "de"), **kw)


def grads_of(torch, bench, synth, w, step):
    """Full-size gradients of one step on the device (the benchmark's generator)."""
    dt = torch.bfloat16 if w.grad_dtype == "bf16" else torch.float32
    return bench.device_grads(torch, w.n, w.grad_kind, w.grad_std, synth.seed_grad(w.config_id, step), dt,
                              bench.sparse_rows_of(w))


# --------------------------------------------------------- config 3, the whole tensor set

def test_config3_whole_tensor_set_flat(so, gpu):
    """All 124 M elements of the GPT-2-125M-shaped set as one flat buffer (2-bit states, block 64,
    fp32 gradients): ten teacher-forced and ten free-running steps, every element compared."""
    import torch
    import bench
    from paper_2505_00347_amd import synth
    solo = gpu
    w = synth.workload("c3_gpt2_125m_2bit")
    n = w.n
    oc, gc = workload_cfgs(so, solo, w)
    p_dev = bench.device_params(torch, w, synth.SEED_PARAM)
    p = p_dev.cpu().numpy()
    st = so.State(n, oc)
    tf_state, fr_state = solo.SoloState(n, gc), solo.SoloState(n, gc)
    p_tf, p_fr = p_dev.clone(), p_dev
    v_tf, v_fr = DeviceView.of(p_tf, tf_state), DeviceView.of(p_fr, fr_state)
    tainted = torch.zeros(st.m_scale.size, dtype=torch.bool, device="cuda")
    flips_tf = flips_fr = 0
    worst_tf = worst_fr = 0.0
    for step in range(1, w.steps + 1):
        g_dev = grads_of(torch, bench, synth, w, step)
        g = g_dev.cpu().numpy()
        v_tf.load(p, st)
        tf_state.step(p_tf, g_dev, step)
        fr_state.step(p_fr, g_dev, step)
        p_before = p.copy()
        margin = so.step_packed(p, g, st, step, oc, want_margin=True, threads=THREADS)
        f, e = compare_on_device(so, oc, v_tf, p, st, margin, 1e-6, 2e-6 * oc.lr, p_before=p_before,
                                 label=f"c3 flat teacher-forced step {step}")
        flips_tf += f; worst_tf = max(worst_tf, e)
        f, e = compare_on_device(so, oc, v_fr, p, st, margin, 1e-5, 1e-5 * oc.lr, tainted=tainted,
                                 label=f"c3 flat free-running step {step}")
        flips_fr += f; worst_fr = e
        progress(f"c3 flat step {step} done")
    diverged = int(tainted.sum())
    note(f"config 3 flat, {n} elements x {w.steps} steps: teacher-forced {flips_tf} flips, worst parameter error "
         f"{worst_tf:.2f} of the one-step bound; free-running {flips_fr} flips, {diverged} of {tainted.numel()} "
         f"blocks diverged, 10-step parameter error {worst_fr:.3f} of 1e-5 (|p| + lr)")
    assert flips_tf <= flip_budget(n * w.steps) and flips_fr <= flip_budget(n * w.steps)
    assert diverged <= flip_budget(n * w.steps)


def test_config3_whole_tensor_set_multi_tensor_launch(so, gpu):
    """The same tensors (99: the embedding, four matrices and four LayerNorm vectors per layer,
    the final LayerNorm), each with buffers of its own, through solo_adamw_step_multi: one
    launch per step; the oracle runs tensor by tensor with the tensor's own xi offset."""
    import torch
    import bench
    from paper_2505_00347_amd import synth
    solo = gpu
    w = synth.workload("c3_gpt2_125m_2bit")
    oc, gc = workload_cfgs(so, solo, w)
    p_all = bench.device_params(torch, w, synth.SEED_PARAM)
    tens = []
    pos = unit0 = 0
    for name, numel, kind in w.tensors:
        cfg_k = so.make_config(bits_m=w.bits_m, bits_v=w.bits_v, block_size=w.block_size, beta1=w.beta1, lr=w.lr,
                               weight_decay=w.weight_decay, eps=w.eps, beta2=w.beta2, quantile_p=w.quantile_p,
                               index_offset=2560 * unit0)
        t = types.SimpleNamespace(n=numel, pos=pos, cfg=cfg_k, p=p_all[pos:pos + numel].cpu().numpy(),
                                  st=so.State(numel, cfg_k),
                                  p_tf=p_all[pos:pos + numel].clone(), p_fr=p_all[pos:pos + numel].clone(),
                                  s_tf=solo.SoloState(numel, gc), s_fr=solo.SoloState(numel, gc))
        t.v_tf, t.v_fr = DeviceView.of(t.p_tf, t.s_tf), DeviceView.of(t.p_fr, t.s_fr)
        t.tainted = torch.zeros(t.st.m_scale.size, dtype=torch.bool, device="cuda")
        tens.append(t)
        pos += numel
        unit0 += -(-numel // 2560)
    flips_tf = flips_fr = 0
    worst_tf = worst_fr = 0.0
    n = w.n
    for step in range(1, w.steps + 1):
        g_dev = grads_of(torch, bench, synth, w, step)
        g = g_dev.cpu().numpy()
        for t in tens:
            t.v_tf.load(t.p, t.st)
        gs = [g_dev[t.pos:t.pos + t.n] for t in tens]
        solo.SoloMultiTable([(t.p_tf, gs[k], t.s_tf) for k, t in enumerate(tens)], gc).step(step)
        solo.SoloMultiTable([(t.p_fr, gs[k], t.s_fr) for k, t in enumerate(tens)], gc).step(step)
        worst_fr = 0.0
        for t in tens:
            p_before = t.p.copy()
            gk = np.ascontiguousarray(g[t.pos:t.pos + t.n])
            margin = so.step_packed(t.p, gk, t.st, step, t.cfg, want_margin=True,
                                    threads=THREADS if t.n > 100000 else 1)
            f, e = compare_on_device(so, oc, t.v_tf, t.p, t.st, margin, 1e-6, 2e-6 * oc.lr, p_before=p_before,
                                     label=f"c3 multi teacher-forced step {step} tensor at {t.pos}")
            flips_tf += f; worst_tf = max(worst_tf, e)
            f, e = compare_on_device(so, oc, t.v_fr, t.p, t.st, margin, 1e-5, 1e-5 * oc.lr, tainted=t.tainted,
                                     label=f"c3 multi free-running step {step} tensor at {t.pos}")
            flips_fr += f; worst_fr = max(worst_fr, e)
        progress(f"c3 multi step {step} done")
    diverged = sum(int(t.tainted.sum()) for t in tens)
    note(f"config 3 as {len(tens)} tensors in one launch, {n} elements x {w.steps} steps: teacher-forced "
         f"{flips_tf} flips, worst parameter error {worst_tf:.2f} of the one-step bound; free-running {flips_fr} "
         f"flips, {diverged} blocks diverged, 10-step parameter error {worst_fr:.3f} of 1e-5 (|p| + lr)")
    assert flips_tf <= flip_budget(n * w.steps) and flips_fr <= flip_budget(n * w.steps)


# ------------------------------------------- configs 4 and 5 at full size: slices per tensor class

def union(intervals):
    out = []
    for a, b in sorted(intervals):
        if out and a <= out[-1][1]:
            out[-1][1] = max(out[-1][1], b)
        else:
            out.append([a, b])
    return [(a, b) for a, b in out]


def protocol_slices(w, class_len=1 << 26, edge_blocks=1024, align=640):
    """(class slices, all slices): up to class_len elements of the first tensor of every size
    class, and those plus the first and last edge_blocks blocks of every tensor; every slice is
    widened to a multiple of 640 elements (whole blocks and whole code words of every width)."""
    n = w.n

    def widen(a, b):
        return (a // align * align, min(n, -(-b // align) * align))

    classes, edges, seen, pos = [], [], set(), 0
    e = edge_blocks * w.block_size
    for _, numel, _ in w.tensors:
        if numel not in seen:
            seen.add(numel)
            classes.append(widen(pos, pos + min(numel, class_len)))
        if numel <= 2 * e:
            edges.append(widen(pos, pos + numel))
        else:
            edges += [widen(pos, pos + e), widen(pos + numel - e, pos + numel)]
        pos += numel
    classes = union(classes)
    return classes, union(classes + edges)


class PackedSlices:
    """Slices of a large flat device buffer and its state, packed one behind the other: on the
    host as numpy arrays the oracle steps slice by slice (each with its global xi offset), on
    the device as gathered copies for the comparison."""

    def __init__(self, so, oc, slices):
        self.so, self.oc, self.slices = so, oc, slices
        self.B, self.cm, self.cv = oc.block_size, 32 // oc.bits_m, 32 // oc.bits_v
        self.total = sum(b - a for a, b in slices)
        self.off = np.cumsum([0] + [b - a for a, b in slices])[:-1]
        for a, b in slices[:-1]:
            assert (b - a) % 640 == 0 and a % 640 == 0
        self.p = np.zeros(self.total, np.float32)
        self.st = so.State(self.total, oc)               # the packed state (zero state to start with)
        self.margin = np.zeros(self.total, np.float64)

    def gather(self, torch, p, state):
        """Packed device copies (a DeviceView) of the slices of (p, state)."""
        B, cm, cv = self.B, self.cm, self.cv
        cat = torch.cat
        sl = self.slices
        return DeviceView(cat([p[a:b] for a, b in sl]),
                          cat([state.m_codes[a // cm:-(-b // cm)] for a, b in sl]),
                          cat([state.m_scale[a // B:-(-b // B)] for a, b in sl]),
                          cat([state.v_codes[a // cv:-(-b // cv)] for a, b in sl]),
                          cat([state.v_scale[a // B:-(-b // B)] for a, b in sl]),
                          cat([state.v_base[a // B:-(-b // B)] for a, b in sl]))

    def gather_grads(self, torch, g):
        return torch.cat([g[a:b] for a, b in self.slices]).float().cpu().numpy()

    def take(self, view):
        """Host state := the packed device copies."""
        self.p[:] = view.p.cpu().numpy()
        st = view.to_host_state(self.so, self.oc)
        for k in ("m_words", "v_words", "m_scale", "v_scale", "v_base"):
            getattr(self.st, k)[:] = getattr(st, k)

    def oracle_step(self, g, step, make_cfg):
        """One oracle step on every slice, in place; fills the margins."""
        B, cm, cv = self.B, self.cm, self.cv
        for (a, b), o in zip(self.slices, self.off):
            ln = b - a
            view = types.SimpleNamespace(
                m_words=self.st.m_words[o // cm:o // cm - (-ln // cm)], v_words=self.st.v_words[o // cv:o // cv - (-ln // cv)],
                m_scale=self.st.m_scale[o // B:o // B - (-ln // B)], v_scale=self.st.v_scale[o // B:o // B - (-ln // B)],
                v_base=self.st.v_base[o // B:o // B - (-ln // B)])
            m = self.so.step_packed(self.p[o:o + ln], g[o:o + ln], view, step, make_cfg(a), want_margin=True,
                                    threads=THREADS if ln > 100000 else 1)
            self.margin[o:o + ln] = m


def run_full_size_protocol(so, solo, name, steps=10):
    import torch
    import bench
    from paper_2505_00347_amd import synth
    w = synth.workload(name)
    n = w.n
    free, _ = torch.cuda.mem_get_info()
    if free < 60 * 2 ** 30:
        pytest.skip("needs 60 GiB of free HBM")
    oc, gc = workload_cfgs(so, solo, w)

    def cfg_at(a):
        return so.make_config(bits_m=w.bits_m, bits_v=w.bits_v, block_size=w.block_size, beta1=w.beta1, lr=w.lr,
                              weight_decay=w.weight_decay, eps=w.eps, beta2=w.beta2, quantile_p=w.quantile_p,
                              index_offset=a, m_codebook=1 if w.m_codebook == "de" else 0)

    classes, everything = protocol_slices(w)
    fr = PackedSlices(so, oc, classes)       # the oracle's own trajectory
    tf = PackedSlices(so, oc, everything)    # recomputed every step from the GPU's state
    p = bench.device_params(torch, w, synth.SEED_PARAM)
    state = solo.SoloState(n, gc)
    fr.p[:] = fr.gather(torch, p, state).p.cpu().numpy()
    tainted = torch.zeros(fr.st.m_scale.size, dtype=torch.bool, device="cuda")
    flips_tf = flips_fr = 0
    worst_tf = worst_fr = 0.0
    for step in range(1, steps + 1):
        g = grads_of(torch, bench, synth, w, step)
        tf.take(tf.gather(torch, p, state))
        p_before = tf.p.copy()
        g_tf, g_fr = tf.gather_grads(torch, g), fr.gather_grads(torch, g)
        state.step(p, g, step)                         # the whole flat buffer, one call, as the benchmark launches it
        del g
        tf.oracle_step(g_tf, step, cfg_at)
        f, e = compare_on_device(so, oc, tf.gather(torch, p, state), tf.p, tf.st, tf.margin, 1e-6, 2e-6 * oc.lr,
                                 p_before=p_before, label=f"{name} step {step} from the GPU's state")
        flips_tf += f; worst_tf = max(worst_tf, e)
        fr.oracle_step(g_fr, step, cfg_at)
        f, e = compare_on_device(so, oc, fr.gather(torch, p, state), fr.p, fr.st, fr.margin, 1e-5, 1e-5 * oc.lr,
                                 tainted=tainted, label=f"{name} free-running step {step}")
        flips_fr += f; worst_fr = e
        progress(f"{name} step {step} done")
    diverged = int(tainted.sum())
    note(f"{name} at full size ({n} elements, {steps} steps): {tf.total} elements in {len(everything)} slices "
         f"recomputed every step from the GPU's state: {flips_tf} flips, worst parameter error {worst_tf:.2f} of "
         f"the one-step bound; {fr.total} elements of {len(classes)} tensor classes free-running: {flips_fr} flips, "
         f"{diverged} blocks diverged, 10-step parameter error {worst_fr:.3f} of 1e-5 (|p| + lr)")
    assert flips_tf <= flip_budget(tf.total * steps) and flips_fr <= flip_budget(fr.total * steps)
    assert diverged <= flip_budget(fr.total * steps)


def test_config4_full_size_slices_per_tensor_class(so, gpu):
    run_full_size_protocol(so, gpu, "c4_1p3b_3bit")


def test_config5_full_size_slices_per_tensor_class(so, gpu):
    run_full_size_protocol(so, gpu, "c5_llama7b_2bit_3bit")


# --------------------------------------------------------------- exactly once, at full size

@pytest.mark.parametrize("name", ("c5_llama7b_2bit_3bit", "c5_llama7b_block2048"))
def test_config5_full_size_every_tile_exactly_once(so, gpu, name):
    """Whole-buffer properties of the metric's launch (6.7e9 elements, one call; also with blocks
    of 2048 elements, where a "tile" below is a run of five blocks).  (1) From the
    zero state under a constant gradient every block must land on the one state the oracle
    computes for a single block, and every parameter on p (1 - lr wd) - u with the one update u:
    a tile that is skipped, or stepped twice, shows.  (2) With random gradients, a step from a
    warmed-up state changes every 5120-element tile (parameters, Delta_v and code words), is
    reproduced bit for bit from restored inputs, and equals bit for bit the same step made in
    about twenty unequal pieces (each a call of its own with its index_offset: other grids, other
    tile-to-workgroup maps, and the short-tensor path for the small pieces)."""
    import torch
    import bench
    from paper_2505_00347_amd import synth
    solo = gpu
    w = synth.workload(name)
    n = w.n
    free, _ = torch.cuda.mem_get_info()
    if free < 130 * 2 ** 30:
        pytest.skip("needs 130 GiB of free HBM")
    oc, gc = workload_cfgs(so, solo, w)
    B, cm, cv = w.block_size, 32 // w.bits_m, 32 // w.bits_v
    tile, PIECE = (5120, 2560) if B != 2048 else (5 * 2048, 5 * 2048)   # whole blocks and whole words of both streams
    p = bench.device_params(torch, w, synth.SEED_PARAM)
    state = solo.SoloState(n, gc)

    # (1) constant gradient from the zero state
    c = 2.0 ** -10
    g = torch.full((n,), c, dtype=torch.bfloat16, device="cuda")
    p0 = p.clone()
    state.step(p, g, 1)
    torch.cuda.synchronize()
    one = so.State(B, oc)
    pb = np.zeros(B, np.float32)
    so.step_packed(pb, np.full(B, c, np.float32), one, 1, oc)
    u = -float(pb[0])                                   # the update of a parameter that starts at 0
    for got, want in ((state.m_scale, one.m_scale), (state.v_scale, one.v_scale), (state.v_base, one.v_base)):
        assert bool((got.view(torch.int32) == int(want.view(np.int32)[0])).all())
    assert bool((state.m_codes == int(one.m_words.view(np.int32)[0])).all())
    assert bool((state.v_codes == int(one.v_words.view(np.int32)[0])).all())
    decay = 1.0 - oc.lr * oc.weight_decay
    chunk = 1 << 28
    for a in range(0, n, chunk):
        want = p0[a:a + chunk].double() * decay - u
        err = (p[a:a + chunk].double() - want).abs()
        assert bool((err <= 1e-6 * want.abs() + 2e-6 * oc.lr).all()), f"constant-gradient update wrong in [{a}, {a + chunk})"
    del p0, g
    progress(f"{name} exactly-once: constant gradient done")

    # (2) random gradients from a warmed-up state
    for step in (2, 3):
        g = grads_of(torch, bench, synth, w, step)
        state.step(p, g, step)
        del g
    g = grads_of(torch, bench, synth, w, 4)
    names = ("m_codes", "m_scale", "v_codes", "v_scale", "v_base")
    before = [p.clone()] + [getattr(state, k).clone() for k in names]

    def restore():
        p.copy_(before[0])
        for k, t in zip(names, before[1:]):
            getattr(state, k).copy_(t)

    state.step(p, g, 4)
    torch.cuda.synchronize()
    whole = [p.clone()] + [getattr(state, k).clone() for k in names]
    nt = n // tile
    assert bool((whole[0][:nt * tile].view(nt, tile) != before[0][:nt * tile].view(nt, tile)).any(1).all()), \
        "a tile's parameters did not change"
    assert bool((whole[4][:nt * (tile // B)].view(nt, -1) != before[4][:nt * (tile // B)].view(nt, -1)).any(1).all()), \
        "a tile's Delta_v did not change"
    mch = (whole[1][:nt * (tile // cm)].view(nt, -1) != before[1][:nt * (tile // cm)].view(nt, -1)).any(1)
    vch = (whole[3][:nt * (tile // cv)].view(nt, -1) != before[3][:nt * (tile // cv)].view(nt, -1)).any(1)
    assert bool((mch | vch).all()), "a tile's code words did not change"
    progress(f"{name} exactly-once: every tile changed")
    restore()
    state.step(p, g, 4)
    torch.cuda.synchronize()
    for t, ref in zip([p] + [getattr(state, k) for k in names], whole):
        assert torch.equal(t, ref), "the step is not reproducible"
    progress(f"{name} exactly-once: reproducible")
    # the same step in unequal pieces
    restore()
    rng = np.random.default_rng(5)
    units = n // PIECE
    cuts = sorted(set([0, units] + [int(x) for x in rng.integers(1, units, 12)] +
                      [int(x) for x in (units // 3 + np.array([1, 3, 4, 9, 12, 100, 1000, 5000]))]))
    cuts = [PIECE * x for x in cuts]
    if n % PIECE:
        cuts[-1] = n
    for a, b in zip(cuts[:-1], cuts[1:]):
        cfg = solo.make_config(w.bits_m, w.bits_v, B, solo.SOLO_GRAD_BF16, lr=w.lr, beta1=w.beta1, beta2=w.beta2,
                               eps=w.eps, weight_decay=w.weight_decay, quantile_p=w.quantile_p, index_offset=a)
        v = DeviceView.of(p, state, a, b - a)
        solo.solo_adamw_step(v.p, g[a:b], v.m_codes, v.m_scale, v.v_codes, v.v_scale, v.v_base, b - a, 4, cfg)
    torch.cuda.synchronize()
    for t, ref, k in zip([p] + [getattr(state, k) for k in names], whole, ("p",) + names):
        assert torch.equal(t, ref), f"{k}: the step in {len(cuts) - 1} pieces differs from the step of the whole buffer"
    note(f"{name} at full size: constant-gradient closed form on all {n // B} blocks, every one of {nt} tiles changed, "
         f"step reproducible, and equal bit for bit to the same step in {len(cuts) - 1} pieces "
         f"(sizes {min(b - a for a, b in zip(cuts[:-1], cuts[1:]))} .. {max(b - a for a, b in zip(cuts[:-1], cuts[1:]))})")


# ------------------------------------------------------- sparse embedding rows (Sec. 3.2.2)

@pytest.mark.parametrize("launch", ("flat", "table"))
def test_config5_sparse_embedding_rows(so, gpu, launch):
    """2048 rows of the LLaMA embedding (4096 wide): every step, 90 % of the rows (drawn afresh)
    receive no gradient, the case Sec. 3.2.2 raises for the adaptive base: their v^ = beta2 v~
    sit on at most eight distinct values per block (every extraction round of the quantile is
    a tie), blocks go to and come from the zero state, x_p = 0 blocks clamp the base.  Ten
    teacher-forced and ten free-running steps, every element.  The flat buffer (8.4 M elements)
    runs one wavefront per 512 elements; as a table of one tensor it runs the streaming kernel
    of the metric's format, 16 elements per lane."""
    from paper_2505_00347_amd import synth
    from test_gpu_parity import GpuSide
    solo = gpu
    w = synth.workload("c5_sparse_embed")
    rows, row_len = 2048, 4096
    n = rows * row_len
    oc, gc = workload_cfgs(so, solo, w)
    p = synth.make_params(n)
    st = so.State(n, oc)
    multi = launch == "table"
    tf, fr = GpuSide(solo, n, gc, multi=multi), GpuSide(solo, n, gc, multi=multi)
    fr.p = dev(p)
    tainted = np.zeros(st.m_scale.size, bool)
    flips_tf = flips_fr = 0
    idle_seen = 0
    for step in range(1, 11):
        g = synth.make_grads(n, w.grad_kind, w.grad_std, synth.seed_grad(w.config_id, step))
        idle = synth.zero_row_mask(rows, 0.9, synth.seed_grad(w.config_id, step))
        g.reshape(rows, row_len)[idle] = 0
        idle_seen += int(idle.sum())
        bits, g = synth.round_to_bf16(g)
        g_dev = dev(bits)
        tf.load(p, st)
        tf.step(g_dev, step)
        fr.step(g_dev, step)
        p_before = p.astype(np.float64)
        margin = so.step_packed(p, g, st, step, oc, want_margin=True, threads=THREADS)
        flips_tf += compare_step(so, oc, n, p, st, margin, tf.fetch(), 1e-6, 2e-6 * oc.lr, p_before=p_before)
        flips_fr += compare_step(so, oc, n, p, st, margin, fr.fetch(), 1e-5, 1e-5 * oc.lr, tainted)
    zero_blocks = int((st.v_scale == 0).sum())
    note(f"c5 sparse embedding rows, {launch} ({rows} x {row_len}, {idle_seen / (10 * rows):.0%} of the rows idle per step): "
         f"teacher-forced {flips_tf} flips, free-running {flips_fr} flips, {int(tainted.sum())} blocks diverged; "
         f"{zero_blocks} of {st.v_scale.size} blocks still in the zero state after 10 steps")
    assert flips_tf <= flip_budget(10 * n) and flips_fr <= flip_budget(10 * n)
