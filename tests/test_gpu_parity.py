"""GPU parity: the HIP library (through its C-ABI) against the CPU oracle, element by element,
on sizes the oracle finishes in seconds: every format, ragged sizes, degenerate blocks, the step
variants, many tensors in one launch, randomized sweeps.  The bar is stated in parity_common.py;
the named configurations at their full sizes are in test_gpu_protocol.py.
"""
import numpy as np
import pytest

from parity_common import (TILE, FLIP_MARGIN, FLIP_RATE, flip_budget, flip_allowance, dev, host_words,
                           make_cfgs, bits_equal, compare_step, note)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2505_00347_amd import solo
    solo.lib()                       # fails loudly if the library is not built
    return solo


class GpuSide:
    """Device copy of (param, state) plus the C-ABI calls."""

    def __init__(self, solo, n, cfg, grad_scale=None, bf16_copy=False, multi=False):
        import torch
        self.solo, self.n, self.cfg = solo, n, cfg
        # multi: the buffer goes through solo_adamw_step_multi as a table of one tensor, which runs
        # the streaming kernels on its full units whatever the size (a flat buffer of a test's
        # size runs one wavefront per 512 elements)
        self.multi = multi
        self.state = solo.SoloState(n, cfg)
        self.p = None
        self.grad_scale = None if grad_scale is None else torch.tensor([grad_scale], dtype=torch.float32,
                                                                       device="cuda")
        # poisoned, so that an element the kernel skips shows
        self.p_bf16 = torch.full((n,), float("nan"), dtype=torch.bfloat16, device="cuda") if bf16_copy else None

    def load(self, p, st):
        self.p = dev(p)
        s = self.state
        s.m_codes.copy_(dev(st.m_words)); s.v_codes.copy_(dev(st.v_words))
        s.m_scale.copy_(dev(st.m_scale)); s.v_scale.copy_(dev(st.v_scale)); s.v_base.copy_(dev(st.v_base))

    def step(self, g_dev, step):
        if self.multi:
            table = self.solo.SoloMultiTable([(self.p, g_dev, self.state, self.p_bf16)], self.cfg)
            table.step(step, grad_scale=self.grad_scale)
            return
        self.state.step(self.p, g_dev, step, param_bf16=self.p_bf16, grad_scale=self.grad_scale)

    def check_bf16_copy(self, so):
        """The 16-bit copy is the kernel's own new parameter rounded to nearest-even, bit for bit."""
        import torch
        if self.p_bf16 is None:
            return
        torch.cuda.synchronize()
        got = self.p_bf16.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, so.round_bf16(self.p.cpu().numpy())), "bf16 copy differs"

    def fetch(self):
        import torch
        torch.cuda.synchronize()
        s = self.state
        return (self.p.cpu().numpy(), host_words(s.m_codes), s.m_scale.cpu().numpy(),
                host_words(s.v_codes), s.v_scale.cpu().numpy(), s.v_base.cpu().numpy())


def grads_for(kind, n, std, seed, bf16):
    from paper_2505_00347_amd import synth
    g = synth.make_grads(n, kind, std, seed)
    if bf16:
        bits, g = synth.round_to_bf16(g)
        return g, dev(bits)
    return g, dev(g)


def run_teacher_forced(so, solo, n, bm, bv, B, bf16=False, steps=3, kind="normal", std=1e-3,
                       seed0=100, bf16_copy=False, multi=False, **kw):
    from paper_2505_00347_amd import synth
    oc, gc = make_cfgs(so, solo, bm, bv, B, bf16, **kw)
    p = synth.make_params(n)
    st = so.State(n, oc)
    side = GpuSide(solo, n, gc, kw.get("grad_scale"), bf16_copy, multi)
    flips = 0
    for step in range(1, steps + 1):
        g, g_dev = grads_for(kind, n, std, seed0 + step, bf16)
        side.load(p, st)
        side.step(g_dev, step)
        p_before = p.astype(np.float64)
        margin = so.step_packed(p, g, st, step, oc, want_margin=True, threads=8)
        flips += compare_step(so, oc, n, p, st, margin, side.fetch(), 1e-6, 2e-6 * oc.lr, p_before=p_before)
        side.check_bf16_copy(so)
    assert flips <= flip_budget(n * steps), f"{flips} flips in {n * steps} codes"
    return flips


def run_free(so, solo, n, bm, bv, B, bf16=False, steps=10, kind="normal", std=1e-3, seed0=100,
             bf16_copy=False, multi=False, **kw):
    from paper_2505_00347_amd import synth
    oc, gc = make_cfgs(so, solo, bm, bv, B, bf16, **kw)
    p = synth.make_params(n)
    st = so.State(n, oc)
    side = GpuSide(solo, n, gc, kw.get("grad_scale"), bf16_copy, multi)
    side.p = dev(p)
    got = side.fetch()                       # solo_state_init against the oracle's zero state
    assert np.array_equal(got[1], st.m_words) and np.array_equal(got[3], st.v_words)
    assert bits_equal(got[2], st.m_scale) and bits_equal(got[4], st.v_scale) and bits_equal(got[5], st.v_base)
    tainted = np.zeros(st.m_scale.size, bool)
    flips = 0
    for step in range(1, steps + 1):
        g, g_dev = grads_for(kind, n, std, seed0 + step, bf16)
        side.step(g_dev, step)
        margin = so.step_packed(p, g, st, step, oc, want_margin=True, threads=8)
        got = side.fetch()
        flips += compare_step(so, oc, n, p, st, margin, got, 1e-5, 1e-5 * oc.lr, tainted)
        side.check_bf16_copy(so)
        if kw.get("optimizer") == "adam_l2":
            # coupled decay feeds the parameter back into both EMAs: the last-bit differences of
            # the two parameter updates would leak into the states, so the oracle continues from
            # the kernel's parameters (the states stay free-running)
            p[:] = got[0]
    assert flips <= flip_budget(n * steps), f"{flips} flips in {n * steps} codes"
    assert tainted.mean() <= max(2.0 / tainted.size, 2 * FLIP_RATE * B * steps)
    return flips, int(tainted.sum())


# ------------------------------------------------------------ the named configs

def test_config1_4bit_normal_ten_steps(so, gpu):
    """2^20 parameters, 4-bit m + 4-bit log v, block 128, beta1 0.8, N(0,1e-3) gradients."""
    run_teacher_forced(so, gpu, 1 << 20, 4, 4, 128, steps=10, seed0=1000)
    flips, tainted = run_free(so, gpu, 1 << 20, 4, 4, 128, steps=10, seed0=1000)
    print(f"config 1 free-running: {flips} flips, {tainted} blocks diverged")


def test_config2_3bit_student_t_ten_steps(so, gpu):
    """Same tensor, 3-bit states (ten codes per word), heavy-tailed Student-t(3) gradients."""
    run_teacher_forced(so, gpu, 1 << 20, 3, 3, 128, steps=10, kind="student_t3", seed0=2000)
    flips, tainted = run_free(so, gpu, 1 << 20, 3, 3, 128, steps=10, kind="student_t3", seed0=2000)
    print(f"config 2 free-running: {flips} flips, {tainted} blocks diverged")


def test_config3_shape_2bit_block64(so, gpu):
    """GPT-2-125M-shaped: a slice of a matrix plus LayerNorm-sized vectors (768), 2-bit, B=64."""
    run_teacher_forced(so, gpu, 768 * 2304 // 4, 2, 2, 64, steps=4, seed0=3000)
    run_free(so, gpu, 768, 2, 2, 64, steps=10, seed0=3100)           # a LayerNorm vector
    run_free(so, gpu, 50257 * 8, 2, 2, 64, steps=5, seed0=3200)      # odd vocabulary rows: ragged tail


def test_config4_shape_3bit_bf16_outliers(so, gpu):
    """1.3B-shaped slice: bf16 gradients N(0,1e-4) with 1 % outliers x100, 3-bit, B=128."""
    run_teacher_forced(so, gpu, 2048 * 1024, 3, 3, 128, bf16=True, steps=4, kind="normal_outliers",
                       std=1e-4, seed0=4000)
    run_free(so, gpu, 2048 * 256 + 2048, 3, 3, 128, bf16=True, steps=10, kind="normal_outliers",
             std=1e-4, seed0=4100)


def test_config5_shape_2bit_m_3bit_v_bf16(so, gpu):
    """LLaMA-7B-shaped slice: 2-bit m, 3-bit log v, bf16 gradients, B=128."""
    run_teacher_forced(so, gpu, 4096 * 1024, 2, 3, 128, bf16=True, steps=4, kind="normal_outliers",
                       std=1e-4, seed0=5000)
    run_free(so, gpu, 4096 * 96 + 4096, 2, 3, 128, bf16=True, steps=10, kind="normal_outliers",
             std=1e-4, seed0=5100)


# ------------------------------------- the paper's own variants: dynamic-exponent 1st moment

def test_paper_4_2bit_adamw_de_first_moment(so, gpu):
    """SOLO 4/2-bit AdamW (Sec. 3.4): 4-bit signed dynamic-exponent m with beta1 = 0.8,
    2-bit logarithmic v, block 128."""
    run_teacher_forced(so, gpu, 1 << 20, 4, 2, 128, steps=6, seed0=6000, de=True, beta1=0.8)
    flips, tainted = run_free(so, gpu, 1 << 19, 4, 2, 128, steps=10, seed0=6100, de=True, beta1=0.8)
    print(f"4/2-bit free-running: {flips} flips, {tainted} blocks diverged")


def test_paper_2bit_adamw_de_first_moment(so, gpu):
    """SOLO 2-bit AdamW (Sec. 3.4): 2-bit signed dynamic-exponent m with beta1 = 0.5 (0.1 from
    scratch), 2-bit logarithmic v."""
    run_teacher_forced(so, gpu, 1 << 20, 2, 2, 128, steps=6, seed0=6200, de=True, beta1=0.5, bf16=True, std=1e-4,
                       kind="normal_outliers")
    run_free(so, gpu, 1 << 19, 2, 2, 128, steps=10, seed0=6300, de=True, beta1=0.1)


@pytest.mark.parametrize("bm", (2, 3, 4))
def test_dynamic_exponent_all_formats(so, gpu, bm):
    for bv, B, bf16, n in ((3, 128, False, 3 * TILE + 777), (4, 64, True, 2 * TILE + 1283), (2, 64, False, 641)):
        run_teacher_forced(so, gpu, n, bm, bv, B, bf16=bf16, steps=4, seed0=50 + bm, de=True)


# ------------------------------------------------------ every format, ragged sizes

@pytest.mark.parametrize("bm", (2, 3, 4))
@pytest.mark.parametrize("bv", (2, 3, 4))
def test_all_formats(so, gpu, bm, bv):
    for B, bf16, n in ((128, False, 3 * TILE + 777), (64, True, 2 * TILE + 1283)):
        run_teacher_forced(so, gpu, n, bm, bv, B, bf16=bf16, steps=3, seed0=7 * bm + bv)


@pytest.mark.parametrize("bm", (2, 3, 4))
@pytest.mark.parametrize("bv", (2, 3, 4))
def test_streaming_kernels_all_formats(so, gpu, bm, bv):
    """The kernels that own a whole super-tile per wavefront (8 or 16 elements per lane, chosen by
    the format) serve flat buffers only from 2^25 elements on; through a table of one tensor they
    run at any size.  Every format, both block sizes, both codebooks with bf16 gradients, the
    dynamic-exponent codebook with fp32 gradients, plain and with every extra: several super-tiles
    and a ragged end."""
    n = 3 * TILE + 2 * 2560 + 1283
    for B in (128, 64):
        for de, bf16 in ((False, True), (True, True), (True, False)):
            run_teacher_forced(so, gpu, n, bm, bv, B, bf16=bf16, steps=3, seed0=300 + 10 * bm + bv + B, de=de, multi=True,
                               kind="normal_outliers" if bf16 else "student_t3", std=1e-4 if bf16 else 1e-3)
    run_teacher_forced(so, gpu, n, bm, bv, 128, bf16=True, steps=3, seed0=400 + 10 * bm + bv, multi=True,
                       optimizer="adam_l2", grad_scale=0.25, bf16_copy=True, wd=0.1)


WIDE_FORMATS = [(bm, bv, 128, de) for de in (False, True)
                for bm, bv in ((2, 2), (2, 3), (2, 4), (3, 2), (3, 3), (4, 2))] + \
               [(bm, bv, 64, de) for de in (False, True) for bm, bv in ((2, 2), (2, 3), (3, 2))]


@pytest.mark.parametrize("bm,bv,B,de", WIDE_FORMATS)
def test_wide_path_formats(so, gpu, bm, bv, B, de):
    """The formats whose full super-tiles run 16 elements per lane (8 lanes per 128-element
    block, 4 per 64-element block): both gradient types, the plain step and the one with every
    extra, four full tiles and a ragged end (which runs the 8-elements-per-lane code on the same
    state).  A flat buffer reaches these kernels only from 2^25 elements on, so the buffer goes in
    as a table of one tensor, whose full units run them at any size (fp32 gradients with the linear
    codebook have no such kernels in use: their flat and multi-tensor launches run one wavefront
    per 512 elements, which the flat call here covers)."""
    n = 4 * TILE + 3000
    for bf16 in (True, False):
        multi = bf16 or de
        run_teacher_forced(so, gpu, n, bm, bv, B, bf16=bf16, steps=3, seed0=900 + 10 * bm + bv, de=de, multi=multi,
                           std=1e-4 if bf16 else 1e-3, kind="normal_outliers" if bf16 else "student_t3")
        run_free(so, gpu, n, bm, bv, B, bf16=bf16, steps=5, seed0=950 + 10 * bm + bv, de=de, multi=multi,
                 optimizer="adabelief", grad_scale=0.5, bf16_copy=True, eps=1e-12)


# ------------------------------------------------- variants of the step (one fused pass each)

@pytest.mark.parametrize("optimizer", ("adamw", "adam_l2", "adabelief"))
@pytest.mark.parametrize("bm,bv,B,bf16,de", [(2, 3, 128, True, False), (4, 2, 128, True, True),
                                             (3, 3, 64, False, False), (4, 4, 128, False, False)])
def test_step_variants(so, gpu, optimizer, bm, bv, B, bf16, de):
    """Coupled decay, AdaBelief, a gradient scale read from device memory and the bf16 weight
    copy, together, over several super-tiles and a ragged tail."""
    n = 5 * TILE + 1234
    kw = dict(optimizer=optimizer, grad_scale=1.0 / 1024, wd=0.1, de=de, bf16_copy=True,
              eps=1e-12 if optimizer == "adabelief" else 1e-8, std=1.024)
    run_teacher_forced(so, gpu, n, bm, bv, B, bf16, steps=3, **kw)
    run_free(so, gpu, n, bm, bv, B, bf16, steps=10, **kw)


def test_bf16_copy_alone_and_scale_alone(so, gpu):
    n = 3 * TILE + 77
    run_teacher_forced(so, gpu, n, 2, 3, 128, True, steps=2, bf16_copy=True)
    run_teacher_forced(so, gpu, n, 2, 3, 128, True, steps=2, grad_scale=0.37, std=3e-3)
    run_teacher_forced(so, gpu, n, 4, 4, 64, False, steps=2, grad_scale=1.0, optimizer="adabelief")


def test_variants_reject_misaligned_extras(gpu):
    import torch
    n = 2560
    cfg = gpu.make_config(bits_m=2, bits_v=3)
    st = gpu.SoloState(n, cfg)
    p = torch.zeros(n, device="cuda")
    g = torch.zeros(n, device="cuda")
    h = torch.zeros(n + 8, dtype=torch.bfloat16, device="cuda")
    s = torch.ones(4, device="cuda")
    bad_h = h.data_ptr() + 2
    bad_s = s.data_ptr() + 2
    assert gpu.solo_adamw_step_mp(p, bad_h, g, None, *st.buffers(), n, 1, cfg, check=False) == gpu.SOLO_E_INVALID
    assert gpu.solo_adamw_step_mp(p, None, g, bad_s, *st.buffers(), n, 1, cfg, check=False) == gpu.SOLO_E_INVALID
    assert gpu.solo_adamw_step_mp(p, h, g, s, *st.buffers(), n, 1, cfg, check=False) == gpu.SOLO_OK
    torch.cuda.synchronize()


@pytest.mark.parametrize("n", (1, 7, 8, 9, 63, 64, 65, 127, 128, 129, 641, 2559, 2560, 2561, 5119, 5120, 5121, 7681, 10240, 15361))
def test_ragged_sizes(so, gpu, n):
    run_free(so, gpu, n, 2, 3, 128, bf16=True, steps=3, std=1e-4, seed0=n)
    run_free(so, gpu, n, 3, 4, 64, steps=3, seed0=n + 1)


def test_quantile_settings_and_nearest_rounding(so, gpu):
    n = 4 * TILE + 300
    for p in (0.0, 0.05, 0.3, 0.5):
        run_teacher_forced(so, gpu, n, 4, 2, 128, steps=3, p=p, seed0=int(p * 100))
        run_teacher_forced(so, gpu, n, 2, 3, 64, steps=3, p=p, seed0=int(p * 100) + 1)
    run_teacher_forced(so, gpu, n, 3, 3, 128, steps=4, stochastic=0, seed0=77)
    run_free(so, gpu, n, 2, 4, 128, steps=6, stochastic=0, seed0=78)
    # the same on the streaming kernels (a table of one tensor): 16 and 8 elements per lane
    for p in (0.0, 0.05, 0.3, 0.5, 0.95):
        run_teacher_forced(so, gpu, n, 2, 3, 128, bf16=True, steps=3, p=p, seed0=int(p * 100) + 2, multi=True, std=1e-4)
        run_teacher_forced(so, gpu, n, 4, 4, 64, bf16=True, steps=3, p=p, seed0=int(p * 100) + 3, multi=True, de=True)
    run_free(so, gpu, n, 3, 3, 128, bf16=True, steps=6, stochastic=0, seed0=79, multi=True)


def test_index_offset_and_seed(so, gpu):
    run_teacher_forced(so, gpu, 6000, 2, 3, 128, steps=3, off=8 * (1 << 33) + 2560 * 7, seed=123456789)
    run_teacher_forced(so, gpu, 6000, 4, 4, 64, steps=3, off=8, seed=0)
    # the streaming kernels (a table of one tensor), with an offset whose group index crosses 2^32 inside the buffer
    run_teacher_forced(so, gpu, 3 * TILE + 100, 2, 3, 128, bf16=True, steps=3, off=8 * ((1 << 32) - 700), seed=987654321,
                       multi=True, std=1e-4)
    run_teacher_forced(so, gpu, 3 * TILE + 100, 2, 3, 2048, bf16=True, steps=3, off=8 * ((1 << 32) - 700), seed=5,
                       std=1e-4)


def test_hyperparameter_ranges(so, gpu):
    run_teacher_forced(so, gpu, 5000, 4, 4, 128, steps=3, beta1=0.0, beta2=0.0, lr=1e-2, wd=0.0, eps=1e-6)
    run_teacher_forced(so, gpu, 5000, 2, 2, 128, steps=3, beta1=0.1, beta2=0.98, lr=3e-4, wd=0.1)
    run_teacher_forced(so, gpu, 5000, 3, 3, 64, steps=3, std=30.0)            # large gradients
    run_teacher_forced(so, gpu, 5000, 3, 3, 64, steps=3, std=1e-9, bf16=True)  # tiny gradients
    for kw in (dict(beta1=0.0, beta2=0.0, lr=1e-2, wd=0.0, eps=1e-6), dict(beta1=0.1, beta2=0.98, lr=3e-4, wd=0.1),
               dict(std=30.0), dict(std=1e-9)):                                # the same on the streaming kernels
        run_teacher_forced(so, gpu, 2 * TILE + 5000, 2, 3, 128, bf16=True, steps=3, multi=True, **kw)


# ------------------------------------------------------------ degenerate inputs

def special_grads(n, B, seed):
    rng = np.random.default_rng(seed)
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    g[0 * B:1 * B] = 0                         # all-zero block
    g[1 * B:2 * B] = 2e-3                      # constant block
    g[2 * B:3 * B] = -2e-3
    g[3 * B + 5:4 * B] = 0                     # sparse block: x_p = 0
    g[4 * B:5 * B] = np.where(rng.random(B) < 0.5, 1e-3, -1e-3)   # equal magnitudes: all ties
    g[5 * B:6 * B] = 1e-18                     # underflows to the zero block
    g[6 * B:7 * B:2] = 0                       # half zeros
    return g


@pytest.mark.parametrize("eps", (1e-12, 1e-13))
def test_nearly_constant_blocks(so, gpu, eps):
    """AdaBelief whose eps dwarfs the squared residuals (gradients of 5e-8 after the scale): every
    v^ of a block lies within 1e-5 of eps, the base alpha within a few dozen ulps of 1, and the
    code of an element hangs on the last bit of v^/Delta.  Scales and bases still agree bit for
    bit, codes differ by at most one, and only within the margin flip_allowance grants."""
    kw = dict(de=True, optimizer="adabelief", p=0.02, eps=eps, grad_scale=1.0 / 1024, seed=146131703902,
              off=265625140904, kind="student_t3", std=5.4e-5)
    run_teacher_forced(so, gpu, 13899, 2, 3, 128, bf16=True, steps=3, seed0=358133, **kw)
    run_teacher_forced(so, gpu, 3 * TILE + 100, 4, 4, 64, bf16=False, steps=2, seed0=11, **kw)
    run_teacher_forced(so, gpu, 3 * TILE + 100, 2, 3, 128, bf16=True, steps=3, seed0=358134, multi=True, **kw)   # streaming kernels
    run_teacher_forced(so, gpu, 3 * TILE + 100, 4, 4, 64, bf16=False, steps=2, seed0=12, multi=True, **kw)


@pytest.mark.parametrize("bm,bv,B,bf16,de", [(2, 3, 128, False, False), (4, 4, 64, False, False),
                                              (3, 2, 128, True, False), (4, 2, 128, False, True),
                                              (2, 2, 64, True, True)])
@pytest.mark.parametrize("multi", (False, True))
def test_degenerate_blocks(so, gpu, bm, bv, B, bf16, de, multi):
    """Constant, zero and sparse blocks, an all-zero step, rows that stay idle.  multi: as a table
    of one tensor, two super-tiles longer, so that the streaming kernels (or, with fp32 gradients
    and the linear codebook, the multi-tensor form of the one-wavefront-per-512 kernels) see them."""
    from paper_2505_00347_amd import synth
    n = 24 * B + 11 + (2 * TILE if multi else 0)
    oc, gc = make_cfgs(so, gpu, bm, bv, B, bf16, de=de)
    p = synth.make_params(n)
    st = so.State(n, oc)
    side = GpuSide(gpu, n, gc, multi=multi)
    for step in range(1, 9):
        g = special_grads(n, B, step) if step != 5 else np.zeros(n, np.float32)   # one all-zero step
        if step in (6, 7):
            g[: 8 * B] = 0                                                         # rows that stay idle
        if bf16:
            bits, g = synth.round_to_bf16(g)
            g_dev = dev(bits)
        else:
            g_dev = dev(g)
        side.load(p, st)
        side.step(g_dev, step)
        margin = so.step_packed(p, g, st, step, oc, want_margin=True)
        compare_step(so, oc, n, p, st, margin, side.fetch(), 1e-6, 2e-6 * oc.lr)
        assert np.all(np.isfinite(p))


def test_empty_and_invalid_arguments(gpu):
    import torch
    solo = gpu
    cfg = solo.make_config(2, 3, 128, 1)
    p = torch.zeros(2560, device="cuda")
    g = torch.zeros(2560, device="cuda", dtype=torch.bfloat16)
    st = solo.SoloState(2560, cfg)
    args = (p, g, *st.buffers())
    assert solo.solo_adamw_step(*args, 0, 1, cfg, check=False) == solo.SOLO_OK          # n = 0
    assert solo.solo_adamw_step(*args, 2560, 0, cfg, check=False) == solo.SOLO_E_INVALID  # step 0
    assert solo.solo_adamw_step(p.data_ptr() + 4, g, *st.buffers(), 2560, 1, cfg, check=False) == solo.SOLO_E_INVALID
    assert solo.solo_adamw_step(0, g, *st.buffers(), 2560, 1, cfg, check=False) == solo.SOLO_E_INVALID
    for field, value in (("bits_m", 5), ("bits_v", 1), ("block_size", 96), ("grad_dtype", 2),
                         ("beta1", 1.0), ("beta2", -0.1), ("quantile_p", 1.0), ("eps", -1.0),
                         ("flags", 16), ("reserved", 1), ("index_offset", 4), ("lr", float("nan"))):
        bad = solo.make_config(2, 3, 128, 1)
        setattr(bad, field, value)
        assert solo.solo_adamw_step(*args, 2560, 1, bad, check=False) == solo.SOLO_E_INVALID, field
        assert solo.solo_state_init(*st.buffers(), 2560, bad, check=False) == solo.SOLO_E_INVALID, field
    torch.cuda.synchronize()
    assert torch.all(p == 0)                                # nothing was enqueued by the failed calls
    with pytest.raises(solo.SoloError):
        solo.solo_adamw_step(*args, 2560, 0, cfg)


def test_state_region_allocates_and_returns_its_spacer(gpu):
    """The placement helper of the binding: inside it the state is allocated behind a spacer that
    fills the first 96 GiB of the process's allocations; the spacer goes back to the driver on
    exit, the state stays usable."""
    import torch
    solo = gpu
    cfg = solo.make_config(2, 3, 128, 1)
    n = 1 << 20
    p = torch.zeros(n, device="cuda")
    g = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    free0 = torch.cuda.mem_get_info()[0]
    with solo.state_region(6 * n) as region:
        had_spacer = region.spacer is not None
        assert had_spacer == (free0 > solo.HBM_REGION_BYTES + (8 << 30))
        if had_spacer:
            assert torch.cuda.mem_get_info()[0] < free0 - (90 << 30)
        st = solo.SoloState(n, cfg)
    assert region.spacer is None
    assert torch.cuda.mem_get_info()[0] > free0 - (1 << 30)          # only the state (and torch's block for it) is left
    st.step(p, g, 1)
    torch.cuda.synchronize()
    assert bool((st.v_scale == 0).all())                             # zero gradients: the zero state stays


def test_runs_on_the_callers_stream(so, gpu):
    import torch
    from paper_2505_00347_amd import synth
    n = 3 * TILE + 100
    oc, gc = make_cfgs(so, gpu, 4, 4, 128)
    p = synth.make_params(n)
    g = synth.make_grads(n, "normal", 1e-3, 5)
    st = so.State(n, oc)
    side = GpuSide(gpu, n, gc)
    side.load(p, st)
    g_dev = dev(g)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        side.state.step(side.p, g_dev, 1)          # binding picks up the current stream
    s.synchronize()
    margin = so.step_packed(p, g, st, 1, oc, want_margin=True)
    compare_step(so, oc, n, p, st, margin, side.fetch(), 1e-6, 2e-6 * oc.lr)


@pytest.mark.parametrize("B", (128, 2048))
def test_step_can_be_captured_in_a_hip_graph(so, gpu, B):
    """The library allocates nothing, synchronises nothing and enqueues only kernels (two for a
    buffer with a ragged end), so a step can be recorded into a HIP graph.  The replayed step
    (same step number, inputs restored by eager copies between the replays) must reproduce the
    eager step bit for bit, every time."""
    import torch
    from paper_2505_00347_amd import synth
    solo = gpu
    n = 3 * TILE + 777
    _, gc = make_cfgs(so, solo, 2, 3, B, True)
    p0 = dev(synth.make_params(n))
    g_host, g = grads_for("normal", n, 1e-3, 4242, True)
    st = solo.SoloState(n, gc)
    for step in (1, 2):                                   # a non-trivial state to start from
        st.step(p0, g, step)
    torch.cuda.synchronize()
    init = [t.clone() for t in (p0, *st.buffers())]

    def restore():
        for dst, src in zip((p0, *st.buffers()), init):
            dst.copy_(src)

    st.step(p0, g, 3)                                     # eager result of step 3
    torch.cuda.synchronize()
    want = [t.clone() for t in (p0, *st.buffers())]

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    restore()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        graph.capture_begin()
        st.step(p0, g, 3)                                 # launches on the capturing (current) stream
        graph.capture_end()
    torch.cuda.synchronize()
    for _ in range(3):
        restore()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((p0, *st.buffers()), want):
            assert torch.equal(got, ref)


# --------------------------- blocks of 2048 elements (the large-block setting of Sec. 4.2)

@pytest.mark.parametrize("bm", (2, 3, 4))
@pytest.mark.parametrize("bv", (2, 3, 4))
def test_block_2048_all_formats(so, gpu, bm, bv):
    """One workgroup per block: maxima across four wavefronts, the quantile (rank 205 of 2048) by
    radix select.  Every format, both gradient types and codebooks, full blocks and a ragged end."""
    for bf16, n, de in ((False, 5 * 2048 + 777, False), (True, 3 * 2048, True), (True, 11 * 2048 + 1283, False)):
        run_teacher_forced(so, gpu, n, bm, bv, 2048, bf16=bf16, steps=3, seed0=40 + 7 * bm + bv, de=de,
                           std=1e-4 if bf16 else 1e-3, kind="normal_outliers" if bf16 else "student_t3")


@pytest.mark.parametrize("n", (1, 7, 8, 511, 512, 513, 1023, 2047, 2048, 2049, 2560, 4095, 4097, 6143, 20481))
def test_block_2048_ragged_sizes(so, gpu, n):
    run_free(so, gpu, n, 2, 3, 2048, bf16=True, steps=3, std=1e-4, seed0=n)
    run_free(so, gpu, n, 3, 4, 2048, steps=3, seed0=n + 1)


def test_block_2048_quantile_settings_variants_and_degenerate_blocks(so, gpu):
    n = 9 * 2048 + 300
    for p in (0.0, 0.02, 0.3, 0.5, 0.95):
        run_teacher_forced(so, gpu, n, 4, 2, 2048, steps=3, p=p, seed0=int(p * 100))
        run_teacher_forced(so, gpu, n, 2, 3, 2048, steps=3, p=p, seed0=int(p * 100) + 1, bf16=True, std=1e-4)
    run_teacher_forced(so, gpu, n, 3, 3, 2048, steps=4, stochastic=0, seed0=77)
    for optimizer in ("adam_l2", "adabelief"):
        kw = dict(optimizer=optimizer, grad_scale=1.0 / 1024, wd=0.1, bf16_copy=True,
                  eps=1e-12 if optimizer == "adabelief" else 1e-8, std=1.024)
        run_teacher_forced(so, gpu, n, 2, 3, 2048, True, steps=3, **kw)
        run_free(so, gpu, n, 4, 2, 2048, True, steps=6, de=True, **kw)
    run_teacher_forced(so, gpu, 6000, 2, 3, 2048, steps=3, off=8 * (1 << 33) + 2560 * 7, seed=123456789)
    # constant blocks (every key equal: the radix select walks one bin per pass), zero blocks, sparse blocks
    from paper_2505_00347_amd import synth
    B = 2048
    nn = 12 * B + 11
    oc, gc = make_cfgs(so, gpu, 2, 3, B, True)
    p = synth.make_params(nn)
    st = so.State(nn, oc)
    side = GpuSide(gpu, nn, gc)
    for step in range(1, 7):
        g = special_grads(nn, B, step) if step != 4 else np.zeros(nn, np.float32)
        bits, g = synth.round_to_bf16(g)
        side.load(p, st)
        side.step(dev(bits), step)
        margin = so.step_packed(p, g, st, step, oc, want_margin=True)
        compare_step(so, oc, nn, p, st, margin, side.fetch(), 1e-6, 2e-6 * oc.lr)


def test_block_2048_config5_shape_ten_steps(so, gpu):
    """The metric's format with blocks of 2048 on a LLaMA-7B-shaped slice: ten teacher-forced and
    ten free-running steps."""
    run_teacher_forced(so, gpu, 4096 * 512, 2, 3, 2048, bf16=True, steps=10, kind="normal_outliers", std=1e-4, seed0=8000)
    flips, tainted = run_free(so, gpu, 4096 * 512 + 4096, 2, 3, 2048, bf16=True, steps=10, kind="normal_outliers",
                              std=1e-4, seed0=8100)
    note(f"block 2048, config-5 format, 2.1 M elements x 10 free-running steps: {flips} flips, {tainted} blocks diverged")


@pytest.mark.parametrize("B,bm,bv,multi", ((2048, 2, 3, False), (2048, 4, 2, False), (128, 2, 3, False),
                                             (128, 2, 3, True), (2048, 2, 3, True)))
def test_trained_state_with_clustered_second_moments(so, gpu, B, bm, bv, multi):
    """After some hundred updates the second moments of a block sit in a few tight clusters (beta2
    times one of the 2^b decoded levels, plus a small fresh term): most keys of the quantile
    selection then share their leading bits, the case the histograms of the large-block kernels
    are laid out for.  300 steps on the GPU alone, then three steps compared with the oracle,
    each starting from the GPU's own state."""
    import torch
    from paper_2505_00347_amd import synth
    from parity_common import DeviceView
    n = 40 * 2048 + 1283
    oc, gc = make_cfgs(so, gpu, bm, bv, B, True)
    side = GpuSide(gpu, n, gc, multi=multi)              # multi: a table of one tensor (the streaming kernels for B = 128)
    side.p = dev(synth.make_params(n))
    grads = [grads_for("normal_outliers", n, 1e-4, 5000 + k, True) for k in range(8)]
    for step in range(1, 301):
        side.step(grads[step % 8][1], step)
    view = DeviceView.of(side.p, side.state)
    flips = 0
    for step in range(301, 304):
        torch.cuda.synchronize()
        p = side.p.cpu().numpy()
        st = view.to_host_state(so, oc)
        vc = so.unpack(st.v_words, n, bv)
        g, g_dev = grads[step % 8]
        side.step(g_dev, step)
        p_before = p.astype(np.float64)
        margin = so.step_packed(p, g, st, step, oc, want_margin=True, threads=8)
        flips += compare_step(so, oc, n, p, st, margin, side.fetch(), 1e-6, 2e-6 * oc.lr, p_before=p_before)
    assert flips <= flip_budget(3 * n)
    # the premise: the codes of the trained state use the levels of a block unevenly
    top = np.bincount(vc[:2048], minlength=1 << bv).max()
    assert top > 2 * 2048 // (1 << bv), "the trained state is not clustered"


@pytest.mark.parametrize("B,n,bm,bv", ((128, 70000, 2, 3), (64, 70000, 4, 4), (2048, 70000, 2, 3), (2048, 70000, 3, 3),
                                       (128, (1 << 25) + 3 * TILE + 17, 2, 3)))
def test_non_finite_gradients_stay_inside_their_blocks(so, gpu, B, n, bm, bv):
    """A NaN or an infinity in the gradient spoils its own block and nothing else: the step
    completes, and every block without such an entry equals the oracle's result for the same
    gradients with the bad entries removed.
    (The last case is large enough for the streaming kernels; the others run one wavefront per
    512 elements, or one workgroup per block of 2048.)"""
    import torch
    from paper_2505_00347_amd import synth
    oc, gc = make_cfgs(so, gpu, bm, bv, B, True)
    p = synth.make_params(n)
    st = so.State(n, oc)
    side = GpuSide(gpu, n, gc)
    rng = np.random.default_rng(B + bm)
    g1, _ = grads_for("normal", n, 1e-3, 9100, True)
    so.step_packed(p, g1, st, 1, oc, threads=8)            # a clean first step, so that the state is not the zero state
    side.load(p, st)
    g, _ = grads_for("normal", n, 1e-3, 9101, True)
    bad = rng.choice(n, 24, replace=False)
    dirty = g.copy()
    dirty[bad[:8]] = np.nan
    dirty[bad[8:16]] = np.inf
    dirty[bad[16:]] = -np.inf
    bits = (dirty.view(np.uint32) >> 16).astype(np.uint16)   # bf16 patterns of the (bf16-representable) values
    side.step(dev(bits), 2)
    torch.cuda.synchronize()
    got = side.fetch()
    p_before = p.astype(np.float64)
    margin = so.step_packed(p, g, st, 2, oc, want_margin=True, threads=8)   # the oracle sees the clean gradients
    spoiled = np.zeros(-(-n // B), bool)
    spoiled[bad // B] = True
    assert not np.isfinite(got[0][bad]).any()                # the parameters under the bad entries are lost
    tainted = spoiled.copy()
    flips = compare_step(so, oc, n, p, st, margin, got, 1e-6, 2e-6 * oc.lr, tainted, p_before=p_before)
    assert flips <= flip_budget(n) and (tainted & ~spoiled).sum() <= flips


# ------------------------------------------------------- many tensors in one launch

@pytest.mark.parametrize("bm,bv,B,bf16,de,optimizer,extras", [(2, 3, 128, True, False, "adamw", False),
                                                             (2, 3, 128, True, False, "adamw", True),
                                                             (4, 2, 128, True, True, "adamw", True),
                                                             (3, 3, 64, False, False, "adabelief", True),
                                                             (2, 2, 64, False, True, "adamw", True),
                                                             (4, 4, 128, False, False, "adam_l2", False),
                                                             (2, 3, 2048, True, False, "adamw", False),
                                                             (4, 2, 2048, True, True, "adabelief", True),
                                                             (3, 3, 2048, False, False, "adam_l2", True)])
def test_multi_tensor_step_equals_per_tensor_steps(so, gpu, bm, bv, B, bf16, de, optimizer, extras):
    """solo_adamw_step_multi over tensors of awkward sizes (empty, smaller than a block, one
    element past a unit, several units) against the oracle run on every tensor alone with the
    tensor's own xi offset; three steps from equal states, with and without the bf16 copy and the
    gradient scale."""
    import torch
    from paper_2505_00347_amd import synth
    solo = gpu
    sizes = [1, 127, 128, 0, 2559, 2560, 2561, 4096, 5000, 12800, 3 * 2560 + 1, 20017, 64]
    off0 = 8 * 1000
    scale = 0.5 if extras else 1.0
    kw = dict(optimizer=optimizer, de=de, off=off0, grad_scale=scale, eps=1e-12 if optimizer == "adabelief" else 1e-8)
    oc, gc = make_cfgs(so, solo, bm, bv, B, bf16, **kw)
    sides, ps, sts, offs = [], [], [], []
    unit0 = 0
    for k, n in enumerate(sizes):
        sides.append(GpuSide(solo, n, gc, None, extras))
        ps.append(synth.make_params(n, stream=k))
        cfg_k = so.make_config(bits_m=bm, bits_v=bv, block_size=B, beta1=oc.beta1, eps=oc.eps,
                               index_offset=off0 + 2560 * unit0, m_codebook=1 if de else 0,
                               optimizer=oc.optimizer, grad_scale=scale)
        offs.append(cfg_k)
        sts.append(so.State(n, cfg_k))
        unit0 += -(-n // 2560)
    gscale = torch.tensor([scale], dtype=torch.float32, device="cuda") if extras else None
    flips = 0
    for step in (1, 2, 3):
        gs = []
        for k, n in enumerate(sizes):
            g, g_dev = grads_for("normal", n, 2e-3, 700 + 10 * step + k, bf16)
            gs.append((g, g_dev))
            sides[k].load(ps[k], sts[k])
        items = [(sides[k].p, gs[k][1], sides[k].state, sides[k].p_bf16) for k in range(len(sizes))]
        table = solo.SoloMultiTable(items, gc)
        table.step(step, grad_scale=gscale)
        for k, n in enumerate(sizes):
            if n == 0:
                continue
            margin = so.step_packed(ps[k], gs[k][0], sts[k], step, offs[k], want_margin=True)
            flips += compare_step(so, offs[k], n, ps[k], sts[k], margin, sides[k].fetch(), 1e-6, 2e-6 * oc.lr)
            sides[k].check_bf16_copy(so)
    assert flips <= 2


def test_multi_tensor_table_rejects_bad_descriptors(gpu):
    import ctypes as C
    import torch
    solo = gpu
    cfg = solo.make_config(bits_m=2, bits_v=3, flags=solo.SOLO_FLAG_STOCHASTIC | solo.SOLO_FLAG_M_DYNAMIC_EXPONENT)
    n = 3000
    st = solo.SoloState(n, cfg)
    p = torch.zeros(n, device="cuda")
    g = torch.zeros(n, device="cuda")
    arr = (solo.solo_tensor * 1)()
    arr[0] = solo.solo_tensor(p.data_ptr(), None, g.data_ptr(), st.m_codes.data_ptr(), st.m_scale.data_ptr(),
                              st.v_codes.data_ptr(), st.v_scale.data_ptr(), st.v_base.data_ptr(), n)
    units = solo.solo_multi_units(arr, 1, cfg)
    assert units == 6                            # 3000 elements, all of them a ragged end: one unit per 512 elements
    # fp32 gradients with the linear codebook: units of 2560 elements, the shorter end included
    assert solo.solo_multi_units(arr, 1, solo.make_config(bits_m=2, bits_v=3)) == 2
    nbytes = solo.solo_multi_table_bytes(1, units)
    assert nbytes == 96 + 4 * units
    buf = (C.c_uint8 * nbytes)()
    assert solo.solo_multi_table_build(arr, 1, cfg, buf, nbytes, check=False) == (solo.SOLO_OK, 0)
    assert solo.solo_multi_table_build(arr, 1, cfg, buf, nbytes - 1, check=False)[0] == solo.SOLO_E_INVALID
    arr[0].param = p.data_ptr() + 4
    assert solo.solo_multi_table_build(arr, 1, cfg, buf, nbytes, check=False)[0] == solo.SOLO_E_INVALID
    arr[0].param = p.data_ptr()
    arr[0].m_scale = None
    assert solo.solo_multi_table_build(arr, 1, cfg, buf, nbytes, check=False)[0] == solo.SOLO_E_INVALID
    assert solo.solo_adamw_step_multi(0, 1, 2, 0, None, 1, cfg, check=False) == solo.SOLO_E_INVALID
    assert solo.solo_adamw_step_multi(0, 1, 0, 0, None, 1, cfg, check=False) == solo.SOLO_OK
    assert solo.solo_adamw_step_multi(p.data_ptr(), 1, 2, 0, None, 0, cfg, check=False) == solo.SOLO_E_INVALID


# ------------------------------------------------------------------- randomized sweep

def random_cases(so, gpu, seed, blocks, cases):
    """Seeded random combinations of format, block size, codebook, gradient type and distribution,
    optimizer, quantile, size (ragged ends included), hyper-parameters, xi on/off, stream position
    and extras, with gradient magnitudes from 1e-15 to 1e6: three steps each from equal states."""
    rng = np.random.default_rng(seed)
    for c in range(cases):
        bm, bv = int(rng.integers(2, 5)), int(rng.integers(2, 5))
        B = int(rng.choice(blocks))
        de, bf16 = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        opt = str(rng.choice(["adamw", "adamw", "adam_l2", "adabelief"]))
        n = int(rng.choice([rng.integers(1, 3000), rng.integers(3000, 40000),
                            TILE * int(rng.integers(1, 6)) + int(rng.integers(0, TILE))]))
        kind = str(rng.choice(["normal", "student_t3", "normal_outliers"]))
        std = float(10.0 ** rng.uniform(-15, 6)) if rng.integers(0, 3) == 0 else float(10.0 ** rng.uniform(-6, 0))
        kw = dict(de=de, optimizer=opt, p=float(rng.choice([0.0, 0.02, 0.1, 0.1, 0.25, 0.6, 0.95])),
                  stochastic=int(rng.integers(0, 4) > 0), seed=int(rng.integers(0, 2 ** 40)),
                  off=8 * int(rng.integers(0, 2 ** 36)), eps=1e-12 if opt == "adabelief" else 1e-8)
        if rng.integers(0, 2):
            kw.update(beta1=float(rng.choice([0.0, 0.1, 0.5, 0.9, 0.95])),
                      beta2=float(rng.choice([0.0, 0.9, 0.98, 0.999, 0.9999])),
                      lr=float(rng.choice([0.0, 1e-5, 1e-3, 1e-1])), wd=float(rng.choice([0.0, 0.01, 0.5])))
        if rng.integers(0, 2):
            kw.update(grad_scale=float(rng.choice([1.0, 0.5, 1.0 / 1024])), bf16_copy=True)
        try:
            # every other case as a table of one tensor (the streaming kernels on its full units)
            run_teacher_forced(so, gpu, n, bm, bv, B, bf16=bf16, steps=3, kind=kind, std=std,
                               seed0=int(rng.integers(0, 10 ** 6)), multi=c % 2 == 1, **kw)
        except AssertionError as e:
            raise AssertionError(f"case {c}: n={n} m{bm} v{bv} B{B} bf16={bf16} {kind} std={std:.3g} table={c % 2 == 1} {kw}: {e}") from e


@pytest.mark.parametrize("seed", (1, 2, 3))
def test_randomized_sweep(so, gpu, seed):
    """Forty random combinations per seed with blocks of 64 and 128 elements.  (Sweeps of this kind
    are what found the nearly-constant-block regime.)"""
    random_cases(so, gpu, seed, [64, 128], 40)


@pytest.mark.parametrize("seed", (11, 12))
def test_randomized_sweep_block_2048(so, gpu, seed):
    """Thirty random combinations per seed with blocks of 2048 elements."""
    random_cases(so, gpu, seed, [2048, 2048], 30)


# ---------------------------------- the benchmark's workload at its full size, sampled

@pytest.mark.parametrize("name,variant", [("c5_llama7b_2bit_3bit", "plain"), ("paper_4_2bit_llama7b", "mp"),
                                          ("c5_llama7b_block2048", "plain")])
def test_full_size_7b_workload_sampled_tiles(so, gpu, name, variant):
    """The LLaMA-7B-shaped workloads exactly as bench.py launches them (6,738,415,616 elements,
    one call): the metric's format, and the paper's own 4/2-bit format (dynamic-exponent m)
    through solo_adamw_step_mp with the bf16 weight copy and a gradient scale.  The oracle cannot
    run 6.7e9 elements in seconds, so the third step is checked on sampled 5120-element
    super-tiles (first, last full, the ragged tail, tensor boundaries and random ones; with blocks
    of 2048 elements, slices of five blocks): inputs of
    those slices are copied out before the step, the oracle runs on each slice with the slice's
    global offset, and every output byte of the slice is compared.  Properties that hold at any
    size are checked on the whole buffer."""
    import torch
    import bench
    from paper_2505_00347_amd import synth
    solo = gpu
    free, _ = torch.cuda.mem_get_info()
    w = synth.workload(name)
    n = w.n
    if free < 80 * 2 ** 30:
        pytest.skip("needs 80 GiB of free HBM")
    de = w.m_codebook == "de"
    mp = variant == "mp"
    scale = 0.25 if mp else None
    oc, gc = make_cfgs(so, solo, w.bits_m, w.bits_v, w.block_size, bf16=True, beta1=w.beta1, de=de,
                       grad_scale=scale, lr=w.lr)
    cm, cv, B = 32 // w.bits_m, 32 // w.bits_v, w.block_size
    p = bench.device_params(torch, w, synth.SEED_PARAM)
    state = solo.SoloState(n, gc)
    extras = {}
    if mp:
        extras = {"param_bf16": torch.full((n,), float("nan"), dtype=torch.bfloat16, device="cuda"),
                  "grad_scale": torch.tensor([scale], dtype=torch.float32, device="cuda")}
    gstd = w.grad_std / (scale or 1.0)
    for step in (1, 2):
        g = bench.device_grads(torch, n, w.grad_kind, gstd, synth.seed_grad(w.config_id, step), torch.bfloat16)
        state.step(p, g, step, **extras)
        del g
    g = bench.device_grads(torch, n, w.grad_kind, gstd, synth.seed_grad(w.config_id, 3), torch.bfloat16)
    T = TILE if B != 2048 else 5 * 2048          # slices start on a block and on a word of both streams
    n_tiles = n // T
    rng = np.random.default_rng(0)
    tiles = {0, 1, n_tiles - 1, n_tiles}                         # n_tiles = the ragged tail
    pos = 0
    for _, numel, _ in w.tensors[:12]:                           # tiles that straddle tensors
        pos += numel
        tiles.add(pos // T)
    tiles |= set(int(t) for t in rng.integers(0, n_tiles, 40))
    tiles = sorted(tiles)

    def state_slices(a, st):
        nb = st.m_scale.size
        return (host_words(state.m_codes[a // cm:a // cm + st.m_words.size]),
                state.m_scale[a // B:a // B + nb].cpu().numpy(),
                host_words(state.v_codes[a // cv:a // cv + st.v_words.size]),
                state.v_scale[a // B:a // B + nb].cpu().numpy(),
                state.v_base[a // B:a // B + nb].cpu().numpy())

    def grab(t):
        a, b = t * T, min(n, (t + 1) * T)
        cnt = b - a
        st = so.State(cnt, oc)
        st.m_words[:], st.m_scale[:], st.v_words[:], st.v_scale[:], st.v_base[:] = state_slices(a, st)
        return a, cnt, p[a:b].cpu().numpy(), g[a:b].float().cpu().numpy(), st

    before = [grab(t) for t in tiles]
    assert float(state.v_base.min()) > 0 and float(state.v_base.max()) <= 1
    state.step(p, g, 3, **extras)
    torch.cuda.synchronize()
    flips = 0
    for a, cnt, p0, g0, st in before:
        cfg_t = so.make_config(bits_m=w.bits_m, bits_v=w.bits_v, block_size=B, beta1=w.beta1, lr=w.lr,
                               index_offset=a, m_codebook=1 if de else 0, grad_scale=scale or 1.0)
        margin = so.step_packed(p0, g0, st, 3, cfg_t, want_margin=True)
        got = (p[a:a + cnt].cpu().numpy(),) + state_slices(a, st)
        flips += compare_step(so, oc, cnt, p0, st, margin, got, 1e-6, 2e-6 * oc.lr)
        if mp:
            h = extras["param_bf16"][a:a + cnt].view(torch.int16).cpu().numpy().view(np.uint16)
            assert np.array_equal(h, so.round_bf16(got[0])), "bf16 copy differs"
    assert flips <= 2
    # whole-buffer properties: codes in range, pad bits zero, scales finite and ordered
    vw, mw = state.v_codes, state.m_codes
    if w.bits_v == 3:
        assert int((vw >> 30).abs().max()) == 0                  # two pad bits of every 3-bit word
    if w.bits_m == 2 and not de:
        both = mw & (mw >> 1) & 0x55555555                       # a 2-bit field equal to 3 is never produced
        assert int(both.abs().max()) == 0
    assert bool(torch.isfinite(state.m_scale).all()) and bool(torch.isfinite(state.v_scale).all())
    K = 2 ** w.bits_v - 1
    assert float(state.v_base.min()) >= 2.0 ** (-64 / K) * (1 - 1e-6) and float(state.v_base.max()) <= 1
    assert bool(torch.isfinite(p).all())
    if mp:
        assert bool(torch.isfinite(extras["param_bf16"]).all())     # poisoned with NaN before the steps
