"""The C-ABI without PyTorch: the stand-alone caller (plain HIP memory, its own stream) must leave
the same bytes as the same inputs through the Python binding."""
import os
import re
import subprocess

import numpy as np
import pytest

from conftest import ROOT

pytestmark = pytest.mark.gpu

EXE = os.path.join(ROOT, "paper_2505_00347_amd", "lib", "solo_c_example")


def lcg_units(x0, count):
    """The example's generator, vectorized: x <- 1664525 x + 1013904223 (mod 2^32), `count` values
    in [-1, 1) from the top 24 bits; returns them and the last state."""
    a = np.uint32(1664525)
    pw = np.cumprod(np.full(count, a, np.uint32), dtype=np.uint32)            # a^k, k = 1..count
    geo = np.concatenate(([np.uint32(1)], (np.cumsum(pw[:-1], dtype=np.uint32) + np.uint32(1)).astype(np.uint32)))  # sum_{i<k} a^i
    x = (pw * np.uint32(x0) + np.uint32(1013904223) * geo).astype(np.uint32)
    vals = (x >> np.uint32(8)).astype(np.int32).astype(np.float32) * np.float32(1.0 / 8388608.0) - np.float32(1.0)
    return vals, int(x[-1])


def fold_hash(h, words):
    for w in words.tolist():
        h = (((h << 7) | (h >> 57)) & 0xFFFFFFFFFFFFFFFF) ^ w
    return h


def test_c_caller_equals_python_binding():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    if not os.path.exists(EXE):
        pytest.fail("solo_c_example is not built (python -m paper_2505_00347_amd.build)")
    n, steps = 300007, 3
    out = subprocess.run([EXE, str(n), str(steps)], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stderr
    m = re.search(r"param_sum (\d+) state_hash ([0-9a-f]+)", out.stdout)
    assert m, out.stdout
    from paper_2505_00347_amd import solo, synth
    cfg = solo.make_config(2, 3, 128, solo.SOLO_GRAD_BF16, lr=1e-3, beta1=solo.solo_beta1_default(2, 0), beta2=0.999,
                           eps=1e-8, weight_decay=0.01, quantile_p=0.1, seed=42)
    vals, x = lcg_units(12345, n)
    p = torch.from_numpy((np.float32(0.02) * vals).astype(np.float32)).cuda()
    st = solo.SoloState(n, cfg)
    for step in range(1, steps + 1):
        vals, x = lcg_units(x, n)
        bits, _ = synth.round_to_bf16((np.float32(1e-3) * vals).astype(np.float32))
        g = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
        st.step(p, g, step)
    torch.cuda.synchronize()
    sum_p = int(p.cpu().numpy().view(np.uint32).astype(np.uint64).sum())
    h = 0
    for t in (st.m_codes, st.v_codes, st.m_scale, st.v_scale, st.v_base):
        h = fold_hash(h, t.cpu().numpy().view(np.uint32))
    assert (sum_p, "%016x" % h) == (int(m.group(1)), m.group(2))
