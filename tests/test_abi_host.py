"""Host-side checks of libsolo that need no GPU: the library loads, exports every symbol that
include/solo.h declares, and its pure host helpers agree with the paper's printed values."""
import ctypes
import os
import re
import sys

import pytest

from conftest import ROOT, read_golden


@pytest.fixture(scope="module")
def solo():
    from paper_2505_00347_amd import solo as s
    if not os.path.exists(s.LIB_PATH):
        from paper_2505_00347_amd import build
        build.build(force=True)
    s.lib()
    return s


def declared_functions():
    text = open(os.path.join(ROOT, "include", "solo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(solo_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(solo):
    names = declared_functions()
    assert {"solo_adamw_step", "solo_adamw_step_mp", "solo_adamw_step_multi", "solo_multi_units",
            "solo_multi_table_bytes", "solo_multi_table_build", "solo_state_init", "solo_code_words", "solo_num_blocks",
            "solo_state_bytes", "solo_beta1_default", "solo_beta1_bound", "solo_strerror"} <= set(names)
    raw = ctypes.CDLL(solo.LIB_PATH)
    for name in names:
        assert hasattr(raw, name), name


def test_config_struct_matches_header(solo):
    """Field order and sizes of the ctypes mirror follow the C declaration."""
    text = open(os.path.join(ROOT, "include", "solo.h")).read()
    body = re.search(r"typedef struct solo_config \{(.*?)\} solo_config;", text, re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in body.split(";"):
        decl = decl.strip()
        if decl:
            typ, names = decl.split(None, 1)
            fields += [(n.strip(), typ) for n in names.split(",")]
    ctype = {"uint32_t": ctypes.c_uint32, "uint64_t": ctypes.c_uint64, "float": ctypes.c_float}
    assert [(n, ctype[t]) for n, t in fields] == list(solo.solo_config._fields_)
    assert ctypes.sizeof(solo.solo_config) == 64


def test_size_queries(solo):
    assert solo.solo_code_words(2560, 2) == 160 and solo.solo_code_words(2560, 3) == 256
    assert solo.solo_code_words(2560, 4) == 320 and solo.solo_code_words(11, 3) == 2
    assert solo.solo_code_words(0, 4) == 0 and solo.solo_code_words(100, 5) == 0
    assert solo.solo_num_blocks(129, 128) == 2 and solo.solo_num_blocks(0, 64) == 0
    # Sec. 4.2: the scale costs 1/4 bit per element at block 128 and the buffered base
    # doubles it: (b_m + b_v)/8 + 12/B bytes per parameter
    n = 128 * 2560
    cfg = solo.make_config(2, 2, 128)
    assert solo.solo_state_bytes(n, cfg) == n * (2 + 2) // 8 + 12 * n // 128
    cfg = solo.make_config(4, 3, 64)
    assert solo.solo_state_bytes(n, cfg) == n * 4 // 8 + 4 * n // 10 + 12 * n // 64
    # the memory table of the paper (LLaMA-7B): SOLO 2-bit AdamW holds 3.61 GB, 0.20 GB more
    # than 2-bit AdamW without a buffered base (3.41 GB): one float per block of 128
    n7b = 6738415616
    total = solo.solo_state_bytes(n7b, solo.make_config(2, 2, 128))
    without_base = n7b * 4 // 8 + 8 * (n7b // 128)
    assert abs((total - without_base) / 2 ** 30 - (3.61 - 3.41)) < 0.006
    assert abs(total / 2 ** 30 - 3.61) < 0.15


def test_beta1_defaults(solo):
    """Sec. 3.4: 0.8 / 0.3 for 4-bit, 0.5 / 0.1 for 2-bit first moments."""
    assert solo.solo_beta1_default(4, 0) == pytest.approx(0.8) and solo.solo_beta1_default(4, 1) == pytest.approx(0.3)
    assert solo.solo_beta1_default(2, 0) == pytest.approx(0.5) and solo.solo_beta1_default(2, 1) == pytest.approx(0.1)
    assert solo.solo_beta1_default(3, 0) == pytest.approx(0.6) and solo.solo_beta1_default(3, 1) == pytest.approx(0.2)


def test_beta_prime_bound_reproduces_the_papers_table(solo):
    rows = read_golden("beta_prime_table.txt")
    rmed = {int(r[1]): float(r[2]) for r in rows if r[0] == "rmed"}
    bounds = [(int(r[1]), int(r[2]), float(r[3])) for r in rows if r[0] == "bound"]
    assert len(bounds) == 12
    for bprime, b, want in bounds:
        got = solo.solo_beta1_bound(0.9, rmed[b], rmed[bprime])
        assert abs(got - want) < 6e-4, (bprime, b, got, want)
    # the paper's defaults sit just under the b = 5 (fine-tuning) and b = 8 (scratch) columns
    assert solo.solo_beta1_default(4, 0) <= solo.solo_beta1_bound(0.9, rmed[5], rmed[4])
    assert solo.solo_beta1_default(2, 0) <= solo.solo_beta1_bound(0.9, rmed[5], rmed[2])
    assert solo.solo_beta1_default(4, 1) <= solo.solo_beta1_bound(0.9, rmed[8], rmed[4])
    assert solo.solo_beta1_default(2, 1) <= solo.solo_beta1_bound(0.9, rmed[8], rmed[2])
    assert solo.solo_beta1_bound(1.5, 0.1, 0.1) == 0.0


def test_error_strings_and_host_side_rejections(solo):
    assert "success" in solo.solo_strerror(0)
    for code in (-1, -2, -3, -99):
        assert solo.solo_strerror(code)
    cfg = solo.make_config(2, 3, 128, 1)
    # rejected on the host before any HIP call: works without a GPU
    assert solo.solo_adamw_step(0, 0, 0, 0, 0, 0, 0, 100, 1, cfg, stream=0, check=False) == solo.SOLO_E_INVALID
    assert solo.solo_adamw_step(0, 0, 0, 0, 0, 0, 0, 0, 1, cfg, stream=0, check=False) == solo.SOLO_OK
    bad = solo.make_config(2, 3, 100, 1)
    assert solo.solo_state_init(16, 16, 16, 16, 16, 100, bad, stream=0, check=False) == solo.SOLO_E_INVALID


def test_multi_tensor_table_layout(solo):
    """The table of solo_adamw_step_multi is built by host code alone: 96 bytes per tensor
    (eight pointers, n, first unit, xi offset, a reserved word), then one 32-bit entry per unit: the
    tensor's index, and for the 512-element pieces of a ragged end also the piece and a flag.  The pointers are made-up, suitably aligned addresses; nothing touches a GPU."""
    import numpy as np
    cfg = solo.make_config(2, 3, 128, 1, index_offset=8 * 77)
    sizes = [3000, 0, 5120, 12800 + 1, 64]
    arr = (solo.solo_tensor * len(sizes))()
    for k, n in enumerate(sizes):
        base = 0x10000000 * (k + 1)
        arr[k] = solo.solo_tensor(base, base + 0x1000000 if k == 2 else None, base + 0x2000000, base + 0x3000000,
                                  base + 0x4000000, base + 0x5000000, base + 0x6000000, base + 0x7000000, n)
    units = solo.solo_multi_units(arr, len(sizes), cfg)
    unit = 5120                       # the super-tile of this format; a ragged end counts one unit per 512
    full = [n // unit for n in sizes]   # elements, up to the end of its last code word (a multiple of 80)
    ragged = [-(-(-(-n // 80) * 80 - n // unit * unit) // 512) if n % unit else 0 for n in sizes]
    per_tensor = [f + r for f, r in zip(full, ragged)]
    assert ragged == [6, 0, 0, 6, 1] and units == sum(per_tensor)
    nbytes = solo.solo_multi_table_bytes(len(sizes), units)
    assert nbytes == 96 * len(sizes) + 4 * units
    buf = np.zeros(nbytes, np.uint8)
    rc, flags = solo.solo_multi_table_build(arr, len(sizes), cfg, buf.ctypes.data, nbytes)
    assert rc == solo.SOLO_OK and flags == 1                      # tensor 2 has a bf16 copy
    entries = buf[:96 * len(sizes)].view(np.uint64).reshape(len(sizes), 12)
    unit_map = buf[96 * len(sizes):].view(np.uint32)
    unit0, xi = 0, 8 * 77
    for k, n in enumerate(sizes):
        base = 0x10000000 * (k + 1)
        want_ptrs = [base, base + 0x1000000 if k == 2 else 0] + [base + 0x1000000 * j for j in range(2, 8)]
        assert list(entries[k, :8]) == want_ptrs
        assert entries[k, 8] == n and entries[k, 9] == unit0 and entries[k, 10] == xi
        assert np.all(unit_map[unit0:unit0 + full[k]] == k)
        want = [k | (c << 24) | 0x80000000 for c in range(ragged[k])]
        assert list(unit_map[unit0 + full[k]:unit0 + per_tensor[k]]) == want
        unit0 += per_tensor[k]
        xi += -(-n // 2560) * 2560                               # xi offsets advance in 2560-element steps
    # a misaligned or missing pointer of a non-empty tensor is refused; an empty tensor's are ignored
    arr[0].grad = arr[0].grad + 8
    assert solo.solo_multi_table_build(arr, len(sizes), cfg, buf.ctypes.data, nbytes, check=False)[0] == solo.SOLO_E_INVALID
    arr[0].grad = arr[0].grad - 8
    arr[1].param = None
    assert solo.solo_multi_table_build(arr, len(sizes), cfg, buf.ctypes.data, nbytes, check=False)[0] == solo.SOLO_OK
    assert solo.solo_multi_units(arr, len(sizes), solo.make_config(2, 3, 100, 1)) == 0


def test_multi_table_of_a_chunked_format_and_large_blocks(solo):
    """With fp32 gradients and the linear codebook a table holds one entry per 2560-element unit
    (the shorter end of a tensor included); with blocks of 2048 elements one entry per block."""
    import numpy as np
    cfg = solo.make_config(bits_m=2, bits_v=2, block_size=64, grad_dtype=solo.SOLO_GRAD_FP32)
    sizes = [1, 2559, 2560, 2561, 0, 7680, 12801]
    arr = (solo.solo_tensor * len(sizes))()
    for k, n in enumerate(sizes):
        base = 0x10000000 * (k + 1)
        arr[k] = solo.solo_tensor(base, None, *[base + 0x1000000 * j for j in range(2, 8)], n)
    want_units = [-(-n // 2560) for n in sizes]
    units = solo.solo_multi_units(arr, len(sizes), cfg)
    assert units == sum(want_units)
    nbytes = solo.solo_multi_table_bytes(len(sizes), units)
    buf = np.zeros(nbytes, np.uint8)
    rc, flags = solo.solo_multi_table_build(arr, len(sizes), cfg, buf.ctypes.data, nbytes)
    assert rc == solo.SOLO_OK and flags == 0
    unit_map = buf[96 * len(sizes):].view(np.uint32)
    assert list(unit_map) == [k for k, u in enumerate(want_units) for _ in range(u)]
    # the same tensors with bf16 gradients: super-tiles plus one entry per 512 elements of a ragged end
    cfg16 = solo.make_config(bits_m=2, bits_v=2, block_size=64, grad_dtype=solo.SOLO_GRAD_BF16)
    assert solo.solo_multi_units(arr, len(sizes), cfg16) != units
    # blocks of 2048 elements: one entry per block, a shorter last block flagged (bit 31) and
    # announced in the table's flags, since it takes a second launch
    big = solo.make_config(bits_m=2, bits_v=3, block_size=2048, grad_dtype=solo.SOLO_GRAD_BF16)
    want_units = [-(-n // 2048) for n in sizes]
    units = solo.solo_multi_units(arr, len(sizes), big)
    assert units == sum(want_units)
    nbytes = solo.solo_multi_table_bytes(len(sizes), units)
    buf = np.zeros(nbytes, np.uint8)
    rc, flags = solo.solo_multi_table_build(arr, len(sizes), big, buf.ctypes.data, nbytes)
    assert rc == solo.SOLO_OK and flags == solo.SOLO_TABLE_SHORT_BLOCK
    want_map = []
    for k, n in enumerate(sizes):
        want_map += [k] * (n // 2048) + ([k | 0x80000000] if n % 2048 else [])
    assert list(buf[96 * len(sizes):].view(np.uint32)) == want_map
    for k in range(len(sizes)):
        arr[k].n = 2048 * k
    units = solo.solo_multi_units(arr, len(sizes), big)
    assert units == sum(range(len(sizes)))
    buf = np.zeros(solo.solo_multi_table_bytes(len(sizes), units), np.uint8)
    assert solo.solo_multi_table_build(arr, len(sizes), big, buf.ctypes.data, buf.size) == (solo.SOLO_OK, 0)
    assert solo.solo_num_blocks(5000, 2048) == 3
    assert solo.solo_state_bytes(4096, big) == 4 * (256 + 410) + 12 * 2


def test_binding_loads_torch_before_the_library():
    """The torch wheel carries a HIP runtime of its own; libsolo must be loaded after it so that
    both use the same one (a process that loaded libsolo first failed every launch on a torch
    stream).  The binding therefore imports torch itself before it opens the library."""
    import subprocess
    code = ("import sys; from paper_2505_00347_amd import solo; assert 'torch' not in sys.modules; "
            "solo.lib(); assert 'torch' in sys.modules")
    subprocess.run([sys.executable, "-c", code], cwd=ROOT, check=True, timeout=300)


def test_product_does_not_import_the_oracle():
    """The library and its binding must not reach into oracle/ (tests, smoke and the
    benchmark's cpu_baseline leg are the only users)."""
    pkg = os.path.join(ROOT, "paper_2505_00347_amd")
    for base, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(base, f)).read()
                assert "oracle" not in text.lower() or f == "synth.py", f
    text = open(os.path.join(pkg, "synth.py")).read()
    assert "import oracle" not in text and "from oracle" not in text
    src = open(os.path.join(ROOT, "oracle", "solo_oracle.py")).read() + open(os.path.join(ROOT, "oracle", "solo_oracle.c")).read()
    assert "paper_2505_00347_amd" not in src and "solo.h" not in src
