"""Thin Python binding of libsolo (see include/solo.h): argument marshalling only.

Every function has the name and meaning of the C entry point it calls; all of the
optimizer step runs in the HIP kernels of the library.  Tensors are torch tensors
on an AMD GPU (torch is used for device memory and streams only); a tensor is
passed as its device pointer, the stream as the current torch stream's handle.
The module fails loudly when the library has not been built: there is no
fallback path.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libsolo.so")

SOLO_OK, SOLO_E_INVALID, SOLO_E_UNSUPPORTED, SOLO_E_HIP = 0, -1, -2, -3
SOLO_GRAD_FP32, SOLO_GRAD_BF16 = 0, 1
SOLO_FLAG_STOCHASTIC = 1
SOLO_FLAG_M_DYNAMIC_EXPONENT = 2
SOLO_FLAG_ADABELIEF = 4
SOLO_FLAG_COUPLED_DECAY = 8
SOLO_TABLE_BF16_COPY, SOLO_TABLE_SHORT_BLOCK = 1, 2


class solo_config(C.Structure):
    _fields_ = [("bits_m", C.c_uint32), ("bits_v", C.c_uint32), ("block_size", C.c_uint32),
                ("grad_dtype", C.c_uint32),
                ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("quantile_p", C.c_float),
                ("flags", C.c_uint32), ("reserved", C.c_uint32),
                ("seed", C.c_uint64), ("index_offset", C.c_uint64)]


def make_config(bits_m=4, bits_v=4, block_size=128, grad_dtype=SOLO_GRAD_FP32, lr=1e-3,
                beta1=None, beta2=0.999, eps=1e-8, weight_decay=0.01, quantile_p=0.1,
                flags=SOLO_FLAG_STOCHASTIC, seed=42, index_offset=0):
    if beta1 is None:
        beta1 = solo_beta1_default(bits_m, 0)
    return solo_config(bits_m, bits_v, block_size, grad_dtype, lr, beta1, beta2, eps,
                       weight_decay, quantile_p, flags, 0, seed, index_offset)


class solo_tensor(C.Structure):
    _fields_ = [("param", C.c_void_p), ("param_bf16", C.c_void_p), ("grad", C.c_void_p),
                ("m_codes", C.c_void_p), ("m_scale", C.c_void_p), ("v_codes", C.c_void_p),
                ("v_scale", C.c_void_p), ("v_base", C.c_void_p), ("n", C.c_uint64)]


class SoloError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__(f"libsolo error {code}: {solo_strerror(code)}")


_lib = None


def lib():
    """Load libsolo.so (built by ``python -m paper_2505_00347_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with "
                              "`python -m paper_2505_00347_amd.build` (needs hipcc)")
        # torch first: the wheel brings a HIP runtime of its own and exports it to the process.
        # Loaded after it, libsolo binds to that runtime, the one the tensors and streams of the
        # callers belong to; loaded before it, libsolo would bind to the system's copy, and every
        # launch on a torch stream would fail.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, u32, u64, cfgp = C.c_void_p, C.c_uint32, C.c_uint64, C.POINTER(solo_config)
        L.solo_code_words.restype = C.c_size_t; L.solo_code_words.argtypes = [u64, u32]
        L.solo_num_blocks.restype = C.c_size_t; L.solo_num_blocks.argtypes = [u64, u32]
        L.solo_state_bytes.restype = C.c_size_t; L.solo_state_bytes.argtypes = [u64, cfgp]
        L.solo_beta1_default.restype = C.c_float; L.solo_beta1_default.argtypes = [u32, C.c_int]
        L.solo_beta1_bound.restype = C.c_float
        L.solo_beta1_bound.argtypes = [C.c_float, C.c_float, C.c_float]
        L.solo_strerror.restype = C.c_char_p; L.solo_strerror.argtypes = [C.c_int]
        L.solo_state_init.restype = C.c_int
        L.solo_state_init.argtypes = [vp, vp, vp, vp, vp, u64, cfgp, vp]
        L.solo_adamw_step.restype = C.c_int
        L.solo_adamw_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, u64, u64, cfgp, vp]
        L.solo_adamw_step_mp.restype = C.c_int
        L.solo_adamw_step_mp.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, u64, u64, cfgp, vp]
        tp = C.POINTER(solo_tensor)
        L.solo_multi_units.restype = C.c_uint64; L.solo_multi_units.argtypes = [tp, u32, cfgp]
        L.solo_multi_table_bytes.restype = C.c_size_t; L.solo_multi_table_bytes.argtypes = [u32, u64]
        L.solo_multi_table_build.restype = C.c_int
        L.solo_multi_table_build.argtypes = [tp, u32, cfgp, vp, C.c_size_t, C.POINTER(C.c_uint32)]
        L.solo_adamw_step_multi.restype = C.c_int
        L.solo_adamw_step_multi.argtypes = [vp, u32, u64, u32, vp, u64, cfgp, vp]
        _lib = L
    return _lib


def _ptr(t):
    """Device pointer of a torch tensor (or a raw integer address)."""
    if t is None:
        return None
    return t if isinstance(t, int) else t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def solo_code_words(n, bits): return lib().solo_code_words(n, bits)
def solo_num_blocks(n, block_size): return lib().solo_num_blocks(n, block_size)
def solo_state_bytes(n, cfg): return lib().solo_state_bytes(n, C.byref(cfg))
def solo_beta1_default(bits_m, from_scratch=0): return lib().solo_beta1_default(bits_m, from_scratch)
def solo_beta1_bound(beta, r_median_b, r_median_bprime): return lib().solo_beta1_bound(beta, r_median_b, r_median_bprime)
def solo_strerror(code): return lib().solo_strerror(code).decode()


def solo_state_init(m_codes, m_scale, v_codes, v_scale, v_base, n, cfg, stream=None, check=True):
    rc = lib().solo_state_init(_ptr(m_codes), _ptr(m_scale), _ptr(v_codes), _ptr(v_scale),
                               _ptr(v_base), n, C.byref(cfg), _stream(stream) if n else None)
    if check and rc != SOLO_OK:
        raise SoloError(rc)
    return rc


def solo_adamw_step(param, grad, m_codes, m_scale, v_codes, v_scale, v_base, n, step, cfg,
                    stream=None, check=True):
    rc = lib().solo_adamw_step(_ptr(param), _ptr(grad), _ptr(m_codes), _ptr(m_scale),
                               _ptr(v_codes), _ptr(v_scale), _ptr(v_base), n, step,
                               C.byref(cfg), _stream(stream) if n else None)
    if check and rc != SOLO_OK:
        raise SoloError(rc)
    return rc


def solo_adamw_step_mp(param, param_bf16, grad, grad_scale, m_codes, m_scale, v_codes, v_scale,
                       v_base, n, step, cfg, stream=None, check=True):
    """param_bf16 (bf16 tensor) and grad_scale (one-element float32 device tensor) may be None."""
    rc = lib().solo_adamw_step_mp(_ptr(param), _ptr(param_bf16), _ptr(grad), _ptr(grad_scale),
                                  _ptr(m_codes), _ptr(m_scale), _ptr(v_codes), _ptr(v_scale),
                                  _ptr(v_base), n, step, C.byref(cfg), _stream(stream) if n else None)
    if check and rc != SOLO_OK:
        raise SoloError(rc)
    return rc


def solo_multi_units(tensors, count, cfg): return lib().solo_multi_units(tensors, count, C.byref(cfg))
def solo_multi_table_bytes(count, units): return lib().solo_multi_table_bytes(count, units)


def solo_multi_table_build(tensors, count, cfg, table_host, table_bytes, check=True):
    """Returns (return code, table flags)."""
    flags = C.c_uint32(0)
    rc = lib().solo_multi_table_build(tensors, count, C.byref(cfg), table_host, table_bytes, C.byref(flags))
    if check and rc != SOLO_OK:
        raise SoloError(rc)
    return rc, flags.value


def solo_adamw_step_multi(table_device, count, units, table_flags, grad_scale, step, cfg, stream=None,
                          check=True):
    rc = lib().solo_adamw_step_multi(_ptr(table_device), count, units, table_flags, _ptr(grad_scale), step,
                                     C.byref(cfg), _stream(stream) if units else None)
    if check and rc != SOLO_OK:
        raise SoloError(rc)
    return rc


class SoloMultiTable:
    """The device table of a multi-tensor step, built from per-tensor (param, grad, SoloState[,
    param_bf16]) tuples of torch tensors: marshals the descriptors, lets the library build the
    table in host memory and copies it to the device."""

    def __init__(self, items, cfg, device="cuda"):
        import torch
        self.cfg, self.count = cfg, len(items)
        arr = (solo_tensor * self.count)()
        for k, it in enumerate(items):
            p, g, st = it[0], it[1], it[2]
            h = it[3] if len(it) > 3 else None
            arr[k] = solo_tensor(_ptr(p), _ptr(h), _ptr(g), _ptr(st.m_codes), _ptr(st.m_scale),
                                 _ptr(st.v_codes), _ptr(st.v_scale), _ptr(st.v_base), st.n)
        self.units = solo_multi_units(arr, self.count, cfg)
        nbytes = solo_multi_table_bytes(self.count, self.units)
        host = torch.empty((nbytes + 15) // 16 * 16, dtype=torch.uint8)
        _, self.flags = solo_multi_table_build(arr, self.count, cfg, host.data_ptr(), nbytes)
        self.table = host.to(device)
        self._keep = items                         # the buffers the table points to

    def step(self, step, grad_scale=None, stream=None):
        return solo_adamw_step_multi(self.table, self.count, self.units, self.flags, grad_scale, step,
                                     self.cfg, stream)


HBM_REGION_BYTES = 96 << 30      # an MI355X behaves as three such regions of physical memory


class state_region:
    """Context manager for the placement rule of include/solo.h (performance note): tensors that
    are allocated inside it come to lie behind the first 96 GiB that this process has allocated on
    the device, i.e. (in a process that started on an idle GPU, which receives physical memory in
    allocation order) in another third of HBM than the parameters allocated before it.

        p, g = ...                                   # resident_bytes of them, allocated first
        with solo.state_region(resident_bytes):
            state = solo.SoloState(n, cfg)

    It allocates a spacer up to the region boundary on entry and returns it to the driver on exit.
    Nothing happens if the resident bytes already fill a region, or if the device has no room."""

    def __init__(self, resident_bytes, keep_free=8 << 30):
        self.resident, self.keep_free, self.spacer = int(resident_bytes), keep_free, None

    def __enter__(self):
        import torch
        gap = HBM_REGION_BYTES - self.resident
        if 0 < gap < torch.cuda.mem_get_info()[0] - self.keep_free:
            self.spacer = torch.empty(gap, dtype=torch.uint8, device="cuda")
        return self

    def __exit__(self, *exc):
        import torch
        if self.spacer is not None:
            self.spacer = None
            torch.cuda.empty_cache()     # the spacer goes back to the driver, not into torch's cache
        return False


class SoloState:
    """Device buffers of the packed optimizer state of n elements (caller-owned memory:
    plain torch tensors; int32 tensors carry the uint32 code words)."""

    def __init__(self, n, cfg, device="cuda", init=True):
        import torch
        self.n, self.cfg = n, cfg
        nb = solo_num_blocks(n, cfg.block_size)
        self.m_codes = torch.empty(solo_code_words(n, cfg.bits_m), dtype=torch.int32, device=device)
        self.v_codes = torch.empty(solo_code_words(n, cfg.bits_v), dtype=torch.int32, device=device)
        self.m_scale = torch.empty(nb, dtype=torch.float32, device=device)
        self.v_scale = torch.empty(nb, dtype=torch.float32, device=device)
        self.v_base = torch.empty(nb, dtype=torch.float32, device=device)
        if init:
            solo_state_init(self.m_codes, self.m_scale, self.v_codes, self.v_scale, self.v_base,
                            n, cfg)

    def buffers(self):
        return (self.m_codes, self.m_scale, self.v_codes, self.v_scale, self.v_base)

    def step(self, param, grad, step, stream=None, param_bf16=None, grad_scale=None):
        if param_bf16 is None and grad_scale is None:
            return solo_adamw_step(param, grad, *self.buffers(), self.n, step, self.cfg, stream)
        return solo_adamw_step_mp(param, param_bf16, grad, grad_scale, *self.buffers(), self.n, step,
                                  self.cfg, stream)
