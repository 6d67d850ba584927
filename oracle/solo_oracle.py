"""ctypes front end of the CPU oracle (``solo_oracle.c``).

TEST INFRASTRUCTURE ONLY.  The oracle is a plain scalar restatement of the SOLO
low-bit AdamW step written from the paper; the tests, the smoke check and the
benchmark's cpu_baseline leg compare the GPU library against it.  Nothing in the
GPU library imports this module and this module imports nothing from it.

Every function here is argument marshalling around one C function of the same
name (prefix ``so_``); the arithmetic lives in the C file, where each routine
cites the passage of the paper it follows.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "solo_oracle.c")
_LIB = os.path.join(_HERE, "libsolo_oracle.so")

CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
          "-Wall", "-Wextra", "-std=c11"]


def build(force=False):
    """Compile the oracle with gcc (strict IEEE binary32, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


class Config(C.Structure):
    _fields_ = [("bits_m", C.c_uint32), ("bits_v", C.c_uint32), ("block_size", C.c_uint32),
                ("stochastic", C.c_uint32),
                ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float), ("quantile_p", C.c_float),
                ("seed", C.c_uint64), ("index_offset", C.c_uint64),
                ("m_codebook", C.c_uint32), ("optimizer", C.c_uint32),
                ("grad_scale", C.c_float), ("pad_", C.c_uint32)]


ADAMW, ADAM_L2, ADABELIEF = 0, 1, 2


def make_config(bits_m=4, bits_v=4, block_size=128, stochastic=1, lr=1e-3, beta1=0.8,
                beta2=0.999, eps=1e-8, weight_decay=0.01, quantile_p=0.1, seed=42,
                index_offset=0, m_codebook=0, optimizer=ADAMW, grad_scale=1.0):
    return Config(bits_m, bits_v, block_size, stochastic, lr, beta1, beta2, eps,
                  weight_decay, quantile_p, seed, index_offset, m_codebook, optimizer,
                  grad_scale, 0)


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _declare(_lib)
    return _lib


_f32p = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")
_u16p = np.ctypeslib.ndpointer(np.uint16, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(np.uint32, flags="C_CONTIGUOUS")


def _declare(L):
    L.so_L.restype = C.c_int; L.so_L.argtypes = [C.c_uint32]
    L.so_K.restype = C.c_int; L.so_K.argtypes = [C.c_uint32]
    L.so_signed_level.restype = C.c_double; L.so_signed_level.argtypes = [C.c_uint32, C.c_uint32]
    L.so_dequant_m.restype = C.c_float; L.so_dequant_m.argtypes = [C.c_uint32, C.c_float, C.c_uint32]
    L.so_log_level.restype = C.c_float; L.so_log_level.argtypes = [C.c_float, C.c_uint32, C.c_uint32]
    L.so_dequant_v.restype = C.c_float
    L.so_dequant_v.argtypes = [C.c_uint32, C.c_float, C.c_float, C.c_uint32]
    L.so_de_levels.restype = C.c_int
    L.so_de_levels.argtypes = [C.c_uint32, C.c_int, np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")]
    L.so_de_signed_level.restype = C.c_double; L.so_de_signed_level.argtypes = [C.c_uint32, C.c_uint32]
    L.so_dequant_m_de.restype = C.c_float; L.so_dequant_m_de.argtypes = [C.c_uint32, C.c_float, C.c_uint32]
    L.so_quant_m_de_block.restype = None
    L.so_quant_m_de_block.argtypes = [_f32p, C.c_uint32, C.c_uint32, _u16p, C.POINTER(C.c_float)]
    L.so_xi_keys.restype = None; L.so_xi_keys.argtypes = [C.c_uint64, C.c_uint64, _u32p]
    L.so_xi_bits.restype = C.c_uint32; L.so_xi_bits.argtypes = [_u32p, C.c_uint64]
    L.so_xi.restype = C.c_float; L.so_xi.argtypes = [_u32p, C.c_uint64]
    L.so_xi_fill.restype = None; L.so_xi_fill.argtypes = [_u32p, C.c_uint64, C.c_uint64, _f32p]
    L.so_rank.restype = C.c_uint32; L.so_rank.argtypes = [C.c_float, C.c_uint32]
    L.so_root.restype = C.c_float; L.so_root.argtypes = [C.c_float, C.c_uint32]
    L.so_quant_m_block.restype = None
    L.so_quant_m_block.argtypes = [_f32p, C.c_uint32, C.c_uint32, _u16p, C.POINTER(C.c_float)]
    L.so_quant_v_elem.restype = C.c_uint32
    L.so_quant_v_elem.argtypes = [C.c_float, C.c_float, C.c_float, C.c_float, C.c_uint32]
    L.so_quant_v_margin.restype = C.c_double
    L.so_quant_v_margin.argtypes = [C.c_float, C.c_float, C.c_float, C.c_float, C.c_uint32]
    L.so_order_statistic.restype = C.c_float
    L.so_order_statistic.argtypes = [_f32p, C.c_uint32, C.c_uint32]
    L.so_quant_v_block.restype = None
    L.so_quant_v_block.argtypes = [_f32p, C.c_uint32, C.c_uint32, C.c_float, C.c_uint32, _u32p,
                                   C.c_uint64, _u16p, C.POINTER(C.c_float), C.POINTER(C.c_float),
                                   C.c_void_p]
    L.so_step_unpacked.restype = C.c_int
    L.so_step_unpacked.argtypes = [_f32p, _f32p, _u16p, _f32p, _u16p, _f32p, _f32p, C.c_uint64,
                                   C.c_uint64, C.POINTER(Config), C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_int]
    L.so_codes_per_word.restype = C.c_uint32; L.so_codes_per_word.argtypes = [C.c_uint32]
    L.so_code_words.restype = C.c_uint64; L.so_code_words.argtypes = [C.c_uint64, C.c_uint32]
    L.so_pack.restype = None; L.so_pack.argtypes = [_u16p, C.c_uint64, C.c_uint32, _u32p]
    L.so_unpack.restype = None; L.so_unpack.argtypes = [_u32p, C.c_uint64, C.c_uint32, _u16p]
    L.so_state_init.restype = None
    L.so_state_init.argtypes = [_u32p, _f32p, _u32p, _f32p, _f32p, C.c_uint64, C.POINTER(Config)]
    L.so_step_packed.restype = C.c_int
    L.so_step_packed.argtypes = [_f32p, _f32p, _u32p, _f32p, _u32p, _f32p, _f32p, C.c_uint64,
                                 C.c_uint64, C.POINTER(Config), C.c_void_p, C.c_int]
    L.so_max_threads.restype = C.c_int; L.so_max_threads.argtypes = []
    L.so_round_bf16.restype = None; L.so_round_bf16.argtypes = [_f32p, _u16p, C.c_uint64]
    L.so_unsigned_levels.restype = C.c_int
    L.so_unsigned_levels.argtypes = [C.c_uint32, C.c_int, C.POINTER(C.c_double)]
    L.so_dequant_unsigned.restype = C.c_float
    L.so_dequant_unsigned.argtypes = [C.c_uint32, C.c_float, C.c_uint32, C.c_int]
    L.so_quant_unsigned_block.restype = None
    L.so_quant_unsigned_block.argtypes = [_f32p, C.c_uint32, C.c_uint32, C.c_int, _u16p, C.POINTER(C.c_float)]
    L.so_unsigned_ema_step.restype = C.c_int
    L.so_unsigned_ema_step.argtypes = [_u16p, _f32p, _f32p, _f32p, C.c_uint64, C.c_uint32, C.c_float,
                                       C.c_uint32, C.c_int, C.c_float, C.c_uint32, C.c_uint64, C.c_uint64]


# ------------------------------------------------------------ scalar helpers

def L_of(bits): return lib().so_L(bits)
def K_of(bits): return lib().so_K(bits)
def signed_level(code, bits): return lib().so_signed_level(code, bits)
def dequant_m(code, scale, bits): return np.float32(lib().so_dequant_m(code, scale, bits))
def log_level(alpha, code, bits): return np.float32(lib().so_log_level(alpha, code, bits))
def dequant_v(code, scale, alpha, bits): return np.float32(lib().so_dequant_v(code, scale, alpha, bits))
def rank(p, nb): return lib().so_rank(p, nb)
def root(rho, bits): return np.float32(lib().so_root(rho, bits))
def quant_v_elem(x, scale, alpha, xi, bits): return lib().so_quant_v_elem(x, scale, alpha, xi, bits)
def quant_v_margin(x, scale, alpha, xi, bits): return lib().so_quant_v_margin(x, scale, alpha, xi, bits)
def codes_per_word(bits): return lib().so_codes_per_word(bits)
def code_words(n, bits): return int(lib().so_code_words(n, bits))
def max_threads(): return lib().so_max_threads()


def xi_keys(seed, step):
    k = np.zeros(4, np.uint32)
    lib().so_xi_keys(seed, step, k)
    return k


def xi(keys, i):
    return np.float32(lib().so_xi(np.ascontiguousarray(keys, np.uint32), int(i)))


def xi_bits(keys, i):
    return lib().so_xi_bits(np.ascontiguousarray(keys, np.uint32), int(i))


def xi_array(seed, step, i0, count):
    out = np.zeros(count, np.float32)
    lib().so_xi_fill(xi_keys(seed, step), i0, count, out)
    return out


def xi_bits_array(seed, step, i0, count):
    keys = xi_keys(seed, step)
    return np.array([lib().so_xi_bits(keys, i0 + k) for k in range(count)], np.uint32)


# ------------------------------------------------------------- block helpers

def de_levels(bits, signed=True):
    out = np.zeros(256, np.float64)
    n = lib().so_de_levels(bits, 1 if signed else 0, out)
    return out[:n].copy()


def dequant_m_de(code, scale, bits): return np.float32(lib().so_dequant_m_de(code, scale, bits))


def quant_m_de_block(x, bits):
    x = np.ascontiguousarray(x, np.float32)
    codes = np.zeros(x.size, np.uint16)
    scale = C.c_float()
    lib().so_quant_m_de_block(x, x.size, bits, codes, C.byref(scale))
    return codes, np.float32(scale.value)


def quant_m_block(x, bits):
    x = np.ascontiguousarray(x, np.float32)
    codes = np.zeros(x.size, np.uint16)
    scale = C.c_float()
    lib().so_quant_m_block(x, x.size, bits, codes, C.byref(scale))
    return codes, np.float32(scale.value)


def order_statistic(x, r):
    x = np.ascontiguousarray(x, np.float32)
    return np.float32(lib().so_order_statistic(x, x.size, r))


def quant_v_block(x, bits, p=0.1, stochastic=1, seed=42, step=1, i0=0, want_margin=False):
    x = np.ascontiguousarray(x, np.float32)
    codes = np.zeros(x.size, np.uint16)
    scale, base = C.c_float(), C.c_float()
    margin = np.zeros(x.size, np.float64) if want_margin else None
    lib().so_quant_v_block(x, x.size, bits, p, stochastic, xi_keys(seed, step), i0, codes,
                           C.byref(scale), C.byref(base),
                           margin.ctypes.data if want_margin else None)
    out = (codes, np.float32(scale.value), np.float32(base.value))
    return out + (margin,) if want_margin else out


U_LOG, U_LINEAR, U_LINEAR_NOZERO, U_DE = 0, 1, 2, 3


def unsigned_levels(bits, kind):
    out = (C.c_double * 256)()
    n = lib().so_unsigned_levels(bits, kind, out)
    return np.array(out[:n])


def quant_unsigned_block(x, bits, kind):
    x = np.ascontiguousarray(x, np.float32)
    codes = np.zeros(x.size, np.uint16)
    scale = C.c_float(0)
    lib().so_quant_unsigned_block(x, x.size, bits, kind, codes, C.byref(scale))
    return codes, np.float32(scale.value)


def dequant_unsigned(codes, scale, bits, kind):
    return np.array([lib().so_dequant_unsigned(int(c), float(scale), bits, kind) for c in codes], np.float32)


class UnsignedEma:
    """A quantized unsigned EMA on its own (no optimizer around it): codes, one scale (and for the
    logarithmic quantizer one base) per block."""

    def __init__(self, x0, block, bits, kind, p=0.1, stochastic=1, seed=42):
        x0 = np.ascontiguousarray(x0, np.float32)
        self.n, self.block, self.bits, self.kind = x0.size, block, bits, kind
        self.p, self.stochastic, self.seed, self.t = p, stochastic, seed, 0
        nblk = -(-self.n // block)
        self.codes = np.zeros(self.n, np.uint16)
        self.scale = np.zeros(nblk, np.float32)
        self.base = np.ones(nblk, np.float32)
        # quantize the initial state: an EMA step with beta = 0 from the zero state
        self.step(x0, 0.0)

    def step(self, z, beta):
        self.t += 1
        rc = lib().so_unsigned_ema_step(self.codes, self.scale, self.base, np.ascontiguousarray(z, np.float32),
                                        self.n, self.block, beta, self.bits, self.kind, self.p,
                                        self.stochastic, self.seed, self.t)
        assert rc == 0

    def values(self):
        out = np.empty(self.n, np.float32)
        for b in range(self.scale.size):
            sl = slice(b * self.block, min(self.n, (b + 1) * self.block))
            if self.kind == U_LOG:
                out[sl] = [dequant_v(int(c), self.scale[b], self.base[b], self.bits) for c in self.codes[sl]]
            else:
                out[sl] = dequant_unsigned(self.codes[sl], self.scale[b], self.bits, self.kind)
        return out


def round_bf16(x):
    """bfloat16 bit patterns nearest to the float32 values (ties to even)."""
    x = np.ascontiguousarray(x, np.float32)
    out = np.zeros(x.size, np.uint16)
    lib().so_round_bf16(x.reshape(-1), out, x.size)
    return out


# ------------------------------------------------------------------ packing

def pack(codes, bits):
    codes = np.ascontiguousarray(codes, np.uint16)
    words = np.zeros(code_words(codes.size, bits), np.uint32)
    lib().so_pack(codes, codes.size, bits, words)
    return words


def unpack(words, n, bits):
    words = np.ascontiguousarray(words, np.uint32)
    assert words.size >= code_words(n, bits)
    codes = np.zeros(n, np.uint16)
    lib().so_unpack(words, n, bits, codes)
    return codes


# ------------------------------------------------------------------- states

class State:
    """Packed optimizer state of n elements as numpy arrays (2/3/4-bit codes)."""

    def __init__(self, n, cfg):
        nblk = (n + cfg.block_size - 1) // cfg.block_size
        self.n = n
        self.m_words = np.zeros(code_words(n, cfg.bits_m), np.uint32)
        self.v_words = np.zeros(code_words(n, cfg.bits_v), np.uint32)
        self.m_scale = np.zeros(nblk, np.float32)
        self.v_scale = np.zeros(nblk, np.float32)
        self.v_base = np.zeros(nblk, np.float32)
        lib().so_state_init(self.m_words, self.m_scale, self.v_words, self.v_scale,
                            self.v_base, n, C.byref(cfg))

    def copy(self):
        s = State.__new__(State)
        s.n = self.n
        for k in ("m_words", "v_words", "m_scale", "v_scale", "v_base"):
            setattr(s, k, getattr(self, k).copy())
        return s


def step_packed(param, grad, state, step, cfg, want_margin=False, threads=1):
    """In-place step on float32 ``param`` and ``state``; ``grad`` float32."""
    assert param.dtype == np.float32 and grad.dtype == np.float32
    n = param.size
    margin = np.zeros(n, np.float64) if want_margin else None
    rc = lib().so_step_packed(param, np.ascontiguousarray(grad), state.m_words, state.m_scale,
                              state.v_words, state.v_scale, state.v_base, n, step,
                              C.byref(cfg), margin.ctypes.data if want_margin else None,
                              threads)
    if rc != 0:
        raise ValueError("so_step_packed rejected its arguments")
    return margin


def step_unpacked(param, grad, m_codes, m_scale, v_codes, v_scale, v_base, step, cfg,
                  want_margin=False, want_ema=False, threads=1):
    """In-place step with one code per uint16 (any code width from 2 to 16)."""
    n = param.size
    margin = np.zeros(n, np.float64) if want_margin else None
    mh = np.zeros(n, np.float32) if want_ema else None
    vh = np.zeros(n, np.float32) if want_ema else None
    rc = lib().so_step_unpacked(param, np.ascontiguousarray(grad, np.float32), m_codes, m_scale,
                                v_codes, v_scale, v_base, n, step, C.byref(cfg),
                                margin.ctypes.data if want_margin else None,
                                mh.ctypes.data if want_ema else None,
                                vh.ctypes.data if want_ema else None, threads)
    if rc != 0:
        raise ValueError("so_step_unpacked rejected its arguments")
    return margin, mh, vh
