"""Seeded synthetic inputs for the SOLO AdamW step: shapes and value recipes only.

This module holds NONE of the method's arithmetic.  It produces parameters and
gradients with the shapes and value distributions of the five benchmark
configurations (a 2^20-element tensor, GPT-2-125M-, 1.3B- and LLaMA-7B-shaped
tensor sets), so that the GPU library and the CPU oracle can be fed the same
numbers.  The models' real weights and data sets are not used anywhere; these
stand in for them.

All generators are counter based (numpy Philox keyed by (seed, stream)), so any
slice of a large flat buffer can be regenerated without materialising the rest.
"""
from dataclasses import dataclass, field

import numpy as np

SEED_PARAM = 1234
SEED_XI = 42


def seed_grad(config_id, step):
    return 1000 * config_id + step


# ------------------------------------------------------------------ shapes

def gpt2_125m_shapes():
    h, layers, vocab = 768, 12, 50257
    t = [("wte", vocab * h, "matrix")]
    for l in range(layers):
        t += [(f"h{l}.ln1.g", h, "ones"), (f"h{l}.ln1.b", h, "zeros"),
              (f"h{l}.qkv", h * 3 * h, "matrix"), (f"h{l}.proj", h * h, "matrix"),
              (f"h{l}.ln2.g", h, "ones"), (f"h{l}.ln2.b", h, "zeros"),
              (f"h{l}.fc", h * 4 * h, "matrix"), (f"h{l}.fc2", 4 * h * h, "matrix")]
    t += [("ln_f.g", h, "ones"), ("ln_f.b", h, "zeros")]
    return t


def transformer_1p3b_shapes():
    h, layers, vocab, ff = 2048, 24, 50304, 8192
    t = [("embed", vocab * h, "matrix")]
    for l in range(layers):
        t += [(f"l{l}.ln1.g", h, "ones"), (f"l{l}.ln1.b", h, "zeros"),
              (f"l{l}.qkv", h * 3 * h, "matrix"), (f"l{l}.proj", h * h, "matrix"),
              (f"l{l}.ln2.g", h, "ones"), (f"l{l}.ln2.b", h, "zeros"),
              (f"l{l}.fc", h * ff, "matrix"), (f"l{l}.fc2", ff * h, "matrix")]
    t += [("ln_f.g", h, "ones"), ("ln_f.b", h, "zeros")]
    return t


def llama_7b_shapes():
    h, layers, vocab, ff = 4096, 32, 32000, 11008
    t = [("embed", vocab * h, "matrix")]
    for l in range(layers):
        t += [(f"l{l}.norm1", h, "ones"),
              (f"l{l}.q", h * h, "matrix"), (f"l{l}.k", h * h, "matrix"),
              (f"l{l}.v", h * h, "matrix"), (f"l{l}.o", h * h, "matrix"),
              (f"l{l}.norm2", h, "ones"),
              (f"l{l}.gate", h * ff, "matrix"), (f"l{l}.up", h * ff, "matrix"),
              (f"l{l}.down", ff * h, "matrix")]
    t += [("norm_f", h, "ones"), ("lm_head", vocab * h, "matrix")]
    return t


@dataclass
class Workload:
    """One benchmark configuration: tensor set, state format, value recipe."""
    name: str
    config_id: int
    tensors: list                 # (name, numel, kind) in flat-buffer order
    bits_m: int
    bits_v: int
    block_size: int
    beta1: float
    grad_dtype: str               # "fp32" | "bf16"
    grad_kind: str                # "normal" | "student_t3" | "normal_outliers"
    grad_std: float
    lr: float = 1e-3
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    quantile_p: float = 0.1
    steps: int = 10
    m_codebook: str = "linear"   # "linear" | "de" (signed dynamic exponent, the paper's own variants)
    extra: dict = field(default_factory=dict)

    @property
    def n(self):
        return sum(t[1] for t in self.tensors)


def workload(name):
    """The five configurations (precision-specific beta1: 0.8 for 4-bit,
    0.6 for 3-bit, 0.5 for 2-bit first moments)."""
    if name == "c1_1m_4bit":
        return Workload(name, 1, [("w", 1 << 20, "matrix")], 4, 4, 128, 0.8, "fp32", "normal", 1e-3)
    if name == "c2_1m_3bit_t3":
        return Workload(name, 2, [("w", 1 << 20, "matrix")], 3, 3, 128, 0.6, "fp32", "student_t3", 1e-3)
    if name == "c3_gpt2_125m_2bit":
        return Workload(name, 3, gpt2_125m_shapes(), 2, 2, 64, 0.5, "fp32", "normal", 1e-3)
    if name == "c4_1p3b_3bit":
        return Workload(name, 4, transformer_1p3b_shapes(), 3, 3, 128, 0.6, "bf16",
                        "normal_outliers", 1e-4)
    if name == "c5_llama7b_2bit_3bit":
        return Workload(name, 5, llama_7b_shapes(), 2, 3, 128, 0.5, "bf16",
                        "normal_outliers", 1e-4)
    # the paper's own two variants (Sec. 3.4) on the LLaMA-7B shapes
    if name == "paper_4_2bit_llama7b":
        return Workload(name, 6, llama_7b_shapes(), 4, 2, 128, 0.8, "bf16", "normal_outliers", 1e-4,
                        m_codebook="de")
    if name == "paper_2bit_llama7b":
        return Workload(name, 7, llama_7b_shapes(), 2, 2, 128, 0.5, "bf16", "normal_outliers", 1e-4,
                        m_codebook="de")
    # C5 with blocks of 2048 elements (the large-block setting of the block-size comparison, Sec. 4.2)
    if name == "c5_llama7b_block2048":
        return Workload(name, 5, llama_7b_shapes(), 2, 3, 2048, 0.5, "bf16", "normal_outliers", 1e-4)
    # C5 with the sparse-embedding stress of Sec. 3.2.2: per step, 90 % of the rows of the
    # embedding matrix (the first tensor) receive no gradient at all
    if name == "c5_sparse_embed":
        return Workload(name, 5, llama_7b_shapes(), 2, 3, 128, 0.5, "bf16", "normal_outliers", 1e-4,
                        extra={"sparse_rows": {"tensor": 0, "row_len": 4096, "zero_frac": 0.9}})
    raise KeyError(name)


WORKLOADS = ["c1_1m_4bit", "c2_1m_3bit_t3", "c3_gpt2_125m_2bit", "c4_1p3b_3bit",
             "c5_llama7b_2bit_3bit"]


# ------------------------------------------------------------------ values

def _rng(seed, stream):
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, stream]))


def round_to_bf16(x):
    """Round float32 to the nearest bfloat16 (ties to even); returns the uint16
    bit patterns and the float32 values they widen to."""
    b = np.ascontiguousarray(x, np.float32).view(np.uint32)
    r = ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).astype(np.uint16)
    return r, (r.astype(np.uint32) << 16).view(np.float32)


def make_params(n, seed=SEED_PARAM, stream=0, kind="matrix"):
    if kind == "ones":
        return np.ones(n, np.float32)
    if kind == "zeros":
        return np.zeros(n, np.float32)
    return (_rng(seed, stream).standard_normal(n, np.float32) * np.float32(0.02))


def make_grads(n, kind, std, seed, stream=0):
    """float32 gradients: N(0, std^2); std * Student-t(nu=3); or N(0, std^2)
    with 1 % of the entries multiplied by 100."""
    g = _rng(seed, stream)
    if kind == "normal":
        x = g.standard_normal(n, np.float32)
    elif kind == "student_t3":
        x = g.standard_t(3.0, n).astype(np.float32)
    elif kind == "normal_outliers":
        x = g.standard_normal(n, np.float32)
        x = np.where(g.random(n, np.float32) < 0.01, x * np.float32(100.0), x)
    else:
        raise KeyError(kind)
    return (x * np.float32(std)).astype(np.float32)


def zero_row_mask(rows, zero_frac, seed, stream=0):
    """Which rows of an embedding-shaped matrix receive no gradient in one step (True = all
    zeros): each row independently with probability zero_frac, fresh per (seed, stream)."""
    return _rng(seed ^ 0x5EED, stream).random(rows, np.float32) < np.float32(zero_frac)


def workload_slice(w, step, count=None, tensor_index=0):
    """(params, grads) of the first `count` elements of one tensor of a workload
    at one step, as float32 numpy arrays; bf16 workloads get gradients already
    rounded to bf16 (bit patterns returned as third item, else None)."""
    name, numel, kind = w.tensors[tensor_index]
    count = numel if count is None else min(count, numel)
    p = make_params(count, SEED_PARAM, tensor_index, kind)
    g = make_grads(count, w.grad_kind, w.grad_std, seed_grad(w.config_id, step), tensor_index)
    bits = None
    if w.grad_dtype == "bf16":
        bits, g = round_to_bf16(g)
    return p, g, bits
