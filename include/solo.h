/*
 * libsolo — the SOLO low-bit AdamW optimizer step for AMD MI355X (gfx950).
 *
 * One call performs, in a single pass over HBM, the whole quantized-state
 * update of "Pushing the Limits of Low-Bit Optimizers: A Focus on EMA
 * Dynamics" (SOLO) for one flat buffer of parameters:
 *
 *   dequantize both moments  ->  EMA update  ->  AdamW parameter update
 *   ->  per-block scale / quantile / log base  ->  re-quantize  ->  re-pack
 *
 *   1st moment  m : b_m-bit signed linear codes, or the signed dynamic-
 *                   exponent codes of the paper's own variants (App. A, Eq. 1)
 *   2nd moment  v : b_v-bit unsigned logarithmic codes, levels alpha^k,
 *                   log-domain stochastic rounding, per-block base alpha
 *                   from the p-quantile                     (Sec. 3.2.2)
 *   block-wise quantization, one scale per block            (Sec. 3.4)
 *
 * Conventions for every entry point
 *   - Pointers named param / grad / *_codes / *_scale / v_base are DEVICE
 *     pointers; `cfg` is a HOST pointer, read during the call only.
 *   - All buffers are owned by the caller.  The library never allocates,
 *     frees or keeps a pointer, and never synchronises: work is enqueued on
 *     `stream` (a hipStream_t passed as void*; NULL = the default stream) and
 *     the call returns at once.
 *   - Return value: SOLO_OK (0) or a negative error code; nothing is enqueued
 *     when an error is returned.  n == 0 is a successful no-op.
 *   - The library uses the HIP runtime it finds in the process.  A process
 *     that brings one of its own (a PyTorch wheel does) loads that first, so
 *     that the streams it passes and the launches belong to the same runtime.
 *
 * State layout for n elements, block size B, nb = ceil(n / B) blocks
 *   m_codes  uint32[solo_code_words(n, bits_m)]   element i lives in word
 *   v_codes  uint32[solo_code_words(n, bits_v)]   i / c at bit bits*(i mod c),
 *            c = 16 (2-bit), 10 (3-bit, two pad bits), 8 (4-bit); unused bits 0
 *   m_scale  float[nb]   Delta_m = max |m| of the block
 *   v_scale  float[nb]   Delta_v = max v of the block
 *   v_base   float[nb]   alpha of the block, in (0, 1]
 *   A 1st-moment code c in [0, 2L], L = 2^(bits_m-1)-1, stands for the level
 *   (c - L) / L; with SOLO_FLAG_M_DYNAMIC_EXPONENT a code in [0, 2L+1] indexes the
 *   increasing signed dynamic-exponent levels (code L is 0, code 2L+1 is +1, there
 *   is no level -1).  A 2nd-moment code q in [0, 2^bits_v - 1] stands for alpha^q.
 *   param, grad and the code buffers must be 16-byte aligned, the scale
 *   buffers 4-byte aligned.
 *   The unused bits of the code words (the two pad bits of every 3-bit word, the
 *   fields behind element n-1 of the last word) must be zero on entry to a step;
 *   solo_state_init and every step leave them zero.
 */
#ifndef SOLO_H
#define SOLO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SOLO_OK = 0,
    SOLO_E_INVALID = -1,      /* null/misaligned pointer, value out of range   */
    SOLO_E_UNSUPPORTED = -2,  /* legal value this build has no kernel for      */
    SOLO_E_HIP = -3           /* the HIP runtime refused the launch            */
};

enum { SOLO_GRAD_FP32 = 0, SOLO_GRAD_BF16 = 1 };

/* flags */
#define SOLO_FLAG_STOCHASTIC 1u   /* xi ~ U(-0.5, 0.5); clear = xi = 0 */
#define SOLO_FLAG_M_DYNAMIC_EXPONENT 2u /* 1st moment uses the signed dynamic-exponent levels of
                                          App. A (the paper's own 4/2-bit and 2-bit AdamW, Sec. 3.4)
                                          instead of the signed linear ones */

#define SOLO_FLAG_ADABELIEF 4u     /* AdaBelief instead of Adam (Sec. 4.2, "Generalizability"): the
                                     unsigned EMA follows (g - m^)^2, m^ the fresh 1st moment, and
                                     eps is added to that EMA itself at every step */
#define SOLO_FLAG_COUPLED_DECAY 8u /* plain Adam: weight_decay * p is added to the gradient before
                                     both EMAs and the parameter is not decayed separately */

typedef struct solo_config {
    uint32_t bits_m;       /* 2, 3 or 4: signed linear or dynamic-exponent codes (App. A) */
    uint32_t bits_v;       /* 2, 3 or 4: logarithmic codes (Sec. 3.2.2)                */
    uint32_t block_size;   /* 64, 128 or 2048 elements per block (Sec. 3.4 uses 128;   */
                           /* 2048 is the large-block setting of Sec. 4.2)             */
    uint32_t grad_dtype;   /* SOLO_GRAD_FP32 or SOLO_GRAD_BF16                         */
    float lr;              /* learning rate                                            */
    float beta1;           /* momentum of the signed EMA, in [0,1); use the precision- */
                           /* specific value of Sec. 3.3 (solo_beta1_default)          */
    float beta2;           /* momentum of the unsigned EMA, in [0,1)                   */
    float eps;             /* added to the bias-corrected root, >= 0                   */
    float weight_decay;    /* decoupled decay                                          */
    float quantile_p;      /* p of the quantile that sets alpha, in [0,1); paper: 0.1  */
    uint32_t flags;        /* SOLO_FLAG_*                                              */
    uint32_t reserved;     /* must be 0                                                */
    uint64_t seed;         /* key of the xi stream                                     */
    uint64_t index_offset; /* global index of element 0 of this buffer; multiple of 8. */
                           /* xi is a function of (seed, step, index_offset + i), so a */
                           /* shard of a larger buffer reproduces the unsharded result */
} solo_config;

/* Number of uint32 words that hold n codes of the given width (2, 3 or 4);
 * 0 for an unsupported width.  Sec. 3.4 packs several low-bit codes into one
 * storage element (two 4-bit or four 2-bit codes per byte; a word of this library
 * is four such bytes, little-endian); 3-bit codes, which Sec. 3.4 leaves out for
 * lack of a packing, go ten to a word with two unused bits. */
size_t solo_code_words(uint64_t n, uint32_t bits);

/* Number of quantization blocks of n elements, ceil(n / block_size) (block-wise
 * quantization, Sec. 3.4: every block of block_size consecutive elements has its
 * own scale; a shorter last block is a block of its own); 0 if block_size is 0. */
size_t solo_num_blocks(uint64_t n, uint32_t block_size);

/* Bytes of optimizer state for n elements: both code buffers plus three
 * floats per block (Sec. 4.2: the scale costs 32/B bits per element and the
 * buffered log base doubles that). 0 if cfg is invalid. */
size_t solo_state_bytes(uint64_t n, const solo_config *cfg);

/* Default momentum of the signed EMA for a code width (Sec. 3.4): 4-bit 0.8
 * (fine-tuning) / 0.3 (from scratch), 2-bit 0.5 / 0.1; 3-bit, which the paper
 * does not list, takes 0.6 / 0.2 by the same rule.  Other widths: 0.9. */
float solo_beta1_default(uint32_t bits_m, int from_scratch);

/* Largest beta' with beta'/(1-beta') * r_median(b') <= beta/(1-beta) * r_median(b)
 * (Sec. 3.3, Eq. "beta-prime"), given the two median radii. */
float solo_beta1_bound(float beta, float r_median_b, float r_median_bprime);

/* Write the zero state m = v = 0 of a fresh optimizer.  The paper does not say how
 * the zero state is encoded; this library's reading: every 1st-moment code = L (the
 * code of level 0 of either codebook, not a zero byte), every 2nd-moment code = 0,
 * Delta_m = Delta_v = 0, alpha = 1 (a block whose maximum is zero has no levels to
 * tell apart; the step treats Delta = 0 as "all elements are exactly 0").  Unused
 * bits of the code words are written as zeros. */
int solo_state_init(uint32_t *m_codes, float *m_scale,
                    uint32_t *v_codes, float *v_scale, float *v_base,
                    uint64_t n, const solo_config *cfg, void *stream);

/* One optimizer step (Sec. 3.1 Eqs. 2-4 for both moments, Sec. 3.2.2 for the
 * 2nd-moment quantizer, Sec. 3.4 for blocks), in place:
 *   param   float[n], read and written
 *   grad    float[n] or bf16[n] per cfg->grad_dtype, read only
 *   states  as laid out above, read and written
 *   step    1-based count of this update (bias correction and xi stream)
 * Gradients must be finite and so must their squares in binary32 (|g| < 1.8e19);
 * the result for other inputs is unspecified for the blocks that hold them and
 * unchanged for every other block (no call hangs or faults: every loop of the
 * kernels is bounded and every table index is clamped).  A block whose new
 * maximum is below 2^-100 is stored as a zero block.
 * Performance note: on MI355X the 288 GiB of HBM behave as three regions of 96 GiB of physical
 * memory (a third of every stack).  The step of a large buffer is about 8 % slower when the two
 * code buffers lie in the same region as `param` (the one large stream that is both read and
 * written) than when they lie in another one; where `grad` and the three scale buffers lie does
 * not matter.  A process that starts on an idle GPU receives physical memory in allocation order:
 * a long-lived optimizer does well to allocate its state so that it does not end up in the
 * third of HBM that holds the parameters (python -m paper_2505_00347_amd.hbm_regions measures
 * the effect; state_region of the Python binding does it, and bench.py allocates that way). */
int solo_adamw_step(float *param, const void *grad,
                    uint32_t *m_codes, float *m_scale,
                    uint32_t *v_codes, float *v_scale, float *v_base,
                    uint64_t n, uint64_t step,
                    const solo_config *cfg, void *stream);

/* The same step with the two extras of a mixed-precision training loop (Sec. 1: 16-bit weights
 * and gradients beside the 32-bit parameters) fused into the one pass:
 *   param_bf16  bf16[n] DEVICE, 16-byte aligned, or NULL: receives every new parameter rounded
 *               to bfloat16 (nearest, ties to even), so the 16-bit weights of the next forward
 *               pass need no second sweep over the parameters
 *   grad_scale  DEVICE pointer to one float, or NULL (= 1): every gradient is multiplied by it,
 *               rounded to binary32, before anything else (reciprocal of the loss scale, a
 *               clipping coefficient computed on the GPU); must be finite
 * All other arguments, the return value and the state are those of solo_adamw_step, which is
 * this call with both pointers NULL. */
int solo_adamw_step_mp(float *param, uint16_t *param_bf16, const void *grad, const float *grad_scale,
                       uint32_t *m_codes, float *m_scale,
                       uint32_t *v_codes, float *v_scale, float *v_base,
                       uint64_t n, uint64_t step,
                       const solo_config *cfg, void *stream);

/* ---- many tensors in one launch ------------------------------------------------------------
 * A model is a set of tensors, each quantized on its own (Sec. 3.4: block-wise, small tensors
 * included), and most of them are small: one launch per tensor is bound by launch latency.
 * solo_adamw_step_multi runs the step of the same configuration over all tensors of a table in
 * one launch.  The table is built on the host from `count` descriptors of DEVICE buffers and
 * copied to device memory by the caller (who owns it, like every other buffer):
 *
 *   units = solo_multi_units(tensors, count, cfg);
 *   bytes = solo_multi_table_bytes(count, units);
 *   solo_multi_table_build(tensors, count, cfg, host_buffer, bytes, &table_flags);   // host -> host
 *   copy host_buffer to a 16-byte aligned device buffer `table`
 *   solo_adamw_step_multi(table, count, units, table_flags, grad_scale, step, cfg, stream);   // every step
 *
 * A tensor's buffers are laid out and aligned like those of solo_adamw_step (state sized by
 * solo_code_words / solo_num_blocks for its own n); param_bf16 may be NULL per tensor; tensors
 * with n == 0 are allowed.  Tensor k uses the xi stream of the flat step at
 * index_offset = cfg->index_offset + sum over the tensors before it of n rounded up to a multiple
 * of 2560, so its result is that of solo_adamw_step_mp on the tensor alone with that
 * index_offset.  The table depends on the pointers, the sizes, cfg's state format (code widths,
 * block size, codebook), grad_dtype and index_offset; it need not be rebuilt when only scalars of
 * cfg or the step change. */
typedef struct solo_tensor {
    float *param;          /* fp32[n], read and written                      */
    void *param_bf16;      /* bf16[n] or NULL: bf16 copy of the new parameters */
    const void *grad;      /* fp32[n] or bf16[n] per cfg->grad_dtype          */
    uint32_t *m_codes;
    float *m_scale;
    uint32_t *v_codes;
    float *v_scale;
    float *v_base;
    uint64_t n;            /* elements                                       */
} solo_tensor;

/* Number of work units the tensors are cut into for cfg's state format and gradient type (a unit
 * is the 2560 or 5120 elements one wavefront of that format's kernel owns, the ragged end of a
 * tensor counts one unit per 512 elements; with fp32 gradients and the linear codebook a unit is
 * 2560 elements or a tensor's shorter end, shared by five wavefronts); 0 if cfg is invalid.  At
 * most 2^24 tensors per table.  With blocks of 2048 elements a unit is one block. */
uint64_t solo_multi_units(const solo_tensor *tensors, uint32_t count, const solo_config *cfg);

/* Bytes of the table for `count` tensors and `units` units. */
size_t solo_multi_table_bytes(uint32_t count, uint64_t units);

/* Fill `table_host` (HOST memory, table_bytes >= solo_multi_table_bytes) from `tensors` (HOST
 * array of descriptors holding DEVICE pointers) and set *table_flags (SOLO_TABLE_*), which
 * solo_adamw_step_multi takes back.  Checks every pointer's alignment. */
#define SOLO_TABLE_BF16_COPY 1u   /* some tensor has a bf16 copy to write */
#define SOLO_TABLE_SHORT_BLOCK 2u /* blocks of 2048: some tensor ends in a shorter block (a second launch) */
int solo_multi_table_build(const solo_tensor *tensors, uint32_t count, const solo_config *cfg,
                           void *table_host, size_t table_bytes, uint32_t *table_flags);

/* One optimizer step over every tensor of `table_device` (DEVICE copy of a built table, 16-byte
 * aligned; `count`, `units` and `table_flags` as at build time).  grad_scale as in solo_adamw_step_mp. */
int solo_adamw_step_multi(const void *table_device, uint32_t count, uint64_t units,
                          uint32_t table_flags, const float *grad_scale, uint64_t step,
                          const solo_config *cfg, void *stream);

/* Static, human-readable text for a return code. */
const char *solo_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SOLO_H */
