// Host side of libsolo: argument checks, per-step scalars, kernel dispatch.
// See include/solo.h for the contract of every entry point.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/solo.h"
#include "solo_step.h"

namespace solo {

template <int BM, bool MDE>
hipError_t launch_step(uint32_t bits_v, uint32_t block_size, bool bf16, const StepArgs &args,
                       hipStream_t stream);
template <> hipError_t launch_step<2, false>(uint32_t, uint32_t, bool, const StepArgs &, hipStream_t);
template <> hipError_t launch_step<3, false>(uint32_t, uint32_t, bool, const StepArgs &, hipStream_t);
template <> hipError_t launch_step<4, false>(uint32_t, uint32_t, bool, const StepArgs &, hipStream_t);
template <> hipError_t launch_step<2, true>(uint32_t, uint32_t, bool, const StepArgs &, hipStream_t);
template <> hipError_t launch_step<3, true>(uint32_t, uint32_t, bool, const StepArgs &, hipStream_t);
template <> hipError_t launch_step<4, true>(uint32_t, uint32_t, bool, const StepArgs &, hipStream_t);

template <int BM, bool MDE>
hipError_t launch_multi(uint32_t bits_v, uint32_t block_size, bool bf16, const MultiArgs &args,
                        hipStream_t stream);
template <> hipError_t launch_multi<2, false>(uint32_t, uint32_t, bool, const MultiArgs &, hipStream_t);
template <> hipError_t launch_multi<3, false>(uint32_t, uint32_t, bool, const MultiArgs &, hipStream_t);
template <> hipError_t launch_multi<4, false>(uint32_t, uint32_t, bool, const MultiArgs &, hipStream_t);
template <> hipError_t launch_multi<2, true>(uint32_t, uint32_t, bool, const MultiArgs &, hipStream_t);
template <> hipError_t launch_multi<3, true>(uint32_t, uint32_t, bool, const MultiArgs &, hipStream_t);
template <> hipError_t launch_multi<4, true>(uint32_t, uint32_t, bool, const MultiArgs &, hipStream_t);

template <int BM, bool MDE>
hipError_t launch_big(uint32_t bits_v, bool bf16, const StepArgs &args, hipStream_t stream);
template <> hipError_t launch_big<2, false>(uint32_t, bool, const StepArgs &, hipStream_t);
template <> hipError_t launch_big<3, false>(uint32_t, bool, const StepArgs &, hipStream_t);
template <> hipError_t launch_big<4, false>(uint32_t, bool, const StepArgs &, hipStream_t);
template <> hipError_t launch_big<2, true>(uint32_t, bool, const StepArgs &, hipStream_t);
template <> hipError_t launch_big<3, true>(uint32_t, bool, const StepArgs &, hipStream_t);
template <> hipError_t launch_big<4, true>(uint32_t, bool, const StepArgs &, hipStream_t);

template <int BM, bool MDE>
hipError_t launch_multi_big(uint32_t bits_v, bool bf16, const MultiArgs &args, uint32_t count, bool ragged,
                            hipStream_t stream);
template <> hipError_t launch_multi_big<2, false>(uint32_t, bool, const MultiArgs &, uint32_t, bool, hipStream_t);
template <> hipError_t launch_multi_big<3, false>(uint32_t, bool, const MultiArgs &, uint32_t, bool, hipStream_t);
template <> hipError_t launch_multi_big<4, false>(uint32_t, bool, const MultiArgs &, uint32_t, bool, hipStream_t);
template <> hipError_t launch_multi_big<2, true>(uint32_t, bool, const MultiArgs &, uint32_t, bool, hipStream_t);
template <> hipError_t launch_multi_big<3, true>(uint32_t, bool, const MultiArgs &, uint32_t, bool, hipStream_t);
template <> hipError_t launch_multi_big<4, true>(uint32_t, bool, const MultiArgs &, uint32_t, bool, hipStream_t);

constexpr uint32_t kLargeBlock = 2048;      // the large-block setting (one workgroup per block)

static bool bits_ok(uint32_t b) { return b >= 2 && b <= 4; }

static bool config_ok(const solo_config *c)
{
    if (!c) return false;
    if (!bits_ok(c->bits_m) || !bits_ok(c->bits_v)) return false;
    if (c->block_size != 64 && c->block_size != 128 && c->block_size != kLargeBlock) return false;
    if (c->grad_dtype != SOLO_GRAD_FP32 && c->grad_dtype != SOLO_GRAD_BF16) return false;
    if (!(c->beta1 >= 0.0f && c->beta1 < 1.0f) || !(c->beta2 >= 0.0f && c->beta2 < 1.0f)) return false;
    if (!(c->quantile_p >= 0.0f && c->quantile_p < 1.0f)) return false;
    if (!(c->eps >= 0.0f) || !isfinite(c->eps)) return false;
    if (!isfinite(c->lr) || !isfinite(c->weight_decay)) return false;
    const uint32_t known = SOLO_FLAG_STOCHASTIC | SOLO_FLAG_M_DYNAMIC_EXPONENT | SOLO_FLAG_ADABELIEF |
                           SOLO_FLAG_COUPLED_DECAY;
    if ((c->flags & ~known) != 0 || c->reserved != 0) return false;
    if (c->index_offset % 8 != 0) return false;
    return true;
}

static bool aligned(const void *p, uintptr_t a) { return p && (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// One code word with the code of level 0 in each of `fields` slots.
__host__ __device__ static uint32_t zero_level_word(uint32_t bits, uint32_t fields)
{
    const uint32_t L = (1u << (bits - 1)) - 1u;
    uint32_t w = 0;
    for (uint32_t k = 0; k < fields; ++k) w |= L << (bits * k);
    return w;
}

__global__ void init_kernel(uint32_t *m_words, float *m_scale, uint32_t *v_words, float *v_scale,
                            float *v_base, uint64_t m_total, uint64_t v_total, uint64_t nblk,
                            uint32_t full_word, uint32_t last_word)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < m_total; i += stride)
        m_words[i] = (i + 1 == m_total) ? last_word : full_word;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < v_total; i += stride)
        v_words[i] = 0u;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nblk; i += stride) {
        m_scale[i] = 0.0f; v_scale[i] = 0.0f; v_base[i] = 1.0f;
    }
}

// 64-bit finalizer used to derive the per-step keys of the xi stream.
static uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// The scalars of one step that do not depend on the buffer: momenta, the folded step size and
// bias corrections (binary64 on the host), the rank of the quantile, the keys of the xi stream.
static void step_scalars(StepArgs &a, const solo_config *cfg, uint64_t step)
{
    a = StepArgs{};                 // pointers, n, index_offset: the caller; the tiling: the launcher of the instantiation
    a.beta1 = cfg->beta1; a.omb1 = 1.0f - cfg->beta1;
    a.beta2 = cfg->beta2; a.omb2 = 1.0f - cfg->beta2;
    const double bc1 = 1.0 - pow((double)cfg->beta1, (double)step);
    const double bc2 = 1.0 - pow((double)cfg->beta2, (double)step);
    const bool coupled = (cfg->flags & SOLO_FLAG_COUPLED_DECAY) != 0;
    const bool belief = (cfg->flags & SOLO_FLAG_ADABELIEF) != 0;
    a.decay = coupled ? 1.0f : (float)(1.0 - (double)cfg->lr * (double)cfg->weight_decay);
    a.l2 = coupled ? cfg->weight_decay : 0.0f;
    a.belief = belief ? 1u : 0u;
    a.eps_state = belief ? cfg->eps : 0.0f;
    // p <- p * decay - m^ / (sqrt(v^) * denom_scale + denom_eps): the step size lr / bc1 is folded
    // into the denominator; a step size too small to divide by (|.| < 2^-100) means no update
    const double step_size = (double)cfg->lr / bc1;
    if (fabs(step_size) < 0x1p-100) {
        a.denom_scale = 0.0f;
        a.denom_eps = INFINITY;
    } else {
        a.denom_scale = (float)(1.0 / sqrt(bc2) / step_size);
        a.denom_eps = (float)((double)cfg->eps / step_size);
    }
    a.quantile_p = cfg->quantile_p;
    // r = max(1, ceil(p * B)) with the product in binary32
    float x = ceilf(cfg->quantile_p * (float)cfg->block_size);
    a.rank_full = x < 1.0f ? 1u : (uint32_t)x;
    if (a.rank_full > cfg->block_size) a.rank_full = cfg->block_size;
    // keys of this step's xi stream
    const uint64_t gamma = 0x9E3779B97F4A7C15ull;
    const uint64_t z = cfg->seed + gamma * step;
    const uint64_t ka = mix64(z + gamma), kb = mix64(z + 2 * gamma);
    a.key0 = (uint32_t)ka; a.key1 = (uint32_t)(ka >> 32); a.key2 = (uint32_t)kb;
    a.stochastic = (cfg->flags & SOLO_FLAG_STOCHASTIC) ? 1u : 0u;
}

// Layout of a multi-tensor table: `count` entries, then one uint32 tensor index per unit.
static size_t multi_map_offset(uint32_t count) { return (size_t)count * sizeof(TensorEntry); }

}  // namespace solo

extern "C" {

size_t solo_code_words(uint64_t n, uint32_t bits)
{
    if (!solo::bits_ok(bits)) return 0;
    const uint64_t c = 32u / bits;
    return (size_t)((n + c - 1) / c);
}

size_t solo_num_blocks(uint64_t n, uint32_t block_size)
{
    return block_size ? (size_t)((n + block_size - 1) / block_size) : 0;
}

size_t solo_state_bytes(uint64_t n, const solo_config *cfg)
{
    if (!solo::config_ok(cfg)) return 0;
    return 4 * (solo_code_words(n, cfg->bits_m) + solo_code_words(n, cfg->bits_v)) +
           12 * solo_num_blocks(n, cfg->block_size);
}

float solo_beta1_default(uint32_t bits_m, int from_scratch)
{
    switch (bits_m) {
    case 4: return from_scratch ? 0.3f : 0.8f;
    case 3: return from_scratch ? 0.2f : 0.6f;
    case 2: return from_scratch ? 0.1f : 0.5f;
    default: return 0.9f;
    }
}

float solo_beta1_bound(float beta, float r_median_b, float r_median_bprime)
{
    if (!(beta >= 0.0f && beta < 1.0f) || !(r_median_b > 0.0f) || !(r_median_bprime > 0.0f)) return 0.0f;
    const double x = (double)beta / (1.0 - (double)beta) * (double)r_median_b / (double)r_median_bprime;
    return (float)(x / (1.0 + x));
}

const char *solo_strerror(int code)
{
    switch (code) {
    case SOLO_OK: return "success";
    case SOLO_E_INVALID: return "invalid argument (null or misaligned pointer, or a value out of range)";
    case SOLO_E_UNSUPPORTED: return "configuration not supported by this build";
    case SOLO_E_HIP: return "the HIP runtime reported an error at launch";
    default: return "unknown error code";
    }
}

int solo_state_init(uint32_t *m_codes, float *m_scale, uint32_t *v_codes, float *v_scale,
                    float *v_base, uint64_t n, const solo_config *cfg, void *stream)
{
    if (!solo::config_ok(cfg)) return SOLO_E_INVALID;
    if (n == 0) return SOLO_OK;
    if (!solo::aligned(m_codes, 16) || !solo::aligned(v_codes, 16) || !solo::aligned(m_scale, 4) ||
        !solo::aligned(v_scale, 4) || !solo::aligned(v_base, 4))
        return SOLO_E_INVALID;
    const uint32_t cm = 32u / cfg->bits_m;
    const uint64_t m_total = solo_code_words(n, cfg->bits_m), v_total = solo_code_words(n, cfg->bits_v);
    const uint64_t nblk = solo_num_blocks(n, cfg->block_size);
    const uint32_t rem = (uint32_t)(n % cm);
    const uint32_t full = solo::zero_level_word(cfg->bits_m, cm);
    const uint32_t last = solo::zero_level_word(cfg->bits_m, rem ? rem : cm);
    uint64_t blocks = (m_total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(solo::init_kernel, dim3((uint32_t)blocks), dim3(256), 0, (hipStream_t)stream,
                       m_codes, m_scale, v_codes, v_scale, v_base, m_total, v_total, nblk, full, last);
    return hipGetLastError() == hipSuccess ? SOLO_OK : SOLO_E_HIP;
}

int solo_adamw_step(float *param, const void *grad, uint32_t *m_codes, float *m_scale,
                    uint32_t *v_codes, float *v_scale, float *v_base, uint64_t n, uint64_t step,
                    const solo_config *cfg, void *stream)
{
    return solo_adamw_step_mp(param, nullptr, grad, nullptr, m_codes, m_scale, v_codes, v_scale, v_base,
                              n, step, cfg, stream);
}

int solo_adamw_step_mp(float *param, uint16_t *param_bf16, const void *grad, const float *grad_scale,
                       uint32_t *m_codes, float *m_scale, uint32_t *v_codes, float *v_scale,
                       float *v_base, uint64_t n, uint64_t step, const solo_config *cfg, void *stream)
{
    if (!solo::config_ok(cfg) || step == 0) return SOLO_E_INVALID;
    if (n == 0) return SOLO_OK;
    if ((param_bf16 && !solo::aligned(param_bf16, 16)) || (grad_scale && !solo::aligned(grad_scale, 4)))
        return SOLO_E_INVALID;
    if (!solo::aligned(param, 16) || !solo::aligned(grad, 16) || !solo::aligned(m_codes, 16) ||
        !solo::aligned(v_codes, 16) || !solo::aligned(m_scale, 4) || !solo::aligned(v_scale, 4) ||
        !solo::aligned(v_base, 4))
        return SOLO_E_INVALID;
    if (n > (1ull << 40)) return SOLO_E_UNSUPPORTED;

    solo::StepArgs a;
    solo::step_scalars(a, cfg, step);
    a.param = param; a.grad = grad;
    a.m_words = m_codes; a.m_scale = m_scale;
    a.v_words = v_codes; a.v_scale = v_scale; a.v_base = v_base;
    a.n = n;
    a.index_offset = cfg->index_offset;
    a.param_bf16 = param_bf16;
    a.grad_scale = grad_scale;

    const bool bf16 = cfg->grad_dtype == SOLO_GRAD_BF16;
    const bool mde = (cfg->flags & SOLO_FLAG_M_DYNAMIC_EXPONENT) != 0;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    if (cfg->block_size == solo::kLargeBlock) {
        switch (cfg->bits_m) {
        case 2: e = mde ? solo::launch_big<2, true>(cfg->bits_v, bf16, a, s) : solo::launch_big<2, false>(cfg->bits_v, bf16, a, s); break;
        case 3: e = mde ? solo::launch_big<3, true>(cfg->bits_v, bf16, a, s) : solo::launch_big<3, false>(cfg->bits_v, bf16, a, s); break;
        case 4: e = mde ? solo::launch_big<4, true>(cfg->bits_v, bf16, a, s) : solo::launch_big<4, false>(cfg->bits_v, bf16, a, s); break;
        default: return SOLO_E_UNSUPPORTED;
        }
        return e == hipSuccess ? SOLO_OK : SOLO_E_HIP;
    }
    switch (cfg->bits_m) {
    case 2: e = mde ? solo::launch_step<2, true>(cfg->bits_v, cfg->block_size, bf16, a, s)
                    : solo::launch_step<2, false>(cfg->bits_v, cfg->block_size, bf16, a, s); break;
    case 3: e = mde ? solo::launch_step<3, true>(cfg->bits_v, cfg->block_size, bf16, a, s)
                    : solo::launch_step<3, false>(cfg->bits_v, cfg->block_size, bf16, a, s); break;
    case 4: e = mde ? solo::launch_step<4, true>(cfg->bits_v, cfg->block_size, bf16, a, s)
                    : solo::launch_step<4, false>(cfg->bits_v, cfg->block_size, bf16, a, s); break;
    default: return SOLO_E_UNSUPPORTED;
    }
    return e == hipSuccess ? SOLO_OK : SOLO_E_HIP;
}

uint64_t solo_multi_units(const solo_tensor *tensors, uint32_t count, const solo_config *cfg)
{
    if (!tensors || !solo::config_ok(cfg)) return 0;
    const bool mde = (cfg->flags & SOLO_FLAG_M_DYNAMIC_EXPONENT) != 0;
    uint64_t units = 0;
    if (cfg->block_size == solo::kLargeBlock) {                  // one unit per block
        for (uint32_t k = 0; k < count; ++k) units += (tensors[k].n + solo::kLargeBlock - 1) / solo::kLargeBlock;
        return units;
    }
    if (solo::multi_chunked(cfg->grad_dtype == SOLO_GRAD_BF16, mde)) {
        for (uint32_t k = 0; k < count; ++k) units += (tensors[k].n + solo::kTileUnit - 1) / solo::kTileUnit;
        return units;
    }
    const uint64_t unit = (uint64_t)solo::unit_elems(cfg->bits_m, cfg->bits_v, cfg->block_size, mde);
    for (uint32_t k = 0; k < count; ++k) units += solo::multi_full_units(tensors[k].n, unit) + solo::multi_ragged_chunks(tensors[k].n, unit);
    return units;
}

size_t solo_multi_table_bytes(uint32_t count, uint64_t units)
{
    return solo::multi_map_offset(count) + (size_t)units * sizeof(uint32_t);
}

int solo_multi_table_build(const solo_tensor *tensors, uint32_t count, const solo_config *cfg,
                           void *table_host, size_t table_bytes, uint32_t *table_flags)
{
    if (!solo::config_ok(cfg) || !tensors || !table_host || !table_flags || count == 0) return SOLO_E_INVALID;
    if (count > solo::kMapTensorMask) return SOLO_E_UNSUPPORTED;      // the map keeps the tensor index in 24 bits
    const uint64_t units = solo_multi_units(tensors, count, cfg);
    if (table_bytes < solo_multi_table_bytes(count, units)) return SOLO_E_INVALID;
    if (units > (1ull << 31)) return SOLO_E_UNSUPPORTED;
    const bool big = cfg->block_size == solo::kLargeBlock;
    const uint64_t unit = big ? solo::kLargeBlock
                              : (uint64_t)solo::unit_elems(cfg->bits_m, cfg->bits_v, cfg->block_size,
                                                           (cfg->flags & SOLO_FLAG_M_DYNAMIC_EXPONENT) != 0);
    const bool chunked = !big && solo::multi_chunked(cfg->grad_dtype == SOLO_GRAD_BF16,
                                             (cfg->flags & SOLO_FLAG_M_DYNAMIC_EXPONENT) != 0);
    solo::TensorEntry *entries = static_cast<solo::TensorEntry *>(table_host);
    uint32_t *map = reinterpret_cast<uint32_t *>(static_cast<char *>(table_host) + solo::multi_map_offset(count));
    uint64_t unit0 = 0, xi_offset = cfg->index_offset;
    uint32_t flags = 0;
    for (uint32_t k = 0; k < count; ++k) {
        const solo_tensor &t = tensors[k];
        if (t.n > (1ull << 40)) return SOLO_E_UNSUPPORTED;
        if (t.n != 0 && (!solo::aligned(t.param, 16) || !solo::aligned(t.grad, 16) ||
                         !solo::aligned(t.m_codes, 16) || !solo::aligned(t.v_codes, 16) ||
                         !solo::aligned(t.m_scale, 4) || !solo::aligned(t.v_scale, 4) ||
                         !solo::aligned(t.v_base, 4) || (t.param_bf16 && !solo::aligned(t.param_bf16, 16))))
            return SOLO_E_INVALID;
        if (t.n != 0 && t.param_bf16) flags |= SOLO_TABLE_BF16_COPY;
        solo::TensorEntry &e = entries[k];
        e.param = t.param; e.param_bf16 = static_cast<uint16_t *>(t.param_bf16); e.grad = t.grad;
        e.m_words = t.m_codes; e.m_scale = t.m_scale;
        e.v_words = t.v_codes; e.v_scale = t.v_scale; e.v_base = t.v_base;
        e.n = t.n; e.unit0 = unit0;
        e.index_offset = xi_offset;
        e.reserved = 0;
        // full units first, then the 512-element iterations of the ragged end, one entry each
        // (chunked formats: one entry per 2560-element unit, the shorter last one included)
        // (blocks of 2048: one entry per full block, then one flagged entry for a shorter last block)
        const uint64_t nf = chunked ? (t.n + solo::kTileUnit - 1) / solo::kTileUnit : solo::multi_full_units(t.n, unit);
        const uint64_t nc = chunked ? 0 : big ? (t.n % unit ? 1 : 0) : solo::multi_ragged_chunks(t.n, unit);
        if (big && nc) flags |= SOLO_TABLE_SHORT_BLOCK;
        for (uint64_t u = 0; u < nf; ++u) map[unit0 + u] = k;
        for (uint64_t c = 0; c < nc; ++c) map[unit0 + nf + c] = k | ((uint32_t)c << solo::kMapChunkShift) | solo::kMapRagged;
        unit0 += nf + nc;
        xi_offset += (t.n + solo::kTileUnit - 1) / solo::kTileUnit * (uint64_t)solo::kTileUnit;
    }
    *table_flags = flags;
    return SOLO_OK;
}

int solo_adamw_step_multi(const void *table_device, uint32_t count, uint64_t units, uint32_t table_flags,
                          const float *grad_scale, uint64_t step, const solo_config *cfg, void *stream)
{
    if (!solo::config_ok(cfg) || step == 0) return SOLO_E_INVALID;
    if (units == 0) return SOLO_OK;
    if (count == 0 || !solo::aligned(table_device, 16) || (grad_scale && !solo::aligned(grad_scale, 4)))
        return SOLO_E_INVALID;
    if (units > (1ull << 31)) return SOLO_E_UNSUPPORTED;
    solo::MultiArgs ma;
    solo::step_scalars(ma.common, cfg, step);
    ma.common.grad_scale = grad_scale;
    ma.entries = static_cast<const solo::TensorEntry *>(table_device);
    ma.unit_map = reinterpret_cast<const uint32_t *>(static_cast<const char *>(table_device) +
                                                     solo::multi_map_offset(count));
    ma.total_units = units;
    ma.any_bf16_copy = (table_flags & SOLO_TABLE_BF16_COPY) ? 1u : 0u;
    const bool bf16 = cfg->grad_dtype == SOLO_GRAD_BF16;
    const bool mde = (cfg->flags & SOLO_FLAG_M_DYNAMIC_EXPONENT) != 0;
    // wavefronts of the launch: one per unit, or five per 2560-element unit of a chunked format
    const uint64_t slots = solo::multi_chunked(bf16, mde) ? units * (solo::kTileUnit / solo::kIter) : units;
    ma.groups_per_xcd = ((slots + solo::kWaves - 1) / solo::kWaves + solo::kXcds - 1) / solo::kXcds;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    if (cfg->block_size == solo::kLargeBlock) {
        const bool ragged = (table_flags & SOLO_TABLE_SHORT_BLOCK) != 0;
        switch (cfg->bits_m) {
        case 2: e = mde ? solo::launch_multi_big<2, true>(cfg->bits_v, bf16, ma, count, ragged, s)
                        : solo::launch_multi_big<2, false>(cfg->bits_v, bf16, ma, count, ragged, s); break;
        case 3: e = mde ? solo::launch_multi_big<3, true>(cfg->bits_v, bf16, ma, count, ragged, s)
                        : solo::launch_multi_big<3, false>(cfg->bits_v, bf16, ma, count, ragged, s); break;
        case 4: e = mde ? solo::launch_multi_big<4, true>(cfg->bits_v, bf16, ma, count, ragged, s)
                        : solo::launch_multi_big<4, false>(cfg->bits_v, bf16, ma, count, ragged, s); break;
        default: return SOLO_E_UNSUPPORTED;
        }
        return e == hipSuccess ? SOLO_OK : SOLO_E_HIP;
    }
    switch (cfg->bits_m) {
    case 2: e = mde ? solo::launch_multi<2, true>(cfg->bits_v, cfg->block_size, bf16, ma, s)
                    : solo::launch_multi<2, false>(cfg->bits_v, cfg->block_size, bf16, ma, s); break;
    case 3: e = mde ? solo::launch_multi<3, true>(cfg->bits_v, cfg->block_size, bf16, ma, s)
                    : solo::launch_multi<3, false>(cfg->bits_v, cfg->block_size, bf16, ma, s); break;
    case 4: e = mde ? solo::launch_multi<4, true>(cfg->bits_v, cfg->block_size, bf16, ma, s)
                    : solo::launch_multi<4, false>(cfg->bits_v, cfg->block_size, bf16, ma, s); break;
    default: return SOLO_E_UNSUPPORTED;
    }
    return e == hipSuccess ? SOLO_OK : SOLO_E_HIP;
}

}  // extern "C"
