// Device code of the fused SOLO AdamW step for gfx950 (wave64).
//
// Work decomposition.  A buffer is cut into super-tiles of 2560 or 5120
// elements (2560 is a multiple of every block size and of 16, 10 and 8 codes
// per word, so a super-tile owns whole blocks and whole code words; the
// larger size is used wherever the LDS image of the tile's state still lets
// five workgroups share a CU).  One wavefront owns one super-tile and walks
// it in iterations of 512 elements; a lane owns 8 consecutive elements per
// iteration, so a block of 128 (64) elements is held by 16 (8) neighbouring
// lanes, i.e. one DPP row (half row), and every per-block reduction is a few
// DPP steps.  Nothing is shared between wavefronts but a constant table: the
// only workgroup barrier sits before the first tile is touched.
//
// step_tile() is the whole step for one super-tile; step_kernel runs it over
// a flat buffer (full tiles, and the ragged end with bounds checks),
// multi_kernel over the tensors of a caller-built table.  Full super-tiles of
// formats whose state image is small enough take step_tile16() instead: 16
// elements per lane, 8 (4) lanes per block, 1024 elements per iteration, four
// wavefronts per SIMD instead of five (fewer instructions per element; see
// there).  A ragged end, a short or mid-size buffer (chunked_up_to()) and the
// formats whose streaming code sits at the register limit run step_tile() in
// its `alone` form: one wavefront per 512-element iteration, which stages and
// writes back only its own words (multi_chunk_kernel: the same over a table).
// The pieces that these functions and the large-block functions of
// solo_step_big.h have in common (layout transposition, level tables, EMAs
// and parameter, encoders, image update, write-back) exist once, as inlined
// helpers in front of step_tile().
//
// The kernel is bound by vector-ALU issue as much as by HBM (packed FP32 is
// off, so a CU retires 64 lane-operations per clock: about 80 per parameter at
// 70 % of the HBM peak).  Everything below is shaped by instruction count:
//   * both dequantizers are table look-ups: the lanes of a group compute the
//     block's level tables (alpha^q * Delta_v, (c-L) * Delta_m/L) once and park
//     them in LDS; an element costs one bit-field extract, one address add and
//     one ds_read per moment;
//   * the p-quantile is exact: each lane sorts its 8 values with min3/med3/max3
//     (32 instructions), parks the sorted column in LDS, and the group runs r
//     rounds of "row minimum by DPP, the lane that holds it pops its column";
//     a scalar population count detects the rounds in which two lanes tie and
//     only those rounds pay for the tie-break;
//   * the two per-block divisions share one IEEE division sequence (even lanes
//     divide x_p by Delta_v, odd lanes L by Delta_m);
//   * the base alpha = rho^(1/K) is found by testing G consecutive binary32
//     candidates around a hardware exp2/log2 guess, one per lane;
//   * codes are rounded in the float domain and accumulated with FMAs
//     (acc += code * 2^(b j)); xi is built as a float in [1, 2) by one
//     bit-align of the element's finalized word of the xi stream (one hash
//     per 8 elements gives a start and a stride, every word is then mixed
//     on its own).
//
// Arithmetic contract (what makes the stored bytes reproducible): every value
// that decides a code or a scale is computed in binary32, one rounding per
// operation in a fixed order, no contraction except the two explicit fused
// multiply-adds of the EMAs.  Only the 2nd-moment code decision uses the
// hardware log2 (a result can differ from another implementation at an exact
// rounding tie), and the parameter update uses the hardware sqrt/rcp.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#ifndef SOLO_MIN_WAVES
#define SOLO_MIN_WAVES 5   // wavefronts per SIMD the register allocator must leave room for
#endif

namespace solo {

constexpr int kTileUnit = 2560;    // lcm of the block sizes and of 16, 10 and 8 codes per word
constexpr int kIter = 512;         // elements per iteration (64 lanes x 8)
constexpr int kLdsPerCu = 160 * 1024;
#ifndef SOLO_WAVES
#define SOLO_WAVES 4
#endif
constexpr int kWaves = SOLO_WAVES; // wavefronts per workgroup
constexpr int kXcds = 8;           // accelerator dies of an MI355X (each has its own L2)
constexpr int kColStride = 12;     // words per lane in the sorted-column area (8 keys, +inf, pad)
constexpr int kIter16 = 1024;      // elements per iteration of the wide path (64 lanes x 16)
constexpr int kColStride16 = 18;   // its column stride (16 keys, +inf, pad; columns are written 8 bytes at a time)
constexpr int kWideWaves = 4;      // wavefronts per SIMD the wide path is compiled for
constexpr float kTiny = 0x1p-100f; // block maxima below this are stored as 0
constexpr float kRhoMin = 0x1p-64f;
constexpr uint32_t kInfBits = 0x7F800000u;
constexpr uint32_t kOneBits = 0x3F800000u;

struct StepArgs {
    float *param;
    const void *grad;
    uint32_t *m_words;
    float *m_scale;
    uint32_t *v_words;
    float *v_scale;
    float *v_base;
    uint64_t n;             // elements
    uint64_t n_tiles_full;  // super-tiles that lie entirely inside [0, n)
    uint64_t tail_tile0;    // first 2560-element unit behind them (the ragged end)
    uint64_t tail_chunks;   // 512-element iterations of the ragged end, one wavefront each
    uint64_t wg_per_xcd;    // workgroups per XCD: ceil(ceil(n_tiles_full / kWaves) / 8)
    uint64_t index_offset;  // global index of element 0 (multiple of 8)
    float beta1, omb1, beta2, omb2;
    float decay;            // 1 - lr * weight_decay
    float denom_scale;      // (1 / sqrt(1 - beta2^t)) / step_size, step_size = lr / (1 - beta1^t)
    float denom_eps;        // eps / step_size  (lr == 0: scale 0 and eps +inf, the update vanishes)
    float quantile_p;
    uint32_t rank_full;     // rank of the quantile in a full block
    uint32_t key0, key1, key2;
    uint32_t stochastic;    // 0: xi = 0
    // variants of the step (all uniform over the launch)
    uint16_t *param_bf16;   // bf16 copy of the new parameters, written beside them (null: none)
    const float *grad_scale;// device scalar every gradient is multiplied by first (null: 1)
    float l2;               // Adam with coupled decay: weight_decay, g <- g + l2 * p; otherwise 0
    float eps_state;        // AdaBelief: eps, added to the 2nd EMA itself at every step
    uint32_t belief;        // AdaBelief: the 2nd EMA follows (g - m^)^2 instead of g^2
};

// One tensor of a multi-tensor launch, as the kernel reads it from the caller's table
// (device memory; built on the host by solo_multi_table_build).
struct TensorEntry {
    float *param;
    uint16_t *param_bf16;   // may be null
    const void *grad;
    uint32_t *m_words;
    float *m_scale;
    uint32_t *v_words;
    float *v_scale;
    float *v_base;
    uint64_t n;             // elements of the tensor
    uint64_t unit0;         // index of the tensor's first unit among all units of the table
    uint64_t index_offset;  // global index of the tensor's element 0 in the xi stream
    uint64_t reserved;
};
static_assert(sizeof(TensorEntry) == 96, "table layout");

// An entry of the unit map: the tensor's index; for the ragged end of a tensor, which is cut into
// its 512-element iterations with one entry (one wavefront) each, also the iteration and a flag.
constexpr uint32_t kMapTensorMask = 0x00FFFFFFu, kMapRagged = 0x80000000u;
constexpr int kMapChunkShift = 24;
inline uint64_t multi_full_units(uint64_t n, uint64_t unit) { return n / unit; }
inline uint64_t multi_ragged_chunks(uint64_t n, uint64_t unit)
{
    // up to the end of the last code word (80 = lcm of 16, 10 and 8 codes per word), whose unused
    // fields are written as zeros like every other field
    return n % unit ? ((n + 79) / 80 * 80 - n / unit * unit + 511) / 512 : 0;
}

struct MultiArgs {
    StepArgs common;              // the scalars of the step; pointers, n and index_offset come from the table
    const TensorEntry *entries;
    const uint32_t *unit_map;     // tensor index of every unit
    uint64_t total_units;
    uint64_t groups_per_xcd;      // groups of kWaves units per XCD
    uint32_t any_bf16_copy;       // some tensor of the table has a bf16 copy to write
};

// Elements per unit of a multi-tensor table for a format: the super-tile size of its kernels.
inline int unit_elems(uint32_t bits_m, uint32_t bits_v, uint32_t block_size, bool mde);

// ---------------------------------------------------------------- cross-lane

template <int CTRL>
__device__ __forceinline__ uint32_t dpp(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, false);
}

// Butterfly over the G (4, 8 or 16) lanes that hold one block: lane^1 and lane^2
// by quad permutes, then mirror inside the half row, then inside the row.
// Every lane ends with the result of its whole group.
template <int G, typename Op>
__device__ __forceinline__ uint32_t group_reduce(uint32_t x, Op op)
{
    x = op(x, dpp<0xB1>(x));    // quad_perm [1,0,3,2]
    x = op(x, dpp<0x4E>(x));    // quad_perm [2,3,0,1]
    if (G >= 8) x = op(x, dpp<0x141>(x));   // row_half_mirror
    if (G == 16) x = op(x, dpp<0x140>(x));  // row_mirror
    return x;
}

struct UMin { __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a < b ? a : b; } };
struct UMax { __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a > b ? a : b; } };

__device__ __forceinline__ uint32_t f2u(float x) { return __builtin_bit_cast(uint32_t, x); }
__device__ __forceinline__ float u2f(uint32_t x) { return __builtin_bit_cast(float, x); }
__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }
__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
// Median of three bit patterns of non-negative floats (they order like the floats).
__device__ __forceinline__ uint32_t umed3(uint32_t a, uint32_t b, uint32_t c)
{
    return f2u(__builtin_amdgcn_fmed3f(u2f(a), u2f(b), u2f(c)));
}

// The bits of a wave-wide ballot that belong to this lane's group, shifted down.
__device__ __forceinline__ uint32_t group_bits(uint64_t ballot, uint32_t lane, uint32_t gshift, uint32_t gmask)
{
    const uint32_t half = lane < 32u ? (uint32_t)ballot : (uint32_t)(ballot >> 32);
    return (half >> gshift) & gmask;
}

__device__ __forceinline__ void cswap(uint32_t &a, uint32_t &b)
{
    const uint32_t lo = umin(a, b), hi = umax(a, b);
    a = lo; b = hi;
}

// Sorts four keys with seven instructions: a three-sort (min3, med3, max3),
// then the fourth key is placed by one min, two med3 and one max.
__device__ __forceinline__ void sort4(uint32_t &a, uint32_t &b, uint32_t &c, uint32_t &d)
{
    const uint32_t lo = umin(umin(a, b), c), mid = umed3(a, b, c), hi = umax(umax(a, b), c);
    a = umin(lo, d); b = umed3(lo, mid, d); c = umed3(mid, hi, d); d = umax(hi, d);
}

// Eight keys: two four-sorts and Batcher's odd-even merge of the halves.
__device__ __forceinline__ void sort8(uint32_t (&k)[8])
{
    sort4(k[0], k[1], k[2], k[3]);
    sort4(k[4], k[5], k[6], k[7]);
    cswap(k[0], k[4]); cswap(k[1], k[5]); cswap(k[2], k[6]); cswap(k[3], k[7]);
    cswap(k[2], k[4]); cswap(k[3], k[5]);
    cswap(k[1], k[2]); cswap(k[3], k[4]); cswap(k[5], k[6]);
}

// ------------------------------------------------------------------- pieces

__device__ __forceinline__ uint32_t mix32(uint32_t h)
{
    h ^= h >> 16; h *= 0x85EBCA6Bu;
    h ^= h >> 13; h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h;
}

// Finalizer of an element's word of the xi stream: the group's words X + j Y lie on an arithmetic
// progression; xorshift and one 24-bit multiplication (full rate; the low 24 bits of the
// xorshifted word contain every bit of w) make the eight elements of a group jointly independent.
constexpr uint32_t kXiMul = 0xC2B2AFu;
__host__ __device__ constexpr uint32_t xi_finalize_ref(uint32_t w)
{
    return ((w ^ (w >> 15)) & 0xFFFFFFu) * kXiMul;
}
__device__ __forceinline__ uint32_t xi_finalize(uint32_t w)
{
    return __umul24(w ^ (w >> 15), kXiMul);
}
// A word whose finalized top 23 bits are 100...0, i.e. xi = 0 (deterministic rounding).
constexpr uint32_t kXiZeroWord = 0x1B29A9u;
static_assert((xi_finalize_ref(kXiZeroWord) >> 9) == 0x400000u, "xi = 0 word");

// Level alpha^q of the log codebook for a run-time q, by binary powering in the
// dequantizer's fixed order: the selected powers a, a^2, a^4, a^8 are
// multiplied from the lowest bit of q up.
template <int BV>
__device__ __forceinline__ float log_level(uint32_t q, float P1, float P2, float P4, float P8)
{
    float y = (q & 1u) ? P1 : 1.0f;
    y = (q & 2u) ? y * P2 : y;
    if (BV >= 3) y = (q & 4u) ? y * P4 : y;
    if (BV >= 4) y = (q & 8u) ? y * P8 : y;
    return y;
}

// Last level alpha^K, K = 2^BV - 1: ((a * a^2) * a^4) * a^8.
template <int BV>
__device__ __forceinline__ float last_level(float a)
{
    const float a2 = a * a;
    float r = a * a2;
    if (BV >= 3) { const float a4 = a2 * a2; r = r * a4; if (BV >= 4) { const float a8 = a4 * a4; r = r * a8; } }
    return r;
}

// Walks y (bits of a binary32 in (0, 1]) to the largest value whose last level
// does not exceed rho.  Both walks are bounded; used only when the parallel
// candidate test did not bracket the answer.
template <int BV>
__device__ __noinline__ uint32_t walk_base(uint32_t y, float rho)
{
    for (int i = 0; i < 4096 && last_level<BV>(u2f(y)) > rho; ++i) --y;
    for (int i = 0; i < 4096 && y < kOneBits && last_level<BV>(u2f(y + 1)) <= rho; ++i) ++y;
    return y;
}

// The base alpha = rho^(1/K) as stored: the largest binary32 whose last level does not exceed rho.
// The hardware exp2/log2 give a guess that is a few units in the last place off; the lanes of the
// group test the 16 consecutive binary32 values yb - 8 .. yb + 7 around it in parallel (one per
// lane in a group of 16, two or four per lane in a group of 8 or 4) and count those that fit.  Only a guess
// further off than that takes the bounded walk.  Returns the bit pattern; meaningful if rho < 1.
template <int BV, int G>
__device__ __forceinline__ uint32_t search_base(float rho, bool need, uint32_t lane, uint32_t lig, uint32_t gshift)
{
    constexpr int K = (1 << BV) - 1;
    constexpr float invK = 1.0f / (float)K;
    constexpr uint32_t GMASK = (1u << G) - 1u;
    static_assert(G == 4 || G == 8 || G == 16, "group of 4, 8 or 16 lanes");
    const float y0 = __builtin_amdgcn_exp2f(__builtin_amdgcn_logf(rho) * invK);
    const uint32_t yb = umed3(f2u(y0), 0x00800000u, kOneBits);
    uint32_t cnt;
    if (G == 16) {
        const uint32_t cand = umin(yb + lig - 8u, kOneBits);
        const bool fits = last_level<BV>(u2f(cand)) <= rho;
        cnt = (uint32_t)__builtin_popcount(group_bits(__builtin_amdgcn_ballot_w64(fits), lane, gshift, GMASK));
    } else {                                   // 16 / G candidates per lane
        cnt = 0;
#pragma unroll
        for (int c = 0; c < 16 / G; ++c) {
            const uint32_t cand = umin(yb + lig + (uint32_t)(c * G) - 8u, kOneBits);
            const bool fits = last_level<BV>(u2f(cand)) <= rho;
            cnt += (uint32_t)__builtin_popcount(group_bits(__builtin_amdgcn_ballot_w64(fits), lane, gshift, GMASK));
        }
    }
    uint32_t ab = umin(yb + cnt - 9u, kOneBits);
    // not bracketed (all or none of the candidates fit): walk from the nearest end
    const bool open = need && (cnt == 0u || cnt == 16u);
    if (__builtin_amdgcn_ballot_w64(open) != 0) {
        if (open) ab = walk_base<BV>(cnt == 0u ? yb - 8u : ab, rho);
    }
    return ab;
}

// Eight consecutive BITS-wide codes starting at slot `slot` of word w0 (the
// run may continue in w1 for 3-bit codes, ten to a word).
template <int BITS>
__device__ __forceinline__ uint32_t extract8(uint32_t w0, uint32_t w1, uint32_t slot)
{
    if (BITS == 3) {
        const uint64_t both = (uint64_t)w0 | ((uint64_t)w1 << 30);
        return (uint32_t)(both >> (3u * slot)) & 0xFFFFFFu;
    }
    return w0 >> (BITS * slot);   // 2-bit: slot 0 or 8; 4-bit: slot 0
}

// Signed dynamic-exponent (DE) levels of the 1st moment (App. A of the paper): the first bit
// is the sign, the other b-1 bits spend E leading zeros on the exponent 10^-E, one indicator
// bit, and the rest on a linear fraction over [0.1, 1].  Exponent step i (scale 10^(-(b-2)+i))
// owns 2^i fraction cells, each represented by the mean of its boundaries, and the two codes
// left over are the levels 0 and 1.  Non-negative levels in increasing order:
// pos(0) = 0, pos(1..L) the cell means, pos(L+1) = 1, L = 2^(b-1) - 1; the negative side
// mirrors pos(1..L) (there is no level -1).
template <int BM>
struct DeLevels {
    static constexpr int L = (1 << (BM - 1)) - 1;
    static constexpr double pos(int j)
    {
        if (j <= 0) return 0.0;
        if (j > L) return 1.0;
        constexpr double tenth[8] = {1.0, 0.1, 0.01, 0.001, 1e-4, 1e-5, 1e-6, 1e-7};
        int i = 0, first = 1;                       // exponent step i holds cells [first, first + 2^i)
        while (j >= first + (1 << i)) { first += (1 << i); ++i; }
        const int cells = 1 << i, c = j - first;
        const double lo = 0.1 + 0.9 * (double)c / (double)cells;
        const double hi = 0.1 + 0.9 * (double)(c + 1) / (double)cells;
        return tenth[(BM - 2) - i] * (lo + hi) / 2.0;
    }
    // Tables evaluated at compile time: the signed levels by code (2L + 2 of them) and the
    // midpoints between neighbouring non-negative levels (the rounding boundaries of |z|).
    struct Tables {
        float level[2 * L + 2];
        float mid[L + 1];
        constexpr Tables() : level(), mid()
        {
            for (int c = 0; c < 2 * L + 2; ++c) level[c] = c >= L ? (float)pos(c - L) : -(float)pos(L - c);
            for (int k = 0; k <= L; ++k) mid[k] = (float)((pos(k) + pos(k + 1)) / 2.0);
        }
    };
    static constexpr Tables tab = Tables();
    // level of a run-time code (used once per wavefront): a select chain over literals
    __device__ static float level(uint32_t code)
    {
        float r = 0.0f;
#pragma unroll
        for (int c = 0; c < 2 * L + 2; ++c) r = (code == (uint32_t)c) ? tab.level[c] : r;
        return r;
    }
};

// Rounding to the DE levels by one table look-up.  |z| <= 1 is cut into buckets by the top of
// its binary32 pattern (the exponent and two fraction bits); the buckets are narrow enough that
// none holds more than one rounding boundary, so a bucket knows the two neighbouring codes its
// values can take.  One 8-byte entry per bucket and sign, { t, base }: the code is
// base + (z > t).  For z >= 0, t is the boundary and base the code at or below it.  For z < 0
// the code falls as |z| grows, so base is the code beyond the boundary and t = -nextup(boundary):
// z > t exactly when |z| <= boundary.  Buckets without a boundary (and the negative buckets
// beyond the last negative level) have t = +inf.  Entry 0 also serves every smaller magnitude.
template <int BM>
struct DeBuckets {
    static constexpr int L = DeLevels<BM>::L;
    static constexpr uint32_t bucket(float x) { return (__builtin_bit_cast(uint32_t, x) >> 21) & 0x3FFu; }
    static constexpr uint32_t kLo = bucket(DeLevels<BM>::tab.mid[0]) - 1u;
    static constexpr uint32_t kHi = bucket(1.0f);       // |z| can reach 1 + 2^-23
    static constexpr int N = (int)(kHi - kLo) + 1;
    struct Table {
        uint32_t w[2 * N][2];
        bool one_boundary_per_bucket;
        constexpr Table() : w(), one_boundary_per_bucket(true)
        {
            constexpr uint32_t kInf = 0x7F800000u;
            for (int b = 0; b < N; ++b) {
                int below = 0, inside = 0;              // boundaries in lower buckets / in this one
                uint32_t thr = kInf;
                for (int k = 0; k <= L; ++k) {
                    const uint32_t bk = bucket(DeLevels<BM>::tab.mid[k]);
                    if (bk < kLo + (uint32_t)b) ++below;
                    if (bk == kLo + (uint32_t)b) { ++inside; thr = __builtin_bit_cast(uint32_t, DeLevels<BM>::tab.mid[k]); }
                }
                if (inside > 1) one_boundary_per_bucket = false;
                const int j0 = below, j1 = below + inside;
                w[2 * b][0] = thr;                                       // z >= 0
                w[2 * b][1] = (uint32_t)(L + j0);
                const int n0 = L - (j0 < L ? j0 : L), n1 = L - (j1 < L ? j1 : L);   // z < 0: no level -1
                w[2 * b + 1][0] = n0 != n1 ? ((thr + 1u) | 0x80000000u) : kInf;
                w[2 * b + 1][1] = (uint32_t)n1;
            }
        }
    };
    static constexpr Table tab = Table();
    static_assert(tab.one_boundary_per_bucket, "two fraction bits must separate the boundaries");
};

// ------------------------------------------------------------------- kernel

// LDS accessed through 32-bit byte addresses, so that a table index can be
// OR-ed into an aligned base with one v_and_or_b32.
typedef __attribute__((address_space(3))) float lds_f32_t;
typedef __attribute__((address_space(3))) uint32_t lds_u32_t;
__device__ __forceinline__ uint32_t lds_addr(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}
__device__ __forceinline__ float lds_f32(uint32_t addr) { return *(lds_f32_t *)(uintptr_t)addr; }
__device__ __forceinline__ uint32_t lds_u32(uint32_t addr) { return *(lds_u32_t *)(uintptr_t)addr; }

// Streaming accesses: 128-bit, every instruction covers one contiguous kilobyte of the
// wavefront's chunk, non-temporal (nothing of p or g is touched twice).
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) u32x2_t lds_u32x2_t;
__device__ __forceinline__ float4 stream_load_f4(const float *p)
{
    const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint4 stream_load_u4(const void *p)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
// Streaming stores are non-temporal and written through at device scope (sc1): the data leaves
// the L2 at once instead of waiting for an eviction, which drains the write stream more evenly
// (0.5-1 % on the whole step over a plain non-temporal store).
// (Written as assembly because no builtin sets sc1.  The s_nop covers the two wait states that a
// store of more than 64 bits needs before its data registers may be overwritten: the compiler
// keeps that distance for its own stores but does not look inside an asm block.)
__device__ __forceinline__ void stream_store_u4(void *p, u32x4_t v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void stream_store_f4(float *p, float4 x)
{
    const u32x4_t v = {__builtin_bit_cast(uint32_t, x.x), __builtin_bit_cast(uint32_t, x.y),
                       __builtin_bit_cast(uint32_t, x.z), __builtin_bit_cast(uint32_t, x.w)};
    stream_store_u4(p, v);
}

// Two binary32 values rounded to bfloat16 (nearest, ties to even: the hardware conversion),
// the first in the low half.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const bf16x2_t v = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, v);
}

template <bool V> struct BoolTag { static constexpr bool value = V; };

// Parameters and gradients of one lane and iteration as they come from memory.  In the
// full-tile kernel the fp32 streams arrive in the coalesced layout (lane l holds elements
// 4l..4l+3 and 256+4l..256+4l+3 of the 512-element chunk) and are transposed through LDS
// to the lane's 8 consecutive elements; bf16 gradients (16 bytes per lane) already are
// both.  The tail kernel loads element by element with bounds checks.
struct RawPG { float4 p0, p1; uint4 g0, g1; };

template <bool BF16, bool TAIL>
__device__ __forceinline__ RawPG load_pg(const StepArgs &a, uint64_t chunk_e0, uint32_t lane)
{
    RawPG r;
    if (!TAIL) {
        const float *pp = a.param + chunk_e0 + lane * 4u;
        r.p0 = stream_load_f4(pp); r.p1 = stream_load_f4(pp + 256);
        if (BF16) {
            r.g0 = stream_load_u4(static_cast<const uint16_t *>(a.grad) + chunk_e0 + lane * 8u);
            r.g1 = make_uint4(0, 0, 0, 0);
        } else {
            const float *gp = static_cast<const float *>(a.grad) + chunk_e0 + lane * 4u;
            r.g0 = stream_load_u4(gp); r.g1 = stream_load_u4(gp + 256);
        }
    } else {                                   // element-wise, bounds-checked
        const uint64_t e0 = chunk_e0 + lane * 8u;
        float p[8]; uint32_t g[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool ok = (e0 + j) < a.n;
            p[j] = ok ? a.param[e0 + j] : 0.0f;
            if (BF16) g[j] = ok ? (uint32_t)static_cast<const uint16_t *>(a.grad)[e0 + j] : 0u;
            else      g[j] = ok ? static_cast<const uint32_t *>(a.grad)[e0 + j] : 0u;
        }
        r.p0 = make_float4(p[0], p[1], p[2], p[3]); r.p1 = make_float4(p[4], p[5], p[6], p[7]);
        if (BF16) { r.g0 = make_uint4(g[0] | (g[1] << 16), g[2] | (g[3] << 16), g[4] | (g[5] << 16), g[6] | (g[7] << 16)); r.g1 = make_uint4(0, 0, 0, 0); }
        else      { r.g0 = make_uint4(g[0], g[1], g[2], g[3]); r.g1 = make_uint4(g[4], g[5], g[6], g[7]); }
    }
    return r;
}

// Wave-level ordering point for LDS traffic between lanes of one wavefront (LDS executes a
// wavefront's operations in order; this only stops the compiler from moving them).
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// LDS of one wavefront, one contiguous slab of 32-bit words (all offsets are compile-time
// constants, so the sub-arrays are reached with instruction offsets from very few address
// registers):
//   columns   64 x 12 words  per-lane sorted keys + sentinel; doubles as the staging area of
//                            the layout transposition at the start of an iteration
//                            (E = 16, the wide path: 64 x 18 words)
//   img_m/v   the super-tile's code words (loaded once, updated in place, written back once)
//   tv, tm    level tables of the blocks of the current iteration
//   sc        3 block scalars (Delta_m, Delta_v, alpha) per block of the super-tile
template <int BM, int BV, int B, bool MDE, int TILE, int E = 8>
struct SlabLayout {
    static constexpr int NG = 64 / (B / E);
    static constexpr int kCol = E == 8 ? kColStride : kColStride16;
    static constexpr int NBT = TILE / B;
    static constexpr int MW = TILE / (32 / BM), VW = TILE / (32 / BV);
    static constexpr int VT = 1 << BV;
    static constexpr int MTS = BM == 2 ? 4 : BM == 3 ? 8 : 16;   // stride of the m tables: a power of two >= their entries
    static constexpr int kOffCol = 0;
    static constexpr int kOffImgM = 64 * kCol;
    static constexpr int kOffImgV = kOffImgM + ((MW + 4 + 3) / 4) * 4;
    static constexpr int kOffTv = ((kOffImgV + VW + 4 + 15) / 16) * 16;      // 64-byte aligned
    static constexpr int kOffTm = kOffTv + ((NG * VT + 15) / 16) * 16;
    static constexpr int kOffSc = kOffTm + NG * MTS;
    static constexpr int kSlab = ((kOffSc + 3 * NBT + 15) / 16) * 16;
    static constexpr bool kDeTable = MDE && BM >= 3;     // DE rounding by bucket table (two boundaries: compares are cheaper)
    static constexpr int kDeWords = kDeTable ? 4 * DeBuckets<BM>::N : 16;
    static constexpr int kBytesPerWg = 4 * (kWaves * kSlab + kDeWords);
};

// Elements per wavefront super-tile: a longer tile spreads a wavefront's start-up (kernel
// arguments, first loads) over more work, so the tile is doubled wherever the larger state
// image still leaves room for SOLO_MIN_WAVES wavefronts per SIMD.
// The wide path (16 elements per lane, see step_tile16) serves the full super-tiles of a format
// whenever its larger LDS slab lets kWideWaves wavefronts per SIMD run.
#ifndef SOLO_WIDE
#define SOLO_WIDE 1
#endif
// Up to how many elements a flat buffer runs one wavefront per 512-element iteration instead of
// one per super-tile.  Measured on MI355X (per-call time over sizes from 2^12 to 2^29, every
// format): the one-iteration wavefronts need about 60 registers and run seven to a SIMD, which
// hides the memory latency without any software prefetch, so a tensor of 2^20 elements takes
// 8-9 us instead of 22-30.  With fp32 gradients and the linear codebook they stay ahead of the
// streaming kernels at every size (by 13 % at 2^26, 5 % at 2^29 elements: the streaming kernels
// of these formats sit at the register limit), with fp32 gradients and the dynamic-exponent
// codebook up to 2^28; with bf16 gradients the streaming kernels take over between 2^25
// (128-element blocks) and 2^27 elements (64-element blocks) and lead by 2-15 % at 2^29.
#ifndef SOLO_MID_SCALE
#define SOLO_MID_SCALE 1
#endif
template <int B, bool BF16, bool MDE>
constexpr uint64_t chunked_up_to()
{
    if (SOLO_MID_SCALE == 0) return 4 * (uint64_t)kTileUnit;           // (tuning builds: streaming wherever possible)
    if (SOLO_MID_SCALE < 0) return ~0ull;                               // (tuning builds: never streaming)
    if (!BF16) return MDE ? (256ull << 20) : ~0ull;
    return B == 64 ? (128ull << 20) : (32ull << 20);
}

#ifndef SOLO_WIDE_B64
#define SOLO_WIDE_B64 1
#endif
template <int BM, int BV, int B, bool MDE>
constexpr bool wide_path()
{
    constexpr int wgs = kWideWaves * 4 / kWaves;
    return SOLO_WIDE && (SOLO_WIDE_B64 || B == 128) && SlabLayout<BM, BV, B, MDE, 2 * kTileUnit, 16>::kBytesPerWg * wgs <= kLdsPerCu;
}

template <int BM, int BV, int B, bool MDE>
constexpr int tile_elems()
{
    constexpr int wgs = SOLO_MIN_WAVES * 4 / kWaves;              // workgroups per CU at that occupancy
    if (wide_path<BM, BV, B, MDE>()) return 2 * kTileUnit;
    return SlabLayout<BM, BV, B, MDE, 2 * kTileUnit>::kBytesPerWg * wgs <= kLdsPerCu ? 2 * kTileUnit : kTileUnit;
}

inline int unit_elems(uint32_t bits_m, uint32_t bits_v, uint32_t block_size, bool mde)
{
#define SOLO_U(BM_, BV_, B_)                                                                  \
    if (bits_m == BM_ && bits_v == BV_ && block_size == B_)                                   \
        return mde ? tile_elems<BM_, BV_, B_, true>() : tile_elems<BM_, BV_, B_, false>();
#define SOLO_UB(BM_, BV_) SOLO_U(BM_, BV_, 64) SOLO_U(BM_, BV_, 128)
    SOLO_UB(2, 2) SOLO_UB(2, 3) SOLO_UB(2, 4) SOLO_UB(3, 2) SOLO_UB(3, 3) SOLO_UB(3, 4)
    SOLO_UB(4, 2) SOLO_UB(4, 3) SOLO_UB(4, 4)
#undef SOLO_UB
#undef SOLO_U
    return 0;
}

// The formats whose flat buffers run one wavefront per 512-element iteration at every size do so
// in a multi-tensor launch as well: their tables hold one entry per 2560-element unit (a tensor's
// shorter end included), and five wavefronts share a unit.
inline bool multi_chunked(bool bf16, bool mde)
{
    return bf16 ? chunked_up_to<128, true, false>() == ~0ull
                : (mde ? chunked_up_to<128, false, true>() == ~0ull : chunked_up_to<128, false, false>() == ~0ull);
}

// ---- pieces shared by the two tile functions

// Stages a full super-tile's state in LDS (coalesced, 16 bytes per lane): every load is issued
// before the first one is waited for, one memory round trip instead of five.
template <int BM, int BV, int MW, int VW, int NBT>
__device__ __forceinline__ void load_state_image(const StepArgs &a, uint64_t tile, uint32_t lane,
                                                 uint32_t *img_m, uint32_t *img_v, float *sc)
{
    static_assert(MW % 4 == 0 && VW % 4 == 0, "128-bit staging");
    constexpr int RM = (MW / 4 + 63) / 64, RV = (VW / 4 + 63) / 64, RS = (NBT + 63) / 64;
    const u32x4_t *gm = reinterpret_cast<const u32x4_t *>(a.m_words + tile * MW);
    const u32x4_t *gv = reinterpret_cast<const u32x4_t *>(a.v_words + tile * VW);
    u32x4_t xm[RM], xv[RV];
    float s_dm[RS], s_dv[RS], s_al[RS];
#pragma unroll
    for (int r = 0; r < RM; ++r) {
        const uint32_t q = lane + 64u * r;
        if (q < MW / 4) xm[r] = __builtin_nontemporal_load(gm + q);
    }
#pragma unroll
    for (int r = 0; r < RV; ++r) {
        const uint32_t q = lane + 64u * r;
        if (q < VW / 4) xv[r] = __builtin_nontemporal_load(gv + q);
    }
#pragma unroll
    for (int r = 0; r < RS; ++r) {
        const uint32_t bb = lane + 64u * r;
        if (bb < NBT) {
            const uint64_t gb = tile * NBT + bb;
            s_dm[r] = a.m_scale[gb]; s_dv[r] = a.v_scale[gb]; s_al[r] = a.v_base[gb];
        }
    }
#pragma unroll
    for (int r = 0; r < RM; ++r) {
        const uint32_t q = lane + 64u * r;
        if (q < MW / 4) {
            if (BM == 3) xm[r] &= 0x3FFFFFFFu;
            *reinterpret_cast<u32x4_t *>(img_m + 4 * q) = xm[r];
        }
    }
#pragma unroll
    for (int r = 0; r < RV; ++r) {
        const uint32_t q = lane + 64u * r;
        if (q < VW / 4) {
            if (BV == 3) xv[r] &= 0x3FFFFFFFu;
            *reinterpret_cast<u32x4_t *>(img_v + 4 * q) = xv[r];
        }
    }
#pragma unroll
    for (int r = 0; r < RS; ++r) {
        const uint32_t bb = lane + 64u * r;
        if (bb < NBT) { sc[bb] = s_dm[r]; sc[NBT + bb] = s_dv[r]; sc[2 * NBT + bb] = s_al[r]; }
    }
}

// Writes a full super-tile's state back (coalesced, streamed).
template <int MW, int VW, int NBT>
__device__ __forceinline__ void store_state_image(const StepArgs &a, uint64_t tile, uint32_t lane,
                                                  const uint32_t *img_m, const uint32_t *img_v, const float *sc)
{
    u32x4_t *gm = reinterpret_cast<u32x4_t *>(a.m_words + tile * MW);
    u32x4_t *gv = reinterpret_cast<u32x4_t *>(a.v_words + tile * VW);
    for (uint32_t q = lane; q < MW / 4; q += 64)
        stream_store_u4(gm + q, *reinterpret_cast<const u32x4_t *>(img_m + 4 * q));
    for (uint32_t q = lane; q < VW / 4; q += 64)
        stream_store_u4(gv + q, *reinterpret_cast<const u32x4_t *>(img_v + 4 * q));
    for (uint32_t b = lane; b < NBT; b += 64) {
        const uint64_t gb = tile * NBT + b;
        a.m_scale[gb] = sc[b];
        a.v_scale[gb] = sc[NBT + b];
        a.v_base[gb] = sc[2 * NBT + b];
    }
}

// The r-th smallest key of every group of G lanes (full blocks).  Each lane has parked its sorted
// column at col_addr (the +inf sentinel behind it) and passes its two smallest keys.  A round:
// group minimum of the heads by DPP; the lane that holds it pops its column.  The pop is written
// out (the holders run under their own exec mask), so a round is straight-line code with the
// loop's back edge as its only branch.  A lane keeps the key behind its head in a register: a pop
// moves it up and fetches the one after it, whose LDS latency then lies outside the chain of
// rounds (it is waited for only when the same lane pops again).  A scalar population count
// detects the rounds in which two lanes of a group tie; then only the lowest holder of a group
// pops, so exactly one key leaves a group per round: a lane counts the holders below it in the
// wavefront (two mbcnt), the count of the group's first lane is spread over the group by DPP,
// and the lowest holder is the one whose count equals it.  A few vector instructions, no loop
// over the groups and no register that lives across the rounds.
template <int G>
__device__ __forceinline__ uint32_t extract_rth(uint32_t head, uint32_t behind, uint32_t haddr, uint32_t rank)
{
    constexpr int NG = 64 / G;
    uint32_t xp_bits = 0;
    for (uint32_t k = 0; k < rank; ++k) {
        const uint32_t mn = group_reduce<G>(head, UMin());
        uint64_t holders = __builtin_amdgcn_ballot_w64(head == mn);
        if (__builtin_expect(__builtin_popcountll(holders) != NG, 0)) {
            const uint32_t c = __builtin_amdgcn_mbcnt_hi((uint32_t)(holders >> 32),
                                                         __builtin_amdgcn_mbcnt_lo((uint32_t)holders, 0u));
            uint32_t c0 = dpp<0x00>(c);                     // quad_perm [0,0,0,0]
            if (G >= 8)                                     // lanes 4-7 and 12-15 of a row <- four lanes down
                c0 = (uint32_t)__builtin_amdgcn_update_dpp((int)c0, (int)c0, 0x114, 0xF, 0xA, false);
            if (G == 16)                                    // lanes 8-15 of a row <- eight lanes down
                c0 = (uint32_t)__builtin_amdgcn_update_dpp((int)c0, (int)c0, 0x118, 0xF, 0xC, false);
            holders &= __builtin_amdgcn_ballot_w64(c == c0);
        }
        xp_bits = mn;
        uint64_t saved;
        asm volatile("s_mov_b64 %[saved], exec\n\t"
                     "s_mov_b64 exec, %[holders]\n\t"
                     "s_waitcnt lgkmcnt(0)\n\t"
                     "v_mov_b32_e32 %[head], %[behind]\n\t"
                     "ds_read_b32 %[behind], %[haddr] offset:8\n\t"
                     "v_add_u32_e32 %[haddr], 4, %[haddr]\n\t"
                     "s_mov_b64 exec, %[saved]"
                     : [head] "+v"(head), [behind] "+v"(behind), [haddr] "+v"(haddr), [saved] "=&s"(saved)
                     : [holders] "s"(holders)
                     : "memory");
    }
    // the last fetch may still be in flight: its register is free only once it has landed
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(behind) : : "memory");
    return xp_bits;
}

// Per-block constants of the two encoders, from the new block statistics.
struct BlockCodec {
    float inv_s;     // L / Delta_m (DE: 1 / Delta_m); 0 for an all-zero block
    float alpha;     // the stored base; 1 for a degenerate block
    float inv_l2a;   // 1 / log2(alpha); 0 for a degenerate block
    float rdv;       // 1 / Delta_v;      0 for a degenerate block (with bias 1 the ratio is then 1)
    float bias;
};

// rho = x_p / Delta_v (even lanes) and L / Delta_m (odd lanes) share one IEEE division, then a
// quad permute hands every lane both; alpha by search_base.
template <int BV, int G, int L, bool MDE>
__device__ __forceinline__ BlockCodec block_codec(uint32_t xp_bits, float dm, float dv, uint32_t lane,
                                                  uint32_t lig, uint32_t gshift)
{
    const float num = (lane & 1u) ? (MDE ? 1.0f : (float)L) : u2f(xp_bits);
    const float den = (lane & 1u) ? dm : dv;
    const float quo = num / den;
    float rho = u2f(dpp<0xA0>(f2u(quo)));        // quad_perm [0,0,2,2]
    float inv_s = u2f(dpp<0xF5>(f2u(quo)));      // quad_perm [1,1,3,3]
    inv_s = dm > 0.0f ? inv_s : 0.0f;
    rho = dv > 0.0f ? rho : 1.0f;
    rho = rho < kRhoMin ? kRhoMin : rho;
    BlockCodec c = {inv_s, 1.0f, 0.0f, 0.0f, 1.0f};
    const bool need = rho < 1.0f;
    const uint32_t ab = search_base<BV, G>(rho, need, lane, lig, gshift);
    // the two reciprocals of the 2nd-moment encoder, correctly rounded, again by one shared
    // division: 1 / log2(alpha) on the even lanes, 1 / Delta_v on the odd ones (a block that
    // does not need them divides by harmless stand-ins)
    const float den2 = (lane & 1u) ? (need ? dv : 1.0f) : __builtin_amdgcn_logf(need ? u2f(ab) : 0.5f);
    const float quo2 = 1.0f / den2;
    const float inv_l2a = u2f(dpp<0xA0>(f2u(quo2)));
    const float rdv = u2f(dpp<0xF5>(f2u(quo2)));
    if (need) {
        c.alpha = u2f(ab);
        c.inv_l2a = inv_l2a;
        c.rdv = rdv;
        c.bias = 0.0f;
    }
    return c;
}

// Encodes a lane's run of 8 consecutive elements starting at global element index e (a multiple
// of 8): returns the packed 1st- and 2nd-moment codes (element j in bits [b j, b j + b)).
// xi: one hashed start and stride per 8 elements, every element's word finalized on its own;
// 1.5 + xi - 2^-24 is built as a float in [1,2) by one bit-align of the finalized word.
// Codes are rounded in the float domain, four to an
// accumulator (element j weighs 2^(b (j mod 4))): m: code - L = rint(m^ * L/Delta_m) in [-L, L];
// v: code + 1 = floor(log_alpha(v^/Delta_v) + 1.5 + xi).  `ok` (TAIL only): the elements that exist.
template <int BM, int BV, bool MDE, bool TAIL>
__device__ __forceinline__ void encode_run(const StepArgs &a, uint64_t e, const float *mh, const float *vh,
                                           const bool *ok, const BlockCodec &c, uint32_t de_base,
                                           uint32_t &m8, uint32_t &v8)
{
    constexpr int L = (1 << (BM - 1)) - 1;
    constexpr int K = (1 << BV) - 1;
    constexpr bool kDeTable = MDE && BM >= 3;
    const uint64_t gidx = (a.index_offset + e) >> 3;
    uint32_t X = mix32(((uint32_t)gidx ^ a.key0) + (uint32_t)(gidx >> 32) * a.key2);
    uint32_t Y = mix32(X ^ a.key1) | 1u;
    if (!a.stochastic) { X = kXiZeroWord; Y = 0u; }     // xi = 0: the float is 1.5
    uint32_t xj = X;                                    // X + j Y, walked up from j = 0
    float am_lo = 0.0f, am_hi = 0.0f, av_lo = 0.0f, av_hi = 0.0f;
    uint32_t m8_de = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j, xj += Y) {
        float tm = 0.0f;
        if (!MDE) {
            tm = __builtin_rintf(mh[j] * c.inv_s);
        } else {
            // DE: nearest level on the magnitude; inv_s = 1/Delta_m
            const float z = mh[j] * c.inv_s;
            uint32_t code;
            if (kDeTable) {
                // entry of the bucket of |z| (16 bytes per bucket: z >= 0, then z < 0)
                // (clamped on both sides: a non-finite input must not leave the table)
                const uint32_t bk = umin(umax(__builtin_amdgcn_ubfe(f2u(z), 21u, 10u), DeBuckets<BM>::kLo),
                                         DeBuckets<BM>::kHi);
                const uint32_t addr = ((f2u(z) >> 28) & 8u) | ((bk << 4) + de_base);
                const u32x2_t en = *(lds_u32x2_t *)(uintptr_t)addr;
                code = en.y + (z > u2f(en.x) ? 1u : 0u);
            } else {
                // few levels: the code is the number of rounding boundaries below z.  A value
                // on a boundary keeps the level of smaller magnitude: '>' on the positive side,
                // '>=' on the negative one (z = -0 is above every negative boundary: code L).
                code = 0;
#pragma unroll
                for (int k = 0; k < L; ++k) code += (z >= -DeLevels<BM>::tab.mid[k]) ? 1u : 0u;
#pragma unroll
                for (int k = 0; k <= L; ++k) code += (z > DeLevels<BM>::tab.mid[k]) ? 1u : 0u;
            }
            if (TAIL && !ok[j]) code = 0;
            m8_de |= code << (BM * j);
        }
        const float f = u2f(__builtin_amdgcn_alignbit(0x7Fu, xi_finalize(xj), 9u));
        const float ratio = __builtin_fmaf(vh[j], c.rdv, c.bias);
        float tv = __builtin_floorf(__builtin_fmaf(__builtin_amdgcn_logf(ratio), c.inv_l2a, f));
        tv = __builtin_amdgcn_fmed3f(tv, 1.0f, (float)(K + 1));   // +inf (v^ = 0) takes the last code
        if (TAIL && !ok[j]) { tm = -(float)L; tv = 1.0f; }
        // (sums of at most four small integers times powers of two: exact)
        const float wm = (float)(1 << (BM * (j & 3))), wv = (float)(1 << (BV * (j & 3)));
        if (j == 0)      { am_lo = tm; av_lo = tv; }
        else if (j < 4)  { am_lo = __builtin_fmaf(tm, wm, am_lo); av_lo = __builtin_fmaf(tv, wv, av_lo); }
        else if (j == 4) { am_hi = tm; av_hi = tv; }
        else             { am_hi = __builtin_fmaf(tm, wm, am_hi); av_hi = __builtin_fmaf(tv, wv, av_hi); }
    }
    constexpr float OFFM = (float)(L * ((1 << (4 * BM)) - 1) / ((1 << BM) - 1));   // L * sum 2^(BM j), j < 4
    constexpr float OFFV = (float)(((1 << (4 * BV)) - 1) / ((1 << BV) - 1));        // sum 2^(BV j), j < 4
    m8 = MDE ? m8_de : ((uint32_t)(am_lo + OFFM) | ((uint32_t)(am_hi + OFFM) << (4 * BM)));
    v8 = (uint32_t)(av_lo - OFFV) | ((uint32_t)(av_hi - OFFV) << (4 * BV));
}

// ---- pieces shared by the tile functions and the large-block functions (solo_step_big.h)

// The level tables of a block that G lanes share (decode by table look-up): lane `lig` of the group
// fills entries lig, lig + G, ... of the 2nd-moment table (Delta_v alpha^q, alpha^q by binary
// powering) and of the 1st-moment table (linear: (c - L) (Delta_m / L); dynamic exponent: the
// lane's levels `de_level` times Delta_m).
template <int BM, int BV, bool MDE, int G>
__device__ __forceinline__ void fill_level_tables(float *const my_tv, float *const my_tm, const uint32_t lig,
                                                  const float dm_old, const float dv_old, const float al_old,
                                                  const float *de_level)
{
    constexpr int L = (1 << (BM - 1)) - 1;
    constexpr int VT = 1 << BV;
    constexpr int MT = MDE ? 2 * L + 2 : 2 * L + 1;
    const float s_m = (L == 1) ? dm_old : dm_old / (float)L;
    const float P1 = al_old, P2 = P1 * P1, P4 = P2 * P2, P8 = P4 * P4;
#pragma unroll
    for (int r = 0; r < (VT + G - 1) / G; ++r) {
        const uint32_t q = lig + r * G;
        if (q < VT) my_tv[q] = log_level<BV>(q, P1, P2, P4, P8) * dv_old;
    }
#pragma unroll
    for (int r = 0; r < (MT + G - 1) / G; ++r) {
        const uint32_t c = lig + r * G;
        if (c < MT) my_tm[c] = MDE ? de_level[r] * dm_old : (float)((int)c - L) * s_m;
    }
}


// A lane's 8 consecutive elements out of the coalesced layout they were loaded in, through the
// wavefront's staging area: st_c = stage + lane + lane / 8 (coalesced slots st_c[0], st_c[72]),
// st_l = stage + 2 lane + lane / 4 (the lane's own two vectors).  TAIL: loaded per lane already.
template <bool BF16, bool TAIL>
__device__ __forceinline__ void lane_layout8(const RawPG &raw, float4 *const st_c, float4 *const st_l,
                                             float (&p)[8], float (&g)[8])
{
    float4 pa = raw.p0, pb = raw.p1;
    uint4 ga = raw.g0, gb = raw.g1;
    if (!TAIL) {                       // coalesced layout -> 8 consecutive elements per lane
        st_c[0] = pa; st_c[72] = pb;
        wave_lds_sync();
        pa = st_l[0]; pb = st_l[1];
        if (!BF16) {
            wave_lds_sync();
            st_c[0] = make_float4(u2f(ga.x), u2f(ga.y), u2f(ga.z), u2f(ga.w));
            st_c[72] = make_float4(u2f(gb.x), u2f(gb.y), u2f(gb.z), u2f(gb.w));
            wave_lds_sync();
            const float4 t0 = st_l[0], t1 = st_l[1];
            ga = make_uint4(f2u(t0.x), f2u(t0.y), f2u(t0.z), f2u(t0.w));
            gb = make_uint4(f2u(t1.x), f2u(t1.y), f2u(t1.z), f2u(t1.w));
        }
    }
    p[0] = pa.x; p[1] = pa.y; p[2] = pa.z; p[3] = pa.w;
    p[4] = pb.x; p[5] = pb.y; p[6] = pb.z; p[7] = pb.w;
    if (BF16) {
        g[0] = u2f(ga.x << 16); g[1] = u2f(ga.x & 0xFFFF0000u);
        g[2] = u2f(ga.y << 16); g[3] = u2f(ga.y & 0xFFFF0000u);
        g[4] = u2f(ga.z << 16); g[5] = u2f(ga.z & 0xFFFF0000u);
        g[6] = u2f(ga.w << 16); g[7] = u2f(ga.w & 0xFFFF0000u);
    } else {
        g[0] = u2f(ga.x); g[1] = u2f(ga.y); g[2] = u2f(ga.z); g[3] = u2f(ga.w);
        g[4] = u2f(gb.x); g[5] = u2f(gb.y); g[6] = u2f(gb.z); g[7] = u2f(gb.w);
    }
}

// Dequantize (table look-up: byte offset 4 * code, OR-ed into the aligned table base), both EMAs
// and the parameter for a lane's N = 8 or 16 consecutive elements; mc8 / vc8: the packed old
// codes of every run of 8.  VMAX: also the largest v^ (the callers that sort take it from the
// sorted keys).  TAIL: elements that do not exist (`ok`) leave zeros in m^ and v^.
// AdaBelief without a branch: d = g - kb * m^ is g itself when kb = 0 and fl(g - m^) when kb = 1
// (one rounding either way), and eps_state = 0 leaves v^ unchanged.
// Parameter: decoupled decay, bias-corrected Adam direction,
// p <- p * decay - step_size * m^ / (sqrt(v^ / bc2) + eps), with step_size folded into the denominator.
template <int N, int BM, int BV, bool EXT, bool TAIL, bool VMAX>
__device__ __forceinline__ void ema_param(const StepArgs &a, const uint32_t tm_addr, const uint32_t tv_addr,
                                          const uint32_t *mc8, const uint32_t *vc8, const bool *ok,
                                          float (&p)[N], const float (&g)[N], float (&mh)[N], float (&vh)[N],
                                          float &m_absmax, float &v_max)
{
    constexpr uint32_t MIDX = ((1u << BM) - 1u) << 2, VIDX = ((1u << BV) - 1u) << 2;   // byte-index masks
    float mt[N], vt[N];
    if (N == 8) {                              // (the narrow code fetches all levels first)
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const uint32_t om = (j == 0) ? (mc8[0] << 2) : (mc8[0] >> (BM * j - 2));
            const uint32_t ov = (j == 0) ? (vc8[0] << 2) : (vc8[0] >> (BV * j - 2));
            mt[j] = lds_f32(tm_addr | (om & MIDX));
            vt[j] = lds_f32(tv_addr | (ov & VIDX));
        }
    }
    m_absmax = 0.0f;
    v_max = 0.0f;
    const float kb = a.belief ? 1.0f : 0.0f;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        if (N != 8) {
            const int r = j / 8, jj = j % 8;
            const uint32_t om = (jj == 0) ? (mc8[r] << 2) : (mc8[r] >> (BM * jj - 2));
            const uint32_t ov = (jj == 0) ? (vc8[r] << 2) : (vc8[r] >> (BV * jj - 2));
            mt[j] = lds_f32(tm_addr | (om & MIDX));
            vt[j] = lds_f32(tv_addr | (ov & VIDX));
        }
        mh[j] = __builtin_fmaf(a.beta1, mt[j], a.omb1 * g[j]);
        if (EXT) {
            const float d = __builtin_fmaf(-kb, mh[j], g[j]);
            vh[j] = __builtin_fmaf(a.beta2, vt[j], a.omb2 * (d * d)) + a.eps_state;
        } else {
            vh[j] = __builtin_fmaf(a.beta2, vt[j], a.omb2 * (g[j] * g[j]));
        }
        const float denom = __builtin_fmaf(__builtin_amdgcn_sqrtf(vh[j]), a.denom_scale, a.denom_eps);
        p[j] = __builtin_fmaf(p[j], a.decay, -(mh[j] * __builtin_amdgcn_rcpf(denom)));
        if (TAIL && !ok[j]) { mh[j] = 0.0f; vh[j] = 0.0f; }
        m_absmax = __builtin_fmaxf(m_absmax, __builtin_fabsf(mh[j]));
        if (VMAX) v_max = __builtin_fmaxf(v_max, vh[j]);
    }
}

// The new parameters of a lane's 8 elements (and their bf16 copy, if asked for) back to the
// coalesced layout and streamed out; chunk_e0: first element of the wavefront's 512, e0: of the lane.
template <bool EXT, bool TAIL>
__device__ __forceinline__ void store_params8(const StepArgs &a, const uint64_t chunk_e0, const uint64_t e0,
                                              const uint32_t lane, const bool *ok, const float (&p)[8],
                                              float4 *const st_c, float4 *const st_l)
{
    if (EXT && a.param_bf16) {                    // 16-bit copy of the new parameters, 16 bytes per lane
        if (!TAIL) {
            const u32x4_t h = {pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]),
                             pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])};
            stream_store_u4(a.param_bf16 + e0, h);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (ok[j]) a.param_bf16[e0 + j] = (uint16_t)pack_bf16(p[j], 0.0f);
        }
    }
    if (!TAIL) {                           // back to the coalesced layout, streamed out
        wave_lds_sync();
        st_l[0] = make_float4(p[0], p[1], p[2], p[3]);
        st_l[1] = make_float4(p[4], p[5], p[6], p[7]);
        wave_lds_sync();
        float *pp = a.param + chunk_e0 + lane * 4u;
        stream_store_f4(pp, st_c[0]);
        stream_store_f4(pp + 256, st_c[72]);
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) if (ok[j]) a.param[e0 + j] = p[j];
    }
}

// A lane's run of 8 new codes into the LDS image of the code words (wm / sm, wv / sv: word and
// slot of the run's first code; xm, xv: old codes XOR new codes): the XOR turns this lane's old
// fields into the new ones and leaves the neighbours' fields of a shared word alone.
template <int BM, int BV>
__device__ __forceinline__ void xor_into_image8(uint32_t *const img_m, uint32_t *const img_v, const uint32_t wm,
                                                const uint32_t sm, const uint32_t wv, const uint32_t sv,
                                                const uint32_t xm, const uint32_t xv)
{
    const uint32_t xm0 = (BM == 3) ? (xm << (3u * sm)) & 0x3FFFFFFFu : xm << (BM * sm);
    const uint32_t xm1 = (BM == 3) ? (uint32_t)(((uint64_t)xm << (3u * sm)) >> 30) : 0u;
    const uint32_t xv0 = (BV == 3) ? (xv << (3u * sv)) & 0x3FFFFFFFu : xv << (BV * sv);
    const uint32_t xv1 = (BV == 3) ? (uint32_t)(((uint64_t)xv << (3u * sv)) >> 30) : 0u;
    atomicXor(&img_m[wm], xm0);
    if (BM == 3) atomicXor(&img_m[wm + 1], xm1);
    atomicXor(&img_v[wv], xv0);
    if (BV == 3) atomicXor(&img_v[wv + 1], xv1);
}

// A lane writes back the code word it staged (`own`: as it was loaded; `fin`: as it is in the
// image now).  Two- and four-bit words are whole words of whole lines and are stored plainly.
// Ten-to-a-word codes do not end on a line (or even on a word) at the end of a wavefront's share:
// their words take this wavefront's changes by atomic XOR (the fields that two wavefronts own in
// a shared word are disjoint), which is carried out at the memory side and leaves no partly
// written line behind in the L2 of this die.
template <int BITS>
__device__ __forceinline__ void write_back_word(uint32_t *const word, const uint32_t fin, const uint32_t own)
{
    if (BITS != 3) *word = fin;
    else if (fin != own) atomicXor(word, fin ^ own);
}

// One super-tile of TILE elements, processed by the calling wavefront: the whole step for the
// elements [tile * TILE, (tile + 1) * TILE) of the buffers in `a` (TAIL: clipped to a.n, with
// bounds checks on every element).  `slab` is this wavefront's LDS, `lds_de` the workgroup's DE
// bucket table.
// EXT: the code that also serves the variants of the step (gradient scale, coupled decay,
// AdaBelief, bf16 weight copy); the plain AdamW step runs the one without them.
template <int BM, int BV, int B, bool BF16, bool MDE, bool TAIL, bool EXT, int TILE, bool ALONE = TAIL>
__device__ __forceinline__ void step_tile(const StepArgs &a, const uint64_t tile, const uint32_t lane,
                                          uint32_t *const slab, const uint32_t *const lds_de, const int chunk = -1)
{
    // ALONE: this wavefront runs iteration `chunk` of the tile alone, next to other wavefronts
    // that run the other iterations (short and mid-size tensors, whose super-tiles are too few to
    // fill the machine; always so for a ragged end).  It stages the tile's state for reading and
    // applies its code changes to the global words directly (atomic XOR: the fields that
    // different wavefronts own in a shared word are disjoint) instead of writing the tile back.
    static_assert(ALONE || !TAIL, "a ragged end is always cut into its iterations");
    constexpr bool alone = ALONE;
    constexpr int G = B / 8;                       // lanes per block
    constexpr int NG = 64 / G;                     // blocks per iteration
    constexpr int kTile = TILE;
    using Lay = SlabLayout<BM, BV, B, MDE, kTile>;
    constexpr int NBT = kTile / B;                 // blocks per super-tile
    constexpr int L = (1 << (BM - 1)) - 1;
    constexpr int K = (1 << BV) - 1;
    constexpr int CM = 32 / BM, CV = 32 / BV;      // codes per word
    constexpr int MW = kTile / CM, VW = kTile / CV; // words per super-tile
    constexpr int VT = K + 1;                      // entries of a block's v level table (4, 8, 16)
    constexpr int MT = MDE ? 2 * L + 2 : 2 * L + 1; // entries of a block's m level table (3, 7, 15; DE: 4, 8, 16)
    constexpr int MTS = Lay::MTS;                  // stride of the m tables
    constexpr uint32_t GMASK = (G == 16) ? 0xFFFFu : 0xFFu;
    // A runaway column address (possible only with non-finite input) stays inside the slab.
    constexpr int kOffCol = Lay::kOffCol, kOffImgM = Lay::kOffImgM, kOffImgV = Lay::kOffImgV;
    constexpr int kOffTv = Lay::kOffTv, kOffTm = Lay::kOffTm, kOffSc = Lay::kOffSc, kSlab = Lay::kSlab;
    constexpr bool kDeTable = Lay::kDeTable;
    static_assert(kSlab >= 64 * kColStride + 140, "column slack");

    const uint64_t nblk = (a.n + B - 1) / B;
    const uint64_t m_total = (a.n + CM - 1) / CM, v_total = (a.n + CV - 1) / CV;
    const uint64_t tile_e0 = tile * kTile;

    uint32_t *const img_m = slab + kOffImgM, *const img_v = slab + kOffImgV;
    float *const sc = reinterpret_cast<float *>(slab + kOffSc);
    uint32_t *const col = slab + kOffCol + lane * kColStride;

    // first parameters and gradients: in flight while the state image is staged
    const int it_begin = alone ? chunk : 0, it_end = alone ? chunk + 1 : TILE / kIter;
    RawPG raw = load_pg<BF16, TAIL>(a, tile_e0 + (uint32_t)it_begin * kIter, lane);
    const float gscale = (EXT && a.grad_scale) ? *a.grad_scale : 1.0f;      // uniform: the gradient is transformed first
    // one pad vector after every 8 keeps both the coalesced (index = lane) and the per-lane
    // (index = 2 lane, 2 lane + 1) accesses of the transposition free of bank conflicts
    static_assert((kIter / 4 + kIter / 32) * 4 <= 64 * kColStride, "staging must fit the column area");
    float4 *const stage = reinterpret_cast<float4 *>(slab + kOffCol);
    float4 *const st_c = stage + (lane + lane / 8u);        // coalesced slots: st_c[0] and st_c[72] (= slot 64 + lane)
    float4 *const st_l = stage + (2u * lane + lane / 4u);   // this lane's 8 elements: st_l[0], st_l[1]

    // ---- stage the state in LDS.  A wavefront that owns the super-tile stages all of it (coalesced,
    // 16 bytes per lane).  One that runs a single iteration stages that iteration's part: at most
    // 64 words of each code stream, one per lane, which the same lane writes back at the end (the
    // first and the last 3-bit word may be shared with the neighbouring iterations' wavefronts),
    // and the scalars of its blocks.
    static_assert(kOffImgM % 4 == 0 && kOffImgV % 4 == 0, "128-bit staging");
    static_assert(kIter / 8 <= 64, "one staged word per lane and code stream");
    uint32_t own_m = 0, own_v = 0;                 // the staged words as they were loaded
    const uint32_t e_lo = alone ? (uint32_t)chunk * kIter : 0u, e_hi = e_lo + kIter - 1u;
    const uint32_t wm_lo = e_lo / CM, wm_hi = e_hi / CM, wv_lo = e_lo / CV, wv_hi = e_hi / CV;
    if (alone) {
        const uint32_t w_m = wm_lo + lane, w_v = wv_lo + lane;
        const uint64_t gw_m = tile * MW + w_m, gw_v = tile * VW + w_v;
        const uint32_t b = (uint32_t)chunk * (kIter / B) + lane;
        const uint64_t gb = tile * NBT + b;
        const bool has_m = w_m <= wm_hi && (!TAIL || gw_m < m_total);
        const bool has_v = w_v <= wv_hi && (!TAIL || gw_v < v_total);
        const bool has_b = lane < (uint32_t)(kIter / B) && (!TAIL || gb < nblk);
        // every load is issued before the first one is waited for
        float s_dm = 0.0f, s_dv = 0.0f, s_al = 1.0f;
        if (has_m) own_m = a.m_words[gw_m];
        if (has_v) own_v = a.v_words[gw_v];
        if (has_b) { s_dm = a.m_scale[gb]; s_dv = a.v_scale[gb]; s_al = a.v_base[gb]; }
        if (BM == 3) own_m &= 0x3FFFFFFFu;
        if (BV == 3) own_v &= 0x3FFFFFFFu;
        if (w_m <= wm_hi) img_m[w_m] = own_m;
        if (w_v <= wv_hi) img_v[w_v] = own_v;
        if (lane < (uint32_t)(kIter / B)) { sc[b] = s_dm; sc[NBT + b] = s_dv; sc[2 * NBT + b] = s_al; }
        // (a 3-bit run that ends with its word reads the word behind it without using it)
        if (lane == 0) { img_m[wm_hi + 1] = 0; img_v[wv_hi + 1] = 0; }
    } else {
        load_state_image<BM, BV, MW, VW, NBT>(a, tile, lane, img_m, img_v, sc);
    }
    if (!alone && lane < 4) { img_m[MW + lane] = 0; img_v[VW + lane] = 0; }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    const uint32_t lig = lane & (G - 1);               // lane in group
    const uint32_t grp = lane / G;                     // group (block) inside the iteration
    const uint32_t gshift = lane & 31u & ~(uint32_t)(G - 1);   // group's first lane inside its 32-lane half
    const uint32_t below = (1u << lig) - 1u;
    float *const my_tv = reinterpret_cast<float *>(slab + kOffTv) + grp * VT;
    float *const my_tm = reinterpret_cast<float *>(slab + kOffTm) + grp * MTS;
    const uint32_t tv_addr = lds_addr(my_tv), tm_addr = lds_addr(my_tm);   // aligned to the table size
    const uint32_t col_addr = lds_addr(col);

    // DE codebook: the levels of the table entries this lane fills (entries lig, lig + G)
    float de_level[(16 + G - 1) / G];
    uint32_t de_base = 0;                              // bucket table address, less the first bucket's index
    if (MDE) {
#pragma unroll
        for (int r = 0; r < (MT + G - 1) / G; ++r) de_level[r] = DeLevels<BM>::level(lig + r * G);
        if (kDeTable) de_base = lds_addr(lds_de) - 16u * DeBuckets<BM>::kLo;
    }

#pragma unroll 1
    for (int it = it_begin; it < it_end; ++it) {
        const uint32_t e_loc = (uint32_t)it * kIter + lane * 8u;   // element inside the tile
        const uint64_t e0 = tile_e0 + e_loc;
        const uint32_t bl = (uint32_t)it * NG + grp;               // block inside the tile
        // word and slot of this lane's first code (recomputed in every iteration: cheaper in
        // registers than carrying them; e / 10 by multiplication, exact far beyond the tile size)
        static_assert(kTile <= 20480, "range of the division by 10");
        const uint32_t wm = (CM == 10) ? __umul24(e_loc, 52429u) >> 19 : e_loc / CM, sm = e_loc - wm * CM;
        const uint32_t wv = (CV == 10) ? __umul24(e_loc, 52429u) >> 19 : e_loc / CV, sv = e_loc - wv * CV;
        // elements of this lane's block that exist (B except in the last block)
        uint32_t nb = B;
        bool blk_ok = true;
        bool ok[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) ok[j] = !TAIL || (e0 + j) < a.n;
        if (TAIL) {
            const uint64_t blk = tile * NBT + bl;
            blk_ok = blk < nblk;
            const uint64_t bstart = blk * B;
            nb = blk_ok ? (uint32_t)((a.n - bstart) < (uint64_t)B ? (a.n - bstart) : (uint64_t)B) : 0u;
        }

        // ---- old state of the block and of this lane's elements (LDS)
        const float dm_old = sc[bl], dv_old = sc[NBT + bl], al_old = sc[2 * NBT + bl];
        const uint32_t mw0 = img_m[wm], mw1 = (BM == 3) ? img_m[wm + 1] : 0u;
        const uint32_t vw0 = img_v[wv], vw1 = (BV == 3) ? img_v[wv + 1] : 0u;
        const uint32_t mc8 = extract8<BM>(mw0, mw1, sm) & (uint32_t)((1ull << (8 * BM)) - 1ull);
        const uint32_t vc8 = extract8<BV>(vw0, vw1, sv) & (uint32_t)((1ull << (8 * BV)) - 1ull);

        // ---- level tables of this lane's block: entries lig, lig + G, ...
        {
            fill_level_tables<BM, BV, MDE, G>(my_tv, my_tm, lig, dm_old, dv_old, al_old, de_level);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }

        // ---- dequantize (table look-up), EMA, parameter
        float p[8], g[8];
        lane_layout8<BF16, TAIL>(raw, st_c, st_l, p, g);
        if (EXT) {                             // g <- fl(g * scale), then one fused g + l2 * p (l2 = 0: exact)
#pragma unroll
            for (int j = 0; j < 8; ++j) g[j] = __builtin_fmaf(a.l2, p[j], g[j] * gscale);
        }
        // next iteration's parameters and gradients, a whole iteration ahead of their use
        if (it + 1 < it_end) raw = load_pg<BF16, TAIL>(a, tile_e0 + (uint32_t)(it + 1) * kIter, lane);
        float mh[8], vh[8];
        float m_absmax, v_max;                 // (v_max of full tiles: the last sorted key below)
        ema_param<8, BM, BV, EXT, TAIL, TAIL>(a, tm_addr, tv_addr, &mc8, &vc8, ok, p, g, mh, vh, m_absmax, v_max);
        store_params8<EXT, TAIL>(a, tile_e0 + (uint32_t)it * kIter, e0, lane, ok, p, st_c, st_l);

        // ---- the lane's v^ sorted (non-negative floats order like their bit patterns); block maxima
        uint32_t key[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) key[j] = (TAIL && !ok[j]) ? kInfBits : f2u(vh[j]);
        sort8(key);
        float dm = u2f(group_reduce<G>(f2u(m_absmax), UMax()));
        float dv = u2f(group_reduce<G>(TAIL ? f2u(v_max) : key[7], UMax()));
        if (dm < kTiny) dm = 0.0f;
        if (dv < kTiny) dv = 0.0f;

        // ---- the r-th smallest v^ of the block
        col[8] = kInfBits;                      // sentinel behind the lane's 8 keys (the staging overwrote it)
        *reinterpret_cast<uint4 *>(col) = make_uint4(key[0], key[1], key[2], key[3]);
        *reinterpret_cast<uint4 *>(col + 4) = make_uint4(key[4], key[5], key[6], key[7]);
        uint32_t r_mine = a.rank_full;
        if (TAIL) {
            const float x = __builtin_ceilf(a.quantile_p * (float)nb);
            r_mine = x < 1.0f ? 1u : (uint32_t)x;
            r_mine = r_mine > nb ? nb : r_mine;
        }
        uint32_t head = key[0], haddr = col_addr, xp_bits = 0;
        auto extract_round = [&](uint32_t k) {
            const uint32_t mn = group_reduce<G>(head, UMin());
            bool pop = head == mn;
            const uint64_t holders = __builtin_amdgcn_ballot_w64(pop);
            // one holder per group is the common case; a tie costs three more instructions:
            // only the lowest holder of a group pops, so exactly one key leaves per round
            if (__builtin_popcountll(holders) != NG)
                pop = pop && (group_bits(holders, lane, gshift, GMASK) & below) == 0u;
            if (TAIL) { if (k + 1 == r_mine) xp_bits = mn; } else xp_bits = mn;
            if (pop) {
                haddr = TAIL ? umin(haddr + 4u, col_addr + 32u) : haddr + 4u;
                head = lds_u32(haddr);
            }
        };
        if (!TAIL) {
            xp_bits = extract_rth<G>(key[0], key[1], col_addr, a.rank_full);
        } else {
            for (uint32_t k = 0; k < a.rank_full; ++k) extract_round(k);
        }

        // ---- the block's encoder constants, then this lane's 8 codes of each moment
        const BlockCodec codec = block_codec<BV, G, L, MDE>(xp_bits, dm, dv, lane, lig, gshift);
        const float alpha = codec.alpha;
        uint32_t m8, v8;
        encode_run<BM, BV, MDE, TAIL>(a, e0, mh, vh, ok, codec, de_base, m8, v8);

        xor_into_image8<BM, BV>(img_m, img_v, wm, sm, wv, sv, mc8 ^ m8, vc8 ^ v8);
        if (alone) {
            if (lig == 0 && blk_ok) {
                const uint64_t gb = tile * NBT + bl;
                a.m_scale[gb] = dm; a.v_scale[gb] = dv; a.v_base[gb] = alpha;
            }
        } else {
            if (lig == 0) { sc[bl] = dm; sc[NBT + bl] = dv; sc[2 * NBT + bl] = alpha; }
        }
        (void)blk_ok;
    }

    // ---- write the super-tile's state back (coalesced)
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (alone) {
        // every lane writes back the word it staged
        const uint32_t w_m = wm_lo + lane, w_v = wv_lo + lane;
        const uint64_t gw_m = tile * MW + w_m, gw_v = tile * VW + w_v;
        if (w_m <= wm_hi && (!TAIL || gw_m < m_total)) write_back_word<BM>(&a.m_words[gw_m], img_m[w_m], own_m);
        if (w_v <= wv_hi && (!TAIL || gw_v < v_total)) write_back_word<BV>(&a.v_words[gw_v], img_v[w_v], own_v);
    } else {
        store_state_image<MW, VW, NBT>(a, tile, lane, img_m, img_v, sc);
    }
}

// Sixteen keys: two eight-sorts and Batcher's odd-even merge of the halves (25 exchanges).
__device__ __forceinline__ void sort16(uint32_t (&k)[16])
{
    uint32_t lo[8], hi[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { lo[i] = k[i]; hi[i] = k[i + 8]; }
    sort8(lo); sort8(hi);
#pragma unroll
    for (int i = 0; i < 8; ++i) { k[i] = lo[i]; k[i + 8] = hi[i]; }
#pragma unroll
    for (int i = 0; i < 8; ++i) cswap(k[i], k[i + 8]);
#pragma unroll
    for (int i = 4; i < 8; ++i) cswap(k[i], k[i + 4]);
#pragma unroll
    for (int i = 2; i < 12; i += 4) { cswap(k[i], k[i + 2]); cswap(k[i + 1], k[i + 3]); }
#pragma unroll
    for (int i = 1; i < 15; i += 2) cswap(k[i], k[i + 1]);
}

// Parameters and gradients of one lane and one 1024-element iteration of the wide path, in the
// coalesced layout they are loaded in (vector k of a lane is vector lane + 64 k of the chunk).
template <bool BF16>
struct RawPG16 { float4 p[4]; uint4 g[BF16 ? 2 : 4]; };

template <bool BF16>
__device__ __forceinline__ RawPG16<BF16> load_pg16(const StepArgs &a, uint64_t chunk_e0, uint32_t lane)
{
    RawPG16<BF16> r;
    const float *pp = a.param + chunk_e0 + lane * 4u;
#pragma unroll
    for (int k = 0; k < 4; ++k) r.p[k] = stream_load_f4(pp + 256 * k);
    if (BF16) {
        const uint16_t *gp = static_cast<const uint16_t *>(a.grad) + chunk_e0 + lane * 8u;
#pragma unroll
        for (int k = 0; k < 2; ++k) r.g[k] = stream_load_u4(gp + 512 * k);
    } else {
        const float *gp = static_cast<const float *>(a.grad) + chunk_e0 + lane * 4u;
#pragma unroll
        for (int k = 0; k < (BF16 ? 2 : 4); ++k) r.g[k] = stream_load_u4(gp + 256 * k);
    }
    return r;
}

// The staging slots of a lane for the layout transposition of a 1024-element iteration, 16-byte
// vectors.  Vector i of the chunk sits in slot i + i / 8 (one pad vector after every 8): eight
// neighbouring lanes then cover all banks both on the coalesced side (i = lane + 64 k) and on the
// lane's own side (fp32: i = 4 lane + c, slot 4 lane + lane / 2 + c; bf16: i = 2 lane + c,
// slot 2 lane + lane / 4 + c).  288 vectors.
struct Stage16 {
    float4 *c4, *l4, *c2, *l2;     // c4[72 k], l4[c]: 32-bit elements; c2[72 k], l2[c]: 16-bit elements
    __device__ __forceinline__ Stage16(float4 *stage, uint32_t lane)
        : c4(stage + (lane + lane / 8u)), l4(stage + (4u * lane + lane / 2u)),
          c2(stage + (lane + lane / 8u)), l2(stage + (2u * lane + lane / 4u)) {}
};

// A lane's 16 consecutive elements out of the coalesced layout they were loaded in.
template <bool BF16>
__device__ __forceinline__ void lane_layout16(const RawPG16<BF16> &raw, const Stage16 &st,
                                              float (&p)[16], float (&g)[16])
{
#pragma unroll
    for (int k = 0; k < 4; ++k) st.c4[72 * k] = raw.p[k];
    wave_lds_sync();                   // (also orders the level tables before their readers)
    float4 t[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) t[c] = st.l4[c];
#pragma unroll
    for (int c = 0; c < 4; ++c) { p[4 * c] = t[c].x; p[4 * c + 1] = t[c].y; p[4 * c + 2] = t[c].z; p[4 * c + 3] = t[c].w; }
    wave_lds_sync();
    if (BF16) {
#pragma unroll
        for (int k = 0; k < 2; ++k)
            st.c2[72 * k] = make_float4(u2f(raw.g[k].x), u2f(raw.g[k].y), u2f(raw.g[k].z), u2f(raw.g[k].w));
        wave_lds_sync();
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const float4 x = st.l2[c];
            const uint32_t w[4] = {f2u(x.x), f2u(x.y), f2u(x.z), f2u(x.w)};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                g[8 * c + 2 * i] = u2f(w[i] << 16);
                g[8 * c + 2 * i + 1] = u2f(w[i] & 0xFFFF0000u);
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < (BF16 ? 2 : 4); ++k)
            st.c4[72 * k] = make_float4(u2f(raw.g[k].x), u2f(raw.g[k].y), u2f(raw.g[k].z), u2f(raw.g[k].w));
        wave_lds_sync();
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float4 x = st.l4[c];
            g[4 * c] = x.x; g[4 * c + 1] = x.y; g[4 * c + 2] = x.z; g[4 * c + 3] = x.w;
        }
    }
}

// The new parameters of a lane's 16 elements (and their bf16 copy, if asked for: 32 bytes per
// lane, two vectors, first) back to the coalesced layout and streamed out; chunk_e0: first
// element of the wavefront's 1024.
template <bool EXT>
__device__ __forceinline__ void store_params16(const StepArgs &a, const uint64_t chunk_e0, const uint32_t lane,
                                               const float (&p)[16], const Stage16 &st)
{
    wave_lds_sync();
    if (EXT && a.param_bf16) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const uint32_t h0 = pack_bf16(p[8 * c], p[8 * c + 1]), h1 = pack_bf16(p[8 * c + 2], p[8 * c + 3]);
            const uint32_t h2 = pack_bf16(p[8 * c + 4], p[8 * c + 5]), h3 = pack_bf16(p[8 * c + 6], p[8 * c + 7]);
            st.l2[c] = make_float4(u2f(h0), u2f(h1), u2f(h2), u2f(h3));
        }
        wave_lds_sync();
        uint16_t *hp = a.param_bf16 + chunk_e0 + lane * 8u;
#pragma unroll
        for (int k = 0; k < 2; ++k) stream_store_f4(reinterpret_cast<float *>(hp + 512 * k), st.c2[72 * k]);
        wave_lds_sync();
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) st.l4[c] = make_float4(p[4 * c], p[4 * c + 1], p[4 * c + 2], p[4 * c + 3]);
    wave_lds_sync();
    float *pp = a.param + chunk_e0 + lane * 4u;
#pragma unroll
    for (int k = 0; k < 4; ++k) stream_store_f4(pp + 256 * k, st.c4[72 * k]);
}

// Codes of a lane's 16 elements (two runs of 8: e0 is the first element, wm / sm / wv / sv the
// word and slot of each run's first code in the image, mc8 / vc8 the old codes) into the LDS
// image of the code words.  3-bit codes share words between lanes: XOR turns this lane's old
// fields into the new ones and leaves the neighbours' alone.  2- and 4-bit words belong to one lane
// (2-bit: both runs lie in word wm[0]).
template <int BM, int BV, bool MDE>
__device__ __forceinline__ void encode_into_image16(const StepArgs &a, const uint64_t e0, const float *mh, const float *vh,
                                                    const BlockCodec &codec, const uint32_t de_base,
                                                    uint32_t *const img_m, uint32_t *const img_v,
                                                    const uint32_t (&wm)[2], const uint32_t (&sm)[2],
                                                    const uint32_t (&wv)[2], const uint32_t (&sv)[2],
                                                    const uint32_t (&mc8)[2], const uint32_t (&vc8)[2])
{
    uint32_t m_word = 0, v_word = 0;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        uint32_t m8, v8;
        encode_run<BM, BV, MDE, false>(a, e0 + 8u * r, mh + 8 * r, vh + 8 * r, nullptr, codec, de_base, m8, v8);
        if (BM == 3) {
            const uint32_t xm = mc8[r] ^ m8;
            atomicXor(&img_m[wm[r]], (xm << (3u * sm[r])) & 0x3FFFFFFFu);
            atomicXor(&img_m[wm[r] + 1], (uint32_t)(((uint64_t)xm << (3u * sm[r])) >> 30));
        } else if (BM == 4) {
            img_m[wm[r]] = m8;
        } else {
            m_word |= m8 << (16 * r);
            if (r == 1) img_m[wm[0]] = m_word;
        }
        if (BV == 3) {
            const uint32_t xv = vc8[r] ^ v8;
            atomicXor(&img_v[wv[r]], (xv << (3u * sv[r])) & 0x3FFFFFFFu);
            atomicXor(&img_v[wv[r] + 1], (uint32_t)(((uint64_t)xv << (3u * sv[r])) >> 30));
        } else if (BV == 4) {
            img_v[wv[r]] = v8;
        } else {
            v_word |= v8 << (16 * r);
            if (r == 1) img_v[wv[0]] = v_word;
        }
    }
}

// The wide path: the same step as step_tile() for a full super-tile, with 16 consecutive
// elements per lane and 1024 per iteration.  A block is held by 8 lanes (4 for B = 64), so the
// work that is done once per lane and block (level tables, the division, the base, the hash,
// packing) is spread over twice as many elements, a group reduction is three DPP steps instead
// of four, and a block still needs only r extraction rounds.  The price is registers (four
// wavefronts per SIMD instead of five) and a 16-key sort per lane.
template <int BM, int BV, int B, bool BF16, bool MDE, bool EXT, int TILE>
__device__ __forceinline__ void step_tile16(const StepArgs &a, const uint64_t tile, const uint32_t lane,
                                            uint32_t *const slab, const uint32_t *const lds_de)
{
    constexpr int E = 16;
    constexpr int G = B / E;                       // lanes per block (8; 4 for 64-element blocks)
    constexpr int NG = 64 / G;                     // blocks per iteration (8; 16)
    constexpr int kTile = TILE;
    constexpr int kIters = kTile / kIter16;
    static_assert(kTile % kIter16 == 0, "whole iterations");
    using Lay = SlabLayout<BM, BV, B, MDE, kTile, E>;
    constexpr int NBT = kTile / B;
    constexpr int L = (1 << (BM - 1)) - 1;
    constexpr int K = (1 << BV) - 1;
    constexpr int CM = 32 / BM, CV = 32 / BV;
    constexpr int MW = kTile / CM, VW = kTile / CV;
    constexpr int VT = K + 1;
    constexpr int MT = MDE ? 2 * L + 2 : 2 * L + 1;
    constexpr int MTS = Lay::MTS;
    constexpr int kOffCol = Lay::kOffCol, kOffImgM = Lay::kOffImgM, kOffImgV = Lay::kOffImgV;
    constexpr int kOffTv = Lay::kOffTv, kOffTm = Lay::kOffTm, kOffSc = Lay::kOffSc, kSlab = Lay::kSlab;
    constexpr bool kDeTable = Lay::kDeTable;
    // A runaway column address (possible only with non-finite input) stays inside the slab.
    static_assert(kSlab >= 64 * kColStride16 + 140, "column slack");

    const uint64_t tile_e0 = tile * kTile;
    uint32_t *const img_m = slab + kOffImgM, *const img_v = slab + kOffImgV;
    float *const sc = reinterpret_cast<float *>(slab + kOffSc);
    uint32_t *const col = slab + kOffCol + lane * kColStride16;

    RawPG16<BF16> raw = load_pg16<BF16>(a, tile_e0, lane);
    const float gscale = (EXT && a.grad_scale) ? *a.grad_scale : 1.0f;
    static_assert(288 * 4 <= 64 * kColStride16, "staging must fit the column area");
    const Stage16 st(reinterpret_cast<float4 *>(slab + kOffCol), lane);

    // ---- stage the super-tile's state in LDS
    static_assert(kOffImgM % 4 == 0 && kOffImgV % 4 == 0, "128-bit staging");
    load_state_image<BM, BV, MW, VW, NBT>(a, tile, lane, img_m, img_v, sc);
    if (lane < 4) { img_m[MW + lane] = 0; img_v[VW + lane] = 0; }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    const uint32_t lig = lane & (G - 1);
    const uint32_t grp = lane / G;
    const uint32_t gshift = lane & 31u & ~(uint32_t)(G - 1);
    float *const my_tv = reinterpret_cast<float *>(slab + kOffTv) + grp * VT;
    float *const my_tm = reinterpret_cast<float *>(slab + kOffTm) + grp * MTS;
    const uint32_t tv_addr = lds_addr(my_tv), tm_addr = lds_addr(my_tm);
    const uint32_t col_addr = lds_addr(col);

    float de_level[(16 + G - 1) / G];
    uint32_t de_base = 0;
    if (MDE) {
#pragma unroll
        for (int r = 0; r < (MT + G - 1) / G; ++r) de_level[r] = DeLevels<BM>::level(lig + r * G);
        if (kDeTable) de_base = lds_addr(lds_de) - 16u * DeBuckets<BM>::kLo;
    }

#pragma unroll 1
    for (int it = 0; it < kIters; ++it) {
        const uint32_t e_loc = (uint32_t)it * kIter16 + lane * 16u;
        const uint64_t e0 = tile_e0 + e_loc;
        const uint32_t bl = (uint32_t)it * NG + grp;
        // word and slot of the first code of the lane's two runs of 8 (recomputed in every
        // iteration: cheaper in registers than carrying them; e / 10 by multiplication, exact far
        // beyond the tile size)
        static_assert(kTile <= 20480, "range of the division by 10");
        uint32_t wm[2], sm[2], wv[2], sv[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const uint32_t e = e_loc + 8u * r;
            wm[r] = (CM == 10) ? __umul24(e, 52429u) >> 19 : e / CM; sm[r] = e - wm[r] * CM;
            wv[r] = (CV == 10) ? __umul24(e, 52429u) >> 19 : e / CV; sv[r] = e - wv[r] * CV;
        }

        // ---- old state of the block and of this lane's elements (LDS)
        const float dm_old = sc[bl], dv_old = sc[NBT + bl], al_old = sc[2 * NBT + bl];
        uint32_t mc8[2], vc8[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            // (2-bit codes: both runs of the lane lie in one word)
            const uint32_t mw0 = img_m[wm[BM == 2 ? 0 : r]], mw1 = (BM == 3) ? img_m[wm[r] + 1] : 0u;
            const uint32_t vw0 = img_v[wv[BV == 2 ? 0 : r]], vw1 = (BV == 3) ? img_v[wv[r] + 1] : 0u;
            mc8[r] = extract8<BM>(mw0, mw1, BM == 2 ? 8u * r : sm[r]) & (uint32_t)((1ull << (8 * BM)) - 1ull);
            vc8[r] = extract8<BV>(vw0, vw1, BV == 2 ? 8u * r : sv[r]) & (uint32_t)((1ull << (8 * BV)) - 1ull);
        }

        // ---- level tables of this lane's block: entries lig, lig + G
        fill_level_tables<BM, BV, MDE, G>(my_tv, my_tm, lig, dm_old, dv_old, al_old, de_level);

        // ---- coalesced layout -> 16 consecutive elements per lane
        float p[16], g[16];
        lane_layout16<BF16>(raw, st, p, g);
        if (EXT) {
#pragma unroll
            for (int j = 0; j < 16; ++j) g[j] = __builtin_fmaf(a.l2, p[j], g[j] * gscale);
        }
        // next iteration's parameters and gradients, a whole iteration ahead of their use
        if (it + 1 < kIters) raw = load_pg16<BF16>(a, tile_e0 + (uint32_t)(it + 1) * kIter16, lane);

        // ---- dequantize (table look-up), EMA, parameter; new parameters streamed out
        float mh[16], vh[16];
        float m_absmax, v_unused;               // (the largest v^ is the lane's last sorted key below)
        ema_param<16, BM, BV, EXT, false, false>(a, tm_addr, tv_addr, mc8, vc8, nullptr, p, g, mh, vh, m_absmax, v_unused);
        store_params16<EXT>(a, tile_e0 + (uint32_t)it * kIter16, lane, p, st);
        wave_lds_sync();                        // the staging area becomes the column area

        // ---- the lane's v^ sorted (non-negative floats order like their bit patterns), the block
        // maxima (the lane's largest v^ is its last key), the r-th smallest v^ of the block
        float dm = u2f(group_reduce<G>(f2u(m_absmax), UMax()));
        if (dm < kTiny) dm = 0.0f;
        float dv;
        uint32_t xp_bits = 0;
        {
            uint32_t key[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) key[j] = f2u(vh[j]);
            sort16(key);
            dv = u2f(group_reduce<G>(key[15], UMax()));
            if (dv < kTiny) dv = 0.0f;
            col[16] = kInfBits;
#pragma unroll
            for (int c = 0; c < 8; ++c) *reinterpret_cast<uint2 *>(col + 2 * c) = make_uint2(key[2 * c], key[2 * c + 1]);
            xp_bits = extract_rth<G>(key[0], key[1], col_addr, a.rank_full);
        }

        // ---- the block's encoder constants
        const BlockCodec codec = block_codec<BV, G, L, MDE>(xp_bits, dm, dv, lane, lig, gshift);
        const float alpha = codec.alpha;

        // ---- encode and update the state image, one run of 8 elements at a time
        encode_into_image16<BM, BV, MDE>(a, e0, mh, vh, codec, de_base, img_m, img_v, wm, sm, wv, sv, mc8, vc8);
        if (lig == 0) { sc[bl] = dm; sc[NBT + bl] = dv; sc[2 * NBT + bl] = alpha; }
    }

    // ---- write the super-tile's state back (coalesced)
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    store_state_image<MW, VW, NBT>(a, tile, lane, img_m, img_v, sc);
}

// The DE bucket table of a workgroup: copied from constant memory once, before any wavefront
// of the workgroup can leave.
template <int BM, bool MDE, int WORDS>
__device__ __forceinline__ void load_de_table(uint32_t *lds_de)
{
    if (MDE && BM >= 3) {
        const uint32_t *src = &DeBuckets<BM>::tab.w[0][0];
        for (uint32_t w = threadIdx.x; w < (uint32_t)WORDS; w += blockDim.x) lds_de[w] = src[w];
        __syncthreads();
    }
}

// The step over one flat buffer.  Full super-tiles: one workgroup per kWaves of them.  TAIL: the
// ragged end, cut into 2560-element units and these into their 512-element iterations, one
// wavefront each (a short tensor is a latency problem: five iterations in sequence would take
// five times as long).
template <int BM, int BV, int B, bool BF16, bool MDE, bool TAIL, bool EXT>
__global__ __launch_bounds__(kWaves * 64, (!TAIL && wide_path<BM, BV, B, MDE>()) ? kWideWaves : SOLO_MIN_WAVES)
void step_kernel(const StepArgs a)
{
    constexpr int kTile = TAIL ? kTileUnit : tile_elems<BM, BV, B, MDE>();
    constexpr bool kWide = !TAIL && wide_path<BM, BV, B, MDE>();
    using Lay = SlabLayout<BM, BV, B, MDE, kTile, kWide ? 16 : 8>;
    __shared__ __attribute__((aligned(64))) uint32_t lds_slab[kWaves * Lay::kSlab];
    __shared__ __attribute__((aligned(64))) uint32_t lds_de[Lay::kDeWords];
    load_de_table<BM, MDE, Lay::kDeWords>(lds_de);

    const uint32_t lane = threadIdx.x & 63u;
    // the wavefront index is uniform: keeping it (and every address derived from the tile) in
    // scalar registers frees vector registers
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // Workgroup ids are dealt round-robin to the 8 XCDs; workgroup (x + 8 i) takes the i-th
    // group of super-tiles of XCD x's contiguous eighth of the buffer, so the wavefronts that
    // run at the same time on one XCD stream through one narrow address window.
    const uint64_t wg = (uint64_t)(blockIdx.x & (kXcds - 1)) * a.wg_per_xcd + (blockIdx.x / kXcds);
    if (TAIL) {
        // one wavefront per 512-element iteration of the 2560-element units from tail_tile0 on:
        // the ragged end of a large buffer, or the whole of a short or mid-size one.  A unit that
        // lies inside the buffer runs the code without bounds checks.
        constexpr int kChunks = kTileUnit / kIter;
        const uint64_t c = (uint64_t)blockIdx.x * kWaves + wave;
        if (c >= a.tail_chunks) return;
        const uint64_t unit = a.tail_tile0 + c / kChunks;
        if ((unit + 1) * kTileUnit <= a.n)
            step_tile<BM, BV, B, BF16, MDE, false, EXT, kTileUnit, true>(a, unit, lane, lds_slab + wave * Lay::kSlab,
                                                                         lds_de, (int)(c % kChunks));
        else
            step_tile<BM, BV, B, BF16, MDE, true, EXT, kTileUnit>(a, unit, lane, lds_slab + wave * Lay::kSlab,
                                                                  lds_de, (int)(c % kChunks));
        return;
    }
    const uint64_t tile = wg * kWaves + wave;
    if (tile >= a.n_tiles_full) return;
    if constexpr (kWide)
        step_tile16<BM, BV, B, BF16, MDE, EXT, kTile>(a, tile, lane, lds_slab + wave * Lay::kSlab, lds_de);
    else if constexpr (!TAIL)
        step_tile<BM, BV, B, BF16, MDE, false, EXT, kTile>(a, tile, lane, lds_slab + wave * Lay::kSlab, lds_de);
}

// The step over many tensors in one launch.  Every tensor is cut into units of the format's
// super-tile size and its ragged end into 512-element iterations; one wavefront takes one entry
// of the map, finds its tensor in the table (a scalar look-up) and runs the full-tile code on a
// unit or the bounds-checked code on one iteration of a ragged end.  Blocks never span tensors:
// each tensor is quantized on its own.
template <int BM, int BV, int B, bool BF16, bool MDE, bool EXT>
__global__ __launch_bounds__(kWaves * 64, (wide_path<BM, BV, B, MDE>() ? kWideWaves : SOLO_MIN_WAVES))
void multi_kernel(const MultiArgs ma)
{
    constexpr int kUnit = tile_elems<BM, BV, B, MDE>();
    constexpr bool kWide = wide_path<BM, BV, B, MDE>();
    using Lay = SlabLayout<BM, BV, B, MDE, kUnit, kWide ? 16 : 8>;        // the wide slab is the larger one
    static_assert(Lay::kSlab >= SlabLayout<BM, BV, B, MDE, kUnit, 8>::kSlab, "one slab serves both code paths");
    __shared__ __attribute__((aligned(64))) uint32_t lds_slab[kWaves * Lay::kSlab];
    __shared__ __attribute__((aligned(64))) uint32_t lds_de[Lay::kDeWords];
    load_de_table<BM, MDE, Lay::kDeWords>(lds_de);

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint64_t wg = (uint64_t)(blockIdx.x & (kXcds - 1)) * ma.groups_per_xcd + (blockIdx.x / kXcds);
    const uint64_t unit = wg * kWaves + wave;
    if (unit >= ma.total_units) return;
    const uint32_t me = ma.unit_map[unit];                      // uniform: scalar loads
    const TensorEntry &e = ma.entries[me & kMapTensorMask];
    StepArgs a = ma.common;
    a.param = e.param; a.param_bf16 = e.param_bf16; a.grad = e.grad;
    a.m_words = e.m_words; a.m_scale = e.m_scale;
    a.v_words = e.v_words; a.v_scale = e.v_scale; a.v_base = e.v_base;
    a.n = e.n; a.index_offset = e.index_offset;
    uint32_t *const slab = lds_slab + wave * Lay::kSlab;
    if (!(me & kMapRagged)) {
        const uint64_t tile = unit - e.unit0;
        if constexpr (kWide) step_tile16<BM, BV, B, BF16, MDE, EXT, kUnit>(a, tile, lane, slab, lds_de);
        else step_tile<BM, BV, B, BF16, MDE, false, EXT, kUnit>(a, tile, lane, slab, lds_de);
    } else {
        step_tile<BM, BV, B, BF16, MDE, true, true, kUnit>(a, a.n / kUnit, lane, slab, lds_de,
                                                           (int)((me >> kMapChunkShift) & 0x7Fu));
    }
}

// The multi-tensor step of the formats that always run one wavefront per 512-element iteration:
// a map entry stands for a 2560-element unit of its tensor (the last one of a tensor may be
// shorter), five consecutive wavefronts take its five iterations.
template <int BM, int BV, int B, bool BF16, bool MDE, bool EXT>
__global__ __launch_bounds__(kWaves * 64, SOLO_MIN_WAVES)
void multi_chunk_kernel(const MultiArgs ma)
{
    constexpr int kChunks = kTileUnit / kIter;
    using Lay = SlabLayout<BM, BV, B, MDE, kTileUnit, 8>;
    __shared__ __attribute__((aligned(64))) uint32_t lds_slab[kWaves * Lay::kSlab];
    __shared__ __attribute__((aligned(64))) uint32_t lds_de[Lay::kDeWords];
    load_de_table<BM, MDE, Lay::kDeWords>(lds_de);

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint64_t slot = (uint64_t)blockIdx.x * kWaves + wave;
    const uint64_t unit = slot / kChunks;
    const int chunk = (int)(slot % kChunks);
    if (unit >= ma.total_units) return;
    const uint32_t me = ma.unit_map[unit];                      // uniform: scalar loads
    const TensorEntry &e = ma.entries[me & kMapTensorMask];
    StepArgs a = ma.common;
    a.param = e.param; a.param_bf16 = e.param_bf16; a.grad = e.grad;
    a.m_words = e.m_words; a.m_scale = e.m_scale;
    a.v_words = e.v_words; a.v_scale = e.v_scale; a.v_base = e.v_base;
    a.n = e.n; a.index_offset = e.index_offset;
    uint32_t *const slab = lds_slab + wave * Lay::kSlab;
    const uint64_t tile = unit - e.unit0;
    if ((tile + 1) * kTileUnit <= a.n)
        step_tile<BM, BV, B, BF16, MDE, false, EXT, kTileUnit, true>(a, tile, lane, slab, lds_de, chunk);
    else if (tile * kTileUnit + (uint64_t)chunk * kIter < (a.n + 79) / 80 * 80)   // up to the end of the last code word
        step_tile<BM, BV, B, BF16, MDE, true, true, kTileUnit>(a, tile, lane, slab, lds_de, chunk);
}

// Host-side launcher of one instantiation family (fixed bits_m and 1st-moment codebook);
// defined in solo_step_m{2,3,4}{,_de}.hip so that the families compile in parallel.
template <int BM, bool MDE>
hipError_t launch_step(uint32_t bits_v, uint32_t block_size, bool bf16, const StepArgs &args,
                       hipStream_t stream);

template <int BM, int BV, int B, bool BF16, bool MDE>
hipError_t launch_one(const StepArgs &args_in, hipStream_t stream)
{
    StepArgs args = args_in;                   // the tiling belongs to the instantiation
    constexpr int kTile = tile_elems<BM, BV, B, MDE>();
    // A short or mid-size tensor is all latency: its super-tiles would be too few to fill the
    // machine (a wavefront walks a super-tile in 5 or 10 dependent iterations), so it goes as a
    // whole, in one launch, to the kernel of the ragged end: one wavefront per 512 elements.
    const bool small = args.n <= chunked_up_to<B, BF16, MDE>();
    args.n_tiles_full = small ? 0 : args.n / kTile;
    args.wg_per_xcd = ((args.n_tiles_full + kWaves - 1) / kWaves + kXcds - 1) / kXcds;
    const bool has_tail = small ? args.n != 0 : (args.n % kTile) != 0;
    args.tail_tile0 = args.n_tiles_full * (kTile / kTileUnit);
    // its 512-element iterations, up to the end of the last code word (80 = lcm of 16, 10 and 8
    // codes per word): the unused fields of that word are written as zeros like every other field
    const uint64_t tail_e0 = args.tail_tile0 * kTileUnit;
    args.tail_chunks = ((args.n + 79) / 80 * 80 - tail_e0 + kIter - 1) / kIter;
    const bool ext = args.param_bf16 || args.grad_scale || args.belief || args.l2 != 0.0f;
    if (args.n_tiles_full) {
        const uint64_t grid = args.wg_per_xcd * kXcds;
        if (grid > 0x7FFFFFFFull) return hipErrorInvalidValue;
        if (ext)
            hipLaunchKernelGGL((step_kernel<BM, BV, B, BF16, MDE, false, true>), dim3((uint32_t)grid), dim3(kWaves * 64), 0, stream, args);
        else
            hipLaunchKernelGGL((step_kernel<BM, BV, B, BF16, MDE, false, false>), dim3((uint32_t)grid), dim3(kWaves * 64), 0, stream, args);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (has_tail) {                            // the ragged end: one wavefront per 512 elements, always the full-featured kernel
        if ((args.tail_chunks + kWaves - 1) / kWaves > 0x7FFFFFFFull) return hipErrorInvalidValue;
        const uint32_t tail_groups = (uint32_t)((args.tail_chunks + kWaves - 1) / kWaves);
        hipLaunchKernelGGL((step_kernel<BM, BV, B, BF16, MDE, true, true>), dim3(tail_groups), dim3(kWaves * 64), 0, stream, args);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <int BM, bool MDE>
hipError_t launch_multi(uint32_t bits_v, uint32_t block_size, bool bf16, const MultiArgs &args,
                        hipStream_t stream);

template <int BM, bool MDE>
hipError_t launch_multi_impl(uint32_t bits_v, uint32_t block_size, bool bf16, const MultiArgs &args,
                             hipStream_t stream)
{
    const uint64_t grid = args.groups_per_xcd * kXcds;
    if (grid == 0 || grid > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const StepArgs &c = args.common;
    const bool ext = args.any_bf16_copy || c.grad_scale || c.belief || c.l2 != 0.0f;
    const bool chunked = multi_chunked(bf16, MDE);
#define SOLO_LAUNCH(BV_, B_, BF_, EXT_)                                                                 \
    do {                                                                                                \
        if (chunked)                                                                                    \
            hipLaunchKernelGGL((multi_chunk_kernel<BM, BV_, B_, BF_, MDE, EXT_>), dim3((uint32_t)grid), \
                               dim3(kWaves * 64), 0, stream, args);                                     \
        else                                                                                            \
            hipLaunchKernelGGL((multi_kernel<BM, BV_, B_, BF_, MDE, EXT_>), dim3((uint32_t)grid),       \
                               dim3(kWaves * 64), 0, stream, args);                                     \
    } while (0)
#define SOLO_CASE(BV_, B_)                                                                              \
    if (bits_v == BV_ && block_size == B_) {                                                            \
        if (bf16) { if (ext) SOLO_LAUNCH(BV_, B_, true, true); else SOLO_LAUNCH(BV_, B_, true, false); } \
        else      { if (ext) SOLO_LAUNCH(BV_, B_, false, true); else SOLO_LAUNCH(BV_, B_, false, false); } \
        return hipGetLastError();                                                                       \
    }
    SOLO_CASE(2, 64) SOLO_CASE(2, 128) SOLO_CASE(3, 64) SOLO_CASE(3, 128) SOLO_CASE(4, 64) SOLO_CASE(4, 128)
#undef SOLO_CASE
#undef SOLO_LAUNCH
    return hipErrorInvalidValue;
}

template <int BM, bool MDE>
hipError_t launch_step_impl(uint32_t bits_v, uint32_t block_size, bool bf16, const StepArgs &args,
                            hipStream_t stream)
{
#define SOLO_CASE(BV_, B_)                                                             \
    if (bits_v == BV_ && block_size == B_)                                             \
        return bf16 ? launch_one<BM, BV_, B_, true, MDE>(args, stream)                 \
                    : launch_one<BM, BV_, B_, false, MDE>(args, stream);
    SOLO_CASE(2, 64) SOLO_CASE(2, 128) SOLO_CASE(3, 64) SOLO_CASE(3, 128) SOLO_CASE(4, 64) SOLO_CASE(4, 128)
#undef SOLO_CASE
    return hipErrorInvalidValue;
}

}  // namespace solo
