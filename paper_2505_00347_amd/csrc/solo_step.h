// Device code of the fused SOLO AdamW step for gfx950 (wave64).
//
// Work decomposition.  The flat buffer is cut into super-tiles of 2560
// elements (a multiple of every block size and of 16, 10 and 8 codes per
// word, so a super-tile owns whole blocks and whole code words).  One
// wavefront owns one super-tile and walks it in five iterations of 512
// elements; a lane owns 8 consecutive elements per iteration, so a block of
// 128 (64) elements is held by 16 (8) neighbouring lanes, i.e. one DPP row
// (half row), and every per-block reduction is a few DPP steps.  Nothing is
// shared between wavefronts: there is no workgroup barrier in the kernel.
//
// Per iteration and lane: 128-bit loads of 8 parameters and 8 gradients, the
// one or two code words that hold its 8+8 codes, the three block scalars;
// unpack, dequantize, both EMAs, parameter update and 128-bit store; block
// maxima by DPP butterflies; the quantile by a per-lane sorting network and
// r rounds of "extract the block minimum"; the base alpha; both encoders;
// codes OR-ed into an LDS image of the super-tile's code words, which is
// written out with coalesced stores after the fifth iteration.
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

namespace solo {

constexpr int kTile = 2560;        // elements per wavefront super-tile
constexpr int kIter = 512;         // elements per iteration (64 lanes x 8)
constexpr int kIters = kTile / kIter;
constexpr int kWaves = 4;          // wavefronts per workgroup
constexpr float kTiny = 0x1p-100f; // block maxima below this are stored as 0
constexpr float kRhoMin = 0x1p-64f;
constexpr uint32_t kInfBits = 0x7F800000u;

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
    uint64_t index_offset;  // global index of element 0 (multiple of 8)
    float beta1, omb1, beta2, omb2;
    float decay;            // 1 - lr * weight_decay
    float step_size;        // lr / (1 - beta1^t)
    float inv_sqrt_bc2;     // 1 / sqrt(1 - beta2^t)
    float eps;
    float quantile_p;
    uint32_t rank_full;     // rank of the quantile in a full block
    uint32_t key0, key1, key2;
    float xi_scale, xi_offset;  // 2^-24 and 2^-25 - 0.5, or 0 and 0 (xi off)
};

// ---------------------------------------------------------------- cross-lane

template <int CTRL>
__device__ __forceinline__ uint32_t dpp(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, false);
}

// Butterfly over the G (8 or 16) lanes that hold one block: lane^1 and lane^2
// by quad permutes, then mirror inside the half row, then inside the row.
// Every lane ends with the result of its whole group.
template <int G, typename Op>
__device__ __forceinline__ uint32_t group_reduce(uint32_t x, Op op)
{
    x = op(x, dpp<0xB1>(x));    // quad_perm [1,0,3,2]
    x = op(x, dpp<0x4E>(x));    // quad_perm [2,3,0,1]
    x = op(x, dpp<0x141>(x));   // row_half_mirror
    if (G == 16) x = op(x, dpp<0x140>(x));  // row_mirror
    return x;
}

struct UMin { __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a < b ? a : b; } };
struct UMax { __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a > b ? a : b; } };

__device__ __forceinline__ uint32_t f2u(float x) { return __builtin_bit_cast(uint32_t, x); }
__device__ __forceinline__ float u2f(uint32_t x) { return __builtin_bit_cast(float, x); }

__device__ __forceinline__ void cswap(uint32_t &a, uint32_t &b)
{
    uint32_t lo = a < b ? a : b, hi = a < b ? b : a;
    a = lo; b = hi;
}

// Batcher's odd-even merge sort for 8 keys, 19 compare-exchanges.
__device__ __forceinline__ void sort8(uint32_t (&k)[8])
{
    cswap(k[0], k[1]); cswap(k[2], k[3]); cswap(k[4], k[5]); cswap(k[6], k[7]);
    cswap(k[0], k[2]); cswap(k[1], k[3]); cswap(k[4], k[6]); cswap(k[5], k[7]);
    cswap(k[1], k[2]); cswap(k[5], k[6]);
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

// Last level alpha^K of the log codebook, K = 2^BV - 1, multiplied in the same
// order as the dequantizer: ((a * a^2) * a^4) * a^8.
template <int BV>
__device__ __forceinline__ float last_level(float a)
{
    float a2 = a * a;
    float r = a * a2;
    if (BV >= 3) { float a4 = a2 * a2; r = r * a4; if (BV >= 4) { float a8 = a4 * a4; r = r * a8; } }
    return r;
}

// alpha = rho^(1/K): the largest binary32 in (0,1] whose last level does not
// exceed rho (0 < rho < 1).  A hardware exp2/log2 guess is walked to that value
// one ulp at a time; both walks are bounded.
template <int BV>
__device__ __forceinline__ float solve_base(float rho)
{
    constexpr float invK = 1.0f / (float)((1 << BV) - 1);
    float y0 = __builtin_amdgcn_exp2f(__builtin_amdgcn_logf(rho) * invK);
    uint32_t y = f2u(y0);
    if (!(y <= 0x3F800000u)) y = 0x3F800000u;
    if (y < 0x00800000u) y = 0x00800000u;
    for (int i = 0; i < 512 && last_level<BV>(u2f(y)) > rho; ++i) --y;
    for (int i = 0; i < 512 && y < 0x3F800000u && last_level<BV>(u2f(y + 1)) <= rho; ++i) ++y;
    return u2f(y);
}

// Eight consecutive BITS-wide codes starting at slot `slot` of word w0 (the
// run may continue in w1 for 3-bit codes, ten to a word).
template <int BITS>
__device__ __forceinline__ uint32_t extract8(uint32_t w0, uint32_t w1, uint32_t slot)
{
    if (BITS == 3) {
        uint64_t both = (uint64_t)w0 | ((uint64_t)w1 << 30);
        return (uint32_t)(both >> (3u * slot)) & 0xFFFFFFu;
    }
    return w0 >> (BITS * slot);   // 2-bit: slot 0 or 8; 4-bit: slot 0
}

// ------------------------------------------------------------------- kernel

template <int BM, int BV, int B, bool BF16, bool TAIL>
__global__ __launch_bounds__(kWaves * 64) void step_kernel(const StepArgs a)
{
    constexpr int G = B / 8;                       // lanes per block
    constexpr int L = (1 << (BM - 1)) - 1;
    constexpr int K = (1 << BV) - 1;
    constexpr int CM = 32 / BM, CV = 32 / BV;      // codes per word
    constexpr int MW = kTile / CM, VW = kTile / CV; // words per super-tile
    constexpr uint32_t MMASK = (1u << BM) - 1u, VMASK = (1u << BV) - 1u;

    __shared__ uint32_t lds_m[kWaves][MW + 1];     // new code words of the super-tile
    __shared__ uint32_t lds_v[kWaves][VW + 1];
    __shared__ uint32_t lds_sort[kWaves][9 * 64];  // per-lane sorted columns + sentinel row

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = threadIdx.x >> 6;
    const uint64_t tile = TAIL ? a.n_tiles_full : (uint64_t)blockIdx.x * kWaves + wave;
    if (!TAIL && tile >= a.n_tiles_full) return;

    uint32_t *out_m = lds_m[wave], *out_v = lds_v[wave];
    uint32_t *col = &lds_sort[wave][lane];
    for (uint32_t w = lane; w < MW + 1; w += 64) out_m[w] = 0;
    for (uint32_t w = lane; w < VW + 1; w += 64) out_v[w] = 0;
    col[8 * 64] = kInfBits;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    const uint64_t nblk = (a.n + B - 1) / B;
    const uint64_t m_total = (a.n + CM - 1) / CM, v_total = (a.n + CV - 1) / CV;
    const uint64_t tile_e0 = tile * kTile;
    const uint32_t lig = lane & (G - 1);               // lane in group
    const uint32_t gbase = lane & ~(uint32_t)(G - 1);
    const uint32_t below = (1u << lig) - 1u;
    const uint32_t gmask = (G == 16) ? 0xFFFFu : 0xFFu;

#pragma unroll 1
    for (int it = 0; it < kIters; ++it) {
        const uint32_t e_loc = (uint32_t)it * kIter + lane * 8u;   // element inside the tile
        const uint64_t e0 = tile_e0 + e_loc;
        uint64_t blk = e0 / B;
        // elements of this lane's block that exist (B except in the last block)
        uint32_t nb = B;
        bool blk_ok = true;
        if (TAIL) {
            blk_ok = blk < nblk;
            const uint64_t bstart = blk * B;
            nb = blk_ok ? (uint32_t)((a.n - bstart) < (uint64_t)B ? (a.n - bstart) : (uint64_t)B) : 0u;
            if (!blk_ok) blk = nblk - 1;                   // keep the loads in bounds
        }

        // ---- loads
        float p[8], g[8];
        bool ok[8];
        if (!TAIL) {
            const float4 *pp = reinterpret_cast<const float4 *>(a.param + e0);
            float4 p0 = pp[0], p1 = pp[1];
            p[0] = p0.x; p[1] = p0.y; p[2] = p0.z; p[3] = p0.w;
            p[4] = p1.x; p[5] = p1.y; p[6] = p1.z; p[7] = p1.w;
            if (BF16) {
                const uint4 gb = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(a.grad) + e0);
                g[0] = u2f(gb.x << 16); g[1] = u2f(gb.x & 0xFFFF0000u);
                g[2] = u2f(gb.y << 16); g[3] = u2f(gb.y & 0xFFFF0000u);
                g[4] = u2f(gb.z << 16); g[5] = u2f(gb.z & 0xFFFF0000u);
                g[6] = u2f(gb.w << 16); g[7] = u2f(gb.w & 0xFFFF0000u);
            } else {
                const float4 *gp = reinterpret_cast<const float4 *>(static_cast<const float *>(a.grad) + e0);
                float4 g0 = gp[0], g1 = gp[1];
                g[0] = g0.x; g[1] = g0.y; g[2] = g0.z; g[3] = g0.w;
                g[4] = g1.x; g[5] = g1.y; g[6] = g1.z; g[7] = g1.w;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) ok[j] = true;
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                ok[j] = (e0 + j) < a.n;
                p[j] = ok[j] ? a.param[e0 + j] : 0.0f;
                if (BF16) g[j] = ok[j] ? u2f((uint32_t)static_cast<const uint16_t *>(a.grad)[e0 + j] << 16) : 0.0f;
                else      g[j] = ok[j] ? static_cast<const float *>(a.grad)[e0 + j] : 0.0f;
            }
        }
        const uint32_t wm = e_loc / CM, sm = e_loc % CM;    // word and slot inside the tile
        const uint32_t wv = e_loc / CV, sv = e_loc % CV;
        uint64_t gm0 = tile * MW + wm, gm1 = tile * MW + (wm + 1 < MW ? wm + 1 : wm);
        uint64_t gv0 = tile * VW + wv, gv1 = tile * VW + (wv + 1 < VW ? wv + 1 : wv);
        if (TAIL) {
            gm0 = gm0 < m_total ? gm0 : m_total - 1; gm1 = gm1 < m_total ? gm1 : m_total - 1;
            gv0 = gv0 < v_total ? gv0 : v_total - 1; gv1 = gv1 < v_total ? gv1 : v_total - 1;
        }
        const uint32_t mw0 = a.m_words[gm0], mw1 = (BM == 3) ? a.m_words[gm1] : 0u;
        const uint32_t vw0 = a.v_words[gv0], vw1 = (BV == 3) ? a.v_words[gv1] : 0u;
        const float dm_old = a.m_scale[blk], dv_old = a.v_scale[blk], al_old = a.v_base[blk];

        // ---- dequantize, EMA, parameter
        const uint32_t mc8 = extract8<BM>(mw0, mw1, sm);
        const uint32_t vc8 = extract8<BV>(vw0, vw1, sv);
        const float s_m = dm_old / (float)L;
        const float P1 = al_old, P2 = P1 * P1, P4 = P2 * P2, P8 = P4 * P4;
        float mh[8], vh[8];
        uint32_t m_absmax = 0, v_max = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int cm = (int)((mc8 >> (BM * j)) & MMASK);
            const uint32_t cv = (vc8 >> (BV * j)) & VMASK;
            const float mt = (float)(cm - L) * s_m;
            float y = (cv & 1u) ? P1 : 1.0f;
            if (cv & 2u) y = y * P2;
            if (BV >= 3) { if (cv & 4u) y = y * P4; }
            if (BV >= 4) { if (cv & 8u) y = y * P8; }
            const float vt = y * dv_old;
            mh[j] = __builtin_fmaf(a.beta1, mt, a.omb1 * g[j]);
            vh[j] = __builtin_fmaf(a.beta2, vt, a.omb2 * (g[j] * g[j]));
            // parameter: decoupled decay, bias-corrected Adam direction
            const float denom = __builtin_fmaf(__builtin_amdgcn_sqrtf(vh[j]), a.inv_sqrt_bc2, a.eps);
            p[j] = __builtin_fmaf(p[j], a.decay, -(a.step_size * mh[j]) * __builtin_amdgcn_rcpf(denom));
            if (TAIL && !ok[j]) { mh[j] = 0.0f; vh[j] = 0.0f; }
            const uint32_t am = f2u(mh[j]) & 0x7FFFFFFFu;
            m_absmax = am > m_absmax ? am : m_absmax;
            v_max = f2u(vh[j]) > v_max ? f2u(vh[j]) : v_max;
        }
        if (!TAIL) {
            float4 *pp = reinterpret_cast<float4 *>(a.param + e0);
            pp[0] = make_float4(p[0], p[1], p[2], p[3]);
            pp[1] = make_float4(p[4], p[5], p[6], p[7]);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) if (ok[j]) a.param[e0 + j] = p[j];
        }

        // ---- block statistics: maxima, then the r-th smallest v^
        float dm = u2f(group_reduce<G>(m_absmax, UMax()));
        float dv = u2f(group_reduce<G>(v_max, UMax()));
        if (dm < kTiny) dm = 0.0f;
        if (dv < kTiny) dv = 0.0f;

        uint32_t key[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) key[j] = (TAIL && !ok[j]) ? kInfBits : f2u(vh[j]);
        sort8(key);
#pragma unroll
        for (int j = 0; j < 8; ++j) col[j * 64] = key[j];
        uint32_t r_mine = a.rank_full;
        if (TAIL) {
            float x = __builtin_ceilf(a.quantile_p * (float)nb);
            r_mine = x < 1.0f ? 1u : (uint32_t)x;
            r_mine = r_mine > nb ? nb : r_mine;
        }
        uint32_t head = key[0], ptr = 0, xp_bits = 0;
        for (uint32_t k = 0; k < a.rank_full; ++k) {
            const uint32_t mn = group_reduce<G>(head, UMin());
            const bool is_min = head == mn;
            const uint64_t bal = __builtin_amdgcn_ballot_w64(is_min);
            const uint32_t grp = (uint32_t)(bal >> gbase) & gmask;
            const bool win = is_min && ((grp & below) == 0u);   // lowest lane of the group pops
            if (k + 1 == r_mine) xp_bits = mn;
            ptr += (win && ptr < 8u) ? 1u : 0u;   // row 8 is the +inf sentinel
            head = col[ptr * 64];
        }

        // ---- log base of the block
        float alpha = 1.0f, inv_l2a = 0.0f, rdv = 0.0f, bias = 1.0f;
        if (dv > 0.0f) {
            float rho = u2f(xp_bits) / dv;
            rho = rho < kRhoMin ? kRhoMin : rho;
            if (rho < 1.0f) {
                alpha = solve_base<BV>(rho);
                inv_l2a = __builtin_amdgcn_rcpf(__builtin_amdgcn_logf(alpha));
                rdv = __builtin_amdgcn_rcpf(dv);
                bias = 0.0f;
            }
        }

        // ---- xi: one hashed start and stride per 8 elements
        const uint64_t gidx = (a.index_offset + e0) >> 3;
        const uint32_t X = mix32(((uint32_t)gidx ^ a.key0) + (uint32_t)(gidx >> 32) * a.key2);
        const uint32_t Y = mix32(X ^ a.key1) | 1u;

        // ---- encode and pack
        const float inv_s = dm > 0.0f ? (float)L / dm : 0.0f;
        uint32_t m8 = 0, v8 = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float tm = __builtin_rintf(mh[j] * inv_s);
            tm = tm > (float)L ? (float)L : tm;
            tm = tm < -(float)L ? -(float)L : tm;
            uint32_t cm = (uint32_t)(L + (int)tm);
            const uint32_t u = (X + (uint32_t)j * Y) >> 8;
            const float xi = __builtin_fmaf((float)u, a.xi_scale, a.xi_offset);
            const float ratio = __builtin_fmaf(vh[j], rdv, bias);
            float tv = __builtin_fmaf(__builtin_amdgcn_logf(ratio), inv_l2a, xi);
            tv = __builtin_rintf(tv);
            tv = tv < (float)K ? tv : (float)K;     // also catches +inf (v^ = 0) and NaN
            tv = tv > 0.0f ? tv : 0.0f;
            uint32_t cv = (uint32_t)tv;
            if (TAIL && !ok[j]) { cm = 0; cv = 0; }
            m8 |= cm << (BM * j);
            v8 |= cv << (BV * j);
        }
        if (BM == 3) {
            atomicOr(&out_m[wm], (m8 << (3u * sm)) & 0x3FFFFFFFu);
            atomicOr(&out_m[wm + 1], (uint32_t)(((uint64_t)m8 << (3u * sm)) >> 30));
        } else {
            atomicOr(&out_m[wm], m8 << (BM * sm));
        }
        if (BV == 3) {
            atomicOr(&out_v[wv], (v8 << (3u * sv)) & 0x3FFFFFFFu);
            atomicOr(&out_v[wv + 1], (uint32_t)(((uint64_t)v8 << (3u * sv)) >> 30));
        } else {
            atomicOr(&out_v[wv], v8 << (BV * sv));
        }
        if (lig == 0 && blk_ok) {
            a.m_scale[blk] = dm;
            a.v_scale[blk] = dv;
            a.v_base[blk] = alpha;
        }
    }

    // ---- write the super-tile's code words
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    for (uint32_t w = lane; w < MW; w += 64) {
        const uint64_t gw = tile * MW + w;
        if (!TAIL || gw < m_total) a.m_words[gw] = out_m[w];
    }
    for (uint32_t w = lane; w < VW; w += 64) {
        const uint64_t gw = tile * VW + w;
        if (!TAIL || gw < v_total) a.v_words[gw] = out_v[w];
    }
}

// Host-side launcher of one instantiation family (fixed bits_m); defined in
// solo_step_m{2,3,4}.hip so that the families compile in parallel.
template <int BM>
hipError_t launch_step(uint32_t bits_v, uint32_t block_size, bool bf16, const StepArgs &args,
                       bool has_tail, hipStream_t stream);

template <int BM, int BV, int B, bool BF16>
hipError_t launch_one(const StepArgs &args, bool has_tail, hipStream_t stream)
{
    if (args.n_tiles_full) {
        const uint64_t grid = (args.n_tiles_full + kWaves - 1) / kWaves;
        hipLaunchKernelGGL((step_kernel<BM, BV, B, BF16, false>), dim3((uint32_t)grid), dim3(kWaves * 64), 0, stream, args);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (has_tail) {
        hipLaunchKernelGGL((step_kernel<BM, BV, B, BF16, true>), dim3(1), dim3(64), 0, stream, args);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <int BM>
hipError_t launch_step_impl(uint32_t bits_v, uint32_t block_size, bool bf16, const StepArgs &args,
                            bool has_tail, hipStream_t stream)
{
#define SOLO_CASE(BV_, B_)                                                             \
    if (bits_v == BV_ && block_size == B_)                                             \
        return bf16 ? launch_one<BM, BV_, B_, true>(args, has_tail, stream)            \
                    : launch_one<BM, BV_, B_, false>(args, has_tail, stream);
    SOLO_CASE(2, 64) SOLO_CASE(2, 128) SOLO_CASE(3, 64) SOLO_CASE(3, 128) SOLO_CASE(4, 64) SOLO_CASE(4, 128)
#undef SOLO_CASE
    return hipErrorInvalidValue;
}

}  // namespace solo
