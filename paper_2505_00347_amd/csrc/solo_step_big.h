// The fused SOLO AdamW step for blocks of 2048 elements (the large-block setting of the paper's
// block-size comparison, Sec. 4.2), gfx950, wave64.
//
// A block of 2048 elements is held by one workgroup of four wavefronts, 512 elements each, eight
// consecutive elements per lane: the element-wise part (decode by table look-up, both EMAs, the
// parameter, the encoders, the 32-bit words of the code streams) is that of the 512-element
// iterations of solo_step.h, one iteration per wavefront, and runs without any exchange between
// the wavefronts.  What a block of this size changes is the block statistics:
//   * Delta_m' and Delta_v' are maxima over four wavefronts: DPP inside a row, four lane reads
//     across the rows, four words of LDS and one barrier across the wavefronts;
//   * the p-quantile is the rank-205 element of 2048 values (p = 0.1), far too deep for rounds
//     of "extract the minimum".  It is found by a radix select on the bit patterns (non-negative
//     floats order like their bits): three passes over 11 + 10 + 10 bits, each a histogram of the
//     keys that still match the selected prefix (LDS atomics), one barrier, and two prefix sums
//     (DPP scans) that every wavefront runs for itself to find the bin that holds the rank.
//     After the third pass the prefix is the order statistic itself, multiplicities included,
//     exactly.  Four barriers per block in all.
//   * the base alpha, the division and the level tables are computed by every wavefront (every
//     16 lanes) for itself: cheaper than another barrier.
// One workgroup per block, every wavefront stages and writes back the words of its own 512
// elements (whole 128-byte lines for 2- and 4-bit codes; ten-to-a-word codes by one atomic XOR
// per word at the memory side, since a block does not end on a word).
#pragma once
#include "solo_step.h"

namespace solo {

constexpr int kBigBlock = 2048;
constexpr int kBigWaves = kBigBlock / kIter;      // 4 wavefronts, one workgroup per block
static_assert(kBigWaves == 4, "one workgroup of four wavefronts per block");

// LDS of a workgroup (32-bit words).  `work` first serves the four wavefronts as the staging
// areas of their layout transpositions (64 x 12 words each), then, behind the barrier of the block
// maxima, the whole workgroup as the histograms of the selection.  A histogram keeps 4 pad words
// after the 32 (16) bins that one lane sums, so that the lanes' 128-bit reads spread over the banks.
struct BigLayout {
    static constexpr int kStage = 64 * kColStride;            // per wavefront
    static constexpr int kHist0 = 0, kHist1 = 2048 + 4 * 64, kHist2 = kHist1 + 1024 + 4 * 64;
    static constexpr int kWork = kHist2 + 1024 + 4 * 64;      // 4864 words
    static constexpr int kOffImgM = 0;                        // per wavefront: its words of each code stream (<= 64, + 1)
    static constexpr int kOffImgV = 68;
    static constexpr int kOffTv = 144;                        // level tables, 64-byte aligned
    static constexpr int kOffTm = 160;
    static constexpr int kSlab = 176;
};
static_assert(BigLayout::kWork >= kBigWaves * BigLayout::kStage, "the staging areas lie inside the work area");

// Maximum over the 64 lanes of a wavefront (uniform result).
__device__ __forceinline__ uint32_t wave_max(uint32_t x)
{
    x = group_reduce<16>(x, UMax());
    const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)x, 0), b = (uint32_t)__builtin_amdgcn_readlane((int)x, 16);
    const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)x, 32), d = (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
    return umax(umax(a, b), umax(c, d));
}

// Inclusive prefix sum over the 64 lanes of a wavefront: four shifted adds inside every row of 16
// lanes, then the last lane of a row is added to the rows behind it.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t x)
{
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xF, 0xF, true);   // row_shr:1
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xF, 0xF, true);   // row_shr:2
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xF, 0xF, true);   // row_shr:4
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xF, 0xF, true);   // row_shr:8
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xA, 0xF, false);  // row_bcast:15 into rows 1 and 3
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xC, 0xF, false);  // row_bcast:31 into rows 2 and 3
    return x;
}

// The rank-th smallest (1-based, uniform over the workgroup) of the 8 keys that each of the 256
// threads holds: bit patterns of non-negative floats, +inf for absent elements (the rank never
// reaches those).  Radix select over 11 + 10 + 10 bits.  A pass: every thread adds its keys that
// still match the selected prefix to the pass's histogram (in `work`, zeroed before
// the workgroup's previous barrier), one barrier, and then every wavefront finds the bin of the
// rank for itself: a lane sums 32 (16) consecutive bins, a prefix sum over the wavefront names
// the lane whose bins hold the rank, and a second prefix sum over that lane's bins, one per
// lane, names the bin.  No exchange between the wavefronts beyond the histogram.
__device__ __forceinline__ uint32_t select_rank(const uint32_t (&key)[8], uint32_t rank, uint32_t lane, uint32_t *work)
{
    uint32_t prefix = 0;                          // the bits selected so far (bit 31 of a key is 0)
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
        constexpr int kBits[3] = {11, 10, 10}, kShift[3] = {20, 10, 0};
        constexpr int kOff[3] = {BigLayout::kHist0, BigLayout::kHist1, BigLayout::kHist2};
        const int bits = kBits[pass], sh = kShift[pass];
        const uint32_t bins = 1u << bits, per = bins / 64u;          // 32, 16, 16 bins per lane
        const int lper = bits - 6;                                   // log2(per)
        uint32_t *const h = work + kOff[pass];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const bool match = pass == 0 || (key[j] >> (sh + bits)) == prefix;
            const uint32_t b = (key[j] >> sh) & (bins - 1u);
            if (match) atomicAdd(&h[b + ((b >> lper) << 2)], 1u);
        }
        __syncthreads();
        uint32_t s = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if ((uint32_t)(4 * i) < per) {
                const uint4 c4 = reinterpret_cast<const uint4 *>(h)[lane * (per / 4u + 1u) + (uint32_t)i];
                s += (c4.x + c4.y) + (c4.z + c4.w);
            }
        }
        const uint32_t incl = wave_inclusive_sum(s);
        const uint64_t holder = __builtin_amdgcn_ballot_w64(incl - s < rank && rank <= incl);   // one lane
        const uint32_t sel = (uint32_t)__builtin_ctzll(holder | (1ull << 63));
        rank -= (uint32_t)__builtin_amdgcn_readlane((int)(incl - s), (int)sel);
        const uint32_t c = lane < per ? h[sel * (per + 4u) + lane] : 0u;
        const uint32_t incl2 = wave_inclusive_sum(c);
        const uint64_t holder2 = __builtin_amdgcn_ballot_w64(incl2 - c < rank && rank <= incl2);
        const uint32_t sel2 = (uint32_t)__builtin_ctzll(holder2 | (1ull << 63));
        rank -= (uint32_t)__builtin_amdgcn_readlane((int)(incl2 - c), (int)sel2);
        prefix = (prefix << bits) | (sel * per + sel2);
    }
    return prefix;
}

// The whole step for block `blk` of 2048 elements (TAIL: the last, shorter block of the buffer,
// with bounds checks on every element), executed by the four wavefronts of the calling workgroup.
template <int BM, int BV, bool BF16, bool MDE, bool TAIL, bool EXT>
__device__ __forceinline__ void step_block_big(const StepArgs &a, const uint64_t blk, const uint32_t lane,
                                               const uint32_t wave, uint32_t *const slab, uint32_t *const work,
                                               uint32_t *const xch, const uint32_t *const lds_de)
{
    constexpr int L = (1 << (BM - 1)) - 1;
    constexpr int K = (1 << BV) - 1;
    constexpr int CM = 32 / BM, CV = 32 / BV;
    constexpr int VT = K + 1;
    constexpr int MT = MDE ? 2 * L + 2 : 2 * L + 1;
    constexpr uint32_t MIDX = ((1u << BM) - 1u) << 2, VIDX = ((1u << BV) - 1u) << 2;
    constexpr bool kDeTable = MDE && BM >= 3;

    const uint32_t tid = wave * 64u + lane;
    const uint64_t m_total = (a.n + CM - 1) / CM, v_total = (a.n + CV - 1) / CV;
    const uint64_t ew0 = blk * kBigBlock + (uint64_t)wave * kIter;    // first element of this wavefront
    const uint64_t e0 = ew0 + lane * 8u;                              // first element of this lane
    uint32_t *const img_m = slab + BigLayout::kOffImgM, *const img_v = slab + BigLayout::kOffImgV;
    float *const my_tv = reinterpret_cast<float *>(slab + BigLayout::kOffTv);
    float *const my_tm = reinterpret_cast<float *>(slab + BigLayout::kOffTm);
    const uint32_t tv_addr = lds_addr(my_tv), tm_addr = lds_addr(my_tm);

    // ---- loads: parameters and gradients, the wavefront's code words, the block's scalars
    RawPG raw = load_pg<BF16, TAIL>(a, ew0, lane);
    const float gscale = (EXT && a.grad_scale) ? *a.grad_scale : 1.0f;
    float4 *const stage = reinterpret_cast<float4 *>(work + wave * BigLayout::kStage);
    float4 *const st_c = stage + (lane + lane / 8u);
    float4 *const st_l = stage + (2u * lane + lane / 4u);
    // words of the wavefront's 512 elements: the first may start inside a word (ten-to-a-word codes)
    const uint64_t gm_lo = ew0 / CM, gv_lo = ew0 / CV;
    const uint32_t rm0 = (uint32_t)(ew0 - gm_lo * CM), rv0 = (uint32_t)(ew0 - gv_lo * CV);   // slot of the first element
    const uint32_t nwm = (rm0 + kIter + CM - 1) / CM, nwv = (rv0 + kIter + CV - 1) / CV;      // words touched (<= 64)
    const uint64_t gw_m = gm_lo + lane, gw_v = gv_lo + lane;
    const bool has_m = lane < nwm && (!TAIL || gw_m < m_total);
    const bool has_v = lane < nwv && (!TAIL || gw_v < v_total);
    uint32_t own_m = 0, own_v = 0;
    if (has_m) own_m = a.m_words[gw_m];
    if (has_v) own_v = a.v_words[gw_v];
    const float dm_old = a.m_scale[blk], dv_old = a.v_scale[blk], al_old = a.v_base[blk];
    if (BM == 3) own_m &= 0x3FFFFFFFu;
    if (BV == 3) own_v &= 0x3FFFFFFFu;
    img_m[lane] = own_m;
    img_v[lane] = own_v;
    if (lane == 0) { img_m[64] = 0; img_v[64] = 0; }

    // ---- level tables of the block (every wavefront its own copy)
    {
        const float s_m = (L == 1) ? dm_old : dm_old / (float)L;
        const float P1 = al_old, P2 = P1 * P1, P4 = P2 * P2, P8 = P4 * P4;
        if (lane < (uint32_t)VT) my_tv[lane] = log_level<BV>(lane, P1, P2, P4, P8) * dv_old;
        if (lane < (uint32_t)MT) my_tm[lane] = MDE ? DeLevels<BM>::level(lane) * dm_old : (float)((int)lane - L) * s_m;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    // word and slot of this lane's first code inside the wavefront's words
    const uint32_t qm = rm0 + lane * 8u, qv = rv0 + lane * 8u;
    const uint32_t wm = qm / CM, sm = qm - wm * CM, wv = qv / CV, sv = qv - wv * CV;
    const uint32_t mw0 = img_m[wm], mw1 = (BM == 3) ? img_m[wm + 1] : 0u;
    const uint32_t vw0 = img_v[wv], vw1 = (BV == 3) ? img_v[wv + 1] : 0u;
    const uint32_t mc8 = extract8<BM>(mw0, mw1, sm) & (uint32_t)((1ull << (8 * BM)) - 1ull);
    const uint32_t vc8 = extract8<BV>(vw0, vw1, sv) & (uint32_t)((1ull << (8 * BV)) - 1ull);

    bool ok[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) ok[j] = !TAIL || (e0 + j) < a.n;
    uint32_t nb = kBigBlock;                       // elements of the block that exist
    if (TAIL) nb = (uint32_t)(a.n - blk * kBigBlock);

    // ---- coalesced layout -> 8 consecutive elements per lane
    float p[8], g[8];
    {
        float4 pa = raw.p0, pb = raw.p1;
        uint4 ga = raw.g0, gb = raw.g1;
        if (!TAIL) {
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
    if (EXT) {
#pragma unroll
        for (int j = 0; j < 8; ++j) g[j] = __builtin_fmaf(a.l2, p[j], g[j] * gscale);
    }

    // ---- dequantize (table look-up), EMA, parameter
    float mh[8], vh[8];
    float m_absmax = 0.0f, v_max = 0.0f;
    const float kb = a.belief ? 1.0f : 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t om = (j == 0) ? (mc8 << 2) : (mc8 >> (BM * j - 2));
        const uint32_t ov = (j == 0) ? (vc8 << 2) : (vc8 >> (BV * j - 2));
        const float mt = lds_f32(tm_addr | (om & MIDX));
        const float vt = lds_f32(tv_addr | (ov & VIDX));
        mh[j] = __builtin_fmaf(a.beta1, mt, a.omb1 * g[j]);
        if (EXT) {
            const float d = __builtin_fmaf(-kb, mh[j], g[j]);
            vh[j] = __builtin_fmaf(a.beta2, vt, a.omb2 * (d * d)) + a.eps_state;
        } else {
            vh[j] = __builtin_fmaf(a.beta2, vt, a.omb2 * (g[j] * g[j]));
        }
        const float denom = __builtin_fmaf(__builtin_amdgcn_sqrtf(vh[j]), a.denom_scale, a.denom_eps);
        p[j] = __builtin_fmaf(p[j], a.decay, -(mh[j] * __builtin_amdgcn_rcpf(denom)));
        if (TAIL && !ok[j]) { mh[j] = 0.0f; vh[j] = 0.0f; }
        m_absmax = __builtin_fmaxf(m_absmax, __builtin_fabsf(mh[j]));
        v_max = __builtin_fmaxf(v_max, vh[j]);
    }
    if (EXT && a.param_bf16) {
        if (!TAIL) {
            const u32x4_t h = {pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7])};
            stream_store_u4(a.param_bf16 + e0, h);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (ok[j]) a.param_bf16[e0 + j] = (uint16_t)pack_bf16(p[j], 0.0f);
        }
    }
    if (!TAIL) {
        wave_lds_sync();
        st_l[0] = make_float4(p[0], p[1], p[2], p[3]);
        st_l[1] = make_float4(p[4], p[5], p[6], p[7]);
        wave_lds_sync();
        float *pp = a.param + ew0 + lane * 4u;
        stream_store_f4(pp, st_c[0]);
        stream_store_f4(pp + 256, st_c[72]);
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) if (ok[j]) a.param[e0 + j] = p[j];
    }

    // ---- the work area becomes the histograms of the selection: a wavefront clears its own staging
    // area (it is done with it; the others may still be using theirs) and its share of the rest
    {
        uint4 *const own = reinterpret_cast<uint4 *>(work + wave * BigLayout::kStage);
        wave_lds_sync();
#pragma unroll
        for (int i = 0; i < BigLayout::kStage / 4 / 64; ++i) own[lane + 64u * (uint32_t)i] = make_uint4(0, 0, 0, 0);
        constexpr int kRest = (BigLayout::kWork - kBigWaves * BigLayout::kStage) / 4;    // 128-bit words behind the staging areas
        uint4 *const rest = reinterpret_cast<uint4 *>(work + kBigWaves * BigLayout::kStage);
        for (uint32_t i = tid; i < (uint32_t)kRest; i += kBigWaves * 64) rest[i] = make_uint4(0, 0, 0, 0);
    }

    // ---- block maxima over the four wavefronts
    {
        const uint32_t wm_max = wave_max(f2u(m_absmax)), wv_max = wave_max(f2u(v_max));
        if (lane == 0) { xch[wave] = wm_max; xch[4 + wave] = wv_max; }
    }
    __syncthreads();
    float dm = u2f(umax(umax(xch[0], xch[1]), umax(xch[2], xch[3])));
    float dv = u2f(umax(umax(xch[4], xch[5]), umax(xch[6], xch[7])));
    if (dm < kTiny) dm = 0.0f;
    if (dv < kTiny) dv = 0.0f;

    // ---- the r-th smallest v^ of the block
    uint32_t rank = a.rank_full;
    if (TAIL) {
        const float x = __builtin_ceilf(a.quantile_p * (float)nb);
        rank = x < 1.0f ? 1u : (uint32_t)x;
        rank = rank > nb ? nb : rank;
    }
    uint32_t key[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) key[j] = (TAIL && !ok[j]) ? kInfBits : f2u(vh[j]);
    const uint32_t xp_bits = select_rank(key, rank, lane, work);

    // ---- encoder constants (every 16 lanes for themselves), codes, the wavefront's words
    const uint32_t lig = lane & 15u, gshift = lane & 16u;
    uint32_t de_base = 0;
    if (kDeTable) de_base = lds_addr(lds_de) - 16u * DeBuckets<BM>::kLo;
    const BlockCodec codec = block_codec<BV, 16, L, MDE>(xp_bits, dm, dv, lane, lig, gshift);
    uint32_t m8, v8;
    encode_run<BM, BV, MDE, TAIL>(a, e0, mh, vh, ok, codec, de_base, m8, v8);
    const uint32_t xm = mc8 ^ m8, xv = vc8 ^ v8;
    const uint32_t xm0 = (BM == 3) ? (xm << (3u * sm)) & 0x3FFFFFFFu : xm << (BM * sm);
    const uint32_t xm1 = (BM == 3) ? (uint32_t)(((uint64_t)xm << (3u * sm)) >> 30) : 0u;
    const uint32_t xv0 = (BV == 3) ? (xv << (3u * sv)) & 0x3FFFFFFFu : xv << (BV * sv);
    const uint32_t xv1 = (BV == 3) ? (uint32_t)(((uint64_t)xv << (3u * sv)) >> 30) : 0u;
    atomicXor(&img_m[wm], xm0);
    if (BM == 3) atomicXor(&img_m[wm + 1], xm1);
    atomicXor(&img_v[wv], xv0);
    if (BV == 3) atomicXor(&img_v[wv + 1], xv1);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (has_m) {
        const uint32_t fin = img_m[lane];
        if (BM != 3) a.m_words[gw_m] = fin;
        else if (fin != own_m) atomicXor(&a.m_words[gw_m], fin ^ own_m);
    }
    if (has_v) {
        const uint32_t fin = img_v[lane];
        if (BV != 3) a.v_words[gw_v] = fin;
        else if (fin != own_v) atomicXor(&a.v_words[gw_v], fin ^ own_v);
    }
    if (tid == 0) { a.m_scale[blk] = dm; a.v_scale[blk] = dv; a.v_base[blk] = codec.alpha; }
}

// One workgroup per block of 2048 elements.
template <int BM, int BV, bool BF16, bool MDE, bool EXT>
__global__ __launch_bounds__(kBigWaves * 64, SOLO_MIN_WAVES)
void big_kernel(const StepArgs a)
{
    constexpr int kDeWords = (MDE && BM >= 3) ? 4 * DeBuckets<BM>::N : 16;
    __shared__ __attribute__((aligned(64))) uint32_t lds_work[BigLayout::kWork];
    __shared__ __attribute__((aligned(64))) uint32_t lds_slab[kBigWaves * BigLayout::kSlab];
    __shared__ __attribute__((aligned(64))) uint32_t lds_xch[8];
    __shared__ __attribute__((aligned(64))) uint32_t lds_de[kDeWords];
    load_de_table<BM, MDE, kDeWords>(lds_de);
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint64_t blk = blockIdx.x;
    uint32_t *const slab = lds_slab + wave * BigLayout::kSlab;
    if ((blk + 1) * kBigBlock <= a.n)
        step_block_big<BM, BV, BF16, MDE, false, EXT>(a, blk, lane, wave, slab, lds_work, lds_xch, lds_de);
    else
        step_block_big<BM, BV, BF16, MDE, true, EXT>(a, blk, lane, wave, slab, lds_work, lds_xch, lds_de);
}

template <int BM, bool MDE>
hipError_t launch_big(uint32_t bits_v, bool bf16, const StepArgs &args, hipStream_t stream);

template <int BM, bool MDE>
hipError_t launch_big_impl(uint32_t bits_v, bool bf16, const StepArgs &args, hipStream_t stream)
{
    const uint64_t grid = (args.n + kBigBlock - 1) / kBigBlock;
    if (grid == 0 || grid > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const bool ext = args.param_bf16 || args.grad_scale || args.belief || args.l2 != 0.0f;
#define SOLO_LAUNCH(BV_, BF_, EXT_)                                                                 \
    hipLaunchKernelGGL((big_kernel<BM, BV_, BF_, MDE, EXT_>), dim3((uint32_t)grid), dim3(kBigWaves * 64), 0, stream, args)
#define SOLO_CASE(BV_)                                                                              \
    if (bits_v == BV_) {                                                                            \
        if (bf16) { if (ext) SOLO_LAUNCH(BV_, true, true); else SOLO_LAUNCH(BV_, true, false); }    \
        else      { if (ext) SOLO_LAUNCH(BV_, false, true); else SOLO_LAUNCH(BV_, false, false); }  \
        return hipGetLastError();                                                                   \
    }
    SOLO_CASE(2) SOLO_CASE(3) SOLO_CASE(4)
#undef SOLO_CASE
#undef SOLO_LAUNCH
    return hipErrorInvalidValue;
}

}  // namespace solo
