// The fused SOLO AdamW step for blocks of 2048 elements (the large-block setting of the paper's
// block-size comparison, Sec. 4.2), gfx950, wave64.
//
// A block of 2048 elements is held by one workgroup.  Two forms:
//   * a full block: two wavefronts, 1024 elements each, sixteen consecutive elements per lane
//     (step_block_wide, big_wide_kernel);
//   * the shorter last block of a buffer: four wavefronts, 512 elements each, eight per lane,
//     bounds checks on every element (step_block_big, big_kernel; a launch of its own).
// The element-wise part (decode by table look-up, both EMAs, the parameter, the encoders, the
// 32-bit words of the code streams) is that of an iteration of solo_step.h, one iteration per
// wavefront, and runs without any exchange between the wavefronts.  What a block of this size
// changes is the block statistics:
//   * Delta_m' and Delta_v' are maxima over the wavefronts: DPP inside a row, four lane reads
//     across the rows, a few words of LDS and one barrier across the wavefronts;
//   * the p-quantile is the rank-205 element of 2048 values (p = 0.1), far too deep for rounds
//     of "extract the minimum".  It is found by a radix select on the bit patterns (non-negative
//     floats order like their bits): four passes over 8 + 8 + 8 + 7 bits, each a histogram of the
//     keys that still match the selected prefix (LDS atomics), one barrier, a prefix sum (DPP
//     scan) by which one wavefront finds the bin that holds the rank, and a second barrier.
//     After the last pass the prefix is the order statistic itself, multiplicities included,
//     exactly.  Nine barriers per block in all.
//   * the base alpha, the divisions and the level tables are computed by every wavefront (every
//     16 lanes) for itself: cheaper than another barrier.
// LDS sets the number of workgroups on a CU, and that the speed (measured on MI355X: 17.3 ms for
// 6.7e9 parameters at 3.5 wavefronts per SIMD, 15.7 ms at 5), so the histograms are kept small:
// see BigLayout.  Every wavefront stages and writes back the words of its own elements (whole
// 128-byte lines for 2- and 4-bit codes; ten-to-a-word codes by one atomic XOR per word at the
// memory side, since a wavefront's share does not end on a word).
#pragma once
#include "solo_step.h"

namespace solo {

constexpr int kBigBlock = 2048;
constexpr int kBigWaves = kBigBlock / kIter;      // 4 wavefronts, one workgroup per block
static_assert(kBigWaves == 4, "one workgroup of four wavefronts per block");

// LDS of a workgroup (32-bit words).  `work` first serves the wavefronts as the staging areas of
// their layout transpositions, then, behind the barrier of the block maxima, the whole workgroup as
// the histograms of the selection (four passes over 8 + 8 + 8 + 7 bits).
// The second moments of a block that has been trained for a while sit in a few tight clusters, one
// per level of the previous code, so most of the 64 lanes of an instruction add to the same one or
// two bins, and LDS applies the adds to one bank one after the other (measured on MI355X with one
// counter per bin: the step slowed down by half between the first and the thousandth update of a
// state, all of it LDS bank conflicts).  Every bin therefore has 8 (4) counters in neighbouring
// words, i.e. in different banks, and a lane always uses the one its number selects.
//   hist A: 256 bins x 8 counters; the lower halves of its words count the first pass, the upper
//           halves the second (a count is at most 2048, so the halves do not carry into each
//           other, and a wavefront that is still reading the lower halves is not disturbed by one
//           that already counts the next pass in the upper ones);
//   hist B: 256 bins x 4 counters; lower halves: third pass, upper halves: fourth (128 bins).
// Four pad words follow every 64 words: the rows that the 64 lanes sum with 128-bit reads (32 or
// 16 words each) then start in 16 different groups of four banks.
struct BigLayout {
    static constexpr int kStage = 64 * kColStride;            // per wavefront
    static constexpr int kHistA = 0, kHistB = 2048 + 2048 / 64 * 4;
    static constexpr int kHists = kHistB + 1024 + 1024 / 64 * 4;                // 3264 words
    static constexpr int kWork = kHists > 4 * kStage ? kHists : 4 * kStage;
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

// The rank-th smallest (1-based, uniform over the workgroup) of the NK keys that each thread of
// the workgroup holds (2048 in all): bit patterns of non-negative floats, +inf for absent elements
// (the rank never reaches those).  Radix select over 8 + 8 + 8 + 7 bits.  A pass: every thread
// adds its keys that still match the selected prefix to its counters of the pass's histogram (in
// `work`, zeroed before the workgroup's first barrier), one barrier, and then one wavefront finds
// the bin of the rank: a lane sums the counters of its four (two) consecutive bins, a prefix sum
// over the wavefront names the lane whose bins hold the rank, and that lane's bin sums name the
// bin; `res` (8 words of LDS) hands bin and rank to the other wavefronts behind a second barrier.
template <int NK>
__device__ __forceinline__ uint32_t select_rank(const uint32_t (&key)[NK], uint32_t rank, uint32_t lane, uint32_t wave,
                                                uint32_t *work, uint32_t *res)
{
    uint32_t prefix = 0;
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        constexpr int kBits[4] = {8, 8, 8, 7}, kShift[4] = {23, 15, 7, 0};      // (bit 31 of a key is 0)
        const int bits = kBits[pass], sh = kShift[pass];
        const int lr = pass < 2 ? 3 : 2;                                        // log2(counters per bin)
        const uint32_t R = 1u << lr;
        uint32_t *const h = work + (pass < 2 ? BigLayout::kHistA : BigLayout::kHistB);
        const uint32_t one = (pass & 1) ? 0x10000u : 1u;
        const uint32_t mine = lane & (R - 1u);
#pragma unroll
        for (int j = 0; j < NK; ++j) {
            const bool match = pass == 0 || (key[j] >> (sh + bits)) == prefix;
            const uint32_t w = ((((key[j] >> sh) & ((1u << bits) - 1u))) << lr) | mine;
            if (match) atomicAdd(&h[w + ((w >> 6) << 2)], one);
        }
        __syncthreads();
        // One wavefront finds the bin (wavefronts 0 and 1 take turns) and leaves it and the rank
        // inside it in LDS for the others: a second barrier costs less than every wavefront
        // summing the whole histogram for itself.
        if (wave == (uint32_t)(pass & 1)) {
            // this lane's bins: 4 of 256 (2 of 128), `per` words from word per * lane, behind the pads in front of it
            const uint32_t nb = (1u << bits) / 64u;                                 // bins per lane
            const uint32_t per = nb * R;                                            // words per lane: 32, 32, 16, 8
            const uint32_t row = per * lane + (((per * lane) >> 6) << 2);
            uint32_t c[4] = {0, 0, 0, 0};
#pragma unroll
            for (uint32_t k = 0; k < nb; ++k) {
#pragma unroll
                for (uint32_t i = 0; i < R / 4u; ++i) {
                    const uint4 c4 = *reinterpret_cast<const uint4 *>(h + row + k * R + 4u * i);
                    c[k] += (c4.x + c4.y) + (c4.z + c4.w);
                }
                c[k] = (pass & 1) ? c[k] >> 16 : c[k] & 0xFFFFu;
            }
            const uint32_t s = (c[0] + c[1]) + (c[2] + c[3]);
            const uint32_t incl = wave_inclusive_sum(s);
            const uint64_t holder = __builtin_amdgcn_ballot_w64(incl - s < rank && rank <= incl);   // one lane
            const uint32_t sel = (uint32_t)__builtin_ctzll(holder | (1ull << 63));
            rank -= (uint32_t)__builtin_amdgcn_readlane((int)(incl - s), (int)sel);
            uint32_t sel2 = 0;
#pragma unroll
            for (uint32_t k = 0; k + 1 < nb; ++k) {
                const uint32_t e = (uint32_t)__builtin_amdgcn_readlane((int)c[k], (int)sel);
                if (sel2 == k && rank > e) { rank -= e; sel2 = k + 1; }
            }
            if (lane == 0) { res[2 * pass] = sel * nb + sel2; res[2 * pass + 1] = rank; }
        }
        __syncthreads();
        prefix = (prefix << bits) | res[2 * pass];
        rank = res[2 * pass + 1];
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
    constexpr int CM = 32 / BM, CV = 32 / BV;
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
        const float de_level = MDE ? DeLevels<BM>::level(lane) : 0.0f;
        fill_level_tables<BM, BV, MDE, 64>(my_tv, my_tm, lane, dm_old, dv_old, al_old, &de_level);
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
    lane_layout8<BF16, TAIL>(raw, st_c, st_l, p, g);
    if (EXT) {
#pragma unroll
        for (int j = 0; j < 8; ++j) g[j] = __builtin_fmaf(a.l2, p[j], g[j] * gscale);
    }

    // ---- dequantize (table look-up), EMA, parameter; new parameters streamed out
    float mh[8], vh[8];
    float m_absmax, v_max;
    ema_param<8, BM, BV, EXT, TAIL, true>(a, tm_addr, tv_addr, &mc8, &vc8, ok, p, g, mh, vh, m_absmax, v_max);
    store_params8<EXT, TAIL>(a, ew0, e0, lane, ok, p, st_c, st_l);

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
    const uint32_t xp_bits = select_rank<8>(key, rank, lane, wave, work, xch + 8);

    // ---- encoder constants (every 16 lanes for themselves), codes, the wavefront's words
    const uint32_t lig = lane & 15u, gshift = lane & 16u;
    uint32_t de_base = 0;
    if (kDeTable) de_base = lds_addr(lds_de) - 16u * DeBuckets<BM>::kLo;
    const BlockCodec codec = block_codec<BV, 16, L, MDE>(xp_bits, dm, dv, lane, lig, gshift);
    uint32_t m8, v8;
    encode_run<BM, BV, MDE, TAIL>(a, e0, mh, vh, ok, codec, de_base, m8, v8);
    xor_into_image8<BM, BV>(img_m, img_v, wm, sm, wv, sv, mc8 ^ m8, vc8 ^ v8);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (has_m) write_back_word<BM>(&a.m_words[gw_m], img_m[lane], own_m);
    if (has_v) write_back_word<BV>(&a.v_words[gw_v], img_v[lane], own_v);
    if (tid == 0) { a.m_scale[blk] = dm; a.v_scale[blk] = dv; a.v_base[blk] = codec.alpha; }
}

// ---- the wide form of a full block: two wavefronts, 16 consecutive elements per lane
//
// The element-wise part is that of one 1024-element iteration of the wide streaming path
// (step_tile16), the block statistics are those of step_block_big() with two wavefronts instead of
// four.  What is done once per lane and block (level tables, the two divisions, the base, the
// hash of a group of eight, the scans of the selection) is spread over twice as many elements, and
// the scans are run by two wavefronts instead of four.
constexpr int kWideBigWaves = kBigBlock / kIter16;
static_assert(kWideBigWaves == 2, "one workgroup of two wavefronts per block");

#ifndef SOLO_BIG_WIDE
#define SOLO_BIG_WIDE 1            // (tuning builds: 0 runs full blocks on four wavefronts, too)
#endif

struct WideBigLayout {
    static constexpr int kStage = 64 * kColStride16;          // per wavefront: staging of the layout transpositions
    static constexpr int kOffImgM = 0;                        // per wavefront: its words of each code stream (<= 128, + 4)
    static constexpr int kOffImgV = 132;
    static constexpr int kOffTv = 272;                        // level tables, 64-byte aligned
    static constexpr int kOffTm = 288;
    static constexpr int kSlab = 304;
};
static_assert(BigLayout::kWork >= kWideBigWaves * WideBigLayout::kStage, "the staging areas lie inside the work area");
static_assert(288 * 4 <= WideBigLayout::kStage, "the padded transposition (Stage16) fits a staging area");

template <int BM, int BV, bool BF16, bool MDE, bool EXT>
__device__ __forceinline__ void step_block_wide(const StepArgs &a, const uint64_t blk, const uint32_t lane,
                                                const uint32_t wave, uint32_t *const slab, uint32_t *const work,
                                                uint32_t *const xch, const uint32_t *const lds_de)
{
    constexpr int L = (1 << (BM - 1)) - 1;
    constexpr int CM = 32 / BM, CV = 32 / BV;
    constexpr bool kDeTable = MDE && BM >= 3;
    constexpr int KM = CM == 16 ? 1 : 2, KV = CV == 16 ? 1 : 2;      // words of a stream per lane (64 x K >= words of 1024 elements)

    const uint32_t tid = wave * 64u + lane;
    const uint64_t ew0 = blk * kBigBlock + (uint64_t)wave * kIter16;  // first element of this wavefront
    const uint64_t e0 = ew0 + lane * 16u;                             // first element of this lane
    uint32_t *const img_m = slab + WideBigLayout::kOffImgM, *const img_v = slab + WideBigLayout::kOffImgV;
    float *const my_tv = reinterpret_cast<float *>(slab + WideBigLayout::kOffTv);
    float *const my_tm = reinterpret_cast<float *>(slab + WideBigLayout::kOffTm);
    const uint32_t tv_addr = lds_addr(my_tv), tm_addr = lds_addr(my_tm);

    // ---- loads: parameters and gradients, the wavefront's code words, the block's scalars
    RawPG16<BF16> raw = load_pg16<BF16>(a, ew0, lane);
    const float gscale = (EXT && a.grad_scale) ? *a.grad_scale : 1.0f;
    const Stage16 st(reinterpret_cast<float4 *>(work + wave * WideBigLayout::kStage), lane);
    // words of the wavefront's 1024 elements: the first may start inside a word (ten-to-a-word
    // codes); all of them exist, the block is a full one
    const uint64_t gm_lo = ew0 / CM, gv_lo = ew0 / CV;
    const uint32_t rm0 = (uint32_t)(ew0 - gm_lo * CM), rv0 = (uint32_t)(ew0 - gv_lo * CV);   // slot of the first element
    const uint32_t nwm = (rm0 + kIter16 + CM - 1) / CM, nwv = (rv0 + kIter16 + CV - 1) / CV;  // words touched (<= 128)
    uint32_t own_m[KM], own_v[KV];
#pragma unroll
    for (int k = 0; k < KM; ++k) {
        own_m[k] = 0;
        if (lane + 64u * k < nwm) own_m[k] = a.m_words[gm_lo + lane + 64u * k];
    }
#pragma unroll
    for (int k = 0; k < KV; ++k) {
        own_v[k] = 0;
        if (lane + 64u * k < nwv) own_v[k] = a.v_words[gv_lo + lane + 64u * k];
    }
    const float dm_old = a.m_scale[blk], dv_old = a.v_scale[blk], al_old = a.v_base[blk];
#pragma unroll
    for (int k = 0; k < KM; ++k) {
        if (BM == 3) own_m[k] &= 0x3FFFFFFFu;
        img_m[lane + 64u * k] = own_m[k];
    }
#pragma unroll
    for (int k = 0; k < KV; ++k) {
        if (BV == 3) own_v[k] &= 0x3FFFFFFFu;
        img_v[lane + 64u * k] = own_v[k];
    }
    if (lane < 4) { img_m[64 * KM + lane] = 0; img_v[64 * KV + lane] = 0; }

    // ---- level tables of the block (every wavefront its own copy)
    {
        const float de_level = MDE ? DeLevels<BM>::level(lane) : 0.0f;
        fill_level_tables<BM, BV, MDE, 64>(my_tv, my_tm, lane, dm_old, dv_old, al_old, &de_level);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    // word and slot of the first code of the lane's two runs of 8 inside the wavefront's words
    uint32_t wm[2], sm[2], wv[2], sv[2];
    uint32_t mc8[2], vc8[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const uint32_t qm = rm0 + lane * 16u + 8u * r, qv = rv0 + lane * 16u + 8u * r;   // < 1040: e / 10 by multiplication
        wm[r] = (CM == 10) ? __umul24(qm, 52429u) >> 19 : qm / CM; sm[r] = qm - wm[r] * CM;
        wv[r] = (CV == 10) ? __umul24(qv, 52429u) >> 19 : qv / CV; sv[r] = qv - wv[r] * CV;
    }
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        // (2-bit codes: both runs of the lane lie in one word)
        const uint32_t mw0 = img_m[wm[BM == 2 ? 0 : r]], mw1 = (BM == 3) ? img_m[wm[r] + 1] : 0u;
        const uint32_t vw0 = img_v[wv[BV == 2 ? 0 : r]], vw1 = (BV == 3) ? img_v[wv[r] + 1] : 0u;
        mc8[r] = extract8<BM>(mw0, mw1, BM == 2 ? 8u * r : sm[r]) & (uint32_t)((1ull << (8 * BM)) - 1ull);
        vc8[r] = extract8<BV>(vw0, vw1, BV == 2 ? 8u * r : sv[r]) & (uint32_t)((1ull << (8 * BV)) - 1ull);
    }

    // ---- coalesced layout -> 16 consecutive elements per lane
    float p[16], g[16];
    lane_layout16<BF16>(raw, st, p, g);
    if (EXT) {
#pragma unroll
        for (int j = 0; j < 16; ++j) g[j] = __builtin_fmaf(a.l2, p[j], g[j] * gscale);
    }

    // ---- dequantize (table look-up), EMA, parameter; new parameters streamed out
    float mh[16], vh[16];
    float m_absmax, v_max;
    ema_param<16, BM, BV, EXT, false, true>(a, tm_addr, tv_addr, mc8, vc8, nullptr, p, g, mh, vh, m_absmax, v_max);
    store_params16<EXT>(a, ew0, lane, p, st);

    // ---- the work area becomes the histograms of the selection: a wavefront clears its own staging
    // area (it is done with it; the other may still be using its own) and its share of the rest
    {
        uint4 *const own = reinterpret_cast<uint4 *>(work + wave * WideBigLayout::kStage);
        wave_lds_sync();
        constexpr int kOwn = WideBigLayout::kStage / 4;                                     // 128-bit words
#pragma unroll
        for (int i = 0; i < (kOwn + 63) / 64; ++i)
            if (lane + 64u * (uint32_t)i < (uint32_t)kOwn) own[lane + 64u * (uint32_t)i] = make_uint4(0, 0, 0, 0);
        constexpr int kRest = (BigLayout::kWork - kWideBigWaves * WideBigLayout::kStage) / 4;
        uint4 *const rest = reinterpret_cast<uint4 *>(work + kWideBigWaves * WideBigLayout::kStage);
        for (uint32_t i = tid; i < (uint32_t)kRest; i += kWideBigWaves * 64) rest[i] = make_uint4(0, 0, 0, 0);
    }

    // ---- block maxima over the two wavefronts
    {
        const uint32_t wm_max = wave_max(f2u(m_absmax)), wv_max = wave_max(f2u(v_max));
        if (lane == 0) { xch[wave] = wm_max; xch[2 + wave] = wv_max; }
    }
    __syncthreads();
    float dm = u2f(umax(xch[0], xch[1]));
    float dv = u2f(umax(xch[2], xch[3]));
    if (dm < kTiny) dm = 0.0f;
    if (dv < kTiny) dv = 0.0f;

    // ---- the r-th smallest v^ of the block
    uint32_t key[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) key[j] = f2u(vh[j]);
    const uint32_t xp_bits = select_rank<16>(key, a.rank_full, lane, wave, work, xch + 8);

    // ---- encoder constants (every 16 lanes for themselves), codes, the wavefront's words
    const uint32_t lig = lane & 15u, gshift = lane & 16u;
    uint32_t de_base = 0;
    if (kDeTable) de_base = lds_addr(lds_de) - 16u * DeBuckets<BM>::kLo;
    const BlockCodec codec = block_codec<BV, 16, L, MDE>(xp_bits, dm, dv, lane, lig, gshift);
    encode_into_image16<BM, BV, MDE>(a, e0, mh, vh, codec, de_base, img_m, img_v, wm, sm, wv, sv, mc8, vc8);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int k = 0; k < KM; ++k)
        if (lane + 64u * k < nwm) write_back_word<BM>(&a.m_words[gm_lo + lane + 64u * k], img_m[lane + 64u * k], own_m[k]);
#pragma unroll
    for (int k = 0; k < KV; ++k)
        if (lane + 64u * k < nwv) write_back_word<BV>(&a.v_words[gv_lo + lane + 64u * k], img_v[lane + 64u * k], own_v[k]);
    if (tid == 0) { a.m_scale[blk] = dm; a.v_scale[blk] = dv; a.v_base[blk] = codec.alpha; }
}

// One workgroup of two wavefronts per full block of 2048 elements.
// (Registers: the plain step with bf16 gradients fits five wavefronts per SIMD without spilling,
// except with two ten-to-a-word streams; LDS allows five for every format.)
template <int BM, int BV, bool BF16, bool EXT>
constexpr int big_wide_waves() { return (BF16 && !EXT && !(BM == 3 && BV == 3)) ? kWideWaves + 1 : kWideWaves; }

template <int BM, int BV, bool BF16, bool MDE, bool EXT>
__global__ __launch_bounds__(kWideBigWaves * 64, (big_wide_waves<BM, BV, BF16, EXT>()))
void big_wide_kernel(const StepArgs a)
{
    constexpr int kDeWords = (MDE && BM >= 3) ? 4 * DeBuckets<BM>::N : 16;
    __shared__ __attribute__((aligned(64))) uint32_t lds_work[BigLayout::kWork];
    __shared__ __attribute__((aligned(64))) uint32_t lds_slab[kWideBigWaves * WideBigLayout::kSlab];
    __shared__ __attribute__((aligned(64))) uint32_t lds_xch[16];   // block maxima; bin and rank of every pass
    __shared__ __attribute__((aligned(64))) uint32_t lds_de[kDeWords];
    load_de_table<BM, MDE, kDeWords>(lds_de);
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    step_block_wide<BM, BV, BF16, MDE, EXT>(a, blockIdx.x, lane, wave, lds_slab + wave * WideBigLayout::kSlab,
                                            lds_work, lds_xch, lds_de);
}

// One workgroup of four wavefronts per block of 2048 elements, from block a.tail_tile0 on.
template <int BM, int BV, bool BF16, bool MDE, bool EXT>
__global__ __launch_bounds__(kBigWaves * 64, SOLO_MIN_WAVES)
void big_kernel(const StepArgs a)
{
    constexpr int kDeWords = (MDE && BM >= 3) ? 4 * DeBuckets<BM>::N : 16;
    __shared__ __attribute__((aligned(64))) uint32_t lds_work[BigLayout::kWork];
    __shared__ __attribute__((aligned(64))) uint32_t lds_slab[kBigWaves * BigLayout::kSlab];
    __shared__ __attribute__((aligned(64))) uint32_t lds_xch[16];   // block maxima; bin and rank of every pass
    __shared__ __attribute__((aligned(64))) uint32_t lds_de[kDeWords];
    load_de_table<BM, MDE, kDeWords>(lds_de);
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint64_t blk = a.tail_tile0 + blockIdx.x;
    uint32_t *const slab = lds_slab + wave * BigLayout::kSlab;
    if constexpr (!SOLO_BIG_WIDE) {
        if ((blk + 1) * kBigBlock <= a.n) {
            step_block_big<BM, BV, BF16, MDE, false, EXT>(a, blk, lane, wave, slab, lds_work, lds_xch, lds_de);
            return;
        }
    }
    step_block_big<BM, BV, BF16, MDE, true, EXT>(a, blk, lane, wave, slab, lds_work, lds_xch, lds_de);
}

// The step over many tensors in one launch, blocks of 2048 elements.  The map of the table holds
// one entry per block of every tensor (the tensor's index; a shorter last block is flagged).  A
// workgroup of multi_big_wide_kernel takes one entry and, unless it is flagged, runs the full
// block; workgroup k of multi_big_tail_kernel runs the shorter last block of tensor k, if it has
// one.  Blocks never span tensors.
__device__ __forceinline__ StepArgs tensor_args(const MultiArgs &ma, const TensorEntry &e)
{
    StepArgs a = ma.common;
    a.param = e.param; a.param_bf16 = e.param_bf16; a.grad = e.grad;
    a.m_words = e.m_words; a.m_scale = e.m_scale;
    a.v_words = e.v_words; a.v_scale = e.v_scale; a.v_base = e.v_base;
    a.n = e.n; a.index_offset = e.index_offset;
    return a;
}

template <int BM, int BV, bool BF16, bool MDE, bool EXT>
__global__ __launch_bounds__(kWideBigWaves * 64, (big_wide_waves<BM, BV, BF16, EXT>()))
void multi_big_wide_kernel(const MultiArgs ma)
{
    constexpr int kDeWords = (MDE && BM >= 3) ? 4 * DeBuckets<BM>::N : 16;
    __shared__ __attribute__((aligned(64))) uint32_t lds_work[BigLayout::kWork];
    __shared__ __attribute__((aligned(64))) uint32_t lds_slab[kWideBigWaves * WideBigLayout::kSlab];
    __shared__ __attribute__((aligned(64))) uint32_t lds_xch[16];
    __shared__ __attribute__((aligned(64))) uint32_t lds_de[kDeWords];
    const uint64_t unit = blockIdx.x;
    if (unit >= ma.total_units) return;
    const uint32_t me = ma.unit_map[unit];                      // uniform: scalar loads
    if (me & kMapRagged) return;                                // (the whole workgroup: no barrier has been reached)
    load_de_table<BM, MDE, kDeWords>(lds_de);
    const TensorEntry &e = ma.entries[me & kMapTensorMask];
    const StepArgs a = tensor_args(ma, e);
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    step_block_wide<BM, BV, BF16, MDE, EXT>(a, unit - e.unit0, lane, wave, lds_slab + wave * WideBigLayout::kSlab,
                                            lds_work, lds_xch, lds_de);
}

template <int BM, int BV, bool BF16, bool MDE>
__global__ __launch_bounds__(kBigWaves * 64, SOLO_MIN_WAVES)
void multi_big_tail_kernel(const MultiArgs ma, const uint32_t count)
{
    constexpr int kDeWords = (MDE && BM >= 3) ? 4 * DeBuckets<BM>::N : 16;
    __shared__ __attribute__((aligned(64))) uint32_t lds_work[BigLayout::kWork];
    __shared__ __attribute__((aligned(64))) uint32_t lds_slab[kBigWaves * BigLayout::kSlab];
    __shared__ __attribute__((aligned(64))) uint32_t lds_xch[16];
    __shared__ __attribute__((aligned(64))) uint32_t lds_de[kDeWords];
    if (blockIdx.x >= count) return;
    const TensorEntry &e = ma.entries[blockIdx.x];
    if (e.n % kBigBlock == 0) return;                           // (the whole workgroup)
    load_de_table<BM, MDE, kDeWords>(lds_de);
    const StepArgs a = tensor_args(ma, e);
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    step_block_big<BM, BV, BF16, MDE, true, true>(a, e.n / kBigBlock, lane, wave, lds_slab + wave * BigLayout::kSlab,
                                                  lds_work, lds_xch, lds_de);
}

template <int BM, bool MDE>
hipError_t launch_multi_big(uint32_t bits_v, bool bf16, const MultiArgs &args, uint32_t count, bool ragged,
                            hipStream_t stream);

template <int BM, bool MDE>
hipError_t launch_multi_big_impl(uint32_t bits_v, bool bf16, const MultiArgs &args, uint32_t count, bool ragged,
                                 hipStream_t stream)
{
    if (args.total_units == 0 || args.total_units > 0x7FFFFFFFull || count == 0) return hipErrorInvalidValue;
    const StepArgs &c = args.common;
    const bool ext = args.any_bf16_copy || c.grad_scale || c.belief || c.l2 != 0.0f;
#define SOLO_LAUNCH(BV_, BF_, EXT_)                                                                 \
    do {                                                                                            \
        hipLaunchKernelGGL((multi_big_wide_kernel<BM, BV_, BF_, MDE, EXT_>), dim3((uint32_t)args.total_units), \
                           dim3(kWideBigWaves * 64), 0, stream, args);                              \
        if (ragged)                                                                                 \
            hipLaunchKernelGGL((multi_big_tail_kernel<BM, BV_, BF_, MDE>), dim3(count),             \
                               dim3(kBigWaves * 64), 0, stream, args, count);                       \
    } while (0)
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

template <int BM, bool MDE>
hipError_t launch_big(uint32_t bits_v, bool bf16, const StepArgs &args, hipStream_t stream);

// Full blocks run on two wavefronts each; a shorter last block is a launch of its own, one
// workgroup of four wavefronts with bounds checks on every element.
template <int BM, bool MDE>
hipError_t launch_big_impl(uint32_t bits_v, bool bf16, const StepArgs &args, hipStream_t stream)
{
    const uint64_t full = args.n / kBigBlock, blocks = (args.n + kBigBlock - 1) / kBigBlock;
    if (blocks == 0 || blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const bool ext = args.param_bf16 || args.grad_scale || args.belief || args.l2 != 0.0f;
    const uint64_t wide_blocks = SOLO_BIG_WIDE ? full : 0;
    StepArgs rest = args;
    rest.tail_tile0 = wide_blocks;               // the four-wavefront kernel starts behind them
#define SOLO_LAUNCH(BV_, BF_, EXT_)                                                                 \
    do {                                                                                            \
        if (wide_blocks)                                                                            \
            hipLaunchKernelGGL((big_wide_kernel<BM, BV_, BF_, MDE, EXT_>), dim3((uint32_t)wide_blocks),    \
                               dim3(kWideBigWaves * 64), 0, stream, args);                          \
        if (blocks > wide_blocks)                                                                   \
            hipLaunchKernelGGL((big_kernel<BM, BV_, BF_, MDE, EXT_>), dim3((uint32_t)(blocks - wide_blocks)), \
                               dim3(kBigWaves * 64), 0, stream, rest);                              \
    } while (0)
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
