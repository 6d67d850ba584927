/*
 * CPU oracle for the SOLO low-bit AdamW step ("Pushing the Limits of Low-Bit
 * Optimizers: A Focus on EMA Dynamics").
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, scalar restatement
 * of the method, written from the paper, and exists only so that the tests,
 * the smoke check and the benchmark's cpu_baseline leg have something
 * independent to compare the GPU library against.  It shares no code, header,
 * table or helper with the GPU library and the library never calls it.
 *
 * What one step does for every block of `block_size` consecutive elements
 * (block-wise quantization, Sec. 3.4):
 *
 *   1. dequantize   m~ = y_q * Delta_m          (Sec. 3.1, dequantizer Q-dagger)
 *                   v~ = alpha^q * Delta_v      (Sec. 3.2.2, levels y_k = alpha^k)
 *   2. EMA update   m^ = beta1 m~ + (1-beta1) g         (Sec. 3.1, Eqs. 2-4)
 *                   v^ = beta2 v~ + (1-beta2) g^2
 *   3. parameter    decoupled-decay Adam step driven by m^ and v^
 *                   (so_config.optimizer also offers Adam with the decay inside the
 *                   gradient, and AdaBelief, whose 2nd EMA follows (g - m^)^2 + eps)
 *   4. block stats  Delta_m' = max|m^|, Delta_v' = max v^,
 *                   x_p = p-quantile of v^, alpha' = (x_p/Delta_v')^(1/(2^b-1))
 *                                               (Sec. 3.2.2, adaptive base)
 *   5. quantize     m: nearest signed-linear level           (Eq. 1, App. A)
 *                   v: Clip(round(log_alpha(v^/Delta) + xi); 0, 2^b-1),
 *                      xi ~ U(-0.5, 0.5)         (Sec. 3.2.2, log quantizer)
 *
 * Precision.  The optimizer states are binary32 (the paper stores a
 * "full-precision" 32-bit scale per block and counts 1/4 bit per element for
 * it, Sec. 4.2).  Every value that decides a stored code or a stored scale is
 * therefore computed in binary32 with one rounding per operation, in the order
 * written below, so that a second implementation can reproduce the stored
 * bytes.  The parameter update, which decides no code, is evaluated in
 * binary64 from the binary32 m^ and v^ and rounded once.
 *
 * Points on which the paper is silent are decided here and listed in the
 * design notes of the repository (tie rule, quantile rank, degenerate blocks,
 * the exact root, the random stream).
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct so_config {
    uint32_t bits_m;      /* signed-linear code width of the 1st moment        */
    uint32_t bits_v;      /* logarithmic code width of the 2nd moment          */
    uint32_t block_size;  /* elements per quantization block                   */
    uint32_t stochastic;  /* 1: xi ~ U(-.5,.5); 0: xi = 0 (nearest in log dom.) */
    float lr, beta1, beta2, eps, weight_decay;
    float quantile_p;     /* p of the p-quantile that sets the log base        */
    uint64_t seed;        /* key of the xi stream                              */
    uint64_t index_offset;/* global index of element 0 (multiple of 8)         */
    uint32_t m_codebook;  /* 1st-moment levels: 0 signed linear, 1 signed dynamic exponent */
    uint32_t optimizer;   /* SO_ADAMW, SO_ADAM_L2 or SO_ADABELIEF                         */
    float grad_scale;     /* every gradient is multiplied by it first (loss-scale         */
                          /* reciprocal, clipping factor); 1 leaves it unchanged          */
    uint32_t pad_;
} so_config;

/* The EMA optimizers the quantizers are applied to (Sec. 4.2, "Generalizability"):
 * AdamW (decoupled decay), Adam (the decay enters the gradient as lambda * p) and
 * AdaBelief (the unsigned EMA tracks (g - m^)^2 and gains eps at every step). */
enum { SO_ADAMW = 0, SO_ADAM_L2 = 1, SO_ADABELIEF = 2 };

#define SO_MAX_BLOCK 4096
/* A block whose maximum is below this is stored as an all-zero block, so that
 * the reciprocal scales below cannot overflow. */
#define SO_TINY 0x1p-100f
/* Lower clamp of x_p / Delta_v (the log codebook has no zero level). */
#define SO_RHO_MIN 0x1p-64f

/* ------------------------------------------------------------------ levels */

/* Number of non-zero magnitudes of the signed linear set
 * {0, +-1/(2^(b-1)-1), ..., +-1}  (App. A, "Linear mapping"). */
int so_L(uint32_t bits) { return (1 << (bits - 1)) - 1; }
/* Largest code of the unsigned set y_k = alpha^k, k = 0..2^b-1 (Sec. 3.2.2). */
int so_K(uint32_t bits) { return (1 << bits) - 1; }

/* Signed linear level of a code as an exact rational in binary64: codes are
 * assigned in increasing level order (monotone levels, Sec. 3.1), code L is
 * the level 0 and code 2^b-1 is never produced. */
double so_signed_level(uint32_t code, uint32_t bits)
{
    int L = so_L(bits);
    return (double)((int)code - L) / (double)L;
}

/* Q-dagger for the 1st moment: m~ = y_q * Delta (Sec. 3.1).  The level
 * (c-L)/L times Delta is evaluated as (c-L) * (Delta/L): one division per
 * block, one multiplication per element. */
float so_dequant_m(uint32_t code, float scale, uint32_t bits)
{
    int L = so_L(bits);
    float s = scale / (float)L;
    return (float)((int)code - L) * s;
}

/* y_q = alpha^q (Sec. 3.2.2).  Evaluated by binary powering: the powers
 * alpha^(2^j) are formed by repeated squaring and the ones selected by the
 * bits of q are multiplied together from the lowest bit up. */
float so_log_level(float alpha, uint32_t code, uint32_t bits)
{
    float y = 1.0f, pw = alpha;
    for (uint32_t j = 0; j < bits; ++j) {
        if ((code >> j) & 1u) y = y * pw;
        pw = pw * pw;
    }
    return y;
}

/* Q-dagger for the 2nd moment: v~ = alpha^q * Delta. */
float so_dequant_v(uint32_t code, float scale, float alpha, uint32_t bits)
{
    return so_log_level(alpha, code, bits) * scale;
}

/* ------------------------------------------------- dynamic exponent levels */

/* Dynamic exponent (DE) levels (App. A): b bits = E leading zero bits that give the
 * exponent 10^-E, one indicator bit, and the remaining bits as a linear fraction over
 * [0.1, 1]; the signed variant spends the first bit on the sign.  With nsb = b - 1 bits after
 * the first one and exponents 0..nsb-1, exponent step i (scale 10^(-(nsb-1)+i)) owns
 * 2^i fraction cells (signed; 2^(i+1) unsigned), a cell is represented by the mean of its two
 * boundaries on the grid linspace(0.1, 1, cells+1), and the codes left over are the levels 0
 * and 1.  The result has 2^b levels, is not symmetric (+1 exists, -1 does not), and reproduces
 * every radius of Fact A.1 for 2..8 bits.  Writes the levels in increasing order, returns
 * their number. */
int so_de_levels(uint32_t bits, int is_signed, double *out)
{
    const int nsb = (int)bits - 1;
    int n = 0;
    for (int i = 0; i < nsb; ++i) {
        const int cells = is_signed ? (1 << i) : (1 << (i + 1));
        static const double tenth[8] = {1.0, 0.1, 0.01, 0.001, 1e-4, 1e-5, 1e-6, 1e-7};
        const double scale = tenth[(nsb - 1) - i];
        for (int c = 0; c < cells; ++c) {
            const double lo = 0.1 + 0.9 * (double)c / (double)cells;
            const double hi = 0.1 + 0.9 * (double)(c + 1) / (double)cells;
            out[n++] = scale * (lo + hi) / 2.0;
            if (is_signed) out[n++] = -scale * (lo + hi) / 2.0;
        }
    }
    out[n++] = 0.0;
    out[n++] = 1.0;
    for (int i = 1; i < n; ++i) {                 /* insertion sort, n <= 256 */
        double v = out[i]; int j = i - 1;
        while (j >= 0 && out[j] > v) { out[j + 1] = out[j]; --j; }
        out[j + 1] = v;
    }
    return n;
}

/* Signed DE level of a code (codes in increasing level order; code L = 2^(b-1)-1 is 0). */
double so_de_signed_level(uint32_t code, uint32_t bits)
{
    double lv[256];
    so_de_levels(bits, 1, lv);
    return lv[code];
}

/* Q-dagger with the signed DE levels: m~ = fl(fl(y_q) * Delta). */
float so_dequant_m_de(uint32_t code, float scale, uint32_t bits)
{
    return (float)so_de_signed_level(code, bits) * scale;
}

/* Eq. 1 with the signed DE levels, Delta = max|x| over the block.  The nearest level is found
 * on the magnitude: with the non-negative levels P_0 = 0 < P_1 < ... and their midpoints
 * M_j = fl((P_j + P_{j+1}) / 2), j = #{ j : |x * fl(1/Delta)| > M_j }, and the code is
 * L + j for x >= 0 and L - min(j, L) for x < 0 (the negative side has no level -1).  A value
 * exactly on a midpoint takes the level of smaller magnitude. */
void so_quant_m_de_block(const float *x, uint32_t nb, uint32_t bits, uint16_t *codes, float *scale)
{
    const int L = so_L(bits);
    double lv[256];
    so_de_levels(bits, 1, lv);
    float mid[128];
    for (int j = 0; j <= L; ++j) mid[j] = (float)((lv[L + j] + lv[L + j + 1]) / 2.0);
    float d = 0.0f;
    for (uint32_t i = 0; i < nb; ++i) d = fmaxf(d, fabsf(x[i]));
    if (d < SO_TINY) {
        for (uint32_t i = 0; i < nb; ++i) codes[i] = (uint16_t)L;
        *scale = 0.0f;
        return;
    }
    const float inv = 1.0f / d;
    for (uint32_t i = 0; i < nb; ++i) {
        const float z = x[i] * inv;
        const float a = fabsf(z);
        int j = 0;
        for (int k = 0; k <= L; ++k) j += (a > mid[k]) ? 1 : 0;
        if (z < 0.0f) codes[i] = (uint16_t)(L - (j < L ? j : L));
        else          codes[i] = (uint16_t)(L + j);
    }
    *scale = d;
}

/* ------------------------------------------------------------- random xi */

static uint64_t so_mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static uint32_t so_mix32(uint32_t h)
{
    h ^= h >> 16; h *= 0x85EBCA6Bu;
    h ^= h >> 13; h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h;
}

/* Four 32-bit keys of one optimizer step, a function of (seed, step). */
void so_xi_keys(uint64_t seed, uint64_t step, uint32_t keys[4])
{
    const uint64_t gamma = 0x9E3779B97F4A7C15ull;
    uint64_t z = seed + gamma * step;
    uint64_t a = so_mix64(z + gamma);
    uint64_t b = so_mix64(z + 2 * gamma);
    keys[0] = (uint32_t)a; keys[1] = (uint32_t)(a >> 32);
    keys[2] = (uint32_t)b; keys[3] = (uint32_t)(b >> 32);
}

/* 32 uniform bits of element i, a pure function of (seed, step, global element
 * index): xi is drawn independently per element and per update (Sec. 3.2.2;
 * proof of Prop. 3.4).  The construction is that of a split-mix generator, a
 * Weyl sequence whose terms pass through a finalizer: elements are taken in
 * groups of eight; two strong hashes of the group index give a start X and an
 * odd stride Y, element j of the group owns the word w = X + j*Y (mod 2^32),
 * and its bits are w ^ (w >> 15), of which the low 24 bits (they contain every
 * bit of w) are multiplied by an odd 24-bit constant, keeping the low 32 bits
 * of the product.  Without the finalizer the eight words of a group would lie
 * on one arithmetic progression: each uniform, any two independent, but any
 * three linearly dependent (w[j+2] = 2 w[j+1] - w[j]), which shows in every
 * joint statistic of three or more neighbours.  The tests check the joint
 * distribution of neighbours up to all eight of a group. */
uint32_t so_xi_bits(const uint32_t keys[4], uint64_t i)
{
    uint64_t group = i >> 3;
    uint32_t j = (uint32_t)(i & 7u);
    uint32_t glo = (uint32_t)group, ghi = (uint32_t)(group >> 32);
    uint32_t X = so_mix32((glo ^ keys[0]) + ghi * keys[2]);
    uint32_t Y = so_mix32(X ^ keys[1]) | 1u;
    uint32_t w = X + j * Y;
    uint32_t t = w ^ (w >> 15);
    return (t & 0xFFFFFFu) * 0xC2B2AFu;
}

/* xi in the open interval (-0.5, 0.5): the top 23 bits u give
 * (u + 0.5) / 2^23 - 0.5, which binary32 holds exactly (23 bits are what fits
 * the fraction field of a binary32 in [1, 2)). */
float so_xi(const uint32_t keys[4], uint64_t i)
{
    uint32_t u = so_xi_bits(keys, i) >> 9;
    return (float)u * 0x1p-23f + (0x1p-24f - 0.5f);
}

/* xi of n consecutive elements starting at global index i0. */
void so_xi_fill(const uint32_t keys[4], uint64_t i0, uint64_t n, float *out)
{
    for (uint64_t k = 0; k < n; ++k) out[k] = so_xi(keys, i0 + k);
}

/* -------------------------------------------------------------- quantizers */

/* Rank of the p-quantile inside a block of nb values: the r-th smallest with
 * r = max(1, ceil(p * nb)), the product taken in binary32. */
uint32_t so_rank(float p, uint32_t nb)
{
    float x = ceilf(p * (float)nb);
    uint32_t r = x < 1.0f ? 1u : (uint32_t)x;
    return r > nb ? nb : r;
}

/* alpha = rho^(1/K), K = 2^b - 1 (Sec. 3.2.2), made reproducible: alpha is
 * the LARGEST binary32 number in (0, 1] whose last level y_K(alpha), as the
 * dequantizer evaluates it, does not exceed rho.  y_K is non-decreasing in
 * alpha (products of non-negative round-to-nearest factors), so the set is an
 * interval and its maximum is found by stepping from any nearby guess. */
float so_root(float rho, uint32_t bits)
{
    uint32_t K = (uint32_t)so_K(bits);
    if (!(rho < 1.0f)) return 1.0f;
    float y = (float)pow((double)rho, 1.0 / (double)K);
    if (y > 1.0f) y = 1.0f;
    while (so_log_level(y, K, bits) > rho) y = nextafterf(y, 0.0f);
    while (y < 1.0f && so_log_level(nextafterf(y, 2.0f), K, bits) <= rho)
        y = nextafterf(y, 2.0f);
    return y;
}

/* Eq. 1 with the signed linear levels: q = argmin_k |x/Delta - y_k|,
 * Delta = max|x| over the block.  With evenly spaced levels the argmin is
 * round(x * L/Delta); ties go to the even integer.  Writes codes in [0, 2L]
 * and the scale. */
void so_quant_m_block(const float *x, uint32_t nb, uint32_t bits,
                      uint16_t *codes, float *scale)
{
    int L = so_L(bits);
    float d = 0.0f;
    for (uint32_t i = 0; i < nb; ++i) d = fmaxf(d, fabsf(x[i]));
    if (d < SO_TINY) {
        for (uint32_t i = 0; i < nb; ++i) codes[i] = (uint16_t)L;
        *scale = 0.0f;
        return;
    }
    float inv = (float)L / d;
    for (uint32_t i = 0; i < nb; ++i) {
        float t = rintf(x[i] * inv);
        if (t > (float)L) t = (float)L;
        if (t < -(float)L) t = -(float)L;
        codes[i] = (uint16_t)(L + (int)t);
    }
    *scale = d;
}

/* The log quantizer for one value with Delta, alpha and xi given
 * (Sec. 3.2.2, second line of the quantizer equation: rounding happens in the
 * log domain): Clip(round(log_alpha(x/Delta) + xi); 0, K).  A zero x has
 * log_alpha = +infinity and takes the last code. */
uint32_t so_quant_v_elem(float x, float scale, float alpha, float xi, uint32_t bits)
{
    float K = (float)so_K(bits);
    float ratio = x / scale;
    float t = log2f(ratio) / log2f(alpha) + xi;
    t = rintf(t);
    if (!(t < K)) t = K;
    if (t < 0.0f) t = 0.0f;
    return (uint32_t)t;
}

/* Distance, in code units and in binary64, from log_alpha(x/Delta)+xi to the
 * nearest rounding boundary that separates two codes (k+0.5, k = 0..K-1).
 * The tests use it to tell a legitimate flip at a rounding tie from an error. */
double so_quant_v_margin(float x, float scale, float alpha, float xi, uint32_t bits)
{
    int K = so_K(bits);
    if (!(x > 0.0f)) return 1e30;
    double t = log2((double)x / (double)scale) / log2((double)alpha) + (double)xi;
    double best = 1e30;
    for (int k = 0; k < K; ++k) {
        double dist = fabs(t - ((double)k + 0.5));
        if (dist < best) best = dist;
    }
    return best;
}

static int so_cmp_float(const void *a, const void *b)
{
    float x = *(const float *)a, y = *(const float *)b;
    return (x > y) - (x < y);
}

/* The r-th smallest of x[0..nb) (1-based r), by sorting a copy. */
float so_order_statistic(const float *x, uint32_t nb, uint32_t r)
{
    float tmp[SO_MAX_BLOCK];
    memcpy(tmp, x, nb * sizeof(float));
    qsort(tmp, nb, sizeof(float), so_cmp_float);
    return tmp[r - 1];
}

/* Quantize one block of the 2nd moment: Delta = max x, x_p = p-quantile,
 * alpha = (x_p/Delta)^(1/K), then the log quantizer per element.  i0 is the
 * global index of x[0] (for xi).  margin may be NULL. */
void so_quant_v_block(const float *x, uint32_t nb, uint32_t bits, float p,
                      uint32_t stochastic, const uint32_t keys[4], uint64_t i0,
                      uint16_t *codes, float *scale, float *base, double *margin)
{
    float d = 0.0f;
    for (uint32_t i = 0; i < nb; ++i) d = fmaxf(d, x[i]);
    if (d < SO_TINY) {                 /* all-zero block: Delta = 0, alpha = 1 */
        for (uint32_t i = 0; i < nb; ++i) { codes[i] = 0; if (margin) margin[i] = 1e30; }
        *scale = 0.0f; *base = 1.0f;
        return;
    }
    float xp = so_order_statistic(x, nb, so_rank(p, nb));
    float rho = xp / d;
    if (rho < SO_RHO_MIN) rho = SO_RHO_MIN;
    float alpha = so_root(rho, bits);
    *scale = d; *base = alpha;
    if (alpha == 1.0f) {               /* constant block: every value is Delta */
        for (uint32_t i = 0; i < nb; ++i) { codes[i] = 0; if (margin) margin[i] = 1e30; }
        return;
    }
    for (uint32_t i = 0; i < nb; ++i) {
        float xi = stochastic ? so_xi(keys, i0 + i) : 0.0f;
        codes[i] = (uint16_t)so_quant_v_elem(x[i], d, alpha, xi, bits);
        if (margin) margin[i] = so_quant_v_margin(x[i], d, alpha, xi, bits);
    }
}

/* ------------------------------------------- comparison quantizers for v */

/* The unsigned level sets the paper compares against (App. A; used on the 2nd moment by earlier
 * low-bit optimizers), each with nearest rounding (Eq. 1) and Delta = max x:
 *   SO_U_LINEAR         {0, 1/(2^b-1), ..., 1}
 *   SO_U_LINEAR_NOZERO  {1/2^b, 2/2^b, ..., 1}         (the variant that excludes the zero point)
 *   SO_U_DE             unsigned dynamic exponent (so_de_levels with is_signed = 0)
 * They exist for the swamping experiments (Sec. 3.2.1: Cor. 3.2 and the synthetic example); the
 * optimizer step never uses them. */
enum { SO_U_LINEAR = 1, SO_U_LINEAR_NOZERO = 2, SO_U_DE = 3 };

/* Writes the 2^b increasing levels of one of the sets above; returns their number (0: unknown). */
int so_unsigned_levels(uint32_t bits, int kind, double *out)
{
    const int n = 1 << bits;
    if (bits < 1 || bits > 8) return 0;
    if (kind == SO_U_LINEAR) {
        for (int k = 0; k < n; ++k) out[k] = (double)k / (double)(n - 1);
        return n;
    }
    if (kind == SO_U_LINEAR_NOZERO) {
        for (int k = 0; k < n; ++k) out[k] = (double)(k + 1) / (double)n;
        return n;
    }
    if (kind == SO_U_DE) return so_de_levels(bits, 0, out);
    return 0;
}

/* Q-dagger of a comparison quantizer: x~ = fl(fl(y_q) * Delta). */
float so_dequant_unsigned(uint32_t code, float scale, uint32_t bits, int kind)
{
    double lv[256];
    so_unsigned_levels(bits, kind, lv);
    return (float)lv[code] * scale;
}

/* Eq. 1 for a comparison quantizer: Delta = max x over the block, q = argmin_k |x/Delta - y_k|
 * (ties to the lower level), the division in binary32. */
void so_quant_unsigned_block(const float *x, uint32_t nb, uint32_t bits, int kind,
                             uint16_t *codes, float *scale)
{
    double lv[256];
    const int n = so_unsigned_levels(bits, kind, lv);
    float d = 0.0f;
    for (uint32_t i = 0; i < nb; ++i) d = fmaxf(d, x[i]);
    *scale = d;
    for (uint32_t i = 0; i < nb; ++i) {
        const double r = d > 0.0f ? (double)(x[i] / d) : 0.0;
        int best = 0;
        for (int k = 1; k < n; ++k)
            if (fabs(r - lv[k]) < fabs(r - lv[best])) best = k;
        codes[i] = (uint16_t)best;
    }
}

/* One step of the quantized unsigned EMA alone (Sec. 3.1, Eqs. 2-4 with the signal given):
 * dequantize, x^ = fma(beta, x~, fl((1-beta) z)), quantize, block by block.  kind 0 is the
 * paper's logarithmic quantizer (so_quant_v_block; base holds alpha per block), kinds 1..3 the
 * comparison quantizers (base unused).  step and seed feed the xi stream of kind 0. */
int so_unsigned_ema_step(uint16_t *codes, float *scale, float *base, const float *z, uint64_t n,
                         uint32_t block, float beta, uint32_t bits, int kind, float p,
                         uint32_t stochastic, uint64_t seed, uint64_t step)
{
    if (block == 0 || block > SO_MAX_BLOCK || kind < 0 || kind > SO_U_DE) return -1;
    const float omb = 1.0f - beta;
    uint32_t keys[4];
    so_xi_keys(seed, step, keys);
    for (uint64_t i0 = 0, blk = 0; i0 < n; i0 += block, ++blk) {
        float xh[SO_MAX_BLOCK];
        const uint32_t nb = (uint32_t)((n - i0) < block ? (n - i0) : block);
        for (uint32_t k = 0; k < nb; ++k) {
            const float xt = kind == 0 ? so_dequant_v(codes[i0 + k], scale[blk], base[blk], bits)
                                       : so_dequant_unsigned(codes[i0 + k], scale[blk], bits, kind);
            xh[k] = fmaf(beta, xt, omb * z[i0 + k]);
        }
        if (kind == 0)
            so_quant_v_block(xh, nb, bits, p, stochastic, keys, i0, codes + i0, scale + blk, base + blk, NULL);
        else
            so_quant_unsigned_block(xh, nb, bits, kind, codes + i0, scale + blk);
    }
    return 0;
}

/* -------------------------------------------------------------- the step */

/* One optimizer step over n elements with one code per uint16 (any width
 * 2..16).  g is binary32 (a bf16 gradient is widened exactly by the caller).
 * step is 1-based.  margin (n doubles) and mhat/vhat (n floats) may be NULL;
 * when given they receive the tie margins of the v codes and the fresh EMA
 * values m^, v^.  threads <= 1 runs serially. */
int so_step_unpacked(float *param, const float *grad,
                     uint16_t *m_codes, float *m_scale,
                     uint16_t *v_codes, float *v_scale, float *v_base,
                     uint64_t n, uint64_t step, const so_config *cfg,
                     double *margin, float *mhat_out, float *vhat_out, int threads)
{
    const uint32_t B = cfg->block_size;
    if (B == 0 || B > SO_MAX_BLOCK || step == 0) return -1;
    if (cfg->bits_m < 2 || cfg->bits_m > 16 || cfg->bits_v < 2 || cfg->bits_v > 16) return -1;
    if (cfg->m_codebook > 1 || (cfg->m_codebook == 1 && cfg->bits_m > 8)) return -1;
    if (cfg->optimizer > SO_ADABELIEF) return -1;
    const uint64_t nblk = (n + B - 1) / B;
    const float beta1 = cfg->beta1, beta2 = cfg->beta2;
    const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
    /* Adam with decoupled weight decay and bias correction; eps is added to
     * the bias-corrected root. */
    const double bc1 = 1.0 - pow((double)beta1, (double)step);
    const double bc2 = 1.0 - pow((double)beta2, (double)step);
    const double decay = cfg->optimizer == SO_ADAM_L2
                             ? 1.0 : 1.0 - (double)cfg->lr * (double)cfg->weight_decay;
    const double step_size = (double)cfg->lr / bc1;
    uint32_t keys[4];
    so_xi_keys(cfg->seed, step, keys);
#ifdef _OPENMP
    if (threads < 1) threads = 1;
#pragma omp parallel for schedule(static) num_threads(threads)
#endif
    for (int64_t blk = 0; blk < (int64_t)nblk; ++blk) {
        float mh[SO_MAX_BLOCK], vh[SO_MAX_BLOCK];
        const uint64_t i0 = (uint64_t)blk * B;
        const uint32_t nb = (uint32_t)((n - i0) < B ? (n - i0) : B);
        for (uint32_t k = 0; k < nb; ++k) {
            const uint64_t i = i0 + k;
            float g = grad[i] * cfg->grad_scale;
            if (cfg->optimizer == SO_ADAM_L2) g = fmaf(cfg->weight_decay, param[i], g);
            const float mt = cfg->m_codebook ? so_dequant_m_de(m_codes[i], m_scale[blk], cfg->bits_m)
                                             : so_dequant_m(m_codes[i], m_scale[blk], cfg->bits_m);
            const float vt = so_dequant_v(v_codes[i], v_scale[blk], v_base[blk], cfg->bits_v);
            /* EMA (Sec. 3.1): the signal term is rounded, then one fused
             * multiply-add joins it to beta * state. */
            mh[k] = fmaf(beta1, mt, omb1 * g);
            if (cfg->optimizer == SO_ADABELIEF) {
                /* the signal of the unsigned EMA is the squared distance of the gradient
                 * from the fresh 1st moment, and eps is added to the state itself */
                const float d = g - mh[k];
                vh[k] = fmaf(beta2, vt, omb2 * (d * d)) + cfg->eps;
            } else {
                vh[k] = fmaf(beta2, vt, omb2 * (g * g));
            }
            const double denom = sqrt((double)vh[k]) / sqrt(bc2) + (double)cfg->eps;
            const double pd = (double)param[i] * decay - step_size * (double)mh[k] / denom;
            param[i] = (float)pd;
            if (mhat_out) mhat_out[i] = mh[k];
            if (vhat_out) vhat_out[i] = vh[k];
        }
        if (cfg->m_codebook) so_quant_m_de_block(mh, nb, cfg->bits_m, m_codes + i0, m_scale + blk);
        else so_quant_m_block(mh, nb, cfg->bits_m, m_codes + i0, m_scale + blk);
        so_quant_v_block(vh, nb, cfg->bits_v, cfg->quantile_p, cfg->stochastic, keys,
                         cfg->index_offset + i0, v_codes + i0, v_scale + blk, v_base + blk,
                         margin ? margin + i0 : NULL);
    }
    (void)threads;
    return 0;
}

/* ------------------------------------------------------ 16-bit weight copy */

/* The bfloat16 nearest to each binary32 value, ties to the even mantissa (the
 * 16-bit weights that mixed-precision training keeps next to the 32-bit ones,
 * Sec. 1).  The two candidates are x with its low 16 bits cleared and the next
 * larger magnitude; infinities and NaNs keep their upper half. */
void so_round_bf16(const float *x, uint16_t *out, uint64_t n)
{
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t u;
        memcpy(&u, &x[i], 4);
        uint32_t lo = u & 0xFFFF0000u, hi = lo + 0x10000u;
        if ((u & 0x7F800000u) == 0x7F800000u) { out[i] = (uint16_t)(u >> 16) | ((u & 0xFFFFu) ? 0x40u : 0u); continue; }
        float flo, fhi;
        memcpy(&flo, &lo, 4);
        memcpy(&fhi, &hi, 4);                    /* may be +-inf: overflow rounds there */
        double dlo = fabs((double)x[i] - (double)flo);
        double dhi = (hi & 0x7F800000u) == 0x7F800000u
                         ? fabs(ldexp(1.0, 128) - fabs((double)x[i]))   /* distance to the value inf stands for */
                         : fabs((double)fhi - (double)x[i]);
        uint32_t pick = dlo < dhi ? lo : dhi < dlo ? hi : ((lo >> 16) & 1u) ? hi : lo;
        out[i] = (uint16_t)(pick >> 16);
    }
}

/* --------------------------------------------------------------- packing */

/* Codes per 32-bit word: 16 two-bit, 10 three-bit (two pad bits), 8 four-bit
 * (Sec. 3.4 packs 2 or 4 codes per byte; three-bit codes go ten to a word). */
uint32_t so_codes_per_word(uint32_t bits) { return 32u / bits; }

uint64_t so_code_words(uint64_t n, uint32_t bits)
{
    uint32_t c = so_codes_per_word(bits);
    return (n + c - 1) / c;
}

/* Element i sits in word i / c at bit offset bits * (i mod c); unused bits
 * are zero. */
void so_pack(const uint16_t *codes, uint64_t n, uint32_t bits, uint32_t *words)
{
    uint32_t c = so_codes_per_word(bits);
    memset(words, 0, so_code_words(n, bits) * sizeof(uint32_t));
    for (uint64_t i = 0; i < n; ++i)
        words[i / c] |= (uint32_t)codes[i] << (bits * (uint32_t)(i % c));
}

void so_unpack(const uint32_t *words, uint64_t n, uint32_t bits, uint16_t *codes)
{
    uint32_t c = so_codes_per_word(bits);
    uint32_t mask = (1u << bits) - 1u;
    for (uint64_t i = 0; i < n; ++i)
        codes[i] = (uint16_t)((words[i / c] >> (bits * (uint32_t)(i % c))) & mask);
}

/* The zero state: m = 0 is code L with Delta_m = 0; v = 0 is code 0 with
 * Delta_v = 0 and alpha = 1. */
void so_state_init(uint32_t *m_words, float *m_scale, uint32_t *v_words,
                   float *v_scale, float *v_base, uint64_t n, const so_config *cfg)
{
    const uint32_t B = cfg->block_size;
    const uint64_t nblk = (n + B - 1) / B;
    uint16_t *tmp = (uint16_t *)calloc(n ? n : 1, sizeof(uint16_t));
    for (uint64_t i = 0; i < n; ++i) tmp[i] = (uint16_t)so_L(cfg->bits_m);
    so_pack(tmp, n, cfg->bits_m, m_words);
    for (uint64_t i = 0; i < n; ++i) tmp[i] = 0;
    so_pack(tmp, n, cfg->bits_v, v_words);
    free(tmp);
    for (uint64_t b = 0; b < nblk; ++b) { m_scale[b] = 0.0f; v_scale[b] = 0.0f; v_base[b] = 1.0f; }
}

/* One optimizer step on packed states (2-, 3- or 4-bit codes). */
int so_step_packed(float *param, const float *grad,
                   uint32_t *m_words, float *m_scale,
                   uint32_t *v_words, float *v_scale, float *v_base,
                   uint64_t n, uint64_t step, const so_config *cfg,
                   double *margin, int threads)
{
    if (cfg->bits_m < 2 || cfg->bits_m > 4 || cfg->bits_v < 2 || cfg->bits_v > 4) return -1;
    uint16_t *mc = (uint16_t *)calloc(n ? n : 1, sizeof(uint16_t));
    uint16_t *vc = (uint16_t *)calloc(n ? n : 1, sizeof(uint16_t));
    so_unpack(m_words, n, cfg->bits_m, mc);
    so_unpack(v_words, n, cfg->bits_v, vc);
    int rc = so_step_unpacked(param, grad, mc, m_scale, vc, v_scale, v_base, n, step, cfg,
                              margin, NULL, NULL, threads);
    if (rc == 0) {
        so_pack(mc, n, cfg->bits_m, m_words);
        so_pack(vc, n, cfg->bits_v, v_words);
    }
    free(mc); free(vc);
    return rc;
}

int so_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
