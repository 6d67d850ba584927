// A caller of libsolo without PyTorch: plain HIP memory, the C-ABI of include/solo.h, one stream.
//
//   solo_c_example [n] [steps]      (defaults: 1,000,003 elements, 3 steps)
//
// Parameters and bf16 gradients come from a small integer generator, so that another caller (the
// GPU tests, through the Python binding) can produce the same inputs and compare the printed
// checksums: the sum of the parameters' bit patterns and the XOR-rotate of every state word.
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/solo.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)
#define CHECK_SOLO(x) do { int r_ = (x); if (r_ != SOLO_OK) { \
    fprintf(stderr, "%s: %s\n", #x, solo_strerror(r_)); return 1; } } while (0)

// x <- x * 1664525 + 1013904223 (mod 2^32); the value in [-1, 1) from the top 24 bits
static float next_unit(uint32_t &x)
{
    x = x * 1664525u + 1013904223u;
    return (float)(int32_t)(x >> 8) * (1.0f / 8388608.0f) - 1.0f;
}

static uint16_t to_bf16(float f)          // round to nearest, ties to even (finite input)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static uint64_t fold(uint64_t h, uint32_t w) { return ((h << 7) | (h >> 57)) ^ w; }

int main(int argc, char **argv)
{
    const uint64_t n = argc > 1 ? strtoull(argv[1], nullptr, 10) : 1000003ull;
    const int steps = argc > 2 ? atoi(argv[2]) : 3;
    solo_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.bits_m = 2; cfg.bits_v = 3; cfg.block_size = 128; cfg.grad_dtype = SOLO_GRAD_BF16;
    cfg.lr = 1e-3f; cfg.beta1 = solo_beta1_default(2, 0); cfg.beta2 = 0.999f; cfg.eps = 1e-8f;
    cfg.weight_decay = 0.01f; cfg.quantile_p = 0.1f; cfg.flags = SOLO_FLAG_STOCHASTIC; cfg.seed = 42;

    const size_t wm = solo_code_words(n, cfg.bits_m), wv = solo_code_words(n, cfg.bits_v);
    const size_t nb = solo_num_blocks(n, cfg.block_size);
    float *p, *m_scale, *v_scale, *v_base;
    uint16_t *g;
    uint32_t *m_codes, *v_codes;
    CHECK_HIP(hipMalloc(&p, n * 4)); CHECK_HIP(hipMalloc(&g, n * 2));
    CHECK_HIP(hipMalloc(&m_codes, wm * 4)); CHECK_HIP(hipMalloc(&v_codes, wv * 4));
    CHECK_HIP(hipMalloc(&m_scale, nb * 4)); CHECK_HIP(hipMalloc(&v_scale, nb * 4)); CHECK_HIP(hipMalloc(&v_base, nb * 4));
    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));

    std::vector<float> hp(n);
    std::vector<uint16_t> hg(n);
    uint32_t x = 12345u;
    for (uint64_t i = 0; i < n; ++i) hp[i] = 0.02f * next_unit(x);
    CHECK_HIP(hipMemcpyAsync(p, hp.data(), n * 4, hipMemcpyHostToDevice, stream));
    CHECK_SOLO(solo_state_init(m_codes, m_scale, v_codes, v_scale, v_base, n, &cfg, stream));
    for (int step = 1; step <= steps; ++step) {
        for (uint64_t i = 0; i < n; ++i) hg[i] = to_bf16(1e-3f * next_unit(x));
        CHECK_HIP(hipMemcpyAsync(g, hg.data(), n * 2, hipMemcpyHostToDevice, stream));
        CHECK_SOLO(solo_adamw_step(p, g, m_codes, m_scale, v_codes, v_scale, v_base, n, (uint64_t)step, &cfg, stream));
        CHECK_HIP(hipStreamSynchronize(stream));       // hg is refilled next
    }
    std::vector<uint32_t> words(wm > wv ? wm : wv), sc(nb);
    CHECK_HIP(hipMemcpy(hp.data(), p, n * 4, hipMemcpyDeviceToHost));
    uint64_t sum_p = 0, h = 0;
    for (uint64_t i = 0; i < n; ++i) { uint32_t u; memcpy(&u, &hp[i], 4); sum_p += u; }
    CHECK_HIP(hipMemcpy(words.data(), m_codes, wm * 4, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < wm; ++i) h = fold(h, words[i]);
    CHECK_HIP(hipMemcpy(words.data(), v_codes, wv * 4, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < wv; ++i) h = fold(h, words[i]);
    for (float *s : {m_scale, v_scale, v_base}) {
        CHECK_HIP(hipMemcpy(sc.data(), s, nb * 4, hipMemcpyDeviceToHost));
        for (size_t i = 0; i < nb; ++i) h = fold(h, sc[i]);
    }
    printf("n %llu steps %d param_sum %llu state_hash %016llx\n", (unsigned long long)n, steps,
           (unsigned long long)sum_p, (unsigned long long)h);
    return 0;
}
