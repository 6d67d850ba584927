// Memory-ceiling probe for the SOLO step on one MI355X: kernels that move the step's
// dominant traffic and do no arithmetic.  It answers "what does HBM deliver for this mix of
// reads and writes", which is the practical roofline the step kernel is measured against
// next to the 8 TB/s datasheet peak.
//
//   stream_probe [n_elements]        (default: the LLaMA-7B-shaped 6,738,415,616)
//
// Reports GB/s for: read only, write only, copy, and "step-shaped": fp32 parameters read and
// written in place plus bf16 gradients read (10 B/element), with the step kernel's access
// pattern (one wavefront per 2560-element super-tile, 128-bit coalesced non-temporal
// accesses, XCD-aware workgroup-to-tile mapping).
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstdlib>

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)

__global__ void k_read(const f32x4 *__restrict__ a, float *sink, size_t n4)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    float acc = 0.0f;
    for (; i < n4; i += stride) { const f32x4 v = a[i]; acc += v.x + v.y + v.z + v.w; }
    if (acc == 123.456f) sink[0] = acc;
}

__global__ void k_write(f32x4 *__restrict__ b, size_t n4)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const f32x4 v = {1.0f, 2.0f, 3.0f, 4.0f};
    for (; i < n4; i += stride) b[i] = v;
}

__global__ void k_copy(const f32x4 *__restrict__ a, f32x4 *__restrict__ b, size_t n4)
{
    // each workgroup copies a contiguous run of 4 x 256 vectors
    const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
    for (int k = 0; k < 4; ++k) { const size_t i = base + (size_t)k * 256; if (i < n4) b[i] = a[i]; }
}

__global__ __launch_bounds__(256) void k_step_shaped(float *__restrict__ p, const uint16_t *__restrict__ g,
                                                      size_t n_tiles, size_t wg_per_xcd)
{
    const size_t wg = (size_t)(blockIdx.x & 7) * wg_per_xcd + (blockIdx.x >> 3);
    const size_t tile = wg * 4 + (threadIdx.x >> 6);
    if (tile >= n_tiles) return;
    const unsigned lane = threadIdx.x & 63;
    for (int it = 0; it < 5; ++it) {
        const size_t e = tile * 2560 + (size_t)it * 512;
        f32x4 p0 = __builtin_nontemporal_load((const f32x4 *)(p + e + lane * 4));
        f32x4 p1 = __builtin_nontemporal_load((const f32x4 *)(p + e + 256 + lane * 4));
        const u32x4 gg = __builtin_nontemporal_load((const u32x4 *)(g + e + lane * 8));
        p0.x += __uint_as_float(gg.x << 16); p0.y += __uint_as_float(gg.y << 16);
        p1.x += __uint_as_float(gg.z << 16); p1.y += __uint_as_float(gg.w << 16);
        // the step kernel's own store: non-temporal, written through at device scope; two wait
        // states before the data registers of a 128-bit store may be reused
        asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p + e + lane * 4), "v"(p0) : "memory");
        asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p + e + 256 + lane * 4), "v"(p1) : "memory");
    }
}

int main(int argc, char **argv)
{
    size_t n = argc > 1 ? strtoull(argv[1], nullptr, 10) : 6738415616ull;
    n = n / 2560 * 2560;
    const size_t n4 = n / 4;
    float *a, *b, *sink; uint16_t *g;
    CHECK(hipMalloc(&a, n * 4)); CHECK(hipMalloc(&b, n * 4)); CHECK(hipMalloc(&g, n * 2)); CHECK(hipMalloc(&sink, 64));
    CHECK(hipMemset(a, 0, n * 4)); CHECK(hipMemset(b, 0, n * 4)); CHECK(hipMemset(g, 0, n * 2));
    hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    auto timeit = [&](const char *name, double bytes, auto launch) -> int {
        launch(); CHECK(hipDeviceSynchronize());
        float best = 1e30f, total = 0.0f; const int reps = 5;
        for (int r = 0; r < reps; ++r) {
            CHECK(hipEventRecord(e0)); launch(); CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1));
            float ms; CHECK(hipEventElapsedTime(&ms, e0, e1)); best = ms < best ? ms : best; total += ms;
        }
        printf("%-34s %8.3f ms (best of %d, mean %.3f)  %6.0f GB/s  %.1f %% of 8 TB/s\n", name, best, reps,
               total / reps, bytes / best / 1e6, bytes / best / 1e6 / 80.0);
        fflush(stdout);
        return 0;
    };
    printf("stream_probe: n = %zu elements\n", n);
    if (timeit("read only (fp32)", n * 4.0, [&] { hipLaunchKernelGGL(k_read, dim3(262144), dim3(256), 0, 0, (const f32x4 *)a, sink, n4); })) return 1;
    if (timeit("write only (fp32)", n * 4.0, [&] { hipLaunchKernelGGL(k_write, dim3(32768), dim3(256), 0, 0, (f32x4 *)b, n4); })) return 1;
    if (timeit("copy (4 B read + 4 B written)", n * 8.0, [&] { hipLaunchKernelGGL(k_copy, dim3((unsigned)((n4 + 1023) / 1024)), dim3(256), 0, 0, (const f32x4 *)a, (f32x4 *)b, n4); })) return 1;
    const size_t n_tiles = n / 2560, nwg = (n_tiles + 3) / 4, per = (nwg + 7) / 8;
    if (timeit("step-shaped (p rw + bf16 g r)", n * 10.0, [&] { hipLaunchKernelGGL(k_step_shaped, dim3((unsigned)(per * 8)), dim3(256), 0, 0, a, g, n_tiles, per); })) return 1;
    return 0;
}
