// Achievable ceilings of one MI355X for the two resources the grouped GEMM is bound by:
//   1. streaming reads from HBM (a weight-sized buffer per launch, rotating through 1 GiB so that no
//      launch finds its data in the 256 MB last-level cache),
//   2. the FP16 MFMA pipe (v_mfma_f32_32x32x16_f16 on independent accumulators, two wavefronts per
//      SIMD), once with constant and once with normally distributed operands: the chip's clock
//      under matrix load depends on how many bits toggle.
// Prints one line per test.  These are reference points for the roofline fractions bench.py
// reports; they are not used by the library.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <math.h>

#define CK(x)                                                                                   \
    do {                                                                                        \
        hipError_t e_ = (x);                                                                    \
        if (e_ != hipSuccess) {                                                                 \
            fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);     \
            exit(1);                                                                            \
        }                                                                                       \
    } while (0)

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

// consecutive wavefronts read consecutive 1 KB chunks
__global__ __launch_bounds__(256) void read_gridstride(const uint4 *__restrict__ p, size_t nvec, uint32_t *out)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    uint32_t acc = 0;
    for (; i < nvec; i += (size_t)gridDim.x * 256) {
        const uint4 v = p[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x12345678u) out[0] = acc;
}

// every wavefront reads its own contiguous region, sixteen 1 KB loads in flight (the access
// pattern of the weight-streaming GEMM)
__global__ __launch_bounds__(256, 2) void read_regions(const uint4 *__restrict__ p, int kb_per_wave, uint32_t *out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint4 *base = p + ((size_t)blockIdx.x * 4 + wave) * (size_t)kb_per_wave * 64 + lane;
    uint4 w[16];
    uint32_t acc = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) w[i] = base[(size_t)i * 64];
    for (int g = 0; g < kb_per_wave; g += 16) {
        const bool more = g + 32 <= kb_per_wave;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint4 v = w[i];
            if (more) w[i] = base[(size_t)(g + 16 + i) * 64];
            acc ^= v.x ^ v.y ^ v.z ^ v.w;
        }
    }
    if (acc == 0x12345678u) out[0] = acc;
}

// A resident grid that reads 128 MiB in one launch: every wavefront streams UNITS regions of 16 KB, one after the
// other (region u of all wavefronts together is one contiguous range, as the two weight matrices of a decode step
// are), through a ring of RING 16-byte-per-lane loads that is refilled block by block.  The refill's address is made
// to depend on the block just consumed, so that the loads stay in ring order.
// THREADS = 1024 is the decode kernel's own launch shape: one workgroup of sixteen wavefronts per compute unit, all of
// them started at once.
template <int UNITS, int RING, int THREADS = 256>
__global__ __launch_bounds__(THREADS, THREADS == 256 ? 2 : 1) void read_resident(const uint4 *p, uint32_t *out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t nw = (size_t)gridDim.x * (THREADS / 64), w = (size_t)blockIdx.x * (THREADS / 64) + wave;
    const uint4 *base = p + w * 16 * 64 + lane;
    uint4 ring[RING];
    uint32_t acc = 0;
#pragma unroll
    for (int i = 0; i < RING; ++i) ring[i] = base[(size_t)i * 64];
#pragma unroll
    for (int g = 0; g < UNITS * 16; ++g) {
        const uint4 v = ring[g % RING];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
        uint32_t z;
        asm volatile("v_and_b32 %0, 0, %1" : "=v"(z) : "v"(v.x));      // an opaque zero that depends on the block's data
        const int n = g + RING;
        if (n < UNITS * 16) ring[g % RING] = base[((size_t)(n / 16) * nw * 16 + (n % 16)) * 64 + z];
    }
    if (acc == 0x12345678u) out[0] = acc;
}

__global__ __launch_bounds__(256, 2) void mfma_loop(const half8_t *__restrict__ in, float *out, int iters)
{
    const half8_t a = in[threadIdx.x], b = in[256 + threadIdx.x];
    float16_t acc[4];
    for (int q = 0; q < 4; ++q)
        for (int j = 0; j < 16; ++j) acc[q][j] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[q], 0, 0, 0);
    }
    float s = 0.0f;
    for (int q = 0; q < 4; ++q)
        for (int j = 0; j < 16; ++j) s += acc[q][j];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

int main()
{
    const size_t total = (size_t)1 << 30, per_launch = (size_t)64 << 20;
    uint4 *buf;
    uint32_t *sink;
    CK(hipMalloc(&buf, total));
    CK(hipMalloc(&sink, 4));
    CK(hipMemset(buf, 1, total));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    auto timed = [&](int reps, auto launch) {
        for (int i = 0; i < 3; ++i) launch(i);
        CK(hipDeviceSynchronize());
        CK(hipEventRecord(e0));
        for (int i = 0; i < reps; ++i) launch(i);
        CK(hipEventRecord(e1));
        CK(hipEventSynchronize(e1));
        float ms;
        CK(hipEventElapsedTime(&ms, e0, e1));
        return (double)ms / reps * 1e-3;
    };
    for (int grid : {1024, 2048, 4096}) {
        const double s = timed(32, [&](int i) {
            hipLaunchKernelGGL(read_gridstride, dim3(grid), dim3(256), 0, 0,
                               (const uint4 *)((const char *)buf + (size_t)(i % 16) * per_launch), per_launch / 16, sink);
        });
        printf("hbm read, grid-stride, 64 MiB per launch, %d blocks: %.1f us per launch, %.0f GB/s\n", grid, s * 1e6, per_launch / s / 1e9);
    }
    for (int kb : {16, 32, 64}) {
        const int waves = (int)(per_launch / 1024 / kb);
        const double s = timed(32, [&](int i) {
            hipLaunchKernelGGL(read_regions, dim3(waves / 4), dim3(256), 0, 0,
                               (const uint4 *)((const char *)buf + (size_t)(i % 16) * per_launch), kb, sink);
        });
        printf("hbm read, %d KB region per wavefront (%d wavefronts), 64 MiB per launch: %.1f us per launch, %.0f GB/s\n", kb, waves, s * 1e6, per_launch / s / 1e9);
    }
    {
        const size_t big = (size_t)128 << 20;
        auto at = [&](int i) { return (const uint4 *)((const char *)buf + (size_t)(i % 8) * big); };
        double s = timed(32, [&](int i) {
            hipLaunchKernelGGL(read_regions, dim3(1024), dim3(256), 0, 0, (const uint4 *)((const char *)at(i)), 16, sink);
            hipLaunchKernelGGL(read_regions, dim3(1024), dim3(256), 0, 0, (const uint4 *)((const char *)at(i) + per_launch), 16, sink);
        });
        printf("hbm read, 128 MiB in two launches of 4096 wavefronts x 16 KB: %.1f us per pair, %.0f GB/s\n", s * 1e6, big / s / 1e9);
        s = timed(32, [&](int i) { hipLaunchKernelGGL((read_resident<4, 16>), dim3(512), dim3(256), 0, 0, at(i), sink); });
        printf("hbm read, 128 MiB in one launch, 2048 resident wavefronts (8 per CU) x 4 regions of 16 KB, ring of 16: %.1f us, %.0f GB/s\n", s * 1e6, big / s / 1e9);
        s = timed(32, [&](int i) { hipLaunchKernelGGL((read_resident<2, 16>), dim3(1024), dim3(256), 0, 0, at(i), sink); });
        printf("hbm read, 128 MiB in one launch, 4096 resident wavefronts (16 per CU) x 2 regions of 16 KB, ring of 16: %.1f us, %.0f GB/s\n", s * 1e6, big / s / 1e9);
        s = timed(32, [&](int i) { hipLaunchKernelGGL((read_resident<2, 8>), dim3(1024), dim3(256), 0, 0, at(i), sink); });
        printf("hbm read, 128 MiB in one launch, 4096 resident wavefronts (16 per CU) x 2 regions of 16 KB, ring of 8: %.1f us, %.0f GB/s\n", s * 1e6, big / s / 1e9);
        s = timed(32, [&](int i) { hipLaunchKernelGGL((read_resident<2, 8, 512>), dim3(512), dim3(512), 0, 0, at(i), sink); });
        printf("hbm read, 128 MiB in one launch, 512 workgroups of 8 wavefronts x 2 regions of 16 KB, ring of 8: %.1f us, %.0f GB/s\n", s * 1e6, big / s / 1e9);
        s = timed(32, [&](int i) { hipLaunchKernelGGL((read_resident<2, 8, 1024>), dim3(256), dim3(1024), 0, 0, at(i), sink); });
        printf("hbm read, 128 MiB in one launch, 256 workgroups of 16 wavefronts (one per CU, the decode kernel's shape) x 2 regions of 16 KB, ring of 8: %.1f us, %.0f GB/s\n", s * 1e6, big / s / 1e9);
    }
    {
        const double s = timed(4, [&](int) {
            hipLaunchKernelGGL(read_gridstride, dim3(4096), dim3(256), 0, 0, (const uint4 *)buf, total / 16, sink);
        });
        printf("hbm read, grid-stride, 1 GiB per launch: %.1f us per launch, %.0f GB/s\n", s * 1e6, total / s / 1e9);
    }

    // MFMA: 512 blocks = two wavefronts per SIMD
    _Float16 *h_in = (_Float16 *)malloc(512 * 8 * sizeof(_Float16));
    half8_t *d_in;
    float *d_out;
    CK(hipMalloc(&d_in, 512 * 8 * sizeof(_Float16)));
    CK(hipMalloc(&d_out, (size_t)512 * 256 * sizeof(float)));
    const int iters = 20000;
    for (int mode = 0; mode < 2; ++mode) {
        uint64_t st = 88172645463325252ull;
        for (int i = 0; i < 512 * 8; ++i) {
            float v = 1.0f;
            if (mode == 1) {                       // Box-Muller on a xorshift stream
                st ^= st << 13; st ^= st >> 7; st ^= st << 17;
                const double u1 = ((st >> 11) + 1.0) / 9007199254740993.0;
                st ^= st << 13; st ^= st >> 7; st ^= st << 17;
                const double u2 = (st >> 11) / 9007199254740992.0;
                v = (float)(sqrt(-2.0 * log(u1)) * cos(6.283185307179586 * u2));
            }
            h_in[i] = (_Float16)v;
        }
        CK(hipMemcpy(d_in, h_in, 512 * 8 * sizeof(_Float16), hipMemcpyHostToDevice));
        const double s = timed(3, [&](int) { hipLaunchKernelGGL(mfma_loop, dim3(512), dim3(256), 0, 0, d_in, d_out, iters); });
        const double flops = 2.0 * 32 * 32 * 16 * 4 * (double)iters * 512 * 4;
        printf("mfma f32_32x32x16_f16, %s operands, 2 wavefronts per SIMD: %.1f TFLOP/s\n", mode ? "N(0,1)" : "constant", flops / s / 1e12);
    }
    return 0;
}
