// Timeline of the decode kernel (moe_ffn_decode.hip) on the decode workload's shape (64 tokens, top-2, 32 experts,
// d_model 1024, d_ff 4096, int4): the kernel is compiled into this program with its time-stamp hook switched on, every
// workgroup records the chip's constant 100 MHz clock at four points (the time at which the last of its sixteen
// wavefronts got there), and the program prints, over the workgroups, when each point was reached, plus the time per
// call (kernel + slice reduction) of back-to-back calls that cycle through 1 GiB of weight copies.  A study tool for
// the measurements quoted in the design notes; not used by the library.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <vector>
#include <algorithm>
__device__ unsigned long long *g_trace;
#define MOE_DEC_STAMP_INIT unsigned long long *const dec_trace = g_trace
#define MOE_DEC_STAMP(slot) do { if ((threadIdx.x & 63) == 0 && dec_trace) atomicMax(&dec_trace[blockIdx.x * 16 + (slot)], (unsigned long long)wall_clock64()); } while (0)
#include "../csrc/moe_ffn_decode.hip"
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)
using namespace moe;
int main(int argc, char **argv)
{
    const int T = 64, k = 2, E = 32, d = 1024, F = 4096, R = T * k;
    const size_t wbytes = (size_t)E * d * F / 2;
    const int copies = 8;
    uint8_t *w1, *w2; CK(hipMalloc(&w1, wbytes * copies)); CK(hipMalloc(&w2, wbytes * copies));
    CK(hipMemset(w1, 0x77, wbytes * copies)); CK(hipMemset(w2, 0x88, wbytes * copies));
    std::vector<uint16_t> hx((size_t)T * d, 0x3c00), hs((size_t)E * F, 0x3c00);
    std::vector<int32_t> gi(R); std::vector<float> gs(R, 0.5f);
    srand(1);
    for (int t = 0; t < T; ++t) { int a = rand() % E, b = rand() % E; if (b == a) b = (a + 1) % E; gi[2 * t] = a; gi[2 * t + 1] = b; }
    uint16_t *x, *s1, *s2; float *partial; int32_t *gidx, *ps, *ip, *of; float *gsc, *out; unsigned *sync; unsigned long long *trace;
    CK(hipMalloc(&x, hx.size() * 2)); CK(hipMemcpy(x, hx.data(), hx.size() * 2, hipMemcpyHostToDevice));
    CK(hipMalloc(&s1, hs.size() * 2)); CK(hipMemcpy(s1, hs.data(), hs.size() * 2, hipMemcpyHostToDevice));
    CK(hipMalloc(&s2, (size_t)E * d * 2)); CK(hipMemcpy(s2, hs.data(), (size_t)E * d * 2, hipMemcpyHostToDevice));
    CK(hipMalloc(&partial, (size_t)(F / 512) * R * d * 4)); CK(hipMalloc(&gidx, R * 4)); CK(hipMemcpy(gidx, gi.data(), R * 4, hipMemcpyHostToDevice));
    CK(hipMalloc(&gsc, R * 4)); CK(hipMemcpy(gsc, gs.data(), R * 4, hipMemcpyHostToDevice));
    CK(hipMalloc(&out, (size_t)T * d * 4)); CK(hipMalloc(&ps, R * 4)); CK(hipMalloc(&ip, R * 4)); CK(hipMalloc(&of, (E + 1) * 4));
    CK(hipMalloc(&sync, 2048)); CK(hipMemset(sync, 0, 2048));
    CK(hipMalloc(&trace, 256 * 16 * 8)); CK(hipMemset(trace, 0, 256 * 16 * 8));
    DecodeArgs p{};
    p.x = x; p.gate_idx = gidx; p.gate_scale = gsc; p.n_assign = R; p.gate_k = k; p.E = E; p.d = d; p.F = F; p.act = 0;
    p.s1 = (const __half *)s1; p.s2 = (const __half *)s2; p.partial = partial; p.out = out;
    p.perm_src_out = ps; p.inv_perm_out = ip; p.offsets_out = of; 
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    unsigned long long *null_trace = nullptr;
    CK(hipMemcpyToSymbol(HIP_SYMBOL(g_trace), &null_trace, sizeof(null_trace)));
    auto launch = [&](int i) { p.w1 = w1 + (size_t)(i % copies) * wbytes; p.w2 = w2 + (size_t)(i % copies) * wbytes; if (launch_decode_ffn(p, 4, 0)) { fprintf(stderr, "%s\n", error_buffer()); exit(1); } };
    for (int i = 0; i < 10; ++i) launch(i);
    CK(hipDeviceSynchronize());
    const int reps = 40;
    CK(hipEventRecord(e0));
    for (int i = 0; i < reps; ++i) launch(i);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    printf("decode kernel, back to back: %.2f us per launch (%.0f GB/s on %.1f MB)\n", ms / reps * 1e3, 2.0 * wbytes / (ms / reps * 1e-3) / 1e9, 2.0 * wbytes / 1e6);
    // one traced launch
    CK(hipMemcpyToSymbol(HIP_SYMBOL(g_trace), &trace, sizeof(trace)));
    CK(hipMemset(trace, 0, 256 * 16 * 8));
    launch(3);
    CK(hipDeviceSynchronize());
    std::vector<unsigned long long> tr(256 * 16);
    CK(hipMemcpy(tr.data(), trace, tr.size() * 8, hipMemcpyDeviceToHost));
    unsigned long long t0 = ~0ull;
    for (int b = 0; b < 256; ++b) if (tr[b * 16]) t0 = std::min(t0, tr[b * 16]);
    const char *names[16] = {"start", "rows staged", "fc1 done, h in LDS", "fc2 done", "", "", "", "end",
                             "", "", "", "", "", "", "", ""};
    const int order[5] = {0, 1, 2, 3, 7};
    for (int oi = 0; oi < 5; ++oi) { const int s = order[oi];
        std::vector<double> v;
        for (int b = 0; b < 256; ++b) if (tr[b * 16 + s]) v.push_back((tr[b * 16 + s] - t0) * 0.01);   // 100 MHz clock -> us
        if (v.empty()) continue;
        std::sort(v.begin(), v.end());
        printf("  %-24s min %.2f  median %.2f  max %.2f us  (%zu workgroups)\n", names[s], v.front(), v[v.size() / 2], v.back(), v.size());
    }
    return 0;
}
