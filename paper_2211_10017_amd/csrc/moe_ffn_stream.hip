// Weight-streaming grouped GEMM with fused dequantisation, for experts with few rows (the
// decoder-like, bandwidth-bound case the paper measures in Table 1: ~40 tokens spread over
// up to 32 experts; Sec. 3.3, Sec. 3.4).
//
// The job is to pull every active expert's packed weights through the chip once, at HBM
// speed; the arithmetic is small.  A wavefront owns `tpw` consecutive 32-channel slabs of one
// expert.  Thanks to the [slab][k-block] order of the packed layout its whole weight stream is
// one contiguous range, read through a ring of sixteen 16-byte-per-lane loads (16 KB per
// wavefront always in flight): as soon as a fragment block has been unpacked, its ring slot is
// refilled with the block 16 ahead.  The few activation rows are the MFMA A operand; each lane
// reads its 8 consecutive K values directly (they are shared by all wavefronts of the expert
// and stay in L1/L2), prefetched a few blocks ahead.  No LDS, no barriers.
#include <type_traits>

#include "moe_ffn_common.h"

namespace moe {

constexpr int kRing = 16;             // weight fragment blocks in flight per wavefront
#ifndef MOE_STREAM_LDS_KB
#define MOE_STREAM_LDS_KB 72
#endif
constexpr int kStreamLds = MOE_STREAM_LDS_KB * 1024;  // LDS per block for an expert's activation rows (2 blocks per CU)
constexpr int kRowPad = 8;             // halfs of padding per LDS row: rows start 4 banks apart

// Rows of one expert that fit in LDS together, for the whole K range (at most one 32-row tile).
__host__ __device__ inline int stream_fit_rows(int K)
{
    const int r = kStreamLds / (2 * (K + kRowPad));
    return r < 32 ? r : 32;
}

template <int I, int N, class F>
__device__ inline void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

constexpr int kStreamMaxTpw = 4;       // slabs per wavefront (their scales are fetched up front)

template <int BITS>
__global__ __launch_bounds__(256, 2) void stream_gemm_kernel(GemmArgs p, int tpw)
{
    constexpr int STEPS = BITS == 4 ? 4 : 2;          // MFMA steps per fragment block
    constexpr int FK = BITS == 4 ? 64 : 32;           // K values per fragment block
    extern __shared__ __align__(16) uint16_t lds_a[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: scalar control flow below
    const int e = blockIdx.y;
    const int K = p.K, N = p.N;
    const int fit = stream_fit_rows(K);
    // blockIdx.z picks the group of `fit` rows (all rows at once for the few-row experts this
    // kernel is meant for; every further group streams the expert's weights again)
    const int m = p.offsets[e + 1] - p.offsets[e];
    if (m <= 0 || m > p.row_hi || (int)blockIdx.z * fit >= m) return;   // same for the whole block
    const int lo = p.offsets[e] + blockIdx.z * fit;
    const int rows = min(fit, m - (int)blockIdx.z * fit);
    const int KB = K / FK;                              // fragment blocks per slab, a multiple of kRing
    const int ntiles = N / 32;
    const int tile0 = (blockIdx.x * 4 + wave) * tpw;
    const int ntile = max(min(tpw, ntiles - tile0), 0); // 0: this wavefront has no slab (it still helps staging)
    const int t0c = min(tile0, ntiles - 1);
    const int nblk = ntile * KB;
    const int ldr = K + kRowPad;
    const uint4 *wbase = reinterpret_cast<const uint4 *>(p.wq + (size_t)e * packed_bytes_per_expert(K, N, BITS) +
                                                         (size_t)t0c * KB * kFragBytes) + lane;

    // the first run of weight blocks is requested before anything else, so that it is in flight
    // while the rows are staged
    uint4 Wn[kRing];                                    // the run in flight
    if (nblk) {
#pragma unroll
        for (int i = 0; i < kRing; ++i) Wn[i] = wbase[(size_t)i * 64];
    }
    // per-channel scale and bias of this wavefront's slabs (fetched now: a compiler-issued load
    // inside the ring loop would be waited for with vmcnt(0) and drain the ring)
    float cs[kStreamMaxTpw], bias[kStreamMaxTpw];
#pragma unroll
    for (int t = 0; t < kStreamMaxTpw; ++t) {
        const int n = min(t0c + t, ntiles - 1) * 32 + (lane & 31);
        cs[t] = __half2float(p.scales[(size_t)e * N + n]);
        bias[t] = p.bias ? __half2float(p.bias[(size_t)e * N + n]) : 0.0f;
    }
    // the block copies the rows into LDS; every wavefront then reads its MFMA A fragments there
    {
        const int vpr = K / 8;                          // 16-byte vectors per row
        const uint16_t *a_rows = p.a + (size_t)lo * K;
        for (int r = 0; r < rows; ++r)
            for (int col = threadIdx.x; col < vpr; col += 256)
                *reinterpret_cast<uint4 *>(lds_a + r * ldr + col * 8) =
                    *reinterpret_cast<const uint4 *>(a_rows + (size_t)r * K + col * 8);
    }
    __syncthreads();
    if (nblk == 0) return;

    const uint16_t *arow = lds_a + (size_t)min(lane & 31, rows - 1) * ldr + 8 * (lane >> 5);   // clamped to a live row
    uint4 A[2][STEPS];
    float16_t acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
    const uint4 *wnext = wbase + (size_t)kRing * 64;    // next block to fetch into the ring
    void *out_rows = reinterpret_cast<char *>(p.out) + (size_t)lo * N * (p.out_dtype == MOE_F32 ? 4 : 2);

#pragma unroll
    for (int sl = 0; sl < kStreamMaxTpw; ++sl) {
        if (sl >= ntile) break;
        auto fetch_a = [&](int slot, int kb) {          // MFMA A fragments of k-block kb
#pragma unroll
            for (int j = 0; j < STEPS; ++j)
                A[slot][j] = *reinterpret_cast<const uint4 *>(arow + kb * FK + 16 * j);
        };
        // One run = kRing fragment blocks (16 KB per wavefront).  The run that has arrived is moved
        // to Wc and, before any of it is unpacked, all loads of the next run are issued: they are
        // in flight for the whole time this run takes to compute.  (A finer-grained ring, refilled
        // block by block, does not survive the compiler: it waits for every outstanding load at
        // each loop boundary, so the blocks requested last are always waited for in full.)
        for (int kb0 = 0; kb0 < KB; kb0 += kRing) {
            uint4 Wc[kRing];
#pragma unroll
            for (int i = 0; i < kRing; ++i) Wc[i] = Wn[i];
            if (sl * KB + kb0 + 2 * kRing <= nblk) {
#pragma unroll
                for (int i = 0; i < kRing; ++i) Wn[i] = wnext[(size_t)i * 64];
                wnext += (size_t)kRing * 64;
            }
            fetch_a(0, kb0);
#pragma unroll
            for (int i = 0; i < kRing; ++i) {
                __builtin_amdgcn_sched_barrier(0);      // keep each block's work together: short live ranges
                // the next block's fragments are fetched from LDS now and used after this block's MFMAs
                if (i + 1 < kRing) fetch_a((i + 1) & 1, kb0 + i + 1);
                const uint32_t raw[4] = {Wc[i].x, Wc[i].y, Wc[i].z, Wc[i].w};
#pragma unroll
                for (int j = 0; j < STEPS; ++j) {
                    uint32_t bw[4];
                    if (BITS == 4) dequant4(raw[j], bw);
                    else dequant8(raw[2 * j], raw[2 * j + 1], bw);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, A[i & 1][j]),
                                                                 frag_from(bw), acc, 0, 0, 0);
                }
            }
        }
        // slab finished: per-channel scale, bias, ReLU, store the live rows
        const int n = (tile0 + sl) * 32 + (lane & 31);
        const int rbase = 4 * (lane >> 5);
        size_t o = (size_t)rbase * N + n;               // element offset of this lane's first row
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int rl = rbase + 8 * (q >> 2) + (q & 3);
            float v = acc[q] * cs[sl] + bias[sl];
            if (p.relu) v = fmaxf(v, 0.0f);
            acc[q] = 0.0f;
            if (rl < rows) {
                if (p.out_dtype == MOE_F16) reinterpret_cast<_Float16 *>(out_rows)[o] = (_Float16)v;
                else if (p.out_dtype == MOE_F32) reinterpret_cast<float *>(out_rows)[o] = v;
                else reinterpret_cast<uint16_t *>(out_rows)[o] = to_bf16_rne(v);
            }
            o += (q & 3) == 3 ? (size_t)5 * N : (size_t)N;      // rows rbase+0..3, +8..11, +16..19, +24..27
        }
    }
}

template <int BITS>
static void launch_stream(const GemmArgs &p, int tpw, dim3 grid, hipStream_t s)
{
    // more than 64 KB of dynamic LDS has to be asked for once per kernel
    static bool raised = false;
    if (!raised) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&stream_gemm_kernel<BITS>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, kStreamLds);
        raised = true;
    }
    hipLaunchKernelGGL((stream_gemm_kernel<BITS>), grid, dim3(256), kStreamLds, s, p, tpw);
}

// The streaming kernel takes shapes whose slabs are whole rings of fragment blocks.
bool stream_gemm_supports(int K, int bits, int smode)
{
    return smode == SCALE_CHANNEL && K % ((bits == 4 ? 64 : 32) * kRing) == 0 && stream_fit_rows(K) >= 1;
}

int stream_gemm_fit_rows(int K) { return stream_fit_rows(K); }

int launch_stream_gemm(const GemmArgs &p, int bits, int smode, int max_rows, hipStream_t s)
{
    if (!stream_gemm_supports(p.K, bits, smode)) return fail(MOE_ERR_UNSUPPORTED, "streaming GEMM does not take K=%d", p.K);
    const int ntiles = p.N / 32;
    // slabs per wavefront: at least 32 KB of weights each, but keep >= ~2 wavefronts per SIMD
    const size_t slab_bytes = (size_t)p.K * 32 * bits / 8;
    int tpw = (int)((32768 + slab_bytes - 1) / slab_bytes);
    const long total = (long)p.E * ntiles;
    while (tpw > 1 && total / tpw < 2048) --tpw;
    if (tpw < 1) tpw = 1;
    if (tpw > kStreamMaxTpw) tpw = kStreamMaxTpw;
    if (p.E > 65535) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq: E=%d exceeds one launch", p.E);
    // row groups: experts handled here have at most min(row_hi, max_rows) rows
    const int fit = stream_fit_rows(p.K);
    const int most = p.row_hi < max_rows ? p.row_hi : max_rows;
    dim3 grid((ntiles + 4 * tpw - 1) / (4 * tpw), p.E, (most + fit - 1) / fit);
    if (bits == 4) launch_stream<4>(p, tpw, grid, s);
    else launch_stream<8>(p, tpw, grid, s);
    return check_launch("moe_grouped_ffn_wq (streaming gemm)");
}

}  // namespace moe
