// Weight-streaming grouped GEMM with fused dequantisation, for experts with few rows (the
// decoder-like, bandwidth-bound case the paper measures in Table 1: ~40 tokens spread over
// up to 32 experts; Sec. 3.3, Sec. 3.4).
//
// The job is to pull every active expert's packed weights through the chip once, at HBM
// speed; the arithmetic is small.  A wavefront owns whole 32-channel slabs of one expert (or a
// quarter of the K range of one).  Thanks to the [slab][k-block] order of the packed layout its
// weight stream is one contiguous range, read with sixteen 16-byte-per-lane loads (16 KB per
// wavefront) in flight.  The few activation rows of the expert are staged once per block in LDS,
// for the whole K range, and are the MFMA A operand; the weights go from registers through the
// magic-number conversion into the B operand and never touch LDS.  Experts with more rows than a
// block holds take further row groups (grid.z), which stream the same weights again.
//
// Two kernels: stream_gemm_kernel (any K that is a multiple of 16 fragment blocks: a loop over
// runs of 16 blocks) and stream_unrolled_kernel (slabs of at most 64 blocks: straight-line code,
// ring refilled block by block).
#include <type_traits>

#include "moe_ffn_common.h"

namespace moe {

constexpr int kRing = 16;             // weight fragment blocks in flight per wavefront
constexpr int kStreamLds = 72 * 1024;  // LDS per block for an expert's activation rows (2 blocks per CU)
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

// One 16-byte weight load of the ring.  The weights of a launch are read once and are many times the
// L2: loaded as non-temporal they leave it first, so the small arrays every block starts from (gate
// indices, offsets, activation rows) and the gate's inputs of the next step stay cached (decode
// workload: 45.8 -> 43.6 us per step).
__device__ inline uint4 ring_load(const uint4 *p)
{
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

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
    int e_lo, e_hi;
    expert_range(p.offsets, e, p.R, &e_lo, &e_hi);
    const int m = e_hi - e_lo;
    if (m <= 0 || (int)blockIdx.z * fit >= m) return;   // same for the whole block
    const int lo = e_lo + blockIdx.z * fit;
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
    // The first run of weight blocks is requested once the rows are on their way into LDS, not before:
    // the load counter is in order, so rows requested behind 16 KB of weights per wavefront would be
    // waited for until all of those have arrived.
    uint4 Wn[kRing];                                    // the run in flight
    if (nblk) {
#pragma unroll
        for (int i = 0; i < kRing; ++i) Wn[i] = ring_load(wbase + (size_t)i * 64);
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
                for (int i = 0; i < kRing; ++i) Wn[i] = ring_load(wnext + (size_t)i * 64);
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
            v = activate(v, p.act);
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
    // (a function-local static is initialised once, also when several threads call)
    static const hipError_t raised = hipFuncSetAttribute(reinterpret_cast<const void *>(&stream_gemm_kernel<BITS>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, kStreamLds);
    (void)raised;                               // a refusal shows up as the launch's error
    hipLaunchKernelGGL((stream_gemm_kernel<BITS>), grid, dim3(256), kStreamLds, s, p, tpw);
}

// ---- straight-line variant for slabs of at most 64 fragment blocks ------------------------------
// With the K extent a compile-time constant the whole job of a wavefront (TPW slabs of KB blocks)
// is unrolled into one basic block.  The ring of kRing loads is then refilled block by block: the
// slot of the block just consumed is reloaded with the block kRing ahead, and because there is no
// loop edge the compiler's wait before block b is "all but the 15 youngest loads", i.e. only the
// load that block needs.  Every wavefront computes as its data trickles in, and the last wait of
// the kernel is for a single block.
constexpr int kStageVecs = 16;         // 16-byte vectors of activation rows one thread stages (at most)
constexpr int kUnrolledFitCap = 16;    // rows per block: 16 rows of K = 1024 leave LDS for several blocks per CU
// vectors one thread stages for a K extent: all of kUnrolledFitCap rows, but no more than kStageVecs
__host__ __device__ constexpr int stage_vecs(int K) { return kUnrolledFitCap * (K / 8) / 256 < kStageVecs ? kUnrolledFitCap * (K / 8) / 256 : kStageVecs; }

// out[a / out_div][n] += out_scale[a] * v for permuted row r, a = out_dst[r] (hardware fp32 add, no return value)
__device__ inline void add_to_token(const GemmArgs &p, int r, int n, float v)
{
    const int a = p.out_dst[r];
    unsafeAtomicAdd(reinterpret_cast<float *>(p.out) + (size_t)(a / p.out_div) * p.N + n, v * p.out_scale[a]);
}

//
// KS = 4 splits the K range of a slab over the four wavefronts of the block (a slab of 64 blocks
// would otherwise be one long, latency-bound stream per wavefront while most of the chip idles):
// each wavefront accumulates a quarter of K, the four partial tiles meet in LDS and are added in a
// fixed order.  With TPW = 2 the block does this for two slabs in turn and keeps both accumulator
// tiles until the end, because the partial tiles take the LDS space of the rows.
//
// BITS = 16 streams unquantised fp16 weights in the same fragment layout (one MFMA step per block;
// the denominator of the Table 1 comparison).  NATIVE replaces the magic-number conversion by the
// chip's integer-to-float conversion instructions (the variant Sec. 3.4.1 found too slow on its
// hardware; kept for that comparison only).
//
// PERM (decode-sized batches, at most 256 assignments): the launch takes the gate's expert indices
// instead of a permuted copy of the rows.  Every block counts, with two ballots per wavefront, the
// assignments of its expert and of the experts before it (the stable sort of Sec. 3.3 restricted to
// what this block needs), fetches its rows straight from the tokens, and the first block of each
// expert writes that expert's part of perm_src, inv_perm and expert_offsets for the launches after
// this one.  Pruned rows (index E) are numbered behind the active ones by the last expert's block.
template <int BITS, int KB, int TPW, int KS, bool NATIVE = false, bool PERM = false>
__global__ __launch_bounds__(256, 2) void stream_unrolled_kernel(GemmArgs p, int fit)
{
    constexpr int STEPS = BITS == 4 ? 4 : BITS == 8 ? 2 : 1;
    constexpr int FK = BITS == 4 ? 64 : BITS == 8 ? 32 : 16;
    constexpr int K = KB * FK;
    constexpr int KBW = KB / KS;                        // fragment blocks of a slab one wavefront streams
    constexpr int TOT = KBW * TPW;
    constexpr int VPR = K / 8;                          // 16-byte vectors per row
    constexpr int LDR = K + kRowPad;
    extern __shared__ __align__(16) uint16_t lds_a[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int e = blockIdx.y, z = blockIdx.z;
    const int N = p.N;
    int e_lo, e_hi;
    __shared__ int s_cnt[3][4];                 // per wavefront: assignments of this expert, of earlier experts, pruned
    __shared__ int s_tok[kUnrolledFitCap];      // token of each row of this block
    if constexpr (PERM) {
        if (p.zero_out) {                       // every block clears its share of the buffer the next launch adds into
            const long nblk = (long)gridDim.x * gridDim.y * gridDim.z;
            const long blk = ((long)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
            float4 *z4 = reinterpret_cast<float4 *>(p.zero_out);
            for (long i = blk * 256 + threadIdx.x; i < p.zero_count / 4; i += nblk * 256) z4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        const int a = threadIdx.x;
        const int v = a < p.n_assign ? p.gate_idx[a] : 0x7fffffff;
        const bool mine = v == e, before = v < e, pruned = v == p.E;
        const uint64_t m_mine = __ballot(mine), m_before = __ballot(before), m_pruned = __ballot(pruned);
        if (lane == 0) {
            s_cnt[0][wave] = __popcll(m_mine);
            s_cnt[1][wave] = __popcll(m_before);
            s_cnt[2][wave] = __popcll(m_pruned);
        }
        __syncthreads();
        int first = 0, count = 0, lower = 0, pruned_first = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave) { first += s_cnt[0][w]; pruned_first += s_cnt[2][w]; }
            count += s_cnt[0][w];
            lower += s_cnt[1][w];
        }
        const uint64_t below = (1ull << lane) - 1;
        const int rank = first + __popcll(m_mine & below);           // stable: assignments in ascending order
        e_lo = lower;
        e_hi = lower + count;
        if (blockIdx.x == 0 && z == 0) {
            if (threadIdx.x == 0) {
                p.offsets_out[e] = lower;
                if (e == p.E - 1) p.offsets_out[p.E] = lower + count;   // = the active rows
            }
            if (mine) {
                p.inv_perm_out[a] = lower + rank;
                p.perm_src_out[lower + rank] = a;
            }
            if (pruned && e == p.E - 1) {
                const int r = lower + count + pruned_first + __popcll(m_pruned & below);
                p.inv_perm_out[a] = r;
                p.perm_src_out[r] = a;
            }
        }
        if (mine && rank >= z * fit && rank < z * fit + fit) s_tok[rank - z * fit] = a / p.gate_k;
        __syncthreads();
    } else {
        expert_range(p.offsets, e, p.R, &e_lo, &e_hi);
    }
    const int m = e_hi - e_lo;
    if (m <= 0 || z * fit >= m) return;   // same for the whole block
    const int lo = e_lo + z * fit;
    const int rows = min(fit, m - z * fit);
    const int ntiles = N / 32;
    const int tile0 = KS == 1 ? (blockIdx.x * 4 + wave) * TPW : blockIdx.x * TPW;
    const int kq = KS == 1 ? 0 : wave;                  // this wavefront's part of K
    const bool has = tile0 < ntiles;                    // ntiles is a multiple of TPW: all slabs or none
    const int t0c = has ? tile0 : 0;
    const uint4 *wbase = reinterpret_cast<const uint4 *>(p.wq + (size_t)e * packed_bytes_per_expert(K, N, BITS) +
                                                         ((size_t)t0c * KB + kq * KBW) * kFragBytes) + lane;
    // block b of this wavefront's stream, in fragment blocks from wbase
    auto wofs = [](int b) { return (size_t)((b / KBW) * KB + b % KBW) * 64; };

    // activation rows first (they are small and everything waits for them), then the scales, then
    // the first ring of weights, in exactly this order: the scheduler barriers keep the compiler
    // from moving the small loads behind the ring or shuffling the ring's order
    const int total = rows * VPR;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 *a_vec = reinterpret_cast<const u32x4 *>(p.a + (PERM ? 0 : (size_t)lo * K));
    constexpr int NA = stage_vecs(K) < 1 ? 1 : stage_vecs(K);
    u32x4 av[NA];
    static_for<0, NA>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        const int idx = min(j * 256 + (int)threadIdx.x, total - 1);
        if constexpr (PERM) av[j] = a_vec[(size_t)s_tok[idx / VPR] * VPR + idx % VPR];   // row idx / VPR of the block is a token's row
        else av[j] = a_vec[idx];
    });
    float cs[TPW], bias[TPW];
    const __half *bias_or_scale = p.bias ? p.bias : BITS == 16 ? reinterpret_cast<const __half *>(p.wq) : p.scales;   // no branch around a load
    const float bias_on = p.bias ? 1.0f : 0.0f;
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        const int n = (t0c + t) * 32 + (lane & 31);
        cs[t] = BITS == 16 ? 1.0f : __half2float(p.scales[(size_t)e * N + n]);
        bias[t] = __half2float(bias_or_scale[(size_t)e * N + n]) * bias_on;
    }
    __builtin_amdgcn_sched_barrier(0);
    uint4 W[kRing];
    static_for<0, kRing>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        W[i] = ring_load(wbase + wofs(i));
        __builtin_amdgcn_sched_barrier(0);
    });
    // vectors past the live rows (clamped reads above) land in a per-thread dump slot behind the rows
    uint16_t *dump = lds_a + max(fit * LDR, KS == 4 ? TPW * 4 * 16 * 64 * 2 : 0) + threadIdx.x * 8;
    static_for<0, NA>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        const int idx = j * 256 + (int)threadIdx.x;
        uint16_t *dst = idx < total ? lds_a + (idx / VPR) * LDR + (idx % VPR) * 8 : dump;
        *reinterpret_cast<u32x4 *>(dst) = av[j];
    });
    __syncthreads();
    if (!has) return;

    // fused un-permute (KS = 4): the destinations and gate scales of the four rows this lane will
    // finish are fetched now, under the weight stream, not at the end of the kernel
    int dst_tok[4];
    float dst_scale[4];
    if (KS == 4 && p.out_add) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int a = p.out_dst[lo + min(4 * (lane >> 5) + 8 * wave + i, rows - 1)];
            dst_tok[i] = a / p.out_div;
            dst_scale[i] = p.out_scale[a];
        }
    }
    const uint16_t *arow = lds_a + (size_t)min(lane & 31, rows - 1) * LDR + 8 * (lane >> 5) +
                           kq * KBW * FK;               // clamped to a live row
    float *part = reinterpret_cast<float *>(lds_a);    // KS = 4: [slab][wave][16][64] partial tiles, over the rows once they are used up
    uint4 A[2][STEPS];
    // KS = 4 keeps one accumulator tile per slab until the end: the partial tiles meet in the LDS
    // space of the activation rows, which every slab still needs
    constexpr int NACC = KS == 4 ? TPW : 1;
    float16_t accs[NACC];
#pragma unroll
    for (int a = 0; a < NACC; ++a)
#pragma unroll
        for (int i = 0; i < 16; ++i) accs[a][i] = 0.0f;
    void *out_rows = reinterpret_cast<char *>(p.out) + (size_t)lo * N * (p.out_dtype == MOE_F32 ? 4 : 2);
    auto fetch_a = [&](int slot, int kb) {
#pragma unroll
        for (int j = 0; j < STEPS; ++j) A[slot][j] = *reinterpret_cast<const uint4 *>(arow + kb * FK + 16 * j);
    };
    fetch_a(0, 0);
    static_for<0, TOT>([&](auto bc) {
        constexpr int b = decltype(bc)::value;
        constexpr int kb = b % KBW, sl = b / KBW;
        __builtin_amdgcn_sched_barrier(0);
        if (b + 1 < TOT) fetch_a((b + 1) & 1, (b + 1) % KBW);
        const uint32_t raw[4] = {W[b % kRing].x, W[b % kRing].y, W[b % kRing].z, W[b % kRing].w};
#pragma unroll
        for (int j = 0; j < STEPS; ++j) {
            uint32_t bw[4];
            if (BITS == 16) { bw[0] = raw[0]; bw[1] = raw[1]; bw[2] = raw[2]; bw[3] = raw[3]; }
            else if (NATIVE && BITS == 4) dequant4_native(raw[j], bw);
            else if (NATIVE) dequant8_native(raw[2 * j], raw[2 * j + 1], bw);
            else if (BITS == 4) dequant4(raw[j], bw);
            else dequant8(raw[2 * j], raw[2 * j + 1], bw);
            float16_t &acc = accs[KS == 4 ? sl : 0];
            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, A[b & 1][j]), frag_from(bw), acc, 0,
                                                         0, 0);
        }
        if (b + kRing < TOT) W[b % kRing] = ring_load(wbase + wofs(b + kRing));
        if (kb == KBW - 1) {
            // slab finished: per-channel scale, bias, ReLU, store the live rows
            const int n = (tile0 + sl) * 32 + (lane & 31);
            const int rbase = 4 * (lane >> 5);
            if constexpr (KS == 1) {
                float16_t &acc = accs[0];
                float v[16];
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    v[q] = acc[q] * cs[sl] + bias[sl];
                    v[q] = activate(v[q], p.act);
                    acc[q] = 0.0f;
                }
                auto put = [&](auto *out) {             // rows rbase+0..3, +8..11, +16..19, +24..27
                    size_t o = (size_t)rbase * N + n;
#pragma unroll
                    for (int q = 0; q < 16; ++q) {
                        if (rbase + 8 * (q >> 2) + (q & 3) < rows) {
                            if constexpr (std::is_same<decltype(out), uint16_t *>::value) out[o] = to_bf16_rne(v[q]);
                            else out[o] = (std::remove_pointer_t<decltype(out)>)v[q];
                        }
                        o += (q & 3) == 3 ? (size_t)5 * N : (size_t)N;
                    }
                };
                if (p.out_add) {                        // fused un-permute: scaled rows added to their tokens' rows
#pragma unroll
                    for (int q = 0; q < 16; ++q) {
                        const int r = rbase + 8 * (q >> 2) + (q & 3);
                        if (r < rows) add_to_token(p, lo + r, n, v[q]);
                    }
                }
                else if (p.out_dtype == MOE_F16) put(reinterpret_cast<_Float16 *>(out_rows));
                else if (p.out_dtype == MOE_F32) put(reinterpret_cast<float *>(out_rows));
                else put(reinterpret_cast<uint16_t *>(out_rows));
            } else if constexpr (sl == TPW - 1) {
                // after the last slab the four K-quarters of every slab meet in LDS; wavefront w then
                // finishes accumulator registers 4w..4w+3 (rows rbase + 8w + 0..3) of each slab,
                // adding the quarters in the order 0, 1, 2, 3
                __syncthreads();                        // every wavefront is done with the rows
#pragma unroll
                for (int a = 0; a < TPW; ++a)
#pragma unroll
                    for (int q = 0; q < 16; ++q) part[((a * 4 + wave) * 16 + q) * 64 + lane] = accs[a][q];
                __syncthreads();
#pragma unroll
                for (int a = 0; a < TPW; ++a) {
                    const int na = (tile0 + a) * 32 + (lane & 31);
                    float v[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float *src = part + (a * 4 * 16 * 64 + (wave * 4 + i) * 64 + lane);
                        v[i] = ((src[0] + src[16 * 64]) + src[2 * 16 * 64]) + src[3 * 16 * 64];
                        v[i] = v[i] * cs[a] + bias[a];
                        v[i] = activate(v[i], p.act);
                    }
                    auto put = [&](auto *out) {
                        size_t o = (size_t)(rbase + 8 * wave) * N + na;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            if (rbase + 8 * wave + i < rows) {
                                if constexpr (std::is_same<decltype(out), uint16_t *>::value) out[o] = to_bf16_rne(v[i]);
                                else out[o] = (std::remove_pointer_t<decltype(out)>)v[i];
                            }
                            o += N;
                        }
                    };
                    if (p.out_add) {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (rbase + 8 * wave + i < rows)
                                unsafeAtomicAdd(reinterpret_cast<float *>(p.out) + (size_t)dst_tok[i] * N + na, v[i] * dst_scale[i]);
                    }
                    else if (p.out_dtype == MOE_F16) put(reinterpret_cast<_Float16 *>(out_rows));
                    else if (p.out_dtype == MOE_F32) put(reinterpret_cast<float *>(out_rows));
                    else put(reinterpret_cast<uint16_t *>(out_rows));
                }
            }
        }
    });
}

template <int BITS, int KB, int TPW, int KS, bool NATIVE = false, bool PERM = false>
static void launch_unrolled(const GemmArgs &p, int fit, int max_rows, hipStream_t s)
{
    constexpr int K = KB * (BITS == 4 ? 64 : BITS == 8 ? 32 : 16);
    // rows (KS = 4: or the partial tiles that later replace them) + the staging dump slots
    int lds = fit * (K + kRowPad) * 2;
    if (KS == 4 && lds < TPW * 4 * 16 * 64 * 4) lds = TPW * 4 * 16 * 64 * 4;
    lds += 256 * 16;
    static const hipError_t raised = hipFuncSetAttribute(reinterpret_cast<const void *>(&stream_unrolled_kernel<BITS, KB, TPW, KS, NATIVE, PERM>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
    (void)raised;
    const int ntiles = p.N / 32;
    const int per_block = KS == 1 ? 4 * TPW : TPW;
    dim3 grid((ntiles + per_block - 1) / per_block, p.E, (max_rows + fit - 1) / fit);
    hipLaunchKernelGGL((stream_unrolled_kernel<BITS, KB, TPW, KS, NATIVE, PERM>), grid, dim3(256), lds, s, p, fit);
}

// Rows per block of the straight-line kernel: what one staging pass (kStageVecs vectors per
// thread) and 64 KB of LDS hold.
static int unrolled_fit_rows(int K, int max_rows)
{
    const int na = stage_vecs(K) < 1 ? 1 : stage_vecs(K);
    int fit = na * 256 / (K / 8);
    if (fit > kUnrolledFitCap) fit = kUnrolledFitCap;
    if (fit > max_rows) fit = max_rows;
    return fit < 1 ? 1 : fit;
}

bool stream_unrolled_supports(int K, int bits, int smode)
{
    const int fk = bits == 4 ? 64 : bits == 8 ? 32 : 16;
    return smode == SCALE_CHANNEL && K % (fk * kRing) == 0 && K / fk <= 64;
}

int stream_unrolled_fit(int K, int max_rows) { return unrolled_fit_rows(K, max_rows); }

// Slab lengths for which the straight-line kernel is also built with the permutation inside.
bool stream_unrolled_takes_gate(int K, int bits)
{
    const int kb = K / (bits == 4 ? 64 : 32);
    return (bits == 4 || bits == 8) && K % (bits == 4 ? 64 : 32) == 0 && (kb == 16 || kb == 32);
}

// The Table 1 variants: fp16 weights (bits = 16) and the native integer-to-float conversion.
int launch_stream_unrolled_variant(const GemmArgs &p, int bits, bool native, int max_rows, hipStream_t s)
{
    const int kb = p.K / (bits == 4 ? 64 : bits == 8 ? 32 : 16);
    const int fit = unrolled_fit_rows(p.K, max_rows);
    if (p.E > 65535) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_wq: E=%d exceeds one launch", p.E);
    if (bits == 16 && kb == 64 && !native) launch_unrolled<16, 64, 1, 4>(p, fit, max_rows, s);
    else if (bits == 16 && kb == 32 && !native) launch_unrolled<16, 32, 1, 1>(p, fit, max_rows, s);
    else if (bits == 16 && kb == 16 && !native) launch_unrolled<16, 16, 1, 1>(p, fit, max_rows, s);
    else if (bits == 4 && kb == 16 && native) launch_unrolled<4, 16, 1, 1, true>(p, fit, max_rows, s);
    else if (bits == 8 && kb == 32 && native) launch_unrolled<8, 32, 1, 1, true>(p, fit, max_rows, s);
    else return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_wq: no kernel for bits=%d K=%d convert=%d", bits, p.K, (int)native);
    return check_launch("moe_grouped_gemm_wq");
}

int launch_stream_unrolled(const GemmArgs &p, int bits, int max_rows, hipStream_t s)
{
    const int kb = p.K / (bits == 4 ? 64 : 32);
    const int fit = unrolled_fit_rows(p.K, max_rows);
    if (p.E > 65535) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq: E=%d exceeds one launch", p.E);
    // 16 blocks: one slab per wavefront; 64 blocks: K split over the block's wavefronts, two slabs per
    // block (LDS holds two such blocks per CU: with one slab each the launch would need two rounds
    // of blocks on the decode workload's fc2); every entry point takes N in multiples of 64 only
    if (kb == 64 && (p.N / 32) % 2) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq: N=%d is not a multiple of 64", p.N);
    if (p.gate_idx) {                           // permutation rebuilt inside the launch
        if (p.n_assign > kGatedMaxAssign || !stream_unrolled_takes_gate(p.K, bits))
            return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq_gated: no kernel for K=%d bits=%d with %d assignments", p.K, bits, p.n_assign);
        if (bits == 4 && kb == 16) launch_unrolled<4, 16, 1, 1, false, true>(p, fit, max_rows, s);
        else if (bits == 4) launch_unrolled<4, 32, 1, 1, false, true>(p, fit, max_rows, s);
        else if (kb == 16) launch_unrolled<8, 16, 1, 1, false, true>(p, fit, max_rows, s);
        else launch_unrolled<8, 32, 1, 1, false, true>(p, fit, max_rows, s);
        return check_launch("moe_grouped_ffn_wq_gated (straight-line streaming gemm)");
    }
    if (bits == 4) {
        if (kb == 16) launch_unrolled<4, 16, 1, 1>(p, fit, max_rows, s);
        else if (kb == 32) launch_unrolled<4, 32, 1, 1>(p, fit, max_rows, s);
        else if (kb == 48) launch_unrolled<4, 48, 1, 1>(p, fit, max_rows, s);
        else launch_unrolled<4, 64, 2, 4>(p, fit, max_rows, s);
    } else {
        if (kb == 16) launch_unrolled<8, 16, 1, 1>(p, fit, max_rows, s);
        else if (kb == 32) launch_unrolled<8, 32, 1, 1>(p, fit, max_rows, s);
        else if (kb == 48) launch_unrolled<8, 48, 1, 1>(p, fit, max_rows, s);
        else launch_unrolled<8, 64, 2, 4>(p, fit, max_rows, s);
    }
    return check_launch("moe_grouped_ffn_wq (straight-line streaming gemm)");
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
    // row groups: no expert has more than max_rows rows
    const int fit = stream_fit_rows(p.K);
    dim3 grid((ntiles + 4 * tpw - 1) / (4 * tpw), p.E, (max_rows + fit - 1) / fit);
    if (bits == 4) launch_stream<4>(p, tpw, grid, s);
    else launch_stream<8>(p, tpw, grid, s);
    return check_launch("moe_grouped_ffn_wq (streaming gemm)");
}

}  // namespace moe
