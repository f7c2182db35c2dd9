// The expert FFN of a decode-sized batch (Sec. 3.3 steps 2-4 with the fused dequantisation of
// Sec. 3.4) in one streaming launch plus a small reduction: the stable sort by expert is rebuilt from
// the gate's output, and fc1, the activation and fc2 run in one persistent grid.
//
// Such a batch (the decoder-like case of Table 1: a few rows per expert) is bound by pulling every
// active expert's packed weights through the chip once.  The work is cut along d_ff: a workgroup
// item is (expert, 512 channels of d_ff).  Its sixteen wavefronts compute that slice of
// h = act(x W1 + b1) (one 32-channel slab of W1 each), keep it in LDS as fp16, and multiply it at
// once with the matching 512 rows of W2 (each wavefront 64 output channels): h never goes to
// memory and a wavefront's weight stream (16 KB of W1, then 16 KB of W2) runs through one ring of
// eight 16-byte-per-lane loads without a break.  What is left over is a partial sum of y per
// d_ff slice, stored as fp32 rows; decode_reduce_kernel then adds the slices in ascending order,
// applies W2's channel scale, the bias and the gate scale, and sums a token's experts in slot
// order into the layer output (no atomics, nothing to clear, nothing to wait for inside a launch).
//
// The rows of an expert (at most sixteen per pass; more rows take further passes over the same
// weights) are staged in LDS and are the A operand of v_mfma_f32_16x16x32_f16; the weights go
// from the ring through the magic-number conversion into the B operand.
#include <type_traits>

#include "moe_ffn_common.h"

// Hook for timing studies: a harness that includes this file may define these to record a time stamp
// per workgroup at the named points; the library builds them empty.
#ifndef MOE_DEC_STAMP
#define MOE_DEC_STAMP(slot)
#define MOE_DEC_STAMP_INIT
#endif

namespace moe {

constexpr int kDecWaves = 16;            // wavefronts per workgroup
constexpr int kDecThreads = kDecWaves * 64;
#ifndef MOE_DEC_RING
#define MOE_DEC_RING 8
#endif
#ifndef MOE_DEC_AUX
#define MOE_DEC_AUX 2
#endif
constexpr int kDecRing = MOE_DEC_RING;   // weight fragment blocks in flight per wavefront
constexpr int kDecFit = 16;              // rows of an expert per pass (one 16-row matrix tile)
constexpr int kDecRowPad = 8;            // halfs of padding per LDS row: rows start 4 banks apart
constexpr int kDecChunk = 32 * kDecWaves;   // channels of d_ff per item

typedef float float4_t __attribute__((ext_vector_type(4)));

template <int I, int N, class F>
__device__ inline void dec_static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        dec_static_for<I + 1, N>(f);
    }
}

// One 16-byte-per-lane load of the ring through a buffer descriptor: the descriptor (base and extent of
// the wavefront's weight stream) and the block's offset sit in scalar registers, the lane's 16 x lane
// in ONE vector register for all loads (plain pointers would cost two vector registers per block in
// flight).  Loads past the extent return zero instead of touching memory.  Non-temporal: the weights
// of a launch are read once and must not push the small hot arrays out of the caches.
typedef uint32_t dec_u32x4 __attribute__((ext_vector_type(4)));
__device__ inline __amdgpu_buffer_rsrc_t dec_stream_rsrc(const uint8_t *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(base), 0, (int)bytes, 0x00020000);
}
__device__ inline uint4 dec_ring_load(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t block_off)
{
    const dec_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, block_off, MOE_DEC_AUX /* 2 = nt */);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Rows 1 and 3 (of sixteen lanes each) of `a` change places with rows 0 and 2 of `b`.  A fragment
// block holds, per MFMA step j of the 32-row layout, [ch 0-15 | ch 16-31 | ch 0-15 | ch 16-31] x
// [k 0-7, k 0-7, k 8-15, k 8-15]; swapping steps j and j+1 this way leaves `a` with channels 0-15
// and `b` with channels 16-31, each over the four k octets {0-7, 16-23, 8-15, 24-31} of the two
// steps: the B operand of a 16x16x32 instruction whose A operand reads its k octets in that order.
__device__ inline void swap_rows(uint32_t &a, uint32_t &b)
{
    const auto r = __builtin_amdgcn_permlane16_swap(a, b, false, false);
    a = r[0];
    b = r[1];
}

// BITS: weight width.  NB1: fragment blocks of a W1 slab (its whole K range, d_model).  TS: W2 slabs per
// wavefront (d_model / 512).  NBC: fragment blocks of a W2 slab inside one d_ff slice of 512 rows.
template <int BITS, int NB1, int TS, int NBC, bool EARLY>
__global__ __launch_bounds__(kDecThreads, 1) void decode_ffn_kernel(DecodeArgs p)
{
    constexpr int FK = BITS == 4 ? 64 : 32;             // K values per fragment block
    constexpr int PAIRS = BITS == 4 ? 2 : 1;            // 32-deep MFMA steps per fragment block
    constexpr int K1 = NB1 * FK;                        // d_model
    constexpr int LDR1 = K1 + kDecRowPad, LDRH = kDecChunk + kDecRowPad;
    constexpr int VPR1 = K1 / 8;                        // 16-byte vectors per row of x
    constexpr int NA1 = kDecFit * VPR1 / kDecThreads;   // staging vectors per thread
    constexpr int TOT = NB1 + TS * NBC;                 // fragment blocks a wavefront streams per pass
    static_assert(NA1 >= 1 && NBC * FK == kDecChunk && TS * 32 * kDecWaves == K1, "shape of an item");
    static_assert(NB1 >= kDecRing && NBC >= 1, "the ring never holds more than one pass");
    extern __shared__ __align__(16) uint16_t lds_x[];   // [kDecFit][LDR1] rows of x, then [kDecFit][LDRH] the slice of h
    uint16_t *lds_h = lds_x + kDecFit * LDR1;
    __shared__ int s_cnt[3][4];                 // per wavefront 0..3: assignments of the expert, of earlier experts, pruned
    __shared__ int s_tok[kGatedMaxAssign];      // token of each row of the expert

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int E = p.E, F = p.F, d = p.d;
    const int G = gridDim.x, blk = blockIdx.x;
    MOE_DEC_STAMP_INIT;
    MOE_DEC_STAMP(0);

    // the gate's expert of assignment `tid` (one per thread of the first four wavefronts)
    const int a_id = tid;
    const int v_exp = a_id < p.n_assign ? p.gate_idx[a_id] : 0x7fffffff;
    const int a_tok = a_id >> (p.gate_k - 1);           // one or two experts per token

    // Counts of expert e among the assignments: its rows, the rows of experts before it, this thread's
    // rank among its rows (stable: ascending assignment id), and the pruned assignments before this thread.
    auto expert_counts = [&](int e, int &count, int &lower, int &rank, int &pruned_rank, bool &mine, bool &pruned) {
        mine = v_exp == e;
        pruned = v_exp == E;
        const bool before = v_exp < e;
        const uint64_t m_mine = __ballot(mine), m_before = __ballot(before), m_pruned = __ballot(pruned);
        __syncthreads();                        // the previous use of s_cnt is over
        if (lane == 0 && wave < 4) {
            s_cnt[0][wave] = __popcll(m_mine);
            s_cnt[1][wave] = __popcll(m_before);
            s_cnt[2][wave] = __popcll(m_pruned);
        }
        __syncthreads();
        int first = 0, pfirst = 0;
        count = 0, lower = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave) { first += s_cnt[0][w]; pfirst += s_cnt[2][w]; }
            count += s_cnt[0][w];
            lower += s_cnt[1][w];
        }
        const uint64_t below = (1ull << lane) - 1;
        rank = first + __popcll(m_mine & below);
        pruned_rank = pfirst + __popcll(m_pruned & below);
    };

    uint4 W[kDecRing];
    // k octet this lane's quarter of the wavefront reads within a 32-deep step (see swap_rows)
    const int koct = ((lane >> 4) & 1) * 16 + (lane >> 5) * 8;

    const int C = F / kDecChunk;                        // items per expert
    const uint32_t lane_off = (uint32_t)lane * 16u;
    // this wavefront's slab of W1 in item `it` (whole K range)
    auto w1_slab = [&](int it) {
        return p.w1 + (size_t)(it / C) * packed_bytes_per_expert(K1, F, BITS) + (size_t)((it % C) * kDecWaves + wave) * NB1 * kFragBytes;
    };
    // EARLY (the launcher's choice where nearly every expert has rows): an item's first ring is requested before the
    // expert's row count is known (the count needs the gate's indices and two barriers; the weights need neither):
    // for the workgroup's first item at once, for a further item when the item before it has used up its stream.
    // Should the expert turn out empty, this one ring (a quarter of the item's stream) was read in vain.  Past the
    // last item the descriptor has no extent: the same eight loads, no traffic, so that the count of loads in flight
    // does not depend on the path taken.
    auto prime = [&](int it) {
        const __amdgpu_buffer_rsrc_t r1e = dec_stream_rsrc(w1_slab(min(it, p.items1 - 1)), it < p.items1 ? NB1 * kFragBytes : 0);
        dec_static_for<0, kDecRing>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            W[i] = dec_ring_load(r1e, lane_off, i * kFragBytes);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    if constexpr (EARLY) prime(blk);
    for (int it = blk; it < p.items1; it += G) {
        const int e = it / C, c = it % C;
        int count, lower, rank, prank;
        bool mine, pruned;
        // this wavefront's weight stream: its slab of W1 (whole K range), then the slice's rows of its TS slabs of W2
        // (the bases are the same for the whole wavefront, so they live in scalar registers; a lane adds 16 bytes x its number)
        const uint8_t *w1b = w1_slab(it);
        expert_counts(e, count, lower, rank, prank, mine, pruned);
        const uint8_t *w2b = p.w2 + (size_t)e * packed_bytes_per_expert(F, K1, BITS) +
                             ((size_t)(wave * TS) * (F / FK) + (size_t)c * NBC) * kFragBytes;
        const size_t slab2 = (size_t)(F / FK) * kFragBytes;             // bytes between consecutive slabs of W2
        // an expert without rows costs no (further) weight traffic: its descriptors have no extent (loads return zero
        // without touching memory) and the item ends below
        const __amdgpu_buffer_rsrc_t r1 = dec_stream_rsrc(w1b, count ? NB1 * kFragBytes : 0);
        __amdgpu_buffer_rsrc_t r2[TS];
#pragma unroll
        for (int s = 0; s < TS; ++s) r2[s] = dec_stream_rsrc(w2b + (size_t)s * slab2, count ? NBC * kFragBytes : 0);
        auto ring_load = [&](auto gc) {         // block g of the stream
            constexpr int g = decltype(gc)::value;
            if constexpr (g < NB1) return dec_ring_load(r1, lane_off, g * kFragBytes);
            else return dec_ring_load(r2[(g - NB1) / NBC], lane_off, ((g - NB1) % NBC) * kFragBytes);
        };
        // The weights depend on nothing but the item: their first ring is requested as soon as the expert is
        // known to have rows, ahead of everything else the item needs (the rows of x arrive under it).
        auto issue_ring = [&]() {
            dec_static_for<0, kDecRing>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                W[i] = ring_load(ic);
                __builtin_amdgcn_sched_barrier(0);
            });
        };
        if constexpr (!EARLY) issue_ring();
        if (c == 0) {                           // the first item of an expert writes the expert's part of the index arrays
            if (tid == 0) {
                p.offsets_out[e] = lower;
                if (e == E - 1) p.offsets_out[E] = lower + count;       // = the active rows
            }
            if (mine) {
                p.inv_perm_out[a_id] = lower + rank;
                p.perm_src_out[lower + rank] = a_id;
            }
            if (pruned && e == E - 1) {         // pruned rows are numbered behind the active ones
                const int r = lower + count + prank;
                p.inv_perm_out[a_id] = r;
                p.perm_src_out[r] = a_id;
            }
        }
        if (count == 0) {
            if constexpr (EARLY) prime(it + G);
            continue;
        }
        if (mine) s_tok[rank] = a_tok;
        const int n1 = c * kDecChunk + wave * 32 + (lane & 15);        // this lane's fc1 channels: n1, n1 + 16
        const float cs0 = __half2float(p.s1[(size_t)e * F + n1]), cs1 = __half2float(p.s1[(size_t)e * F + n1 + 16]);
        const float bi0 = p.b1 ? __half2float(p.b1[(size_t)e * F + n1]) : 0.0f, bi1 = p.b1 ? __half2float(p.b1[(size_t)e * F + n1 + 16]) : 0.0f;
        __syncthreads();                        // s_tok is written
        for (int z0 = 0; z0 < count; z0 += kDecFit) {   // usually a single pass
            const int rows = min(kDecFit, count - z0);
            if (z0) issue_ring();               // a further pass streams the same weights again
            // rows of x: gathered through the tokens of the expert's rows
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 *xv = reinterpret_cast<const u32x4 *>(p.x);
            const int total = rows * VPR1;
            u32x4 av[NA1];
#pragma unroll
            for (int j = 0; j < NA1; ++j) {
                const int idx = min(j * kDecThreads + tid, total - 1);
                av[j] = xv[(size_t)s_tok[z0 + idx / VPR1] * VPR1 + idx % VPR1];
            }
#pragma unroll
            for (int j = 0; j < NA1; ++j) {
                const int idx = j * kDecThreads + tid;
                if (idx < total) *reinterpret_cast<u32x4 *>(lds_x + (idx / VPR1) * LDR1 + (idx % VPR1) * 8) = av[j];
            }
            __syncthreads();
            MOE_DEC_STAMP(1);

            // ---- fc1: 16 rows x 32 channels per wavefront over the whole K range
            const int arow_i = min(lane & 15, rows - 1);                // clamped to a live row
            const uint16_t *arow = lds_x + (size_t)arow_i * LDR1 + koct;
            uint4 A[2][PAIRS];
            auto fetch_a = [&](const uint16_t *row, int slot, int kb) {
#pragma unroll
                for (int q = 0; q < PAIRS; ++q) A[slot][q] = *reinterpret_cast<const uint4 *>(row + kb * FK + 32 * q);
            };
            // one fragment block: 32 channels x FK k values, into the accumulators of the two channel halves
            auto mac_block = [&](int slot, int g, float4_t &lo, float4_t &hi) {
                uint32_t r0 = W[g % kDecRing].x, r1 = W[g % kDecRing].y, r2 = W[g % kDecRing].z, r3 = W[g % kDecRing].w;
                uint32_t bw[4];
                if constexpr (BITS == 4) {
                    swap_rows(r0, r1);
                    swap_rows(r2, r3);
                    dequant4(r0, bw);
                    lo = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, A[slot][0]), frag_from(bw), lo, 0, 0, 0);
                    dequant4(r1, bw);
                    hi = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, A[slot][0]), frag_from(bw), hi, 0, 0, 0);
                    dequant4(r2, bw);
                    lo = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, A[slot][1]), frag_from(bw), lo, 0, 0, 0);
                    dequant4(r3, bw);
                    hi = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, A[slot][1]), frag_from(bw), hi, 0, 0, 0);
                } else {
                    swap_rows(r0, r2);
                    swap_rows(r1, r3);
                    dequant8(r0, r1, bw);
                    lo = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, A[slot][0]), frag_from(bw), lo, 0, 0, 0);
                    dequant8(r2, r3, bw);
                    hi = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, A[slot][0]), frag_from(bw), hi, 0, 0, 0);
                }
            };
            float4_t h0 = {0.f, 0.f, 0.f, 0.f}, h1 = {0.f, 0.f, 0.f, 0.f};
            fetch_a(arow, 0, 0);
            dec_static_for<0, NB1>([&](auto bc) {
                constexpr int b = decltype(bc)::value;
                __builtin_amdgcn_sched_barrier(0);
                if (b + 1 < NB1) fetch_a(arow, (b + 1) & 1, b + 1);
                mac_block(b & 1, b, h0, h1);
                if constexpr (b + kDecRing < TOT) W[b % kDecRing] = ring_load(std::integral_constant<int, b + kDecRing>{});   // runs on into the W2 blocks
            });
            // rows 4 (lane / 16) + i, channels n1 and n1 + 16: scale, bias, activation, fp16, into the slice of h in LDS
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = 4 * (lane >> 4) + i;
                const _Float16 v0 = (_Float16)activate(h0[i] * cs0 + bi0, p.act), v1 = (_Float16)activate(h1[i] * cs1 + bi1, p.act);
                lds_h[m * LDRH + wave * 32 + (lane & 15)] = __builtin_bit_cast(uint16_t, v0);
                lds_h[m * LDRH + wave * 32 + (lane & 15) + 16] = __builtin_bit_cast(uint16_t, v1);
            }
            __syncthreads();
            MOE_DEC_STAMP(2);

            // ---- fc2 on the slice: 16 rows x (TS x 32) output channels per wavefront, K = the slice's 512 channels
            const uint16_t *hrow = lds_h + (size_t)arow_i * LDRH + koct;
            float4_t y[TS][2];
#pragma unroll
            for (int s = 0; s < TS; ++s) y[s][0] = y[s][1] = float4_t{0.f, 0.f, 0.f, 0.f};
            fetch_a(hrow, 0, 0);
            dec_static_for<0, TS * NBC>([&](auto bc) {
                constexpr int b = decltype(bc)::value, s = b / NBC, g = NB1 + b;
                __builtin_amdgcn_sched_barrier(0);
                if (b + 1 < TS * NBC) fetch_a(hrow, (b + 1) & 1, (b + 1) % NBC);
                mac_block(b & 1, g, y[s][0], y[s][1]);
                if constexpr (g + kDecRing < TOT) W[g % kDecRing] = ring_load(std::integral_constant<int, g + kDecRing>{});
            });
            MOE_DEC_STAMP(3);
            // this slice's part of y, rows lower + z0 + m of the expert-sorted order
            float *prow = p.partial + ((size_t)c * p.n_assign + lower + z0) * d;
#pragma unroll
            for (int s = 0; s < TS; ++s) {
                const int n2 = (wave * TS + s) * 32 + (lane & 15);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int m = 4 * (lane >> 4) + i;
                    if (m < rows) {
                        prow[(size_t)m * d + n2] = y[s][0][i];
                        prow[(size_t)m * d + n2 + 16] = y[s][1][i];
                    }
                }
            }
            if (z0 + kDecFit < count) __syncthreads();      // LDS rows are free for the next pass
        }
        if constexpr (EARLY) prime(it + G);
    }
    MOE_DEC_STAMP(7);
}

// Sum of the d_ff slices and of a token's experts: out[t] = sum_j scale[a] * (W2-scale * sum_c partial[c][row of a] + b2),
// a = t k + j in ascending j, slices in ascending c; pruned assignments (expert index E) add nothing, so a
// pruned token's row is zero.  One workgroup per token, four channels per thread.
__global__ __launch_bounds__(256) void decode_reduce_kernel(DecodeArgs p)
{
    const int t = blockIdx.x, C = p.F / kDecChunk, d = p.d;
    for (int n = threadIdx.x * 4; n < d; n += 256 * 4) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int j = 0; j < p.gate_k; ++j) {
            const int a = t * p.gate_k + j, e = p.gate_idx[a];
            if (e >= p.E) continue;             // pruned
            const int r = p.inv_perm_out[a];
            const float sc = p.gate_scale[a];
            float4 v[8];
#pragma unroll
            for (int c = 0; c < 8; ++c)
                v[c] = c < C ? *reinterpret_cast<const float4 *>(p.partial + ((size_t)c * p.n_assign + r) * d + n) : make_float4(0.f, 0.f, 0.f, 0.f);
            float4 y = v[0];
#pragma unroll
            for (int c = 1; c < 8; ++c) { y.x += v[c].x; y.y += v[c].y; y.z += v[c].z; y.w += v[c].w; }
            const uint2 s2 = *reinterpret_cast<const uint2 *>(p.s2 + (size_t)e * d + n);
            const half2_t s01 = bits_h2(s2.x), s23 = bits_h2(s2.y);
            float b[4] = {0.f, 0.f, 0.f, 0.f};
            if (p.b2) {
                const uint2 bb = *reinterpret_cast<const uint2 *>(p.b2 + (size_t)e * d + n);
                const half2_t b01 = bits_h2(bb.x), b23 = bits_h2(bb.y);
                b[0] = (float)b01[0]; b[1] = (float)b01[1]; b[2] = (float)b23[0]; b[3] = (float)b23[1];
            }
            acc.x += sc * (y.x * (float)s01[0] + b[0]);
            acc.y += sc * (y.y * (float)s01[1] + b[1]);
            acc.z += sc * (y.z * (float)s23[0] + b[2]);
            acc.w += sc * (y.w * (float)s23[1] + b[3]);
        }
        *reinterpret_cast<float4 *>(p.out + (size_t)t * d + n) = acc;
    }
}

// ---- host side -----------------------------------------------------------------------------------

template <int BITS, int NB1, int TS, int NBC>
static int launch_decode(const DecodeArgs &p, int grid, hipStream_t s)
{
    constexpr int FK = BITS == 4 ? 64 : 32;
    constexpr int K1 = NB1 * FK;
    const int lds = kDecFit * (K1 + kDecRowPad) * 2 + kDecFit * (kDecChunk + kDecRowPad) * 2;
    if (p.early_ring) hipLaunchKernelGGL((decode_ffn_kernel<BITS, NB1, TS, NBC, true>), dim3(grid), dim3(kDecThreads), lds, s, p);
    else hipLaunchKernelGGL((decode_ffn_kernel<BITS, NB1, TS, NBC, false>), dim3(grid), dim3(kDecThreads), lds, s, p);
    int rc = check_launch("moe_grouped_ffn_wq_gated (decode kernel)");
    if (rc || !p.out) return rc;                // (no output buffer: the partial sums are all the caller wants)
    hipLaunchKernelGGL(decode_reduce_kernel, dim3(p.n_assign / p.gate_k), dim3(256), 0, s, p);
    return check_launch("moe_grouped_ffn_wq_gated (slice reduction)");
}

// Sizes the decode kernel is built for: d_model of sixteen fragment blocks (1024 with 4-bit, 512 with
// 8-bit weights), d_ff in slices of 512 channels (at most eight), few rows per expert.
bool decode_ffn_supports(int n_assign, int E, int d, int F, int bits)
{
    if (bits != 4 && bits != 8) return false;
    if (n_assign < 1 || n_assign > kGatedMaxAssign || E < 1 || E > kDecMaxExperts) return false;
    if (d != (bits == 4 ? 1024 : 512) || F % kDecChunk || F / kDecChunk > 8 || F < kDecChunk) return false;
    // few rows per expert (a pass takes sixteen) and enough items to give a quarter of the compute units one
    return (long)n_assign <= 8L * E && (long)E * (F / kDecChunk) >= 64;
}

size_t decode_ffn_partial_bytes(int n_assign, int d, int F)
{
    return (size_t)(F / kDecChunk) * n_assign * d * sizeof(float);
}

static int decode_ffn_grid(int items)
{
    static int cus = 0;                          // compute units of the current device (one workgroup fits each)
    if (!cus) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) cus = n;
        else cus = 64;
    }
    return items < cus ? items : cus;
}

int launch_decode_ffn(const DecodeArgs &q, int bits, hipStream_t s)
{
    DecodeArgs p = q;
    p.items1 = p.E * (p.F / kDecChunk);
    // three or more assignments per expert: under uniform routing at most one expert in twenty is empty, and the
    // early ring of such an expert is a quarter of its weights
    p.early_ring = p.n_assign >= 3 * p.E;
    const int grid = decode_ffn_grid(p.items1);
    if (bits == 4) return launch_decode<4, 16, 2, 8>(p, grid, s);
    return launch_decode<8, 16, 1, 16>(p, grid, s);
}

}  // namespace moe
