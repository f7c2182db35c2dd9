// moe_permute: stable counting sort of the (expert, row) tuples by expert and gather of the
// activation rows into expert-contiguous order (Sec. 3.3).
//
// The assignment list a = 0..R-1 is cut into wave-chunks of CH consecutive assignments; a
// wavefront counts its chunk per expert (integer LDS atomics: order-independent), the
// counts are turned into per-chunk start positions by an exclusive scan over (expert, chunk),
// and each wavefront then ranks its assignments in order with ballot-based match masks, so
// the sort is stable and free of global atomics.  Small problems (up to 4096 assignments) take
// a single launch that also copies the rows; larger ones take a count launch, a rank launch and
// a row-copy launch.
//
// Batch pruning (Sec. 3.5): an expert index equal to E marks a row of a finished sentence.  It is
// one more key of the sort, the last one, so such rows end up behind every active row;
// expert_offsets[E] is then the number of active rows, and pruned rows are not copied.
#include "moe_common.h"

namespace moe {

constexpr int kPermMaxE = 1024;

__device__ inline uint64_t lanemask_lt() { return (1ull << (threadIdx.x & 63)) - 1ull; }

// lanes of this wavefront holding the same key (keys < 1024), computed with 10 ballots
__device__ inline uint64_t match_key(int key, int key_bits)
{
    uint64_t m = ~0ull;
    for (int b = 0; b < key_bits; ++b) {
        const uint64_t set = __ballot((key >> b) & 1);
        m &= ((key >> b) & 1) ? set : ~set;
    }
    return m;
}

// FUSED: small problems, one launch: every block repeats count + scan + rank for all
// assignments (cheap), keeps perm_src in LDS and then gathers its share of the rows; block 0
// writes the index outputs.  Otherwise PHASE selects count (0) or rank (1), and the per-chunk
// histograms travel through `hist` [nwc][E].
template <bool FUSED, int PHASE>
__global__ __launch_bounds__(256) void permute_index_kernel(const int32_t *__restrict__ expert_idx,
                                                            int R, int NB, int iters, int nwc,
                                                            int key_bits, int32_t *__restrict__ hist,
                                                            int32_t *__restrict__ perm_src,
                                                            int32_t *__restrict__ inv_perm,
                                                            int32_t *__restrict__ offsets,
                                                            const uint4 *__restrict__ x, int k, int row_vec,
                                                            uint4 *__restrict__ x_perm)
{
    extern __shared__ int32_t sm[];          // [4][NB] per-wave counters, [NB] scratch, (FUSED) [R] perm_src
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int blk = FUSED ? 0 : blockIdx.x;  // FUSED: every block plays block 0 of the index phase
    const bool writer = !FUSED || blockIdx.x == 0;
    int32_t *perm_l = sm + 5 * NB;
    const int wc = blk * 4 + wave;           // wave-chunk id
    const int CH = iters * 64;
    int32_t *cnt = sm + wave * NB;
    int32_t *tot = sm + 4 * NB;

    if (FUSED || PHASE == 0) {
        for (int e = threadIdx.x; e < 4 * NB; e += 256) sm[e] = 0;
        __syncthreads();
        for (int it = 0; it < iters; ++it) {
            const int a = wc * CH + it * 64 + lane;
            if (a < R) atomicAdd(&cnt[min(max(expert_idx[a], 0), NB - 1)], 1);   // clamped: never out of range
        }
        __syncthreads();
        if (!FUSED) {
            for (int e = threadIdx.x; e < 4 * NB; e += 256) hist[(size_t)blk * 4 * NB + e] = sm[e];
            return;
        }
    }

    // start position of every (expert, wave-chunk of this block): cnt[w][e] <- base
    for (int e = threadIdx.x; e < NB; e += 256) {
        int before = 0, total = 0;
        int c[4];
        if (FUSED) {
#pragma unroll
            for (int w = 0; w < 4; ++w) c[w] = sm[w * NB + e];
            total = c[0] + c[1] + c[2] + c[3];
        } else {
#pragma unroll
            for (int w = 0; w < 4; ++w) c[w] = hist[(size_t)(blk * 4 + w) * NB + e];
#pragma unroll 16
            for (int j = 0; j < nwc; ++j) {              // independent loads: many in flight
                const int v = hist[(size_t)j * NB + e];
                before += j < blk * 4 ? v : 0;
                total += v;
            }
        }
        tot[e] = total;
        sm[0 * NB + e] = before;
        sm[1 * NB + e] = before + c[0];
        sm[2 * NB + e] = before + c[0] + c[1];
        sm[3 * NB + e] = before + c[0] + c[1] + c[2];
    }
    __syncthreads();
    // exclusive scan of the totals over experts by wavefront 0 (64 experts per step)
    if (wave == 0) {
        int carry = 0;
        for (int e0 = 0; e0 < NB; e0 += 64) {
            const int e = e0 + lane;
            const int v = e < NB ? tot[e] : 0;
            int incl = v;
            for (int off = 1; off < 64; off <<= 1) {
                const int up = __shfl_up(incl, off);
                if (lane >= off) incl += up;
            }
            if (e < NB) tot[e] = carry + incl - v;
            carry += __shfl(incl, 63);
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < NB; e += 256) {
        const int base = tot[e];
        if (writer && blk == 0) offsets[e] = base;
#pragma unroll
        for (int w = 0; w < 4; ++w) sm[w * NB + e] += base;
    }
    __syncthreads();

    // rank: cnt[key] is the next free position of `key` for this wave-chunk
    for (int it = 0; it < iters; ++it) {
        const int a = wc * CH + it * 64 + lane;
        const bool live = a < R;
        const int key = live ? min(max(expert_idx[a], 0), NB - 1) : 0;
        uint64_t m = match_key(live ? key : (1 << key_bits) - 1, key_bits);
        m &= __ballot(live);                 // idle lanes never share a group with live ones
        const int rank = __popcll(m & lanemask_lt());
        int r = 0;
        if (live) {
            r = cnt[key] + rank;
            if (FUSED) perm_l[r] = a;
            if (writer) {
                perm_src[r] = a;
                inv_perm[a] = r;
            }
        }
        __syncthreads();                     // everyone has read cnt[] before the leaders bump it
        if (live && rank == 0) cnt[key] += __popcll(m);
        __syncthreads();
    }
    if (FUSED && x) {
        // x_perm[r] = x[perm_src[r] / k] for this block's share of the active rows; one wavefront per row
        const int active = tot[NB - 1];
        for (int r = blockIdx.x * 4 + wave; r < active; r += gridDim.x * 4) {
            const uint4 *src = x + (size_t)(perm_l[r] / k) * row_vec;
            uint4 *dst = x_perm + (size_t)r * row_vec;
            for (int v = lane; v < row_vec; v += 64) dst[v] = src[v];
        }
    }
}

// x_perm[r] = x[perm_src[r] / k]; one wavefront per row, 16 bytes per lane per step
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4 *__restrict__ x,
                                                          const int32_t *__restrict__ perm_src,
                                                          const int32_t *__restrict__ active_rows, int R,
                                                          int k, int row_vec, uint4 *__restrict__ x_perm)
{
    const int lane = threadIdx.x & 63;
    const int active = min(*active_rows, R);
    for (int r = blockIdx.x * 4 + (threadIdx.x >> 6); r < active; r += gridDim.x * 4) {
        const int t = perm_src[r] / k;
        const uint4 *src = x + (size_t)t * row_vec;
        uint4 *dst = x_perm + (size_t)r * row_vec;
        for (int v = lane; v < row_vec; v += 64) dst[v] = src[v];
    }
}

static void perm_plan(int R, int *iters, int *nblocks)
{
    // up to 4096 assignments: one block, one launch; beyond: 256 assignments per wavefront
    if (R <= 4096) { *iters = (R + 255) / 256; if (*iters < 1) *iters = 1; *nblocks = 1; }
    else { *iters = 4; *nblocks = (R + 1023) / 1024; }
}

}  // namespace moe

extern "C" size_t moe_permute_workspace_bytes(int T, int k, int E)
{
    if (T <= 0 || k <= 0 || E <= 0) return 16;
    int iters, nblocks;
    moe::perm_plan(T * k, &iters, &nblocks);
    return moe::round_up((size_t)nblocks * 4 * (E + 1) * sizeof(int32_t), 256);
}

extern "C" int moe_permute(const int32_t *expert_idx, const void *x, int act_dtype, int T, int k, int E,
                           int d, void *x_perm, int32_t *perm_src, int32_t *inv_perm,
                           int32_t *expert_offsets, void *workspace, size_t workspace_bytes,
                           void *stream)
{
    using namespace moe;
    if (!expert_offsets || (T > 0 && (!expert_idx || !perm_src || !inv_perm)))
        return fail(MOE_ERR_INVALID_ARG, "moe_permute: NULL index pointer");
    if (T > 0 && (x == nullptr) != (x_perm == nullptr)) return fail(MOE_ERR_INVALID_ARG, "moe_permute: x and x_perm must both be given or both be NULL");
    if (T < 0 || k <= 0 || E <= 0 || d <= 0) return fail(MOE_ERR_INVALID_ARG, "moe_permute: T >= 0 and k, E, d > 0 required");
    if (E > kPermMaxE) return fail(MOE_ERR_UNSUPPORTED, "moe_permute: E=%d above %d", E, kPermMaxE);
    if (act_dtype != MOE_F16 && act_dtype != MOE_BF16 && act_dtype != MOE_F32) return fail(MOE_ERR_UNSUPPORTED, "moe_permute: unknown act_dtype %d", act_dtype);
    const int elt = act_dtype == MOE_F32 ? 4 : 2;
    if (((size_t)d * elt) % 16) return fail(MOE_ERR_INVALID_ARG, "moe_permute: rows must be a multiple of 16 bytes (d=%d)", d);
    if ((long long)T * k > 0x7fffffffLL) return fail(MOE_ERR_INVALID_ARG, "moe_permute: T*k overflows int32");
    if (!aligned16(x) || !aligned16(x_perm)) return fail(MOE_ERR_INVALID_ARG, "moe_permute: x and x_perm must be 16-byte aligned");
    const int R = T * k;
    int iters, nblocks;
    perm_plan(R, &iters, &nblocks);
    const size_t need = moe_permute_workspace_bytes(T, k, E);
    if (nblocks > 1 && (!workspace || workspace_bytes < need))
        return fail(MOE_ERR_WORKSPACE, "moe_permute: workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    const int NB = E + 1;                              // keys: the experts and the pruned-row index E
    int key_bits = 1;
    while ((1 << key_bits) < NB + 1) ++key_bits;       // one spare code for idle lanes
    hipStream_t s = as_stream(stream);
    const size_t smem = (size_t)5 * NB * sizeof(int32_t);
    int32_t *hist = (int32_t *)workspace;
    const int row_vec = (int)((size_t)d * elt / 16);
    if (nblocks == 1) {
        // index and gather in one launch: up to 64 blocks share the row copies
        int gb = x ? (R + 3) / 4 : 1;
        gb = gb < 1 ? 1 : gb > 64 ? 64 : gb;
        hipLaunchKernelGGL((permute_index_kernel<true, 0>), dim3(gb), dim3(256), smem + (size_t)R * sizeof(int32_t), s,
                           expert_idx, R, NB, iters, 4, key_bits, hist, perm_src, inv_perm, expert_offsets,
                           (const uint4 *)x, k, row_vec, (uint4 *)x_perm);
        return check_launch("moe_permute");
    }
    hipLaunchKernelGGL((permute_index_kernel<false, 0>), dim3(nblocks), dim3(256), smem, s, expert_idx, R, NB, iters,
                       nblocks * 4, key_bits, hist, perm_src, inv_perm, expert_offsets, (const uint4 *)nullptr, k,
                       row_vec, (uint4 *)nullptr);
    hipLaunchKernelGGL((permute_index_kernel<false, 1>), dim3(nblocks), dim3(256), smem, s, expert_idx, R, NB, iters,
                       nblocks * 4, key_bits, hist, perm_src, inv_perm, expert_offsets, (const uint4 *)nullptr, k,
                       row_vec, (uint4 *)nullptr);
    int rc = check_launch("moe_permute (index)");
    if (rc != MOE_OK || !x || R == 0) return rc;
    int gblocks = (R + 3) / 4;
    if (gblocks > 4096) gblocks = 4096;
    hipLaunchKernelGGL(gather_rows_kernel, dim3(gblocks), dim3(256), 0, s, (const uint4 *)x, perm_src, expert_offsets + E, R, k,
                       row_vec, (uint4 *)x_perm);
    return check_launch("moe_permute (gather)");
}
