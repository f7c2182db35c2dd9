// moe_gate_topk: router logits, top-k selection and gate probabilities (Sec. 3.3).
//
// Mapping: a lane owns one expert (NE experts when E > 64) for TB tokens (TB = 1 when there are
// few tokens, so that they spread over more blocks); when E < 64 a
// wavefront is cut into 64/EL token groups of EL = pow2ceil(E) lanes.  The four wavefronts of
// a block take the four partial sums of the contract (128-element blocks of the feature axis
// dealt round-robin), so the floating-point order is fixed by the definition, not by the
// launch shape.  Softmax and top-k are butterfly reductions over the EL lanes of a group.
// FP16 batches of 16384 tokens and more with 64 experts take another mapping, a token per lane
// (gate_token_lanes_kernel below), with the same order of the additions.
#include <math.h>

#include <type_traits>

#include "moe_common.h"

namespace moe {

constexpr int kGateBlk = 128;    // feature block of one partial-sum turn
constexpr int kGateWRow = 64;     // LDS row of the staged gate-weight block: 64 experts' weights for one feature

template <bool BF16>
__device__ inline float act_to_float(uint16_t v)
{
    if (BF16) return __uint_as_float((uint32_t)v << 16);
    __half h;
    *reinterpret_cast<uint16_t *>(&h) = v;
    return __half2float(h);
}

// acc + x * w in fp32 with both operands widened exactly (one v_fma_mix_f32 for fp16 inputs).
template <bool BF16>
__device__ inline float mac(uint16_t xb, uint16_t wb, float acc)
{
    if (BF16) return fmaf(__uint_as_float((uint32_t)xb << 16), __uint_as_float((uint32_t)wb << 16), acc);
    return fmaf((float)__builtin_bit_cast(_Float16, xb), (float)__builtin_bit_cast(_Float16, wb), acc);
}

// Value of the partner lane of butterfly step `off` within a lane group.  Steps 1 and 2 are quad
// permutes, 4 and 8 the half-row and row mirrors (the same partner sets once the value is uniform
// over 4 resp. 8 lanes, which the earlier steps have made it), all in the VALU's data-parallel
// primitives, the steps across 16-lane rows and 32-lane halves the row and half swaps.  Used in ascending
// order of `off` by reductions whose operation is commutative.
template <int OFF, typename V>
__device__ inline V butterfly_partner(V v)
{
    const int b = __builtin_bit_cast(int, v);
    int r;
    if (OFF == 1) r = __builtin_amdgcn_update_dpp(0, b, 0xB1, 0xf, 0xf, false);        // quad_perm [1,0,3,2]
    else if (OFF == 2) r = __builtin_amdgcn_update_dpp(0, b, 0x4E, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
    else if (OFF == 4) r = __builtin_amdgcn_update_dpp(0, b, 0x141, 0xf, 0xf, false);  // row_half_mirror
    else if (OFF == 8) r = __builtin_amdgcn_update_dpp(0, b, 0x140, 0xf, 0xf, false);  // row_mirror
    else if (OFF == 16) {
        // rows of 16 lanes: the swap leaves [r0, r0, r2, r2] and [r1, r1, r3, r3]; a lane in an even row
        // takes the second, a lane in an odd row the first
        const auto sw = __builtin_amdgcn_permlane16_swap((unsigned)b, (unsigned)b, false, false);
        r = (int)((threadIdx.x & 16) ? sw[0] : sw[1]);
    } else {
        // halves of 32 lanes: the swap leaves [lo, lo] and [hi, hi]
        const auto sw = __builtin_amdgcn_permlane32_swap((unsigned)b, (unsigned)b, false, false);
        r = (int)((threadIdx.x & 32) ? sw[0] : sw[1]);
    }
    return __builtin_bit_cast(V, r);
}

// f(partner value getter) for every butterfly step of a group of EL lanes (EL = 8, 16, 32 or 64)
template <typename F>
__device__ inline void butterfly_steps(int EL, F &&f)
{
    f(std::integral_constant<int, 1>{});
    f(std::integral_constant<int, 2>{});
    f(std::integral_constant<int, 4>{});
    if (EL > 8) f(std::integral_constant<int, 8>{});
    if (EL > 16) f(std::integral_constant<int, 16>{});
    if (EL > 32) f(std::integral_constant<int, 32>{});
}

// With E <= 64 the 128 x E block of the gate weight that a wavefront needs per turn is copied
// to LDS with 16-byte loads first (one latency per turn instead of one per row).
template <bool BF16, int NE, int TB, int GM>
__global__ __launch_bounds__(256) void gate_kernel(const uint16_t *__restrict__ x,
                                                   const uint16_t *__restrict__ wg,
                                                   const float *__restrict__ bias,
                                                   const uint8_t *__restrict__ finished, int T, int d,
                                                   int E, int EL, int k, int renorm,
                                                   int32_t *__restrict__ expert_idx,
                                                   float *__restrict__ expert_scale)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: addresses built from it are scalar
    const int G = 64 / EL;                        // token groups per wavefront
    const int grp = lane / EL, le = lane % EL;
    const int ntok = G * TB;                 // tokens per block
    const int t0 = blockIdx.x * ntok;

    // wave-private staging areas: x [ntok][128] and (NE == 1) the gate weight block [128][E]
    constexpr bool WLDS = NE == 1;
    const size_t x_halfs = (GM == 1 && NE == 1 && !BF16) ? 0 : (size_t)ntok * kGateBlk;   // (x through scalar loads: no staging)
    const size_t wave_halfs = x_halfs + (WLDS ? (size_t)kGateWRow * kGateBlk : 0);
    uint16_t *xs = reinterpret_cast<uint16_t *>(smem) + (size_t)wave * wave_halfs;
    uint16_t *ws = xs + x_halfs;
    float *part = reinterpret_cast<float *>(smem);   // [4][NE][TB][64], over the staging areas once they are used up

    float acc[NE][TB];
#pragma unroll
    for (int a = 0; a < NE; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b) acc[a][b] = 0.0f;

    const int e_shift = 31 - __builtin_clz(EL);
    const int nblk = (d + kGateBlk - 1) / kGateBlk;
    const int turns = (nblk + 3) / 4;             // same trip count for all four wavefronts
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    // GM == 1 and at most 64 experts (a lane group is the whole wavefront): a token's features are
    // the same for every lane, so they are fetched with scalar loads and feed the MACs from scalar
    // registers; no x staging.  (With more experts per lane the scalar registers run out.)
    constexpr bool SX = GM == 1 && NE == 1 && !BF16;   // (bf16 features would be widened in scalar registers, two per dword: they run out)
    constexpr int XR = SX ? 1 : (GM * TB >= 4 ? GM * TB / 4 : 1);   // x vectors per lane per turn (ntok <= GM * TB rows, 4 rows per pass)
    constexpr int WR = WLDS ? 16 : 1;             // gate-weight vectors per lane per turn (128 x E halfs, E <= 64)
    struct Staged { u32x4 x[XR]; u32x4 w[WR]; };

    // global -> registers for one turn; nothing is waited for here
    auto fetch = [&](int turn, Staged &st) {
        const int blk = min(turn * 4 + wave, max(nblk - 1, 0));     // clamped: a turn past the end re-reads the last block
        const int i0 = blk * kGateBlk;
        const int lim = min(kGateBlk, d - i0);
#pragma unroll
        for (int r = 0; r < (SX ? 0 : XR); ++r) {
            const int row = (lane >> 4) + 4 * r;
            const int seg = (lane & 15) * 8;
            const int t = min(t0 + min(row, ntok - 1), T - 1);
            st.x[r] = *reinterpret_cast<const u32x4 *>(x + (size_t)t * d + i0 + min(seg, lim - 8));
        }
        if (WLDS) {
            const u32x4 *src = reinterpret_cast<const u32x4 *>(wg + (size_t)i0 * E);
            const int nvec = lim * E / 8;
#pragma unroll
            for (int u = 0; u < WR; ++u)
                if (u * 64 < nvec) st.w[u] = src[min(u * 64 + lane, nvec - 1)];
        }
    };
    // registers -> LDS: x rows as they are (zero past the block's end) and the weight block
    auto stash = [&](int turn, const Staged &st) {
        const int blk = turn * 4 + wave;
        const int lim = blk < nblk ? min(kGateBlk, d - blk * kGateBlk) : 0;     // multiple of 8
#pragma unroll
        for (int r = 0; r < (SX ? 0 : XR); ++r) {
            const int row = (lane >> 4) + 4 * r;
            const int seg = (lane & 15) * 8;
            if (row < ntok) {
                u32x4 v = st.x[r];
                if (seg >= lim) v = u32x4{0, 0, 0, 0};
                *reinterpret_cast<u32x4 *>(xs + row * kGateBlk + seg) = v;
            }
        }
        if (WLDS) {
            // rows of the block keep their order, padded to 64 experts: [i][64]
            const int nvec = lim * E / 8;
#pragma unroll
            for (int u = 0; u < WR; ++u) {
                const int v = u * 64 + lane;
                if (v < nvec) {
                    int i, e;
                    if (E == EL) {                               // power of two: shifts
                        i = (v * 8) >> e_shift;
                        e = (v * 8) & (E - 1);
                    } else {                                     // one division per vector
                        i = (v * 8) / E;
                        e = v * 8 - i * E;
                    }
                    if ((E & 7) == 0) {
                        *reinterpret_cast<u32x4 *>(ws + i * kGateWRow + e) = st.w[u];
                    } else {
#pragma unroll
                        for (int q = 0; q < 8; ++q) {
                            ws[i * kGateWRow + e] = (uint16_t)(st.w[u][q >> 1] >> (16 * (q & 1)));
                            if (++e == E) { e = 0; ++i; }
                        }
                    }
                }
            }
        }
    };
    auto compute = [&](int turn) __attribute__((always_inline)) {
        const int blk = turn * 4 + wave;
        const int i0 = blk * kGateBlk;
        const int lim = blk < nblk ? min(kGateBlk, d - i0) : 0;
#pragma unroll 2
        for (int i = 0; i < lim; i += 8) {       // unrolled: several LDS reads in flight per wavefront
            uint16_t wv[NE][8];
#pragma unroll
            for (int a = 0; a < NE; ++a) {
                const int e = min(a * 64 + le, E - 1);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    wv[a][u] = WLDS ? ws[(i + u) * kGateWRow + e] : wg[(size_t)(i0 + i + u) * E + e];
            }
            // tokens in batches of up to eight: their rows are read first, then the features are
            // walked with the tokens innermost, so that consecutive MACs are independent
            constexpr int XB = TB < 8 ? TB : 8;
#pragma unroll
            for (int b0 = 0; b0 < TB; b0 += XB) {
                uint4 raw[XB];
#pragma unroll
                for (int b = 0; b < XB; ++b) {
                    if (SX)     // uniform address: a scalar load
                        raw[b] = *reinterpret_cast<const uint4 *>(x + (size_t)min(t0 + b0 + b, T - 1) * d + i0 + i);
                    else
                        raw[b] = *reinterpret_cast<const uint4 *>(xs + (grp * TB + b0 + b) * kGateBlk + i);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
#pragma unroll
                    for (int b = 0; b < XB; ++b) {
                        const uint32_t r = u < 2 ? raw[b].x : u < 4 ? raw[b].y : u < 6 ? raw[b].z : raw[b].w;
                        const uint16_t xb = (uint16_t)(r >> (16 * (u & 1)));
#pragma unroll
                        for (int a = 0; a < NE; ++a) acc[a][b0 + b] = mac<BF16>(xb, wv[a][u], acc[a][b0 + b]);
                    }
                }
            }
        }
    };
    // The loads of two turns are always in flight: with few tokens the whole kernel is one memory
    // latency long, and two turns cover d = 1024.
    // The staging areas are private to a wavefront, and LDS serves one wavefront's instructions in
    // order, so a turn needs no barrier between its writes and reads.
    Staged s0, s1;
    fetch(0, s0);
    fetch(1, s1);
    for (int turn = 0; turn < turns; turn += 2) {
        stash(turn, s0);
        if (turn + 2 < turns) fetch(turn + 2, s0);
        compute(turn);
        if (turn + 1 < turns) {
            stash(turn + 1, s1);
            if (turn + 3 < turns) fetch(turn + 3, s1);
            compute(turn + 1);
        }
    }

    __syncthreads();                              // every wavefront is done with its staging area
#pragma unroll
    for (int a = 0; a < NE; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b) part[((wave * NE + a) * TB + b) * 64 + lane] = acc[a][b];
    __syncthreads();

    // wavefront `wave` finishes token slots b = wave, wave + 4, ... of every group
    for (int b = wave; b < TB; b += 4) {
    const int t = t0 + grp * TB + b;
    float lg[NE];
    const float NEG = -INFINITY;
#pragma unroll
    for (int a = 0; a < NE; ++a) {
        const int e = a * 64 + le;
        float p0 = part[((0 * NE + a) * TB + b) * 64 + lane];
        float p1 = part[((1 * NE + a) * TB + b) * 64 + lane];
        float p2 = part[((2 * NE + a) * TB + b) * 64 + lane];
        float p3 = part[((3 * NE + a) * TB + b) * 64 + lane];
        float l = ((p0 + p1) + p2) + p3;
        if (e < E && bias) l = l + bias[e];
        lg[a] = e < E ? l : NEG;
    }

    // best (value, index) with ties to the lower index
    int sel[2] = {0, 0};
    float selv[2] = {0.0f, 0.0f};
    for (int j = 0; j < k; ++j) {
        float bv = NEG;
        int be = 0x7fffffff;
#pragma unroll
        for (int a = 0; a < NE; ++a) {
            const int e = a * 64 + le;
            const bool taken = j == 1 && e == sel[0];
            if (e < E && !taken && (lg[a] > bv || be == 0x7fffffff)) { bv = lg[a]; be = e; }
        }
        butterfly_steps(EL, [&](auto off) {
            constexpr int OFF = decltype(off)::value;
            const float ov = butterfly_partner<OFF>(bv);
            const int oe = butterfly_partner<OFF>(be);
            if (oe != 0x7fffffff && (be == 0x7fffffff || ov > bv || (ov == bv && oe < be))) { bv = ov; be = oe; }
        });
        sel[j] = be;
        selv[j] = bv;
    }
    const float lmax = selv[0];
    float den = 0.0f;
#pragma unroll
    for (int a = 0; a < NE; ++a)
        if (a * 64 + le < E) den += expf(lg[a] - lmax);
    butterfly_steps(EL, [&](auto off) { den += butterfly_partner<decltype(off)::value>(den); });

    if (le == 0 && t < T) {
        if (finished && finished[t]) {
            // batch pruning (Sec. 3.5): the row gets an expert index past the real experts, so the
            // sort moves it behind every active row, and a zero scale
            for (int j = 0; j < k; ++j) {
                expert_idx[k * t + j] = E;
                expert_scale[k * t + j] = 0.0f;
            }
        } else if (k == 1) {
            expert_idx[t] = sel[0];
            expert_scale[t] = 1.0f / den;
        } else {
            const float e2 = expf(selv[1] - lmax);
            float s0 = 1.0f / den, s1 = e2 / den;
            if (renorm) { s0 = 1.0f / (1.0f + e2); s1 = e2 / (1.0f + e2); }
            expert_idx[2 * t] = sel[0];
            expert_idx[2 * t + 1] = sel[1];
            expert_scale[2 * t] = s0;
            expert_scale[2 * t + 1] = s1;
        }
    }
    }   // token slots of this wavefront
}

// Many tokens, 64 experts: a lane owns one token.  The block's wavefronts are the four partial sums of
// the contract times 64 / EW slices of the experts; a feature's EW gate weights are the same for every
// lane, so they come through scalar loads and feed the MACs from scalar registers (one row of the gate
// weight is 128 contiguous bytes), while each lane walks its own token's features, 32 at a time, one
// chunk ahead.  Nothing is staged or exchanged until the partial sums meet in LDS; then every wavefront
// finishes the logits of 64 / NW experts for all 64 tokens and the candidates are merged per token.
// Same floating-point order of the logits as gate_kernel.  FP16 only (bf16 weights would be widened in
// scalar registers, which run out).
template <int EW>
__global__ __launch_bounds__(256 * (64 / EW)) void gate_token_lanes_kernel(const uint16_t *__restrict__ x,
                                                               const uint16_t *__restrict__ wg,
                                                               const float *__restrict__ bias,
                                                               const uint8_t *__restrict__ finished, int T, int d,
                                                               int k, int renorm, int32_t *__restrict__ expert_idx,
                                                               float *__restrict__ expert_scale)
{
    constexpr int E = 64, NW = 4 * (E / EW), EPW = E / NW;      // wavefronts per block, experts a wavefront finishes
    extern __shared__ __align__(16) unsigned char smem[];
    float *part = reinterpret_cast<float *>(smem);           // [4 partial sums][64 experts][64 tokens]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int p = wave & 3, slice = wave >> 2;
    const int t = blockIdx.x * 64 + lane;
    const uint4 *xrow = reinterpret_cast<const uint4 *>(x + (size_t)min(t, T - 1) * d);
    float acc[EW];
#pragma unroll
    for (int e = 0; e < EW; ++e) acc[e] = 0.0f;

    const int nblk = d / kGateBlk;                            // d is a multiple of the block here
    const int nch = ((nblk - p + 3) / 4) * 4;                 // 32-feature chunks of this partial sum
    auto first_feature = [&](int c) { return (p + 4 * (c >> 2)) * kGateBlk + (c & 3) * 32; };
    uint4 nxt[4];
    if (nch > 0) {
#pragma unroll
        for (int v = 0; v < 4; ++v) nxt[v] = xrow[first_feature(0) / 8 + v];
    }
#pragma unroll 1
    for (int c = 0; c < nch; ++c) {
        uint4 cur[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) cur[v] = nxt[v];
        const int cn = min(c + 1, nch - 1);
#pragma unroll
        for (int v = 0; v < 4; ++v) nxt[v] = xrow[first_feature(cn) / 8 + v];
        const uint32_t *wrow = reinterpret_cast<const uint32_t *>(wg + (size_t)first_feature(c) * E + slice * EW);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const uint32_t xw[4] = {cur[v].x, cur[v].y, cur[v].z, cur[v].w};
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint16_t xb = (uint16_t)(xw[u >> 1] >> (16 * (u & 1)));
                const uint32_t *w = wrow + (v * 8 + u) * (E / 2);     // uniform address: scalar loads
#pragma unroll
                for (int q = 0; q < EW / 2; ++q) {
                    const uint32_t w2 = w[q];
                    acc[2 * q] = mac<false>(xb, (uint16_t)w2, acc[2 * q]);
                    acc[2 * q + 1] = mac<false>(xb, (uint16_t)(w2 >> 16), acc[2 * q + 1]);
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < EW; ++e) part[(p * E + slice * EW + e) * 64 + lane] = acc[e];
    __syncthreads();

    // wavefront w: logits of experts w * EPW ... for the lane's token, best two of them with ties to
    // the lower index (experts in ascending order, a later one must be strictly larger)
    float lg[EPW];
    float bv = 0.0f, sv = 0.0f;
    int be = 0, se = 0;
#pragma unroll
    for (int j = 0; j < EPW; ++j) {
        const int e = wave * EPW + j;
        float l = ((part[e * 64 + lane] + part[(E + e) * 64 + lane]) + part[(2 * E + e) * 64 + lane]) + part[(3 * E + e) * 64 + lane];
        if (bias) l = l + bias[e];
        lg[j] = l;
        const bool first = j == 0 || l > bv;
        const bool second = !first && (j == 1 || l > sv);
        sv = first ? bv : second ? l : sv;
        se = first ? be : second ? e : se;
        bv = first ? l : bv;
        be = first ? e : be;
    }
    __syncthreads();                                         // the partial sums are used up: candidates take their place
    float *cand_v = part;                                    // [NW][2][64]
    int *cand_e = reinterpret_cast<int *>(part + NW * 2 * 64);      // [NW][2][64]
    float *den_part = part + 2 * NW * 2 * 64;                // [NW][64]
    cand_v[(wave * 2 + 0) * 64 + lane] = bv;
    cand_v[(wave * 2 + 1) * 64 + lane] = sv;
    cand_e[(wave * 2 + 0) * 64 + lane] = be;
    cand_e[(wave * 2 + 1) * 64 + lane] = se;
    __syncthreads();
    // every wavefront merges the candidates of its token, in ascending order of the experts
    bv = cand_v[lane]; sv = cand_v[64 + lane];
    be = cand_e[lane]; se = cand_e[64 + lane];
#pragma unroll
    for (int c = 2; c < 2 * NW; ++c) {
        const float l = cand_v[c * 64 + lane];
        const int e = cand_e[c * 64 + lane];
        const bool first = l > bv;
        const bool second = !first && l > sv;
        sv = first ? bv : second ? l : sv;
        se = first ? be : second ? e : se;
        bv = first ? l : bv;
        be = first ? e : be;
    }
    float den = 0.0f;
#pragma unroll
    for (int j = 0; j < EPW; ++j) den += expf(lg[j] - bv);
    den_part[wave * 64 + lane] = den;
    __syncthreads();
    if (wave != 0 || t >= T) return;
    den = den_part[lane];
#pragma unroll
    for (int w = 1; w < NW; ++w) den += den_part[w * 64 + lane];
    if (finished && finished[t]) {
        // batch pruning (Sec. 3.5): an expert index past the real experts and a zero scale
        for (int j = 0; j < k; ++j) {
            expert_idx[k * t + j] = E;
            expert_scale[k * t + j] = 0.0f;
        }
    } else if (k == 1) {
        expert_idx[t] = be;
        expert_scale[t] = 1.0f / den;
    } else {
        const float e2 = expf(sv - bv);
        float s0 = 1.0f / den, s1 = e2 / den;
        if (renorm) { s0 = 1.0f / (1.0f + e2); s1 = e2 / (1.0f + e2); }
        expert_idx[2 * t] = be;
        expert_idx[2 * t + 1] = se;
        expert_scale[2 * t] = s0;
        expert_scale[2 * t + 1] = s1;
    }
}

}  // namespace moe

extern "C" int moe_gate_topk(const void *x, int act_dtype, const void *wg, const float *bias,
                             const uint8_t *finished, int T, int d, int E, int k, int renormalize,
                             int32_t *expert_idx, float *expert_scale, void *stream)
{
    using namespace moe;
    if (T == 0 && d > 0 && E > 0) return MOE_OK;         // nothing to route (empty buffers may be NULL)
    if (!x || !wg || !expert_idx || !expert_scale) return fail(MOE_ERR_INVALID_ARG, "moe_gate_topk: NULL pointer");
    if (T < 0 || d <= 0 || E <= 0) return fail(MOE_ERR_INVALID_ARG, "moe_gate_topk: T >= 0, d > 0, E > 0 required");
    if (d % 8) return fail(MOE_ERR_INVALID_ARG, "moe_gate_topk: d %% 8 != 0 (d=%d)", d);
    if (k < 1 || k > 2 || k > E) return fail(MOE_ERR_INVALID_ARG, "moe_gate_topk: k must be 1 or 2 and <= E (k=%d E=%d)", k, E);
    if (E > 256) return fail(MOE_ERR_UNSUPPORTED, "moe_gate_topk: E=%d above 256", E);
    if (act_dtype != MOE_F16 && act_dtype != MOE_BF16) return fail(MOE_ERR_UNSUPPORTED, "moe_gate_topk: act_dtype must be fp16 or bf16");
    if (!aligned16(x) || !aligned16(wg)) return fail(MOE_ERR_INVALID_ARG, "moe_gate_topk: x and wg must be 16-byte aligned");
    hipStream_t s = as_stream(stream);
    const bool bf = act_dtype == MOE_BF16;
    if (!bf && E == 64 && d % kGateBlk == 0 && T >= 16384) {     // a token per lane, and a block of 64 tokens for every CU at least
        dim3 grid((T + 63) / 64), block(512);
        const size_t smem = (size_t)4 * 64 * 64 * sizeof(float);
        hipLaunchKernelGGL((gate_token_lanes_kernel<32>), grid, block, smem, s, (const uint16_t *)x, (const uint16_t *)wg,
                           bias, finished, T, d, k, renormalize, expert_idx, expert_scale);
        return check_launch("moe_gate_topk");
    }
    int EL = 8;
    while (EL < E && EL < 64) EL *= 2;
    const int NE = (E + 63) / 64;
    // tokens per lane group: sixteen when every lane group is a whole wavefront and there are
    // enough tokens to fill the chip that way (each block stages the whole gate weight, so more
    // tokens per block mean less staging per token), thirty-two for bf16 rows, which go through
    // LDS (with FP16 rows in scalar registers that many tokens measured twice as slow); else four;
    // one when even that would leave most of the chip idle
    const int tb = (bf && EL == 64 && NE == 1 && T / 32 >= 256) ? 32 : (EL == 64 && T / 16 >= 256) ? 16 : ((long)T * EL / 64 + 3) / 4 >= 256 ? 4 : 1;
    const int ntok = (64 / EL) * tb;
    const size_t wave_halfs = (tb == 16 && NE == 1 && !bf ? 0 : (size_t)ntok * kGateBlk) + (NE == 1 ? (size_t)kGateWRow * kGateBlk : 0);
    const size_t part_bytes = (size_t)4 * (NE == 3 ? 4 : NE) * tb * 64 * 4;      // shares the staging space
    const size_t smem = (size_t)4 * wave_halfs * 2 > part_bytes ? (size_t)4 * wave_halfs * 2 : part_bytes;
    dim3 grid((T + ntok - 1) / ntok), block(256);
    const uint16_t *xp = (const uint16_t *)x, *wp = (const uint16_t *)wg;
#define MOE_GATE_LAUNCH(BF, NEV, TBV, GMV)                                                             \
    do {                                                                                               \
        /* more than 64 KB of dynamic LDS must be asked for once (a local static: once, also across threads) */ \
        static const hipError_t raised = hipFuncSetAttribute(reinterpret_cast<const void *>(&gate_kernel<BF, NEV, TBV, GMV>), \
                                                             hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024); \
        (void)raised;                                                                                  \
        hipLaunchKernelGGL((gate_kernel<BF, NEV, TBV, GMV>), grid, block, smem, s, xp, wp, bias, finished, T, d, E,\
                           EL, k, renormalize, expert_idx, expert_scale);                              \
    } while (0)
#define MOE_GATE_TB(BF, NEV)                                                                           \
    do {                                                                                               \
        if (tb == 16) MOE_GATE_LAUNCH(BF, NEV, 16, 1);                                                 \
        else if (tb == 4) MOE_GATE_LAUNCH(BF, NEV, 4, 8);                                              \
        else MOE_GATE_LAUNCH(BF, NEV, 1, 8);                                                           \
    } while (0)
    if (NE == 1 && tb == 32) MOE_GATE_LAUNCH(true, 1, 32, 1);
    else if (NE == 1) { if (bf) MOE_GATE_TB(true, 1); else MOE_GATE_TB(false, 1); }
    else if (NE == 2) { if (bf) MOE_GATE_TB(true, 2); else MOE_GATE_TB(false, 2); }
    else { if (bf) MOE_GATE_TB(true, 4); else MOE_GATE_TB(false, 4); }
#undef MOE_GATE_TB
#undef MOE_GATE_LAUNCH
    return check_launch("moe_gate_topk");
}
