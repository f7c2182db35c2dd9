// LDS-tiled grouped GEMM with fused dequantisation, for experts with many rows
// (Sec. 3.3 grouped GEMM, Sec. 3.4 fused dequantisation).
//
// Tokens are the MFMA A operand (rows), weights the B operand (columns).  A wavefront fetches
// its weight fragments straight from HBM into registers (one 16-byte load per lane per 1 KB
// fragment block, see moe_common.h), converts the codes to FP16 with the 0x6400 trick and
// feeds v_mfma_f32_32x32x16_f16; only the activations go through LDS (FP16 rows straight from
// global memory, bf16 rows converted on the way), shared by the four wavefronts of a block, each
// of which owns its own 64 output channels.
#pragma once
#include <type_traits>

#include "moe_ffn_common.h"

namespace moe {

constexpr int kLdsRow = 64;              // halfs per LDS row: one K step, no padding; the 16-byte chunks of a row are
                                         // stored at position (k chunk) ^ ((row >> 1) & 7), which makes the b128
                                         // fragment reads conflict-free and keeps a wavefront's 64 chunks contiguous
constexpr int kTN = 2;                   // 32-channel tiles per wavefront

template <int BITS, int SMODE, int TM>
__global__ __launch_bounds__(256, 2) void grouped_gemm_kernel(GemmArgs p)
{
    constexpr int BM = 32 * TM;
    constexpr int NW = BITS == 4 ? 1 : 2;             // 16-byte loads per tile per 64-deep K step
    __shared__ __align__(16) uint16_t lds_a[2][BM * kLdsRow];
    __shared__ int32_t s_dst[BM];          // fused un-permute: destination row and gate scale of each row of the tile
    __shared__ float s_scale[BM];

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: tile addresses stay scalar
    const int K = p.K, N = p.N;
    int e, col, row0, rows;
    if (!find_item(p.offsets, p.E, p.R, 32 * p.tile_units, (N + 255) / 256, blockIdx.x, &e, &col, &row0, &rows)) return;
    e = __builtin_amdgcn_readfirstlane(e), col = __builtin_amdgcn_readfirstlane(col);      // the same in every lane: kept in scalar registers
    row0 = __builtin_amdgcn_readfirstlane(row0), rows = __builtin_amdgcn_readfirstlane(rows);

    if (p.out_dst && (int)threadIdx.x < rows) {       // read long before the epilogue; the K loop's barriers publish it
        const int dst = p.out_dst[row0 + threadIdx.x];
        s_dst[threadIdx.x] = dst;
        s_scale[threadIdx.x] = p.out_scale[dst];
    }
    const int nk = K / 64;
    const int ntile0 = (col * 4 + wave) * kTN;         // first 32-channel tile of this wavefront
    const int ntiles = N / 32;
    bool tile_ok[kTN];
#pragma unroll
    for (int t = 0; t < kTN; ++t) tile_ok[t] = ntile0 + t < ntiles;

    // ---- global addresses
    // A: thread loads 16 bytes = 8 K values of row (tid/8 + 32*pass)
    // thread t fills chunk position t & 7 of LDS row t >> 3 (+ 32 per pass); the K chunk that belongs
    // there is (t & 7) ^ ((row >> 1) & 7), the same for every pass
    const int a_row = threadIdx.x >> 3, a_pos = (threadIdx.x & 7) * 8;
    const int a_seg = ((threadIdx.x & 7) ^ ((threadIdx.x >> 4) & 7)) * 8;
    const uint16_t *a_ptr[TM];
#pragma unroll
    for (int m = 0; m < TM; ++m) {
        const int r = row0 + min(a_row + 32 * m, rows - 1);      // clamped: always a valid row
        const int rs = p.a_src ? p.a_src[r] / p.a_div : r;       // gather fused into the A loads
        a_ptr[m] = p.a + (size_t)rs * K + a_seg;
    }
    // B: fragment blocks of tile t are contiguous along K
    const uint8_t *w_e = p.wq + (size_t)e * packed_bytes_per_expert(K, N, BITS);
    const uint4 *b_ptr[kTN];
#pragma unroll
    for (int t = 0; t < kTN; ++t) {
        const int nt = tile_ok[t] ? ntile0 + t : 0;
        b_ptr[t] = reinterpret_cast<const uint4 *>(w_e + (size_t)nt * (K / frag_k(BITS)) * kFragBytes);   // wave-uniform
    }
    const int G = K / p.g;
    const __half *s_ptr[kTN];
#pragma unroll
    for (int t = 0; t < kTN; ++t) {
        const int nt = tile_ok[t] ? ntile0 + t : 0;
        s_ptr[t] = p.scales + (size_t)e * G * N + nt * 32;              // wave-uniform
    }

    float16_t acc[TM][kTN];
#pragma unroll
    for (int m = 0; m < TM; ++m)
#pragma unroll
        for (int t = 0; t < kTN; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[m][t][i] = 0.0f;

    // SCALE_GROUP_ACC (groups of 128 = the two K steps of one loop trip): the codes enter the MFMAs
    // unscaled (exact), a group's products are summed in accg and folded into acc with the group's
    // scale in fp32.  Exact like the two-term form, at half its MFMA count; needs the registers of a
    // second accumulator set, so it is built for row tiles of at most 64 rows.
    constexpr bool ACC = SMODE == SCALE_GROUP_ACC;
    static_assert(!ACC || TM <= 2, "two accumulator sets fit for TM <= 2 only");
    float16_t accg[ACC ? TM : 1][kTN];

    // Activations are fetched one K step ahead (they come from L2); packed weights and group
    // scales PF = 2 steps ahead, into two register sets used alternately (they come from HBM, and
    // one step of MFMA work is shorter than that latency).  The tallest 8-bit tile has registers
    // for one set only and fetches one step ahead.
    constexpr int PF = (BITS == 8 && TM == 4) ? 1 : 2;
    // The rows (FP16; bf16 rows arrive converted, see rows_to_f16_kernel) go from global memory straight into
    // the LDS stage: no staging registers, no LDS write instructions.
    constexpr int LB = kTN * NW + (SMODE != SCALE_CHANNEL ? kTN : 0);   // loads of one load_b()
    auto dma_a = [&](int kb, uint16_t *stage, int m) {
        load_to_lds16(a_ptr[m] + kb * 64, stage + (32 * m + 8 * wave) * kLdsRow);
    };
    uint4 gb[PF][kTN][NW];
    _Float16 gs[PF][kTN];
    auto load_b = [&](int kb, auto slot_c) {
        constexpr int WS = decltype(slot_c)::value;
#pragma unroll
        for (int t = 0; t < kTN; ++t) {
#pragma unroll
            for (int w = 0; w < NW; ++w) gb[WS][t][w] = (b_ptr[t] + (size_t)(kb * NW + w) * 64)[lane];
            if (SMODE != SCALE_CHANNEL)
                gs[WS][t] = __builtin_bit_cast(_Float16, (s_ptr[t] + (size_t)((kb * 64) / p.g) * N)[lane & 31]);
        }
    };

    const int live = (rows + 31) / 32;
#pragma unroll
    for (int m = 0; m < TM; ++m)
        if (m < live) dma_a(0, lds_a[0], m);
    load_b(0, std::integral_constant<int, 0>{});
    if constexpr (PF == 2) load_b(min(1, nk - 1), std::integral_constant<int, 1>{});
    // Private copies of the steps being computed.  They are taken (and the loads of the next
    // steps issued) once per pair of K steps, at the top of the loop body (PF = 1: at the top of
    // each step): at the loop edge every weight load is then at least a full step old, so the
    // drain of the load counter that the compiler places at a loop head does not wait for fresh loads.
    uint32_t raw2[PF][kTN][NW * 4];
    _Float16 sc2[PF][kTN];
    auto take = [&](auto slot_c) {
        constexpr int WS = decltype(slot_c)::value;
#pragma unroll
        for (int t = 0; t < kTN; ++t) {
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                // real register moves (opaque to the compiler): if it merged these copies with
                // the load registers, the refills would land elsewhere and have to be moved
                // back at the loop edge, i.e. waited for right after being issued
                raw2[WS][t][4 * w + 0] = opaque_copy(gb[WS][t][w].x); raw2[WS][t][4 * w + 1] = opaque_copy(gb[WS][t][w].y);
                raw2[WS][t][4 * w + 2] = opaque_copy(gb[WS][t][w].z); raw2[WS][t][4 * w + 3] = opaque_copy(gb[WS][t][w].w);
            }
            sc2[WS][t] = __builtin_bit_cast(_Float16, (uint16_t)opaque_copy((uint32_t)__builtin_bit_cast(uint16_t, gs[WS][t])));
        }
    };
    // One barrier per step, at its top: it publishes this step's stage (written during the
    // previous step) and tells that every wavefront has left the other stage, which is then
    // refilled at the end of the step, when its rows have had time to arrive; the arrival of
    // the rows is not waited for in front of a barrier.
    auto k_step = [&](int kb, auto slot_c, auto live_c) {
        constexpr int SL = decltype(slot_c)::value;      // = kb & 1: LDS stage and weight register set
        constexpr int LIVE = decltype(live_c)::value;    // row tiles of this block that hold rows
        uint16_t *stage = lds_a[SL];
        // this wavefront's share of the stage has landed once only the weight refills issued after
        // it (in the previous step) are still in flight
        wait_loads<PF == 2 ? (SL == 1 ? 2 * LB : 0) : LB>();
        __syncthreads();
        uint32_t (&raw)[kTN][NW * 4] = raw2[PF == 2 ? SL : 0];
        _Float16 (&sc)[kTN] = sc2[PF == 2 ? SL : 0];
        // The step's loads are dealt over its four MFMA sub-steps, so that the memory pipeline
        // takes a few at a time between matrix instructions: the next step's activation rows in
        // the first two, the weight refills after them (the load counter is in order, so the wait
        // for the rows leaves the younger weight loads in flight).  No branches around the loads:
        // past the end they re-read the last step, which keeps the loop body free of joins and
        // the load counter exact.
        auto issue = [&](int j) {
            const int kn = min(kb + 1, nk - 1);
            if (j < 2) {
#pragma unroll
                for (int m = 0; m < TM; ++m)       // (row tiles past the expert's last row are neither loaded nor written)
                    if (m < LIVE && (TM == 1 ? j == 0 : (m < TM / 2) == (j == 0))) {
                        dma_a(kn, lds_a[1 - SL], m);          // the other stage: every wavefront has left it
                    }
            } else if constexpr (PF == 2) {
                if constexpr (SL == 0) {
                    if (j == 2) load_b(min(kb + 2, nk - 1), std::integral_constant<int, 0>{});
                    else load_b(min(kb + 3, nk - 1), std::integral_constant<int, 1>{});
                }
            } else if (j == 2) {
                load_b(min(kb + 1, nk - 1), std::integral_constant<int, 0>{});
            }
        };

        // unpack + convert one 16-deep step of weight fragments in registers
        auto dequant_step = [&](int j, uint32_t (&bw)[kTN][4], uint32_t (&bl)[kTN][4]) {
#pragma unroll
            for (int t = 0; t < kTN; ++t) {
                if (BITS == 4) dequant4(raw[t][j], bw[t]);
                else dequant8(raw[t][2 * j], raw[t][2 * j + 1], bw[t]);
                if (SMODE == SCALE_GROUP) {
                    const half2_t s2 = {sc[t], sc[t]};
#pragma unroll
                    for (int q = 0; q < 4; ++q) bw[t][q] = h2_bits(bits_h2(bw[t][q]) * s2);
                } else if (SMODE == SCALE_GROUP_SPLIT) {
                    // exact two-term weight: hi = fl(q*s'), lo = q*s' - hi, with s' = 256*s so
                    // that lo stays a normal FP16 number; the epilogue divides by 256
                    const _Float16 s8 = sc[t] * (_Float16)256.0f;
                    const half2_t s2 = {s8, s8};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const half2_t qv = bits_h2(bw[t][q]);
                        const half2_t hi = qv * s2;
                        half2_t lo;
                        lo[0] = __builtin_fmaf16(qv[0], s2[0], -hi[0]);
                        lo[1] = __builtin_fmaf16(qv[1], s2[1], -hi[1]);
                        bw[t][q] = h2_bits(hi);
                        bl[t][q] = h2_bits(lo);
                    }
                }
            }
        };
        // ---- MFMA over the four 16-deep steps of this K slab; the fragments of step j+1 are
        // converted while the MFMAs of step j run (VALU work hides under the matrix pipe)
        // Where the registers allow (PIPE), the A fragments of step j+1 are read from LDS before the
        // MFMAs of step j are issued, so that the LDS latency passes under a full step of matrix
        // work; otherwise each fragment is read just before its MFMAs and the other wavefront of
        // the SIMD covers the wait.
        constexpr bool PIPE = TM < 4 || !(SMODE == SCALE_GROUP_SPLIT || false);
        uint32_t bw[2][kTN][4], bl[2][kTN][4];
        half8_t af[PIPE ? 2 : 1][TM];
        auto read_a = [&](int j, int m) {
            return *reinterpret_cast<const half8_t *>(stage + (32 * m + (lane & 31)) * kLdsRow + 8 * ((2 * j + (lane >> 5)) ^ ((lane >> 1) & 7)));
        };
        auto read_step = [&](int j, half8_t (&dst)[TM]) {
#pragma unroll
            for (int m = 0; m < TM; ++m)
                if (m < LIVE) dst[m] = read_a(j, m);    // row tiles past the expert's last row are skipped
        };
        if (PIPE) read_step(0, af[0]);
        dequant_step(0, bw[0], bl[0]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            issue(j);
            if (PIPE && j + 1 < 4) read_step(j + 1, af[PIPE ? (j + 1) & 1 : 0]);
            __builtin_amdgcn_sched_barrier(0);          // loads and LDS reads stay ahead of this sub-step's MFMAs
            if (j + 1 < 4) dequant_step(j + 1, bw[(j + 1) & 1], bl[(j + 1) & 1]);
#pragma unroll
            for (int m = 0; m < TM; ++m) {
                if (m < LIVE) {
                    const half8_t a = PIPE ? af[PIPE ? j & 1 : 0][m] : read_a(j, m);
#pragma unroll
                    for (int t = 0; t < kTN; ++t) {
                        if constexpr (ACC) {
                            float16_t c = accg[m][t];
                            if (SL == 0 && j == 0)          // first products of a group: start from zero
#pragma unroll
                                for (int i = 0; i < 16; ++i) c[i] = 0.0f;
                            accg[m][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, frag_from(bw[j & 1][t]), c, 0, 0, 0);
                        } else {
                            acc[m][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, frag_from(bw[j & 1][t]), acc[m][t], 0, 0, 0);
                            if (SMODE == SCALE_GROUP_SPLIT)
                                acc[m][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, frag_from(bl[j & 1][t]), acc[m][t], 0, 0, 0);
                        }
                    }
                }
            }
        }
        if constexpr (ACC && SL == 1) {                 // end of the group: acc += scale * accg
#pragma unroll
            for (int t = 0; t < kTN; ++t) {
                const float sf = (float)sc[t];
#pragma unroll
                for (int m = 0; m < TM; ++m)
                    if (m < LIVE)
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[m][t][i] = fmaf(accg[m][t][i], sf, acc[m][t][i]);
            }
        }
    };
    // The K loop exists once per number of live row tiles (the last tile of an expert usually
    // holds few rows): a run-time test inside the loop would cut the MFMA stream into pieces.
    auto k_loop = [&](auto live_c) {
        for (int kb = 0; kb < nk; kb += 2) {
            take(std::integral_constant<int, 0>{});
            if constexpr (PF == 2) take(std::integral_constant<int, PF - 1>{});
            k_step(kb, std::integral_constant<int, 0>{}, live_c);
            if (kb + 1 < nk) {
                if constexpr (PF == 1) take(std::integral_constant<int, 0>{});
                k_step(kb + 1, std::integral_constant<int, 1>{}, live_c);
            }
        }
    };
    if (TM == 1 || live == TM) k_loop(std::integral_constant<int, TM>{});
    else if (TM >= 4 && live == 3) k_loop(std::integral_constant<int, 3>{});
    else if (TM >= 2 && live == 2) k_loop(std::integral_constant<int, 2>{});
    else k_loop(std::integral_constant<int, 1>{});
    wait_loads<0>();      // the last step's (unused) refill of the other stage must land before the block's LDS is given up

    // ---- epilogue: scale (per channel), bias, activation, store.  acc[m][t][i] is row
    // 32*m + 8*(i/4) + 4*(lane/32) + i%4 of the tile, channel lane%32 of tile t.
    // Two channels leave per store: registers i and i+1 are two rows of one channel; a lane
    // hands the row its neighbour (lane ^ 1, the next channel) keeps to that neighbour and gets the
    // other row's value back, so the even lane stores channels (n, n+1) of the first row and the
    // odd lane channels (n-1, n) of the second.
    auto finish = [&](float a, int rl, float cs, float bias) {
        float v = a * cs;
        if (p.row_pow) v *= p.row_pow[row0 + min(rl, rows - 1)].y;     // rows that went in scaled by a power of two (bf16 rows)
        v += bias;
        v = activate(v, p.act);
        if (p.out_dst) v *= s_scale[min(rl, rows - 1)];         // gate scale of the fused un-permute
        return v;
    };
    auto store_tiles = [&](auto out_tag) {
        using OT = decltype(out_tag);                            // float | _Float16 | uint16_t (bf16 bits)
        OT *out = reinterpret_cast<OT *>(p.out);
        // per-channel factors of the wavefront's two tiles first; then, row pair by row pair, both tiles:
        // the two halves of a 128-byte line of the output leave back to back
        float cs[kTN], bias[kTN];
#pragma unroll
        for (int t = 0; t < kTN; ++t) {
            const int n = (tile_ok[t] ? ntile0 + t : 0) * 32 + (lane & 31);       // clamped: always a channel of this expert
            cs[t] = SMODE == SCALE_CHANNEL ? __half2float(p.scales[(size_t)e * N + n]) : SMODE == SCALE_GROUP_SPLIT ? 1.0f / 256.0f : 1.0f;
            bias[t] = p.bias ? __half2float(p.bias[(size_t)e * N + n]) : 0.0f;
        }
#pragma unroll
        for (int m = 0; m < TM; ++m) {
#pragma unroll
            for (int i = 0; i < 16; i += 2) {
                const int rl = 32 * m + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);     // row of register i; i + 1 is the next row
                const bool odd = lane & 1;
                const int rs = rl + (odd ? 1 : 0);
                OT *dst_row = out + (size_t)(p.out_dst ? s_dst[min(rs, rows - 1)] : row0 + rs) * N;
#pragma unroll
                for (int t = 0; t < kTN; ++t) {
                    if (!tile_ok[t]) continue;
                    const int n = (ntile0 + t) * 32 + (lane & 31);
                    const float v0 = finish(acc[m][t][i], rl, cs[t], bias[t]), v1 = finish(acc[m][t][i + 1], rl + 1, cs[t], bias[t]);
                    const float got = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
                                          0, __builtin_bit_cast(int, odd ? v0 : v1), 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
                    const float lo = odd ? got : v0, hi = odd ? v1 : got;
                    if (rs < rows) {
                        OT *dst = dst_row + (n & ~1);
                        if constexpr (std::is_same<OT, float>::value)
                            *reinterpret_cast<float2 *>(dst) = make_float2(lo, hi);
                        else if constexpr (std::is_same<OT, _Float16>::value)
                            *reinterpret_cast<uint32_t *>(dst) = h2_bits(half2_t{(_Float16)lo, (_Float16)hi});
                        else
                            *reinterpret_cast<uint32_t *>(dst) = (uint32_t)to_bf16_rne(lo) | ((uint32_t)to_bf16_rne(hi) << 16);
                    }
                }
            }
        }
    };
    if (p.out_dtype == MOE_F32) store_tiles(float{});
    else if (p.out_dtype == MOE_BF16) store_tiles(uint16_t{});
    else store_tiles(_Float16{});
}

template <int BITS, int SMODE>
static void launch_tm(const GemmArgs &p, int tm, dim3 grid, hipStream_t s)
{
    if (tm == 1) hipLaunchKernelGGL((grouped_gemm_kernel<BITS, SMODE, 1>), grid, dim3(256), 0, s, p);
    else if (tm == 2) hipLaunchKernelGGL((grouped_gemm_kernel<BITS, SMODE, 2>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((grouped_gemm_kernel<BITS, SMODE, 4>), grid, dim3(256), 0, s, p);
}

// All kernels of one weight width and one kind of scale mode (one translation unit each, so that they
// compile side by side): EXACT = the two forms that keep the group scales out of the FP16 weights.
template <int BITS, bool EXACT>
static void launch_tiled_variants(const GemmArgs &p, int smode, int tm, dim3 grid, hipStream_t s)
{
    if constexpr (!EXACT) {
        if (smode == SCALE_CHANNEL) launch_tm<BITS, SCALE_CHANNEL>(p, tm, grid, s);
        else launch_tm<BITS, SCALE_GROUP>(p, tm, grid, s);
    } else if (smode == SCALE_GROUP_ACC) {                 // row tiles of at most 64 rows
        if (tm == 1) hipLaunchKernelGGL((grouped_gemm_kernel<BITS, SCALE_GROUP_ACC, 1>), grid, dim3(256), 0, s, p);
        else hipLaunchKernelGGL((grouped_gemm_kernel<BITS, SCALE_GROUP_ACC, 2>), grid, dim3(256), 0, s, p);
    } else {
        launch_tm<BITS, SCALE_GROUP_SPLIT>(p, tm, grid, s);
    }
}

}  // namespace moe
