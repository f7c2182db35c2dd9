// moe_grouped_ffn_wq: grouped expert GEMM pair with weight-only int4/int8 experts
// (Sec. 3.3 grouped GEMM, Sec. 3.4 fused dequantisation, Sec. 3.4.1-3.4.3 integer-to-FP16
// conversion by magic number).
//
// One GEMM launch computes, for every expert e and its rows r in [off[e], off[e+1]):
//     out[r, n] = epilogue( sum_k A[r, k] * deq(W[e, k, n]) )
// Tokens are the MFMA A operand (rows), weights the B operand (columns).  A wavefront fetches
// its weight fragments straight from HBM into registers (one 16-byte load per lane per 1 KB
// fragment block, see moe_common.h), converts the codes to FP16 with the 0x6400 trick and
// feeds v_mfma_f32_32x32x16_f16; only the activations go through LDS, shared by the four
// wavefronts of a block, each of which owns its own 64 output channels.
#include "moe_common.h"

namespace moe {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

enum { SCALE_CHANNEL = 0, SCALE_GROUP = 1, SCALE_GROUP_SPLIT = 2 };

struct GemmArgs {
    const uint16_t *a;        // [R, K] fp16 or bf16 bit patterns
    const float2 *row_pow;    // bf16 only: per row (2^-p, 2^p) normalisation factors
    const int32_t *offsets;   // [E+1]
    const uint8_t *wq;        // packed codes, [E] x packed_bytes_per_expert
    const __half *scales;     // [E, K/g, N]
    const __half *bias;       // [E, N] or null
    void *out;                // [R, N]
    int E, R, K, N, g;
    int out_dtype, relu;
};

__device__ inline uint32_t h2_bits(half2_t v) { return __builtin_bit_cast(uint32_t, v); }
__device__ inline half2_t bits_h2(uint32_t v) { return __builtin_bit_cast(half2_t, v); }

// Sec. 3.4.1: OR-ing an unsigned code Y < 1024 into the mantissa of FP16 1024.0 (0x6400) gives
// the FP16 number 1024 + Y; an FP16 subtraction of 1024 + offset returns the signed integer,
// exactly.  Two codes are converted per 32-bit register.
//
// 4-bit (Sec. 3.4.3): the eight codes of a dword sit in nibble positions 0,4,1,5,2,6,3,7, so
// (x & 0x000f000f) | 0x64006400 is the pair (i0, i1) + 1024 and (x & 0x00f000f0) | 0x64006400 is
// 16 * (i2, i3) + 1024; the latter is brought back with one fma: v/16 - (64 + 8).
__device__ inline void dequant4(uint32_t x, uint32_t out[4])
{
    const uint32_t magic = 0x64006400u;
    const half2_t sub = {(_Float16)1032.0f, (_Float16)1032.0f};
    const half2_t sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
    const half2_t sub16 = {(_Float16)72.0f, (_Float16)72.0f};
    const uint32_t lo0 = (x & 0x000f000fu) | magic;
    const uint32_t hi0 = (x & 0x00f000f0u) | magic;
    x >>= 8;
    const uint32_t lo1 = (x & 0x000f000fu) | magic;
    const uint32_t hi1 = (x & 0x00f000f0u) | magic;
    out[0] = h2_bits(bits_h2(lo0) - sub);
    out[1] = h2_bits(bits_h2(hi0) * sixteenth - sub16);
    out[2] = h2_bits(bits_h2(lo1) - sub);
    out[3] = h2_bits(bits_h2(hi1) * sixteenth - sub16);
}

// 8-bit (Sec. 3.4.2): four codes (+128) per dword; a byte permute builds 0x64xx64yy for two of
// them at a time, and an FP16 subtraction of 1152 = 1024 + 128 returns the signed integers.
__device__ inline void dequant8(uint32_t w0, uint32_t w1, uint32_t out[4])
{
    const half2_t sub = {(_Float16)1152.0f, (_Float16)1152.0f};
    const uint32_t magic = 0x64646464u;
    out[0] = h2_bits(bits_h2(__builtin_amdgcn_perm(magic, w0, 0x04010400u)) - sub);
    out[1] = h2_bits(bits_h2(__builtin_amdgcn_perm(magic, w0, 0x04030402u)) - sub);
    out[2] = h2_bits(bits_h2(__builtin_amdgcn_perm(magic, w1, 0x04010400u)) - sub);
    out[3] = h2_bits(bits_h2(__builtin_amdgcn_perm(magic, w1, 0x04030402u)) - sub);
}

__device__ inline half8_t frag_from(const uint32_t w[4])
{
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    u4 v = {w[0], w[1], w[2], w[3]};
    return __builtin_bit_cast(half8_t, v);
}

__device__ inline uint16_t to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Finds the (expert, row tile) of tile slot `slot`: experts are walked 64 at a time, each lane
// holding one expert's tile count, with a shuffle scan.  Every wavefront computes the same
// answer; returns false when the slot is past the last tile.
__device__ inline bool find_tile(const int32_t *offsets, int E, int BM, int slot, int *e_out,
                                 int *row0, int *rows)
{
    const int lane = threadIdx.x & 63;
    int base = 0;
    for (int e0 = 0; e0 < E; e0 += 64) {
        const int e = e0 + lane;
        int lo = 0, hi = 0;
        if (e < E) { lo = offsets[e]; hi = offsets[e + 1]; }
        const int tiles = (hi - lo + BM - 1) / BM;
        int incl = tiles;
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        const uint64_t hit = __ballot(base + incl > slot);
        if (hit) {
            const int src = __ffsll((unsigned long long)hit) - 1;
            const int excl = __shfl(incl - tiles, src);
            const int mt = slot - base - excl;
            const int lo_s = __shfl(lo, src), hi_s = __shfl(hi, src);
            *e_out = e0 + src;
            *row0 = lo_s + mt * BM;
            *rows = min(BM, hi_s - (lo_s + mt * BM));
            return true;
        }
        base += __shfl(incl, 63);
    }
    return false;
}

constexpr int kLdsRow = 64 + 8;          // halfs per LDS row: 144-byte stride, conflict-free b128 reads
constexpr int kTN = 2;                   // 32-channel tiles per wavefront

template <int BITS, int SMODE, bool ABF16, int TM>
__global__ __launch_bounds__(256) void grouped_gemm_kernel(GemmArgs p)
{
    constexpr int BM = 32 * TM;
    constexpr int NW = BITS == 4 ? 1 : 2;             // 16-byte loads per tile per 64-deep K step
    __shared__ __align__(16) uint16_t lds_a[2][BM * kLdsRow];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int e, row0, rows;
    if (!find_tile(p.offsets, p.E, BM, blockIdx.y, &e, &row0, &rows)) return;

    const int K = p.K, N = p.N;
    const int nk = K / 64;
    const int ntile0 = (blockIdx.x * 4 + wave) * kTN;  // first 32-channel tile of this wavefront
    const int ntiles = N / 32;
    bool tile_ok[kTN];
#pragma unroll
    for (int t = 0; t < kTN; ++t) tile_ok[t] = ntile0 + t < ntiles;

    // ---- global addresses
    // A: thread loads 16 bytes = 8 K values of row (tid/8 + 32*pass)
    const int a_row = threadIdx.x >> 3, a_seg = (threadIdx.x & 7) * 8;
    const uint16_t *a_ptr[TM];
    float a_down[TM];
#pragma unroll
    for (int m = 0; m < TM; ++m) {
        const int r = row0 + min(a_row + 32 * m, rows - 1);      // clamped: always a valid row
        a_ptr[m] = p.a + (size_t)r * K + a_seg;
        a_down[m] = ABF16 ? p.row_pow[r].x : 1.0f;
    }
    // B: fragment blocks of tile t are contiguous along K
    const uint8_t *w_e = p.wq + (size_t)e * packed_bytes_per_expert(K, N, BITS);
    const uint4 *b_ptr[kTN];
#pragma unroll
    for (int t = 0; t < kTN; ++t) {
        const int nt = tile_ok[t] ? ntile0 + t : 0;
        b_ptr[t] = reinterpret_cast<const uint4 *>(w_e + (size_t)nt * (K / frag_k(BITS)) * kFragBytes) + lane;
    }
    const int G = K / p.g;
    const __half *s_ptr[kTN];
#pragma unroll
    for (int t = 0; t < kTN; ++t) {
        const int nt = tile_ok[t] ? ntile0 + t : 0;
        s_ptr[t] = p.scales + (size_t)e * G * N + nt * 32 + (lane & 31);
    }

    float16_t acc[TM][kTN];
#pragma unroll
    for (int m = 0; m < TM; ++m)
#pragma unroll
        for (int t = 0; t < kTN; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[m][t][i] = 0.0f;

    uint4 ga[TM], gb[kTN][NW];
    _Float16 gs[kTN];
    auto load_global = [&](int kb) {
#pragma unroll
        for (int m = 0; m < TM; ++m) ga[m] = *reinterpret_cast<const uint4 *>(a_ptr[m] + kb * 64);
#pragma unroll
        for (int t = 0; t < kTN; ++t) {
#pragma unroll
            for (int w = 0; w < NW; ++w) gb[t][w] = b_ptr[t][(size_t)(kb * NW + w) * 64];
            if (SMODE != SCALE_CHANNEL) gs[t] = __builtin_bit_cast(_Float16, s_ptr[t][(size_t)((kb * 64) / p.g) * N]);
        }
    };

    load_global(0);
    for (int kb = 0; kb < nk; ++kb) {
        uint16_t *stage = lds_a[kb & 1];
        // ---- activations to LDS (bf16 rows are scaled by a power of two into FP16 range)
#pragma unroll
        for (int m = 0; m < TM; ++m) {
            uint4 v = ga[m];
            if (ABF16) {
                uint32_t in[4] = {v.x, v.y, v.z, v.w}, o[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float f0 = __uint_as_float(in[q] << 16) * a_down[m];
                    const float f1 = __uint_as_float(in[q] & 0xffff0000u) * a_down[m];
                    const half2_t h = {(_Float16)f0, (_Float16)f1};
                    o[q] = h2_bits(h);
                }
                v = make_uint4(o[0], o[1], o[2], o[3]);
            }
            *reinterpret_cast<uint4 *>(stage + (a_row + 32 * m) * kLdsRow + a_seg) = v;
        }
        // ---- this step's weight fragments: unpack + convert in registers
        uint32_t bw[kTN][4][4], bl[kTN][4][4];
#pragma unroll
        for (int t = 0; t < kTN; ++t) {
            uint32_t raw[NW * 4];
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                raw[4 * w + 0] = gb[t][w].x; raw[4 * w + 1] = gb[t][w].y;
                raw[4 * w + 2] = gb[t][w].z; raw[4 * w + 3] = gb[t][w].w;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (BITS == 4) dequant4(raw[j], bw[t][j]);
                else dequant8(raw[2 * j], raw[2 * j + 1], bw[t][j]);
                if (SMODE == SCALE_GROUP) {
                    const half2_t s2 = {gs[t], gs[t]};
#pragma unroll
                    for (int q = 0; q < 4; ++q) bw[t][j][q] = h2_bits(bits_h2(bw[t][j][q]) * s2);
                } else if (SMODE == SCALE_GROUP_SPLIT) {
                    // exact two-term weight: hi = fl(q*s'), lo = q*s' - hi, with s' = 256*s so
                    // that lo stays a normal FP16 number; the epilogue divides by 256
                    const _Float16 s8 = gs[t] * (_Float16)256.0f;
                    const half2_t s2 = {s8, s8};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const half2_t qv = bits_h2(bw[t][j][q]);
                        const half2_t hi = qv * s2;
                        half2_t lo;
                        lo[0] = __builtin_fmaf16(qv[0], s2[0], -hi[0]);
                        lo[1] = __builtin_fmaf16(qv[1], s2[1], -hi[1]);
                        bw[t][j][q] = h2_bits(hi);
                        bl[t][j][q] = h2_bits(lo);
                    }
                }
            }
        }
        __syncthreads();
        if (kb + 1 < nk) load_global(kb + 1);
        // ---- MFMA over the four 16-deep steps of this K slab
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int m = 0; m < TM; ++m) {
                const half8_t af = *reinterpret_cast<const half8_t *>(
                    stage + (32 * m + (lane & 31)) * kLdsRow + 16 * j + 8 * (lane >> 5));
#pragma unroll
                for (int t = 0; t < kTN; ++t) {
                    acc[m][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af, frag_from(bw[t][j]), acc[m][t], 0, 0, 0);
                    if (SMODE == SCALE_GROUP_SPLIT)
                        acc[m][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af, frag_from(bl[t][j]), acc[m][t], 0, 0, 0);
                }
            }
        }
    }

    // ---- epilogue: scale (per channel), bias, ReLU, store.  acc[m][t][i] is row
    // 32*m + 8*(i/4) + 4*(lane/32) + i%4 of the tile, channel lane%32 of tile t.
#pragma unroll
    for (int t = 0; t < kTN; ++t) {
        if (!tile_ok[t]) continue;
        const int n = (ntile0 + t) * 32 + (lane & 31);
        float cs = 1.0f;
        if (SMODE == SCALE_CHANNEL) cs = __half2float(p.scales[(size_t)e * N + n]);
        if (SMODE == SCALE_GROUP_SPLIT) cs = 1.0f / 256.0f;
        const float bias = p.bias ? __half2float(p.bias[(size_t)e * N + n]) : 0.0f;
#pragma unroll
        for (int m = 0; m < TM; ++m) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int rl = 32 * m + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
                if (rl >= rows) continue;
                const int r = row0 + rl;
                float v = acc[m][t][i] * cs;
                if (ABF16) v *= p.row_pow[r].y;
                v += bias;
                if (p.relu) v = fmaxf(v, 0.0f);
                const size_t o = (size_t)r * N + n;
                if (p.out_dtype == MOE_F32) reinterpret_cast<float *>(p.out)[o] = v;
                else if (p.out_dtype == MOE_BF16) reinterpret_cast<uint16_t *>(p.out)[o] = to_bf16_rne(v);
                else reinterpret_cast<_Float16 *>(p.out)[o] = (_Float16)v;
            }
        }
    }
}

// Per-row power-of-two normalisation of bf16 activations: pow.x = 2^-p brings the row's
// largest magnitude into [2^14, 2^15) so that every element converts to FP16 without
// overflow and with its 8-bit significand intact; pow.y = 2^p undoes it after the GEMM.
__global__ __launch_bounds__(256) void row_pow_kernel(const uint16_t *__restrict__ a, int R, int K,
                                                      float2 *__restrict__ row_pow)
{
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= R) return;
    const uint4 *row = reinterpret_cast<const uint4 *>(a + (size_t)r * K);
    uint32_t amax = 0;
    for (int v = lane; v < K / 8; v += 64) {
        const uint4 q = row[v];
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            amax = max(amax, w[i] & 0x7fffu);
            amax = max(amax, (w[i] >> 16) & 0x7fffu);
        }
    }
    for (int off = 32; off > 0; off >>= 1) amax = max(amax, (uint32_t)__shfl_xor((int)amax, off));
    if (lane == 0) {
        int ex = (int)(amax >> 7);                 // biased exponent of the largest magnitude
        if (ex == 255) ex = 141;                   // inf/nan rows: factor 1 (the result is nan anyway)
        int fe = 268 - ex;                         // biased exponent of 2^(14 - (ex - 127))
        fe = min(max(fe, 1), 253);
        row_pow[r] = make_float2(__uint_as_float((uint32_t)fe << 23), __uint_as_float((uint32_t)(254 - fe) << 23));
    }
}

template <int BITS, int SMODE, bool ABF16>
static void launch_tm(const GemmArgs &p, int tm, dim3 grid, hipStream_t s)
{
    if (tm == 1) hipLaunchKernelGGL((grouped_gemm_kernel<BITS, SMODE, ABF16, 1>), grid, dim3(256), 0, s, p);
    else if (tm == 2) hipLaunchKernelGGL((grouped_gemm_kernel<BITS, SMODE, ABF16, 2>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((grouped_gemm_kernel<BITS, SMODE, ABF16, 4>), grid, dim3(256), 0, s, p);
}

template <int BITS>
static void launch_mode(const GemmArgs &p, int smode, bool abf16, int tm, dim3 grid, hipStream_t s)
{
    if (smode == SCALE_CHANNEL) {
        if (abf16) launch_tm<BITS, SCALE_CHANNEL, true>(p, tm, grid, s);
        else launch_tm<BITS, SCALE_CHANNEL, false>(p, tm, grid, s);
    } else if (smode == SCALE_GROUP) {
        if (abf16) launch_tm<BITS, SCALE_GROUP, true>(p, tm, grid, s);
        else launch_tm<BITS, SCALE_GROUP, false>(p, tm, grid, s);
    } else {
        if (abf16) launch_tm<BITS, SCALE_GROUP_SPLIT, true>(p, tm, grid, s);
        else launch_tm<BITS, SCALE_GROUP_SPLIT, false>(p, tm, grid, s);
    }
}

static int launch_gemm(const GemmArgs &p, int bits, int smode, bool abf16, hipStream_t s)
{
    // row-tile height from the mean rows per expert (the offsets themselves stay on the device)
    const int mean = (p.R + p.E - 1) / p.E;
    const int tm = mean <= 32 ? 1 : mean <= 64 ? 2 : 4;
    const int bm = 32 * tm;
    const long slots = (long)p.R / bm + (p.E < p.R ? p.E : p.R);
    if (slots > 65535) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq: %ld row tiles exceed one launch", slots);
    dim3 grid((p.N + 255) / 256, (unsigned)slots);
    if (bits == 4) launch_mode<4>(p, smode, abf16, tm, grid, s);
    else launch_mode<8>(p, smode, abf16, tm, grid, s);
    return check_launch("moe_grouped_ffn_wq (gemm)");
}

struct FfnWorkspace {
    size_t h_off, pow_x_off, pow_h_off, total;
};

static FfnWorkspace ffn_workspace(int R, int d, int F, int act_dtype)
{
    (void)d;
    FfnWorkspace w;
    size_t o = 0;
    w.h_off = o;
    o += round_up((size_t)R * F * 2, 256);
    w.pow_x_off = o;
    if (act_dtype == MOE_BF16) o += round_up((size_t)R * sizeof(float2), 256);
    w.pow_h_off = o;
    if (act_dtype == MOE_BF16) o += round_up((size_t)R * sizeof(float2), 256);
    w.total = o < 256 ? 256 : o;
    return w;
}

}  // namespace moe

extern "C" size_t moe_grouped_ffn_wq_workspace_bytes(int R, int d, int F, int E, int act_dtype)
{
    (void)E;
    if (R <= 0 || d <= 0 || F <= 0) return 256;
    return moe::ffn_workspace(R, d, F, act_dtype).total;
}

extern "C" int moe_grouped_ffn_wq(const void *x_perm, int act_dtype, const int32_t *expert_offsets, int R,
                                  int E, int d, int F, int bits, int group_size, const void *w1_packed,
                                  const void *s1, const void *b1, const void *w2_packed, const void *s2,
                                  const void *b2, void *y_perm, int y_dtype, void *workspace,
                                  size_t workspace_bytes, void *stream)
{
    using namespace moe;
    if (!expert_offsets || !w1_packed || !s1 || !w2_packed || !s2 || (R != 0 && (!x_perm || !y_perm)))
        return fail(MOE_ERR_INVALID_ARG, "moe_grouped_ffn_wq: NULL pointer");
    if (R < 0 || E <= 0 || d <= 0 || F <= 0) return fail(MOE_ERR_INVALID_ARG, "moe_grouped_ffn_wq: R >= 0 and E, d, F > 0 required");
    if (d % 64 || F % 64) return fail(MOE_ERR_INVALID_ARG, "moe_grouped_ffn_wq: d and F must be multiples of 64 (d=%d F=%d)", d, F);
    if (bits != 4 && bits != 8) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq: bits must be 4 or 8 (got %d)", bits);
    if (act_dtype != MOE_F16 && act_dtype != MOE_BF16) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq: act_dtype must be fp16 or bf16");
    if (y_dtype != MOE_F16 && y_dtype != MOE_BF16 && y_dtype != MOE_F32) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq: unknown y_dtype %d", y_dtype);
    if (group_size < 0 || (group_size && (group_size % 64 || d % group_size || F % group_size)))
        return fail(MOE_ERR_INVALID_ARG, "moe_grouped_ffn_wq: group_size %d must be 0 or a multiple of 64 dividing d and F", group_size);
    if (E > 4096) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq: E=%d above 4096", E);
    const void *ptrs[] = {x_perm, w1_packed, s1, b1, w2_packed, s2, b2, y_perm, workspace};
    for (const void *q : ptrs)
        if (!aligned16(q)) return fail(MOE_ERR_INVALID_ARG, "moe_grouped_ffn_wq: buffers must be 16-byte aligned");
    const FfnWorkspace ws = ffn_workspace(R, d, F, act_dtype);
    if (!workspace || workspace_bytes < ws.total)
        return fail(MOE_ERR_WORKSPACE, "moe_grouped_ffn_wq: workspace of %zu bytes needed, %zu given", ws.total, workspace_bytes);
    if (R == 0) return MOE_OK;

    hipStream_t s = as_stream(stream);
    const bool bf = act_dtype == MOE_BF16;
    unsigned char *wsb = (unsigned char *)workspace;
    void *h = wsb + ws.h_off;
    float2 *pow_x = (float2 *)(wsb + ws.pow_x_off), *pow_h = (float2 *)(wsb + ws.pow_h_off);
    const bool grouped = group_size != 0 && !(group_size == d && group_size == F);

    // fc1: h = relu(x_perm @ deq(W1) + b1), stored in the activation dtype.  With bf16
    // activations and group scales the weights go in as an exact two-term FP16 sum, because h
    // is rounded to 8 bits afterwards and a 2^-11 weight rounding would show through.
    GemmArgs g1{};
    g1.a = (const uint16_t *)x_perm; g1.row_pow = pow_x; g1.offsets = expert_offsets;
    g1.wq = (const uint8_t *)w1_packed; g1.scales = (const __half *)s1; g1.bias = (const __half *)b1;
    g1.out = h; g1.E = E; g1.R = R; g1.K = d; g1.N = F; g1.g = grouped ? group_size : d;
    g1.out_dtype = act_dtype; g1.relu = 1;
    if (bf) {
        hipLaunchKernelGGL(row_pow_kernel, dim3((R + 3) / 4), dim3(256), 0, s, (const uint16_t *)x_perm, R, d, pow_x);
        int rc = check_launch("moe_grouped_ffn_wq (row scale x)");
        if (rc) return rc;
    }
    int rc = launch_gemm(g1, bits, grouped ? (bf ? SCALE_GROUP_SPLIT : SCALE_GROUP) : SCALE_CHANNEL, bf, s);
    if (rc) return rc;

    // fc2: y = h @ deq(W2) + b2
    GemmArgs g2 = g1;
    g2.a = (const uint16_t *)h; g2.row_pow = pow_h;
    g2.wq = (const uint8_t *)w2_packed; g2.scales = (const __half *)s2; g2.bias = (const __half *)b2;
    g2.out = y_perm; g2.K = F; g2.N = d; g2.g = grouped ? group_size : F;
    g2.out_dtype = y_dtype; g2.relu = 0;
    if (bf) {
        hipLaunchKernelGGL(row_pow_kernel, dim3((R + 3) / 4), dim3(256), 0, s, (const uint16_t *)h, R, F, pow_h);
        rc = check_launch("moe_grouped_ffn_wq (row scale h)");
        if (rc) return rc;
    }
    return launch_gemm(g2, bits, grouped ? SCALE_GROUP : SCALE_CHANNEL, bf, s);
}
