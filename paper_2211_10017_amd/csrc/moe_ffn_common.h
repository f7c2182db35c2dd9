// Device helpers shared by the grouped-GEMM kernels: argument block, the magic-number
// integer-to-FP16 conversions (Sec. 3.4.1-3.4.3) and the tile lookup.
#pragma once

#include "moe_common.h"

namespace moe {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

enum { SCALE_CHANNEL = 0, SCALE_GROUP = 1, SCALE_GROUP_SPLIT = 2, SCALE_GROUP_ACC = 3 };

struct GemmArgs {
    const uint16_t *a;        // [R, K] fp16 bit patterns (rows that were bf16 come converted, scaled by 2^-p per row)
    const float2 *row_pow;    // null, or per row (2^-p, 2^p): the tiled kernel multiplies its output rows by 2^p
    const int32_t *offsets;   // [E+1]
    const uint8_t *wq;        // packed codes, [E] x packed_bytes_per_expert
    const __half *scales;     // [E, K/g, N]
    const __half *bias;       // [E, N] or null
    void *out;                // [R, N]
    int E, R, K, N, g;
    int out_dtype;
    int act;                  // MOE_ACT_NONE (plain GEMM) | MOE_ACT_RELU | MOE_ACT_GELU applied after the bias
    int tile_units;           // tiled kernel: row tiles of at most 32 * tile_units rows (set by the launcher)
    // tiled kernel only: rows fetched / stored through the routing index instead of a permuted copy
    const int32_t *a_src;     // [R] or null: row r of A is a[a_src[r] / a_div]
    int a_div;
    const int32_t *out_dst;   // [R] or null: row r of the result goes to out[out_dst[r]], times out_scale[out_dst[r]]
    const float *out_scale;
    // straight-line streaming kernel only (decode-sized batches): the permutation is rebuilt from the
    // gate's output inside the launch.  gate_idx[a] is the expert of assignment a (E = pruned row),
    // row a / gate_k of `a` is its token; the first block of every expert writes the index arrays.
    const int32_t *gate_idx;  // [n_assign] or null
    int n_assign, gate_k;
    int32_t *perm_src_out, *inv_perm_out, *offsets_out;
    float *zero_out;          // or null: fp32 buffer the launch clears (zero_count floats, a multiple of 4) for the
    long zero_count;          // launch after it, which adds rows into it
    // straight-line streaming kernel, fused un-permute for k <= 2: with out_add set, row r of the result,
    // times out_scale[a], a = out_dst[r], is ADDED to row a / out_div of the fp32 buffer `out` (cleared
    // before).  A token's at most two terms arrive in either order; fp32 addition of two terms onto
    // zero is commutative, so the sum does not depend on it.
    int out_add, out_div;
};

// FFN of a decode-sized batch: one streaming launch plus a small reduction (moe_ffn_decode.hip).
struct DecodeArgs {
    const uint16_t *x;          // [T, d] fp16, un-permuted
    const int32_t *gate_idx;    // [n_assign] expert of assignment a (E = pruned row)
    const float *gate_scale;    // [n_assign] gate scale of assignment a
    int n_assign, gate_k;
    int E, d, F, act;
    const uint8_t *w1, *w2;     // packed codes
    const __half *s1, *s2;      // per-channel scales [E, F] / [E, d]
    const __half *b1, *b2;      // biases or null
    float *partial;             // [F / 512, n_assign, d] fp32: y summed over one 512-channel slice of d_ff
    float *out;                 // [T, d] fp32 layer output
    int32_t *perm_src_out, *inv_perm_out, *offsets_out;
    int items1;                 // workgroup items (set by the launcher)
    int early_ring;             // an item requests its first weights before it knows the expert's row count (set by the launcher)
};
constexpr int kDecMaxExperts = 4096;
bool decode_ffn_supports(int n_assign, int E, int d, int F, int bits);
size_t decode_ffn_partial_bytes(int n_assign, int d, int F);
int launch_decode_ffn(const DecodeArgs &p, int bits, hipStream_t s);

constexpr int kGatedMaxAssign = 256;    // assignments the fused permutation takes: one per thread of a block

int launch_tiled_gemm(const GemmArgs &p, int bits, int smode, hipStream_t s);
void launch_tiled_4(const GemmArgs &p, int smode, int tm, dim3 grid, hipStream_t s);
void launch_tiled_4_exact(const GemmArgs &p, int smode, int tm, dim3 grid, hipStream_t s);
void launch_tiled_8(const GemmArgs &p, int smode, int tm, dim3 grid, hipStream_t s);
void launch_tiled_8_exact(const GemmArgs &p, int smode, int tm, dim3 grid, hipStream_t s);
int launch_stream_gemm(const GemmArgs &p, int bits, int smode, int max_rows, hipStream_t s);
bool stream_gemm_supports(int K, int bits, int smode);
int stream_gemm_fit_rows(int K);
bool stream_unrolled_supports(int K, int bits, int smode);
int stream_unrolled_fit(int K, int max_rows);
bool stream_unrolled_takes_gate(int K, int bits);
int launch_stream_unrolled(const GemmArgs &p, int bits, int max_rows, hipStream_t s);
int launch_stream_unrolled_variant(const GemmArgs &p, int bits, bool native, int max_rows, hipStream_t s);

enum { MOE_ACT_NONE = -1 };

// The activation between the two GEMMs.  GELU in its exact form x * Phi(x).
__device__ inline float activate(float v, int act)
{
    if (act == MOE_ACT_RELU) return fmaxf(v, 0.0f);
    if (act == MOE_ACT_GELU) return 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f));
    return v;
}

__device__ inline uint32_t h2_bits(half2_t v) { return __builtin_bit_cast(uint32_t, v); }
__device__ inline half2_t bits_h2(uint32_t v) { return __builtin_bit_cast(half2_t, v); }

// Sec. 3.4.1: OR-ing an unsigned code Y < 1024 into the mantissa of FP16 1024.0 (0x6400) gives
// the FP16 number 1024 + Y; an FP16 subtraction of 1024 + offset returns the signed integer,
// exactly.  Two codes are converted per 32-bit register.
//
// 4-bit (Sec. 3.4.3): the eight codes of a dword sit in nibble positions 0,4,1,5,2,6,3,7, so
// (x & 0x000f000f) | 0x64006400 is the pair (i0, i1) + 1024 and (x & 0x00f000f0) | 0x64006400 is
// 16 * (i2, i3) + 1024; the latter is brought back with one fma: v/16 - (64 + 8).
// A register-to-register move that the compiler cannot fold away.
__device__ inline uint32_t opaque_copy(uint32_t x)
{
    uint32_t r;
    asm volatile("v_mov_b32 %0, %1" : "=v"(r) : "v"(x));
    return r;
}

// (x & mask) | magic in one VALU instruction.  The compiler prefers two VOP2 instructions with
// literal operands here (VOP3 cannot encode literals on this target), so the instruction is
// spelled out, with mask and magic held in registers.
__device__ inline uint32_t and_or(uint32_t x, uint32_t mask, uint32_t magic)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(mask), "v"(magic));
    return r;
}

__device__ inline void dequant4(uint32_t x, uint32_t out[4])
{
    const uint32_t magic = 0x64006400u, mlo = 0x000f000fu, mhi = 0x00f000f0u;
    const half2_t sub = {(_Float16)1032.0f, (_Float16)1032.0f};
    const half2_t sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
    const half2_t sub16 = {(_Float16)72.0f, (_Float16)72.0f};
    const uint32_t lo0 = and_or(x, mlo, magic);
    const uint32_t hi0 = and_or(x, mhi, magic);
    x >>= 8;
    const uint32_t lo1 = and_or(x, mlo, magic);
    const uint32_t hi1 = and_or(x, mhi, magic);
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

// The same conversions with the chip's integer-to-float instructions instead of the magic
// number (the variant Sec. 3.4.1 measured as too slow on its hardware): extract the code, convert
// to fp32, remove the offset, round to FP16.  Exact, like the magic-number route.
__device__ inline void dequant4_native(uint32_t x, uint32_t out[4])
{
    // codes of MFMA index i sit in nibble position {0,4,1,5,2,6,3,7}[i]
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float lo = (float)((x >> (4 * q)) & 15u) - 8.0f;        // index 2q
        const float hi = (float)((x >> (4 * q + 16)) & 15u) - 8.0f;   // index 2q + 1
        const half2_t h = {(_Float16)lo, (_Float16)hi};
        out[q] = h2_bits(h);
    }
}

__device__ inline void dequant8_native(uint32_t w0, uint32_t w1, uint32_t out[4])
{
    const uint32_t w[2] = {w0, w1};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float lo = (float)((w[q >> 1] >> (16 * (q & 1))) & 255u) - 128.0f;
        const float hi = (float)((w[q >> 1] >> (16 * (q & 1) + 8)) & 255u) - 128.0f;
        const half2_t h = {(_Float16)lo, (_Float16)hi};
        out[q] = h2_bits(h);
    }
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

__device__ inline void store_out(void *out, int dtype, size_t o, float v)
{
    if (dtype == MOE_F32) reinterpret_cast<float *>(out)[o] = v;
    else if (dtype == MOE_BF16) reinterpret_cast<uint16_t *>(out)[o] = to_bf16_rne(v);
    else reinterpret_cast<_Float16 *>(out)[o] = (_Float16)v;
}

// 16 bytes per lane from global memory straight into LDS: lane l's bytes land at dst + 16 l, dst
// the same for the whole wavefront.  Written as assembly so that the compiler's load counter
// does not see it (it would take loads of two kinds to be in flight and wait for all of them at
// the first use of any).  The caller waits for it by hand with wait_loads<N>(), N = the loads
// issued after it that may stay in flight: the counter retires loads in order, and the waits the
// compiler places for its own loads can only be stricter for the ones it does not see.
__device__ inline void load_to_lds16(const void *src, uint16_t *dst)
{
    const uint32_t l = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)dst;
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(l) : "memory", "m0");
}

// s_waitcnt vmcnt(N) alone (the other counters' fields say "no wait").
// Built with MOE_WAIT_ALL_LOADS every such wait is for ALL outstanding loads: slower, but free of any
// assumption about how many loads the compiler issues after a direct-to-LDS load.  The library is built
// a second time that way (libmoe_wq_waitall.so) and a GPU test compares the two builds bit for bit, so a
// compiler that merges, splits or reorders one of the counted loads shows up as a failing test, not as
// silently stale rows in LDS.
template <int N>
__device__ inline void wait_loads()
{
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
#ifdef MOE_WAIT_ALL_LOADS
    __builtin_amdgcn_s_waitcnt(0x0f70);
#else
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
#endif
}

// Inclusive prefix sum over the 64 lanes in the VALU's data-parallel primitives: shifts by 1, 2, 4
// and 8 inside each row of 16 lanes (zero shifted in), then the last lane of rows 0 and 2 added to rows
// 1 and 3, then lane 31 added to rows 2 and 3.  All lanes must be active.
__device__ inline int wave_inclusive_sum(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);     // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);     // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);     // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);     // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);    // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);    // row_bcast:31 into rows 2 and 3
    return v;
}

// Work distribution of the tiled kernel.  A work item is (expert, column block, row tile); the
// items are ordered expert-major, then by column block, row tile fastest, so that neighbours in
// the order share a weight column block (row tiles of one expert) or an activation row tile
// (column blocks of one expert).  The chip's workgroups go round-robin to its 8 XCDs, each with
// an L2 of its own: workgroup id w runs on XCD w % 8, so XCD x is given the x-th contiguous
// eighth of the order, walked in order by its workgroups w / 8.  What runs together on one XCD
// then streams the same few row tiles and weight blocks through that XCD's L2.
// Every wavefront computes the same answer; returns false when this workgroup has no item.
constexpr int kXcds = 8;

// Expert e's row range, forced into [0, R] and non-negative length: offsets that are not a
// monotone partition of the R rows then give wrong results but no access outside the buffers.
__device__ inline void expert_range(const int32_t *offsets, int e, int R, int *lo, int *hi)
{
    const int l = min(max(offsets[e], 0), R);
    *lo = l;
    *hi = min(max(offsets[e + 1], l), R);
}

__device__ inline bool find_item(const int32_t *offsets, int E, int R, int BM, int ncol, int wg,
                                 int *e_out, int *col, int *row0, int *rows)
{
    const int lane = threadIdx.x & 63;
    // row tiles of the experts of one 64-lane chunk, with their inclusive prefix sum over the chunk
    auto chunk_tiles = [&](int e0, int &lo, int &hi, int &tiles, int &incl) {
        const int e = e0 + lane;
        lo = 0, hi = 0;
        if (e < E) expert_range(offsets, e, R, &lo, &hi);
        tiles = (hi - lo + BM - 1) / BM;
        incl = wave_inclusive_sum(tiles);
    };
    int total = 0;                                     // row tiles of all experts
    int lo0, hi0, tiles0, incl0;                       // the first chunk is kept: with E <= 64 the offsets are read once
    chunk_tiles(0, lo0, hi0, tiles0, incl0);
    total = __shfl(incl0, 63);
    for (int e0 = 64; e0 < E; e0 += 64) {
        int lo, hi, tiles, incl;
        chunk_tiles(e0, lo, hi, tiles, incl);
        total += __shfl(incl, 63);
    }
    const long items = (long)total * ncol;
    const long chunk = (items + kXcds - 1) / kXcds;
    const long s = wg / kXcds;
    const long item = (wg % kXcds) * chunk + s;
    if (s >= chunk || item >= items) return false;
    int base = 0;
    for (int e0 = 0; e0 < E; e0 += 64) {
        int lo = lo0, hi = hi0, tiles = tiles0, incl = incl0;
        if (e0) chunk_tiles(e0, lo, hi, tiles, incl);
        const uint64_t hit = __ballot((long)(base + incl) * ncol > item);
        if (hit) {
            const int src = __ffsll((unsigned long long)hit) - 1;
            const int t_e = __shfl(tiles, src);
            const int excl = __shfl(incl - tiles, src);
            const int local = (int)(item - (long)(base + excl) * ncol);
            const int c = local / t_e, mt = local % t_e;
            const int lo_s = __shfl(lo, src), hi_s = __shfl(hi, src);
            // The expert's rows, in units of 32 (one MFMA row tile), are dealt evenly to its t_e
            // tiles: 270 rows become 96 + 96 + 78 rather than 128 + 128 + 14, the same matrix
            // work without a nearly empty tile that streams a whole weight block for 14 rows.
            const int units = (hi_s - lo_s + 31) / 32, per = units / t_e, extra = units % t_e;
            const int first = lo_s + 32 * (mt * per + min(mt, extra));
            *e_out = e0 + src;
            *col = c;
            *row0 = first;
            *rows = min(32 * (per + (mt < extra ? 1 : 0)), hi_s - first);
            return true;
        }
        base += __shfl(incl, 63);
    }
    return false;
}

}  // namespace moe
