// moe_grouped_ffn_wq: grouped expert GEMM pair with weight-only int4/int8 experts
// (Sec. 3.3 grouped GEMM, Sec. 3.4 fused dequantisation).  This file holds the entry point:
// argument checks, workspace layout and the choice between the weight-streaming kernel
// (experts with few rows, HBM-bound) and the LDS-tiled kernel (experts with many rows,
// MFMA-bound).
#include <mutex>

#include "moe_ffn_common.h"

namespace moe {

// bf16 rows -> FP16 rows scaled by a power of two per row: pow.x = 2^-p brings the row's largest magnitude
// into [2^14, 2^15), so that every element converts to FP16 without overflow; the GEMM takes the result like
// FP16 rows (straight from memory into LDS) and multiplies its output rows by pow.y = 2^p.  A value keeps its 8-bit significand unless it is more than 2^-28 below the row's largest, where FP16
// runs out of exponent.  `out` may be `in`: a lane reads what it converts before it writes it, and the row's
// largest magnitude is known before the first write.
__global__ __launch_bounds__(256) void rows_to_f16_kernel(const uint16_t *in, uint16_t *out, int R, int K, float2 *__restrict__ row_pow)
{
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= R) return;
    const uint4 *row = reinterpret_cast<const uint4 *>(in + (size_t)r * K);
    uint4 *dst = reinterpret_cast<uint4 *>(out + (size_t)r * K);
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
    int ex = (int)(amax >> 7);                     // biased exponent of the largest magnitude
    if (ex == 255) ex = 141;                       // inf/nan rows: factor 1 (the result is nan anyway)
    int fe = 268 - ex;                             // biased exponent of 2^(14 - (ex - 127))
    fe = min(max(fe, 1), 253);
    const float down = __uint_as_float((uint32_t)fe << 23);
    if (lane == 0) row_pow[r] = make_float2(down, __uint_as_float((uint32_t)(254 - fe) << 23));
    for (int v = lane; v < K / 8; v += 64) {
        const uint4 q = row[v];
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
        uint32_t o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const half2_t h = {(_Float16)(__uint_as_float(w[i] << 16) * down), (_Float16)(__uint_as_float(w[i] & 0xffff0000u) * down)};
            o[i] = h2_bits(h);
        }
        dst[v] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

struct FfnWorkspace {
    size_t h_off, pow_x_off, pow_h_off, x16_off, partial_off, total;
};

static FfnWorkspace ffn_workspace(int R, int d, int F, int act_dtype)
{
    FfnWorkspace w;
    size_t o = 0;
    w.h_off = o;
    o += round_up((size_t)R * F * 2, 256);
    w.pow_x_off = o;
    if (act_dtype == MOE_BF16) o += round_up((size_t)R * sizeof(float2), 256);
    w.pow_h_off = o;
    if (act_dtype == MOE_BF16) o += round_up((size_t)R * sizeof(float2), 256);
    w.x16_off = o;                               // bf16 rows: x converted to scaled FP16 (h is converted in place)
    if (act_dtype == MOE_BF16) o += round_up((size_t)R * d * 2, 256);
    w.partial_off = o;                           // decode kernel: partial sums of y per d_ff slice
    if (R <= kGatedMaxAssign && F % 512 == 0) o += round_up(decode_ffn_partial_bytes(R, d, F), 256);
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

// Which kernel one GEMM of the FFN runs in, from what the host knows about the routed loads: an upper
// bound on the rows of any expert and the mean rows per expert.
enum GemmKernel { GEMM_TILED, GEMM_STREAM_UNROLLED, GEMM_STREAM_LOOP };

static GemmKernel choose_kernel(int R, int E, int max_rows, int K, int N, int bits, int smode, bool bf)
{
    using namespace moe;
    if (bf || !stream_gemm_supports(K, bits, smode)) return GEMM_TILED;
    const int mean = (R + E - 1) / E;
    const bool unrolled = stream_unrolled_supports(K, bits, smode);
    // rows of an expert one block of the streaming kernel holds; an expert with more rows takes further
    // blocks (row groups), each of which streams the expert's weights again
    const int fit = unrolled ? stream_unrolled_fit(K, max_rows) : stream_gemm_fit_rows(K);
    // Streaming takes a row bound that needs few row groups: at most 64 rows, or at most 32 rows per
    // expert on average and at most sixteen groups ...
    const bool few = unrolled && mean <= 32 && max_rows <= 16 * fit;
    if (!(max_rows <= 64 || few)) return GEMM_TILED;
    // ... and it pays while the typical expert is one row group (measured on 32 experts of 1024 x 4096:
    // 34 us up to 8 rows per expert, 47 at 16, 69 at 24, against 49 us in row tiles at any of these), or
    // the batch is decode-sized, or row tiles would leave most of the chip idle (one tile per expert and
    // column block: 8 experts of 512 x 2048 stream in 16 us and take 30 us in 64 + 16 tiles).
    const long tiles = (long)(E < R ? E : R) * ((N + 255) / 256);
    if (R <= 256 || mean <= fit || tiles < 128) return unrolled ? GEMM_STREAM_UNROLLED : GEMM_STREAM_LOOP;
    return GEMM_TILED;
}

// bf: the rows were bf16 (they come in converted to scaled FP16, with their factors in g.row_pow, which only the
// tiled kernel applies)
static int run_gemm(moe::GemmArgs g, int bits, int smode, bool bf, int max_rows, hipStream_t s)
{
    using namespace moe;
    const GemmKernel kernel = choose_kernel(g.R, g.E, max_rows, g.K, g.N, bits, smode, bf);
    note_kernel(kernel == GEMM_STREAM_UNROLLED ? "stream_unrolled_kernel" : kernel == GEMM_STREAM_LOOP ? "stream_gemm_kernel" : "grouped_gemm_kernel");
    if (kernel == GEMM_STREAM_UNROLLED) return launch_stream_unrolled(g, bits, max_rows, s);
    if (g.gate_idx || g.out_add) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq_gated: K=%d does not run in the straight-line kernel with these sizes", g.K);
    if (kernel == GEMM_STREAM_LOOP) return launch_stream_gemm(g, bits, smode, max_rows, s);
    // Everything else runs in the tiled kernel, experts with a handful of rows included: their tiles skip
    // the row blocks that hold no rows and stream the weights as fast as the streaming kernel would
    // (sending them there in a launch of their own measured 2-25 % slower on skewed loads).
    return launch_tiled_gemm(g, bits, smode, s);
}

// true when a call with these sizes runs both GEMMs in the tiled kernel (the only kernel that takes
// rows through the routing index)
static bool tiled_only(int R, int E, int max_rows, int d, int F, int bits, bool grouped, bool bf)
{
    using namespace moe;
    const int smode = grouped ? SCALE_GROUP : SCALE_CHANNEL;
    return choose_kernel(R, E, max_rows, d, F, bits, smode, bf) == GEMM_TILED &&
           choose_kernel(R, E, max_rows, F, d, bits, smode, bf) == GEMM_TILED;
}

static int ffn_impl(const void *x_perm, int act_dtype, const int32_t *expert_offsets, int R,
                    int E, int max_rows_per_expert, int d, int F, int bits, int group_size, int activation,
                    const void *w1_packed,
                    const void *s1, const void *b1, const void *w2_packed, const void *s2,
                    const void *b2, void *y_perm, int y_dtype, void *workspace,
                    size_t workspace_bytes, void *stream,
                    const int32_t *perm_src, int k, const float *expert_scale,
                    const int32_t *gate_idx = nullptr, int32_t *perm_src_out = nullptr, int32_t *inv_perm_out = nullptr,
                    int32_t *offsets_out = nullptr)
{
    using namespace moe;
    // (y_perm may be NULL only on the decode kernel's path, where it means "leave out the slice reduction")
    const bool partial_only = !y_perm && gate_idx && expert_scale && act_dtype == MOE_F16 && group_size == 0 &&
                              moe::decode_ffn_supports(R, E, d, F, bits);
    if (!expert_offsets || !w1_packed || !s1 || !w2_packed || !s2 || (R != 0 && (!x_perm || (!y_perm && !partial_only))))
        return fail(MOE_ERR_INVALID_ARG, "moe_grouped_ffn_wq: NULL pointer");
    if (R < 0 || E <= 0 || d <= 0 || F <= 0 || max_rows_per_expert < 0)
        return fail(MOE_ERR_INVALID_ARG, "moe_grouped_ffn_wq: R >= 0, max_rows_per_expert >= 0 and E, d, F > 0 required");
    if (d % 64 || F % 64) return fail(MOE_ERR_INVALID_ARG, "moe_grouped_ffn_wq: d and F must be multiples of 64 (d=%d F=%d)", d, F);
    if (bits != 4 && bits != 8) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq: bits must be 4 or 8 (got %d)", bits);
    if (activation != MOE_ACT_RELU && activation != MOE_ACT_GELU) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq: unknown activation %d", activation);
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
    reset_kernel_notes();
    if (R == 0) return MOE_OK;

    hipStream_t s = as_stream(stream);
    const bool bf = act_dtype == MOE_BF16;
    const int max_rows = max_rows_per_expert > 0 && max_rows_per_expert < R ? max_rows_per_expert : R;
    unsigned char *wsb = (unsigned char *)workspace;
    void *h = wsb + ws.h_off;
    // decode-sized batch with everything fused: one streaming launch for the sort and both GEMMs, then the slice reduction
    if (gate_idx && expert_scale && !bf && group_size == 0 && decode_ffn_supports(R, E, d, F, bits)) {
        DecodeArgs q{};
        q.x = (const uint16_t *)x_perm; q.gate_idx = gate_idx; q.gate_scale = expert_scale; q.n_assign = R; q.gate_k = k;
        q.E = E; q.d = d; q.F = F; q.act = activation;
        q.w1 = (const uint8_t *)w1_packed; q.w2 = (const uint8_t *)w2_packed;
        q.s1 = (const __half *)s1; q.s2 = (const __half *)s2; q.b1 = (const __half *)b1; q.b2 = (const __half *)b2;
        q.partial = (float *)(wsb + ws.partial_off); q.out = (float *)y_perm;
        q.perm_src_out = perm_src_out; q.inv_perm_out = inv_perm_out; q.offsets_out = offsets_out;
        note_kernel("decode_ffn_kernel");
        return launch_decode_ffn(q, bits, as_stream(stream));
    }
    float2 *pow_x = (float2 *)(wsb + ws.pow_x_off), *pow_h = (float2 *)(wsb + ws.pow_h_off);
    const bool grouped = group_size != 0 && !(group_size == d && group_size == F);

    // fc1: h = relu(x_perm @ deq(W1) + b1), stored in the activation dtype.  With bf16
    // activations and group scales the weights go in as an exact two-term FP16 sum, because h
    // is rounded to 8 bits afterwards and a 2^-11 weight rounding would show through.
    GemmArgs g1{};
    g1.a = (const uint16_t *)x_perm; g1.row_pow = bf ? pow_x : nullptr; g1.offsets = expert_offsets;
    g1.wq = (const uint8_t *)w1_packed; g1.scales = (const __half *)s1; g1.bias = (const __half *)b1;
    g1.out = h; g1.E = E; g1.R = R; g1.K = d; g1.N = F; g1.g = grouped ? group_size : d;
    g1.out_dtype = act_dtype; g1.act = activation;
    g1.a_src = perm_src; g1.a_div = k;
    if (gate_idx) {     // decode-sized: fc1 rebuilds the permutation from the gate's output and writes the index arrays
        g1.gate_idx = gate_idx; g1.n_assign = R; g1.gate_k = k;
        g1.perm_src_out = perm_src_out; g1.inv_perm_out = inv_perm_out; g1.offsets_out = offsets_out;
        if (expert_scale) { g1.zero_out = (float *)y_perm; g1.zero_count = (long)(R / k) * d; }   // fc2 adds into it
    }
    if (bf) {           // bf16 rows: converted to power-of-two scaled FP16 rows first, then the GEMM of FP16 rows
        uint16_t *x16 = (uint16_t *)(wsb + ws.x16_off);
        hipLaunchKernelGGL(rows_to_f16_kernel, dim3((R + 3) / 4), dim3(256), 0, s, (const uint16_t *)x_perm, x16, R, d, pow_x);
        int rc = check_launch("moe_grouped_ffn_wq (x to scaled FP16)");
        if (rc) return rc;
        g1.a = x16;
    }
    // (groups of 128: exact codes, group sums folded in fp32; other group sizes: the two-term form)
    const int smode1 = !grouped ? SCALE_CHANNEL : !bf ? SCALE_GROUP : group_size == 128 ? SCALE_GROUP_ACC : SCALE_GROUP_SPLIT;
    int rc = run_gemm(g1, bits, smode1, bf, max_rows, s);
    if (rc) return rc;

    // fc2: y = h @ deq(W2) + b2
    GemmArgs g2 = g1;
    g2.a = (const uint16_t *)h; g2.row_pow = bf ? pow_h : nullptr;
    g2.wq = (const uint8_t *)w2_packed; g2.scales = (const __half *)s2; g2.bias = (const __half *)b2;
    g2.out = y_perm; g2.K = F; g2.N = d; g2.g = grouped ? group_size : F;
    g2.out_dtype = y_dtype; g2.act = MOE_ACT_NONE;
    g2.a_src = nullptr;
    g2.gate_idx = nullptr; g2.zero_out = nullptr;
    if (gate_idx && expert_scale) {     // un-permute fused into fc2: fc1 clears out, fc2 adds scale * y into the tokens' rows
        g2.out_dst = perm_src_out; g2.out_scale = expert_scale; g2.out_add = 1; g2.out_div = k;
    } else if (expert_scale) {
        g2.out_dst = perm_src; g2.out_scale = expert_scale;
    }
    if (bf) {           // h, which fc1 rounded to bf16 (A13), in place
        hipLaunchKernelGGL(rows_to_f16_kernel, dim3((R + 3) / 4), dim3(256), 0, s, (const uint16_t *)h, (uint16_t *)h, R, F, pow_h);
        rc = check_launch("moe_grouped_ffn_wq (h to scaled FP16)");
        if (rc) return rc;
    }
    return run_gemm(g2, bits, grouped ? SCALE_GROUP : SCALE_CHANNEL, bf, max_rows, s);
}

extern "C" int moe_grouped_ffn_wq(const void *x_perm, int act_dtype, const int32_t *expert_offsets, int R,
                                  int E, int max_rows_per_expert, int d, int F, int bits, int group_size,
                                  int activation, const void *w1_packed,
                                  const void *s1, const void *b1, const void *w2_packed, const void *s2,
                                  const void *b2, void *y_perm, int y_dtype, void *workspace,
                                  size_t workspace_bytes, void *stream)
{
    return ffn_impl(x_perm, act_dtype, expert_offsets, R, E, max_rows_per_expert, d, F, bits, group_size, activation, w1_packed,
                    s1, b1, w2_packed, s2, b2, y_perm, y_dtype, workspace, workspace_bytes, stream, nullptr, 1, nullptr);
}

// ---- the entry point for callers that cannot allocate ------------------------------------------
// moe_grouped_ffn_wq with its workspace (h, and for bf16 rows the per-row factors) in a fixed array in
// the library's own device memory.  Every GPU the library runs on holds its own copy of the array
// until the process ends.
constexpr size_t kScratchBytes = (size_t)8 << 20;
constexpr int kScratchMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Device address of `scratch` on the current device, looked up once per device (0 on failure, with
// the error message set).  In host code the array's name is only a handle for this lookup.
static void *scratch_address()
{
    using namespace moe;
    static std::mutex lock;
    static void *address[kScratchMaxDevices];           // zero-initialised: not looked up yet
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess || dev < 0 || dev >= kScratchMaxDevices) {
        fail(MOE_ERR_HIP, "moe_grouped_ffn_wq_noalloc: no current device (%s)", hipGetErrorString(err));
        return nullptr;
    }
    std::lock_guard<std::mutex> guard(lock);
    if (!address[dev]) {
        void *ptr = nullptr;
        err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (err != hipSuccess || !ptr) {
            fail(MOE_ERR_HIP, "moe_grouped_ffn_wq_noalloc: hipGetSymbolAddress failed on device %d (%s)", dev, hipGetErrorString(err));
            return nullptr;
        }
        address[dev] = ptr;
    }
    return address[dev];
}

extern "C" size_t moe_grouped_ffn_wq_noalloc_max_bytes(void) { return kScratchBytes; }

extern "C" int moe_grouped_ffn_wq_noalloc(const void *x_perm, int act_dtype, const int32_t *expert_offsets, int R,
                                          int E, int max_rows_per_expert, int d, int F, int bits, int group_size,
                                          int activation, const void *w1_packed,
                                          const void *s1, const void *b1, const void *w2_packed, const void *s2,
                                          const void *b2, void *y_perm, int y_dtype, void *stream)
{
    using namespace moe;
    if (R > 0 && d > 0 && F > 0) {
        const size_t need = moe_grouped_ffn_wq_workspace_bytes(R, d, F, E, act_dtype);
        if (need > kScratchBytes)
            return fail(MOE_ERR_WORKSPACE, "moe_grouped_ffn_wq_noalloc: R=%d rows of F=%d need %zu bytes of scratch, the built-in "
                                           "array holds %zu: use moe_grouped_ffn_wq with a workspace", R, F, need, kScratchBytes);
    }
    void *ws = scratch_address();
    if (!ws) return MOE_ERR_HIP;
    return ffn_impl(x_perm, act_dtype, expert_offsets, R, E, max_rows_per_expert, d, F, bits, group_size, activation, w1_packed,
                    s1, b1, w2_packed, s2, b2, y_perm, y_dtype, ws, kScratchBytes, stream, nullptr, 1, nullptr);
}

// The same pair of GEMMs with the row gather (and, for k = 1, the un-permute and gate scale) fused
// into them; built on the tiled kernel only.
extern "C" int moe_grouped_ffn_wq_routed_supported(int R, int E, int max_rows_per_expert, int d, int F,
                                                   int bits, int group_size, int act_dtype)
{
    using namespace moe;
    if (R <= 0 || E <= 0 || d <= 0 || F <= 0 || act_dtype != MOE_F16) return 0;
    const int max_rows = max_rows_per_expert > 0 && max_rows_per_expert < R ? max_rows_per_expert : R;
    const bool grouped = group_size != 0 && !(group_size == d && group_size == F);
    return tiled_only(R, E, max_rows, d, F, bits, grouped, false) ? 1 : 0;
}

extern "C" int moe_grouped_ffn_wq_routed(const void *x, int act_dtype, const int32_t *perm_src, int k,
                                         const float *expert_scale, const int32_t *expert_offsets, int R,
                                         int E, int max_rows_per_expert, int d, int F, int bits,
                                         int group_size, int activation, const void *w1_packed, const void *s1,
                                         const void *b1, const void *w2_packed, const void *s2,
                                         const void *b2, void *out, int out_dtype, void *workspace,
                                         size_t workspace_bytes, void *stream)
{
    using namespace moe;
    if (!perm_src) return fail(MOE_ERR_INVALID_ARG, "moe_grouped_ffn_wq_routed: perm_src must not be NULL");
    if (k < 1 || k > 2) return fail(MOE_ERR_INVALID_ARG, "moe_grouped_ffn_wq_routed: k must be 1 or 2 (k=%d)", k);
    if (expert_scale && k != 1)
        return fail(MOE_ERR_INVALID_ARG, "moe_grouped_ffn_wq_routed: the fused un-permute needs k = 1 (one expert per token)");
    if (!moe_grouped_ffn_wq_routed_supported(R, E, max_rows_per_expert, d, F, bits, group_size, act_dtype))
        return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq_routed: these sizes run (partly) in the streaming kernels or in bf16, "
                                         "which take permuted rows only: use moe_permute + moe_grouped_ffn_wq + moe_combine");
    return ffn_impl(x, act_dtype, expert_offsets, R, E, max_rows_per_expert, d, F, bits, group_size, activation, w1_packed, s1, b1,
                    w2_packed, s2, b2, out, out_dtype, workspace, workspace_bytes, stream, perm_src, k, expert_scale);
}

// Decode-sized batches: moe_permute and moe_grouped_ffn_wq in one call.  fc1 runs in the straight-line
// streaming kernel, whose blocks rebuild the permutation from the gate's expert indices, fetch their
// rows from the tokens and write perm_src / inv_perm / expert_offsets on the way; fc2 and moe_combine
// then read those arrays as after moe_permute.
static int gated_shapes(int T, int k, int E, int d, int F, int bits, int group_size, int act_dtype)
{
    using namespace moe;
    if (T <= 0 || k < 1 || k > 2 || E <= 0 || d <= 0 || F <= 0 || act_dtype != MOE_F16) return 0;
    if ((long)T * k > kGatedMaxAssign || (bits != 4 && bits != 8) || d % 64 || F % 64) return 0;
    if (group_size != 0 && !(group_size == d && group_size == F)) return 0;
    if (!stream_unrolled_takes_gate(d, bits)) return 0;
    // fc1 must run in the straight-line streaming kernel (row bound T) ...
    const int R = T * k;
    if (choose_kernel(R, E, T, d, F, bits, SCALE_CHANNEL, false) != GEMM_STREAM_UNROLLED) return 0;
    // ... and fc2 as well, if it is to add its rows straight into the layer output
    const bool fc2 = choose_kernel(R, E, T, F, d, bits, SCALE_CHANNEL, false) == GEMM_STREAM_UNROLLED;
    return fc2 ? 2 : 1;
}

extern "C" int moe_grouped_ffn_wq_gated_supported(int T, int k, int E, int d, int F, int bits, int group_size,
                                                  int act_dtype)
{
    return gated_shapes(T, k, E, d, F, bits, group_size, act_dtype);
}

extern "C" int moe_grouped_ffn_wq_gated(const void *x, int act_dtype, const int32_t *expert_idx,
                                        const float *expert_scale, int T, int k,
                                        int E, int d, int F, int bits, int group_size, int activation,
                                        const void *w1_packed, const void *s1, const void *b1,
                                        const void *w2_packed, const void *s2, const void *b2, void *y_perm,
                                        int y_dtype, int32_t *perm_src, int32_t *inv_perm,
                                        int32_t *expert_offsets, void *workspace, size_t workspace_bytes,
                                        void *stream)
{
    using namespace moe;
    if (!expert_idx || !perm_src || !inv_perm || !expert_offsets)
        return fail(MOE_ERR_INVALID_ARG, "moe_grouped_ffn_wq_gated: NULL pointer");
    const int level = gated_shapes(T, k, E, d, F, bits, group_size, act_dtype);
    if (!level)
        return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq_gated: only decode-sized fp16 batches with per-channel scales "
                                         "(T*k <= %d) are taken: use moe_permute + moe_grouped_ffn_wq", kGatedMaxAssign);
    if (expert_scale && (level < 2 || y_dtype != MOE_F32))
        return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq_gated: the fused un-permute needs an fp32 output and an fc2 that runs "
                                         "in the straight-line streaming kernel: pass expert_scale = NULL and use moe_combine");
    return ffn_impl(x, act_dtype, expert_offsets, T * k, E, T, d, F, bits, group_size, activation, w1_packed, s1, b1,
                    w2_packed, s2, b2, y_perm, y_dtype, workspace, workspace_bytes, stream, nullptr, k, expert_scale,
                    expert_idx, perm_src, inv_perm, expert_offsets);
}

// One grouped GEMM of the decode-sized case, for the comparison of Table 1 (fp16 / int8 / int4
// weights, magic-number or native conversion).
extern "C" int moe_grouped_gemm_wq(const void *x_perm, const int32_t *expert_offsets, int R, int E,
                                   int max_rows_per_expert, int K, int N, int bits, int native_convert,
                                   const void *w_packed, const void *scales, void *y, int y_dtype,
                                   void *stream)
{
    using namespace moe;
    if (!expert_offsets || !w_packed || (bits != 16 && !scales) || (R != 0 && (!x_perm || !y)))
        return fail(MOE_ERR_INVALID_ARG, "moe_grouped_gemm_wq: NULL pointer");
    if (R < 0 || E <= 0 || K <= 0 || N <= 0 || max_rows_per_expert < 0)
        return fail(MOE_ERR_INVALID_ARG, "moe_grouped_gemm_wq: R >= 0, max_rows_per_expert >= 0 and E, K, N > 0 required");
    if (K % 64 || N % 64) return fail(MOE_ERR_INVALID_ARG, "moe_grouped_gemm_wq: K and N must be multiples of 64 (K=%d N=%d)", K, N);
    if (bits != 4 && bits != 8 && bits != 16) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_wq: bits must be 4, 8 or 16 (got %d)", bits);
    if (y_dtype != MOE_F16 && y_dtype != MOE_BF16 && y_dtype != MOE_F32) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_wq: unknown y_dtype %d", y_dtype);
    if (E > 4096) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_wq: E=%d above 4096", E);
    const void *ptrs[] = {x_perm, w_packed, scales, y};
    for (const void *q : ptrs)
        if (!aligned16(q)) return fail(MOE_ERR_INVALID_ARG, "moe_grouped_gemm_wq: buffers must be 16-byte aligned");
    if (R == 0) return MOE_OK;
    const int max_rows = max_rows_per_expert > 0 && max_rows_per_expert < R ? max_rows_per_expert : R;
    if (max_rows > 64) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_wq: only the decode-sized case (at most 64 rows per expert) is built");
    if (!stream_unrolled_supports(K, bits, SCALE_CHANNEL))
        return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_gemm_wq: K=%d is not taken with bits=%d", K, bits);
    GemmArgs g{};
    g.a = (const uint16_t *)x_perm; g.offsets = expert_offsets; g.wq = (const uint8_t *)w_packed;
    g.scales = (const __half *)scales; g.bias = nullptr; g.out = y; g.E = E; g.R = R; g.K = K; g.N = N; g.g = K;
    g.out_dtype = y_dtype; g.act = MOE_ACT_NONE;
    hipStream_t s = as_stream(stream);
    if (bits == 16 || native_convert) return launch_stream_unrolled_variant(g, bits, native_convert != 0, max_rows, s);
    return launch_stream_unrolled(g, bits, max_rows, s);
}
