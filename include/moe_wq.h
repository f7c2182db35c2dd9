/*
 * moe_wq.h - C ABI of the MI355X (gfx950) sparsely activated expert FFN layer with
 * weight-only int4/int8 quantised experts (arXiv 2211.10017, Sec. 3.3 "Optimized GPU kernel
 * design" and Sec. 3.4 "Expert quantization with 4-bit and 8-bit").
 *
 * The layer is five calls, made in this order on one stream:
 *
 *   moe_quantize_experts   offline, once per weight tensor
 *   moe_gate_topk -> moe_permute -> moe_grouped_ffn_wq -> moe_combine     per layer call
 *
 * Conventions common to every entry point
 *   - Every pointer is a DEVICE pointer unless it says otherwise.  The caller allocates and
 *     owns every buffer; the library never allocates, frees or keeps device memory between
 *     calls.  Scratch comes from a caller-provided workspace sized by the *_workspace_bytes
 *     queries (pure host functions).  Buffers must be 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All work is
 *     enqueued on it; no entry point synchronises with the host or reads device memory from
 *     the host (the per-expert offsets stay on the device).
 *   - Return value: MOE_OK or one of the MOE_ERR_* codes.  Arguments, sizes and the choice of
 *     kernels are checked on the host before anything is launched: with MOE_ERR_INVALID_ARG,
 *     MOE_ERR_UNSUPPORTED or MOE_ERR_WORKSPACE nothing has been enqueued.  MOE_ERR_HIP reports a
 *     launch the runtime refused; launches of the same call made before it stay enqueued.
 *     moe_last_error() returns a thread-local message.  No exceptions, no aborts.
 *   - Identical inputs give bit-identical outputs: the sort is stable and no result depends on
 *     the order in which workgroups run.  (One path adds floating-point numbers into shared
 *     memory locations, moe_grouped_ffn_wq_gated with expert_scale: at most two fp32 terms per
 *     element onto a cleared buffer, and the sum of two terms does not depend on their order.)
 *   - Limits of a whole layer call: 1 <= k <= 2 and k <= E <= 256 (the gate's limits; moe_permute
 *     alone takes E <= 1024 and the FFN entry points E <= 4096), d % 64 == 0, F % 64 == 0.
 *   - Notation: T tokens, d = d_model, F = d_ff, E experts, k experts per token,
 *     R = T*k routed rows, assignment id a = t*k + j.  Expert weights are (E, K, N)
 *     row-major with N contiguous, so that a GEMM is A[m x K] @ B[K x N] (Table 1 caption):
 *     fc1 has K = d, N = F; fc2 has K = F, N = d.
 */
#ifndef MOE_WQ_H
#define MOE_WQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = 1,   /* null pointer, non-positive or misaligned dimension, k > E ... */
    MOE_ERR_UNSUPPORTED = 2,   /* bits not in {4,8}, unknown dtype, E above the supported range */
    MOE_ERR_WORKSPACE = 3,     /* workspace missing or smaller than the query says */
    MOE_ERR_HIP = 4            /* a launch failed (hipGetLastError) */
};

/* element types of activation-like tensors */
enum { MOE_F16 = 0, MOE_BF16 = 1, MOE_F32 = 2 };

/* activation between the two GEMMs of the expert FFN */
enum { MOE_ACT_RELU = 0, MOE_ACT_GELU = 1 };

/* Message for the last error returned on this thread ("" if none). */
const char *moe_last_error(void);

/* Names of the GEMM kernels that the last moe_grouped_ffn_wq* call on this thread launched, fc1
 * first, separated by a blank ("" before the first call); for measurement reports. */
const char *moe_last_ffn_kernels(void);

/* What the current device reports (HOST pointers, any may be NULL): compute units, engine and
 * memory clock in kHz, memory bus width in bits; for reports that re-derive the chip's peaks. */
int moe_device_info(int *compute_units, int *engine_clock_khz, int *memory_clock_khz, int *memory_bus_bits);

/* Library ABI version (bumped when a signature or the packed layout changes). */
int moe_abi_version(void);

/*
 * Sec. 3.4: symmetric, range-based quantisation of expert weights, one fp16 scale per output
 * channel n (the paper's (E,1,N) scales for (E,M,N) weights), or per group of `group_size`
 * rows along K.  qmax = 127 (8 bits) / 7 (4 bits); scale = fp16(absmax / qmax);
 * code = clamp(round_half_even(w / scale), -qmax, qmax); an all-zero channel has scale 0 and
 * codes 0.  Dequantisation (Algorithm 1) is code * scale.
 *
 *   w          [E,K,N] fp32
 *   bits       4 or 8
 *   group_size 0 or K: per channel; otherwise must divide K and be a multiple of 64
 *   q_canon    interchange codes: bits=8: int8 [E,K,N]; bits=4: [E,K,N/2] bytes, two's-complement
 *              nibbles, even n in the low nibble.  May be NULL.
 *   scales     fp16 [E, K/group_size, N]
 *   q_packed   the layout moe_grouped_ffn_wq reads: same byte count as q_canon, codes stored
 *              offset-binary (+128 / +8, Sec. 3.4.1) and pre-shuffled into per-wavefront MFMA
 *              operand order; opaque to the caller.  May be NULL.
 * Requires N % 32 == 0 and K % 64 == 0.  E may be a slice: calling once per expert with E = 1
 * and offset pointers gives the same bytes as one call over all experts.
 */
int moe_quantize_experts(const float *w, int E, int K, int N, int bits, int group_size,
                         void *q_canon, void *scales, void *q_packed, void *stream);

/*
 * Sec. 3.3: the top-k gating function.  logit[t,e] = sum_i x[t,i]*wg[i,e] (+ bias[e]); the k
 * largest logits win (ties: lower expert index; slots in descending logit order);
 * expert_scale is the softmax probability (over all E logits, fp32) of each chosen expert,
 * divided by the sum of the k chosen probabilities when renormalize != 0 and k > 1.
 * The logit is accumulated in fp32 as four partial sums (128-element blocks of i dealt
 * round-robin to the four sums, each in increasing i), combined as ((p0+p1)+p2)+p3, then
 * the bias is added: this order is part of the contract, so routing is reproducible.
 *
 * Sec. 3.5 (batch pruning): a row with finished[t] != 0 (a sentence that has ended) gets the
 * expert index E, one past the real experts, and scale 0 in all its k slots; moe_permute sorts
 * such rows behind every active row and nothing downstream touches them.
 *
 *   x [T,d] act_dtype (MOE_F16 | MOE_BF16), wg [d,E] same dtype, bias [E] fp32 or NULL
 *   finished [T] bytes (device) or NULL (no row is pruned)
 *   expert_idx [T,k] int32, expert_scale [T,k] fp32
 * Requires 1 <= k <= 2, k <= E <= 256, d >= 8 and d % 8 == 0.
 */
int moe_gate_topk(const void *x, int act_dtype, const void *wg, const float *bias,
                  const uint8_t *finished, int T, int d, int E, int k, int renormalize,
                  int32_t *expert_idx, float *expert_scale, void *stream);

/*
 * Sec. 3.3: routing.  The (expert, row) tuples are sorted by expert with a stable counting
 * sort and the activation rows are gathered into expert-contiguous order.
 *
 *   expert_idx [T,k]; x [T,d] act_dtype
 *   x_perm [R,d]          x_perm[r] = x[perm_src[r] / k]
 *   perm_src [R]          assignment id held by sorted position r
 *   inv_perm [R]          sorted position of assignment a
 *   expert_offsets [E+1]  rows of expert e are offsets[e] .. offsets[e+1]-1  (start of each
 *                         expert's sub-matrix); stays on the device
 * An entry of expert_idx equal to E marks a pruned row (Sec. 3.5): it is the last key of the
 * sort, so these rows follow all others in perm_src / inv_perm, expert_offsets[E] is the number
 * of active rows (R when nothing is pruned) and their x_perm rows are not written.  Other
 * entries outside [0,E] are a caller error (not checked; they are treated as 0 or E).  d % 8 == 0.
 */
size_t moe_permute_workspace_bytes(int T, int k, int E);
int moe_permute(const int32_t *expert_idx, const void *x, int act_dtype, int T, int k, int E,
                int d, void *x_perm, int32_t *perm_src, int32_t *inv_perm,
                int32_t *expert_offsets, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Sec. 3.3 (grouped GEMM, Fig. 1) + Sec. 3.4 (dequantisation fused into the GEMM): for every
 * expert e and each of its rows r,
 *     h[r] = act(x_perm[r] @ deq(W1[e]) + b1[e])    stored in act_dtype
 *     y[r] = h[r] @ deq(W2[e]) + b2[e]              stored in y_dtype
 * with fp16 MFMA and fp32 accumulation; the packed codes are unpacked and dequantised in
 * registers (never written back to memory).  Experts without rows cost no weight traffic.
 *
 *   activation: MOE_ACT_RELU (the paper does not name the activation; ReLU is the reading
 *       taken) or MOE_ACT_GELU (exact form x * Phi(x), a second choice)
 *   x_perm [R,d] act_dtype
 *   expert_offsets [E+1] (device): a monotone partition of the R rows, offsets[0] = 0 and
 *       offsets[E] = R, as moe_permute writes it.  The host cannot check it; the kernels force
 *       every range into [0, R], so other contents give wrong results but no stray access.
 *   max_rows_per_expert: an upper bound on the rows any one expert receives, if the caller
 *       knows one (T is one: a token visits an expert at most once); 0 = unknown (R is used).
 *       It takes part in the choice between the weight-streaming kernels (which need a bound
 *       <= 64, or a mean of at most 32 rows per expert with a bound of at most sixteen row
 *       groups, and are used while R / E says that the typical expert fits one row group, R <= 256,
 *       or there are too few experts to fill the chip with row tiles) and the tiled kernel, and
 *       it sizes the streaming launch, so it must be a true bound: rows of an expert beyond it
 *       are not computed.
 *   w1_packed / w2_packed: q_packed from moe_quantize_experts for (E,d,F) / (E,F,d)
 *   s1 fp16 [E, d/g, F]; s2 fp16 [E, F/g, d]  (g = group_size, or K when group_size is 0)
 *   b1 [E,F] / b2 [E,d] fp16 or NULL
 *   y_perm [R,d] in y_dtype (MOE_F16 | MOE_BF16 | MOE_F32)
 * Requires d % 64 == 0, F % 64 == 0, bits in {4,8}, group_size 0 or a multiple of 64 dividing
 * both d and F.
 * Workspace: h (R * F elements of act_dtype), for bf16 rows their per-row factors and x_perm converted to
 * scaled FP16 (R * d elements), and for decode-sized batches (R <= 256) the partial sums
 * moe_grouped_ffn_wq_gated keeps (F / 512 x R x d fp32).
 */
size_t moe_grouped_ffn_wq_workspace_bytes(int R, int d, int F, int E, int act_dtype);
int moe_grouped_ffn_wq(const void *x_perm, int act_dtype, const int32_t *expert_offsets, int R,
                       int E, int max_rows_per_expert, int d, int F, int bits, int group_size,
                       int activation, const void *w1_packed,
                       const void *s1, const void *b1, const void *w2_packed, const void *s2,
                       const void *b2, void *y_perm, int y_dtype, void *workspace,
                       size_t workspace_bytes, void *stream);

/*
 * moe_grouped_ffn_wq for callers that cannot allocate device memory or carry a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * and same results (bit for bit: the same kernels run) as moe_grouped_ffn_wq without the
 * workspace pair; h (and what bf16 rows need: their factors and the converted x_perm) live in a fixed array of
 * moe_grouped_ffn_wq_noalloc_max_bytes() = 8 MiB inside the library's own device memory, which
 * every GPU the library is used on holds until the process ends.  The call allocates and frees
 * nothing (its first call on a device looks up the array's address, nothing more).
 *   Sizes whose moe_grouped_ffn_wq_workspace_bytes(R, d, F, E, act_dtype) exceeds the array are
 *   refused with MOE_ERR_WORKSPACE before anything is launched (decode-sized batches fit: 128 rows
 *   of F = 4096 take 1 MiB; R * F <= 4 Mi elements of fp16 in general).
 *   All calls on one GPU share that GPU's array, which keeps the last call's h: nothing in it has
 *   to start from zero (fc1 writes every row fc2 reads), but two calls that overlap in time on one
 *   GPU (different streams or host threads) race on it.  Calls on one stream are safe.
 */
size_t moe_grouped_ffn_wq_noalloc_max_bytes(void);
int moe_grouped_ffn_wq_noalloc(const void *x_perm, int act_dtype, const int32_t *expert_offsets, int R,
                               int E, int max_rows_per_expert, int d, int F, int bits, int group_size,
                               int activation, const void *w1_packed,
                               const void *s1, const void *b1, const void *w2_packed, const void *s2,
                               const void *b2, void *y_perm, int y_dtype, void *stream);

/*
 * moe_grouped_ffn_wq with the routing fused into the GEMMs, for batches large enough to run in
 * the tiled kernel: fc1 fetches row r from x[perm_src[r] / k] (no x_perm copy is needed:
 * moe_permute may be called with x = x_perm = NULL), and, when expert_scale is given (k = 1
 * only, one expert per token), fc2 stores expert_scale[t] * y[r] straight into out[t],
 * t = perm_src[r], which replaces moe_combine.
 *   x [T,d] fp16 (un-permuted); perm_src [R], expert_offsets [E+1] from moe_permute;
 *   expert_scale [T] fp32 or NULL; out: [T,d] when expert_scale is given, else y_perm [R,d].
 *   With pruned rows (Sec. 3.5) and expert_scale given, the rows of pruned tokens in out are
 *   not written: clear out first, or use moe_combine.
 * moe_grouped_ffn_wq_routed_supported returns 1 when a call with these sizes is taken (fp16
 * activations and row counts that run entirely in the tiled kernel); otherwise the call
 * returns MOE_ERR_UNSUPPORTED and the un-fused sequence has to be used.  Workspace as for
 * moe_grouped_ffn_wq.
 */
int moe_grouped_ffn_wq_routed_supported(int R, int E, int max_rows_per_expert, int d, int F, int bits,
                                        int group_size, int act_dtype);
int moe_grouped_ffn_wq_routed(const void *x, int act_dtype, const int32_t *perm_src, int k,
                              const float *expert_scale, const int32_t *expert_offsets, int R, int E,
                              int max_rows_per_expert, int d, int F, int bits, int group_size,
                              int activation, const void *w1_packed, const void *s1, const void *b1,
                              const void *w2_packed, const void *s2, const void *b2, void *out,
                              int out_dtype, void *workspace, size_t workspace_bytes, void *stream);

/*
 * moe_permute and moe_grouped_ffn_wq in one call, for decode-sized batches (Sec. 3.3 steps 2 and
 * 3; the stable sort by expert is rebuilt inside the first GEMM).  fc1's blocks count the
 * assignments of their expert and of the experts before it from expert_idx, fetch their rows
 * straight from x and write the index arrays; fc2 (and moe_combine afterwards) read them as
 * after moe_permute.  No x_perm copy and no permute launch.
 *   x [T,d] fp16 (un-permuted, device); expert_idx [T*k] from moe_gate_topk (E = pruned row);
 *   outputs: y_perm [R,d] in y_dtype, perm_src [R], inv_perm [R], expert_offsets [E+1]
 *   (identical to what moe_permute writes, pruned rows behind the active ones,
 *   expert_offsets[E] = active rows); workspace as for moe_grouped_ffn_wq with R = T*k.
 *   expert_scale [T*k] fp32 or NULL.  When given, moe_combine is fused in as well: y_perm is
 *   then the layer output out [T,d], fp32 (y_dtype must be MOE_F32): fc1 clears it and fc2 adds
 *   expert_scale[a] * y[row of a] into row a / k with hardware fp32 adds.  A token gets at
 *   most two terms and fp32 addition of two terms onto zero is commutative, so the result
 *   does not depend on the order of arrival; rows of pruned tokens stay zero.
 *   With expert_scale given and sizes the decode kernel is built for (4-bit: d = 1024; 8-bit:
 *   d = 512; F a multiple of 512 up to 4096; at most 8 assignments per expert on average and at
 *   least 64 slices of 512 d_ff channels in all), the call is two launches: a persistent grid of one
 *   workgroup per compute unit streams every active expert's W1 and W2 once (fc1, activation and
 *   fc2 per 512-channel slice of d_ff, h staying on chip) and leaves fp32 partial sums of y in the
 *   workspace; a small second launch adds the slices in a fixed order, applies the channel scale,
 *   bias and gate scale and writes out.  No atomics on this path.  (For timing studies y_perm may
 *   be NULL on this path: the second launch is then left out and the partial sums stay in the
 *   workspace.)
 * moe_grouped_ffn_wq_gated_supported returns 0 when a call with these sizes is not taken
 * (it then returns MOE_ERR_UNSUPPORTED and launches nothing), 1 when it is taken with
 * expert_scale = NULL, 2 when expert_scale may be given too.  Taken: fp16 activations,
 * per-channel scales, T*k <= 256, and d such that fc1 runs in the straight-line streaming
 * kernel (d = 1024 or 2048 with 4-bit, 512 or 1024 with 8-bit weights) under the row bound T;
 * for 2, F at most 4096 (4-bit) or 2048 (8-bit) and a multiple of 1024 / 512 as well.
 */
int moe_grouped_ffn_wq_gated_supported(int T, int k, int E, int d, int F, int bits, int group_size,
                                       int act_dtype);
int moe_grouped_ffn_wq_gated(const void *x, int act_dtype, const int32_t *expert_idx,
                             const float *expert_scale, int T, int k,
                             int E, int d, int F, int bits, int group_size, int activation,
                             const void *w1_packed, const void *s1, const void *b1,
                             const void *w2_packed, const void *s2, const void *b2, void *y_perm,
                             int y_dtype, int32_t *perm_src, int32_t *inv_perm,
                             int32_t *expert_offsets, void *workspace, size_t workspace_bytes,
                             void *stream);

/*
 * Table 1 (Sec. 4.1): throughput of one grouped GEMM  y[r] = x_perm[r] @ deq(W[e])  on about 40
 * tokens spread over 1..32 active experts, with fp16, int8 and int4 weights.  This entry runs
 * that single GEMM with the decode-sized streaming kernels of moe_grouped_ffn_wq:
 *   bits 4 | 8: w_packed / scales from moe_quantize_experts (per-channel scales, group_size 0);
 *   bits 16:    w_packed from moe_pack_fp16_experts (unquantised fp16 weights, scales ignored,
 *               may be NULL) - the comparison's denominator;
 *   native_convert != 0: the codes are converted with the chip's integer-to-float instructions
 *               instead of the magic-number trick of Sec. 3.4.1 (same values; the route the
 *               paper found slow), built for the table's shape only (K = 1024).
 *   x_perm [R,K] fp16; expert_offsets [E+1] as for moe_grouped_ffn_wq; y [R,N] y_dtype.
 * Requires at most 64 rows per expert (max_rows_per_expert, 0 = R), K % 64 == 0, N % 64 == 0 and
 * a K the streaming kernel takes (a multiple of 16 fragment blocks, at most 64 of them: K = 1024
 * .. 4096 for int4, 512 .. 2048 for int8, 256 .. 1024 for fp16); otherwise MOE_ERR_UNSUPPORTED.
 *
 * moe_pack_fp16_experts: w fp32 [E,K,N] (device) rounded to fp16 and stored in the fragment
 * layout of the packed weights (E*K*N*2 bytes).  N % 32 == 0, K % 16 == 0.
 */
int moe_pack_fp16_experts(const float *w, int E, int K, int N, void *w_packed, void *stream);
int moe_grouped_gemm_wq(const void *x_perm, const int32_t *expert_offsets, int R, int E,
                        int max_rows_per_expert, int K, int N, int bits, int native_convert,
                        const void *w_packed, const void *scales, void *y, int y_dtype, void *stream);

/*
 * Sec. 3.3, last step: rows return to their original order and are multiplied by
 * expert_scale:  out[t] = sum_j expert_scale[t,j] * y_perm[inv_perm[t*k+j]]  (fp32, j ascending).
 *   y_perm [R,d] y_dtype; out [T,d] out_dtype (each MOE_F16 | MOE_BF16 | MOE_F32); d % 8 == 0.
 *   active_rows: device pointer to the number of active rows (expert_offsets + E) or NULL.
 *       Terms whose row is at or past it belong to pruned tokens (Sec. 3.5): y_perm holds
 *       nothing for them and they are left out, so a fully pruned token gets a zero row.
 */
int moe_combine(const void *y_perm, int y_dtype, const int32_t *inv_perm,
                const float *expert_scale, const int32_t *active_rows, int T, int k, int d,
                void *out, int out_dtype, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_WQ_H */
