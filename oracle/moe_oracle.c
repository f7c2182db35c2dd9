/*
 * CPU oracle for the sparsely activated expert FFN layer (arXiv 2211.10017, Sec. 3.3-3.4).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition of what the layer computes,
 * written as loops so it can be checked against the paper by eye.  It shares no code, table
 * or constant with the HIP library, and nothing in the product path may call it.
 *
 * Conventions
 *   - every real tensor is held in float; values that the method stores in fp16 or bf16
 *     (activations, scales, the hidden activation h) are floats that are exactly
 *     representable in that format, produced by the two rounding routines below;
 *   - sums are carried in double unless the sum decides an integer (the gate logits, see
 *     orc_gate), where the order and precision are part of the definition;
 *   - weights are (E, K, N) row-major with N contiguous: the GEMM is A[m x K] @ B[K x N]
 *     (Table 1 caption), and the scale tensor is (E, K/g, N); g == K is the paper's
 *     per-channel (E, 1, N) case (Sec. 3.4).
 *
 * Pins (tests that do not come from this file): see tests/test_oracle_*.py.
 * Functions whose speed/accuracy figures in the paper cannot be reproduced here
 * (Tables 1-4) are not implemented: parity unpinned, context only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- number formats */

static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* float -> IEEE binary16 bit pattern, round to nearest even, with subnormals, inf, nan. */
uint16_t orc_f32_to_f16_bits(float f)
{
    uint32_t u = f32_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t mag = u & 0x7fffffffu;
    if (mag >= 0x7f800000u)                      /* inf or nan */
        return (uint16_t)(sign | 0x7c00u | (mag > 0x7f800000u ? 0x0200u : 0u));
    double a = fabs((double)f);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                          /* a = m * 2^e, m in [0.5, 1) */
    int exp2 = e - 1;                            /* a in [2^exp2, 2^(exp2+1)) */
    if (exp2 < -14) exp2 = -14;                  /* subnormal range shares the 2^-24 grid */
    double ulp = ldexp(1.0, exp2 - 10);
    double q = nearbyint(a / ulp);               /* default mode: ties to even */
    double r = q * ulp;
    if (r >= 65520.0) return (uint16_t)(sign | 0x7c00u);     /* rounds past max finite */
    if (r < ldexp(1.0, -14))                     /* subnormal or zero: q is the mantissa */
        return (uint16_t)(sign | (uint16_t)q);
    (void)frexp(r, &e);                          /* rounding may have carried to 2^(exp2+1) */
    exp2 = e - 1;
    uint32_t mant = (uint32_t)(r / ldexp(1.0, exp2 - 10)) - 1024u;
    return (uint16_t)(sign | (uint32_t)((exp2 + 15) << 10) | mant);
}

float orc_f16_bits_to_f32(uint16_t h)
{
    int sign = (h >> 15) & 1, e = (h >> 10) & 0x1f, m = h & 0x3ff;
    double v;
    if (e == 0) v = ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexp((double)(1024 + m), e - 25);
    return (float)(sign ? -v : v);
}

float orc_round_f16(float f) { return orc_f16_bits_to_f32(orc_f32_to_f16_bits(f)); }

/* float -> bfloat16 (upper 16 bits of binary32), round to nearest even. */
uint16_t orc_f32_to_bf16_bits(float f)
{
    uint32_t u = f32_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);  /* nan */
    uint32_t lower = u & 0xffffu, upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) upper += 1;
    return (uint16_t)upper;
}

float orc_bf16_bits_to_f32(uint16_t b) { return bits_f32((uint32_t)b << 16); }
float orc_round_bf16(float f) { return orc_bf16_bits_to_f32(orc_f32_to_bf16_bits(f)); }

/* dtype codes shared with the callers: 0 = fp16, 1 = bf16, 2 = fp32 (no rounding) */
static float round_to(float f, int dtype)
{
    if (dtype == 0) return orc_round_f16(f);
    if (dtype == 1) return orc_round_bf16(f);
    return f;
}

void orc_round_array(const float *in, size_t n, int dtype, float *out)
{
    for (size_t i = 0; i < n; ++i) out[i] = round_to(in[i], dtype);
}

/* ---------------------------------------------------------------- quantisation (Sec. 3.4)
 * Symmetric, range-based, per output channel n (and per group of g rows along K when
 * g < K).  The paper fixes: symmetric, range based, scales of shape (E,1,N) in FP16, the
 * same recipe for 4 and 8 bits.  Readings taken where it is silent: qmax = 2^(bits-1)-1,
 * the scale is rounded to fp16 first and the code is the nearest integer (ties to even)
 * to w divided by the scale actually stored; an all-zero column has scale 0 and codes 0.
 */
void orc_quantize(const float *w, int E, int K, int N, int bits, int g,
                  int8_t *q /* [E,K,N], one code per byte */,
                  uint16_t *s_bits /* [E,K/g,N] fp16 bit patterns */)
{
    const int qmax = (1 << (bits - 1)) - 1;
    if (g <= 0 || g > K) g = K;
    const int G = K / g;
#pragma omp parallel for collapse(2) schedule(static)
    for (int e = 0; e < E; ++e)
        for (int gi = 0; gi < G; ++gi) {
            const float *we = w + (size_t)e * K * N;
            int8_t *qe = q + (size_t)e * K * N;
            uint16_t *se = s_bits + ((size_t)e * G + gi) * N;
            float *amax = (float *)calloc((size_t)N, sizeof(float));
            for (int m = gi * g; m < (gi + 1) * g; ++m)          /* range of each channel */
                for (int n = 0; n < N; ++n) {
                    float a = fabsf(we[(size_t)m * N + n]);
                    if (a > amax[n]) amax[n] = a;
                }
            for (int n = 0; n < N; ++n) {
                se[n] = orc_f32_to_f16_bits(amax[n] / (float)qmax);
                amax[n] = orc_f16_bits_to_f32(se[n]);            /* now the stored scale */
            }
            for (int m = gi * g; m < (gi + 1) * g; ++m)
                for (int n = 0; n < N; ++n) {
                    float s = amax[n];
                    float c = 0.0f;
                    if (s != 0.0f) {
                        c = nearbyintf(we[(size_t)m * N + n] / s);
                        if (c > (float)qmax) c = (float)qmax;
                        if (c < (float)-qmax) c = (float)-qmax;
                    }
                    qe[(size_t)m * N + n] = (int8_t)c;
                }
            free(amax);
        }
}

/* Interchange format for 4-bit codes: two's-complement nibbles, even n in the low nibble. */
void orc_pack_int4(const int8_t *q, size_t n_elems, uint8_t *out)
{
    for (size_t i = 0; i < n_elems / 2; ++i)
        out[i] = (uint8_t)((q[2 * i] & 0xf) | ((q[2 * i + 1] & 0xf) << 4));
}

void orc_unpack_int4(const uint8_t *in, size_t n_elems, int8_t *q)
{
    for (size_t i = 0; i < n_elems / 2; ++i) {
        int lo = in[i] & 0xf, hi = in[i] >> 4;
        q[2 * i] = (int8_t)(lo >= 8 ? lo - 16 : lo);
        q[2 * i + 1] = (int8_t)(hi >= 8 ? hi - 16 : hi);
    }
}

/* Algorithm 1: Wdq[e,m,n] = IntToFloat(W[e,m,n]) * S[e,n]  (S indexed by group when g < K).
 * The product of an 8-bit integer and an 11-bit significand is exact in float. */
void orc_dequantize(const int8_t *q, const uint16_t *s_bits, int E, int K, int N, int g,
                    float *wdq)
{
    if (g <= 0 || g > K) g = K;
    const int G = K / g;
#pragma omp parallel for collapse(2) schedule(static)
    for (int e = 0; e < E; ++e)
        for (int gi = 0; gi < G; ++gi) {
            float *sf = (float *)malloc(sizeof(float) * (size_t)N);
            for (int n = 0; n < N; ++n) sf[n] = orc_f16_bits_to_f32(s_bits[((size_t)e * G + gi) * N + n]);
            for (int m = gi * g; m < (gi + 1) * g; ++m)
                for (int n = 0; n < N; ++n) {
                    float f = (float)q[((size_t)e * K + m) * N + n];      /* IntToFloat */
                    wdq[((size_t)e * K + m) * N + n] = f * sf[n];
                }
            free(sf);
        }
}

/* Sec. 3.4.1-3.4.3: integer-to-FP16 conversion without an I2F instruction.  The code is
 * stored offset by `offset` (128 for 8 bits, 8 for 4 bits) so that it is unsigned; OR-ing it
 * into the mantissa of FP16 1024.0 (0x6400) gives the FP16 number 1024 + code_plus, and an
 * FP16 subtraction of (1024 + offset) gives the signed integer as FP16.  Returns the FP16
 * bit pattern of the result; *biased_bits receives the intermediate pattern. */
uint16_t orc_i2f_magic(unsigned code_plus, unsigned offset, uint16_t *biased_bits)
{
    uint16_t biased = (uint16_t)(0x6400u | (code_plus & 0x3ffu));
    if (biased_bits) *biased_bits = biased;
    float diff = orc_f16_bits_to_f32(biased) - (float)(1024u + offset);   /* exact in float */
    return orc_f32_to_f16_bits(diff);                                     /* the FP16 result */
}

/* Sec. 3.4.3: the 4-bit storage order inside each group of eight codes. */
void orc_int4_interleave8(const int8_t *in /*[8]*/, int8_t *out /*[8]*/)
{
    static const int src[8] = {0, 2, 4, 6, 1, 3, 5, 7};
    for (int i = 0; i < 8; ++i) out[i] = in[src[i]];
}

/* ---------------------------------------------------------------- gating (Sec. 3.3)
 * logit[t,e] = sum_i x[t,i] * wg[i,e] + bias[e]; the k largest logits win (ties: lower
 * expert index; slot order: descending logit).  Sec. 3.3 defines the gate only as returning k
 * (scale, index) tuples per token, and Sec. 3.1 names Switch top-1 gating, so: softmax over all E
 * logits, scale = probability of the chosen expert; for k > 1 with `renorm` the k
 * probabilities are divided by their sum.
 *
 * Because the logits decide integers, their arithmetic is part of the definition: products
 * of two fp16 (or bf16) numbers are exact in float; they are added in float into four
 * partial sums, partial p taking the 128-element blocks b = i/128 with b % 4 == p, in
 * increasing i; then logit = ((p0 + p1) + p2) + p3, then + bias.
 */
void orc_gate(const float *x, const float *wg, const float *bias, const uint8_t *finished /*[T] or NULL*/,
              int T, int d, int E, int k,
              int renorm, int32_t *idx /*[T,k]*/, float *scale /*[T,k]*/,
              float *logits /*[T,E] or NULL*/)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        float *lg = (float *)malloc(sizeof(float) * (size_t)E);
        char *taken = (char *)calloc((size_t)E, 1);
        for (int e = 0; e < E; ++e) {
            float p[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            for (int i = 0; i < d; ++i) {
                float prod = x[(size_t)t * d + i] * wg[(size_t)i * E + e];
                int j = (i / 128) % 4;
                p[j] = p[j] + prod;
            }
            float l = ((p[0] + p[1]) + p[2]) + p[3];
            if (bias) l = l + bias[e];
            lg[e] = l;
            if (logits) logits[(size_t)t * E + e] = l;
        }
        float lmax = lg[0];
        for (int e = 1; e < E; ++e) if (lg[e] > lmax) lmax = lg[e];
        double denom = 0.0;
        for (int e = 0; e < E; ++e) denom += exp((double)lg[e] - (double)lmax);
        double psel[8], psum = 0.0;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e)
                if (!taken[e] && (best < 0 || lg[e] > lg[best])) best = e;
            taken[best] = 1;
            idx[(size_t)t * k + j] = best;
            psel[j] = exp((double)lg[best] - (double)lmax) / denom;
            psum += psel[j];
        }
        for (int j = 0; j < k; ++j)
            scale[(size_t)t * k + j] = (float)((k > 1 && renorm) ? psel[j] / psum : psel[j]);
        /* Batch pruning (Sec. 3.5): a finished row gets an expert index past the real experts, so
         * that the sort moves it behind every active row; it contributes nothing. */
        if (finished && finished[t])
            for (int j = 0; j < k; ++j) { idx[(size_t)t * k + j] = E; scale[(size_t)t * k + j] = 0.0f; }
        free(lg);
        free(taken);
    }
}

/* ---------------------------------------------------------------- routing (Sec. 3.3)
 * The (expert, row) tuples, flattened token-major as a = t*k + j, are sorted by expert with
 * a stable sort; perm_src[r] = a, inv_perm[a] = r, offsets[e] = number of tuples whose
 * expert is < e (the start of expert e's sub-matrix).  Tuples of pruned rows carry the index E
 * (Sec. 3.5) and sort behind all others: offsets[E] is the number of active rows (T*k without
 * pruning), and only the rows before it are processed downstream. */
void orc_permute(const int32_t *idx, int T, int k, int E, int32_t *perm_src, int32_t *inv_perm,
                 int32_t *offsets /*[E+1]*/)
{
    const int R = T * k;
    int r = 0;
    for (int e = 0; e < E; ++e) {
        offsets[e] = r;
        for (int a = 0; a < R; ++a)
            if (idx[a] == e) { perm_src[r] = a; inv_perm[a] = r; ++r; }
    }
    offsets[E] = r;
    for (int a = 0; a < R; ++a)
        if (idx[a] == E) { perm_src[r] = a; inv_perm[a] = r; ++r; }
}

void orc_gather_rows(const float *x, const int32_t *perm_src, int R, int k, int d, float *x_perm)
{
    for (int r = 0; r < R; ++r)
        memcpy(x_perm + (size_t)r * d, x + (size_t)(perm_src[r] / k) * d, sizeof(float) * (size_t)d);
}

/* ---------------------------------------------------------------- expert FFN (Sec. 3.3-3.4)
 * One expert, m rows: h = relu(x @ W1dq + b1), stored in the activation dtype (the paper keeps
 * activations in FP16); y = h @ W2dq + b2.  The activation function is not named in the
 * paper; ReLU is the reading taken (activation 0).  Activation 1 is GELU in its exact form,
 * x * Phi(x) = 0.5 x (1 + erf(x / sqrt 2)), offered as the second choice the method allows "without
 * loss of generality".  y is returned unrounded (rounding of the stored y, if
 * any, is the caller's: see orc_round_array). */
void orc_expert_ffn(const float *x /*[m,d]*/, int m, int d, int F,
                    const float *w1 /*[d,F]*/, const float *b1 /*[F] or NULL*/,
                    const float *w2 /*[F,d]*/, const float *b2 /*[d] or NULL*/,
                    int act_dtype, int activation /*0 relu, 1 gelu*/, float *h_out /*[m,F] or NULL*/,
                    float *y /*[m,d]*/)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < m; ++r) {
        double *acc = (double *)malloc(sizeof(double) * (size_t)(F > d ? F : d));
        float *h = (float *)malloc(sizeof(float) * (size_t)F);
        for (int n = 0; n < F; ++n) acc[n] = 0.0;
        for (int i = 0; i < d; ++i) {
            double a = (double)x[(size_t)r * d + i];
            const float *wrow = w1 + (size_t)i * F;
            for (int n = 0; n < F; ++n) acc[n] += a * (double)wrow[n];
        }
        for (int n = 0; n < F; ++n) {
            double v = acc[n] + (b1 ? (double)b1[n] : 0.0);
            double a = activation == 1 ? 0.5 * v * (1.0 + erf(v * 0.70710678118654752440)) : (v > 0.0 ? v : 0.0);
            h[n] = round_to((float)a, act_dtype);
            if (h_out) h_out[(size_t)r * F + n] = h[n];
        }
        for (int n = 0; n < d; ++n) acc[n] = 0.0;
        for (int i = 0; i < F; ++i) {
            double a = (double)h[i];
            const float *wrow = w2 + (size_t)i * d;
            for (int n = 0; n < d; ++n) acc[n] += a * (double)wrow[n];
        }
        for (int n = 0; n < d; ++n)
            y[(size_t)r * d + n] = (float)(acc[n] + (b2 ? (double)b2[n] : 0.0));
        free(acc);
        free(h);
    }
}

/* ---------------------------------------------------------------- combine (Sec. 3.3)
 * Rows go back to their original order and are multiplied by expert_scale; with k > 1 the k
 * scaled rows of a token are added, j ascending. */
void orc_combine(const float *y_perm /*[R,d]*/, const int32_t *inv_perm, const float *scale,
                 int T, int k, int d, int active_rows /* rows at or past it are pruned: they add 0 */,
                 float *out /*[T,d]*/)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < d; ++n) {
            double s = 0.0;
            for (int j = 0; j < k; ++j) {
                const int r = inv_perm[(size_t)t * k + j];
                if (r >= active_rows) continue;
                s += (double)scale[(size_t)t * k + j] * (double)y_perm[(size_t)r * d + n];
            }
            out[(size_t)t * d + n] = (float)s;
        }
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}

/* Threads the parallel loops above use from now on (n >= 1); for timing the oracle on one core.
 * Not part of any computation. */
void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
