// moe_quantize_experts: symmetric range-based weight quantisation (Sec. 3.4) producing the
// interchange codes, the fp16 scales and the pre-shuffled offset-binary layout (Sec. 3.4.1)
// that the grouped FFN kernels stream.
#include "moe_common.h"

namespace moe {

// One block = 64 output channels x one scale group; 4 row phases per channel.
template <int BITS>
__global__ __launch_bounds__(256) void quantize_kernel(const float *__restrict__ w, int K, int N,
                                                       int g, int8_t *__restrict__ q_canon,
                                                       __half *__restrict__ scales,
                                                       uint8_t *__restrict__ q_packed)
{
    constexpr int QMAX = BITS == 8 ? 127 : 7;
    const int c = threadIdx.x & 63, ph = threadIdx.x >> 6;
    const int n = blockIdx.x * 64 + c;
    const int gi = blockIdx.y, e = blockIdx.z;
    const int G = K / g;
    const bool live = n < N;
    const int nc = live ? n : N - 1;             // clamp: idle lanes still read in bounds
    const float *we = w + (size_t)e * K * N;
    const int k0 = gi * g;

    __shared__ float s_amax[4][64];
    float amax = 0.0f;
    for (int m = k0 + ph; m < k0 + g; m += 4) amax = fmaxf(amax, fabsf(we[(size_t)m * N + nc]));
    s_amax[ph][c] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(s_amax[0][c], s_amax[1][c]), fmaxf(s_amax[2][c], s_amax[3][c]));

    const __half sh = __float2half_rn(amax / (float)QMAX);   // IEEE divide, round to nearest even
    const float s = __half2float(sh);
    if (ph == 0 && live) scales[((size_t)e * G + gi) * N + n] = sh;

    const size_t expert_bytes = packed_bytes_per_expert(K, N, BITS);
    const int nb = n >> 5, nl = n & 31;
    for (int ch = ph; ch < g / 8; ch += 4) {
        const int m0 = k0 + ch * 8;
        int code[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float v = 0.0f;
            if (s != 0.0f) {
                v = rintf(we[(size_t)(m0 + i) * N + nc] / s);
                v = fminf(fmaxf(v, (float)-QMAX), (float)QMAX);
            }
            code[i] = (int)v;
        }
        const int half = (m0 >> 3) & 1;
        if (BITS == 8) {
            if (q_canon && live) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    q_canon[((size_t)e * K + m0 + i) * N + n] = (int8_t)code[i];
            }
            if (q_packed && live) {
                const int kb = m0 >> 5, j = (m0 >> 4) & 1;
                uint32_t lo = 0, hi = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    lo |= (uint32_t)((code[i] + 128) & 0xff) << (8 * i);
                    hi |= (uint32_t)((code[i + 4] + 128) & 0xff) << (8 * i);
                }
                uint8_t *dst = q_packed + (size_t)e * expert_bytes +
                               ((size_t)nb * (K / 32) + kb) * kFragBytes + (half * 32 + nl) * 16 + j * 8;
                *reinterpret_cast<uint2 *>(dst) = make_uint2(lo, hi);
            }
        } else {
            if (q_canon) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int other = __shfl_xor(code[i], 1);
                    if (live && !(n & 1))
                        reinterpret_cast<uint8_t *>(q_canon)[((size_t)e * K + m0 + i) * (N / 2) + (n >> 1)] =
                            (uint8_t)((code[i] & 0xf) | ((other & 0xf) << 4));
                }
            }
            if (q_packed && live) {
                const int kb = m0 >> 6, j = (m0 >> 4) & 3;
                uint32_t word = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int pos = (i >> 1) + 4 * (i & 1);      // nibble positions 0,4,1,5,2,6,3,7
                    word |= (uint32_t)((code[i] + 8) & 0xf) << (4 * pos);
                }
                uint8_t *dst = q_packed + (size_t)e * expert_bytes +
                               ((size_t)nb * (K / 64) + kb) * kFragBytes + (half * 32 + nl) * 16 + j * 4;
                *reinterpret_cast<uint32_t *>(dst) = word;
            }
        }
    }
}

// Unquantised fp16 weights in the fragment layout (one MFMA step, 16 K values, per 1 KB block):
// lane l of block (nb, kb) holds w[16 kb + 8 (l >> 5) + 0..7][32 nb + (l & 31)].
__global__ __launch_bounds__(256) void pack_f16_kernel(const float *__restrict__ w, int K, int N,
                                                       uint16_t *__restrict__ packed)
{
    const int e = blockIdx.z, kb = blockIdx.y;
    const int nb = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (nb >= N / 32) return;
    const int n = nb * 32 + (lane & 31), k0 = kb * 16 + 8 * (lane >> 5);
    uint16_t v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const __half h = __float2half_rn(w[((size_t)e * K + k0 + i) * N + n]);
        v[i] = *reinterpret_cast<const uint16_t *>(&h);
    }
    uint16_t *dst = packed + (size_t)e * K * N + (((size_t)nb * (K / 16) + kb) * 64 + lane) * 8;
    *reinterpret_cast<uint4 *>(dst) = make_uint4(v[0] | (uint32_t)v[1] << 16, v[2] | (uint32_t)v[3] << 16,
                                                 v[4] | (uint32_t)v[5] << 16, v[6] | (uint32_t)v[7] << 16);
}

}  // namespace moe

extern "C" int moe_pack_fp16_experts(const float *w, int E, int K, int N, void *w_packed, void *stream)
{
    using namespace moe;
    if (!w || !w_packed) return fail(MOE_ERR_INVALID_ARG, "moe_pack_fp16_experts: NULL pointer");
    if (E <= 0 || K <= 0 || N <= 0) return fail(MOE_ERR_INVALID_ARG, "moe_pack_fp16_experts: E, K, N must be positive");
    if (N % 32 || K % 16) return fail(MOE_ERR_INVALID_ARG, "moe_pack_fp16_experts: need N %% 32 == 0 and K %% 16 == 0 (K=%d N=%d)", K, N);
    if (E > 65535 || K / 16 > 65535) return fail(MOE_ERR_UNSUPPORTED, "moe_pack_fp16_experts: too many experts or K blocks for one launch");
    if (!aligned16(w) || !aligned16(w_packed)) return fail(MOE_ERR_INVALID_ARG, "moe_pack_fp16_experts: buffers must be 16-byte aligned");
    dim3 grid((N / 32 + 3) / 4, K / 16, E);
    hipLaunchKernelGGL(pack_f16_kernel, grid, dim3(256), 0, as_stream(stream), w, K, N, (uint16_t *)w_packed);
    return check_launch("moe_pack_fp16_experts");
}

extern "C" int moe_quantize_experts(const float *w, int E, int K, int N, int bits, int group_size,
                                    void *q_canon, void *scales, void *q_packed, void *stream)
{
    using namespace moe;
    if (!w || !scales) return fail(MOE_ERR_INVALID_ARG, "moe_quantize_experts: w and scales must not be NULL");
    if (E <= 0 || K <= 0 || N <= 0) return fail(MOE_ERR_INVALID_ARG, "moe_quantize_experts: E, K, N must be positive");
    if (bits != 4 && bits != 8) return fail(MOE_ERR_UNSUPPORTED, "moe_quantize_experts: bits must be 4 or 8 (got %d)", bits);
    if (N % 32 || K % 64) return fail(MOE_ERR_INVALID_ARG, "moe_quantize_experts: need N %% 32 == 0 and K %% 64 == 0 (K=%d N=%d)", K, N);
    const int g = (group_size == 0 || group_size == K) ? K : group_size;
    if (g < 0 || g % 64 || K % g) return fail(MOE_ERR_INVALID_ARG, "moe_quantize_experts: group_size %d must be a multiple of 64 dividing K=%d", group_size, K);
    if (E > 65535 || K / g > 65535) return fail(MOE_ERR_UNSUPPORTED, "moe_quantize_experts: too many experts or groups for one launch");
    if (!aligned16(w) || !aligned16(scales) || !aligned16(q_canon) || !aligned16(q_packed))
        return fail(MOE_ERR_INVALID_ARG, "moe_quantize_experts: buffers must be 16-byte aligned");
    dim3 grid((N + 63) / 64, K / g, E);
    if (bits == 8)
        hipLaunchKernelGGL(quantize_kernel<8>, grid, dim3(256), 0, as_stream(stream), w, K, N, g,
                           (int8_t *)q_canon, (__half *)scales, (uint8_t *)q_packed);
    else
        hipLaunchKernelGGL(quantize_kernel<4>, grid, dim3(256), 0, as_stream(stream), w, K, N, g,
                           (int8_t *)q_canon, (__half *)scales, (uint8_t *)q_packed);
    return check_launch("moe_quantize_experts");
}
