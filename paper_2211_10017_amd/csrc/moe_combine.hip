// moe_combine: un-permute the expert outputs and apply expert_scale (Sec. 3.3, last step).
#include "moe_common.h"

namespace moe {

template <int DT>
__device__ inline void load4(const void *base, size_t idx4, float v[4])
{
    if (DT == MOE_F32) {
        const float4 f = reinterpret_cast<const float4 *>(base)[idx4];
        v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
    } else {
        const uint2 u = reinterpret_cast<const uint2 *>(base)[idx4];
        const uint32_t w[2] = {u.x, u.y};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint16_t b = (uint16_t)(w[i >> 1] >> (16 * (i & 1)));
            if (DT == MOE_BF16) v[i] = __uint_as_float((uint32_t)b << 16);
            else { __half h; *reinterpret_cast<uint16_t *>(&h) = b; v[i] = __half2float(h); }
        }
    }
}

__device__ inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int DT>
__device__ inline void store4(void *base, size_t idx4, const float v[4])
{
    if (DT == MOE_F32) {
        reinterpret_cast<float4 *>(base)[idx4] = make_float4(v[0], v[1], v[2], v[3]);
    } else {
        uint16_t b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (DT == MOE_BF16) b[i] = f32_to_bf16_rne(v[i]);
            else { __half h = __float2half_rn(v[i]); b[i] = *reinterpret_cast<uint16_t *>(&h); }
        }
        reinterpret_cast<uint2 *>(base)[idx4] =
            make_uint2((uint32_t)b[0] | ((uint32_t)b[1] << 16), (uint32_t)b[2] | ((uint32_t)b[3] << 16));
    }
}

template <int YDT, int ODT>
__global__ __launch_bounds__(256) void combine_kernel(const void *__restrict__ y_perm,
                                                      const int32_t *__restrict__ inv_perm,
                                                      const float *__restrict__ scale,
                                                      const int32_t *__restrict__ active_rows, int T, int k,
                                                      int d4, void *__restrict__ out)
{
    // rows at or past *active_rows belong to pruned tokens (Sec. 3.5): never computed, they add nothing
    const int active = active_rows ? *active_rows : 0x7fffffff;
    const size_t total = (size_t)T * d4;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const int t = (int)(i / d4), c = (int)(i % d4);
        float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int j = 0; j < k; ++j) {
            const int r = inv_perm[(size_t)t * k + j];
            if (r >= active) continue;
            const float s = scale[(size_t)t * k + j];
            float v[4];
            load4<YDT>(y_perm, (size_t)r * d4 + c, v);
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = fmaf(s, v[q], acc[q]);
        }
        store4<ODT>(out, i, acc);
    }
}

}  // namespace moe

extern "C" int moe_combine(const void *y_perm, int y_dtype, const int32_t *inv_perm,
                           const float *expert_scale, const int32_t *active_rows, int T, int k, int d,
                           void *out, int out_dtype, void *stream)
{
    using namespace moe;
    if (T == 0 && k > 0 && d > 0) return MOE_OK;         // empty buffers may be NULL
    if (!y_perm || !inv_perm || !expert_scale || !out) return fail(MOE_ERR_INVALID_ARG, "moe_combine: NULL pointer");
    if (T < 0 || k <= 0 || d <= 0 || d % 8) return fail(MOE_ERR_INVALID_ARG, "moe_combine: need T >= 0, k > 0, d > 0, d %% 8 == 0");
    if (y_dtype < 0 || y_dtype > 2 || out_dtype < 0 || out_dtype > 2) return fail(MOE_ERR_UNSUPPORTED, "moe_combine: unknown dtype");
    if (!aligned16(y_perm) || !aligned16(out)) return fail(MOE_ERR_INVALID_ARG, "moe_combine: buffers must be 16-byte aligned");
    const int d4 = d / 4;
    size_t blocks = ((size_t)T * d4 + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipStream_t s = as_stream(stream);
#define MOE_COMBINE_CASE(Y, O)                                                                       \
    if (y_dtype == Y && out_dtype == O) {                                                            \
        hipLaunchKernelGGL((combine_kernel<Y, O>), dim3((unsigned)blocks), dim3(256), 0, s, y_perm,  \
                           inv_perm, expert_scale, active_rows, T, k, d4, out);                                   \
        return check_launch("moe_combine");                                                          \
    }
    MOE_COMBINE_CASE(MOE_F16, MOE_F16) MOE_COMBINE_CASE(MOE_F16, MOE_BF16) MOE_COMBINE_CASE(MOE_F16, MOE_F32)
    MOE_COMBINE_CASE(MOE_BF16, MOE_F16) MOE_COMBINE_CASE(MOE_BF16, MOE_BF16) MOE_COMBINE_CASE(MOE_BF16, MOE_F32)
    MOE_COMBINE_CASE(MOE_F32, MOE_F16) MOE_COMBINE_CASE(MOE_F32, MOE_BF16) MOE_COMBINE_CASE(MOE_F32, MOE_F32)
#undef MOE_COMBINE_CASE
    return fail(MOE_ERR_UNSUPPORTED, "moe_combine: dtype combination not supported");
}
