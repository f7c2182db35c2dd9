// Tiled grouped GEMM kernels for 4-bit weights and bf16 activation rows.
#include "moe_ffn_tiled_kernel.h"

namespace moe {
void launch_tiled_4_bf16(const GemmArgs &p, int smode, int tm, dim3 grid, hipStream_t s)
{
    launch_tiled_variants<4, true>(p, smode, tm, grid, s);
}
}  // namespace moe
