// Tiled grouped GEMM kernels for 8-bit weights: per-channel scales and group scales multiplied into the FP16 weights.
#include "moe_ffn_tiled_kernel.h"

namespace moe {
void launch_tiled_8(const GemmArgs &p, int smode, int tm, dim3 grid, hipStream_t s)
{
    launch_tiled_variants<8, false>(p, smode, tm, grid, s);
}
}  // namespace moe
