// Tiled grouped GEMM kernels for 8-bit weights: the two forms that keep the group scales out of the FP16 weights
// (group sums folded in fp32; two-term weights), which fc1 of a bf16 layer needs.
#include "moe_ffn_tiled_kernel.h"

namespace moe {
void launch_tiled_8_exact(const GemmArgs &p, int smode, int tm, dim3 grid, hipStream_t s)
{
    launch_tiled_variants<8, true>(p, smode, tm, grid, s);
}
}  // namespace moe
