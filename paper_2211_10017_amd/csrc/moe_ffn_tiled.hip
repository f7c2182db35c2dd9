// Host side of the LDS-tiled grouped GEMM: tile height, grid size, and the hand-over to the
// translation unit that holds the kernels of the weight width and activation dtype asked for.
#include "moe_ffn_common.h"

namespace moe {

int launch_tiled_gemm(const GemmArgs &p, int bits, int smode, hipStream_t s)
{
    // row-tile height from the mean rows per expert (the offsets themselves stay on the device)
    const int mean = (p.R + p.E - 1) / p.E;
    // 64-row tiles also for taller experts where a third block per CU pays more than halving the
    // dequantisation does: short K loops (the prologue and epilogue of a block then overlap the loops of
    // two others, not of one), and 8-bit weights up to 256 rows per expert (their 128-row tile has
    // registers for one set of weights in flight only)
    int tm = mean <= 32 ? 1 : (mean <= 64 || p.K <= 2048 || (bits == 8 && mean <= 256)) ? 2 : 4;
    if (smode == SCALE_GROUP_ACC && tm > 2) tm = 2;
    const long most = p.R;                                      // experts that can hold rows
    const long ncol = (p.N + 255) / 256;
    // Tiles may be lower than the kernel's 32 * tm rows (it skips row tiles that hold no rows): with few
    // column blocks the launch is a handful of rounds of 512 blocks (two per CU), and 96-row tiles
    // can fill the last round better than 128-row tiles leave it.  Cost model: rounds x tile height,
    // lower tiles charged 6 % per step down for streaming the weights more often.
    int units = tm;
    if (tm == 4) {
        double best = 0;
        for (int u = 4; u >= 2; --u) {
            const long items = ((long)p.R / (32 * u) + (p.E < most ? p.E : most) / 2) * ncol;
            const double cost = (double)((items + 511) / 512) * u * (1.0 + 0.06 * (4 - u));
            if (u == 4 || cost < best) { best = cost; units = u; }
        }
    }
    GemmArgs q = p;
    q.tile_units = units;
    const long slots = (long)p.R / (32 * units) + (p.E < most ? p.E : most);
    if (slots == 0) return MOE_OK;
    const long wgs = (slots * ncol + kXcds - 1) / kXcds * kXcds;   // upper bound of the work items, whole rounds of XCDs
    if (wgs > 0x7fffffffL) return fail(MOE_ERR_UNSUPPORTED, "moe_grouped_ffn_wq: %ld workgroups exceed one launch", wgs);
    dim3 grid((unsigned)wgs);
    const bool exact = smode == SCALE_GROUP_ACC || smode == SCALE_GROUP_SPLIT;
    if (bits == 4) (exact ? launch_tiled_4_exact : launch_tiled_4)(q, smode, tm, grid, s);
    else (exact ? launch_tiled_8_exact : launch_tiled_8)(q, smode, tm, grid, s);
    return check_launch("moe_grouped_ffn_wq (gemm)");
}

}  // namespace moe
