// Shared host/device helpers of the HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <stdio.h>

#include "moe_wq.h"

namespace moe {

constexpr int kWave = 64;

// ---- error reporting (thread-local message behind moe_last_error) -------------------------
char *error_buffer();
int fail(int code, const char *fmt, ...);
int check_launch(const char *what);
void reset_kernel_notes();
void note_kernel(const char *name);

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- packed weight layout ------------------------------------------------------------------
// One matrix of one expert, logical shape [K, N], is cut into fragment blocks of 32 output
// channels.  A block of 1024 bytes is what one wavefront fetches with a single 16-byte load per
// lane, and a lane's 16 bytes are exactly the codes it feeds to v_mfma_f32_32x32x16_f16 as the
// B operand: lane l owns channel n = 32*nb + (l & 31) and, in MFMA step j, the eight K indices
// kbase + 16*j + 8*(l >> 5) + i, i = 0..7.
//   4-bit: a block spans 64 K values (4 MFMA steps); dword j of the lane holds step j, the code
//          for i in nibble position {0,4,1,5,2,6,3,7}[i] (pairs (i, i+1) sit 16 bits apart, so
//          one AND+OR builds two fp16 numbers).  Codes are stored +8.
//   8-bit: a block spans 32 K values (2 MFMA steps); byte 8*j + i of the lane holds the code
//          for step j, index i.  Codes are stored +128.
// Blocks are ordered [expert][nb][kb]: the K-stream of one 32-channel slab is contiguous.
constexpr int kFragN = 32;
constexpr int kFragBytes = 1024;
__host__ __device__ inline int frag_k(int bits) { return bits == 4 ? 64 : 32; }
__host__ __device__ inline size_t packed_bytes_per_expert(int K, int N, int bits)
{
    return (size_t)K * N * bits / 8;
}

}  // namespace moe
