// Packed 4-bit codes (two to a byte, each as code + 8; block rows of 32 bytes) on their way from
// memory through LDS into matrix-instruction fragments.  Shared by the product kernels that read
// packed code tensors.
#pragma once
#include <hip/hip_runtime.h>

namespace lance {
namespace pk {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kRow = 32;  // bytes of a packed block row

// One wave-wide copy moves 32 rows x 32 B = 1 KB; lane l's 16 bytes land at 16*l.  Lane l takes
// chunk (l >> 4) & 1 of row (l & 15) + 16 * (l >> 5), so that the 8-byte fragment reads of 16
// consecutive rows cover all banks.
__device__ __forceinline__ int lane_row(int l) { return (l & 15) + 16 * (l >> 5); }
__device__ __forceinline__ int lane_chunk(int l) { return (l >> 4) & 1; }
// Byte offset, inside its 1 KB piece, of the 8-byte part `half8` of chunk `chunk` of row `row`.
__device__ __forceinline__ unsigned frag_offset(int row, int chunk, int half8) {
  return (unsigned)(((row & 15) + 16 * chunk + 32 * (row >> 4)) * 16 + 8 * half8);
}
// 8 packed bytes -> 16 contraction bytes (the low nibbles of the 8 bytes, then the high ones), as
// the unsigned values code + 8.  Any order serves as long as both operands use the same.
__device__ __forceinline__ v4i unpack(const v2i x) {
  constexpr unsigned kM = 0x0F0F0F0Fu;
  v4i r;
  r[0] = (int)((unsigned)x[0] & kM);
  r[1] = (int)((unsigned)x[1] & kM);
  r[2] = (int)(((unsigned)x[0] >> 4) & kM);
  r[3] = (int)(((unsigned)x[1] >> 4) & kM);
  return r;
}

}  // namespace pk
}  // namespace lance
