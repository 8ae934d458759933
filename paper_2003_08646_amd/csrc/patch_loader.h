// Loading the (m+2)x(m+2) input patch of one tile (Sec. 2.3) straight from an NCHW image into
// registers, one lane per tile, with raw buffer loads.
//
// A lane's offsets are relative to the plane of (first image of the lane's tile block, channel)
// and are computed once per tile block; walking over channels only moves the scalar base of the
// buffer descriptor.  Zero padding comes from buffer range checking: a load whose offset lies
// beyond the descriptor's extent returns 0.
//
// Two ways to load a patch:
//  * rows: one 16-byte (plus one 8-byte for m = 4) load per patch row, starting at the patch's
//    first column wherever that is (4-byte alignment).  Rows outside the image get an offset
//    beyond the extent; columns outside the image are read from the neighbouring row and zeroed
//    afterwards (fix()).  Such a load touches up to 4 bytes before and a few elements after its
//    image row, so the descriptor starts kGuard bytes before the plane, and the caller may use
//    this way only for planes that are neither the first nor the last of the tensor
//    (rows_usable()), and only for layers with pad <= 1.
//  * elements: one dword load per pixel, pixels outside the image at an offset beyond the
//    extent.  Never touches memory outside the image rows; four times the load instructions.
#pragma once
#include "lance_device.h"

namespace lance {
namespace dev {

typedef float pl_f4 __attribute__((ext_vector_type(4)));
typedef float pl_f2 __attribute__((ext_vector_type(2)));

template <int M>
struct PatchLoader {
  static constexpr int A = M + 2;
  static constexpr unsigned kOutside = 0x80000000u;  // extents are below 2^31
  static constexpr unsigned kGuard = 16;

  unsigned rowoff[A];  // kGuard + byte offset of the patch row's first column; kOutside: no such row
  int ix0;             // image column of patch column 0 (negative inside the left padding)
  unsigned colmask;    // bit c: patch column c lies inside the image
  unsigned rowmask;    // bit r: patch row r lies inside the image
  bool first_image, last_image;  // wave-uniform: some lane's tile is in image 0 / image N-1
  unsigned before_mask;  // bit r: a row load of patch row r in the tensor's FIRST plane would start before the tensor
  unsigned after_mask;   // bit r: a row load of patch row r in the tensor's LAST plane would end after the tensor

  // img_elems: (image of the tile - first image of the block) * C * H * W
  __device__ __forceinline__ void setup(unsigned img_elems, int n_first, int n_last_lane, int N,
                                        int ty, int tx, int pad, int H, int W) {
    ix0 = tx * M - pad;
    colmask = 0;
    rowmask = 0;
#pragma unroll
    for (int c = 0; c < A; c++)
      if (ix0 + c >= 0 && ix0 + c < W) colmask |= 1u << c;
#pragma unroll
    for (int r = 0; r < A; r++) {
      const int iy = ty * M - pad + r;
      const bool ok = iy >= 0 && iy < H;
      rowoff[r] = ok ? (img_elems + (unsigned)iy * (unsigned)W + (unsigned)ix0) * 4u + kGuard : kOutside;
      if (ok) rowmask |= 1u << r;
    }
    before_mask = 0;
    after_mask = 0;
#pragma unroll
    for (int r = 0; r < A; r++) {
      const int iy = ty * M - pad + r;
      if (n_last_lane == 0 && iy == 0 && ix0 < 0) before_mask |= 1u << r;
      if (n_last_lane == N - 1 && iy == H - 1 && ix0 + A > W) after_mask |= 1u << r;
    }
    first_image = n_first == 0;
    // the largest image index of the wave sits in its last lane (tiles ascend with the lane)
    last_image = __builtin_amdgcn_readlane(n_last_lane, 63) == N - 1;
  }

  // Wave-uniform: may the planes of a set of channels be loaded by rows?  rows_allowed: the layer
  // permits it at all (pad <= 1, planes of at least 8 pixels); has_first / has_last: the set
  // contains channel 0 / channel C-1.
  __device__ __forceinline__ bool rows_usable(bool rows_allowed, bool has_first, bool has_last) const {
    return rows_allowed && !(first_image && has_first) && !(last_image && has_last);
  }

  // plane: (first image of the block, channel ch), wave-uniform.  extent: bytes from that plane
  // the block's offsets stay below.
  template <bool BY_ROWS>
  __device__ __forceinline__ void issue(const char* plane, unsigned extent, float (&b)[A * A]) const {
    if constexpr (BY_ROWS) {
      const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<char*>(plane - kGuard), 0, extent + 2 * kGuard, 0x00020000);
#pragma unroll
      for (int r = 0; r < A; r++) {
        const pl_f4 v =
            __builtin_bit_cast(pl_f4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, rowoff[r], 0, 0));
        b[r * A + 0] = v[0]; b[r * A + 1] = v[1]; b[r * A + 2] = v[2]; b[r * A + 3] = v[3];
        if constexpr (A == 6) {
          const pl_f2 w = __builtin_bit_cast(
              pl_f2, __builtin_amdgcn_raw_buffer_load_b64(rsrc, rowoff[r] + 16u, 0, 0));
          b[r * A + 4] = w[0]; b[r * A + 5] = w[1];
        }
      }
    } else {
      const __amdgpu_buffer_rsrc_t rsrc =
          __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(plane), 0, extent, 0x00020000);
      // The pixel offsets are formed here, from a copy of ix0 the compiler cannot see through:
      // two calls then share no offsets, so none is kept in registers between them (a kernel
      // that mostly loads by rows calls this for the odd plane only).
      int ix = ix0;
      asm volatile("" : "+v"(ix));
#pragma unroll
      for (int r = 0; r < A; r++) {
        const unsigned row0 = rowoff[r] - kGuard - 4u * (unsigned)ix;  // column 0 of the image row
#pragma unroll
        for (int c = 0; c < A; c++) {
          const bool ok = ((rowmask >> r) & 1u) && ((colmask >> c) & 1u);
          const unsigned o = ok ? row0 + 4u * (unsigned)(ix + c) : kOutside;
          b[r * A + c] = __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc, o, 0, 0));
        }
      }
    }
  }

  // Row loads that are safe in the first (first_plane) or the last (last_plane) plane of the
  // tensor, for layers whose patches stick out of the image by at most one column on either side
  // (patch_edge_cols_only) and whose rows hold at least A pixels (lane_off: a per-lane constant
  // added to every offset, e.g. a channel plane of the lane's own): the one row load that would
  // start before the tensor starts one pixel later, those that would end after the tensor start
  // one pixel earlier; unshift() puts the pixels back into their columns.  Both flags are
  // wave-uniform; the code is branch-free.
  __device__ __forceinline__ void issue_rows_shifted(const char* plane, unsigned extent,
                                                     bool first_plane, bool last_plane,
                                                     float (&b)[A * A], unsigned lane_off = 0) const {
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(plane - kGuard), 0, extent + 2 * kGuard, 0x00020000);
    const unsigned fm = first_plane ? before_mask : 0u, lm = last_plane ? after_mask : 0u;
#pragma unroll
    for (int r = 0; r < A; r++) {
      unsigned o = rowoff[r] + lane_off;
      o = ((fm >> r) & 1u) ? o + 4u : o;
      o = ((lm >> r) & 1u) ? o - 4u : o;
      const pl_f4 v = __builtin_bit_cast(pl_f4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, o, 0, 0));
      b[r * A + 0] = v[0]; b[r * A + 1] = v[1]; b[r * A + 2] = v[2]; b[r * A + 3] = v[3];
      if constexpr (A == 6) {
        const pl_f2 w =
            __builtin_bit_cast(pl_f2, __builtin_amdgcn_raw_buffer_load_b64(rsrc, o + 16u, 0, 0));
        b[r * A + 4] = w[0]; b[r * A + 5] = w[1];
      }
    }
  }
  __device__ __forceinline__ void unshift(bool first_plane, bool last_plane, float (&d)[A][A]) const {
    const unsigned fm = first_plane ? before_mask : 0u, lm = last_plane ? after_mask : 0u;
#pragma unroll
    for (int r = 0; r < A; r++) {
      const bool f = (fm >> r) & 1u, l = (lm >> r) & 1u;
      float v[A];
#pragma unroll
      for (int c = 0; c < A; c++) v[c] = d[r][c];
      // loaded one pixel later: columns move up; one pixel earlier: columns move down; the
      // column that falls outside the image is zeroed by fix()
#pragma unroll
      for (int c = 0; c < A; c++) {
        const float up = c > 0 ? v[c - 1] : v[c], down = c + 1 < A ? v[c + 1] : v[c];
        d[r][c] = f ? up : (l ? down : v[c]);
      }
    }
  }

  // Zero the columns that a row load took from outside the image (harmless after a load by
  // elements).  EDGE_ONLY: the layer guarantees that only columns 0 and A-1 can be outside
  // (see patch_edge_cols_only); branch-free either way, so that the caller's straight-line code
  // stays one basic block.
  template <bool EDGE_ONLY>
  __device__ __forceinline__ void fix(float (&d)[A][A]) const {
#pragma unroll
    for (int r = 0; r < A; r++)
#pragma unroll
      for (int c = 0; c < A; c++)
        if (!EDGE_ONLY || c == 0 || c == A - 1) d[r][c] = ((colmask >> c) & 1u) ? d[r][c] : 0.0f;
  }
};

}  // namespace dev
}  // namespace lance
