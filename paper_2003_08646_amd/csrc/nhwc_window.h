// The (m+2)^2 window of one tile for four consecutive channels of an NHWC tensor, one 16-byte
// buffer load per pixel.  Pixels outside the image (zero padding, ragged last tiles) get an
// offset beyond the buffer, which the load's range check turns into zeros: no select after the
// load, and one add and one select per pixel for its 32-bit offset.
#pragma once
#include "lance_device.h"

namespace lance {
namespace dev {

typedef float nw_f4 __attribute__((ext_vector_type(4)));

// x: the tensor [N][H][W][C], x_bytes its size (below 0xFFFFFFF0), 16-byte aligned, C a multiple
// of 4.  (n, y0, x0): image and top-left pixel of the window (may lie outside the image);
// c0: first of the four channels (a multiple of 4, c0 + 3 < C).
template <int M>
__device__ __forceinline__ void load_window_nhwc(const float* x, unsigned x_bytes, int n, int y0,
                                                 int x0, int c0, int H, int W, int C,
                                                 nw_f4 (&w)[(M + 2) * (M + 2)]) {
  constexpr int A = M + 2;
  constexpr unsigned kOob = 0xFFFFFFF0u;
  const __amdgpu_buffer_rsrc_t rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(x), 0, x_bytes, 0x00020000);
  const unsigned px = (unsigned)C * 4u;  // bytes per pixel
  unsigned coloff[A];
  bool cok[A];
#pragma unroll
  for (int s = 0; s < A; s++) {
    const int gx = x0 + s;
    cok[s] = gx >= 0 && gx < W;
    coloff[s] = (unsigned)gx * px + (unsigned)c0 * 4u;
  }
#pragma unroll
  for (int r = 0; r < A; r++) {
    const int gy = y0 + r;
    const bool rok = gy >= 0 && gy < H;
    const unsigned rowoff = ((unsigned)n * (unsigned)H + (unsigned)gy) * (unsigned)W * px;
#pragma unroll
    for (int s = 0; s < A; s++) {
      const unsigned off = (rok && cok[s]) ? rowoff + coloff[s] : kOob;
      w[r * A + s] = __builtin_bit_cast(nw_f4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0));
    }
  }
}

// One pixel row of a window: four channels of the pixels at byte offsets rowoff + coloff[s]
// (16-byte buffer loads); zeros where the row (rok) or the column (cok[s]) is outside the image.
template <int COLS>
__device__ __forceinline__ void load_row_nhwc(const float* x, unsigned x_bytes, unsigned rowoff,
                                              bool rok, const unsigned (&coloff)[COLS],
                                              const bool (&cok)[COLS], nw_f4 (&row)[COLS]) {
  constexpr unsigned kOob = 0xFFFFFFF0u;
  const __amdgpu_buffer_rsrc_t rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(x), 0, x_bytes, 0x00020000);
#pragma unroll
  for (int s = 0; s < COLS; s++) {
    const unsigned off = (rok && cok[s]) ? rowoff + coloff[s] : kOob;
    row[s] = __builtin_bit_cast(nw_f4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0));
  }
}

// Lane-per-tile form for layers with few channels: the byte offsets of the window's pixels
// (channel 0) are computed once, off[r*(m+2)+s], beyond the buffer for pixels outside the image.
template <int M>
__device__ __forceinline__ void window_offsets_nhwc(int n, int y0, int x0, int H, int W, int C,
                                                    unsigned (&off)[(M + 2) * (M + 2)]) {
  constexpr int A = M + 2;
  constexpr unsigned kOob = 0xFFFFFFF0u;
  const unsigned px = (unsigned)C * 4u;
#pragma unroll
  for (int r = 0; r < A; r++) {
    const int gy = y0 + r;
    const bool rok = gy >= 0 && gy < H;
    const unsigned rowoff = ((unsigned)n * (unsigned)H + (unsigned)gy) * (unsigned)W * px;
#pragma unroll
    for (int s = 0; s < A; s++) {
      const int gx = x0 + s;
      off[r * A + s] = (rok && gx >= 0 && gx < W) ? rowoff + (unsigned)gx * px : kOob;
    }
  }
}

// Channel c of that window: one 4-byte buffer load per pixel, the channel as the (wave-uniform)
// scalar offset.  x_bytes below 0xFFFFFFF0.
template <int M>
__device__ __forceinline__ void load_channel_nhwc(const float* x, unsigned x_bytes,
                                                  const unsigned (&off)[(M + 2) * (M + 2)], int c,
                                                  float (&b)[(M + 2) * (M + 2)]) {
  const __amdgpu_buffer_rsrc_t rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(x), 0, x_bytes, 0x00020000);
#pragma unroll
  for (int i = 0; i < (M + 2) * (M + 2); i++)
    b[i] = __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc, off[i], (unsigned)c * 4u, 0));
}

// All channels of that window's pixels at once for layers with at most four channels (an RGB
// image): one buffer load of 4*C bytes per pixel instead of C loads.  px[i][c] = channel c of
// pixel i (0 for c >= C and for pixels outside the image).  C (1 .. 4) is kernel-uniform.
template <int M>
__device__ __forceinline__ void load_pixels_nhwc(const float* x, unsigned x_bytes,
                                                 const unsigned (&off)[(M + 2) * (M + 2)], int C,
                                                 float (&px)[(M + 2) * (M + 2)][4]) {
  typedef unsigned v2u __attribute__((ext_vector_type(2)));
  typedef unsigned v3u __attribute__((ext_vector_type(3)));
  typedef unsigned v4u __attribute__((ext_vector_type(4)));
  constexpr int NPX = (M + 2) * (M + 2);
  const __amdgpu_buffer_rsrc_t rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(x), 0, x_bytes, 0x00020000);
#pragma unroll
  for (int i = 0; i < NPX; i++)
#pragma unroll
    for (int c = 0; c < 4; c++) px[i][c] = 0.0f;
  if (C == 4) {
#pragma unroll
    for (int i = 0; i < NPX; i++) {
      const v4u v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off[i], 0, 0);
#pragma unroll
      for (int c = 0; c < 4; c++) px[i][c] = __uint_as_float(v[c]);
    }
  } else if (C == 3) {
#pragma unroll
    for (int i = 0; i < NPX; i++) {
      const v3u v = __builtin_amdgcn_raw_buffer_load_b96(rsrc, off[i], 0, 0);
#pragma unroll
      for (int c = 0; c < 3; c++) px[i][c] = __uint_as_float(v[c]);
    }
  } else if (C == 2) {
#pragma unroll
    for (int i = 0; i < NPX; i++) {
      const v2u v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, off[i], 0, 0);
#pragma unroll
      for (int c = 0; c < 2; c++) px[i][c] = __uint_as_float(v[c]);
    }
  } else {
#pragma unroll
    for (int i = 0; i < NPX; i++)
      px[i][0] = __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc, off[i], 0, 0));
  }
}

}  // namespace dev
}  // namespace lance
