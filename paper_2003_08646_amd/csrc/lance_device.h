// Device-side building blocks: Winograd 1-D transforms, the Eq. 7 quantizer, lane reductions.
// Compiled with -ffp-contract=off: every + - * below is one rounded binary32 operation, which
// is what makes the integer codes reproducible.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lance {
namespace dev {

// ---- F(m x m, 3 x 3) transforms (Sec. 2.3, Eq. 4), one dimension at a time ---------------
// The 2-D transform applies the 1-D form to every column (left factor), then to every row of
// the result (right factor).
template <int M> struct Wino;

template <> struct Wino<2> {
  static constexpr int A = 4;
  // t = B^T d, points {0, 1, -1, inf}
  __device__ __forceinline__ static void in1d(const float (&d)[4], float (&t)[4]) {
    t[0] = d[0] - d[2];
    t[1] = d[1] + d[2];
    t[2] = d[2] - d[1];
    t[3] = d[1] - d[3];
  }
  // u = G g
  __device__ __forceinline__ static void flt1d(const float (&g)[3], float (&u)[4]) {
    const float s = g[0] + g[2];
    u[0] = g[0];
    u[1] = (s + g[1]) * 0.5f;
    u[2] = (s - g[1]) * 0.5f;
    u[3] = g[2];
  }
  // A^T rows: {1,1,1,0}, {0,1,-1,-1}
  __device__ __forceinline__ static float at(int o, int i) {
    constexpr float T[2][4] = {{1, 1, 1, 0}, {0, 1, -1, -1}};
    return T[o][i];
  }
};

template <> struct Wino<4> {
  static constexpr int A = 6;
  // t = B^T d, points {0, 1, -1, 2, -2, inf}
  __device__ __forceinline__ static void in1d(const float (&d)[6], float (&t)[6]) {
    t[0] = (4.0f * d[0] - 5.0f * d[2]) + d[4];
    const float p = d[4] - 4.0f * d[2];
    const float q = d[3] - 4.0f * d[1];
    t[1] = p + q;
    t[2] = p - q;
    const float r = d[4] - d[2];
    const float s = 2.0f * (d[3] - d[1]);
    t[3] = r + s;
    t[4] = r - s;
    t[5] = (4.0f * d[1] - 5.0f * d[3]) + d[5];
  }
  __device__ __forceinline__ static void flt1d(const float (&g)[3], float (&u)[6]) {
    const float c6 = (float)(1.0 / 6.0), c24 = (float)(1.0 / 24.0);
    const float s = g[0] + g[2];
    const float a = g[0] + 4.0f * g[2];
    const float b = 2.0f * g[1];
    u[0] = 0.25f * g[0];
    u[1] = (s + g[1]) * (-c6);
    u[2] = (s - g[1]) * (-c6);
    u[3] = (a + b) * c24;
    u[4] = (a - b) * c24;
    u[5] = g[2];
  }
  __device__ __forceinline__ static float at(int o, int i) {
    constexpr float T[4][6] = {
        {1, 1, 1, 1, 1, 0}, {0, 1, -1, 2, -2, 0}, {0, 1, 1, 4, 4, 0}, {0, 1, -1, 8, -8, 1}};
    return T[o][i];
  }
};

// A^T[o][i] of F(m x m, 3 x 3) for run-time indices (o < m, i < m+2).
__device__ __forceinline__ float at_coef(int m, int o, int i) {
  static constexpr float T2[2][4] = {{1, 1, 1, 0}, {0, 1, -1, -1}};
  static constexpr float T4[4][6] = {
      {1, 1, 1, 1, 1, 0}, {0, 1, -1, 2, -2, 0}, {0, 1, 1, 4, 4, 0}, {0, 1, -1, 8, -8, 1}};
  return m == 2 ? T2[o][i] : T4[o][i];
}

// V = B^T d B for one (m+2)x(m+2) patch held in registers (in place).
template <int M>
__device__ __forceinline__ void input_tile_transform(float (&d)[Wino<M>::A][Wino<M>::A]) {
  constexpr int A = Wino<M>::A;
#pragma unroll
  for (int j = 0; j < A; j++) {
    float col[A], out[A];
#pragma unroll
    for (int i = 0; i < A; i++) col[i] = d[i][j];
    Wino<M>::in1d(col, out);
#pragma unroll
    for (int i = 0; i < A; i++) d[i][j] = out[i];
  }
#pragma unroll
  for (int i = 0; i < A; i++) {
    float out[A];
    Wino<M>::in1d(d[i], out);
#pragma unroll
    for (int j = 0; j < A; j++) d[i][j] = out[j];
  }
}

// U = G g G^T for one 3x3 filter.
template <int M>
__device__ __forceinline__ void filter_tile_transform(const float (&g)[3][3],
                                                      float (&u)[Wino<M>::A][Wino<M>::A]) {
  constexpr int A = Wino<M>::A;
  float t[A][3];
#pragma unroll
  for (int s = 0; s < 3; s++) {
    float col[3], out[A];
#pragma unroll
    for (int r = 0; r < 3; r++) col[r] = g[r][s];
    Wino<M>::flt1d(col, out);
#pragma unroll
    for (int i = 0; i < A; i++) t[i][s] = out[i];
  }
#pragma unroll
  for (int i = 0; i < A; i++) {
    float out[A];
    Wino<M>::flt1d(t[i], out);
#pragma unroll
    for (int j = 0; j < A; j++) u[i][j] = out[j];
  }
}

// ---- Eq. 7 / Eq. 8 parameters ------------------------------------------------------------
// inv = (float)(L / (max - min)), scale = (float)((max - min) / L), quotients in binary64.
__device__ __forceinline__ void quant_params(float mn, float mx, int bits, float* inv,
                                             float* scale) {
  const double L = (double)((1 << bits) - 1);
  const double range = (double)mx - (double)mn;
  if (range == 0.0) {
    *inv = 0.0f;
    *scale = 0.0f;
    return;
  }
  float i = (float)(L / range);
  if (!(fabsf(i) <= 3.402823466e+38f)) i = 0.0f;  // not finite
  *inv = i;
  *scale = (float)(range / L);
}

// Signed stored code of Eq. 7: clamp(rne((x - mn) * inv), 0, L) - h.
__device__ __forceinline__ int quantize_code(float x, float mn, float inv, float L, int h) {
  float t = (x - mn) * inv;
  float r = rintf(t);
  r = fminf(fmaxf(r, 0.0f), L);
  return (int)r - h;
}

// ---- lane reductions ---------------------------------------------------------------------
// Sum over each aligned group of 16 lanes, result in every lane of the group (DPP only).
__device__ __forceinline__ int row16_sum(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
  v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, false);  // row_half_mirror
  v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, false);  // row_mirror
  return v;
}

__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

}  // namespace dev
}  // namespace lance
