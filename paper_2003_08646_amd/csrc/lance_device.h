// Device-side building blocks: Winograd 1-D transforms, the Eq. 7 quantizer, lane reductions.
// Compiled with -ffp-contract=off: every + - * below is one rounded binary32 operation, which
// is what makes the integer codes reproducible.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

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

// LDS code rows are 64 bytes (one channel block of one tile or filter).  The 16-byte chunk c of
// row r is stored at chunk position c ^ swizzle(r), with one of two functions:
//  * row_swizzle: rows that the quantize phases write with one 16-byte store per lane (lane =
//    row, a fixed chunk per wave).  Row bits (1,2): the stores of eight consecutive rows cover
//    all banks.
//  * row_swizzle_mfma32: rows that land in LDS through loads that write LDS and are read as
//    32 x 32 matrix-instruction fragments (lane & 31 = row, lane >> 5 = half of the contraction
//    bytes).  Row bits (2,3), found by measurement: on the streaming product kernel of a
//    512-channel layer bits (1,2) give 35 us and 3.2 M quad-cycles of SQ_LDS_BANK_CONFLICT, two
//    of the bits 2, 3, 4 give 32 us and 9 K, no swizzle 48 us.  (The quantize phases lose with
//    that choice: their stores then conflict.)
__device__ __forceinline__ int row_swizzle(int row) { return (row >> 1) & 3; }
__device__ __forceinline__ int row_swizzle_mfma32(int row) { return (row >> 2) & 3; }

// x / d for a divisor known on the host: magic = ceil(2^32 / d) (0 stands for d == 1).
// Exact for x * d < 2^32.
__device__ __forceinline__ int fast_div(int x, unsigned magic) {
  return magic == 0 ? x : (int)__umulhi((unsigned)x, magic);
}

// Workgroups are dealt to the 8 accelerator dies (XCDs, each with its own L2) round robin by
// their index.  This maps workgroup b of n to a work item such that every die gets one contiguous
// range of items: neighbouring items (tile blocks that share halo rows) then share an L2.
__device__ __forceinline__ int xcd_contiguous(int b, int n) {
  constexpr int kXcd = 8;
  const int x = b % kXcd, idx = b / kXcd;
  const int q = n / kXcd, r = n % kXcd;
  return x * q + min(x, r) + idx;
}

// Index of Y[n][k][yy][xx] (of X[n][c][yy][xx] alike): NCHW, or NHWC when nhwc.
__device__ __forceinline__ size_t act_index(bool nhwc, int n, int k, int yy, int xx, int K, int Ho,
                                            int Wo) {
  return nhwc ? (((size_t)n * Ho + yy) * Wo + xx) * K + k
              : (((size_t)n * K + k) * Ho + yy) * Wo + xx;
}

// NHWC output: stores v = the values of filters k .. k+3 of one output pixel at byte offset
// pix_bytes + 4*k of y (Y is [pixel][K]).  pix_ok: the pixel exists; kleft: filters that exist
// from k on; k4 (kernel-uniform): K is a multiple of 4, so the four are stored at once.  Stores
// that must not happen get an offset the buffer's range check drops.  y_bytes < 0xFFFFFFF0.
__device__ __forceinline__ void store_nhwc_k4(float* y, unsigned y_bytes, unsigned pix_bytes,
                                              unsigned k_bytes, bool pix_ok, int kleft, bool k4,
                                              float v0, float v1, float v2, float v3) {
  const __amdgpu_buffer_rsrc_t res = __builtin_amdgcn_make_buffer_rsrc(y, 0, y_bytes, 0x00020000);
  typedef unsigned v4u __attribute__((ext_vector_type(4)));
  constexpr unsigned kOob = 0xFFFFFFF0u;
  if (k4) {
    const v4u v = {__float_as_uint(v0), __float_as_uint(v1), __float_as_uint(v2), __float_as_uint(v3)};
    __builtin_amdgcn_raw_buffer_store_b128(v, res, (pix_ok && kleft >= 4) ? pix_bytes + k_bytes : kOob,
                                           0, 0);
  } else {
    const float vv[4] = {v0, v1, v2, v3};
#pragma unroll
    for (int q = 0; q < 4; q++)
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(vv[q]), res,
                                            (pix_ok && q < kleft) ? pix_bytes + k_bytes + 4u * q : kOob,
                                            0, 0);
  }
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

// Reduce NP (min,max) pairs over the 64 lanes of a wave, scattering the results: afterwards the
// lanes  id*(64/NP) .. id*(64/NP)+64/NP-1  all hold the reduced pair number id in (*lo, *hi).
// NP is 16 or 32.  Each halving step combines two lane groups and keeps half of the values in
// each (v_permlane32_swap, v_permlane16_swap, then DPP inside the rows of 16 lanes), so the cost
// is about 2*NP*2 instructions instead of 2*NP*6 for NP separate full reductions.
template <int NP>
__device__ __forceinline__ void wave_minmax_scatter(const float* mn, const float* mx, int lane,
                                                    float* lo, float* hi) {
  typedef unsigned v2u __attribute__((ext_vector_type(2)));
  // r[2k] = min-type, r[2k+1] = max-type: every pairing below keeps the parity of the index
  float r[2 * NP];
#pragma unroll
  for (int k = 0; k < NP; k++) { r[2 * k] = mn[k]; r[2 * k + 1] = mx[k]; }
  auto op = [](int idx, float a, float b) { return (idx & 1) ? fmaxf(a, b) : fminf(a, b); };
  constexpr int n1 = NP;  // registers after the lane-32 step
#pragma unroll
  for (int j = 0; j < n1; j++) {  // lanes 0-31 keep r[j], lanes 32-63 keep r[j+n1]
    const v2u s = __builtin_amdgcn_permlane32_swap(__float_as_uint(r[j]), __float_as_uint(r[j + n1]),
                                                   false, false);
    r[j] = op(j, __uint_as_float(s[0]), __uint_as_float(s[1]));
  }
  constexpr int n2 = n1 / 2;
#pragma unroll
  for (int j = 0; j < n2; j++) {  // even rows keep r[j], odd rows keep r[j+n2]
    const v2u s = __builtin_amdgcn_permlane16_swap(__float_as_uint(r[j]), __float_as_uint(r[j + n2]),
                                                   false, false);
    r[j] = op(j, __uint_as_float(s[0]), __uint_as_float(s[1]));
  }
  auto dppf = [](float x, auto ctrl) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x),
                                                      decltype(ctrl)::value, 0xF, 0xF, false));
  };
  constexpr int n3 = n2 / 2;
  const bool b3 = lane & 8, b2 = lane & 4;
#pragma unroll
  for (int j = 0; j < n3; j++) {  // partner = lane ^ 8 (rotate the row by 8)
    const float t0 = op(j, r[j], dppf(r[j], std::integral_constant<int, 0x128>{}));
    const float t1 = op(j, r[j + n3], dppf(r[j + n3], std::integral_constant<int, 0x128>{}));
    r[j] = b3 ? t1 : t0;
  }
  constexpr int n4 = n3 / 2;
#pragma unroll
  for (int j = 0; j < n4; j++) {  // partner = lane ^ 4: lane+4 for the keepers of r[j], lane-4 else
    const float t0 = op(j, r[j], dppf(r[j], std::integral_constant<int, 0x104>{}));            // row_shl:4
    const float t1 = op(j, r[j + n4], dppf(r[j + n4], std::integral_constant<int, 0x114>{}));  // row_shr:4
    r[j] = b2 ? t1 : t0;
  }
  if constexpr (NP == 32) {  // four registers left: one more scatter step over lane ^ 2
    const bool b1 = lane & 2;
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const float t0 = op(j, r[j], dppf(r[j], std::integral_constant<int, 0x4E>{}));
      const float t1 = op(j, r[j + 2], dppf(r[j + 2], std::integral_constant<int, 0x4E>{}));
      r[j] = b1 ? t1 : t0;
    }
  } else {  // two registers left: plain reduction over lane ^ 2
    r[0] = op(0, r[0], dppf(r[0], std::integral_constant<int, 0x4E>{}));
    r[1] = op(1, r[1], dppf(r[1], std::integral_constant<int, 0x4E>{}));
  }
  r[0] = op(0, r[0], dppf(r[0], std::integral_constant<int, 0xB1>{}));  // lane ^ 1
  r[1] = op(1, r[1], dppf(r[1], std::integral_constant<int, 0xB1>{}));
  *lo = r[0];
  *hi = r[1];
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
