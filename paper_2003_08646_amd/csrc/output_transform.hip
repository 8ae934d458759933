// Stage 4 alone: m~ = Q'(m^) (Eq. 8 on both operands, expanded), S = A^T m A, tiles merged into
// Y (Eq. 9, Algorithm 1).  One lane per (k, p): reads the E accumulators of that pair (lanes
// run along p, so every read is coalesced), writes an m x m output patch row by row (one store per
// row).  A loop over several filters per workgroup, to form the constants less often, was tried:
// it helps layers whose accumulators fit the last-level cache (cfg2: 34 -> 27 us) and costs more on
// the others (the compiler carries 4*E constants or 3*E addresses in registers across the loop).
#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

constexpr int kThreads = 256;

template <int M>
__global__ __launch_bounds__(kThreads) void output_transform_kernel(
    const int32_t* __restrict__ acc, const float* __restrict__ u_range,
    const int32_t* __restrict__ u_rowsum, const float* __restrict__ v_range,
    const int32_t* __restrict__ v_colsum, float* __restrict__ y, int K, int P, int C, int bits,
    int bits_w, int th, int tw, int Ho, int Wo, int nhwc) {
  constexpr int A = M + 2, E = A * A;
  __shared__ float c_acc[E], c_row[E], c_col[E], c_const[E];
  if (threadIdx.x < E) {
    const int e = threadIdx.x;
    float iu, su, iv, sv;
    dev::quant_params(u_range[2 * e], u_range[2 * e + 1], bits_w, &iu, &su);
    dev::quant_params(v_range[2 * e], v_range[2 * e + 1], bits, &iv, &sv);
    // each operand's stored code is its Eq. 7 code minus its own 2^(b-1)
    const double ou = (double)u_range[2 * e] + (double)su * (double)(1 << (bits_w - 1));
    const double ov = (double)v_range[2 * e] + (double)sv * (double)(1 << (bits - 1));
    c_acc[e] = (float)((double)su * (double)sv);
    c_row[e] = (float)((double)su * ov);
    c_col[e] = (float)((double)sv * ou);
    c_const[e] = (float)((double)C * ou * ov);
  }
  __syncthreads();
  const int p = blockIdx.x * kThreads + threadIdx.x;
  const int k = blockIdx.y;
  if (p >= P) return;
  float mm[A][A];
#pragma unroll
  for (int e = 0; e < E; e++) {
    const float a = (float)acc[((size_t)e * K + k) * P + p];
    const float ru = (float)u_rowsum[(size_t)e * K + k];
    const float cv = (float)v_colsum[(size_t)e * P + p];
    mm[e / A][e % A] = ((c_acc[e] * a + c_row[e] * ru) + c_col[e] * cv) + c_const[e];
  }
  // S = A^T M A : rows first, then columns
  float t[M][A];
#pragma unroll
  for (int o = 0; o < M; o++)
#pragma unroll
    for (int j = 0; j < A; j++) {
      float s = 0.0f;
#pragma unroll
      for (int i = 0; i < A; i++) {
        const float c = dev::Wino<M>::at(o, i);
        if (c != 0.0f) s += c * mm[i][j];
      }
      t[o][j] = s;
    }
  const int tx = p % tw, t2 = p / tw;
  const int ty = t2 % th, n = t2 / th;
  // a tile's row of M outputs is contiguous in an NCHW plane: one store of 4*M bytes when the row
  // lies inside the image (any 4-byte alignment), so that the lanes of a wave write whole lines
  typedef float rowv __attribute__((ext_vector_type(M), aligned(4)));
  const bool row_inside = !nhwc && tx * M + M - 1 < Wo;
#pragma unroll
  for (int o = 0; o < M; o++) {
    const int yy = ty * M + o;
    float s[M];
#pragma unroll
    for (int q = 0; q < M; q++) {
      s[q] = 0.0f;
#pragma unroll
      for (int j = 0; j < A; j++) {
        const float c = dev::Wino<M>::at(q, j);
        if (c != 0.0f) s[q] += c * t[o][j];
      }
    }
    if (yy < Ho) {
      if (row_inside) {
        rowv v;
#pragma unroll
        for (int q = 0; q < M; q++) v[q] = s[q];
        *reinterpret_cast<rowv*>(y + dev::act_index(0, n, k, yy, tx * M, K, Ho, Wo)) = v;
      } else {
#pragma unroll
        for (int q = 0; q < M; q++) {
          const int xx = tx * M + q;
          if (xx < Wo) y[dev::act_index(nhwc, n, k, yy, xx, K, Ho, Wo)] = s[q];
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_output_transform(const Geo& g, const int32_t* acc, const float* u_range,
                                   const int32_t* u_rowsum, const float* v_range,
                                   const int32_t* v_colsum, float* y, hipStream_t s) {
  dim3 grid((g.P + kThreads - 1) / kThreads, g.K, 1);
  if (g.K > 65535) return hipErrorInvalidValue;
  if (g.m == 2)
    output_transform_kernel<2><<<grid, kThreads, 0, s>>>(acc, u_range, u_rowsum, v_range, v_colsum,
                                                         y, g.K, g.P, g.C, g.bits, g.bits_w, g.th, g.tw,
                                                         g.Ho, g.Wo, is_nhwc(g) ? 1 : 0);
  else
    output_transform_kernel<4><<<grid, kThreads, 0, s>>>(acc, u_range, u_rowsum, v_range, v_colsum,
                                                         y, g.K, g.P, g.C, g.bits, g.bits_w, g.th, g.tw,
                                                         g.Ho, g.Wo, is_nhwc(g) ? 1 : 0);
  return hipGetLastError();
}

}  // namespace lance
