// Algorithm 1 taken literally, as an accuracy ablation on the GPU: for every filter k, tile p and
// channel c the transformed filter G g G^T and the transformed patch B^T d B are quantized with
// the range of their own (m+2) x (m+2) matrix (the most literal reading of T, the matrix a value
// belongs to, in Eq. 7), the codes are de-quantized (Eq. 8), multiplied, and the products summed over the
// channels in binary32; then S = A^T m A (Eq. 9).  With ranges of their own per matrix the
// channel sum is no integer product, so this path uses no matrix cores and is not the fast
// path: it exists to measure what the per-position ranges of the GEMM form cost in accuracy.
//
// Lane = tile, a workgroup takes 256 tiles and kFilters filters.  Per channel: every lane forms
// the de-quantized codes of its own patch; the first kFilters lanes form those of the
// workgroup's filters and leave them in LDS; E multiply-adds per filter and lane.
#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

constexpr int kThreads = 256;
constexpr int kFilters = 4;

struct LitArgs {
  const float* x;
  const float* w;
  float* y;
  int N, C, H, W, K, pad, th, tw, P, Ho, Wo, bits, bits_w, nhwc;
};

// v[i][j] <- Q'(Q(v[i][j])) with T = the matrix itself (Eq. 7, Eq. 8), codes of `bits` bits.
template <int A>
__device__ __forceinline__ void fake_quantize_matrix(float (&v)[A][A], int bits) {
  float mn = v[0][0], mx = v[0][0];
#pragma unroll
  for (int i = 0; i < A; i++)
#pragma unroll
    for (int j = 0; j < A; j++) { mn = fminf(mn, v[i][j]); mx = fmaxf(mx, v[i][j]); }
  float inv, scale;
  dev::quant_params(mn, mx, bits, &inv, &scale);
  const float L = (float)((1 << bits) - 1);
#pragma unroll
  for (int i = 0; i < A; i++)
#pragma unroll
    for (int j = 0; j < A; j++) {
      const float code = fminf(fmaxf(rintf((v[i][j] - mn) * inv), 0.0f), L);
      v[i][j] = code * scale + mn;
    }
}

template <int M>
__global__ __launch_bounds__(kThreads) void alg1_literal_kernel(const LitArgs a) {
  constexpr int A = M + 2, E = A * A;
  __shared__ float us[kFilters][E];
  const int tid = threadIdx.x;
  const int p = blockIdx.x * kThreads + tid;
  const int k0 = blockIdx.y * kFilters;
  const bool valid = p < a.P;
  const int pt = min(p, a.P - 1);
  const int tx = pt % a.tw, t2 = pt / a.tw;
  const int ty = t2 % a.th, n = t2 / a.th;
  const int y0 = ty * M - a.pad, x0 = tx * M - a.pad;
  float acc[kFilters][E];
#pragma unroll
  for (int f = 0; f < kFilters; f++)
#pragma unroll
    for (int e = 0; e < E; e++) acc[f][e] = 0.0f;

  for (int c = 0; c < a.C; c++) {
    __syncthreads();  // the previous channel's filter values have been read
    if (tid < kFilters) {
      const int k = min(k0 + tid, a.K - 1);
      float g[3][3], u[A][A];
      const float* src = a.w + ((size_t)k * a.C + c) * 9;
#pragma unroll
      for (int r = 0; r < 3; r++)
#pragma unroll
        for (int s = 0; s < 3; s++) g[r][s] = src[r * 3 + s];
      dev::filter_tile_transform<M>(g, u);
      fake_quantize_matrix<A>(u, a.bits_w);
#pragma unroll
      for (int e = 0; e < E; e++) us[tid][e] = u[e / A][e % A];
    }
    float d[A][A];
#pragma unroll
    for (int r = 0; r < A; r++)
#pragma unroll
      for (int s = 0; s < A; s++) {
        const int gy = y0 + r, gx = x0 + s;
        const bool ok = gy >= 0 && gy < a.H && gx >= 0 && gx < a.W;
        const float v = a.x[dev::act_index(a.nhwc, n, c, min(max(gy, 0), a.H - 1),
                                           min(max(gx, 0), a.W - 1), a.C, a.H, a.W)];
        d[r][s] = ok ? v : 0.0f;
      }
    dev::input_tile_transform<M>(d);
    fake_quantize_matrix<A>(d, a.bits);
    __syncthreads();
#pragma unroll
    for (int f = 0; f < kFilters; f++)
#pragma unroll
      for (int e = 0; e < E; e++) acc[f][e] = __builtin_fmaf(us[f][e], d[e / A][e % A], acc[f][e]);
  }

  if (!valid) return;
#pragma unroll
  for (int f = 0; f < kFilters; f++) {
    const int k = k0 + f;
    if (k >= a.K) break;
    // S = A^T M A: rows first, then columns
    float t[M][A];
#pragma unroll
    for (int o = 0; o < M; o++)
#pragma unroll
      for (int j = 0; j < A; j++) {
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < A; i++) {
          const float cf = dev::Wino<M>::at(o, i);
          if (cf != 0.0f) s += cf * acc[f][i * A + j];
        }
        t[o][j] = s;
      }
#pragma unroll
    for (int o = 0; o < M; o++)
#pragma unroll
      for (int q = 0; q < M; q++) {
        float s = 0.0f;
#pragma unroll
        for (int j = 0; j < A; j++) {
          const float cf = dev::Wino<M>::at(q, j);
          if (cf != 0.0f) s += cf * t[o][j];
        }
        const int yy = ty * M + o, xx = tx * M + q;
        if (yy < a.Ho && xx < a.Wo) a.y[dev::act_index(a.nhwc, n, k, yy, xx, a.K, a.Ho, a.Wo)] = s;
      }
  }
}

}  // namespace

hipError_t launch_alg1_literal(const Geo& g, const float* x, const float* w, float* y,
                               hipStream_t s) {
  const LitArgs a{x, w, y, g.N, g.C, g.H, g.W, g.K, g.pad, g.th, g.tw, g.P, g.Ho, g.Wo, g.bits,
                  g.bits_w, is_nhwc(g) ? 1 : 0};
  const long long bx = ((long long)g.P + kThreads - 1) / kThreads, by = (g.K + kFilters - 1) / kFilters;
  if (bx > 0x7FFFFFFFLL || by > 65535) return hipErrorInvalidValue;
  dim3 grid((unsigned)bx, (unsigned)by, 1);
  if (g.m == 2) alg1_literal_kernel<2><<<grid, kThreads, 0, s>>>(a);
  else alg1_literal_kernel<4><<<grid, kThreads, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace lance
