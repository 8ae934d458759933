// Stage 1: u^ = Q(G g G^T) for every filter (Algorithm 1; Eq. 7).  Runs once per set of
// weights (Sec. 3.4), so it is written for clarity; it still streams W once per pass.
//
//   pass A  one workgroup per filter k: transform every (k,c), reduce (min,max) per position e
//           -> partial[k][e][2]   (kept in the head of the uq buffer, which pass C overwrites)
//   pass B  one workgroup: reduce the K partials -> u_range[e] (one range for all e if
//           LANCE_RANGE_PER_TENSOR)
//   pass C  one workgroup per filter k: transform again, quantize, store the codes in the
//           blocked/permuted layout, reduce the code sums -> u_rowsum[e][k]
#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

constexpr int kThreads = 256;

template <int M>
__device__ __forceinline__ void load_and_transform(const float* __restrict__ w, int k, int c, int C,
                                                   float (&u)[M + 2][M + 2]) {
  float g[3][3];
  const float* src = w + ((size_t)k * C + c) * 9;
#pragma unroll
  for (int r = 0; r < 3; r++)
#pragma unroll
    for (int s = 0; s < 3; s++) g[r][s] = src[r * 3 + s];
  dev::filter_tile_transform<M>(g, u);
}

template <int M>
__global__ __launch_bounds__(kThreads) void filter_range_kernel(const float* __restrict__ w,
                                                                float* __restrict__ partial,
                                                                int C) {
  constexpr int A = M + 2, E = A * A;
  __shared__ float red[kThreads / 64][E][2];
  const int k = blockIdx.x;
  float mn[E], mx[E];
#pragma unroll
  for (int e = 0; e < E; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }
  for (int c = threadIdx.x; c < C; c += kThreads) {
    float u[A][A];
    load_and_transform<M>(w, k, c, C, u);
#pragma unroll
    for (int e = 0; e < E; e++) {
      mn[e] = fminf(mn[e], u[e / A][e % A]);
      mx[e] = fmaxf(mx[e], u[e / A][e % A]);
    }
  }
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
#pragma unroll
  for (int e = 0; e < E; e++) {
    float a = dev::wave_min(mn[e]), b = dev::wave_max(mx[e]);
    if (lane == 0) { red[wave][e][0] = a; red[wave][e][1] = b; }
  }
  __syncthreads();
  if (threadIdx.x < E) {
    float a = red[0][threadIdx.x][0], b = red[0][threadIdx.x][1];
    for (int wv = 1; wv < kThreads / 64; wv++) {
      a = fminf(a, red[wv][threadIdx.x][0]);
      b = fmaxf(b, red[wv][threadIdx.x][1]);
    }
    partial[((size_t)k * E + threadIdx.x) * 2 + 0] = a;
    partial[((size_t)k * E + threadIdx.x) * 2 + 1] = b;
  }
}

template <int M>
__global__ __launch_bounds__(kThreads) void filter_quant_kernel(
    const float* __restrict__ w, const float* __restrict__ range, int8_t* __restrict__ uq,
    int32_t* __restrict__ rowsum, int C, int K, int Cp, int CB, int NB, int Q, int bits,
    int natural, int packed) {
  constexpr int A = M + 2, E = A * A;
  __shared__ float qmn[E], qinv[E];
  __shared__ int red[kThreads / 64][E];
  const int k = blockIdx.x;
  if (threadIdx.x < E) {
    float inv, scale;
    dev::quant_params(range[threadIdx.x * 2], range[threadIdx.x * 2 + 1], bits, &inv, &scale);
    qmn[threadIdx.x] = range[threadIdx.x * 2];
    qinv[threadIdx.x] = inv;
  }
  __syncthreads();
  const float L = (float)((1 << bits) - 1);
  const int h = 1 << (bits - 1);
  int sum[E];
#pragma unroll
  for (int e = 0; e < E; e++) sum[e] = 0;
  if (packed) {
    // two codes per byte (64-channel blocks only): a thread forms the byte that holds the codes
    // at positions q and q + 32 of a block row, each as code + 8 in four bits
    for (int i = threadIdx.x; i < NB * 32; i += kThreads) {
      const int b = i / 32, q = i % 32;
      int8_t* dst = uq + ((size_t)b * K + k) * 32 + q;
      const size_t estride = (size_t)NB * K * 32;
      unsigned byte[E];
#pragma unroll
      for (int e = 0; e < E; e++) byte[e] = 0;
#pragma unroll
      for (int hi = 0; hi < 2; hi++) {
        const int pos = q + 32 * hi;
        const int r = natural ? pos : 16 * (pos % 4) + pos / 4;  // channel of the block at pos
        const int c = b * 64 + r;
        if (c < C) {
          float u[A][A];
          load_and_transform<M>(w, k, c, C, u);
#pragma unroll
          for (int e = 0; e < E; e++) {
            const int code = dev::quantize_code(u[e / A][e % A], qmn[e], qinv[e], L, h);
            byte[e] |= (unsigned)(code + 8) << (4 * hi);
            sum[e] += code;
          }
        } else {
#pragma unroll
          for (int e = 0; e < E; e++) byte[e] |= 8u << (4 * hi);
        }
      }
#pragma unroll
      for (int e = 0; e < E; e++) dst[e * estride] = (int8_t)byte[e];
    }
  } else
  for (int c = threadIdx.x; c < Cp; c += kThreads) {
    const int b = c / CB, r = c % CB;
    const int pos = natural ? r : 4 * (r % Q) + r / Q;  // byte of channel r in its block
    int8_t* dst = uq + ((size_t)b * K + k) * CB + pos;
    const size_t estride = (size_t)NB * K * CB;
    if (c < C) {
      float u[A][A];
      load_and_transform<M>(w, k, c, C, u);
#pragma unroll
      for (int e = 0; e < E; e++) {
        int q = dev::quantize_code(u[e / A][e % A], qmn[e], qinv[e], L, h);
        dst[e * estride] = (int8_t)q;
        sum[e] += q;
      }
    } else {
#pragma unroll
      for (int e = 0; e < E; e++) dst[e * estride] = 0;
    }
  }
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
#pragma unroll
  for (int e = 0; e < E; e++) {
    int v = sum[e];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    if (lane == 0) red[wave][e] = v;
  }
  __syncthreads();
  if (threadIdx.x < E) {
    int v = 0;
    for (int wv = 0; wv < kThreads / 64; wv++) v += red[wv][threadIdx.x];
    rowsum[(size_t)threadIdx.x * K + k] = v;
  }
}

}  // namespace

hipError_t launch_filter_transform(const Geo& g, const float* w, int8_t* uq, float* u_range,
                                   int32_t* u_rowsum, hipStream_t s) {
  // The K partial records (K*E*2 floats = 8*E*K bytes) fit in uq (E*K*Cp >= 16*E*K bytes);
  // pass C rewrites every byte of uq afterwards.
  float* partial = reinterpret_cast<float*>(uq);
  const int per_tensor = (g.flags & LANCE_RANGE_PER_TENSOR) ? 1 : 0;
  if (g.m == 2)
    filter_range_kernel<2><<<g.K, kThreads, 0, s>>>(w, partial, g.C);
  else
    filter_range_kernel<4><<<g.K, kThreads, 0, s>>>(w, partial, g.C);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = launch_range_finalize(partial, g.K, g.E, per_tensor, /*is_static=*/0, g.bits_w, u_range,
                            /*qparams=*/nullptr, /*dqo=*/nullptr, s);
  if (e != hipSuccess) return e;
  if (g.m == 2)
    filter_quant_kernel<2><<<g.K, kThreads, 0, s>>>(w, u_range, uq, u_rowsum, g.C, g.K, g.Cp,
                                                    g.CB, g.NB, g.Q, g.bits_w, is_nhwc(g) ? 1 : 0,
                                                    is_packed(g) ? 1 : 0);
  else
    filter_quant_kernel<4><<<g.K, kThreads, 0, s>>>(w, u_range, uq, u_rowsum, g.C, g.K, g.Cp,
                                                    g.CB, g.NB, g.Q, g.bits_w, is_nhwc(g) ? 1 : 0,
                                                    is_packed(g) ? 1 : 0);
  return hipGetLastError();
}

}  // namespace lance
