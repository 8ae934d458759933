// Small helper kernels: reduction of partial ranges, Eq. 7 / Eq. 8 parameter tables, zero fill.
#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

constexpr int kThreads = 256;

// Reduce `count` partial (min,max) records of E positions each into range[E][2]; optionally
// emit the quantizer parameters {min, inv} of Eq. 7 per position.
__global__ __launch_bounds__(kThreads) void range_finalize_kernel(
    const float* __restrict__ partial, int count, int E, int per_tensor, int is_static, int bits,
    float* __restrict__ range, float* __restrict__ qparams) {
  __shared__ float red[kThreads / 64][2];
  __shared__ float res[36][2];
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  if (is_static) {
    if (threadIdx.x < E) {
      res[threadIdx.x][0] = range[threadIdx.x * 2];
      res[threadIdx.x][1] = range[threadIdx.x * 2 + 1];
    }
    __syncthreads();
  } else {
    for (int e = 0; e < E; e++) {
      float a = INFINITY, b = -INFINITY;
      for (int i = threadIdx.x; i < count; i += kThreads) {
        a = fminf(a, partial[((size_t)i * E + e) * 2 + 0]);
        b = fmaxf(b, partial[((size_t)i * E + e) * 2 + 1]);
      }
      a = dev::wave_min(a);
      b = dev::wave_max(b);
      if (lane == 0) { red[wave][0] = a; red[wave][1] = b; }
      __syncthreads();
      if (threadIdx.x == 0) {
        for (int wv = 1; wv < kThreads / 64; wv++) {
          a = fminf(a, red[wv][0]);
          b = fmaxf(b, red[wv][1]);
        }
        res[e][0] = a;
        res[e][1] = b;
      }
      __syncthreads();
    }
  }
  if (threadIdx.x < E) {
    float a = res[threadIdx.x][0], b = res[threadIdx.x][1];
    if (per_tensor && !is_static) {
      for (int e = 0; e < E; e++) { a = fminf(a, res[e][0]); b = fmaxf(b, res[e][1]); }
    }
    if (!is_static) {
      range[threadIdx.x * 2 + 0] = a;
      range[threadIdx.x * 2 + 1] = b;
    }
    if (qparams) {
      float inv, scale;
      dev::quant_params(a, b, bits, &inv, &scale);
      qparams[threadIdx.x * 2 + 0] = a;
      qparams[threadIdx.x * 2 + 1] = inv;
    }
  }
}

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(int32_t* __restrict__ p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n;
       i += (size_t)gridDim.x * kThreads)
    p[i] = 0;
}

// Per-position constants of the expanded Eq. 8 (formed in binary64, stored as binary32):
//   dq[e] = { su*sv, sv*ou }          rk[e][k] = su*ov*rowsum[e][k] + C*ou*ov
// so that M[e,k,p] = dq[e][0]*ACC + rk[e][k] + dq[e][1]*colsum[e][p].
__global__ __launch_bounds__(kThreads) void dq_prepare_kernel(
    const float* __restrict__ u_range, const int32_t* __restrict__ u_rowsum,
    const float* __restrict__ v_range, float* __restrict__ dq, float* __restrict__ rk, int K, int C,
    int bits) {
  const int e = blockIdx.x;
  float iu, su, iv, sv;
  dev::quant_params(u_range[2 * e], u_range[2 * e + 1], bits, &iu, &su);
  dev::quant_params(v_range[2 * e], v_range[2 * e + 1], bits, &iv, &sv);
  const double h = (double)(1 << (bits - 1));
  const double ou = (double)u_range[2 * e] + (double)su * h;
  const double ov = (double)v_range[2 * e] + (double)sv * h;
  if (threadIdx.x == 0) {
    dq[4 * e + 0] = (float)((double)su * (double)sv);
    dq[4 * e + 1] = (float)((double)sv * ou);
    dq[4 * e + 2] = 0.0f;
    dq[4 * e + 3] = 0.0f;
  }
  const double kconst = (double)C * ou * ov, rmul = (double)su * ov;
  for (int k = threadIdx.x; k < K; k += kThreads)
    rk[(size_t)e * K + k] = (float)(rmul * (double)u_rowsum[(size_t)e * K + k] + kconst);
}

}  // namespace

hipError_t launch_range_finalize(const float* partial, int count, int E, int per_tensor,
                                 int is_static, int bits, float* range, float* qparams,
                                 hipStream_t s) {
  range_finalize_kernel<<<1, kThreads, 0, s>>>(partial, count, E, per_tensor, is_static, bits,
                                               range, qparams);
  return hipGetLastError();
}

hipError_t launch_fill_zero(int32_t* p, size_t n, hipStream_t s) {
  size_t blocks = (n + kThreads - 1) / kThreads;
  if (blocks > 4096) blocks = 4096;
  if (blocks == 0) return hipSuccess;
  fill_zero_kernel<<<(unsigned)blocks, kThreads, 0, s>>>(p, n);
  return hipGetLastError();
}

hipError_t launch_dq_prepare(const Geo& g, const float* u_range, const int32_t* u_rowsum,
                             const float* v_range, float* dq, float* rk, hipStream_t s) {
  dq_prepare_kernel<<<g.E, kThreads, 0, s>>>(u_range, u_rowsum, v_range, dq, rk, g.K, g.C,
                                             g.bits);
  return hipGetLastError();
}

}  // namespace lance
