// Small helper kernels: reduction of partial ranges, Eq. 7 / Eq. 8 parameter tables, zero fill.
#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

constexpr int kThreads = 256;

constexpr int kFinThreads = 1024;

// One workgroup.  (1) Reduce `count` partial (min,max) records of E positions each into
// range[E][2] (skipped when is_static: the caller's ranges are used as they are).
// (2) Optionally emit the quantizer parameters {min, inv} of Eq. 7 per position.
// (3) Optionally (u_range != nullptr) emit the constants of the expanded Eq. 8, formed in
//     binary64 and stored as binary32.  With ou = min_u + su*h, ov = min_v + sv*h:
//       M[e,k,p] = su*sv*ACC + (su*ov*rowsum[e][k] + C*ou*ov) + sv*ou*colsum[e][p]
//     and the output transform S = A^T M A is linear, so the middle term is folded through it
//     here:  dq[e] = { su*sv, sv*ou, 0, 0 },
//            rk[(a*m+b)][k] = sum_e A^T[a][i] A^T[b][j] (su*ov*rowsum[e][k] + C*ou*ov).
//
// The kernel is a chain of dependent steps run by one workgroup, so everything that does not
// depend on the reduced ranges (filter-side parameters, the row sums of the first round of rk
// outputs, the A^T table) is requested or computed before the reduction, under the latency of
// the partial-record loads.
__global__ __launch_bounds__(kFinThreads) void range_finalize_kernel(
    const float* __restrict__ partial, int count, int E, int per_tensor, int is_static, int bits,
    float* __restrict__ range, float* __restrict__ qparams, const float* __restrict__ u_range,
    const int32_t* __restrict__ u_rowsum, float* __restrict__ dq, float* __restrict__ rk,
    double* __restrict__ dqd, int K, int C, int want_rk, int bits_u, int bias) {
  __shared__ float red[kFinThreads];
  __shared__ float res[72];
  __shared__ float at_s[24];
  __shared__ double rmul[36], kconst[36];
  const int tid = threadIdx.x;
  const int cols = 2 * E;            // column = (position, min|max); odd columns are maxima
  const int groups = kFinThreads / cols;
  const int m = E == 16 ? 2 : 4, A = m + 2;
  constexpr int kBatch = 32, kParts = 4, kTerms = 9;  // kParts * kTerms >= 36 positions

  // rk outputs are spread over quads of lanes: lane part handles e = part, part + 4, ...
  const int part = tid & (kParts - 1);
  const int nout = (u_range && want_rk) ? m * m * K : 0;
  const int idx0 = tid / kParts;
  int32_t rs[kTerms];
  float su = 0.0f;
  double ou = 0.0;
  if (u_range) {
    if (tid < m * A) at_s[tid] = dev::at_coef(m, tid / A, tid % A);
    if (idx0 < nout) {
      const int k = idx0 % K;
#pragma unroll
      for (int u = 0; u < kTerms; u++) {
        const int e = part + kParts * u;
        rs[u] = e < E ? u_rowsum[(size_t)e * K + k] : 0;
      }
    }
  }

  if (is_static) {
    if (tid < cols) res[tid] = range[tid];
  } else {
    const int col = tid % cols, grp = tid / cols;
    const bool is_max = col & 1;
    float v = is_max ? -INFINITY : INFINITY;
    if (grp < groups) {
      // all loads of a batch are issued before the first is used: one memory round trip per
      // kBatch records
      for (int row0 = grp; row0 < count; row0 += kBatch * groups) {
        float x[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; u++) {
          const int row = row0 + u * groups;
          x[u] = row < count ? partial[(size_t)row * cols + col] : v;
        }
#pragma unroll
        for (int u = 0; u < kBatch; u++) v = is_max ? fmaxf(v, x[u]) : fminf(v, x[u]);
      }
    }
    red[tid] = v;
  }
  if (u_range && tid < E) {  // filter-side parameters: independent of the reduction
    float iu;
    dev::quant_params(u_range[2 * tid], u_range[2 * tid + 1], bits_u, &iu, &su);
    ou = (double)u_range[2 * tid] + (double)su * (double)(1 << (bits_u - 1));
  }
  __syncthreads();
  if (!is_static && tid < cols) {
    const bool is_max = tid & 1;
    float v = red[tid];
    for (int g2 = 1; g2 < groups; g2++) {
      const float x = red[g2 * cols + tid];
      v = is_max ? fmaxf(v, x) : fminf(v, x);
    }
    res[tid] = v;
  }
  __syncthreads();
  if (tid < E) {
    float a = res[2 * tid], b = res[2 * tid + 1];
    if (per_tensor && !is_static) {
      for (int e = 0; e < E; e++) { a = fminf(a, res[2 * e]); b = fmaxf(b, res[2 * e + 1]); }
    }
    if (!is_static) {
      range[tid * 2 + 0] = a;
      range[tid * 2 + 1] = b;
    }
    float inv, sv;
    dev::quant_params(a, b, bits, &inv, &sv);
    if (qparams) {
      qparams[tid * 2 + 0] = a;
      qparams[tid * 2 + 1] = inv;
    }
    if (u_range) {
      const double h = (double)(1 << (bits - 1));
      const double ov = (double)a + (double)sv * h;
      // (bias: the product kernel multiplies code + bias; see DqOut)
      const double sb = (double)bias * ((double)su * (double)sv);
      dq[4 * tid + 0] = (float)((double)su * (double)sv);
      dq[4 * tid + 1] = (float)((double)sv * ou - sb);
      dq[4 * tid + 2] = 0.0f;
      dq[4 * tid + 3] = 0.0f;
      rmul[tid] = (double)su * ov - sb;
      kconst[tid] = (double)C * ou * ov;
      dqd[2 * tid + 0] = rmul[tid];
      dqd[2 * tid + 1] = kconst[tid];
    }
  }
  if (nout > 0) {
    __syncthreads();
    constexpr int kStride = kFinThreads / kParts;
    // idx is the same in the four lanes of a quad, so the quad shuffles below are convergent
    for (int idx = idx0; idx < nout; idx += kStride) {
      const int k = idx % K, ab = idx / K;
      const int a = ab / m, b = ab % m;
      double acc = 0.0;
#pragma unroll
      for (int u = 0; u < kTerms; u++) {
        const int e = part + kParts * u;
        if (e < E) {
          const int32_t r = idx == idx0 ? rs[u] : u_rowsum[(size_t)e * K + k];
          const double coef = (double)at_s[a * A + e / A] * (double)at_s[b * A + e % A];
          acc += coef * (rmul[e] * (double)r + kconst[e]);
        }
      }
      acc += __shfl_xor(acc, 1, 64);
      acc += __shfl_xor(acc, 2, 64);
      if (part == 0) rk[idx] = (float)acc;
    }
  }
}

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(int32_t* __restrict__ p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n;
       i += (size_t)gridDim.x * kThreads)
    p[i] = 0;
}

}  // namespace

hipError_t launch_range_finalize(const float* partial, int count, int E, int per_tensor,
                                 int is_static, int bits, float* range, float* qparams,
                                 const DqOut* dqo, hipStream_t s) {
  note_kernel("range_finalize_kernel");
  range_finalize_kernel<<<1, kFinThreads, 0, s>>>(
      partial, count, E, per_tensor, is_static, bits, range, qparams,
      dqo ? dqo->u_range : nullptr, dqo ? dqo->u_rowsum : nullptr, dqo ? dqo->dq : nullptr,
      dqo ? dqo->rk : nullptr, dqo ? dqo->dqd : nullptr, dqo ? dqo->K : 0, dqo ? dqo->C : 0,
      dqo ? dqo->want_rk : 0, dqo ? dqo->bits_w : bits, dqo ? dqo->bias : 0);
  return hipGetLastError();
}

hipError_t launch_fill_zero(int32_t* p, size_t n, hipStream_t s) {
  size_t blocks = (n + kThreads - 1) / kThreads;
  if (blocks > 4096) blocks = 4096;
  if (blocks == 0) return hipSuccess;
  fill_zero_kernel<<<(unsigned)blocks, kThreads, 0, s>>>(p, n);
  return hipGetLastError();
}

}  // namespace lance
