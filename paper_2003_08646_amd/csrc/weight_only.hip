// Weight-only quantization (Sec. 4, the 4-32 row of Table 2): filters quantized in the Winograd
// domain (Eq. 7, prepared by the filter transform), inputs transformed but not quantized:
//   M[e,k,p] = sum_c Q'(u^[e,k,c]) * (B^T d_{p,c} B)[e],   S = A^T M A          (Eq. 8, Eq. 9)
// The channel sum is a binary32 product in the Winograd domain, not this library's integer one,
// so the matrix-core kernels do not apply; this is a plain vector-ALU kernel.
//
// Lane = tile, a workgroup takes 256 tiles and kF filters.  Per channel every lane transforms
// its own patch; kF*E threads de-quantize the workgroup's filter codes of that channel into LDS
// (u~ = code * scale_e + min_e with the unsigned code of Eq. 7); E multiply-adds per filter and
// lane follow.  The patch transform is repeated per filter block (K / kF times).
#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

constexpr int kThreads = 256;

struct WoArgs {
  const float* x;
  const int8_t* uq;       // [E][NB][K][CB], layout of lance.h
  const float* u_range;   // [E][2]
  float* y;
  int N, C, H, W, K, pad, th, tw, P, Ho, Wo, bits_w, nhwc, CB, NB;
};

template <int M, int kF>
__global__ __launch_bounds__(kThreads) void weight_only_kernel(const WoArgs a) {
  constexpr int A = M + 2, E = A * A;
  static_assert(kF * E <= kThreads, "one thread per (filter, position)");
  __shared__ float us[kF][E];
  __shared__ float mn_s[E], sc_s[E];
  const int tid = threadIdx.x;
  const int p = blockIdx.x * kThreads + tid;
  const int k0 = blockIdx.y * kF;
  const bool valid = p < a.P;
  const int pt = min(p, a.P - 1);
  const int tx = pt % a.tw, t2 = pt / a.tw;
  const int ty = t2 % a.th, n = t2 / a.th;
  const int y0 = ty * M - a.pad, x0 = tx * M - a.pad;
  if (tid < E) {
    float inv, scale;
    dev::quant_params(a.u_range[2 * tid], a.u_range[2 * tid + 1], a.bits_w, &inv, &scale);
    mn_s[tid] = a.u_range[2 * tid];
    sc_s[tid] = scale;
  }
  float acc[kF][E];
#pragma unroll
  for (int f = 0; f < kF; f++)
#pragma unroll
    for (int e = 0; e < E; e++) acc[f][e] = 0.0f;
  const int h = 1 << (a.bits_w - 1);
  const int fe_f = tid / E, fe_e = tid % E;   // this thread's (filter, position) of the block
  const int kq = min(k0 + fe_f, a.K - 1);
  const int Q = a.CB / 4;

  for (int c = 0; c < a.C; c++) {
    __syncthreads();  // the previous channel's filter values have been read (and mn_s, sc_s set)
    if (tid < kF * E) {
      const int b = c / a.CB, r = c % a.CB;
      const int pos = a.nhwc ? r : 4 * (r % Q) + r / Q;
      const int code = (int)a.uq[(((size_t)fe_e * a.NB + b) * a.K + kq) * a.CB + pos] + h;
      us[fe_f][fe_e] = (float)code * sc_s[fe_e] + mn_s[fe_e];
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
    __syncthreads();
#pragma unroll
    for (int f = 0; f < kF; f++)
#pragma unroll
      for (int e = 0; e < E; e++) acc[f][e] = __builtin_fmaf(us[f][e], d[e / A][e % A], acc[f][e]);
  }

  if (!valid) return;
#pragma unroll
  for (int f = 0; f < kF; f++) {
    const int k = k0 + f;
    if (k >= a.K) break;
    float t[M][A];  // S = A^T M A: rows first, then columns
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

hipError_t launch_weight_only(const Geo& g, const float* x, const int8_t* uq, const float* u_range,
                              float* y, hipStream_t s) {
  const WoArgs a{x, uq, u_range, y, g.N, g.C, g.H, g.W, g.K, g.pad, g.th, g.tw, g.P, g.Ho, g.Wo,
                 g.bits_w, is_nhwc(g) ? 1 : 0, g.CB, g.NB};
  const int kf = g.m == 2 ? 8 : 4;
  const long long bx = ((long long)g.P + kThreads - 1) / kThreads, by = (g.K + kf - 1) / kf;
  if (bx > 0x7FFFFFFFLL || by > 65535) return hipErrorInvalidValue;
  dim3 grid((unsigned)bx, (unsigned)by, 1);
  if (g.m == 2) weight_only_kernel<2, 8><<<grid, kThreads, 0, s>>>(a);
  else weight_only_kernel<4, 4><<<grid, kThreads, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace lance
