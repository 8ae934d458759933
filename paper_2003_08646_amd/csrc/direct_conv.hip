// Full-precision comparator: Eq. 1 evaluated directly in binary32 (stride 1, zero padding).
// A workgroup computes a 16x16 output patch of one image for 32 filters; the input window and
// the filter slab of 8 channels at a time are staged in LDS.  Each lane owns one output pixel
// and 32 filter accumulators.
#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

constexpr int kTile = 16, kKB = 32, kCC = 8;

__global__ __launch_bounds__(kTile* kTile) void direct_conv_kernel(
    const float* __restrict__ x, const float* __restrict__ w, float* __restrict__ y, int N, int C,
    int H, int W, int K, int pad, int Ho, int Wo, int tiles_x, int nhwc) {
  __shared__ float xs[kCC][kTile + 2][kTile + 3];
  __shared__ float ws[kCC][9][kKB];
  const int tid = threadIdx.x;
  const int lx = tid % kTile, ly = tid / kTile;
  const int bx = blockIdx.x % tiles_x, by = blockIdx.x / tiles_x;
  const int k0 = blockIdx.y * kKB, n = blockIdx.z;
  const int oy0 = by * kTile, ox0 = bx * kTile;
  float acc[kKB];
#pragma unroll
  for (int k = 0; k < kKB; k++) acc[k] = 0.0f;
  for (int c0 = 0; c0 < C; c0 += kCC) {
    __syncthreads();
    for (int i = tid; i < kCC * (kTile + 2) * (kTile + 2); i += kTile * kTile) {
      const int cc = i / ((kTile + 2) * (kTile + 2)), rem = i % ((kTile + 2) * (kTile + 2));
      const int r = rem / (kTile + 2), s = rem % (kTile + 2);
      const int gy = oy0 + r - pad, gx = ox0 + s - pad, c = c0 + cc;
      float v = 0.0f;
      if (c < C && gy >= 0 && gy < H && gx >= 0 && gx < W)
        v = x[dev::act_index(nhwc, n, c, gy, gx, C, H, W)];
      xs[cc][r][s] = v;
    }
    for (int i = tid; i < kCC * 9 * kKB; i += kTile * kTile) {
      const int kk = i % kKB, rem = i / kKB;
      const int t = rem % 9, cc = rem / 9;
      const int k = k0 + kk, c = c0 + cc;
      ws[cc][t][kk] = (k < K && c < C) ? w[((size_t)k * C + c) * 9 + t] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int cc = 0; cc < kCC; cc++) {
      float d[9];
#pragma unroll
      for (int r = 0; r < 3; r++)
#pragma unroll
        for (int s = 0; s < 3; s++) d[r * 3 + s] = xs[cc][ly + r][lx + s];
#pragma unroll
      for (int t = 0; t < 9; t++)
#pragma unroll
        for (int k = 0; k < kKB; k++) acc[k] = __builtin_fmaf(d[t], ws[cc][t][k], acc[k]);
    }
  }
  const int oy = oy0 + ly, ox = ox0 + lx;
  if (oy < Ho && ox < Wo) {
#pragma unroll
    for (int k = 0; k < kKB; k++)
      if (k0 + k < K) y[dev::act_index(nhwc, n, k0 + k, oy, ox, K, Ho, Wo)] = acc[k];
  }
}

}  // namespace

hipError_t launch_direct_conv(const Geo& g, const float* x, const float* w, float* y,
                              hipStream_t s) {
  const int tiles_x = (g.Wo + kTile - 1) / kTile, tiles_y = (g.Ho + kTile - 1) / kTile;
  dim3 grid(tiles_x * tiles_y, (g.K + kKB - 1) / kKB, g.N);
  if (g.N > 65535 || (g.K + kKB - 1) / kKB > 65535) return hipErrorInvalidValue;
  direct_conv_kernel<<<grid, kTile * kTile, 0, s>>>(x, w, y, g.N, g.C, g.H, g.W, g.K, g.pad, g.Ho,
                                                    g.Wo, tiles_x, is_nhwc(g) ? 1 : 0);
  return hipGetLastError();
}

}  // namespace lance
