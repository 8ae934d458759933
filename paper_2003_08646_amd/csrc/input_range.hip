// Stage 2, first pass: the (min,max) of every Winograd-domain position of V = B^T d B over the
// whole input (the T of Eq. 7 for the input operand).  A pure reduction: X is read once, nothing
// but one partial record per workgroup is written.
//
// No LDS staging here: a lane owns one tile and walks over a chunk of channels, loading the
// tile's (m+2) rows straight from the image (rows of adjacent tiles overlap, the overlap is
// served by the vector cache).  Lanes run along the tile row, so a wave's loads cover
// contiguous image rows.  The small per-lane state (one patch, 2*E running extrema) lets many
// waves stay resident, which is what hides the load latency.
#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

constexpr int kThreads = 256;

struct RArgs {
  const float* x;
  float* partial;   // [gridDim.x][E][2]
  int32_t* colsum;  // cleared here when the code tensor has several channel blocks
  int N, C, H, W, pad, th, tw, P;
  int CC;           // channels per workgroup
  int cchunks;      // ceil(C / CC)
  int TT;           // tiles per workgroup
  int tchunks;      // ceil(th*tw / TT)
  int units;        // N * cchunks * tchunks work units, taken round robin by the workgroups
  int zero_colsum;
};

// m floats that need only 4-byte alignment (the hardware allows unaligned multi-dword loads)
template <int NV> struct __attribute__((packed, aligned(4))) fvec { float v[NV]; };

// min over the 64 lanes of a wave, result in lane 63 (DPP only, no LDS)
template <bool IS_MAX>
__device__ __forceinline__ float wave_reduce_to_lane63(float v) {
  auto comb = [](float a, float b) { return IS_MAX ? fmaxf(a, b) : fminf(a, b); };
  auto dpp = [](float x, int ctrl_sel) {
    const int i = __float_as_int(x);
    int r;
    switch (ctrl_sel) {
      case 0: r = __builtin_amdgcn_update_dpp(i, i, 0xB1, 0xF, 0xF, false); break;   // xor 1
      case 1: r = __builtin_amdgcn_update_dpp(i, i, 0x4E, 0xF, 0xF, false); break;   // xor 2
      case 2: r = __builtin_amdgcn_update_dpp(i, i, 0x141, 0xF, 0xF, false); break;  // half mirror
      case 3: r = __builtin_amdgcn_update_dpp(i, i, 0x140, 0xF, 0xF, false); break;  // mirror
      case 4: r = __builtin_amdgcn_update_dpp(i, i, 0x142, 0xA, 0xF, false); break;  // row_bcast:15
      default: r = __builtin_amdgcn_update_dpp(i, i, 0x143, 0xC, 0xF, false); break; // row_bcast:31
    }
    return __int_as_float(r);
  };
#pragma unroll
  for (int s = 0; s < 6; s++) v = comb(v, dpp(v, s));
  return v;
}

template <int M>
__global__ __launch_bounds__(kThreads) void input_range_kernel(const RArgs a) {
  constexpr int A = M + 2, E = A * A;
  __shared__ float red[kThreads / 64][E][2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tiles = a.th * a.tw;
  const size_t HW = (size_t)a.H * a.W;

  float mn[E], mx[E];
#pragma unroll
  for (int e = 0; e < E; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }

  for (int unit = blockIdx.x; unit < a.units; unit += gridDim.x) {
    int b = unit;
    const int tchunk = b % a.tchunks; b /= a.tchunks;
    const int cchunk = b % a.cchunks;
    const int n = b / a.cchunks;
    const int c0 = cchunk * a.CC, c1 = min(a.C, c0 + a.CC);
    const int t_end = min(tiles, (tchunk + 1) * a.TT);
    for (int t = tchunk * a.TT + tid; t < t_end; t += kThreads) {
      const int ty = t / a.tw, tx = t - ty * a.tw;
      const int y0 = ty * M - a.pad, x0 = tx * M - a.pad;
      const bool interior = y0 >= 0 && y0 + A <= a.H && x0 >= 0 && x0 + A <= a.W;
      if (a.zero_colsum && cchunk == 0) {
        const unsigned p = (unsigned)((n * a.th + ty) * a.tw + tx);
#pragma unroll
        for (int e = 0; e < E; e++) a.colsum[p + (unsigned)e * a.P] = 0;
      }
      const float* img = a.x + ((size_t)n * a.C + c0) * HW;
      for (int c = c0; c < c1; c++, img += HW) {
        float d[A][A];
        if (interior) {
          const float* src = img + (size_t)y0 * a.W + x0;
#pragma unroll
          for (int r = 0; r < A; r++) {
            const fvec<A> row = *reinterpret_cast<const fvec<A>*>(src + (size_t)r * a.W);
#pragma unroll
            for (int s = 0; s < A; s++) d[r][s] = row.v[s];
          }
        } else {
#pragma unroll
          for (int r = 0; r < A; r++)
#pragma unroll
            for (int s = 0; s < A; s++) {
              const int gy = y0 + r, gx = x0 + s;
              d[r][s] =
                  (gy >= 0 && gy < a.H && gx >= 0 && gx < a.W) ? img[(size_t)gy * a.W + gx] : 0.0f;
            }
        }
        dev::input_tile_transform<M>(d);
#pragma unroll
        for (int e = 0; e < E; e++) {
          mn[e] = fminf(mn[e], d[e / A][e % A]);
          mx[e] = fmaxf(mx[e], d[e / A][e % A]);
        }
      }
    }
  }

#pragma unroll
  for (int e = 0; e < E; e++) {
    const float lo = wave_reduce_to_lane63<false>(mn[e]);
    const float hi = wave_reduce_to_lane63<true>(mx[e]);
    if (lane == 63) { red[wave][e][0] = lo; red[wave][e][1] = hi; }
  }
  __syncthreads();
  if (tid < E) {
    float lo = red[0][tid][0], hi = red[0][tid][1];
    for (int wv = 1; wv < kThreads / 64; wv++) {
      lo = fminf(lo, red[wv][tid][0]);
      hi = fmaxf(hi, red[wv][tid][1]);
    }
    a.partial[((size_t)blockIdx.x * E + tid) * 2 + 0] = lo;
    a.partial[((size_t)blockIdx.x * E + tid) * 2 + 1] = hi;
  }
}

}  // namespace

hipError_t launch_input_range(const Geo& g, const float* x, float* partial, int32_t* colsum,
                              int zero_colsum, int* groups_out, hipStream_t s) {
  RArgs a{};
  a.x = x; a.partial = partial; a.colsum = colsum;
  a.N = g.N; a.C = g.C; a.H = g.H; a.W = g.W; a.pad = g.pad; a.th = g.th; a.tw = g.tw; a.P = g.P;
  a.zero_colsum = zero_colsum;
  const long long tiles = (long long)g.th * g.tw;
  // A work unit is TT tiles x CC channels of one image.  Aim at about kMaxRangeGroups units
  // (one partial record per workgroup is reduced afterwards) with at least one tile per lane;
  // if there are still more units, the workgroups take several each.
  long long TT = tiles < kThreads ? tiles : kThreads;
  long long CC = 1;
  auto units = [&]() {
    return (long long)g.N * ((g.C + CC - 1) / CC) * ((tiles + TT - 1) / TT);
  };
  while (units() > kMaxRangeGroups && CC < g.C) CC *= 2;
  while (units() > kMaxRangeGroups && TT < tiles) TT *= 2;
  if (units() > (1LL << 30)) return hipErrorInvalidValue;
  a.CC = (int)CC; a.cchunks = (int)((g.C + CC - 1) / CC);
  a.TT = (int)TT; a.tchunks = (int)((tiles + TT - 1) / TT);
  a.units = (int)units();
  const int grid = a.units < kMaxRangeGroups ? a.units : kMaxRangeGroups;
  *groups_out = grid;
  if (g.m == 2)
    input_range_kernel<2><<<grid, kThreads, 0, s>>>(a);
  else
    input_range_kernel<4><<<grid, kThreads, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace lance
