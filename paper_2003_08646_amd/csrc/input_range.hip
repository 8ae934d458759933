// Stage 2, first pass: the (min,max) of every Winograd-domain position of V = B^T d B over the
// whole input (the T of Eq. 7 for the input operand).  A pure reduction: X is read once, nothing
// but one partial record per workgroup is written.
//
// No LDS staging: a lane owns one tile of a block of 64 consecutive tiles and walks over
// channels, reading the tile's patch with buffer loads through per-lane offsets that are computed
// once per block (patch_loader.h: zero padding by buffer range checking, no vector address
// arithmetic in the channel walk).  Lanes run along the tile row, so a wave's loads cover
// contiguous image rows; the overlap of adjacent patches is served by the vector cache.  The four waves of a workgroup take the channels of the block round
// robin, loading two channels ahead of the one they transform.
#include "lance_device.h"
#include "lance_internal.h"
#include "patch_loader.h"

namespace lance {
namespace {

constexpr int kThreads = 512;  // two groups of four waves; each group takes a work unit

struct RArgs {
  const float* x;
  float* partial;   // [gridDim.x][E][2]
  int32_t* colsum;  // cleared here when the code tensor has several channel blocks
  int N, C, H, W, pad, th, tw, P;
  int T;            // tiles per image
  int bpi;          // 0: blocks are 64 consecutive tiles of the whole batch; else blocks per image
  int TB;           // tile blocks
  int CC, cchunks;  // channels per work unit, units per tile block
  int units;        // TB * cchunks, taken round robin by the workgroups
  unsigned reach;   // extent of the buffer descriptors (see tile_block_reach)
  int zero_colsum;
};

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


// Work unit = (block of 64 tiles, chunk of CC channels).
// MODE: patch load mode (patch_load_mode): 0 pixel by pixel, 1 by rows, 2 by rows with only
// edge columns ever outside the image.
template <int M, int MODE>
__global__ __launch_bounds__(kThreads, (M == 2 && MODE != 1 ? 4 : 2)) void input_range_kernel(const RArgs a) {
  constexpr int A = M + 2, E = A * A;
  constexpr int kStep = M == 2 ? 2 : 1;  // channels transformed together (min3/max3 for pairs)
  constexpr int kBuf = M == 2 ? 4 : 2;   // patch buffers
  constexpr int kAhead = M == 2 ? 2 : 1; // channels in flight ahead of the transform
  __shared__ float red[kThreads / 64][E][2];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave = wave8 & 3, grp = wave8 >> 2;  // wave inside its group of four; the group
  const unsigned HW = (unsigned)a.H * (unsigned)a.W;

  if (a.zero_colsum) {
    const size_t n = (size_t)E * a.P;
    for (size_t i = (size_t)blockIdx.x * kThreads + tid; i < n; i += (size_t)gridDim.x * kThreads)
      a.colsum[i] = 0;
  }

  float mn[E], mx[E];
#pragma unroll
  for (int e = 0; e < E; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }

  // A workgroup takes pairs of consecutive units, one per wave group: one partial record per
  // PAIR of units keeps the record count (which every consumer reads in full) down.
  const int pairs = (a.units + 1) / 2;
  for (int pr = blockIdx.x; pr < pairs; pr += gridDim.x) {
    // units of one channel chunk are consecutive; within the grid's first round the pairs are
    // dealt so that each die works on a contiguous range of tile blocks
    const int pr2 = pr < (int)gridDim.x ? dev::xcd_contiguous(pr, min((int)gridDim.x, pairs)) : pr;
    const int u2 = 2 * pr2 + grp;
    if (u2 >= a.units) continue;
    const int cc = u2 / a.TB, tb = u2 - cc * a.TB;
    // this lane's tile (lanes past the end repeat the last tile: harmless for min/max)
    int p, n0;
    if (a.bpi == 0) {
      p = min(tb * 64 + lane, a.P - 1);
      n0 = (tb * 64) / a.T;
    } else {
      n0 = tb / a.bpi;
      p = n0 * a.T + min((tb - n0 * a.bpi) * 64 + lane, a.T - 1);
    }
    const int n = p / a.T, t = p - n * a.T;
    const int ty = t / a.tw, tx = t - ty * a.tw;
    dev::PatchLoader<M> pl;
    pl.setup((unsigned)(n - n0) * (unsigned)a.C * HW, n0, n, a.N, ty, tx, a.pad, a.H, a.W);
    // channels of this wave: c0 + wave + 4 i, i < cnt
    const int c0 = cc * a.CC, cend = min(c0 + a.CC, a.C);
    const int cnt = (cend - c0 - wave + 3) >> 2;
    if (cnt <= 0) continue;
    const char* xb = reinterpret_cast<const char*>(a.x + (size_t)n0 * a.C * HW);
    auto chan = [&](int i) { return c0 + wave + 4 * i; };
    auto accumulate = [&](const float (&d)[A][A]) {
#pragma unroll
      for (int e = 0; e < E; e++) {
        mn[e] = fminf(mn[e], d[e / A][e % A]);
        mx[e] = fmaxf(mx[e], d[e / A][e % A]);
      }
    };
    // A wave loads patches by rows, except from the first and the last plane of the tensor
    // (patch_loader.h).  Those can only be the wave's first and last channel; they are taken
    // out of the pipelined walk and done on their own, pixel by pixel.
    int i_lo = 0, i_hi = cnt;
    if constexpr (MODE != 0) {
      const bool first_edge = pl.first_image && chan(0) == 0;
      const bool last_edge = pl.last_image && chan(cnt - 1) == a.C - 1;
      if (first_edge || last_edge) {
        float b[E], d[A][A];
        if (first_edge) {
          pl.template issue<false>(xb + (size_t)chan(0) * HW * 4, a.reach, b);
#pragma unroll
          for (int r = 0; r < A; r++)
#pragma unroll
            for (int c = 0; c < A; c++) d[r][c] = b[r * A + c];
          dev::input_tile_transform<M>(d);
          accumulate(d);
          i_lo = 1;
        }
        if (last_edge && cnt - 1 >= i_lo) {
          pl.template issue<false>(xb + (size_t)chan(cnt - 1) * HW * 4, a.reach, b);
#pragma unroll
          for (int r = 0; r < A; r++)
#pragma unroll
            for (int c = 0; c < A; c++) d[r][c] = b[r * A + c];
          dev::input_tile_transform<M>(d);
          accumulate(d);
          i_hi = cnt - 1;
        }
      }
    }
    if (i_hi <= i_lo) continue;
    // channel of step i of the walk; past the end the last one again (duplicates do not change
    // min/max)
    auto wchan = [&](int i) { return c0 + wave + 4 * min(i_lo + i, i_hi - 1); };
    const int steps = i_hi - i_lo;
    auto walk = [&](auto by_rows_t) {
      constexpr bool BY_ROWS = decltype(by_rows_t)::value;
      float buf[kBuf][E];
      auto issue = [&](int i, float (&b)[E]) {
        pl.template issue<BY_ROWS>(xb + (size_t)wchan(i) * HW * 4, a.reach, b);
      };
#pragma unroll
      for (int u = 0; u < kAhead; u++) issue(u, buf[u]);
      for (int i0 = 0; i0 < steps; i0 += kBuf) {
#pragma unroll
        for (int u = 0; u < kBuf; u += kStep) {
#pragma unroll
          for (int s2 = 0; s2 < kStep; s2++)
            issue(i0 + u + s2 + kAhead, buf[(u + s2 + kAhead) % kBuf]);
          float d[kStep][A][A];
#pragma unroll
          for (int s2 = 0; s2 < kStep; s2++) {
#pragma unroll
            for (int r = 0; r < A; r++)
#pragma unroll
              for (int c = 0; c < A; c++) d[s2][r][c] = buf[(u + s2) % kBuf][r * A + c];
            if constexpr (BY_ROWS) pl.template fix<MODE == 2>(d[s2]);
            dev::input_tile_transform<M>(d[s2]);
          }
#pragma unroll
          for (int e = 0; e < E; e++) {
            if constexpr (kStep == 2) {
              mn[e] = fminf(mn[e], fminf(d[0][e / A][e % A], d[1][e / A][e % A]));
              mx[e] = fmaxf(mx[e], fmaxf(d[0][e / A][e % A], d[1][e / A][e % A]));
            } else {
              mn[e] = fminf(mn[e], d[0][e / A][e % A]);
              mx[e] = fmaxf(mx[e], d[0][e / A][e % A]);
            }
          }
        }
      }
    };
    walk(std::integral_constant<bool, MODE != 0>{});
  }

  // wave reduction: the first NP positions by the scattering butterfly (lane group g ends up
  // with position g), the rest (m = 4 only: positions 32..35) one by one
  constexpr int NP = E >= 32 ? 32 : 16;
  {
    float lo, hi;
    dev::wave_minmax_scatter<NP>(mn, mx, lane, &lo, &hi);
    constexpr int per = 64 / NP;
    if (lane % per == 0) { red[wave8][lane / per][0] = lo; red[wave8][lane / per][1] = hi; }
  }
#pragma unroll
  for (int e = NP; e < E; e++) {
    const float lo = wave_reduce_to_lane63<false>(mn[e]);
    const float hi = wave_reduce_to_lane63<true>(mx[e]);
    if (lane == 63) { red[wave8][e][0] = lo; red[wave8][e][1] = hi; }
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

// Blocks of 64 tiles for kernels that address a block's pixels by 32-bit offsets from the
// (first image of the block, channel) plane: consecutive tiles of the whole batch when all
// images such a block can touch lie within 2^31 bytes (*bpi = 0), else blocks that stay inside
// one image (*bpi = blocks per image; an image plane is below 2^31 bytes by validation).
// Returns the extent in bytes that the offsets stay below.
unsigned tile_block_reach(const Geo& g, int* bpi, int* blocks) {
  const long long T = (long long)g.th * g.tw;
  const long long images = 63 / T + 2;  // images a block of 64 consecutive tiles can touch
  const long long span = images * g.C * g.H * g.W * 4LL;
  if (span < (1LL << 31)) {
    *bpi = 0;
    *blocks = (int)(((long long)g.P + 63) / 64);
    return (unsigned)span;
  }
  *bpi = (int)((T + 63) / 64);
  *blocks = (int)((long long)g.N * *bpi);
  return (unsigned)((long long)g.H * g.W * 4LL);
}

hipError_t launch_input_range(const Geo& g, const float* x, float* partial, int32_t* colsum,
                              int zero_colsum, int* groups_out, hipStream_t s) {
  if (is_nhwc(g)) return launch_input_nhwc_range(g, x, partial, colsum, zero_colsum, groups_out, s);
  if (input_range_strip_applicable(g, x))
    return launch_input_range_strip(g, x, partial, colsum, zero_colsum, groups_out, s);
  RArgs a{};
  a.x = x; a.partial = partial; a.colsum = colsum;
  a.N = g.N; a.C = g.C; a.H = g.H; a.W = g.W; a.pad = g.pad; a.th = g.th; a.tw = g.tw; a.P = g.P;
  a.T = g.th * g.tw;
  a.zero_colsum = zero_colsum;
  a.reach = tile_block_reach(g, &a.bpi, &a.TB);
  // Work units: a tile block with all channels, or, when there are few blocks, with a chunk of
  // channels (a multiple of 4, at least 8) so that about kTargetUnits units exist.
  constexpr int kTargetUnits = 512;  // two units per compute unit
  int cchunks = 1;
  if (a.TB < kTargetUnits) {
    cchunks = kTargetUnits / a.TB;  // rounded down: one round of workgroups, not one and a bit
    const int most = (g.C + 7) / 8;
    if (cchunks > most) cchunks = most;
  }
  a.CC = ((g.C + cchunks - 1) / cchunks + 3) / 4 * 4;
  a.cchunks = (g.C + a.CC - 1) / a.CC;
  const long long units = (long long)a.TB * a.cchunks;
  if (units > (1LL << 30)) return hipErrorInvalidValue;
  a.units = (int)units;
  const int pairs = (a.units + 1) / 2;
  const int grid = pairs < kMaxRangeGroups ? pairs : kMaxRangeGroups;
  *groups_out = grid;
  const int mode = patch_load_mode(g);
  note_kernel("input_range_kernel");
  if (g.m == 2) {
    if (mode == 0) input_range_kernel<2, 0><<<grid, kThreads, 0, s>>>(a);
    else if (mode == 1) input_range_kernel<2, 1><<<grid, kThreads, 0, s>>>(a);
    else input_range_kernel<2, 2><<<grid, kThreads, 0, s>>>(a);
  } else {
    if (mode == 0) input_range_kernel<4, 0><<<grid, kThreads, 0, s>>>(a);
    else if (mode == 1) input_range_kernel<4, 1><<<grid, kThreads, 0, s>>>(a);
    else input_range_kernel<4, 2><<<grid, kThreads, 0, s>>>(a);
  }
  return hipGetLastError();
}

}  // namespace lance
