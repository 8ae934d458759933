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
  // interior tiles: ty in [ty_lo, ty_hi), tx in [tx_lo, tx_hi); n_int of them, w_int per row;
  // border list: nb_top whole rows above, nb_bot below, then sw side tiles per middle row
  int ty_lo, ty_hi, tx_lo, tx_hi, n_int, w_int, nb_top, nb_bot, sw;
  unsigned magic_w_int, magic_tw, magic_sw;  // see dev::fast_div
};

// Vectors of floats that need only 4-byte alignment (the hardware allows unaligned multi-dword
// global loads): a patch row starts at any pixel.
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
typedef float f2u __attribute__((ext_vector_type(2), aligned(4)));

// One patch row from (uniform base) + (per-lane byte offset): the form the compiler turns into
// scalar-base global loads, so the walk over channels costs no vector address arithmetic.
template <int A>
__device__ __forceinline__ void load_row(const char* __restrict__ base, unsigned off,
                                         float (&row)[A]) {
  const f4u v = *reinterpret_cast<const f4u*>(base + off);
  row[0] = v[0]; row[1] = v[1]; row[2] = v[2]; row[3] = v[3];
  if constexpr (A == 6) {
    const f2u w = *reinterpret_cast<const f2u*>(base + off + 16);
    row[4] = w[0]; row[5] = w[1];
  }
}

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

// list index -> tile.  Tiles of an image are enumerated interior first (every pixel of the patch
// inside the image), then the border tiles: whole rows above, whole rows below, side tiles.
__device__ __forceinline__ void list_to_tile(const RArgs& a, int t, int* ty, int* tx) {
  if (t < a.n_int) {
    const int q = dev::fast_div(t, a.magic_w_int);
    *ty = a.ty_lo + q;
    *tx = a.tx_lo + (t - q * a.w_int);
    return;
  }
  int j = t - a.n_int;
  if (j < a.nb_top) {
    *ty = dev::fast_div(j, a.magic_tw); *tx = j - *ty * a.tw;
  } else if (j < a.nb_top + a.nb_bot) {
    j -= a.nb_top;
    const int q = dev::fast_div(j, a.magic_tw);
    *ty = a.ty_hi + q; *tx = j - q * a.tw;
  } else {
    j -= a.nb_top + a.nb_bot;
    const int q = dev::fast_div(j, a.magic_sw);
    const int k = j - q * a.sw;
    *ty = a.ty_lo + q;
    *tx = k < a.tx_lo ? k : a.tx_hi + (k - a.tx_lo);
  }
}

// A work unit is a range of the tile list of one image times a chunk of channels.  Its work
// items are (tile, channel pair) for interior tiles -- plain vector loads, two channels so that
// min/max of three operands are single instructions, the loads of the next item issued before
// the current one is transformed -- and (tile, channel) for border tiles (guarded loads).  Items
// are dealt to the 256 lanes with the tile index fastest, so a wave reads contiguous image rows
// and the few border tiles are spread over all lanes instead of keeping one wave busy.
template <int M>
__global__ __launch_bounds__(kThreads) void input_range_kernel(const RArgs a) {
  constexpr int A = M + 2, E = A * A;
  __shared__ float red[kThreads / 64][E][2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tiles = a.th * a.tw;
  const size_t HWb = (size_t)a.H * a.W * sizeof(float);

  float mn[E], mx[E];
#pragma unroll
  for (int e = 0; e < E; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }

  for (int unit = blockIdx.x; unit < a.units; unit += gridDim.x) {
    int b = unit;
    const int tchunk = b % a.tchunks; b /= a.tchunks;
    const int cchunk = b % a.cchunks;
    const int n = b / a.cchunks;
    const int c0 = cchunk * a.CC, cn = min(a.C, c0 + a.CC) - c0;
    const int t0 = tchunk * a.TT, t1 = min(tiles, t0 + a.TT);
    const char* img0 = reinterpret_cast<const char*>(a.x) + ((size_t)n * a.C + c0) * HWb;

    if (a.zero_colsum && cchunk == 0) {
      for (int t = t0 + tid; t < t1; t += kThreads) {
        int ty, tx;
        list_to_tile(a, t, &ty, &tx);
        const unsigned p = (unsigned)((n * a.th + ty) * a.tw + tx);
#pragma unroll
        for (int e = 0; e < E; e++) a.colsum[p + (unsigned)e * a.P] = 0;
      }
    }

    // ---- interior tiles: items = (tile, channel pair) ----
    const int ti1 = min(t1, a.n_int);
    const int nt_i = max(ti1 - t0, 0);
    const int npair = (cn + 1) / 2;
    const int items_i = nt_i * npair;
    // item = cp * nt_i + tl, walked with stride 256 without dividing again
    const int step_q = nt_i > 0 ? kThreads / nt_i : 0, step_r = nt_i > 0 ? kThreads - step_q * nt_i : 0;
    int cp_next = nt_i > 0 ? tid / nt_i : 0, tl_next = nt_i > 0 ? tid - cp_next * nt_i : 0;
    auto load_item = [&](float (&d0)[A][A], float (&d1)[A][A]) {
      const int cp = cp_next, tl = tl_next;
      tl_next += step_r; cp_next += step_q;
      if (tl_next >= nt_i) { tl_next -= nt_i; cp_next++; }
      int ty, tx;
      list_to_tile(a, t0 + tl, &ty, &tx);
      const unsigned off0 = (unsigned)(((ty * M - a.pad) * a.W + (tx * M - a.pad)) * 4);
      const int ca = 2 * cp, cb2 = min(2 * cp + 1, cn - 1);  // odd tail: the last channel twice
      const char* pa = img0 + (size_t)ca * HWb;
      const char* pb = img0 + (size_t)cb2 * HWb;
#pragma unroll
      for (int r = 0; r < A; r++) {
        load_row<A>(pa, off0 + (unsigned)(r * a.W * 4), d0[r]);
        load_row<A>(pb, off0 + (unsigned)(r * a.W * 4), d1[r]);
      }
    };
    auto reduce_item = [&](float (&d0)[A][A], float (&d1)[A][A]) {
      dev::input_tile_transform<M>(d0);
      dev::input_tile_transform<M>(d1);
#pragma unroll
      for (int e = 0; e < E; e++) {
        mn[e] = fminf(fminf(mn[e], d0[e / A][e % A]), d1[e / A][e % A]);
        mx[e] = fmaxf(fmaxf(mx[e], d0[e / A][e % A]), d1[e / A][e % A]);
      }
    };
    {
      float p0[A][A], p1[A][A], q0[A][A], q1[A][A];
      int item = tid;
      if (item < items_i) load_item(p0, p1);
      while (item < items_i) {
        const int nxt = item + kThreads;
        if (nxt < items_i) load_item(q0, q1);
        reduce_item(p0, p1);
        item = nxt;
        if (item >= items_i) break;
        const int nxt2 = item + kThreads;
        if (nxt2 < items_i) load_item(p0, p1);
        reduce_item(q0, q1);
        item = nxt2;
      }
    }

    // ---- border tiles: items = (tile, channel), guarded loads ----
    const int tb0 = max(t0, a.n_int);
    const int nt_b = max(t1 - tb0, 0);
    const int items_b = nt_b * cn;
    const int bstep_q = nt_b > 0 ? kThreads / nt_b : 0, bstep_r = nt_b > 0 ? kThreads - bstep_q * nt_b : 0;
    int c = nt_b > 0 ? tid / nt_b : 0, tl = nt_b > 0 ? tid - c * nt_b : 0;
    for (int item = tid; item < items_b; item += kThreads) {
      int ty, tx;
      list_to_tile(a, tb0 + tl, &ty, &tx);
      const int y0 = ty * M - a.pad, x0 = tx * M - a.pad;
      const char* img = img0 + (size_t)c * HWb;
      float d[A][A];
#pragma unroll
      for (int r = 0; r < A; r++)
#pragma unroll
        for (int s = 0; s < A; s++) {
          const int gy = y0 + r, gx = x0 + s;
          const bool ok = gy >= 0 && gy < a.H && gx >= 0 && gx < a.W;
          // clamp the address into the image, zero what lies outside
          const float v = *reinterpret_cast<const float*>(img + (ok ? (unsigned)((gy * a.W + gx) * 4) : 0u));
          d[r][s] = ok ? v : 0.0f;
        }
      dev::input_tile_transform<M>(d);
#pragma unroll
      for (int e = 0; e < E; e++) {
        mn[e] = fminf(mn[e], d[e / A][e % A]);
        mx[e] = fmaxf(mx[e], d[e / A][e % A]);
      }
      tl += bstep_r; c += bstep_q;
      if (tl >= nt_b) { tl -= nt_b; c++; }
    }
  }

  // wave reduction: the first NP positions by the scattering butterfly (lane group g ends up
  // with position g), the rest (m = 4 only: positions 32..35) one by one
  constexpr int NP = E >= 32 ? 32 : 16;
  {
    float lo, hi;
    dev::wave_minmax_scatter<NP>(mn, mx, lane, &lo, &hi);
    constexpr int per = 64 / NP;
    if (lane % per == 0) { red[wave][lane / per][0] = lo; red[wave][lane / per][1] = hi; }
  }
#pragma unroll
  for (int e = NP; e < E; e++) {
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
  {
    const int A = g.m + 2;
    auto lo = [&](int pad) { return (pad + g.m - 1) / g.m; };                  // first t with t*m-pad >= 0
    auto hi = [&](int extent, int nt) {                                        // one past last t with t*m-pad+A <= extent
      const int v = extent - A + g.pad;
      int h = v < 0 ? 0 : v / g.m + 1;
      return h > nt ? nt : h;
    };
    a.ty_lo = lo(g.pad); a.tx_lo = lo(g.pad);
    a.ty_hi = hi(g.H, g.th); a.tx_hi = hi(g.W, g.tw);
    if (a.ty_lo > g.th) a.ty_lo = g.th;
    if (a.tx_lo > g.tw) a.tx_lo = g.tw;
    if (a.ty_hi < a.ty_lo) a.ty_hi = a.ty_lo;
    if (a.tx_hi < a.tx_lo) a.tx_hi = a.tx_lo;
    if (a.ty_hi == a.ty_lo || a.tx_hi == a.tx_lo) {   // no interior tile: everything is "top" border
      a.ty_lo = a.ty_hi = g.th; a.tx_lo = 0; a.tx_hi = 0;
    }
    a.w_int = a.tx_hi - a.tx_lo;
    a.n_int = (a.ty_hi - a.ty_lo) * a.w_int;
    a.nb_top = a.ty_lo * g.tw;
    a.nb_bot = (g.th - a.ty_hi) * g.tw;
    a.sw = a.tx_lo + (g.tw - a.tx_hi);
    if (a.w_int == 0) a.w_int = 1;
    if (a.sw == 0) a.sw = 1;
    a.magic_w_int = div_magic(a.w_int); a.magic_tw = div_magic(g.tw); a.magic_sw = div_magic(a.sw);
    if (tiles * g.tw >= (1LL << 32)) return hipErrorInvalidValue;  // fast_div range
  }
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
