// Stage 2, first pass for pad 1 and image widths that are multiples of 4: the (min,max)
// of every Winograd-domain position of V = B^T d B over the whole input (the T of Eq. 7), with
// every input pixel loaded exactly once per strip.
//
// The lane-per-tile range pass (input_range.hip) reads each tile's 4x4 patch with four 16-byte
// row loads: horizontally adjacent patches overlap by half and vertically adjacent ones too, so
// a wave-wide load instruction brings 256 new bytes, and the pass is bound by the rate at which
// the vector memory unit takes load instructions (about 25 cycles per wave-wide load), not by
// HBM.  Here a lane owns one aligned 16-byte column segment (pixels 4q .. 4q+3 of every row,
// i.e. the two tiles 2q and 2q+1 of every tile row) of one channel plane and walks down a strip
// of tile rows: each image row is loaded once, the pixel left of the segment comes from the
// lane below and the pixel right of it from the lane above (whole-wave DPP shifts; zero at the
// image edges), and the two rows a tile row shares with the next one stay in registers.  Rows
// above and below the image are loads whose offset is out of the buffer's range (they return
// zero).  A wave-wide load brings 1 KB of new pixels.
//
// The transform of a patch is the canonical one (columns first, then rows, one rounding per
// operation); the column pass of the six pixel columns of a lane is shared by its two tiles
// (the same operations on the same values as in two separate patches).
//
// F(4x4,3x3) takes the same walk: a lane's 16-byte segment holds exactly the four new pixel
// columns of ONE 6x6 patch (tile column q), the fifth and sixth column are the neighbours'
// pixels, a tile row brings four new image rows (two row pairs) and shares two with the next.
//
// Lanes of a wave: G = 64 / Wq row groups (Wq = W / 4 segments per row), lane = g * Wq + q; each
// row group is one (plane, strip).  Lanes past G * Wq compute on duplicates and their results are
// dropped before the reduction.  Strips have S tile rows; the last strip of a
// plane is moved up to end at the last tile row (its overlap with the one before is computed
// twice, which min/max do not notice).
#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

constexpr int kThreads = 512;
constexpr int kRing = 4;  // row pairs in flight or in use per lane

typedef float v4f __attribute__((ext_vector_type(4)));

struct RsArgs {
  const float* x;
  float* partial;   // [gridDim.x][16][2]
  int32_t* colsum;  // cleared here when the code tensor has several channel blocks
  size_t colsum_n;
  int zero_colsum;
  int H, W, Wq, th;
  int G, S, nstrips;  // row groups per wave, tile rows per strip, strips per plane
  int groups, tasks;  // planes * nstrips; ceil(groups / G)
  unsigned x_bytes;
};

// rows y and y + 1 of the lane's segment (out-of-image rows: zero)
__device__ __forceinline__ void load_pair(const float* x, unsigned x_bytes, unsigned base, int y,
                                          int H, unsigned row_bytes, v4f (&dst)[2]) {
  const __amdgpu_buffer_rsrc_t rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(x), 0, x_bytes, 0x00020000);
  constexpr unsigned kOob = 0xFFFFFFF0u;
#pragma unroll
  for (int i = 0; i < 2; i++) {
    const unsigned off = (unsigned)(y + i) < (unsigned)H ? base + (unsigned)(y + i) * row_bytes : kOob;
    dst[i] = __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0));
  }
}

// value of lane - 1 (zero into lane 0) / of lane + 1 (zero into lane 63)
__device__ __forceinline__ float from_lane_below(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x138, 0xF, 0xF, true));
}
__device__ __forceinline__ float from_lane_above(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x130, 0xF, 0xF, true));
}

__global__ __launch_bounds__(kThreads, 4) void input_range_strip_kernel(const RsArgs a) {
  constexpr int E = 16;
  __shared__ float red[kThreads / 64][E][2];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);

  if (a.zero_colsum) {
    for (size_t i = (size_t)blockIdx.x * kThreads + tid; i < a.colsum_n;
         i += (size_t)gridDim.x * kThreads)
      a.colsum[i] = 0;
  }

  float mn[E], mx[E];
#pragma unroll
  for (int e = 0; e < E; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }

  const int g = lane / a.Wq, q = lane - g * a.Wq;
  const bool active = g < a.G;
  const int gc = min(g, a.G - 1);
  const bool left_edge = q == 0, right_edge = q == a.Wq - 1;
  const unsigned row_bytes = (unsigned)a.W * 4u;
  const int S = a.S;

  // six pixel columns of one image row: [0] left of the segment, [1..4] the segment, [5] right
  auto widen = [&](const v4f& s, float (&r)[6]) {
    const float l = from_lane_below(s[3]), rr = from_lane_above(s[0]);
    r[0] = left_edge ? 0.0f : l;
    r[1] = s[0]; r[2] = s[1]; r[3] = s[2]; r[4] = s[3];
    r[5] = right_edge ? 0.0f : rr;
  };

  const int total_waves = (int)gridDim.x * (kThreads / 64);
  for (int task = (int)blockIdx.x * (kThreads / 64) + wave8; task < a.tasks; task += total_waves) {
    const int group = min(task * a.G + gc, a.groups - 1);
    const int pc = group / a.nstrips, strip = group - pc * a.nstrips;
    const int ty0 = min(strip * S, a.th - S);
    const int y0 = 2 * ty0 - 1;  // first image row of the strip (pad = 1)
    const unsigned base = (unsigned)pc * (unsigned)a.H * row_bytes + (unsigned)q * 16u;

    // Row pair k = rows y0 + 2k, y0 + 2k + 1; tile row t of the strip uses pairs t and t + 1.
    // Pairs past S are never used: they repeat pair S so that every step issues two loads.
    v4f ring[kRing][2];
    auto issue = [&](int k, v4f (&dst)[2]) {
      load_pair(a.x, a.x_bytes, base, y0 + 2 * min(k, S), a.H, row_bytes, dst);
    };
#pragma unroll
    for (int k = 0; k < kRing; k++) issue(k, ring[k]);
    float top[2][6];  // the pair carried over from the tile row above
    widen(ring[0][0], top[0]);
    widen(ring[0][1], top[1]);
    for (int t0 = 0; t0 < S; t0 += kRing) {
#pragma unroll
      for (int u = 0; u < kRing; u++) {
        const int t = t0 + u;
        if (t >= S) break;  // wave-uniform
        float bot[2][6];
        widen(ring[(u + 1) % kRing][0], bot[0]);
        widen(ring[(u + 1) % kRing][1], bot[1]);
        issue(t + kRing, ring[u]);  // pair t has been widened one step ago
        // column pass (B^T d over the four rows) of the six pixel columns
        float c[4][6];
#pragma unroll
        for (int j = 0; j < 6; j++) {
          const float d4[4] = {top[0][j], top[1][j], bot[0][j], bot[1][j]};
          float t4[4];
          dev::Wino<2>::in1d(d4, t4);
#pragma unroll
          for (int i = 0; i < 4; i++) c[i][j] = t4[i];
        }
        // row pass of the two tiles: pixel columns 0..3 and 2..5
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const float ra[4] = {c[i][0], c[i][1], c[i][2], c[i][3]};
          const float rb[4] = {c[i][2], c[i][3], c[i][4], c[i][5]};
          float va[4], vb[4];
          dev::Wino<2>::in1d(ra, va);
          dev::Wino<2>::in1d(rb, vb);
#pragma unroll
          for (int j = 0; j < 4; j++) {
            mn[i * 4 + j] = fminf(mn[i * 4 + j], fminf(va[j], vb[j]));
            mx[i * 4 + j] = fmaxf(mx[i * 4 + j], fmaxf(va[j], vb[j]));
          }
        }
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
          for (int j = 0; j < 6; j++) top[i][j] = bot[i][j];
      }
    }
  }
  if (!active) {
#pragma unroll
    for (int e = 0; e < E; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }
  }

  {
    float lo, hi;
    dev::wave_minmax_scatter<E>(mn, mx, lane, &lo, &hi);
    constexpr int per = 64 / E;
    if (lane % per == 0) { red[wave8][lane / per][0] = lo; red[wave8][lane / per][1] = hi; }
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

// F(4x4,3x3): one tile per lane and tile row; row pair k = rows y0 + 2k, y0 + 2k + 1 with
// y0 = 4 * ty0 - 1; tile row t of the strip uses the pairs 2t (carried over), 2t + 1, 2t + 2.
__global__ __launch_bounds__(kThreads, 2) void input_range_strip_m4_kernel(const RsArgs a) {
  constexpr int E = 36, A = 6;
  __shared__ float red[kThreads / 64][E][2];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);

  if (a.zero_colsum) {
    for (size_t i = (size_t)blockIdx.x * kThreads + tid; i < a.colsum_n;
         i += (size_t)gridDim.x * kThreads)
      a.colsum[i] = 0;
  }

  float mn[E], mx[E];
#pragma unroll
  for (int e = 0; e < E; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }

  const int g = lane / a.Wq, q = lane - g * a.Wq;
  const bool active = g < a.G;
  const int gc = min(g, a.G - 1);
  const bool left_edge = q == 0, right_edge = q == a.Wq - 1;
  const unsigned row_bytes = (unsigned)a.W * 4u;
  const int S = a.S;

  auto widen = [&](const v4f& s, float (&r)[A]) {
    const float l = from_lane_below(s[3]), rr = from_lane_above(s[0]);
    r[0] = left_edge ? 0.0f : l;
    r[1] = s[0]; r[2] = s[1]; r[3] = s[2]; r[4] = s[3];
    r[5] = right_edge ? 0.0f : rr;
  };

  const int total_waves = (int)gridDim.x * (kThreads / 64);
  for (int task = (int)blockIdx.x * (kThreads / 64) + wave8; task < a.tasks; task += total_waves) {
    const int group = min(task * a.G + gc, a.groups - 1);
    const int pc = group / a.nstrips, strip = group - pc * a.nstrips;
    const int ty0 = min(strip * S, a.th - S);
    const int y0 = 4 * ty0 - 1;  // first image row of the strip (pad = 1)
    const unsigned base = (unsigned)pc * (unsigned)a.H * row_bytes + (unsigned)q * 16u;

    // Pairs past 2S are never used: they repeat pair 2S so that every step issues four loads.
    v4f ring[kRing][2];
    auto issue = [&](int k, v4f (&dst)[2]) {
      load_pair(a.x, a.x_bytes, base, y0 + 2 * min(k, 2 * S), a.H, row_bytes, dst);
    };
#pragma unroll
    for (int k = 0; k < kRing; k++) issue(k, ring[k]);
    float d[A][A];  // the patch: rows 0, 1 carried over from the tile row above
    widen(ring[0][0], d[0]);
    widen(ring[0][1], d[1]);
    issue(kRing, ring[0]);
    for (int t0 = 0; t0 < S; t0 += 2) {
#pragma unroll
      for (int u = 0; u < 2; u++) {
        const int t = t0 + u;
        if (t >= S) break;  // wave-uniform
        // pairs 2t + 1 and 2t + 2 sit in ring slots (2u + 1) and (2u + 2) % 4
        widen(ring[2 * u + 1][0], d[2]);
        widen(ring[2 * u + 1][1], d[3]);
        widen(ring[(2 * u + 2) % kRing][0], d[4]);
        widen(ring[(2 * u + 2) % kRing][1], d[5]);
        issue(2 * t + 1 + kRing, ring[2 * u + 1]);
        if (u == 0) issue(2 * t + 2 + kRing, ring[2]);  // slot 0 is refilled after the next step
        float v[A][A];
#pragma unroll
        for (int i = 0; i < A; i++)
#pragma unroll
          for (int j = 0; j < A; j++) v[i][j] = d[i][j];
        dev::input_tile_transform<4>(v);
#pragma unroll
        for (int i = 0; i < A; i++)
#pragma unroll
          for (int j = 0; j < A; j++) {
            mn[i * A + j] = fminf(mn[i * A + j], v[i][j]);
            mx[i * A + j] = fmaxf(mx[i * A + j], v[i][j]);
          }
#pragma unroll
        for (int j = 0; j < A; j++) { d[0][j] = d[4][j]; d[1][j] = d[5][j]; }
        if (u == 1) issue(2 * t + 2 + kRing, ring[0]);  // pair 2t + 2 has been widened and carried over
      }
    }
  }
  if (!active) {
#pragma unroll
    for (int e = 0; e < E; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }
  }

  {
    float lo, hi;
    dev::wave_minmax_scatter<32>(mn, mx, lane, &lo, &hi);
    if (lane % 2 == 0) { red[wave8][lane / 2][0] = lo; red[wave8][lane / 2][1] = hi; }
  }
#pragma unroll
  for (int e = 32; e < E; e++) {
    float lo = mn[e], hi = mx[e];
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      lo = fminf(lo, __shfl_xor(lo, o, 64));
      hi = fmaxf(hi, __shfl_xor(hi, o, 64));
    }
    if (lane == 0) { red[wave8][e][0] = lo; red[wave8][e][1] = hi; }
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

// Pad 1, rows of whole 16-byte segments that fit a wave, at least four tile rows, the whole tensor
// addressable by 32-bit byte offsets from a 16-byte aligned start.
bool input_range_strip_applicable(const Geo& g, const float* x) {
  if (is_nhwc(g)) return false;  // this kernel addresses NCHW tensors
  const long long bytes = (long long)g.N * g.C * g.H * g.W * 4LL;
  return g.pad == 1 && g.W % 4 == 0 && g.W <= 256 && g.th >= 4 &&
         bytes < 0xFFFFFFF0LL && (reinterpret_cast<uintptr_t>(x) & 15) == 0;
}

hipError_t launch_input_range_strip(const Geo& g, const float* x, float* partial, int32_t* colsum,
                                    int zero_colsum, int* groups_out, hipStream_t s) {
  if (!input_range_strip_applicable(g, x)) return hipErrorInvalidValue;
  RsArgs a{};
  a.x = x; a.partial = partial; a.colsum = colsum;
  a.colsum_n = (size_t)g.E * g.P; a.zero_colsum = zero_colsum;
  a.H = g.H; a.W = g.W; a.Wq = g.W / 4; a.th = g.th;
  a.G = 64 / a.Wq;
  a.x_bytes = (unsigned)((long long)g.N * g.C * g.H * g.W * 4LL);
  // Strips per plane: every strip re-reads two rows and starts with an empty load pipeline (about
  // ten tile rows' worth of time, from the measured durations of launches with strips of
  // different lengths); about 2048 waves (eight per compute unit) work at a time - launches with
  // 2300 .. 3600 tasks were measured 40-70 % slower than ones with 2048 tasks of the same length -
  // and fewer than about 1024 busy waves leave the memory system short of requests.  Cost of a
  // choice = rounds of 2048 tasks x (strip length + 10) x that shortage; the cheapest wins (at
  // least four tile rows per strip).
  const long long planes = (long long)g.N * g.C;
  constexpr long long kBusyWaves = 2048;
  double best_cost = 0.0;
  for (int want = 1; want <= (g.th / 4 > 1 ? g.th / 4 : 1); want++) {
    const int S = (g.th + want - 1) / want, nstrips = (g.th + S - 1) / S;
    const long long tasks = (planes * nstrips + a.G - 1) / a.G;
    const long long rounds = (tasks + kBusyWaves - 1) / kBusyWaves;
    const double cost = (double)rounds * (S + 10) * (tasks < 1024 ? 1024.0 / (double)tasks : 1.0);
    if (want == 1 || cost < best_cost) {
      best_cost = cost;
      a.S = S;
      a.nstrips = nstrips;
    }
  }
  const long long groups = planes * a.nstrips;
  if (groups > (1LL << 30)) return hipErrorInvalidValue;
  a.groups = (int)groups;
  a.tasks = (a.groups + a.G - 1) / a.G;
  const int waves_per_wg = kThreads / 64;
  int grid = (a.tasks + waves_per_wg - 1) / waves_per_wg;
  if (grid > 512) grid = 512;
  *groups_out = grid;
  note_kernel(g.m == 2 ? "input_range_strip_kernel" : "input_range_strip_m4_kernel");
  if (g.m == 2) input_range_strip_kernel<<<grid, kThreads, 0, s>>>(a);
  else input_range_strip_m4_kernel<<<grid, kThreads, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace lance
