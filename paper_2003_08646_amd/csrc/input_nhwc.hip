// Stage 2 for NHWC activations (the layout of Sec. 3.3): v^ = Q(B^T d B) for every input patch
// (Algorithm 1; Eq. 7), X fp32 [N][H][W][C] in, blocked int8 codes out.  Two passes as for NCHW:
// the range pass (per-position min and max of V over real channels and all tiles) and the
// quantize pass (codes and their column sums); fp32 V is never stored.
//
// 16 lanes per (tile, channel block): lane cl holds the channels cl, cl+Q, cl+2Q, cl+3Q of the
// block, so its four codes are one dword of the blocked layout (byte i of dword cl = channel
// cl + i*Q) and the 16 lanes write one 64-byte code row per position.  In NHWC the channels of
// a pixel are contiguous: the 16 lanes read 64 contiguous bytes of a pixel per load, straight
// from memory; nothing is staged in LDS and nothing is transposed.  A tile's pixels are loaded
// once per tile (neighbouring tiles overlap by two rows and columns; those loads hit in cache).
//
// Column sums of the codes: 16-lane DPP reduction; atomic add when the channel axis spans
// several blocks (the sums are cleared before the pass).
#include <limits.h>

#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

constexpr int kThreads = 256;
constexpr int kGroupsPerWg = kThreads / 16;  // (tile, block) groups a workgroup handles at once

struct NhArgs {
  const float* x;
  int8_t* vq;
  int32_t* colsum;
  const float* qparams;  // quantize pass: [E][2] = {min, inv}
  float* partial;        // range pass: records [grid][E][2]
  int C, H, W, pad, th, tw, P, CB, NB, Q, bits;
  long long groups;  // P * NB
};

// Loads the (m+2)^2 window of tile p, channel c (clamped by the caller to a real channel), zero
// outside the image.
template <int M>
__device__ __forceinline__ void load_window(const NhArgs& a, int n, int y0, int x0, int c,
                                            float (&d)[M + 2][M + 2]) {
  constexpr int A = M + 2;
  const float* img = a.x + (size_t)n * a.H * a.W * a.C + c;
#pragma unroll
  for (int r = 0; r < A; r++) {
    const int gy = y0 + r;
    const bool rok = gy >= 0 && gy < a.H;
    const size_t rowoff = (size_t)min(max(gy, 0), a.H - 1) * a.W;
#pragma unroll
    for (int s = 0; s < A; s++) {
      const int gx = x0 + s;
      const bool ok = rok && gx >= 0 && gx < a.W;
      const float v = img[(rowoff + (size_t)min(max(gx, 0), a.W - 1)) * a.C];
      d[r][s] = ok ? v : 0.0f;
    }
  }
}

// What a lane works on: group index -> tile, block, window origin, real channels.
struct Group {
  int p, cb, n, y0, x0;
  int c[4];      // channel of byte i, clamped to a real one
  bool real[4];  // byte i holds a real channel
};

template <int M>
__device__ __forceinline__ Group decode_group(const NhArgs& a, long long grp, int cl) {
  Group g;
  g.cb = (int)(grp % a.NB);
  g.p = (int)(grp / a.NB);
  const int tx = g.p % a.tw, t2 = g.p / a.tw;
  const int ty = t2 % a.th;
  g.n = t2 / a.th;
  g.y0 = ty * M - a.pad;
  g.x0 = tx * M - a.pad;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int c = g.cb * a.CB + cl + a.Q * i;
    g.real[i] = cl < a.Q && c < a.C;
    g.c[i] = min(c, a.C - 1);
  }
  return g;
}

// Range pass: every workgroup leaves one record [E][2] = {min, max} over the groups it walked.
template <int M>
__global__ __launch_bounds__(kThreads) void input_nhwc_range_kernel(const NhArgs a) {
  constexpr int A = M + 2, E = A * A;
  __shared__ float red[kThreads / 64][E][2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cl = lane & 15;
  float mn[E], mx[E];
#pragma unroll
  for (int e = 0; e < E; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }
  for (long long grp = (long long)blockIdx.x * kGroupsPerWg + (tid >> 4); grp < a.groups;
       grp += (long long)gridDim.x * kGroupsPerWg) {
    const Group g = decode_group<M>(a, grp, cl);
#pragma unroll
    for (int i = 0; i < 4; i++) {
      float d[A][A];
      load_window<M>(a, g.n, g.y0, g.x0, g.c[i], d);
      dev::input_tile_transform<M>(d);
      if (g.real[i]) {
#pragma unroll
        for (int e = 0; e < E; e++) {
          mn[e] = fminf(mn[e], d[e / A][e % A]);
          mx[e] = fmaxf(mx[e], d[e / A][e % A]);
        }
      }
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
    const float lo = dev::wave_min(mn[e]);
    const float hi = dev::wave_max(mx[e]);
    if (lane == 0) { red[wave][e][0] = lo; red[wave][e][1] = hi; }
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

// Quantize pass.  B8: the code width is 8 bits.
template <int M, bool B8>
__global__ __launch_bounds__(kThreads) void input_nhwc_quant_kernel(const NhArgs a) {
  constexpr int A = M + 2, E = A * A;
  const int tid = threadIdx.x, cl = tid & 15;
  const long long grp = (long long)blockIdx.x * kGroupsPerWg + (tid >> 4);
  // Eq. 7 parameters as wave-uniform scalars
  float qmn[E], qinv[E];
#pragma unroll
  for (int e = 0; e < E; e++) {
    qmn[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a.qparams[2 * e])));
    qinv[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a.qparams[2 * e + 1])));
  }
  const bool valid = grp < a.groups;
  const Group g = decode_group<M>(a, valid ? grp : a.groups - 1, cl);
  const float L = (float)((1 << a.bits) - 1);
  const unsigned h = 1u << (a.bits - 1);
  const size_t estride = (size_t)a.NB * (size_t)a.P * (size_t)a.CB;  // bytes per position

  unsigned pk[E];  // unsigned codes of Eq. 7, byte i = channel cl + i*Q
#pragma unroll
  for (int e = 0; e < E; e++) pk[e] = 0;
  unsigned realmask = 0;
  int nreal = 0;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    if (g.real[i]) { realmask |= 0xFFu << (8 * i); nreal++; }
    float d[A][A];
    load_window<M>(a, g.n, g.y0, g.x0, g.c[i], d);
    dev::input_tile_transform<M>(d);
#pragma unroll
    for (int e = 0; e < E; e++) {
      // clamp(rne((x - min) * inv), 0, L): v_cvt_pk_u8_f32 rounds to nearest even and saturates
      // to [0, 255], so only the upper clamp of narrower codes needs an instruction of its own
      float tq = (d[e / A][e % A] - qmn[e]) * qinv[e];
      if constexpr (!B8) tq = fminf(tq, L);
      pk[e] = __builtin_amdgcn_cvt_pk_u8_f32(tq, i, pk[e]);
    }
  }
  const unsigned H8 = 0x80808080u, hh = h * 0x01010101u;
  int tot[E];
#pragma unroll
  for (int e = 0; e < E; e++) {
    // bytes of channels that do not exist are dropped before the sum
    pk[e] &= realmask;
    // column sum of the signed codes: (sum of the unsigned bytes) - nreal*h
    tot[e] = dev::row16_sum((int)__builtin_amdgcn_sad_u8(pk[e], 0u, 0u) - nreal * (int)h);
    // per-byte (code - h) mod 256 without borrows between bytes (for h = 128 that is a flip of
    // the top bit), padding bytes -> 0
    if constexpr (B8)
      pk[e] = (pk[e] ^ H8) & realmask;
    else
      pk[e] = (((pk[e] | H8) - (hh & ~H8)) ^ ((pk[e] ^ ~hh) & H8)) & realmask;
  }
  if (!valid) return;
  char* row = reinterpret_cast<char*>(a.vq) + ((size_t)g.cb * a.P + g.p) * a.CB + 4u * cl;
  if (cl < a.Q) {
#pragma unroll
    for (int e = 0; e < E; e++) *reinterpret_cast<unsigned*>(row + e * estride) = pk[e];
  }
  if (cl == 0) {
    if (a.NB > 1) {
#pragma unroll
      for (int e = 0; e < E; e++) atomicAdd(a.colsum + ((size_t)e * a.P + g.p), tot[e]);
    } else {
#pragma unroll
      for (int e = 0; e < E; e++) a.colsum[(size_t)e * a.P + g.p] = tot[e];
    }
  }
}

NhArgs make_args(const Geo& g, const float* x) {
  NhArgs a{};
  a.x = x;
  a.C = g.C; a.H = g.H; a.W = g.W; a.pad = g.pad; a.th = g.th; a.tw = g.tw; a.P = g.P;
  a.CB = g.CB; a.NB = g.NB; a.Q = g.Q; a.bits = g.bits;
  a.groups = (long long)g.P * g.NB;
  return a;
}

}  // namespace

hipError_t launch_input_nhwc_range(const Geo& g, const float* x, float* partial, int32_t* colsum,
                                   int zero_colsum, int* groups_out, hipStream_t s) {
  if (zero_colsum) {
    const hipError_t e = launch_fill_zero(colsum, (size_t)g.E * g.P, s);
    if (e != hipSuccess) return e;
  }
  NhArgs a = make_args(g, x);
  a.partial = partial;
  const long long wgs = (a.groups + kGroupsPerWg - 1) / kGroupsPerWg;
  const int grid = (int)(wgs < kMaxRangeGroups ? wgs : kMaxRangeGroups);
  *groups_out = grid;
  if (g.m == 2) input_nhwc_range_kernel<2><<<grid, kThreads, 0, s>>>(a);
  else input_nhwc_range_kernel<4><<<grid, kThreads, 0, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_input_nhwc_quant(const Geo& g, const float* x, const float* qparams, int8_t* vq,
                                   int32_t* colsum, hipStream_t s) {
  NhArgs a = make_args(g, x);
  a.qparams = qparams; a.vq = vq; a.colsum = colsum;
  const long long wgs = (a.groups + kGroupsPerWg - 1) / kGroupsPerWg;
  if (wgs > INT_MAX) return hipErrorInvalidValue;
  const unsigned grid = (unsigned)wgs;
  const bool b8 = g.bits == 8;
  if (g.m == 2) {
    if (b8) input_nhwc_quant_kernel<2, true><<<grid, kThreads, 0, s>>>(a);
    else input_nhwc_quant_kernel<2, false><<<grid, kThreads, 0, s>>>(a);
  } else {
    if (b8) input_nhwc_quant_kernel<4, true><<<grid, kThreads, 0, s>>>(a);
    else input_nhwc_quant_kernel<4, false><<<grid, kThreads, 0, s>>>(a);
  }
  return hipGetLastError();
}

}  // namespace lance
