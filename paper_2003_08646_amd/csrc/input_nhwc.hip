// Stage 2 for NHWC activations (the layout of Sec. 3.3): v^ = Q(B^T d B) for every input patch
// (Algorithm 1; Eq. 7), X fp32 [N][H][W][C] in, blocked int8 codes out.  Two passes as for NCHW:
// the range pass (per-position min and max of V over real channels and all tiles) and the
// quantize pass (codes and their column sums); fp32 V is never stored.
//
// 16 lanes per (tile, channel block): lane cl holds the channels 4*cl .. 4*cl+3 of the block.
// With NHWC the code blocks keep the channels in their natural order, so the lane's four codes
// are dword cl of the code row and the 16 lanes write one 64-byte row per position.  The
// channels of a pixel are contiguous in X: a lane reads its four with one 16-byte load (four
// 4-byte loads when C is not a multiple of 4 or X is not 16-byte aligned), the 16 lanes 256
// contiguous bytes, straight from memory; nothing is staged in LDS and nothing is transposed.
// A tile's pixels are loaded once per tile (neighbouring tiles overlap by two rows and columns;
// those loads hit in cache), except in the rolling range pass of F(2x2,3x3), which keeps the
// rows two vertically adjacent tiles share in registers.  Layers with at most 16 channels have
// a range pass of their own (lane = tile).
//
// Column sums of the codes: 16-lane DPP reduction.  With several channel blocks the groups of
// one tile are neighbours in a workgroup (16 groups): when NB divides 16 their sums are added
// through LDS and stored once; otherwise they are added with atomics (the sums are cleared
// before the pass).
#include <limits.h>

#include <atomic>

#include "lance_device.h"
#include "lance_internal.h"
#include "nhwc_window.h"

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
  int R, strips, units;  // rolling range pass: tile rows per strip, strips per image column, work units
  int groups;        // P * NB
  unsigned x_bytes;  // size of X (used by the 16-byte loads: below 0xFFFFFFF0 then)
  int packed;        // quantize pass: vq is [E][NB][P][32], two 4-bit codes per byte
};

typedef float f4 __attribute__((ext_vector_type(4)));

// What a lane works on: group index -> tile, block, window origin, real channels.
struct Group {
  int p, cb, n, y0, x0;
  int c[4];      // channel of byte i, clamped to a real one (c[0] .. c[0]+3 all real with VEC)
  bool real[4];  // byte i holds a real channel
};

// Loads the lane's four channels of the (m+2)^2 window of its tile, zero outside the image.
// VEC: C is a multiple of 4 and X is 16-byte aligned: one load per pixel.
template <int M, bool VEC>
__device__ __forceinline__ void load_window(const NhArgs& a, const Group& g,
                                            f4 (&d)[M + 2][M + 2]) {
  constexpr int A = M + 2;
  if constexpr (VEC) {
    f4 w[A * A];
    dev::load_window_nhwc<M>(a.x, a.x_bytes, g.n, g.y0, g.x0, g.c[0], a.H, a.W, a.C, w);
#pragma unroll
    for (int r = 0; r < A; r++)
#pragma unroll
      for (int s = 0; s < A; s++) d[r][s] = w[r * A + s];
    return;
  }
  const float* img = a.x + (size_t)g.n * a.H * a.W * a.C;
#pragma unroll
  for (int r = 0; r < A; r++) {
    const int gy = g.y0 + r;
    const bool rok = gy >= 0 && gy < a.H;
    const size_t rowoff = (size_t)min(max(gy, 0), a.H - 1) * a.W;
#pragma unroll
    for (int s = 0; s < A; s++) {
      const int gx = g.x0 + s;
      const bool ok = rok && gx >= 0 && gx < a.W;
      const float* px = img + (rowoff + (size_t)min(max(gx, 0), a.W - 1)) * a.C;
      f4 v;
      if constexpr (VEC) {
        v = *reinterpret_cast<const f4*>(px + g.c[0]);
      } else {
#pragma unroll
        for (int i = 0; i < 4; i++) v[i] = px[g.c[i]];
      }
      d[r][s] = ok ? v : f4{0.0f, 0.0f, 0.0f, 0.0f};
    }
  }
}

// The same for the channels i0, i0+1 of the lane's four (i0 = 0 or 2).
typedef float f2 __attribute__((ext_vector_type(2)));
template <int M, bool VEC>
__device__ __forceinline__ void load_window_pair(const NhArgs& a, const Group& g, int i0,
                                                 f2 (&d)[M + 2][M + 2]) {
  constexpr int A = M + 2;
  const float* img = a.x + (size_t)g.n * a.H * a.W * a.C;
#pragma unroll
  for (int r = 0; r < A; r++) {
    const int gy = g.y0 + r;
    const bool rok = gy >= 0 && gy < a.H;
    const size_t rowoff = (size_t)min(max(gy, 0), a.H - 1) * a.W;
#pragma unroll
    for (int s = 0; s < A; s++) {
      const int gx = g.x0 + s;
      const bool ok = rok && gx >= 0 && gx < a.W;
      const float* px = img + (rowoff + (size_t)min(max(gx, 0), a.W - 1)) * a.C;
      f2 v;
      if constexpr (VEC) {
        v = *reinterpret_cast<const f2*>(px + g.c[i0]);
      } else {
        v[0] = px[g.c[i0]];
        v[1] = px[g.c[i0 + 1]];
      }
      d[r][s] = ok ? v : f2{0.0f, 0.0f};
    }
  }
}

template <int M, bool VEC>
__device__ __forceinline__ Group decode_group(const NhArgs& a, int grp, int cl) {
  Group g;
  g.p = grp / a.NB;
  g.cb = grp - g.p * a.NB;
  const int tx = g.p % a.tw, t2 = g.p / a.tw;
  const int ty = t2 % a.th;
  g.n = t2 / a.th;
  g.y0 = ty * M - a.pad;
  g.x0 = tx * M - a.pad;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int c = g.cb * a.CB + 4 * cl + i;
    g.real[i] = cl < a.Q && c < a.C;
    g.c[i] = VEC ? min(c - i, a.C - 4) + i : min(c, a.C - 1);
  }
  return g;
}

// One record [E][2] = {min, max} per workgroup from the lanes' running extrema.
template <int E>
__device__ __forceinline__ void write_range_record(const float (&mn)[E], const float (&mx)[E],
                                                   float (&red)[kThreads / 64][E][2],
                                                   float* partial, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
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
    partial[((size_t)blockIdx.x * E + tid) * 2 + 0] = lo;
    partial[((size_t)blockIdx.x * E + tid) * 2 + 1] = hi;
  }
}

// Range pass: every workgroup leaves one record [E][2] = {min, max} over the groups it walked.
template <int M, bool VEC>
__global__ __launch_bounds__(kThreads, 2) void input_nhwc_range_kernel(const NhArgs a) {
  constexpr int A = M + 2, E = A * A;
  __shared__ float red[kThreads / 64][E][2];
  const int tid = threadIdx.x, cl = tid & 15;
  float mn[E], mx[E];
#pragma unroll
  for (int e = 0; e < E; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }
  for (int grp = blockIdx.x * kGroupsPerWg + (tid >> 4); grp < a.groups;
       grp += gridDim.x * kGroupsPerWg) {
    const Group g = decode_group<M, VEC>(a, grp, cl);
    auto fold = [&](const float (&d)[A][A], bool real) {
      if (real) {
#pragma unroll
        for (int e = 0; e < E; e++) {
          mn[e] = fminf(mn[e], d[e / A][e % A]);
          mx[e] = fmaxf(mx[e], d[e / A][e % A]);
        }
      }
    };
    if constexpr (M == 2) {
      f4 w[A][A];
      load_window<M, VEC>(a, g, w);
      float d[4][A][A];
#pragma unroll
      for (int i = 0; i < 4; i++) {
#pragma unroll
        for (int r = 0; r < A; r++)
#pragma unroll
          for (int s2 = 0; s2 < A; s2++) d[i][r][s2] = w[r][s2][i];
        dev::input_tile_transform<M>(d[i]);
      }
      if (VEC) {
        // the lane's four channels exist together or not at all: two values per
        // three-operand minimum / maximum
        if (g.real[0]) {
#pragma unroll
          for (int e = 0; e < E; e++) {
            const int r = e / A, c = e % A;
            mn[e] = fminf(mn[e], fminf(d[0][r][c], d[1][r][c]));
            mn[e] = fminf(mn[e], fminf(d[2][r][c], d[3][r][c]));
            mx[e] = fmaxf(mx[e], fmaxf(d[0][r][c], d[1][r][c]));
            mx[e] = fmaxf(mx[e], fmaxf(d[2][r][c], d[3][r][c]));
          }
        }
      } else {
#pragma unroll
        for (int i = 0; i < 4; i++) fold(d[i], g.real[i]);
      }
    } else {
      // 36 running minima and maxima leave no room for a 36-pixel window of four channels:
      // two channels at a time
#pragma unroll
      for (int hf = 0; hf < 2; hf++) {
        f2 w[A][A];
        load_window_pair<M, VEC>(a, g, 2 * hf, w);
#pragma unroll
        for (int i = 0; i < 2; i++) {
          float d[A][A];
#pragma unroll
          for (int r = 0; r < A; r++)
#pragma unroll
            for (int s2 = 0; s2 < A; s2++) d[r][s2] = w[r][s2][i];
          dev::input_tile_transform<M>(d);
          fold(d, g.real[2 * hf + i]);
          // one channel's transform at a time, and the second pair's loads behind the first's
          // folds: left alone the scheduler interleaves them all and runs out of registers
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  }
  write_range_record<E>(mn, mx, red, a.partial, tid);
}

// Range pass of F(2x2,3x3) layers whose channels come four at a time (16-byte loads): the pass
// above issues 16 loads per tile of which a quarter of the bytes are new, and measured it is
// bound by the rate at which the vector memory unit takes load instructions, not by bytes or
// arithmetic.  Here a lane group (16 lanes, four channels each) walks down a strip of R tile
// rows of one tile column: the two pixel rows a tile shares with the one below stay in
// registers, so a tile costs two new rows (8 loads), requested before the current tile is
// transformed.  Work unit = (image, strip, tile column, channel block), tile columns and blocks
// of a wave next to each other.
template <int UNUSED = 0>
__global__ __launch_bounds__(kThreads, 2) void input_nhwc_range_roll_kernel(const NhArgs a) {
  constexpr int M = 2, A = 4, E = 16;
  __shared__ float red[kThreads / 64][E][2];
  const int tid = threadIdx.x, cl = tid & 15;
  float mn[E], mx[E];
#pragma unroll
  for (int e = 0; e < E; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }
  const unsigned px = (unsigned)a.C * 4u;
  for (int u = blockIdx.x * kGroupsPerWg + (tid >> 4); u < a.units; u += gridDim.x * kGroupsPerWg) {
    int t = u / a.NB;
    const int cb = u - t * a.NB;
    const int tx = t % a.tw; t /= a.tw;
    const int st = t % a.strips, n = t / a.strips;
    const int c0 = cb * a.CB + 4 * cl;
    const bool real = cl < a.Q && c0 < a.C;  // C is a multiple of 4: all four channels or none
    const int cc = min(c0, a.C - 4);
    const int ty0 = st * a.R, ty1 = min(ty0 + a.R, a.th);
    unsigned coloff[A];
    bool cok[A];
#pragma unroll
    for (int s = 0; s < A; s++) {
      const int gx = tx * M - a.pad + s;
      cok[s] = gx >= 0 && gx < a.W;
      coloff[s] = (unsigned)gx * px + (unsigned)cc * 4u;
    }
    auto load_row = [&](int gy, f4 (&row)[A]) {
      const unsigned rowoff = ((unsigned)n * (unsigned)a.H + (unsigned)gy) * (unsigned)a.W * px;
      dev::load_row_nhwc<A>(a.x, a.x_bytes, rowoff, gy >= 0 && gy < a.H, coloff, cok, row);
    };
    f4 w[A][A], nxt[2][A];
#pragma unroll
    for (int s = 0; s < A; s++) nxt[0][s] = nxt[1][s] = f4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int r = 0; r < A; r++) load_row(ty0 * M - a.pad + r, w[r]);
    for (int ty = ty0; ty < ty1; ty++) {
      if (ty + 1 < ty1) {  // the next tile's two new rows
        load_row((ty + 1) * M - a.pad + 2, nxt[0]);
        load_row((ty + 1) * M - a.pad + 3, nxt[1]);
      }
#pragma unroll
      for (int hf = 0; hf < 2; hf++) {  // two channels at a time: three-operand minima and maxima
        float d[2][A][A];
#pragma unroll
        for (int i = 0; i < 2; i++) {
#pragma unroll
          for (int r = 0; r < A; r++)
#pragma unroll
            for (int s = 0; s < A; s++) d[i][r][s] = w[r][s][2 * hf + i];
          dev::input_tile_transform<M>(d[i]);
        }
        if (real) {
#pragma unroll
          for (int e = 0; e < E; e++) {
            mn[e] = fminf(mn[e], fminf(d[0][e / A][e % A], d[1][e / A][e % A]));
            mx[e] = fmaxf(mx[e], fmaxf(d[0][e / A][e % A], d[1][e / A][e % A]));
          }
        }
      }
#pragma unroll
      for (int s = 0; s < A; s++) {
        w[0][s] = w[2][s]; w[1][s] = w[3][s];
        w[2][s] = nxt[0][s]; w[3][s] = nxt[1][s];
      }
    }
  }
  write_range_record<E>(mn, mx, red, a.partial, tid);
}

// Range pass of layers with at most 16 channels: with 16 lanes per tile most lanes would hold no
// channel at all.  Lane = tile instead, the channels one after the other (4-byte buffer loads at
// per-pixel offsets computed once per tile, the channel as the scalar offset); a wave takes
// blocks of 64 consecutive tiles with a grid stride.  X below 4 GB.
template <int M>
__global__ __launch_bounds__(kThreads) void input_nhwc_range_small_kernel(const NhArgs a) {
  constexpr int A = M + 2, E = A * A;
  __shared__ float red[kThreads / 64][E][2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float mn[E], mx[E];
#pragma unroll
  for (int e = 0; e < E; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }
  const int stride = gridDim.x * (kThreads / 64) * 64;
  for (int p0 = (blockIdx.x * (kThreads / 64) + wave) * 64; p0 < a.P; p0 += stride) {
    const bool valid = p0 + lane < a.P;
    const int pt = min(p0 + lane, a.P - 1);
    const int tx = pt % a.tw, t2 = pt / a.tw;
    const int ty = t2 % a.th, n = t2 / a.th;
    unsigned off[A * A];
    dev::window_offsets_nhwc<M>(n, ty * M - a.pad, tx * M - a.pad, a.H, a.W, a.C, off);
    auto fold = [&](float (&d)[A][A]) {
      dev::input_tile_transform<M>(d);
      if (valid) {
#pragma unroll
        for (int e = 0; e < E; e++) {
          mn[e] = fminf(mn[e], d[e / A][e % A]);
          mx[e] = fmaxf(mx[e], d[e / A][e % A]);
        }
      }
    };
    if (M == 2 && a.C <= 4) {  // an RGB image: a pixel is one load
      float px[A * A][4];
      dev::load_pixels_nhwc<M>(a.x, a.x_bytes, off, a.C, px);
#pragma unroll
      for (int c = 0; c < 4; c++) {
        if (c < a.C) {
          float d[A][A];
#pragma unroll
          for (int r = 0; r < A; r++)
#pragma unroll
            for (int s2 = 0; s2 < A; s2++) d[r][s2] = px[r * A + s2][c];
          fold(d);
        }
      }
    } else {
      for (int c = 0; c < a.C; c++) {
        float b[A * A], d[A][A];
        dev::load_channel_nhwc<M>(a.x, a.x_bytes, off, c, b);
#pragma unroll
        for (int r = 0; r < A; r++)
#pragma unroll
          for (int s2 = 0; s2 < A; s2++) d[r][s2] = b[r * A + s2];
        fold(d);
      }
    }
  }
  write_range_record<E>(mn, mx, red, a.partial, tid);
}

// Quantize pass.  B8: the code width is 8 bits.
template <int M, bool B8, bool VEC>
__global__ __launch_bounds__(kThreads) void input_nhwc_quant_kernel(const NhArgs a) {
  constexpr int A = M + 2, E = A * A;
  const int tid = threadIdx.x, cl = tid & 15;
  const int grp = blockIdx.x * kGroupsPerWg + (tid >> 4);
  // Eq. 7 parameters as wave-uniform scalars
  float qmn[E], qinv[E];
#pragma unroll
  for (int e = 0; e < E; e++) {
    qmn[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a.qparams[2 * e])));
    qinv[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a.qparams[2 * e + 1])));
  }
  const bool valid = grp < a.groups;
  const Group g = decode_group<M, VEC>(a, valid ? grp : a.groups - 1, cl);
  const float L = (float)((1 << a.bits) - 1);
  const unsigned h = 1u << (a.bits - 1);
  const size_t estride = (size_t)a.NB * (size_t)a.P * (size_t)a.CB;  // bytes per position

  f4 w[A][A];
  load_window<M, VEC>(a, g, w);
  unsigned pk[E];  // unsigned codes of Eq. 7, byte i = channel 4*cl + i of the block
#pragma unroll
  for (int e = 0; e < E; e++) pk[e] = 0;
  unsigned realmask = 0;
  int nreal = 0;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    if (g.real[i]) { realmask |= 0xFFu << (8 * i); nreal++; }
    float d[A][A];
#pragma unroll
    for (int r = 0; r < A; r++)
#pragma unroll
      for (int s2 = 0; s2 < A; s2++) d[r][s2] = w[r][s2][i];
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
  if (a.packed) {
    // two codes per byte (64-channel blocks): the lane's four codes become four nibbles
    // code + 8 (one bit flip of the two's-complement nibble; a padding byte 0 becomes 8), and the
    // lanes of channels 0..31 take those of channels 32..63 (eight lanes up) into the high bits
    char* prow = reinterpret_cast<char*>(a.vq) + ((size_t)g.cb * a.P + g.p) * 32 + 4u * cl;
#pragma unroll
    for (int e = 0; e < E; e++) {
      const unsigned n = (pk[e] ^ 0x08080808u) & 0x0F0F0F0Fu;
      const unsigned up = (unsigned)__builtin_amdgcn_update_dpp(0, (int)n, 0x108, 0xF, 0xF, false);  // row_shl:8
      pk[e] = n | (up << 4);
    }
    if (valid && cl < 8) {
#pragma unroll
      for (int e = 0; e < E; e++) *reinterpret_cast<unsigned*>(prow + e * (estride / 2)) = pk[e];
    }
  } else {
    char* row = reinterpret_cast<char*>(a.vq) + ((size_t)g.cb * a.P + g.p) * a.CB + 4u * cl;
    if (valid && cl < a.Q) {
#pragma unroll
      for (int e = 0; e < E; e++) *reinterpret_cast<unsigned*>(row + e * estride) = pk[e];
    }
  }
  if (a.NB == 1) {
    if (valid && cl == 0) {
#pragma unroll
      for (int e = 0; e < E; e++) a.colsum[(size_t)e * a.P + g.p] = tot[e];
    }
  } else if (kGroupsPerWg % a.NB == 0) {
    // the workgroup holds all blocks of kGroupsPerWg / NB tiles
    __shared__ int sums[kGroupsPerWg][E];
    if (cl == 0) {
#pragma unroll
      for (int e = 0; e < E; e++) sums[tid >> 4][e] = valid ? tot[e] : 0;
    }
    __syncthreads();
    const int tiles = kGroupsPerWg / a.NB;
    for (int t = tid; t < tiles * E; t += kThreads) {
      const int tl = t / E, e = t - tl * E;
      const int p = blockIdx.x * tiles + tl;
      if (p < a.P) {
        int s = 0;
        for (int b = 0; b < a.NB; b++) s += sums[tl * a.NB + b][e];
        a.colsum[(size_t)e * a.P + p] = s;
      }
    }
  } else if (valid && cl == 0) {
#pragma unroll
    for (int e = 0; e < E; e++) atomicAdd(a.colsum + ((size_t)e * a.P + g.p), tot[e]);
  }
}

NhArgs make_args(const Geo& g, const float* x) {
  NhArgs a{};
  a.x = x;
  a.C = g.C; a.H = g.H; a.W = g.W; a.pad = g.pad; a.th = g.th; a.tw = g.tw; a.P = g.P;
  a.CB = g.CB; a.NB = g.NB; a.Q = g.Q; a.bits = g.bits;
  a.groups = g.P * g.NB;  // below 2^30: checked by the launchers
  const long long xb = (long long)g.N * g.C * g.H * g.W * 4;
  a.x_bytes = xb < 0xFFFFFFF0LL ? (unsigned)xb : 0u;
  a.packed = is_packed(g) ? 1 : 0;
  return a;
}

}  // namespace

bool input_nhwc_adds_colsum_atomically(const Geo& g) { return g.NB > 1 && kGroupsPerWg % g.NB != 0; }

namespace {

bool groups_fit(const Geo& g) { return (long long)g.P * g.NB < (1LL << 30); }

bool vec_loads(const Geo& g, const float* x) {
  return g.C % 4 == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0 &&
         (long long)g.N * g.C * g.H * g.W * 4 < 0xFFFFFFF0LL;
}

}  // namespace

hipError_t launch_input_nhwc_range(const Geo& g, const float* x, float* partial, int32_t* colsum,
                                   int zero_colsum, int* groups_out, hipStream_t s) {
  if (zero_colsum) {
    const hipError_t e = launch_fill_zero(colsum, (size_t)g.E * g.P, s);
    if (e != hipSuccess) return e;
  }
  if (!groups_fit(g)) return hipErrorInvalidValue;
  NhArgs a = make_args(g, x);
  a.partial = partial;
  if (g.CB == 16 && a.x_bytes != 0) {  // at most 16 channels: lane = tile
    const long long blocks = ((long long)g.P + kThreads - 1) / kThreads;
    const int grid = (int)(blocks < kMaxRangeGroups ? blocks : kMaxRangeGroups);
    *groups_out = grid;
    note_kernel("input_nhwc_range_small_kernel");
    if (g.m == 2) input_nhwc_range_small_kernel<2><<<grid, kThreads, 0, s>>>(a);
    else input_nhwc_range_small_kernel<4><<<grid, kThreads, 0, s>>>(a);
    return hipGetLastError();
  }
  const bool vec = vec_loads(g, x);
  // (small layers keep the tile-per-group pass: with fewer than 4096 strips the chip is not full)
  const bool roll = g.m == 2 && vec &&
                    (long long)g.N * g.tw * g.NB * ((g.th + 3) / 4) >= 4096;
  if (roll) {
    // Strips of four tile rows: 10 loads per tile instead of 16.  Longer strips save little more
    // and were slower (measured: a lane has one tile's loads in flight, so a strip is a chain of
    // memory latencies and there must be many strips to overlap them).
    const long long cols = (long long)g.N * g.tw * g.NB;
    int R = 4;
    if (R > g.th) R = g.th;
    a.R = R;
    a.strips = (g.th + R - 1) / R;
    const long long units = cols * a.strips;
    if (units >= (1LL << 30)) return hipErrorInvalidValue;
    a.units = (int)units;
  }
  const int wgs = roll ? (a.units + kGroupsPerWg - 1) / kGroupsPerWg
                       : (a.groups + kGroupsPerWg - 1) / kGroupsPerWg;
  // The workgroups walk the groups with a grid stride: as many as are resident at once (one
  // round, no tail), at most one record each of kMaxRangeGroups.
  // Resident workgroups of each kernel variant on each device: a property of the kernel and the
  // chip, asked for once per device and kept (a cache of a constant: concurrent callers may both
  // ask and store the same value).  [device][m == 4, or 2 for the rolling kernel][vec]
  constexpr int kMaxDevices = 64;
  static std::atomic<int> resident[kMaxDevices][3][2];
  const int which = roll ? 2 : (g.m == 4 ? 1 : 0);
  auto run = [&](auto kern) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::atomic<int>* slot = (dev >= 0 && dev < kMaxDevices) ? &resident[dev][which][vec] : nullptr;
    int res = slot ? slot->load(std::memory_order_relaxed) : 0;
    if (res == 0) {
      int per_cu = 0, cus = 0;
      e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, kThreads, 0);
      if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
      if (e != hipSuccess) return e;
      res = per_cu * cus;
      if (slot) slot->store(res, std::memory_order_relaxed);
    }
    int grid = res;
    if (grid < 1) grid = 1;
    if (grid > kMaxRangeGroups) grid = kMaxRangeGroups;
    if (grid > wgs) grid = wgs;
    *groups_out = grid;
    kern<<<grid, kThreads, 0, s>>>(a);
    return hipGetLastError();
  };
  note_kernel(roll ? "input_nhwc_range_roll_kernel" : "input_nhwc_range_kernel");
  if (roll) return run(input_nhwc_range_roll_kernel<0>);
  if (g.m == 2) return vec ? run(input_nhwc_range_kernel<2, true>) : run(input_nhwc_range_kernel<2, false>);
  return vec ? run(input_nhwc_range_kernel<4, true>) : run(input_nhwc_range_kernel<4, false>);
}

hipError_t launch_input_nhwc_quant(const Geo& g, const float* x, const float* qparams, int8_t* vq,
                                   int32_t* colsum, hipStream_t s) {
  if (!groups_fit(g)) return hipErrorInvalidValue;
  NhArgs a = make_args(g, x);
  a.qparams = qparams; a.vq = vq; a.colsum = colsum;
  const unsigned grid = (unsigned)((a.groups + kGroupsPerWg - 1) / kGroupsPerWg);
  const bool b8 = g.bits == 8, vec = vec_loads(g, x);
#define LANCE_NHWC_QUANT(MM)                                                                 \
  do {                                                                                       \
    if (b8 && vec) input_nhwc_quant_kernel<MM, true, true><<<grid, kThreads, 0, s>>>(a);     \
    else if (b8) input_nhwc_quant_kernel<MM, true, false><<<grid, kThreads, 0, s>>>(a);      \
    else if (vec) input_nhwc_quant_kernel<MM, false, true><<<grid, kThreads, 0, s>>>(a);     \
    else input_nhwc_quant_kernel<MM, false, false><<<grid, kThreads, 0, s>>>(a);             \
  } while (0)
  note_kernel("input_nhwc_quant_kernel");
  if (g.m == 2) LANCE_NHWC_QUANT(2); else LANCE_NHWC_QUANT(4);
#undef LANCE_NHWC_QUANT
  return hipGetLastError();
}

}  // namespace lance
