// Stage 2, second pass for F(2x2,3x3) layers of any channel count: v^ = Q(B^T d B) for every
// input patch (Algorithm 1; Eq. 7), NCHW fp32 in, blocked int8 codes and their column sums out.
// The ranges come from the first pass (input_range.hip) and its reduction.
//
// A workgroup takes 64 consecutive tiles and one block of 64 channels, transforms and quantizes
// them into LDS code rows (quant_phase.h: lane = tile, no pixel staging), then copies the 16
// position planes of 64 rows x 64 bytes to vq with fully coalesced 16-byte stores (the rows of
// consecutive tiles are contiguous in vq).  Each XCD takes a contiguous range of tile blocks.
//
// F(4x4,3x3) layers (36 positions, 6x6 patches) use the same scheme with blocks of 32 tiles: lane
// = (tile, half of the wave's 16-byte chunk), eight channels per lane, two channels' pixels in
// registers at a time.
#include "lance_device.h"
#include "lance_internal.h"
#include "quant_phase.h"
#include "quant_phase32.h"
#include "range_reduce.h"

namespace lance {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

struct QArgs {
  dev::QuantBlockGeo g;
  int8_t* vq;             // [E][NB][P][64]
  int32_t* colsum;        // [E][P]
  dev::RangeSource rs;     // Eq. 7 parameters: finished, or the range pass's records
  int NB, TB;             // channel blocks, tile blocks
  int packed;             // vq is [E][NB][P][32]: two 4-bit codes per byte
};

// Packed form of a 64-byte code row: byte q of the result = (byte q of `lo`, byte q of `hi`) as
// low and high four bits, each the signed code + 8 (for a two's-complement nibble that is one
// bit flip).  lo = chunks 0-1 of the row, hi = chunks 2-3.
__device__ __forceinline__ v4i pack_nibbles(const v4i lo, const v4i hi) {
  v4i r;
#pragma unroll
  for (int d = 0; d < 4; d++) {
    const unsigned l = ((unsigned)lo[d] ^ 0x08080808u) & 0x0F0F0F0Fu;
    const unsigned h = ((unsigned)hi[d] ^ 0x08080808u) & 0x0F0F0F0Fu;
    r[d] = (int)(l | (h << 4));
  }
  return r;
}

template <bool B8, bool FULL, int MODE>
__global__ __launch_bounds__(kThreads, 2) void input_quant_m2_kernel(const QArgs a) {
  constexpr int E = 16, kPlanes = 8;
  extern __shared__ char smem[];
  char* ring = smem;                                          // [kPlanes][64 rows][64 B]
  int* cs_s = reinterpret_cast<int*>(smem + kPlanes * 4096);  // [E][64]
  float* res_s = reinterpret_cast<float*>(cs_s + E * 64);  // [E][2] reduced ranges
  float* qp_s = res_s + 2 * E;                           // [E][2] = {min, inv} of Eq. 7
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // work item = (channel block, tile block); tile blocks of one channel block are consecutive
  const int item = dev::xcd_contiguous(blockIdx.x, gridDim.x);
  const int cb = item / a.TB, tb = item - cb * a.TB;
  const int p0 = tb * 64;
  const int P = a.g.P;

  for (int i = tid; i < E * 64; i += kThreads) cs_s[i] = 0;
  // Eq. 7 parameters under the latency of the first patch loads (the ring is free until the
  // codes are written); its barriers also order the zeroing of the column sums
  auto mid = [&]() {
    dev::ranges_to_lds<E>(a.rs, reinterpret_cast<float*>(ring), res_s, qp_s, tid, item == 0);
  };
  auto qp = [&](int e, float* mn, float* inv) { *mn = qp_s[2 * e]; *inv = qp_s[2 * e + 1]; };
  // copy-out of eight positions at a time (the ring holds eight planes: half the LDS, twice the
  // workgroups per compute unit): thread = (row, chunk) of a plane; 256 threads move one 4 KB
  // plane per pass
  const int row = tid >> 2, chunk = tid & 3;
  auto flush = [&](int e0) {
    __syncthreads();  // the planes are complete
    if (a.packed) {
      if (p0 + row < P && chunk < 2) {  // chunks 0 and 1 take chunks 2 and 3 into their high bits
        const unsigned src = dev::code_row_offset(row, chunk), src2 = dev::code_row_offset(row, chunk + 2);
        int8_t* dst = a.vq + ((size_t)cb * P + p0 + row) * 32 + chunk * 16;
        const size_t plane = (size_t)a.NB * P * 32;
#pragma unroll
        for (int i = 0; i < kPlanes; i++)
          *reinterpret_cast<v4i*>(dst + (size_t)(e0 + i) * plane) =
              pack_nibbles(*reinterpret_cast<const v4i*>(ring + i * 4096 + src),
                           *reinterpret_cast<const v4i*>(ring + i * 4096 + src2));
      }
    } else if (p0 + row < P) {
      const unsigned src = dev::code_row_offset(row, chunk);
      int8_t* dst = a.vq + ((size_t)cb * P + p0 + row) * 64 + chunk * 16;
      const size_t plane = (size_t)a.NB * P * 64;  // bytes per position
      v4i v[kPlanes];
#pragma unroll
      for (int i = 0; i < kPlanes; i++) v[i] = *reinterpret_cast<const v4i*>(ring + i * 4096 + src);
#pragma unroll
      for (int i = 0; i < kPlanes; i++) *reinterpret_cast<v4i*>(dst + (size_t)(e0 + i) * plane) = v[i];
    }
    __syncthreads();  // the planes are free again (and, the last time, the column sums complete)
  };
  dev::quantize_block_to_lds<B8, FULL, MODE, kPlanes>(a.g, p0, cb * 64, ring, cs_s, lane, wave, mid,
                                                      qp, flush);

  // column sums of the signed codes: (sum of the unsigned bytes) - h * (channels of the block)
  const int cbn = min(64, a.g.C - cb * 64);
  const int hsum = cbn * (1 << (a.g.bits - 1));
  for (int i = tid; i < E * 64; i += kThreads) {
    const int e = i >> 6, t = i & 63;
    if (p0 + t < P) {
      const int v = cs_s[i] - hsum;
      if (a.NB > 1)
        atomicAdd(a.colsum + (size_t)e * P + p0 + t, v);
      else
        a.colsum[(size_t)e * P + p0 + t] = v;
    }
  }
}

// The same pass on blocks of 32 tiles (quant_phase32.h: a lane quantizes eight channels of one
// tile) for layers whose 64-tile blocks would leave most of the chip idle: twice the workgroups,
// half the chain of loads and arithmetic in each.
template <bool B8, bool FULL, int MODE>
__global__ __launch_bounds__(kThreads, 2) void input_quant_m2_half_kernel(const QArgs a) {
  constexpr int E = 16, kTiles = 32, kPlane = kTiles * 64;
  extern __shared__ char smem[];
  char* ring = smem;                                          // [E][32 rows][64 B]
  int* cs_s = reinterpret_cast<int*>(smem + E * kPlane);      // [E][32]
  float* res_s = reinterpret_cast<float*>(cs_s + E * kTiles);  // [E][2] reduced ranges
  float* qp_s = res_s + 2 * E;                                 // [E][2] = {min, inv} of Eq. 7
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int item = dev::xcd_contiguous(blockIdx.x, gridDim.x);
  const int cb = item / a.TB, tb = item - cb * a.TB;
  const int p0 = tb * kTiles;
  const int P = a.g.P;

  for (int i = tid; i < E * kTiles; i += kThreads) cs_s[i] = 0;
  auto mid = [&]() {
    dev::ranges_to_lds<E>(a.rs, reinterpret_cast<float*>(ring), res_s, qp_s, tid, item == 0);
  };
  auto qp = [&](int e, float* mn, float* inv) { *mn = qp_s[2 * e]; *inv = qp_s[2 * e + 1]; };
  dev::quantize_half_block_to_lds<B8, FULL, MODE, 3>(a.g, p0, cb * 64, ring, cs_s, lane, wave, mid, qp);
  __syncthreads();

  // copy-out: thread = (plane parity, row, chunk); 256 threads move two 2 KB planes per pass
  const int par = tid >> 7, row = (tid >> 2) & 31, chunk = tid & 3;
  if (a.packed) {
    if (p0 + row < P && chunk < 2) {
      const unsigned src = dev::code_row_offset(row, chunk), src2 = dev::code_row_offset(row, chunk + 2);
      int8_t* dst = a.vq + ((size_t)cb * P + p0 + row) * 32 + chunk * 16;
      const size_t plane = (size_t)a.NB * P * 32;
#pragma unroll
      for (int i = 0; i < E / 2; i++)
        *reinterpret_cast<v4i*>(dst + (size_t)(2 * i + par) * plane) =
            pack_nibbles(*reinterpret_cast<const v4i*>(ring + (2 * i + par) * kPlane + src),
                         *reinterpret_cast<const v4i*>(ring + (2 * i + par) * kPlane + src2));
    }
  } else if (p0 + row < P) {
    const unsigned src = dev::code_row_offset(row, chunk);
    int8_t* dst = a.vq + ((size_t)cb * P + p0 + row) * 64 + chunk * 16;
    const size_t plane = (size_t)a.NB * P * 64;  // bytes per position
    v4i v[E / 2];
#pragma unroll
    for (int i = 0; i < E / 2; i++)
      v[i] = *reinterpret_cast<const v4i*>(ring + (2 * i + par) * kPlane + src);
#pragma unroll
    for (int i = 0; i < E / 2; i++) *reinterpret_cast<v4i*>(dst + (size_t)(2 * i + par) * plane) = v[i];
  }
  // column sums of the signed codes: (sum of the unsigned bytes) - h * (channels of the block)
  const int cbn = min(64, a.g.C - cb * 64);
  const int hsum = cbn * (1 << (a.g.bits - 1));
  for (int i = tid; i < E * kTiles; i += kThreads) {
    const int e = i / kTiles, t = i - e * kTiles;
    if (p0 + t < P) {
      const int v = cs_s[i] - hsum;
      if (a.NB > 1)
        atomicAdd(a.colsum + (size_t)e * P + p0 + t, v);
      else
        a.colsum[(size_t)e * P + p0 + t] = v;
    }
  }
}

// ---- F(4x4,3x3) ----------------------------------------------------------------------------
// Block = 32 consecutive tiles x one 64-channel block.  Wave w owns the 16-byte chunk w of every
// code row; lanes 0..31 own its dwords 0,1, lanes 32..63 its dwords 2,3 (tile = lane % 32), i.e.
// a lane quantizes the channels c_base + 4w + d + 16q with d = 2*(lane/32) + {0,1}, q = 0..3.
// The two lane halves read different channel planes with one buffer descriptor: the upper half
// carries the two planes' distance in its offsets.
template <bool B8, bool FULL, int MODE>
__global__ __launch_bounds__(kThreads, 2) void input_quant_m4_kernel(const QArgs a) {
  typedef int v2i __attribute__((ext_vector_type(2)));
  constexpr int M = 4, A = 6, E = 36, kTiles = 32, kSteps = 8;
  constexpr bool kRows = MODE == 2;
  extern __shared__ char smem[];
  char* ring = smem;                                             // [E][32 rows][64 B]
  int* cs_s = reinterpret_cast<int*>(smem + E * kTiles * 64);    // [E][32]
  float* res_s = reinterpret_cast<float*>(cs_s + E * kTiles);    // [E][2] reduced ranges
  float* qp_s = res_s + 2 * E;                                   // [E][2] = {min, inv} of Eq. 7
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int item = dev::xcd_contiguous(blockIdx.x, gridDim.x);
  const int cb = item / a.TB, tb = item - cb * a.TB;
  const int p0 = tb * kTiles, c_base = cb * 64;
  const dev::QuantBlockGeo& g = a.g;
  const int P = g.P;
  const unsigned HW = (unsigned)g.H * (unsigned)g.W;
  const int trow = lane & 31, hd = lane >> 5;

  for (int i = tid; i < E * kTiles; i += kThreads) cs_s[i] = 0;

  const int pt = min(p0 + trow, P - 1);
  const int tx = pt % g.tw, t2 = pt / g.tw;
  const int ty = t2 % g.th, n = t2 / g.th;
  const int n0 = p0 / (g.th * g.tw);  // image of the block's first tile (wave-uniform)
  dev::PatchLoader<M> pl;
  // the wave's last lane (tile 31, upper half) holds the largest image index, as setup() expects
  pl.setup((unsigned)(n - n0) * (unsigned)g.C * HW, n0, n, g.N, ty, tx, g.pad, g.H, g.W);
  const char* xb = reinterpret_cast<const char*>(g.x + (size_t)n0 * g.C * HW);

  // step k: dword d = 2 hd + k / 4, byte q = k % 4.  chan_lo: the channel of the lower lane half
  // (the descriptor's plane); the upper half is two channels above.
  auto chan_lo = [&](int k) { return c_base + 4 * wave + (k >> 2) + 16 * (k & 3); };
  auto chan_own = [&](int k) { return chan_lo(k) + 2 * hd; };
  // channels beyond C (FULL is false) read the last plane; their bytes are masked below
  const unsigned plane_bytes = HW * 4u;
  auto lane_off = [&](int k) -> unsigned {  // per-lane distance from the descriptor's plane
    if constexpr (FULL) return hd ? 2u * plane_bytes : 0u;
    const int lo = min(chan_lo(k), g.C - 1), own = min(chan_own(k), g.C - 1);
    return (unsigned)(own - lo) * plane_bytes;
  };
  auto plane_lo = [&](int k) { return FULL ? chan_lo(k) : min(chan_lo(k), g.C - 1); };
  auto plane_own = [&](int k) { return FULL ? chan_own(k) : min(chan_own(k), g.C - 1); };
  // first / last plane of the tensor (per lane: the halves differ): shifted row loads
  // With all 64 channels present only the first step can meet the tensor's first plane and only
  // the last step its last one (the channel order of the steps): the other steps carry no test.
  auto may_be_first = [&](int k) { return !FULL || k == 0; };
  auto may_be_last = [&](int k) { return !FULL || k == kSteps - 1; };
  auto is_first = [&](int k) { return may_be_first(k) && pl.first_image && plane_own(k) == 0; };
  auto is_last = [&](int k) { return may_be_last(k) && pl.last_image && plane_own(k) == g.C - 1; };

  float buf[2][E];
  auto issue = [&](int k) {
    const char* plane = xb + (size_t)plane_lo(k) * plane_bytes;
    if constexpr (kRows) {
      pl.issue_rows_shifted(plane, g.reach, is_first(k), is_last(k), buf[k & 1], lane_off(k));
    } else {
      // pixel by pixel: the element loader takes the plane of the lower half; shift the offsets
      dev::PatchLoader<M> pl2 = pl;
      const unsigned lo = lane_off(k);
#pragma unroll
      for (int r = 0; r < A; r++)
        if ((pl2.rowmask >> r) & 1u) pl2.rowoff[r] += lo;
      pl2.template issue<false>(plane, g.reach, buf[k & 1]);
    }
  };
  issue(0);
  // Eq. 7 parameters under the latency of the first patch loads (the ring is free until the
  // codes are written); its barriers also order the zeroing of the column sums
  dev::ranges_to_lds<E>(a.rs, reinterpret_cast<float*>(ring), res_s, qp_s, tid, item == 0);

  float qmn[E], qinv[E];
#pragma unroll
  for (int e = 0; e < E; e++) {
    qmn[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(qp_s[2 * e])));
    qinv[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(qp_s[2 * e + 1])));
  }
  const float L = (float)((1 << g.bits) - 1);
  const unsigned h = 1u << (g.bits - 1);
  const unsigned H8 = 0x80808080u, hh = h * 0x01010101u;

  v2i codes[E];
#pragma unroll
  for (int k = 0; k < kSteps; k++) {
    if (k + 1 < kSteps) issue(k + 1);
    const int q = k & 3, dd = k >> 2;
    float d[A][A];
#pragma unroll
    for (int r = 0; r < A; r++)
#pragma unroll
      for (int c = 0; c < A; c++) d[r][c] = buf[k & 1][r * A + c];
    if constexpr (kRows) {
      if (may_be_first(k) || may_be_last(k)) pl.unshift(is_first(k), is_last(k), d);
      pl.template fix<true>(d);
    }
    dev::input_tile_transform<M>(d);
#pragma unroll
    for (int e = 0; e < E; e++) {
      float tq = (d[e / A][e % A] - qmn[e]) * qinv[e];
      if constexpr (!B8) tq = fminf(tq, L);
      codes[e][dd] = (int)__builtin_amdgcn_cvt_pk_u8_f32(tq, q, q == 0 ? 0u : (unsigned)codes[e][dd]);
    }
    // pin this channel's arithmetic to its step (see quant_phase.h)
#pragma unroll
    for (int e = 0; e < E; e++) asm volatile("" : "+v"(codes[e][dd]));
    __builtin_amdgcn_sched_barrier(0);
  }
  unsigned realmask[2];
#pragma unroll
  for (int dd = 0; dd < 2; dd++) {
    realmask[dd] = 0;
#pragma unroll
    for (int i = 0; i < 4; i++)
      if (c_base + 4 * wave + 2 * hd + dd + 16 * i < g.C) realmask[dd] |= 0xFFu << (8 * i);
  }
  const unsigned l_off = dev::code_row_offset(trow, wave) + 8u * (unsigned)hd;
#pragma unroll
  for (int e = 0; e < E; e++) {
    unsigned cs = 0;
    v2i sg;
#pragma unroll
    for (int dd = 0; dd < 2; dd++) {
      unsigned u = (unsigned)codes[e][dd];
      if constexpr (!FULL) u &= realmask[dd];
      cs = __builtin_amdgcn_sad_u8(u, 0u, cs);
      unsigned v;
      if constexpr (B8)
        v = u ^ H8;
      else
        v = ((u | H8) - (hh & ~H8)) ^ ((u ^ ~hh) & H8);
      if constexpr (!FULL) v &= realmask[dd];
      sg[dd] = (int)v;
    }
    *reinterpret_cast<v2i*>(ring + e * (kTiles * 64) + l_off) = sg;
    atomicAdd(&cs_s[e * kTiles + trow], (int)cs);
  }
  __syncthreads();

  // copy-out: 128 threads move one 2 KB plane; the two halves of the workgroup alternate planes
  {
    const int t7 = tid & 127, row = t7 >> 2, chunk = t7 & 3, half = tid >> 7;
    if (a.packed) {
      if (p0 + row < P && chunk < 2) {  // chunks 0 and 1 take chunks 2 and 3 into their high bits
        const unsigned src = dev::code_row_offset(row, chunk), src2 = dev::code_row_offset(row, chunk + 2);
        int8_t* dst = a.vq + ((size_t)cb * P + p0 + row) * 32 + chunk * 16;
        const size_t plane = (size_t)a.NB * P * 32;
#pragma unroll
        for (int i = 0; i < E / 2; i++)
          *reinterpret_cast<v4i*>(dst + (size_t)(2 * i + half) * plane) =
              pack_nibbles(*reinterpret_cast<const v4i*>(ring + (2 * i + half) * (kTiles * 64) + src),
                           *reinterpret_cast<const v4i*>(ring + (2 * i + half) * (kTiles * 64) + src2));
      }
    } else if (p0 + row < P) {
      const unsigned src = dev::code_row_offset(row, chunk);
      int8_t* dst = a.vq + ((size_t)cb * P + p0 + row) * 64 + chunk * 16;
      const size_t plane = (size_t)a.NB * P * 64;  // bytes per position
      v4i v[E / 2];
#pragma unroll
      for (int i = 0; i < E / 2; i++)
        v[i] = *reinterpret_cast<const v4i*>(ring + (2 * i + half) * (kTiles * 64) + src);
#pragma unroll
      for (int i = 0; i < E / 2; i++)
        *reinterpret_cast<v4i*>(dst + (size_t)(2 * i + half) * plane) = v[i];
    }
  }
  const int cbn = min(64, g.C - cb * 64);
  const int hsum = cbn * (1 << (g.bits - 1));
  for (int i = tid; i < E * kTiles; i += kThreads) {
    const int e = i >> 5, t = i & 31;
    if (p0 + t < P) {
      const int v = cs_s[i] - hsum;
      if (a.NB > 1)
        atomicAdd(a.colsum + (size_t)e * P + p0 + t, v);
      else
        a.colsum[(size_t)e * P + p0 + t] = v;
    }
  }
}

constexpr size_t kLdsBytesM4 =
    36 * 32 * 64 + 36 * 32 * sizeof(int) + dev::range_reduce_lds_floats<36>() * sizeof(float);

constexpr size_t kLdsBytes =
    8 * 4096 + 16 * 64 * sizeof(int) + dev::range_reduce_lds_floats<16>() * sizeof(float);

constexpr size_t kLdsBytesHalf =
    16 * 2048 + 16 * 32 * sizeof(int) + dev::range_reduce_lds_floats<16>() * sizeof(float);

// m: 2, 4, or 1 for F(2x2,3x3) on blocks of 32 tiles
template <bool B8, bool FULL, int MODE>
hipError_t launch_variant(const QArgs& a, unsigned grid, hipStream_t s, int m) {
  const size_t lds = m == 2 ? kLdsBytes : (m == 4 ? kLdsBytesM4 : kLdsBytesHalf);
  auto kern = m == 2 ? input_quant_m2_kernel<B8, FULL, MODE>
                     : (m == 4 ? input_quant_m4_kernel<B8, FULL, MODE>
                               : input_quant_m2_half_kernel<B8, FULL, MODE>);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  note_kernel(m == 2 ? "input_quant_m2_kernel" : (m == 4 ? "input_quant_m4_kernel" : "input_quant_m2_half_kernel"));
  kern<<<grid, kThreads, lds, s>>>(a);
  return hipGetLastError();
}

// Tiles per workgroup: 32 for F(4x4,3x3); for F(2x2,3x3) 64, or 32 when 64-tile blocks would
// give fewer than 192 workgroups (most compute units idle).
int tile_block(const Geo& g) {
  if (g.m == 4) return 32;
  return (long long)g.NB * ((g.P + 63) / 64) < 192 ? 32 : 64;
}

template <bool B8, bool FULL>
hipError_t launch_rows(const Geo& g, const QArgs& a, unsigned grid, hipStream_t s) {
  const int m = (g.m == 2 && tile_block(g) == 32) ? 1 : g.m;
  switch (patch_load_mode(g)) {
    case 0: return launch_variant<B8, FULL, 0>(a, grid, s, m);
    case 1: return launch_variant<B8, FULL, 1>(a, grid, s, m);
    default: return launch_variant<B8, FULL, 2>(a, grid, s, m);
  }
}

long long block_reach_bytes(const Geo& g) {
  const long long tiles = (long long)g.th * g.tw;
  const int block = tile_block(g);
  const long long images = (block - 1) / tiles + 2;  // images a block of consecutive tiles can touch
  // + two channel planes: the upper lane half of the 32-tile kernels reads two channels above
  return images * g.C * g.H * g.W * 4LL + (block == 32 ? 2LL * g.H * g.W * 4LL : 0LL);
}

}  // namespace

// 64-channel code blocks, and byte offsets below 2^31 from the first image of a tile block to
// every pixel it reads.
bool input_quant_applicable(const Geo& g) {
  if (is_nhwc(g)) return false;  // this kernel addresses NCHW tensors
  const int block = tile_block(g);
  return g.CB == 64 && block_reach_bytes(g) < (1LL << 31) &&
         (long long)g.NB * ((g.P + block - 1) / block) < (1LL << 31);
}

// Every workgroup reads all records: worth it while that stays a small part of the pass
// (measured: a gain of 4-6 us per layer up to about 20 MB of record reads, a loss of 2-4 us at 78 MB).
bool input_quant_can_merge(const Geo& g, int count) {
  const int block = tile_block(g);
  const long long grid = (long long)g.NB * ((g.P + block - 1) / block);
  return grid * count * (8LL * g.E) <= (32LL << 20);
}

// colsum must have been cleared when NB > 1 (the range pass does it).
// src: finished Eq. 7 parameters (src.merge == 0), or the records of the range pass / the static
// ranges, from which every workgroup forms the parameters itself and the first one also writes
// v_range and, if asked for, the Eq. 8 constants (src.merge == 1).
hipError_t launch_input_quant(const Geo& g, const float* x, const QuantSource& src, int8_t* vq,
                              int32_t* colsum, hipStream_t s) {
  if (!input_quant_applicable(g)) return hipErrorInvalidValue;
  QArgs a{};
  a.g = dev::QuantBlockGeo{x, g.N, g.C, g.H, g.W, g.pad, g.th, g.tw, g.P, g.bits,
                           (unsigned)block_reach_bytes(g)};
  a.vq = vq; a.colsum = colsum;
  a.rs.qparams = src.qparams; a.rs.partial = src.partial; a.rs.v_range = src.v_range;
  a.rs.u_range = src.dqo ? src.dqo->u_range : nullptr;
  a.rs.dq = src.dqo ? src.dqo->dq : nullptr;
  a.rs.dqd = src.dqo ? src.dqo->dqd : nullptr;
  a.rs.count = src.count; a.rs.merge = src.merge;
  a.rs.is_static = (g.flags & LANCE_INPUT_RANGE_STATIC) ? 1 : 0;
  a.rs.per_tensor = (g.flags & LANCE_RANGE_PER_TENSOR) ? 1 : 0;
  a.rs.bits = g.bits; a.rs.C = g.C; a.rs.bits_w = g.bits_w;
  a.rs.bias = src.dqo ? src.dqo->bias : 0;
  a.packed = is_packed(g) ? 1 : 0;
  const int block = tile_block(g);
  a.NB = g.NB; a.TB = (g.P + block - 1) / block;
  const unsigned grid = (unsigned)(a.NB * a.TB);
  const bool b8 = g.bits == 8, full = g.C % 64 == 0;
  if (b8) return full ? launch_rows<true, true>(g, a, grid, s) : launch_rows<true, false>(g, a, grid, s);
  return full ? launch_rows<false, true>(g, a, grid, s) : launch_rows<false, false>(g, a, grid, s);
}

}  // namespace lance
