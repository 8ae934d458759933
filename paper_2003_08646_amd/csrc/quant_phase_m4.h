// Transform + quantize of one block of 16 tiles x 64 channels of F(4x4,3x3) into LDS, for kernels
// that keep the codes of V on chip: v^ = Q(B^T d B) (Algorithm 1; Eq. 7) formed in registers, the
// signed 8-bit codes written as code rows [36][16 tiles][64 B], the column sums of the unsigned
// codes accumulated in LDS.
//
// Called by all 256 threads (4 waves) of a workgroup.  Wave w owns the 16-byte chunk w of every
// code row and lane = (tile = lane % 16, dword hd = lane / 16 of that chunk): a lane quantizes
// the four channels c_base + 4w + hd + 16q, q = 0..3 (byte q of its dword; the blocked channel
// order of the code layout), one channel's 6x6 patch in registers while the next one's loads are
// in flight.  The four lane groups read four different channel planes with one buffer
// descriptor: a group carries its plane's distance from the first one in its offsets.  After its
// four channels a lane owns one dword of all 36 positions: 36 ds_write_b32.  Column sums:
// v_sad_u8, then LDS atomics.
//
// LDS code rows are 64 bytes; the 16-byte chunk c of row p is stored at chunk c ^ row_swizzle(p)
// (quant_phase.h).
#pragma once
#include "lance_device.h"
#include "patch_loader.h"
#include "quant_phase.h"

namespace lance {
namespace dev {

// B8: 8-bit codes.  FULL: all 64 channels c_base .. c_base+63 exist.  MODE: load mode of the
// patches (patch_load_mode): by rows when it is 2, pixel by pixel otherwise.
// p0: first tile of the block.  planes: [36][16][64 B].  cs_s: [36][16] int, zeroed by the caller
// before a barrier that precedes the first atomic below (mid() contains one).
// mid(): run once after the first loads have been requested (all threads; may use barriers);
// after it qp_s[2e], qp_s[2e+1] = {min, inv} of Eq. 7 for position e.
// g.reach must cover three channel planes beyond the block's images (the lane groups' planes).
template <bool B8, bool FULL, int MODE, class Mid>
__device__ __forceinline__ void quantize_m4_block16_to_lds(const QuantBlockGeo& g, int p0,
                                                           int c_base, char* planes, int* cs_s,
                                                           const float* qp_s, int lane, int wave,
                                                           Mid&& mid) {
  constexpr int M = 4, A = 6, E = 36, kTiles = 16, kSteps = 4, kPlane = kTiles * 64;
  constexpr bool kRows = MODE == 2;
  const int P = g.P;
  const unsigned HW = (unsigned)g.H * (unsigned)g.W;
  const int trow = lane & 15, hd = lane >> 4;

  const int pt = min(p0 + trow, P - 1);
  const int tx = pt % g.tw, t2 = pt / g.tw;
  const int ty = t2 % g.th, n = t2 / g.th;
  const int n0 = p0 / (g.th * g.tw);  // image of the block's first tile (wave-uniform)
  PatchLoader<M> pl;
  // the wave's last lane (tile 15 of the block) holds the largest image index, as setup() expects
  pl.setup((unsigned)(n - n0) * (unsigned)g.C * HW, n0, n, g.N, ty, tx, g.pad, g.H, g.W);
  const char* xb = reinterpret_cast<const char*>(g.x + (size_t)n0 * g.C * HW);

  // step k = byte k of the lane's dword.  chan_lo: the channel of lane group 0 (the descriptor's
  // plane); group hd is hd channels above.
  auto chan_lo = [&](int k) { return c_base + 4 * wave + 16 * k; };
  auto chan_own = [&](int k) { return chan_lo(k) + hd; };
  // channels beyond C (FULL is false) read the last plane; their bytes are masked below
  const unsigned plane_bytes = HW * 4u;
  auto lane_off = [&](int k) -> unsigned {  // per-lane distance from the descriptor's plane
    if constexpr (FULL) return (unsigned)hd * plane_bytes;
    const int lo = min(chan_lo(k), g.C - 1), own = min(chan_own(k), g.C - 1);
    return (unsigned)(own - lo) * plane_bytes;
  };
  auto plane_lo = [&](int k) { return FULL ? chan_lo(k) : min(chan_lo(k), g.C - 1); };
  auto plane_own = [&](int k) { return FULL ? chan_own(k) : min(chan_own(k), g.C - 1); };
  // first / last plane of the tensor (per lane: the groups differ): shifted row loads
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
      // pixel by pixel: the element loader takes the plane of group 0; shift the offsets
      PatchLoader<M> pl2 = pl;
      const unsigned lo = lane_off(k);
#pragma unroll
      for (int r = 0; r < A; r++)
        if ((pl2.rowmask >> r) & 1u) pl2.rowoff[r] += lo;
      pl2.template issue<false>(plane, g.reach, buf[k & 1]);
    }
  };
  issue(0);
  mid();

  float qmn[E], qinv[E];
#pragma unroll
  for (int e = 0; e < E; e++) {
    qmn[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(qp_s[2 * e])));
    qinv[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(qp_s[2 * e + 1])));
  }
  const float L = (float)((1 << g.bits) - 1);
  const unsigned h = 1u << (g.bits - 1);
  const unsigned H8 = 0x80808080u, hh = h * 0x01010101u;

  unsigned codes[E];
#pragma unroll
  for (int k = 0; k < kSteps; k++) {
    if (k + 1 < kSteps) issue(k + 1);
    float d[A][A];
#pragma unroll
    for (int r = 0; r < A; r++)
#pragma unroll
      for (int c = 0; c < A; c++) d[r][c] = buf[k & 1][r * A + c];
    if constexpr (kRows) {
      if (may_be_first(k) || may_be_last(k)) pl.unshift(is_first(k), is_last(k), d);
      pl.template fix<true>(d);
    }
    input_tile_transform<M>(d);
#pragma unroll
    for (int e = 0; e < E; e++) {
      float tq = (d[e / A][e % A] - qmn[e]) * qinv[e];
      if constexpr (!B8) tq = fminf(tq, L);
      codes[e] = __builtin_amdgcn_cvt_pk_u8_f32(tq, k, k == 0 ? 0u : codes[e]);
    }
    // pin this channel's arithmetic to its step (see quant_phase.h)
#pragma unroll
    for (int e = 0; e < E; e++) asm volatile("" : "+v"(codes[e]));
    __builtin_amdgcn_sched_barrier(0);
  }
  unsigned realmask = 0;
#pragma unroll
  for (int i = 0; i < 4; i++)
    if (c_base + 4 * wave + hd + 16 * i < g.C) realmask |= 0xFFu << (8 * i);
  const unsigned l_off = code_row_offset(trow, wave) + 4u * (unsigned)hd;
#pragma unroll
  for (int e = 0; e < E; e++) {
    unsigned u = codes[e];
    if constexpr (!FULL) u &= realmask;
    const unsigned cs = __builtin_amdgcn_sad_u8(u, 0u, 0u);
    unsigned v;
    if constexpr (B8)
      v = u ^ H8;
    else
      v = ((u | H8) - (hh & ~H8)) ^ ((u ^ ~hh) & H8);
    if constexpr (!FULL) v &= realmask;
    *reinterpret_cast<unsigned*>(planes + e * kPlane + l_off) = v;
    atomicAdd(&cs_s[e * kTiles + trow], (int)cs);
  }
}

}  // namespace dev
}  // namespace lance
