// Transform + quantize of one block of 32 tiles x 64 channels of F(2x2,3x3) into LDS: the variant
// of quant_phase.h for workgroups that own 32 tiles (half the LDS per channel block, so that two
// workgroups with two channel blocks each share a compute unit).  v^ = Q(B^T d B) (Algorithm 1;
// Eq. 7) formed in registers, the signed 8-bit codes written as code rows [E][32 tiles][64 B], the
// column sums of the unsigned codes accumulated in LDS.
//
// Called by all 256 threads (4 waves) of a workgroup.  Wave w owns the 16-byte chunk w of every
// code row; lanes 0..31 own its dwords 0,1, lanes 32..63 its dwords 2,3 (tile = lane % 32), i.e. a
// lane quantizes the channels c_base + 4w + d + 16q with d = 2*(lane/32) + {0,1}, q = 0..3: eight
// channels, two channels' pixels in registers at a time.  The two lane halves read different
// channel planes with one buffer descriptor: the upper half carries the two planes' distance in
// its offsets.  After its eight channels a lane owns 8 bytes (tile, chunk w, its half) of all 16
// positions: 16 ds_write_b64.  Column sums: v_sad_u8, then LDS atomics.
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
// p0: first tile of the block.  ring: [16][32][64 B].  cs_s: [16][32] int, zeroed by the caller
// before a barrier that precedes the first atomic below (mid() contains one).
// mid(): run once after the first loads have been requested (all threads; may use barriers).
// qp(e, &mn, &inv): the Eq. 7 parameters of position e (wave-uniform), valid after mid().
// AHEAD: channels whose loads are in flight ahead of the one being transformed (16 registers each).
template <bool B8, bool FULL, int MODE, int AHEAD, class Mid, class Qp>
__device__ __forceinline__ void quantize_half_block_to_lds(const QuantBlockGeo& g, int p0,
                                                           int c_base, char* ring, int* cs_s,
                                                           int lane, int wave, Mid&& mid, Qp&& qp) {
  typedef int v2i __attribute__((ext_vector_type(2)));
  constexpr int M = 2, A = 4, E = 16, kTiles = 32, kSteps = 8, kBuf = AHEAD + 1;
  constexpr bool kRows = MODE == 2;
  const int P = g.P;
  const unsigned HW = (unsigned)g.H * (unsigned)g.W;
  const int trow = lane & 31, hd = lane >> 5;

  const int pt = min(p0 + trow, P - 1);
  const int tx = pt % g.tw, t2 = pt / g.tw;
  const int ty = t2 % g.th, n = t2 / g.th;
  const int n0 = p0 / (g.th * g.tw);  // image of the block's first tile (wave-uniform)
  PatchLoader<M> pl;
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

  float buf[kBuf][E];
  auto issue = [&](int k) {
    const char* plane = xb + (size_t)plane_lo(k) * plane_bytes;
    if constexpr (kRows) {
      pl.issue_rows_shifted(plane, g.reach, is_first(k), is_last(k), buf[k % kBuf], lane_off(k));
    } else {
      // pixel by pixel: the element loader takes the plane of the lower half; shift the offsets
      PatchLoader<M> pl2 = pl;
      const unsigned lo = lane_off(k);
#pragma unroll
      for (int r = 0; r < A; r++)
        if ((pl2.rowmask >> r) & 1u) pl2.rowoff[r] += lo;
      pl2.template issue<false>(plane, g.reach, buf[k % kBuf]);
    }
  };
#pragma unroll
  for (int k = 0; k < AHEAD; k++) issue(k);

  mid();

  float qmn[E], qinv[E];
#pragma unroll
  for (int e = 0; e < E; e++) {
    float mn, inv;
    qp(e, &mn, &inv);
    qmn[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(mn)));
    qinv[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(inv)));
  }
  const float L = (float)((1 << g.bits) - 1);
  const unsigned h = 1u << (g.bits - 1);
  const unsigned H8 = 0x80808080u, hh = h * 0x01010101u;

  v2i codes[E];
#pragma unroll
  for (int k = 0; k < kSteps; k++) {
    if (k + AHEAD < kSteps) issue(k + AHEAD);
    const int q = k & 3, dd = k >> 2;
    float d[A][A];
#pragma unroll
    for (int r = 0; r < A; r++)
#pragma unroll
      for (int c = 0; c < A; c++) d[r][c] = buf[k % kBuf][r * A + c];
    if constexpr (kRows) {
      if (may_be_first(k) || may_be_last(k)) pl.unshift(is_first(k), is_last(k), d);
      pl.template fix<true>(d);
    }
    input_tile_transform<M>(d);
#pragma unroll
    for (int e = 0; e < E; e++) {
      // clamp(rne((x - min) * inv), 0, L): v_cvt_pk_u8_f32 rounds to nearest even and saturates
      // to [0, 255]; only the upper clamp of narrower codes needs an instruction
      float tq = (d[e / A][e % A] - qmn[e]) * qinv[e];
      if constexpr (!B8) tq = fminf(tq, L);
      codes[e][dd] = (int)__builtin_amdgcn_cvt_pk_u8_f32(tq, q, q == 0 ? 0u : (unsigned)codes[e][dd]);
    }
    // pin this channel's arithmetic to its step (see quant_phase.h)
#pragma unroll
    for (int e = 0; e < E; e++) asm volatile("" : "+v"(codes[e][dd]));
    __builtin_amdgcn_sched_barrier(0);
  }
  unsigned realmask[2];  // bytes of channels that exist
#pragma unroll
  for (int dd = 0; dd < 2; dd++) {
    realmask[dd] = 0;
#pragma unroll
    for (int i = 0; i < 4; i++)
      if (c_base + 4 * wave + 2 * hd + dd + 16 * i < g.C) realmask[dd] |= 0xFFu << (8 * i);
  }
  const unsigned l_off = code_row_offset(trow, wave) + 8u * (unsigned)hd;
#pragma unroll
  for (int e = 0; e < E; e++) {
    unsigned cs = 0;
    v2i sg;
#pragma unroll
    for (int dd = 0; dd < 2; dd++) {
      unsigned u = (unsigned)codes[e][dd];
      if constexpr (!FULL) u &= realmask[dd];
      cs = __builtin_amdgcn_sad_u8(u, 0u, cs);
      // per-byte (code - h) mod 256 without borrows between bytes (h = 128: flip the top bit)
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
}

}  // namespace dev
}  // namespace lance
