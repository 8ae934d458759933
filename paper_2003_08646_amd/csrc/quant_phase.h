// Transform + quantize of one block of 64 tiles x 64 channels of F(2x2,3x3) into LDS:
// v^ = Q(B^T d B) (Algorithm 1; Eq. 7) formed in registers, the signed 8-bit codes written as
// code rows [E][64 tiles][64 B] (the layout the matrix-core fragments read), the column sums of
// the unsigned codes accumulated in LDS.  Used by the one-kernel plan (conv_fused_c64.hip) and by
// the quantize pass that writes the codes to memory (input_quant.hip).
//
// Called by all 256 threads (4 waves) of a workgroup.  Lane = tile, wave w = the 16-byte chunk w
// of every code row, i.e. the channels c_base + 4w+d+16q (d, q = 0..3: dword d of the chunk,
// byte q of the dword -- the blocked code layout the filter codes use).  A lane reads its 4x4
// patch of one channel through per-lane offsets that are computed once (patch_loader.h), kAhead
// channels ahead of the one it transforms.  The four codes of a dword are packed by
// v_cvt_pk_u8_f32 straight into the lane's code registers; after 16 channels the lane owns the
// 16 bytes (tile, chunk w) of all 16 positions: 16 ds_write_b128.  Column sums: v_sad_u8, then
// LDS atomics.  No cross-lane traffic, no LDS staging of pixels.
//
// LDS code rows are 64 bytes; the 16-byte chunk c of row p is stored at chunk
// c ^ row_swizzle(p) (lance_device.h).
#pragma once
#include "lance_device.h"
#include "patch_loader.h"

namespace lance {
namespace dev {

struct QuantBlockGeo {
  const float* x;
  int N, C, H, W, pad, th, tw, P, bits;
  unsigned reach;  // extent of the buffer descriptors (bytes a block's offsets stay below)
};

// Swizzled byte offset of the 16-byte chunk `chunk` of code row `row` inside a 4 KB position plane.
__device__ __forceinline__ unsigned code_row_offset(int row, int chunk) {
  return (unsigned)row * 64u + (unsigned)((chunk ^ row_swizzle(row)) * 16);
}

// B8: 8-bit codes.  FULL: all 64 channels c_base .. c_base+63 exist.  MODE: load mode of the
// patches (patch_load_mode): by rows when it is 2, pixel by pixel otherwise.
// p0: first tile of the block.  ring: [16][64][64 B].  cs_s: [16][64] int, zeroed by the caller
// before its last barrier ahead of this call's end... (the atomics below are the only writers).
// mid(): run once after the first loads have been requested (all threads; may use barriers).
// qp(e, &mn, &inv): the Eq. 7 parameters of position e (wave-uniform), valid after mid().
// PLANES (16 or 8): planes the ring holds.  With 8, position e goes to plane e % 8 and
// flush(first_position) is called after positions 0..7 have been written and again after 8..15
// (all threads; it must empty the planes behind barriers of its own): a pass that only copies the
// codes out needs half the LDS that way.
struct NoFlush {
  __device__ __forceinline__ void operator()(int) const {}
};
template <bool B8, bool FULL, int MODE, int PLANES = 16, class Mid, class Qp, class Flush = NoFlush>
__device__ __forceinline__ void quantize_block_to_lds(const QuantBlockGeo& g, int p0, int c_base,
                                                      char* ring, int* cs_s, int lane, int wave,
                                                      Mid&& mid, Qp&& qp, Flush&& flush = NoFlush()) {
  static_assert(PLANES == 16 || PLANES == 8, "whole or half the positions at a time");
  typedef int v4i __attribute__((ext_vector_type(4)));
  constexpr int M = 2, A = 4, E = 16;
  constexpr int kAhead = 2;  // channels whose loads are in flight ahead of the transform
  constexpr int kBuf = kAhead + 1;
  const unsigned HW = (unsigned)g.H * (unsigned)g.W;
  const int pt = min(p0 + lane, g.P - 1);
  const int tx = pt % g.tw, t2 = pt / g.tw;
  const int ty = t2 % g.th, n = t2 / g.th;
  const int n0 = p0 / (g.th * g.tw);  // image of the block's first tile (wave-uniform)
  PatchLoader<M> pl;
  pl.setup((unsigned)(n - n0) * (unsigned)g.C * HW, n0, n, g.N, ty, tx, g.pad, g.H, g.W);
  const char* xb = reinterpret_cast<const char*>(g.x + (size_t)n0 * g.C * HW);

  // channel of step k: dword d = k / 4, byte q = k % 4
  auto chan = [&](int k) { return c_base + 4 * wave + (k >> 2) + 16 * (k & 3); };
  // channels beyond C (FULL is false) read the last plane; their bytes are masked below
  auto plane_of = [&](int k) { return FULL ? chan(k) : min(chan(k), g.C - 1); };
  // MODE 2: patches are loaded by rows; the first and the last plane of the tensor need the
  // shifted form (patch_loader.h).  With all 64 channels present those can only be step 0 of
  // wave 0 and step 15 of wave 3, so every other step carries no test at all.  Everything here
  // is branch-free: one branch inside the 16 steps would let the compiler sink the arithmetic
  // of all steps below it, with the pixels of all 16 channels held in registers.
  constexpr bool kRows = MODE == 2;
  auto may_be_first = [&](int k) { return !FULL || k == 0; };
  auto may_be_last = [&](int k) { return !FULL || k == 15; };
  auto is_first = [&](int k) { return may_be_first(k) && pl.first_image && plane_of(k) == 0; };
  auto is_last = [&](int k) { return may_be_last(k) && pl.last_image && plane_of(k) == g.C - 1; };
  v4i codes[E];  // codes[e][d] = dword d of this lane's chunk: bytes = channels 4w+d+16q
  float buf[kBuf][E];
  auto issue = [&](int k) {
    const char* plane = xb + (size_t)plane_of(k) * HW * 4;
    if constexpr (!kRows)
      pl.template issue<false>(plane, g.reach, buf[k % kBuf]);
    else if (may_be_first(k) || may_be_last(k))
      pl.issue_rows_shifted(plane, g.reach, is_first(k), is_last(k), buf[k % kBuf]);
    else
      pl.template issue<true>(plane, g.reach, buf[k % kBuf]);
  };
#pragma unroll
  for (int k = 0; k < kAhead; k++) issue(k);

  mid();

  // Eq. 7 parameters as wave-uniform scalars
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

#pragma unroll
  for (int k = 0; k < 16; k++) {
    if (k + kAhead < 16) issue(k + kAhead);
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
      // clamp(rne((x - min) * inv), 0, L): v_cvt_pk_u8_f32 rounds to nearest even and
      // saturates to [0, 255]; only the upper clamp of narrower codes needs an instruction
      float tq = (d[e / A][e % A] - qmn[e]) * qinv[e];
      if constexpr (!B8) tq = fminf(tq, L);
      codes[e][dd] = (int)__builtin_amdgcn_cvt_pk_u8_f32(tq, q, q == 0 ? 0u : (unsigned)codes[e][dd]);
    }
    // Pin this channel's arithmetic here.  Its results are first needed after the last step,
    // and left alone the compiler moves the arithmetic of all 16 steps down there, below all the
    // loads, with the pixels of all channels held in registers (or spilled) meanwhile.
#pragma unroll
    for (int e = 0; e < E; e++) asm volatile("" : "+v"(codes[e][dd]));
    __builtin_amdgcn_sched_barrier(0);
  }
  // column sums of the unsigned codes, then unsigned -> signed; this lane's 16 bytes
  // (row = lane, chunk = wave) of every position go to LDS
  unsigned realmask[4];  // bytes of channels that exist (wave-uniform)
#pragma unroll
  for (int dd = 0; dd < 4; dd++) {
    realmask[dd] = 0;
#pragma unroll
    for (int i = 0; i < 4; i++)
      if (c_base + 4 * wave + dd + 16 * i < g.C) realmask[dd] |= 0xFFu << (8 * i);
  }
  const unsigned l_off = code_row_offset(lane, wave);
#pragma unroll
  for (int e = 0; e < E; e++) {
    unsigned cs = 0;
    v4i sg;
#pragma unroll
    for (int dd = 0; dd < 4; dd++) {
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
    *reinterpret_cast<v4i*>(ring + (e % PLANES) * 4096 + l_off) = sg;
    atomicAdd(&cs_s[e * 64 + lane], (int)cs);
    if (PLANES < E && (e + 1) % PLANES == 0) flush(e + 1 - PLANES);
  }
}

}  // namespace dev
}  // namespace lance
