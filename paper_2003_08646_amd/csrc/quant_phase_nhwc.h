// Transform + quantize of one block of TILES tiles x NBLK 64-channel blocks of F(2x2,3x3) into
// LDS from NHWC pixels: v^ = Q(B^T d B) (Algorithm 1; Eq. 7) formed in registers, the signed 8-bit
// codes written as code rows [NBLK][E][TILES][64 B] with the channels in their natural order (the
// order of the filter codes of an NHWC layer), the column sums of the unsigned codes left in LDS.
// The NHWC counterpart of quant_phase.h / quant_phase32.h, used by the one-kernel plans
// (conv_fused_c64.hip: 64 tiles x 1 block; conv_fused_c128.hip: 32 tiles x 2 blocks).
//
// Called by all 256 threads of a workgroup.  16 * NBLK lanes per tile: lane j holds the channels
// 4j .. 4j+3 (one 16-byte load per pixel of the 4x4 window; C is a multiple of 4), a thread
// group takes four tiles one after the other; the window of the next tile is requested before
// the current one is transformed.  The lane's four codes of a position are one dword of the
// code row; the column sum is a 16-lane DPP sum (added to LDS with an atomic when a tile has
// two blocks).
//
// LDS code rows are 64 bytes; the 16-byte chunk c of row p is stored at chunk c ^ row_swizzle(p)
// (what the fragment reads of the product phase expect).
#pragma once
#include "lance_device.h"
#include "nhwc_window.h"
#include "quant_phase.h"

namespace lance {
namespace dev {

// B8: 8-bit codes.  p0: first tile of the block.  ring: [NBLK][16][TILES][64 B].  cs_s:
// [16][TILES] int: every entry written here (NBLK = 1), or added to (NBLK = 2: zeroed by the caller
// before a barrier inside mid()).  mid(): run once after the first loads have been requested (all
// threads; may use barriers).  qp(e, &mn, &inv): the Eq. 7 parameters of position e, valid
// after mid().  Uses g.x as [N][H][W][C] (16-byte aligned), g.reach = its size in bytes.
template <bool B8, int TILES, int NBLK, class Mid, class Qp>
__device__ __forceinline__ void quantize_block_nhwc_to_lds(const QuantBlockGeo& g, int p0,
                                                           char* ring, int* cs_s, int tid,
                                                           Mid&& mid, Qp&& qp) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  constexpr int M = 2, A = 4, E = 16;
  constexpr int kLanes = 16 * NBLK, kGroups = 256 / kLanes, kItems = TILES / kGroups;
  static_assert(kItems * kGroups == TILES, "tiles split evenly over the thread groups");
  constexpr unsigned kPlane = TILES * 64u, kBlock = E * kPlane;
  const int j = tid % kLanes, grp = tid / kLanes;
  const int jj = j & 15, blk = j >> 4;  // dword of the code row, channel block
  const bool lane_real = 4 * j < g.C;            // C is a multiple of 4: all four or none
  const int c0 = min(4 * j, g.C - 4);            // a real quad for the loads of padding lanes
  auto load = [&](int it, f4 (&w)[A * A]) {
    const int pt = min(p0 + kGroups * it + grp, g.P - 1);
    const int tx = pt % g.tw, t2 = pt / g.tw;
    const int ty = t2 % g.th, n = t2 / g.th;
    load_window_nhwc<M>(g.x, g.reach, n, ty * M - g.pad, tx * M - g.pad, c0, g.H, g.W, g.C, w);
  };
  f4 win[2][A * A];
  load(0, win[0]);

  mid();
  __syncthreads();  // mid() may still read scratch inside the ring after its last barrier

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
  const unsigned realmask = lane_real ? 0xFFFFFFFFu : 0u;

#pragma unroll
  for (int it = 0; it < kItems; it++) {
    if (it + 1 < kItems) load(it + 1, win[(it + 1) & 1]);
    const int t = kGroups * it + grp;  // code row of this item
    unsigned pk[E];               // unsigned codes of Eq. 7, byte i = channel 4j + i
#pragma unroll
    for (int e = 0; e < E; e++) pk[e] = 0;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      float d[A][A];
#pragma unroll
      for (int r = 0; r < A; r++)
#pragma unroll
        for (int s = 0; s < A; s++) d[r][s] = win[it & 1][r * A + s][i];
      input_tile_transform<M>(d);
#pragma unroll
      for (int e = 0; e < E; e++) {
        // clamp(rne((x - min) * inv), 0, L): v_cvt_pk_u8_f32 rounds to nearest even and
        // saturates to [0, 255]; only the upper clamp of narrower codes needs an instruction
        float tq = (d[e / A][e % A] - qmn[e]) * qinv[e];
        if constexpr (!B8) tq = fminf(tq, L);
        pk[e] = __builtin_amdgcn_cvt_pk_u8_f32(tq, i, pk[e]);
      }
    }
    char* row = ring + (unsigned)blk * kBlock + (unsigned)t * 64u +
                (unsigned)(((jj >> 2) ^ row_swizzle(t)) * 16 + (jj & 3) * 4);
#pragma unroll
    for (int e = 0; e < E; e++) {
      const unsigned u = pk[e] & realmask;
      const int tot = row16_sum((int)__builtin_amdgcn_sad_u8(u, 0u, 0u));
      // per-byte (code - h) mod 256 without borrows between bytes (h = 128: flip the top bit)
      unsigned v;
      if constexpr (B8)
        v = u ^ H8;
      else
        v = ((u | H8) - (hh & ~H8)) ^ ((u ^ ~hh) & H8);
      *reinterpret_cast<unsigned*>(row + e * kPlane) = v & realmask;
      if (jj == 0) {
        if constexpr (NBLK == 1) cs_s[e * TILES + t] = tot;
        else atomicAdd(&cs_s[e * TILES + t], tot);
      }
    }
    // keep this tile's arithmetic here: left alone the compiler interleaves all four tiles and
    // holds their windows at once
    __builtin_amdgcn_sched_barrier(0);
  }
}

}  // namespace dev
}  // namespace lance
