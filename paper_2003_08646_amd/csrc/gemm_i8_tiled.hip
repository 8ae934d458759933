// Stage 3 alone for 64-channel code blocks: the low-precision products of Algorithm 1 (Sec. 3.3)
// as E integer GEMMs acc[e] = uq[e] . vq[e]^T with int32 accumulation, LDS-tiled.
//
// Without an epilogue to carry, a wave can own a large accumulator tile: 128 filters x 64 tiles
// (4 x 2 matrix tiles of 32 x 32, 128 accumulator registers) in workgroups of 2 x 2 waves = 256 x
// 128, two workgroups per compute unit so that one's barrier waits, fragment reads and final
// stores hide under the other's matrix instructions; or 64 x 64 per wave (128 x 128 per
// workgroup) for small problems.  Per 64-channel block a wave reads 12 KB of fragments from LDS
// for 16 matrix instructions, which leaves the matrix units, not LDS or the path from L2, as
// the limit.
//
// Per block the workgroup's pieces (TK x 64 B of uq, TP x 64 B of vq) are copied into a ring of
// three LDS slots by loads that write LDS directly (lane l's 16 bytes land at base + 16*l, so the
// bank swizzle - chunk c of row r stored at c ^ row_swizzle_mfma32(r) - is applied to the address the
// lane reads from), two blocks ahead; one barrier per block.
//
// Packed 4-bit codes (PK): block rows of 32 bytes, copied in 1 KB pieces of 32 rows in the
// arrangement of packed_codes.h; a fragment is 8 bytes per lane, unpacked to 16 contraction bytes
// and turned back into signed codes in registers (two operations per register), so that acc is
// the exact product of the codes as with 8-bit rows.
#include "lance_device.h"
#include "lance_internal.h"
#include "packed_codes.h"

namespace lance {
namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Four bytes code + 8 (0..15 each) -> the four signed codes: + 120 carries into no neighbour, and
// flipping bit 7 then subtracts 128 modulo 256.
__device__ __forceinline__ int nibbles_to_signed(int x) {
  return (int)(((unsigned)x + 0x78787878u) ^ 0x80808080u);
}
__device__ __forceinline__ v4i packed_fragment(const char* p) {
  v4i r = pk::unpack(*reinterpret_cast<const v2i*>(p));
#pragma unroll
  for (int i = 0; i < 4; i++) r[i] = nibbles_to_signed(r[i]);
  return r;
}

constexpr int kSlots = 3;

struct GbArgs {
  const int8_t* uq;
  const int8_t* vq;
  int32_t* acc;
  int K, P, NB, nkt, npt;
  unsigned uq_bytes, vq_bytes, acc_bytes;
};

// Waits until at most N (< 64) of this wave's vector-memory operations are outstanding and all
// its LDS operations are done, then meets the other waves.  The copies into LDS count as
// vector-memory operations and complete in order; nothing else is in flight in the product loop.
template <int N>
__device__ __forceinline__ void wait_copies_and_barrier() {
  static_assert(N >= 0 && N < 64, "vmcnt field");
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt((N & 15) | 0x70 | ((N >> 4) << 14));  // vmcnt(N) lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// One block's copies of this wave: NC pieces of 1 KB to slot + (NW*j + wave)*1024 (+ 16 bytes per
// lane), NW = waves of the workgroup; the first NA from uq, the others from vq.
template <int NC, int NA, int NW>
__device__ __forceinline__ void copy_block(const int8_t* uq, unsigned uq_bytes, const int8_t* vq,
                                           unsigned vq_bytes, char* slot_wave,
                                           const unsigned (&voff)[NC], unsigned off_u,
                                           unsigned off_v) {
  const __amdgpu_buffer_rsrc_t res_u =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(uq), 0, uq_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t res_v =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(vq), 0, vq_bytes, 0x00020000);
  auto* dst = (__attribute__((address_space(3))) char*)slot_wave;
#pragma unroll
  for (int j = 0; j < NC; j++) {
    if (j < NA)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(res_u, dst + j * (NW * 1024), 16, voff[j], off_u, 0, 0);
    else
      __builtin_amdgcn_raw_ptr_buffer_load_lds(res_v, dst + j * (NW * 1024), 16, voff[j], off_v, 0, 0);
  }
}

// acc registers of one wave -> acc_out.  Register r of matrix tile (i, j) is row
// 32*i + 8*(r/4) + 4*half + r%4, column 32*j + col of the wave's tile.  Rows past K and columns
// past P get an offset the buffer's range check drops.
template <int WK, int WP>
__device__ __forceinline__ void store_acc(int32_t* acc_out, unsigned acc_bytes,
                                          const v16i (&acc)[WK][WP], unsigned row0_bytes,
                                          unsigned lane_bytes, unsigned row_bytes, int rows_left,
                                          int cols_left, int half) {
  const __amdgpu_buffer_rsrc_t res =
      __builtin_amdgcn_make_buffer_rsrc(acc_out, 0, acc_bytes, 0x00020000);
  constexpr unsigned kOob = 0xFFFFFFF0u;
#pragma unroll
  for (int j = 0; j < WP; j++) {
    const unsigned vj = (32 * j < cols_left) ? lane_bytes + 128u * j : kOob;  // lane's column exists
#pragma unroll
    for (int i = 0; i < WK; i++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int row = 32 * i + 8 * (r / 4) + (r % 4);  // + 4*half: part of lane_bytes
        const unsigned v = (row + 4 * half < rows_left) ? vj : kOob;
        __builtin_amdgcn_raw_buffer_store_b32((unsigned)acc[i][j][r], res, v,
                                              row0_bytes + (unsigned)row * row_bytes, 0);
      }
  }
}

// WK x WP matrix tiles per wave, NWK x NWP waves per workgroup; PK: packed 4-bit code rows.
template <int WK, int WP, int NWK, int NWP, bool PK>
__global__ __launch_bounds__(64 * NWK * NWP, 2) void gemm_i8_tiled_kernel(
    const GbArgs a) {
  constexpr int NW = NWK * NWP;
  constexpr int TK = 32 * WK * NWK, TP = 32 * WP * NWP;  // workgroup tile
  constexpr int RB = PK ? pk::kRow : 64;                 // bytes of a block row
  constexpr int kBlockBytes = (TK + TP) * RB;            // one channel block of both pieces
  constexpr int NC = kBlockBytes / (NW * 1024);          // copy instructions per wave and block
  constexpr int NA = TK * RB / (NW * 1024);              // ... of which from uq
  static_assert(NA * NW * 1024 == TK * RB && NC * NW * 1024 == kBlockBytes, "whole instructions");
  extern __shared__ char smem[];                         // [kSlots][kBlockBytes]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = a.K, P = a.P, NB = a.NB;
  // work item = (position, tile column block, filter row block), filter blocks fastest: the
  // workgroups of one die that run together share their vq piece and cycle through uq in L2
  const int item = dev::xcd_contiguous(blockIdx.x, gridDim.x);
  const int kt = item % a.nkt, rest = item / a.nkt;
  const int pt = rest % a.npt, e = rest / a.npt;
  const int k0 = kt * TK, p0 = pt * TP;

  // Copies: instruction j of wave w fills the chunk slots (NW*j + w)*64 .. +63; slot q is row q/4
  // (TK filter rows, then TP tile rows), stored chunk q%4 = the row's chunk (q%4) ^ row_swizzle_mfma32(row).
  // Packed rows: instruction j of wave w fills the 1 KB piece NW*j + w = rows 32*piece .. +31,
  // lane by lane as packed_codes.h lays a piece out.
  unsigned voff[NC];
#pragma unroll
  for (int j = 0; j < NC; j++) {
    int row, c;
    if constexpr (PK) {
      row = (NW * j + wave) * 32 + pk::lane_row(lane);
      c = pk::lane_chunk(lane);
    } else {
      const int q = (NW * j + wave) * 64 + lane;
      row = q >> 2;
      c = (q & 3) ^ dev::row_swizzle_mfma32(row);
    }
    voff[j] = (unsigned)(j < NA ? min(k0 + row, K - 1) : min(p0 + row - TK, P - 1)) * (unsigned)RB +
              (unsigned)c * 16u;
  }
  const unsigned su = (unsigned)K * RB, sv = (unsigned)P * RB;  // bytes between blocks
  unsigned off_u = (unsigned)(e * NB) * su, off_v = (unsigned)(e * NB) * sv;
  const unsigned last_u = off_u + (unsigned)(NB - 1) * su, last_v = off_v + (unsigned)(NB - 1) * sv;
  int slot_w = 0;
  // Copies past the last block re-read it (into a slot nobody reads any more): every step then
  // issues the same number of copies and the waits stay exact.
  auto issue = [&]() {
    copy_block<NC, NA, NW>(a.uq, a.uq_bytes, a.vq, a.vq_bytes,
                       smem + slot_w * kBlockBytes + wave * 1024, voff, off_u, off_v);
    off_u = min(off_u + su, last_u);
    off_v = min(off_v + sv, last_v);
    slot_w = slot_w + 1 == kSlots ? 0 : slot_w + 1;
  };
#pragma unroll
  for (int d = 0; d < kSlots - 1; d++) issue();

  // this wave's WK x WP matrix tiles: fragment addresses inside a slot (k-halves 0 and 1)
  const int kw = wave % NWK, pw = wave / NWK;
  const int col = lane & 31, half = lane >> 5;
  // (packed rows: the two steps are the two 16-byte chunks of the row, each lane half its 8 bytes;
  // both operands meet the same contraction order)
  unsigned fa[WK][2], fb[WP][2];
#pragma unroll
  for (int i = 0; i < WK; i++) {
    const int r = (kw * WK + i) * 32 + col;
    if constexpr (PK) {
      fa[i][0] = (unsigned)(r >> 5) * 1024u + pk::frag_offset(col, 0, half);
      fa[i][1] = (unsigned)(r >> 5) * 1024u + pk::frag_offset(col, 1, half);
    } else {
      fa[i][0] = (unsigned)r * 64u + (unsigned)(((0 + half) ^ dev::row_swizzle_mfma32(r)) * 16);
      fa[i][1] = (unsigned)r * 64u + (unsigned)(((2 + half) ^ dev::row_swizzle_mfma32(r)) * 16);
    }
  }
#pragma unroll
  for (int j = 0; j < WP; j++) {
    const int r = TK + (pw * WP + j) * 32 + col;
    if constexpr (PK) {
      fb[j][0] = (unsigned)(r >> 5) * 1024u + pk::frag_offset(col, 0, half);
      fb[j][1] = (unsigned)(r >> 5) * 1024u + pk::frag_offset(col, 1, half);
    } else {
      fb[j][0] = (unsigned)r * 64u + (unsigned)(((0 + half) ^ dev::row_swizzle_mfma32(r)) * 16);
      fb[j][1] = (unsigned)r * 64u + (unsigned)(((2 + half) ^ dev::row_swizzle_mfma32(r)) * 16);
    }
  }

  v16i acc[WK][WP];
#pragma unroll
  for (int i = 0; i < WK; i++)
#pragma unroll
    for (int j = 0; j < WP; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0;

  int slot_r = 0;
  for (int t = 0; t < NB; t++) {
    // Every thread's copies of block t have landed, and every wave has read block t - 1 (its
    // matrix instructions have been issued): that slot takes block t + kSlots - 1.
    wait_copies_and_barrier<(kSlots - 2) * NC>();
    issue();
    const char* blk = smem + slot_r * kBlockBytes;
    slot_r = slot_r + 1 == kSlots ? 0 : slot_r + 1;
    v4i xa[WK][2], xb[WP][2];
#pragma unroll
    for (int h = 0; h < 2; h++) {
#pragma unroll
      for (int j = 0; j < WP; j++)
        xb[j][h] = PK ? packed_fragment(blk + fb[j][h]) : *reinterpret_cast<const v4i*>(blk + fb[j][h]);
#pragma unroll
      for (int i = 0; i < WK; i++)
        xa[i][h] = PK ? packed_fragment(blk + fa[i][h]) : *reinterpret_cast<const v4i*>(blk + fa[i][h]);
    }
    // all fragment reads of the block are requested before its first matrix instruction (left
    // alone the compiler keeps two fragments in flight to save registers, and every group of
    // matrix instructions then waits for an LDS round trip)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int h = 0; h < 2; h++)
#pragma unroll
      for (int i = 0; i < WK; i++)
#pragma unroll
        for (int j = 0; j < WP; j++)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xa[i][h], xb[j][h], acc[i][j], 0, 0, 0);
  }
  // the copies past the end must have landed before the workgroup's LDS is given away
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0) only
  asm volatile("" ::: "memory");

  const int krow0 = k0 + kw * WK * 32, pcol0 = p0 + pw * WP * 32;
  store_acc<WK, WP>(a.acc, a.acc_bytes, acc,
                    (unsigned)(((size_t)e * K + krow0) * P + pcol0) * 4u,
                    ((unsigned)(4 * half) * (unsigned)P + (unsigned)col) * 4u, (unsigned)P * 4u,
                    K - krow0, P - pcol0 - col, half);
}

}  // namespace

// 64-channel code blocks and 32-bit byte offsets into all three tensors.
bool gemm_i8_tiled_applicable(const Geo& g) {
  const int rb = code_row_bytes(g);
  const long long ub = (long long)g.E * g.NB * g.K * rb, vb = (long long)g.E * g.NB * g.P * rb;
  const long long ab = (long long)g.E * g.K * g.P * 4;
  return g.CB == 64 && ub < (1LL << 32) && vb < (1LL << 32) && ab < 0xFFFFFFF0LL;
}

template <int WK, int WP, int NWK, int NWP, bool PK>
static hipError_t launch_variant(GbArgs a, const Geo& g, hipStream_t s) {
  constexpr int TK = 32 * WK * NWK, TP = 32 * WP * NWP;
  a.nkt = (g.K + TK - 1) / TK;
  a.npt = (g.P + TP - 1) / TP;
  const long long items = (long long)g.E * a.nkt * a.npt;
  if (items >= (1LL << 31)) return hipErrorInvalidValue;
  const size_t lds = (size_t)kSlots * (TK + TP) * (PK ? pk::kRow : 64);
  auto kern = gemm_i8_tiled_kernel<WK, WP, NWK, NWP, PK>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  kern<<<(unsigned)items, 64 * NWK * NWP, lds, s>>>(a);
  return hipGetLastError();
}

hipError_t launch_gemm_i8_tiled(const Geo& g, const int8_t* uq, const int8_t* vq, int32_t* acc,
                                hipStream_t s) {
  if (!gemm_i8_tiled_applicable(g)) return hipErrorInvalidValue;
  const size_t rb = (size_t)code_row_bytes(g);
  GbArgs a{uq, vq, acc, g.K, g.P, g.NB, 0, 0, (unsigned)((size_t)g.E * g.NB * g.K * rb),
           (unsigned)((size_t)g.E * g.NB * g.P * rb), (unsigned)((size_t)g.E * g.K * g.P * 4)};
  // 256 x 128 tiles when they still fill the chip twice (two workgroups per compute unit)
  const long long big = (long long)g.E * ((g.K + 255) / 256) * ((g.P + 127) / 128);
  if (is_packed(g))
    return big >= 1024 ? launch_variant<4, 2, 2, 2, true>(a, g, s)
                       : launch_variant<2, 2, 2, 2, true>(a, g, s);
  return big >= 1024 ? launch_variant<4, 2, 2, 2, false>(a, g, s)
                     : launch_variant<2, 2, 2, 2, false>(a, g, s);
}

}  // namespace lance
