// Stages 3+4 fused for F(2x2,3x3) layers with several 64-channel blocks (C > 64): the int8
// products of Algorithm 1 (Sec. 3.3), the de-quantization (Eq. 8) and the output transform
// (Eq. 9) applied to the register accumulators.
//
// For such layers the product is a real dense contraction (E GEMMs of K x P x C).  A workgroup
// of four waves owns 64 filters x 32 tiles.  The 16 positions form a 4 x 4 grid (i, j) and
// S = A^T M A = sum_i A^T[.][i] (sum_j M[i][j] A^T[.][j]): wave i owns grid row i, all channels.
// It needs only the two row sums R_i[b] = sum_j A^T[b][j] s_e ACC_e per element (half the
// registers of the four outputs), and the four waves work independently - no barrier in the
// product loop, four times the waves of a layout that gives every wave all positions - until
// the end, where the row sums are exchanged through LDS and each wave finishes and stores a
// quarter of the workgroup's outputs.
//
// A wave walks its 4*NB blocks (block = (position, channel block), position-major; in both code
// tensors consecutive blocks are a constant stride apart: [E][NB][rows][64]).  Each block's
// 64 x 64 B piece of uq and 32 x 64 B piece of vq are copied into a wave-private ring of three
// LDS slots by loads that write LDS directly (no registers, no LDS store instructions), two
// blocks ahead of the block whose matrix-instruction fragments are being read.  LDS is a
// prefetch buffer here: pieces are shared between workgroups through L2, not between waves.
// LDS rows are 64 bytes with the 16-byte chunk c of row r stored at c ^ row_swizzle_mfma32(r)
// (lance_device.h).
//
// Epilogue algebra (as in gemm_i8.hip): M[e,k,p] = s_e*ACC + f[e,k] + g[e,p]; the three terms go
// through the linear map S = A^T M A separately.  f is formed here from the filter row sums, in
// binary64; g is formed from the column sums.
#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kTileK = 64, kTileP = 32;
constexpr int kBlockBytes = (kTileK + kTileP) * 64;  // one channel block of both pieces: 6 KB
constexpr int kCopies = kBlockBytes / 1024;          // copy instructions per block (1 KB each)
constexpr int kSlots = 3;                            // ring slots per wave (deeper rings measured no faster)
constexpr int kWaveRing = kSlots * kBlockBytes;      // 18 KB
constexpr int kRingBytes = 4 * kWaveRing;            // 72 KB; the exchange reuses 64 KB of it

struct GrArgs {
  const int8_t* uq;
  const int8_t* vq;
  const int32_t* colsum;
  const float* dq;          // [E][4]
  const double* dqd;        // [E][2] = {su*ov, C*ou*ov}
  const int32_t* u_rowsum;  // [E][K]
  float* y;
  int K, P, NB, th, tw, Ho, Wo;
  int nky;  // filter tiles
  unsigned uq_bytes, vq_bytes, y_bytes;
  int nhwc;  // Y is [N][Ho][Wo][K]
};

// Waits until at most N (< 64) of this wave's vector-memory operations are outstanding.  The
// copies into LDS count as vector-memory operations and complete in order; nothing else is in
// flight in the product loop.  The compiler's own builtin, so that its bookkeeping stays exact;
// the empty statements keep memory accesses on their side.
template <int N>
__device__ __forceinline__ void wait_copies() {
  static_assert(N >= 0 && N < 64, "vmcnt field");
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt((N & 15) | 0x0F70 | ((N >> 4) << 14));  // vmcnt(N) only
  asm volatile("" ::: "memory");
}

// One block's copies of this wave: kCopies pieces of 1 KB to slot + j*1024 (+ 16 bytes per
// lane): the first four from uq, the last two from vq.  voff: the lane's byte offsets within a
// block; off_u / off_v: the block's offsets (wave-uniform).
__device__ __forceinline__ void copy_block(const int8_t* uq, unsigned uq_bytes, const int8_t* vq,
                                           unsigned vq_bytes, char* slot,
                                           const unsigned (&voff)[kCopies], unsigned off_u,
                                           unsigned off_v) {
  const __amdgpu_buffer_rsrc_t res_u =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(uq), 0, uq_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t res_v =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(vq), 0, vq_bytes, 0x00020000);
  auto* dst = (__attribute__((address_space(3))) char*)slot;
#pragma unroll
  for (int j = 0; j < kCopies; j++) {
    if (j < kTileK / 16)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(res_u, dst + j * 1024, 16, voff[j], off_u, 0, 0);
    else
      __builtin_amdgcn_raw_ptr_buffer_load_lds(res_v, dst + j * 1024, 16, voff[j], off_v, 0, 0);
  }
}

// The tail's stores: out[t][q][aa] = the two pixels of row aa of the 2x2 patch of filter
// 32*t + q (counted from the lane's first filter), at base + (32*t + q)*plane_bytes +
// aa*row_bytes.  kleft: filters that exist from the lane's first one on.  even_w (kernel-uniform):
// the output width is even, so a patch never loses its second column and the pair is stored
// as one 8-byte store.
__device__ __forceinline__ void store_patches(float* y, unsigned y_bytes, const v4f (&out)[2][4][2],
                                              unsigned base, unsigned plane_bytes,
                                              unsigned row_bytes, int kleft, bool tile_ok,
                                              bool row1, bool col1, bool even_w, unsigned oob) {
  const __amdgpu_buffer_rsrc_t res = __builtin_amdgcn_make_buffer_rsrc(y, 0, y_bytes, 0x00020000);
  typedef unsigned v2u __attribute__((ext_vector_type(2)));
  unsigned off[2][4][2];  // [t][q][aa]
#pragma unroll
  for (int t = 0; t < 2; t++)
#pragma unroll
    for (int q = 0; q < 4; q++) {
      const bool k_ok = tile_ok && (32 * t + q) < kleft;
#pragma unroll
      for (int aa = 0; aa < 2; aa++)
        off[t][q][aa] = (k_ok && (aa == 0 || row1)) ? base + (unsigned)aa * row_bytes : oob;
    }
  if (even_w) {
#pragma unroll
    for (int t = 0; t < 2; t++)
#pragma unroll
      for (int q = 0; q < 4; q++)
#pragma unroll
        for (int aa = 0; aa < 2; aa++) {
          const v2u v = {__float_as_uint(out[t][q][aa][0]), __float_as_uint(out[t][q][aa][1])};
          __builtin_amdgcn_raw_buffer_store_b64(v, res, off[t][q][aa],
                                                (unsigned)(32 * t + q) * plane_bytes, 0);
        }
  } else {
#pragma unroll
    for (int t = 0; t < 2; t++)
#pragma unroll
      for (int q = 0; q < 4; q++)
#pragma unroll
        for (int aa = 0; aa < 2; aa++) {
          const unsigned so = (unsigned)(32 * t + q) * plane_bytes;  // wave-uniform
          __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(out[t][q][aa][0]), res,
                                                off[t][q][aa], so, 0);
          __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(out[t][q][aa][1]), res,
                                                col1 ? off[t][q][aa] + 4u : oob, so, 0);
        }
  }
}

__global__ __launch_bounds__(kThreads, 2) void gemm_fused_rows_kernel(const GrArgs a) {
  constexpr int M = 2, A = 4, E = 16;
  extern __shared__ char smem[];
  float* rk_s = reinterpret_cast<float*>(smem + kRingBytes);  // [kTileK][M*M]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // = grid row i of this wave
  const int K = a.K, P = a.P, NB = a.NB;
  // work item = (tile block, filter tile), the filter tiles of a tile block next to each other
  // on one die so that they share the block's codes in its L2
  const int item = dev::xcd_contiguous(blockIdx.x, gridDim.x);
  const int tb = item / a.nky, ky = item - tb * a.nky;
  const int k0w = ky * kTileK, p0w = tb * kTileP;
  char* ring = smem + wave * kWaveRing;

  // Copies.  A block's piece is 384 chunks of 16 bytes; copy instruction j fills the 64
  // consecutive chunk slots starting at 64*j, lane l the slot of its own number (that is how a
  // load into LDS places its data).  Slot q is row q/4 (64 filter rows, then 32 tile rows),
  // stored chunk q%4, and holds the row's chunk (q%4) ^ row_swizzle_mfma32(row): the swizzle is applied
  // to the address the lane reads from.  Rows past K or P re-read the last row.  A lane's
  // offsets within a block never change; the block offsets advance in scalar registers.
  unsigned voff[kCopies];
#pragma unroll
  for (int j = 0; j < kCopies; j++) {
    const int q = 64 * j + lane;
    const int row = q >> 2, c = (q & 3) ^ dev::row_swizzle_mfma32(row);
    voff[j] = (unsigned)(row < kTileK ? min(k0w + row, K - 1) : min(p0w + row - kTileK, P - 1)) * 64u +
              (unsigned)c * 16u;
  }
  const unsigned su = (unsigned)K * 64u, sv = (unsigned)P * 64u;  // bytes between blocks
  const int T = A * NB;                                           // this wave's blocks, >= 8
  // Copies past the wave's last block re-read it (into a slot nobody reads any more): every
  // step then issues the same number of copies and the waits below stay exact.
  unsigned off_u = (unsigned)(wave * T) * su, off_v = (unsigned)(wave * T) * sv;
  const unsigned last_u = off_u + (unsigned)(T - 1) * su, last_v = off_v + (unsigned)(T - 1) * sv;
  int slot_w = 0;  // ring slot of the next copy
  auto issue = [&]() {  // the next block -> the next ring slot
    copy_block(a.uq, a.uq_bytes, a.vq, a.vq_bytes, ring + slot_w * kBlockBytes, voff, off_u, off_v);
    off_u = min(off_u + su, last_u);
    off_v = min(off_v + sv, last_v);
    slot_w = slot_w + 1 == kSlots ? 0 : slot_w + 1;
  };
#pragma unroll
  for (int d = 0; d < kSlots - 1; d++) issue();  // blocks 0 .. kSlots-2 (T >= 8)

  // filter-side terms f[e,k] = su*ov*rowsum[e][k] + C*ou*ov through A^T . A, in binary64:
  // thread = (filter = lane, output ab = wave), so that all four waves enter the product loop
  // together
  {
    const int k = min(k0w + lane, K - 1);
    const int aa = wave >> 1, b = wave & 1;
    double accd = 0.0;
#pragma unroll
    for (int e2 = 0; e2 < E; e2++) {
      // A^T = [1 1 1 0; 0 1 -1 -1]: coefficient of position (i, j) for output (aa, b)
      const int i = e2 / A, j = e2 % A;
      const double ci = aa == 0 ? (i < 3 ? 1.0 : 0.0) : (i == 0 ? 0.0 : (i == 1 ? 1.0 : -1.0));
      const double cj = b == 0 ? (j < 3 ? 1.0 : 0.0) : (j == 0 ? 0.0 : (j == 1 ? 1.0 : -1.0));
      const double f = a.dqd[2 * e2] * (double)a.u_rowsum[(size_t)e2 * K + k] + a.dqd[2 * e2 + 1];
      accd += (ci * cj) * f;
    }
    rk_s[4 * lane + wave] = (float)accd;
  }

  // this lane's tile (column of the matrix tiles) and its input-side term through A^T . A
  const int col = lane & 31, half = lane >> 5;
  const int p = min(p0w + col, P - 1);
  float gp[M][M];
#pragma unroll
  for (int aa = 0; aa < M; aa++)
#pragma unroll
    for (int b = 0; b < M; b++) gp[aa][b] = 0.0f;
#pragma unroll
  for (int e2 = 0; e2 < E; e2++) {
    const float g = a.dq[4 * e2 + 1] * (float)a.colsum[(size_t)e2 * P + p];
#pragma unroll
    for (int aa = 0; aa < M; aa++)
#pragma unroll
      for (int b = 0; b < M; b++) {
        const float coef = dev::Wino<M>::at(aa, e2 / A) * dev::Wino<M>::at(b, e2 % A);
        if (coef != 0.0f) gp[aa][b] = __builtin_fmaf(coef, g, gp[aa][b]);
      }
  }
  // the scales s_e of this wave's four positions (wave-uniform)
  float sj[A];
#pragma unroll
  for (int j = 0; j < A; j++) {
    const float s = a.dq[4 * (wave * A + j)];
    sj[j] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(s)));
  }

  // fragment addresses within a slot: two filter tiles of 32 rows, one tile of 32 tile rows
  unsigned fa[2][2], fb[2];
#pragma unroll
  for (int t = 0; t < 2; t++) {
    const int r = t * 32 + col;
    fa[t][0] = (unsigned)r * 64u + (unsigned)(((0 + half) ^ dev::row_swizzle_mfma32(r)) * 16);
    fa[t][1] = (unsigned)r * 64u + (unsigned)(((2 + half) ^ dev::row_swizzle_mfma32(r)) * 16);
  }
  fb[0] = (unsigned)(kTileK + col) * 64u + (unsigned)(((0 + half) ^ dev::row_swizzle_mfma32(col)) * 16);
  fb[1] = (unsigned)(kTileK + col) * 64u + (unsigned)(((2 + half) ^ dev::row_swizzle_mfma32(col)) * 16);

  float rowacc[M][2][16];  // R_i[b] of the two filter tiles
#pragma unroll
  for (int b = 0; b < M; b++)
#pragma unroll
    for (int t = 0; t < 2; t++)
#pragma unroll
      for (int r = 0; r < 16; r++) rowacc[b][t][r] = 0.0f;

  // One block.  All earlier fragment reads are complete (the matrix instructions consumed
  // them; the explicit wait states it), so the slot of the previous block is free: it takes
  // the block kSlots - 1 ahead.  Then wait until this block has landed (the copies of the
  // kSlots - 1 blocks after it may stay in flight), read its fragments, multiply.
  int slot_r = 0;
  auto block = [&](v16i (&acc)[2], bool first) {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0) only
    asm volatile("" ::: "memory");
    issue();
    wait_copies<(kSlots - 1) * kCopies>();
    const char* blk = ring + slot_r * kBlockBytes;
    slot_r = slot_r + 1 == kSlots ? 0 : slot_r + 1;
    v4i xa[2][2], xb[2];
#pragma unroll
    for (int h = 0; h < 2; h++) {
      xb[h] = *reinterpret_cast<const v4i*>(blk + fb[h]);
#pragma unroll
      for (int t = 0; t < 2; t++) xa[t][h] = *reinterpret_cast<const v4i*>(blk + fa[t][h]);
    }
    if (first) {  // the accumulators start from zero
      const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int t = 0; t < 2; t++)
        acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xa[t][0], xb[0], zero, 0, 0, 0);
    } else {
#pragma unroll
      for (int t = 0; t < 2; t++)
        acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xa[t][0], xb[0], acc[t], 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < 2; t++)
      acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(xa[t][1], xb[1], acc[t], 0, 0, 0);
  };
  // Positions (i, j = 0..3): R_i[b] += A^T[b][j] * s_e * ACC with A^T = [1 1 1 0; 0 1 -1 -1].
#pragma unroll
  for (int j = 0; j < A; j++) {
    v16i acc[2];
    block(acc, true);
#pragma nounroll
    for (int cb = 1; cb < NB; cb++) block(acc, false);
    const float s = sj[j];
#pragma unroll
    for (int b = 0; b < M; b++) {
      const float coef = dev::Wino<M>::at(b, j);  // compile-time
      if (coef != 0.0f) {
        const float c = coef * s;
#pragma unroll
        for (int t = 0; t < 2; t++)
#pragma unroll
          for (int r = 0; r < 16; r++)
            rowacc[b][t][r] = __builtin_fmaf(c, (float)acc[t][r], rowacc[b][t][r]);
      }
    }
  }
  wait_copies<0>();  // the copies past the end must not land on the exchange area

  // ---- exchange: every wave leaves its row sums in LDS (the rings are done with) -------------
  // chunk ((i*2 + b)*2 + t)*4 + rq holds, lane by lane, R_i[b] of tile t, registers 4rq .. 4rq+3
  __syncthreads();
  v4f* xch = reinterpret_cast<v4f*>(smem);
#pragma unroll
  for (int b = 0; b < M; b++)
#pragma unroll
    for (int t = 0; t < 2; t++)
#pragma unroll
      for (int rq = 0; rq < 4; rq++) {
        v4f v;
#pragma unroll
        for (int q = 0; q < 4; q++) v[q] = rowacc[b][t][4 * rq + q];
        xch[(((wave * 2 + b) * 2 + t) * 4 + rq) * 64 + lane] = v;
      }
  __syncthreads();

  // ---- tail: this wave finishes registers 4*wave .. 4*wave+3 of both tiles: S[a][b] =
  // sum_i A^T[a][i] R_i[b], plus the two separable terms; stores the 2x2 patches.  Stores that
  // must not happen (tiles past P, filters past K, the second row or column of a patch cut by
  // an odd output size) get an offset beyond the buffer instead of a branch. ----
  {
    const int pt = p0w + col;
    const int pc = min(pt, P - 1);
    const int tx = pc % a.tw, t2 = pc / a.tw;
    const int ty = t2 % a.th, n = t2 / a.th;
    const unsigned Wo = (unsigned)a.Wo, plane = (unsigned)a.Ho * Wo;
    const bool row1 = ty * M + 1 < a.Ho, col1 = tx * M + 1 < a.Wo;  // row 0 / column 0 always exist
    const unsigned kOob = 0xFFFFFFF0u;
    // byte offset of the patch's first pixel in the plane of this lane's first filter
    const unsigned base = (((unsigned)n * (unsigned)K + (unsigned)(k0w + 4 * half + 8 * wave)) * plane +
                           (unsigned)(ty * M) * Wo + (unsigned)(tx * M)) * 4u;
    const int kleft = K - (k0w + 4 * half + 8 * wave);  // filters from the lane's first one on
    v4f out[2][4][M];  // [t][q][aa] = {o(aa,0), o(aa,1)} in [0], [1]
#pragma unroll
    for (int t = 0; t < 2; t++) {
      v4f s4[M][M];  // [a][b], four filters each
#pragma unroll
      for (int b = 0; b < M; b++) {
        v4f x[A];
#pragma unroll
        for (int i = 0; i < A; i++) x[i] = xch[(((i * 2 + b) * 2 + t) * 4 + wave) * 64 + lane];
        s4[0][b] = (x[0] + x[1]) + x[2];
        s4[1][b] = (x[1] - x[2]) - x[3];
      }
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const v4f f4 = *reinterpret_cast<const v4f*>(rk_s + 4 * (t * 32 + 4 * half + 8 * wave + q));
#pragma unroll
        for (int aa = 0; aa < M; aa++) {
          out[t][q][aa][0] = (s4[aa][0][q] + f4[aa * M + 0]) + gp[aa][0];
          out[t][q][aa][1] = (s4[aa][1][q] + f4[aa * M + 1]) + gp[aa][1];
        }
      }
    }
    if (a.nhwc) {
      // the lane's filters come in groups of four consecutive ones: one store per group and pixel
      const bool k4 = (K & 3) == 0;
#pragma unroll
      for (int aa = 0; aa < M; aa++)
#pragma unroll
        for (int b = 0; b < M; b++) {
          const int oy = ty * M + aa, ox = tx * M + b;
          const bool pix_ok = pt < P && oy < a.Ho && ox < a.Wo;
          const unsigned pix = (((unsigned)n * (unsigned)a.Ho + (unsigned)oy) * Wo + (unsigned)ox) *
                               (unsigned)K * 4u;
#pragma unroll
          for (int t = 0; t < 2; t++)
            dev::store_nhwc_k4(a.y, a.y_bytes, pix, (unsigned)(K - kleft + 32 * t) * 4u, pix_ok,
                               kleft - 32 * t, k4, out[t][0][aa][b], out[t][1][aa][b],
                               out[t][2][aa][b], out[t][3][aa][b]);
        }
      return;
    }
    store_patches(a.y, a.y_bytes, out, base, plane * 4u, Wo * 4u, kleft, pt < P, row1, col1,
                  (a.Wo & 1) == 0, kOob);
  }
}

constexpr size_t kLdsBytes = kRingBytes + 2 * 2 * kTileK * sizeof(float);

}  // namespace

// For layers with too few tiles for the 128 x 64 workgroup tiles of gemm_fused_tiled.hip (which
// share their pieces between waves and win as soon as they fill half the chip), up to kMaxItems
// workgroups; the copies and the stores address the code tensors and Y with 32-bit byte offsets.
constexpr long long kMaxItems = 2048;
bool gemm_fused_rows_applicable(const Geo& g) {
  const long long items = (long long)((g.P + kTileP - 1) / kTileP) * ((g.K + kTileK - 1) / kTileK);
  const long long ub = (long long)g.E * g.NB * g.K * 64, vb = (long long)g.E * g.NB * g.P * 64;
  const long long yb = (long long)g.N * g.K * g.Ho * g.Wo * 4;
  return g.m == 2 && g.CB == 64 && g.NB >= 2 && items <= kMaxItems &&
         !(g.flags & LANCE_PLAN_WIDE_TILES) && !gemm_fused_stream_m2_preferred(g) &&
         ub < (1LL << 32) && vb < (1LL << 32) && yb < 0xFFFFFFF0LL;
}

hipError_t launch_gemm_fused_rows(const Geo& g, const int8_t* uq, const int8_t* vq,
                                   const int32_t* colsum, const float* dq, const double* dqd,
                                   const int32_t* u_rowsum, float* y, hipStream_t s) {
  if (!gemm_fused_rows_applicable(g)) return hipErrorInvalidValue;
  GrArgs a{uq, vq, colsum, dq, dqd, u_rowsum, y, g.K, g.P, g.NB, g.th, g.tw, g.Ho, g.Wo,
           (g.K + kTileK - 1) / kTileK,
           (unsigned)((size_t)g.E * g.NB * g.K * 64), (unsigned)((size_t)g.E * g.NB * g.P * 64),
           (unsigned)((size_t)g.N * g.K * g.Ho * g.Wo * 4), is_nhwc(g) ? 1 : 0};
  const unsigned grid = (unsigned)(((g.P + kTileP - 1) / kTileP) * a.nky);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_fused_rows_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes);
  if (e != hipSuccess) return e;
  note_kernel("gemm_fused_rows_kernel");
  gemm_fused_rows_kernel<<<grid, kThreads, kLdsBytes, s>>>(a);
  return hipGetLastError();
}

}  // namespace lance
