// Stages 3+4 fused for F(2x2,3x3) layers with several 64-channel blocks (C > 64): the int8
// products of Algorithm 1 (Sec. 3.3) with both operands staged through LDS, the de-quantization
// (Eq. 8) and the output transform (Eq. 9) applied to the register accumulators.
//
// For such layers the product is a real dense contraction (E GEMMs of K x P x C) and what limits
// a kernel that reads its fragments from memory is the number of vector-memory instructions per
// matrix instruction.  Here a workgroup of eight waves owns 128 filters x 64 tiles (one
// 32 x 32 x 32 accumulator tile per wave); the pieces of uq (128 x 64 B per channel block) and vq
// (64 x 64 B) go through LDS and every wave reads its four fragments from there, and each piece
// of vq is fetched by K/128 workgroups instead of K/64.
//
// The pieces go from memory straight into LDS (buffer loads that write LDS: no registers, no LDS
// store instructions) through a ring of 72 KB: steps of two channel blocks (24 KB) with two
// steps in flight ahead of the one being multiplied when NB is even, steps of one block with
// five ahead when it is odd.  (A first version kept two 16-byte loads per thread two stages
// ahead in registers and waited for memory at every stage.)  The blocks of all positions are a
// constant stride apart in both code tensors ([E][NB][rows][64]), so a step is simply the next
// blocks.  One barrier per step.
// LDS rows are 64 bytes with the 16-byte chunk c of row r stored at c ^ row_swizzle_mfma32(r)
// (lance_device.h).
//
// Epilogue algebra (as in gemm_i8.hip): M[e,k,p] = s_e*ACC + f[e,k] + g[e,p]; the three terms go
// through the linear map S = A^T M A separately.  The first is accumulated position by position;
// the 16 positions are unrolled, so the coefficients A^T[a][i] A^T[b][j] s_e are +-s_e or absent
// at compile time.  f is formed here from the filter row sums (binary64), g from the column
// sums.
#include "lance_device.h"
#include "lance_internal.h"
#include "packed_codes.h"
#include <utility>

namespace lance {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 512;
constexpr int kTileK = 128, kTileP = 64;
constexpr int kBlockBytes = (kTileK + kTileP) * 64;  // one channel block of both pieces: 12 KB

struct GtArgs {
  const int8_t* uq;
  const int8_t* vq;
  const int32_t* colsum;
  const float* dq;          // [E][4]
  const double* dqd;        // [E][2] = {su*ov, C*ou*ov}
  const int32_t* u_rowsum;  // [E][K]
  float* y;
  int K, P, NB, th, tw, Ho, Wo;
  int nky;  // filter tiles (ceil(K / 128))
  unsigned y_bytes;
  int nhwc;  // Y is [N][Ho][Wo][K]
};

// The tail's stores: o[r][aa] = the two pixels of row aa of the 2x2 patch of filter
// 8*(r/4) + r%4 (counted from the lane's first filter), at base + filter*plane_bytes +
// aa*row_bytes.  kleft: filters that exist from the lane's first one on.  even_w (kernel-uniform):
// the output width is even, so a patch never loses its second column and the pair is stored as
// one 8-byte store.  Masked stores get an offset the buffer's range check drops.
__device__ __forceinline__ void store_patches(float* y, unsigned y_bytes, const float (&o)[16][2][2],
                                              unsigned base, unsigned plane_bytes,
                                              unsigned row_bytes, int kleft, bool tile_ok,
                                              bool row1, bool col1, bool even_w) {
  const __amdgpu_buffer_rsrc_t res = __builtin_amdgcn_make_buffer_rsrc(y, 0, y_bytes, 0x00020000);
  typedef unsigned v2u __attribute__((ext_vector_type(2)));
  constexpr unsigned kOob = 0xFFFFFFF0u;
  if (even_w) {
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int kk = 8 * (r / 4) + (r % 4);
      const bool k_ok = tile_ok && kk < kleft;
#pragma unroll
      for (int aa = 0; aa < 2; aa++) {
        const unsigned off = (k_ok && (aa == 0 || row1)) ? base + (unsigned)aa * row_bytes : kOob;
        const v2u v = {__float_as_uint(o[r][aa][0]), __float_as_uint(o[r][aa][1])};
        __builtin_amdgcn_raw_buffer_store_b64(v, res, off, (unsigned)kk * plane_bytes, 0);
      }
    }
  } else {
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int kk = 8 * (r / 4) + (r % 4);
      const bool k_ok = tile_ok && kk < kleft;
#pragma unroll
      for (int aa = 0; aa < 2; aa++) {
        const unsigned off = (k_ok && (aa == 0 || row1)) ? base + (unsigned)aa * row_bytes : kOob;
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o[r][aa][0]), res, off,
                                              (unsigned)kk * plane_bytes, 0);
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o[r][aa][1]), res,
                                              col1 ? off + 4u : kOob, (unsigned)kk * plane_bytes, 0);
      }
    }
  }
}

typedef float v16f __attribute__((ext_vector_type(16)));

template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{})
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// A^T of F(2x2,3x3) (points 0, 1, -1, inf), for compile-time indices.
constexpr float kAt2[2][4] = {{1, 1, 1, 0}, {0, 1, -1, -1}};

struct GsArgs {
  GtArgs g;
  unsigned uq_bytes, vq_bytes;
};
// This wave's copies of one step of SB channel blocks, 1 KB each (lane l = row l/4, stored chunk
// l%4): the uq rows 16*wave .. 16*wave+15 of every block, and the vq rows 16*(wave%4) .. of block
// wave/4 (SB = 2) or of the one block (SB = 1: the upper four waves copy what the lower four
// copy, so that every wave has the same number of copies in flight).
template <int SB>
__device__ __forceinline__ void m2_copy_step(const int8_t* uq, unsigned uq_bytes, const int8_t* vq,
                                             unsigned vq_bytes, char* slot, int wave,
                                             const unsigned (&voff)[3], unsigned off_u,
                                             unsigned off_v) {
  const __amdgpu_buffer_rsrc_t res_u =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(uq), 0, uq_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t res_v =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(vq), 0, vq_bytes, 0x00020000);
#pragma unroll
  for (int j = 0; j < SB; j++) {
    auto* dst = (__attribute__((address_space(3))) char*)(slot + j * kBlockBytes + wave * 1024);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(res_u, dst, 16, voff[j], off_u, 0, 0);
  }
  auto* dst = (__attribute__((address_space(3))) char*)(slot + (SB == 2 ? wave >> 2 : 0) * kBlockBytes +
                                                        kTileK * 64 + (wave & 3) * 1024);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(res_v, dst, 16, voff[2], off_v, 0, 0);
}

// At most N of this wave's copies outstanding, all its LDS reads done; then the other waves.
template <int N>
__device__ __forceinline__ void m2_wait_and_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt((N & 15) | 0x70 | ((N >> 4) << 14));  // vmcnt(N) lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Position e is complete: out[ab] += A^T[a][i] A^T[b][j] s_e ACC (coefficients +-1 or 0).
// bias2: what every integer sum carries beyond the product of the stored codes (0, or
// 64 * Cp for packed codes, which are multiplied as code + 8).
template <int e>
__device__ __forceinline__ void m2_fold(const v16i& acc, const float* sc_s, v16f (&out)[4],
                                        const int bias2 = 0) {
  constexpr int A = 4, gi = e / A, gj = e % A;
  // The outputs are first read in the tail, in another basic block: left alone the compiler
  // sinks the folds of all positions down there and keeps every position's accumulators until
  // then.  The empty statements tie them to their position.
  __builtin_amdgcn_sched_barrier(0);
  const float se = sc_s[e];
  v16f accf;
#pragma unroll
  for (int r = 0; r < 16; r++) accf[r] = (float)(acc[r] - bias2);
  static_for<4>([&](auto abc) {
    constexpr int ab = decltype(abc)::value;
    constexpr float coef = kAt2[ab >> 1][gi] * kAt2[ab & 1][gj];
    if constexpr (coef != 0.0f) {
      const float c = coef * se;
#pragma unroll
      for (int r = 0; r < 16; r++) out[ab][r] = __builtin_fmaf(c, accf[r], out[ab][r]);
      asm volatile("" : "+v"(out[ab]));
    }
  });
  __builtin_amdgcn_sched_barrier(0);
}

// Filter-side terms f[e,k] = su*ov*rowsum[e][k] + C*ou*ov through A^T . A, in binary64, for the
// workgroup's 128 filters (thread = (ab, filter): ab is wave-uniform) into rk_s[128][4], and the
// scales s_e into sc_s[16].  Called by all 512 threads; visible after the next barrier.
__device__ __forceinline__ void m2_filter_terms(const GtArgs& a, float* rk_s, float* sc_s, int tid,
                                                int wave, int k0w) {
  constexpr int M = 2, A = 4, E = 16;
  const int K = a.K;
  {
    const int ab = wave >> 1, kk = tid & (kTileK - 1);
    const int k = min(k0w + kk, K - 1);
    double accd = 0.0;
#pragma unroll
    for (int e2 = 0; e2 < E; e2++) {
      const double coef =
          (double)dev::at_coef(M, ab >> 1, e2 / A) * (double)dev::at_coef(M, ab & 1, e2 % A);
      accd += coef * (a.dqd[2 * e2] * (double)a.u_rowsum[(size_t)e2 * K + k] + a.dqd[2 * e2 + 1]);
    }
    rk_s[4 * kk + ab] = (float)accd;
  }
  if (tid < E) sc_s[tid] = a.dq[4 * tid];
}

// Tail of a workgroup: adds the two separable terms of the expanded Eq. 8 to the folded products
// and stores the 2x2 patches.  Stores that must not happen (tiles past P, filters past K, the
// second row or column of a patch cut by an odd output size) get an offset beyond the buffer
// instead of a branch.  kw, half, brow_l: the lane's place in its wave's 32 x 32 tile.
__device__ __forceinline__ void m2_tail(const GtArgs& a, const v16f (&out)[4], const float* rk_s,
                                        int kw, int half, int brow_l, int k0w, int p0w) {
  constexpr int M = 2, A = 4, E = 16;
  const int K = a.K, P = a.P;
    typedef float v4f __attribute__((ext_vector_type(4)));
    const int p = p0w + brow_l;
    const int pc = min(p, P - 1);
    float gp[M][M];  // input-side term of this lane's tile through A^T . A
#pragma unroll
    for (int aa = 0; aa < M; aa++)
#pragma unroll
      for (int b = 0; b < M; b++) gp[aa][b] = 0.0f;
#pragma unroll
    for (int e2 = 0; e2 < E; e2++) {
      const float g = a.dq[4 * e2 + 1] * (float)a.colsum[(size_t)e2 * P + pc];
#pragma unroll
      for (int aa = 0; aa < M; aa++)
#pragma unroll
        for (int b = 0; b < M; b++) {
          const float coef = dev::Wino<M>::at(aa, e2 / A) * dev::Wino<M>::at(b, e2 % A);
          if (coef != 0.0f) gp[aa][b] = __builtin_fmaf(coef, g, gp[aa][b]);
        }
    }
    const int tx = pc % a.tw, t2 = pc / a.tw;
    const int ty = t2 % a.th, n = t2 / a.th;
    const int kfirst = k0w + kw * 32 + 4 * half;  // this lane's first filter
    float o[16][M][M];
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int kk = 8 * (r / 4) + (r % 4);
      const v4f f4 = *reinterpret_cast<const v4f*>(rk_s + 4 * (kw * 32 + 4 * half + kk));
#pragma unroll
      for (int aa = 0; aa < M; aa++)
#pragma unroll
        for (int b = 0; b < M; b++) o[r][aa][b] = (out[aa * M + b][r] + f4[aa * M + b]) + gp[aa][b];
    }
    if (a.nhwc) {
      // the lane's filters come in groups of four consecutive ones: one store per group and pixel
      const bool k4 = (K & 3) == 0;
#pragma unroll
      for (int aa = 0; aa < M; aa++)
#pragma unroll
        for (int b = 0; b < M; b++) {
          const int oy = ty * M + aa, ox = tx * M + b;
          const bool pix_ok = p < P && oy < a.Ho && ox < a.Wo;
          const unsigned pix = (((unsigned)n * (unsigned)a.Ho + (unsigned)oy) * (unsigned)a.Wo +
                                (unsigned)ox) * (unsigned)K * 4u;
#pragma unroll
          for (int rq = 0; rq < 4; rq++)
            dev::store_nhwc_k4(a.y, a.y_bytes, pix, (unsigned)(kfirst + 8 * rq) * 4u, pix_ok,
                               K - (kfirst + 8 * rq), k4, o[4 * rq][aa][b], o[4 * rq + 1][aa][b],
                               o[4 * rq + 2][aa][b], o[4 * rq + 3][aa][b]);
        }
      return;
    }
    const unsigned Wo_u = (unsigned)a.Wo, plane = (unsigned)a.Ho * Wo_u;
    const unsigned base = (((unsigned)n * (unsigned)K + (unsigned)kfirst) * plane +
                           (unsigned)(ty * M) * Wo_u + (unsigned)(tx * M)) * 4u;
    store_patches(a.y, a.y_bytes, o, base, plane * 4u, Wo_u * 4u, K - kfirst, p < P,
                  ty * M + 1 < a.Ho, tx * M + 1 < a.Wo, (a.Wo & 1) == 0);
}

// SB: channel blocks per step (2: NB even; 1: NB odd).  NBT: NB if a variant is compiled for it
// (then no loop is left in the product phase), else 0.
template <int SB, int NBT>
__global__ __launch_bounds__(kThreads, 4) void gemm_fused_m2_stream_kernel(const GsArgs as) {
  constexpr int M = 2, E = 16;
  constexpr int kStepBytes = SB * kBlockBytes;
  constexpr int kRing = SB == 2 ? 3 : 6;  // slots of the ring (72 KB)
  constexpr int kCopies = SB + 1;         // copies per wave and step
  const GtArgs& a = as.g;
  extern __shared__ char smem[];
  char* ring = smem;                                                  // [kRing][kStepBytes]
  float* rk_s = reinterpret_cast<float*>(smem + kRing * kStepBytes);  // [128 filters][M*M]
  float* sc_s = rk_s + M * M * kTileK;                                // [E] s_e

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = a.K, P = a.P;
  const int NB = NBT > 0 ? NBT : a.NB;
  const int item = dev::xcd_contiguous(blockIdx.x, gridDim.x);
  const int tb = item / a.nky, ky = item - tb * a.nky;
  const int k0w = ky * kTileK, p0w = tb * kTileP;

  // lane offsets of the copies inside a step (block stride included)
  const unsigned su = (unsigned)K * 64u, sv = (unsigned)P * 64u;  // bytes between blocks
  unsigned voff[3];
  {
    const int r16 = lane >> 2, cpos = lane & 3;
    const int rowu = 16 * wave + r16;
    const unsigned vu = (unsigned)min(k0w + rowu, K - 1) * 64u +
                        (unsigned)((cpos ^ dev::row_swizzle_mfma32(rowu)) * 16);
    voff[0] = vu;
    voff[1] = su + vu;
    const int rowv = 16 * (wave & 3) + r16;
    voff[2] = (SB == 2 ? (unsigned)(wave >> 2) * sv : 0u) + (unsigned)min(p0w + rowv, P - 1) * 64u +
              (unsigned)((cpos ^ dev::row_swizzle_mfma32(rowv)) * 16);
  }
  const int steps = E * NB / SB;
  unsigned off_u = 0, off_v = 0;
  const unsigned last_u = (unsigned)(steps - 1) * SB * su, last_v = (unsigned)(steps - 1) * SB * sv;
  int slot_w = 0, slot_r = 0;
  // Copies past the last step read it again (into a slot nobody reads any more): every step
  // issues the same number of copies and the waits stay exact.
  auto issue = [&]() {
    m2_copy_step<SB>(a.uq, as.uq_bytes, a.vq, as.vq_bytes, ring + slot_w * kStepBytes, wave, voff,
                     off_u, off_v);
    off_u = min(off_u + SB * su, last_u);
    off_v = min(off_v + SB * sv, last_v);
    slot_w = slot_w + 1 == kRing ? 0 : slot_w + 1;
  };
#pragma unroll
  for (int d = 0; d < kRing - 1; d++) issue();

  m2_filter_terms(a, rk_s, sc_s, tid, wave, k0w);

  // this wave's 32 x 32 tile
  const int kw = wave & 3, pw = wave >> 2;
  const int col = lane & 31, half = lane >> 5;
  const int arow_l = kw * 32 + col, brow_l = pw * 32 + col;
  const unsigned fa0 = (unsigned)arow_l * 64u + (unsigned)(((0 + half) ^ dev::row_swizzle_mfma32(arow_l)) * 16);
  const unsigned fa1 = (unsigned)arow_l * 64u + (unsigned)(((2 + half) ^ dev::row_swizzle_mfma32(arow_l)) * 16);
  const unsigned fb0 =
      (unsigned)(kTileK + brow_l) * 64u + (unsigned)(((0 + half) ^ dev::row_swizzle_mfma32(brow_l)) * 16);
  const unsigned fb1 =
      (unsigned)(kTileK + brow_l) * 64u + (unsigned)(((2 + half) ^ dev::row_swizzle_mfma32(brow_l)) * 16);

  v16f out[M * M];
#pragma unroll
  for (int ab = 0; ab < M * M; ab++)
#pragma unroll
    for (int r = 0; r < 16; r++) out[ab][r] = 0.0f;
  v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

  auto step = [&]() {
    // This wave's copies of this step have landed and so have, after the barrier, everybody's
    // (rk_s and sc_s too, the first time); every wave has read the step before, whose slot
    // takes the step kRing - 1 ahead.
    m2_wait_and_barrier<(kRing - 2) * kCopies>();
    issue();
    const char* blk = ring + slot_r * kStepBytes;
    slot_r = slot_r + 1 == kRing ? 0 : slot_r + 1;
    v4i fa[SB][2], fb[SB][2];
#pragma unroll
    for (int i = 0; i < SB; i++) {
      fa[i][0] = *reinterpret_cast<const v4i*>(blk + i * kBlockBytes + fa0);
      fb[i][0] = *reinterpret_cast<const v4i*>(blk + i * kBlockBytes + fb0);
      fa[i][1] = *reinterpret_cast<const v4i*>(blk + i * kBlockBytes + fa1);
      fb[i][1] = *reinterpret_cast<const v4i*>(blk + i * kBlockBytes + fb1);
    }
#pragma unroll
    for (int i = 0; i < SB; i++) {
      acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i][0], fb[i][0], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i][1], fb[i][1], acc, 0, 0, 0);
    }
  };
  static_for<E>([&](auto ec) {
    constexpr int e = decltype(ec)::value;
    if constexpr (NBT > 0) {
#pragma unroll
      for (int i = 0; i < NBT / SB; i++) step();
    } else {
      for (int i = 0; i < NB / SB; i++) step();
    }
    m2_fold<e>(acc, sc_s, out);
#pragma unroll
    for (int r = 0; r < 16; r++) acc[r] = 0;
  });
  // the copies past the end are still in flight: they must have landed before the workgroup
  // ends (its LDS is handed to the next one)
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)

  m2_tail(a, out, rk_s, kw, half, brow_l, k0w, p0w);
}

// ---- the same product on packed 4-bit codes ---------------------------------------------------
// Block rows are 32 bytes (two codes per byte, each as code + 8): per channel block a workgroup
// brings 4 KB of uq and 2 KB of vq into LDS instead of 8 + 4, and a lane reads 8 bytes per
// fragment instead of 16 -- LDS traffic, which bounds the unpacked kernel, is halved.  The
// nibbles are split in registers (three operations per packed dword) and go to the matrix cores
// as they are, unsigned: sum (cu+8)(cv+8) = sum cu*cv + 8*RU + 8*CV + 64*Cp, where the last
// term is taken off the integer sums before they are converted and the middle ones are part of
// the filter-side and input-side constants the host-side caller asked for (DqOut::bias).
// Any assignment of a block's channels to the contraction index is as good as another as long
// as both operands use the same one; here contraction bytes come in the order (low nibbles of
// the lane's 8 bytes, high nibbles of the lane's 8 bytes).
constexpr int kPkRow = pk::kRow;
constexpr int kPkBlockBytes = (kTileK + kTileP) * kPkRow;    // 6 KB
typedef pk::v2i v2i;

// This wave's copies of one step (the buffer descriptors live in a helper: a kernel body that
// names their type loses its host stub).
__device__ __forceinline__ void pk_copy_step(const int8_t* uq, unsigned uq_bytes, const int8_t* vq,
                                             unsigned vq_bytes, char* slot, unsigned dst_u0,
                                             unsigned voff_u0, unsigned dst_u1, unsigned voff_u1,
                                             bool two_u, unsigned dst_v, unsigned voff_v,
                                             unsigned off_u, unsigned off_v) {
  const __amdgpu_buffer_rsrc_t res_u =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(uq), 0, uq_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t res_v =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(vq), 0, vq_bytes, 0x00020000);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(
      res_u, (__attribute__((address_space(3))) char*)(slot + dst_u0), 16, voff_u0, off_u, 0, 0);
  if (two_u)  // (a compile-time constant of the calling kernel)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(
        res_u, (__attribute__((address_space(3))) char*)(slot + dst_u1), 16, voff_u1, off_u, 0, 0);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(
      res_v, (__attribute__((address_space(3))) char*)(slot + dst_v), 16, voff_v, off_v, 0, 0);
}

struct GpArgs {
  GtArgs g;
  unsigned uq_bytes, vq_bytes;
  int bias2;  // 64 * Cp
};

// SB: channel blocks per step (4: NB a multiple of 4; 2: NB even; 1: NB odd).  A step's pieces
// of 32 rows (4*SB of uq, 2*SB of vq) are dealt to the eight waves, every wave issuing the same
// number of copies per step (SB = 4: two of uq and one of vq; else one of each); where that is
// more waves than pieces, waves copy the same piece twice (same bytes to the same place).
template <int SB>
__global__ __launch_bounds__(kThreads, 4) void gemm_fused_m2_packed_kernel(const GpArgs as) {
  constexpr int M = 2, E = 16;
  constexpr int kStepBytes = SB * kPkBlockBytes;
  constexpr int kRing = SB == 4 ? 3 : (SB == 2 ? 4 : 8);  // 72 KB or 48 KB
  constexpr int kUCopies = SB == 4 ? 2 : 1;
  constexpr int kCopies = kUCopies + 1;
  const GtArgs& a = as.g;
  extern __shared__ char smem[];
  char* ring = smem;
  float* rk_s = reinterpret_cast<float*>(smem + kRing * kStepBytes);  // [128 filters][M*M]
  float* sc_s = rk_s + M * M * kTileK;                                // [E] s_e

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = a.K, P = a.P, NB = a.NB;
  const int item = dev::xcd_contiguous(blockIdx.x, gridDim.x);
  const int tb = item / a.nky, ky = item - tb * a.nky;
  const int k0w = ky * kTileK, p0w = tb * kTileP;

  const unsigned su = (unsigned)K * kPkRow, sv = (unsigned)P * kPkRow;  // bytes between blocks
  unsigned voff_u[kUCopies], dst_u[kUCopies];
#pragma unroll
  for (int j = 0; j < kUCopies; j++) {
    const int q = SB == 1 ? (wave & 3) : wave + 8 * j;  // piece of the step: block q/4, rows 32*(q%4)..
    voff_u[j] = (unsigned)(q >> 2) * su +
                (unsigned)min(k0w + 32 * (q & 3) + pk::lane_row(lane), K - 1) * kPkRow +
                (unsigned)pk::lane_chunk(lane) * 16u;
    dst_u[j] = (unsigned)((q >> 2) * kPkBlockBytes + (q & 3) * 1024);
  }
  const int qv = SB == 4 ? wave : (SB == 2 ? (wave & 3) : (wave & 1));  // block qv/2, rows 32*(qv%2)..
  const unsigned voff_v = (unsigned)(qv >> 1) * sv +
                          (unsigned)min(p0w + 32 * (qv & 1) + pk::lane_row(lane), P - 1) * kPkRow +
                          (unsigned)pk::lane_chunk(lane) * 16u;
  const unsigned dst_v = (unsigned)((qv >> 1) * kPkBlockBytes + kTileK * kPkRow + (qv & 1) * 1024);
  const int steps = E * NB / SB;
  unsigned off_u = 0, off_v = 0;
  const unsigned last_u = (unsigned)(steps - 1) * SB * su, last_v = (unsigned)(steps - 1) * SB * sv;
  int slot_w = 0, slot_r = 0;
  // Copies past the last step read it again (into a slot nobody reads any more): every step
  // issues the same number of copies and the waits stay exact.
  auto issue = [&]() {
    pk_copy_step(a.uq, as.uq_bytes, a.vq, as.vq_bytes, ring + slot_w * kStepBytes, dst_u[0],
                 voff_u[0], dst_u[kUCopies - 1], voff_u[kUCopies - 1], kUCopies == 2, dst_v, voff_v,
                 off_u, off_v);
    off_u = min(off_u + SB * su, last_u);
    off_v = min(off_v + SB * sv, last_v);
    slot_w = slot_w + 1 == kRing ? 0 : slot_w + 1;
  };
#pragma unroll
  for (int d = 0; d < kRing - 1; d++) issue();

  m2_filter_terms(a, rk_s, sc_s, tid, wave, k0w);

  // this wave's 32 x 32 tile
  const int kw = wave & 3, pw = wave >> 2;
  const int col = lane & 31, half = lane >> 5;
  const int brow_l = pw * 32 + col;
  const unsigned fa[2] = {(unsigned)(kw * 1024) + pk::frag_offset(col, 0, half),
                          (unsigned)(kw * 1024) + pk::frag_offset(col, 1, half)};
  const unsigned fb[2] = {(unsigned)(kTileK * kPkRow + pw * 1024) + pk::frag_offset(col, 0, half),
                          (unsigned)(kTileK * kPkRow + pw * 1024) + pk::frag_offset(col, 1, half)};

  v16f out[M * M];
#pragma unroll
  for (int ab = 0; ab < M * M; ab++)
#pragma unroll
    for (int r = 0; r < 16; r++) out[ab][r] = 0.0f;
  v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

  auto step = [&]() {
    m2_wait_and_barrier<(kRing - 2) * kCopies>();
    issue();
    const char* blk = ring + slot_r * kStepBytes;
    slot_r = slot_r + 1 == kRing ? 0 : slot_r + 1;
    // two blocks' fragments at a time: more would not fit the registers beside the outputs
    constexpr int kG = SB == 1 ? 1 : 2;
#pragma unroll
    for (int i0 = 0; i0 < SB; i0 += kG) {
      v2i xa[kG][2], xb[kG][2];
#pragma unroll
      for (int i = 0; i < kG; i++)
#pragma unroll
        for (int c = 0; c < 2; c++) {
          xa[i][c] = *reinterpret_cast<const v2i*>(blk + (i0 + i) * kPkBlockBytes + fa[c]);
          xb[i][c] = *reinterpret_cast<const v2i*>(blk + (i0 + i) * kPkBlockBytes + fb[c]);
        }
#pragma unroll
      for (int i = 0; i < kG; i++)
#pragma unroll
        for (int c = 0; c < 2; c++)
          acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(pk::unpack(xa[i][c]), pk::unpack(xb[i][c]),
                                                      acc, 0, 0, 0);
      if (i0 + kG < SB) __builtin_amdgcn_sched_barrier(0);
    }
  };
  static_for<E>([&](auto ec) {
    constexpr int e = decltype(ec)::value;
    for (int i = 0; i < NB / SB; i++) step();
    m2_fold<e>(acc, sc_s, out, as.bias2);
#pragma unroll
    for (int r = 0; r < 16; r++) acc[r] = 0;
  });
  // the copies past the end are still in flight: they must have landed before the workgroup
  // ends (its LDS is handed to the next one)
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)

  m2_tail(a, out, rk_s, kw, half, brow_l, k0w, p0w);
}

constexpr size_t kTailBytes = (2 * 2 * kTileK + 16 * 4) * sizeof(float);

}  // namespace

// The streaming kernel addresses both code tensors by 32-bit byte offsets.
static bool stream_m2_fits(const Geo& g) {
  // (NCHW layers with one block have a plan of their own: conv_fused_c64.hip)
  return !is_packed(g) && g.m == 2 && g.CB == 64 && g.NB >= (is_nhwc(g) ? 1 : 2) && (long long)g.E * g.NB * g.K * 64 < (1LL << 32) &&
         (long long)g.E * g.NB * g.P * 64 < (1LL << 32) &&
         (long long)g.N * g.K * g.Ho * g.Wo * 4 < 0xFFFFFFF0LL;
}

// Layers for which the streaming kernel on 128 x 64 tiles is the fastest product kernel: at
// least 128 such tiles (measured: 196 tiles beat the 784 small workgroups of
// gemm_fused_rows.hip by 18 %, 52 tiles lose to 200 of them by 40 %).
bool gemm_fused_stream_m2_preferred(const Geo& g) {
  const long long items = (long long)((g.P + kTileP - 1) / kTileP) * ((g.K + kTileK - 1) / kTileK);
  return stream_m2_fits(g) && items >= 128 && items < (1LL << 31);
}

bool gemm_fused_tiled_applicable(const Geo& g) {
  const long long items = (long long)((g.P + kTileP - 1) / kTileP) * ((g.K + kTileK - 1) / kTileK);
  return stream_m2_fits(g) && items < (1LL << 31);
}

hipError_t launch_gemm_fused_tiled(const Geo& g, const int8_t* uq, const int8_t* vq,
                                   const int32_t* colsum, const float* dq, const double* dqd,
                                   const int32_t* u_rowsum, float* y, hipStream_t s) {
  if (!gemm_fused_tiled_applicable(g)) return hipErrorInvalidValue;
  GtArgs a{uq, vq, colsum, dq, dqd, u_rowsum, y, g.K, g.P, g.NB, g.th, g.tw, g.Ho, g.Wo,
           (g.K + kTileK - 1) / kTileK, (unsigned)((size_t)g.N * g.K * g.Ho * g.Wo * 4),
           is_nhwc(g) ? 1 : 0};
  const unsigned grid = (unsigned)(((g.P + kTileP - 1) / kTileP) * a.nky);
  // Variants without any loop for the usual block counts; steps of one block when NB is odd.
  {
    const GsArgs as{a, (unsigned)((long long)g.E * g.NB * g.K * 64),
                    (unsigned)((long long)g.E * g.NB * g.P * 64)};
    const size_t lds = 3 * 2 * (size_t)kBlockBytes + kTailBytes;
    auto run = [&](auto kern) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
      note_kernel("gemm_fused_m2_stream_kernel");
      kern<<<grid, kThreads, lds, s>>>(as);
      return hipGetLastError();
    };
    if (g.NB == 2) return run(gemm_fused_m2_stream_kernel<2, 2>);
    if (g.NB == 4) return run(gemm_fused_m2_stream_kernel<2, 4>);
    if (g.NB == 8) return run(gemm_fused_m2_stream_kernel<2, 8>);
    if (g.NB % 2 == 0) return run(gemm_fused_m2_stream_kernel<2, 0>);
    return run(gemm_fused_m2_stream_kernel<1, 0>);
  }
}

bool gemm_fused_packed_applicable(const Geo& g) {
  const long long items = (long long)((g.P + kTileP - 1) / kTileP) * ((g.K + kTileK - 1) / kTileK);
  return is_packed(g) && g.m == 2 && g.CB == 64 && items < (1LL << 31);
}

hipError_t launch_gemm_fused_packed(const Geo& g, const int8_t* uq, const int8_t* vq,
                                    const int32_t* colsum, const float* dq, const double* dqd,
                                    const int32_t* u_rowsum, float* y, hipStream_t s) {
  if (!gemm_fused_packed_applicable(g)) return hipErrorInvalidValue;
  GtArgs a{uq, vq, colsum, dq, dqd, u_rowsum, y, g.K, g.P, g.NB, g.th, g.tw, g.Ho, g.Wo,
           (g.K + kTileK - 1) / kTileK, (unsigned)((size_t)g.N * g.K * g.Ho * g.Wo * 4),
           is_nhwc(g) ? 1 : 0};
  const unsigned grid = (unsigned)(((g.P + kTileP - 1) / kTileP) * a.nky);
  const GpArgs as{a, (unsigned)((long long)g.E * g.NB * g.K * kPkRow),
                  (unsigned)((long long)g.E * g.NB * g.P * kPkRow), 64 * g.Cp};
  const size_t lds = (g.NB % 4 == 0 ? 12 : 8) * (size_t)kPkBlockBytes + kTailBytes;
  auto run = [&](auto kern) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    note_kernel("gemm_fused_m2_packed_kernel");
    kern<<<grid, kThreads, lds, s>>>(as);
    return hipGetLastError();
  };
  if (g.NB % 4 == 0) return run(gemm_fused_m2_packed_kernel<4>);
  return g.NB % 2 == 0 ? run(gemm_fused_m2_packed_kernel<2>) : run(gemm_fused_m2_packed_kernel<1>);
}

}  // namespace lance
