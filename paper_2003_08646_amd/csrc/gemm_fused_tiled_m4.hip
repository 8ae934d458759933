// Stages 3+4 fused for F(4x4,3x3) layers with 64-channel code blocks: the int8 products of
// Algorithm 1 (Sec. 3.3) with both operands staged through LDS, the de-quantization (Eq. 8) and
// the output transform (Eq. 9) applied to the register accumulators.
//
// F(4x4,3x3) has 36 positions and 16 outputs per tile and filter, so what a lane carries across
// the positions is 16 output values (plus 4 row sums) per accumulator element.  That rules out
// 32 x 32 matrix tiles (16 accumulator registers each); the kernel uses v_mfma_i32_16x16x64_i8
// (4 accumulator registers, the whole 64-channel block in one instruction).  A workgroup of four
// waves owns 64 filters x 32 tiles; wave w takes filters 16w.. and both 16-tile groups, so its
// two products of a stage share the A fragment.
//
// Stage = two channel blocks (one if NB is odd) of one position e: a 64 x 64 B piece of uq and a
// 32 x 64 B piece of vq per block; consecutive stages are a constant stride apart in both code
// tensors ([E][NB][rows][64]).  The copies run two stages ahead in registers, every thread moves
// the same number of 16-byte chunks (no thread-dependent branches, so the memory counters of
// the pipeline stay exact), one barrier per stage.  LDS rows are 64 bytes with the 16-byte chunk
// c of row r stored at c ^ ((r >> 2) & 3): the fragment reads of 16 consecutive rows cover all
// banks.
//
// Epilogue algebra: M[e,k,p] = s_e*ACC + f[e,k] + g[e,p]; the three terms go through the linear
// map S = A^T M A separately.  The first: per position (i, j), rowacc[b] += A^T[b][j] s_e ACC, and
// at the end of grid row i, out[a][b] += A^T[a][i] rowacc[b] (zero coefficients skipped by
// wave-uniform branches).  f is formed here from the filter row sums (binary64); g from the
// column sums of the input codes.
#include "lance_device.h"
#include "lance_internal.h"
#include "m4_fold.h"
#include "packed_codes.h"

namespace lance {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
using m4e::kAt;
using m4e::m4_fold;
using m4e::static_for;
using m4e::v4f;

constexpr int kThreads = 512;
constexpr int kTileK = 64, kTileP = 32;
constexpr int kBlockBytes = (kTileK + kTileP) * 64;  // one channel block of both pieces: 6 KB

struct G4Args {
  const int8_t* uq;
  const int8_t* vq;
  const int32_t* colsum;
  const float* dq;          // [E][4]
  const double* dqd;        // [E][2] = {su*ov, C*ou*ov}
  const int32_t* u_rowsum;  // [E][K]
  float* y;
  int K, P, NB, th, tw, Ho, Wo;
  int nky;  // filter tiles (ceil(K / 64))
  int nhwc;  // Y is [N][Ho][Wo][K]
};


// Filter-side terms f[e,k] = su*ov*rowsum[e][k] + C*ou*ov through A^T . A, in binary64, for the 64
// filters of the workgroup: rk_s[(a*4 + b)*64 + filter].  Thread = (a = kw, b pair = tg, filter =
// lane) of a workgroup of eight waves.
__device__ __forceinline__ void m4_filter_terms(const G4Args& a, float* rk_s, int k0w, int kw,
                                                int tg, int lane) {
  constexpr int M = 4, A = 6, E = 36;
  const int kk = lane, k = min(k0w + kk, a.K - 1);
  // Everything is unrolled: the 36 row sums and constants are requested at once (a loop over
  // the positions waits for memory 36 times), and the coefficient rows are looked up once.
  double ca[A], cb[2][A];
#pragma unroll
  for (int i = 0; i < A; i++) {
    ca[i] = (double)dev::at_coef(M, kw, i);  // a = kw
    cb[0][i] = (double)dev::at_coef(M, 2 * tg, i);
    cb[1][i] = (double)dev::at_coef(M, 2 * tg + 1, i);
  }
  int32_t rs[E];
#pragma unroll
  for (int e2 = 0; e2 < E; e2++) rs[e2] = a.u_rowsum[(size_t)e2 * a.K + k];
  double accd[2] = {0.0, 0.0};
#pragma unroll
  for (int e2 = 0; e2 < E; e2++) {
    const double f = a.dqd[2 * e2] * (double)rs[e2] + a.dqd[2 * e2 + 1];
    const double ci = ca[e2 / A];
#pragma unroll
    for (int b = 0; b < 2; b++) accd[b] += ci * cb[b][e2 % A] * f;
  }
#pragma unroll
  for (int b = 0; b < 2; b++) rk_s[(kw * 4 + 2 * tg + b) * kTileK + kk] = (float)accd[b];
}

// Tail: add the two separable terms and store the 4x4 patches.  The lane holds filters
// k0w + 16*kw + 4*kq + r (r = register) of tile p0w + 16*tg + col.
__device__ __forceinline__ void m4_tail(const G4Args& a, const v4f (&out)[4][4], const float* rk_s,
                                        int k0w, int p0w, int kw, int tg, int kq, int col) {
  constexpr int M = 4, A = 6;
  const int K = a.K, P = a.P;
  const int k0 = k0w + kw * 16 + 4 * kq;
  const int Ho = a.Ho, Wo = a.Wo;
  const bool vec_ok = (Wo % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.y) & 15) == 0);
  const int p = p0w + tg * 16 + col;
  if (p < P && k0 < K) {
    float gp[M][M];  // input-side term of this lane's tile through A^T . A
#pragma unroll
    for (int aa = 0; aa < M; aa++)
#pragma unroll
      for (int b = 0; b < M; b++) gp[aa][b] = 0.0f;
    // unrolled: the 36 column sums are requested at once
    int32_t cs[A * A];
#pragma unroll
    for (int e2 = 0; e2 < A * A; e2++) cs[e2] = a.colsum[(size_t)e2 * P + p];
#pragma unroll
    for (int i = 0; i < A; i++) {
      float gr[M] = {0.0f, 0.0f, 0.0f, 0.0f};  // sum_j A^T[b][j] g[(i, j)]
#pragma unroll
      for (int j = 0; j < A; j++) {
        const int e2 = i * A + j;
        const float g = a.dq[4 * e2 + 1] * (float)cs[e2];
#pragma unroll
        for (int b = 0; b < M; b++) {
          const float coef = dev::Wino<M>::at(b, j);
          if (coef != 0.0f) gr[b] = __builtin_fmaf(coef, g, gr[b]);
        }
      }
#pragma unroll
      for (int aa = 0; aa < M; aa++) {
        const float ca = dev::Wino<M>::at(aa, i);
#pragma unroll
        for (int b = 0; b < M; b++) gp[aa][b] = __builtin_fmaf(ca, gr[b], gp[aa][b]);
      }
    }
    const int tx = p % a.tw, t2 = p / a.tw;
    const int ty = t2 % a.th, n = t2 / a.th;
    const float* rk_l = rk_s + kw * 16 + 4 * kq;
    if (a.nhwc) {
      // the lane's four filters are consecutive: one 16-byte store per output pixel
      typedef float f4 __attribute__((ext_vector_type(4)));
      const bool k4 = (K & 3) == 0 && (reinterpret_cast<uintptr_t>(a.y) & 15) == 0;
#pragma unroll
      for (int aa = 0; aa < M; aa++) {
        const int yy = ty * M + aa;
        if (yy < Ho) {
#pragma unroll
          for (int b = 0; b < M; b++) {
            const int xx = tx * M + b;
            if (xx < Wo) {
              float o[4];
#pragma unroll
              for (int r = 0; r < 4; r++)
                o[r] = (out[aa][b][r] + rk_l[(aa * M + b) * kTileK + r]) + gp[aa][b];
              float* dst = a.y + (((size_t)n * Ho + yy) * Wo + xx) * K + k0;
              if (k4) {
                *reinterpret_cast<f4*>(dst) = f4{o[0], o[1], o[2], o[3]};
              } else {
#pragma unroll
                for (int r = 0; r < 4; r++)
                  if (k0 + r < K) dst[r] = o[r];
              }
            }
          }
        }
      }
      return;
    }
#pragma unroll
    for (int r = 0; r < 4; r++) {
      const int k = k0 + r;
      if (k < K) {
        float* yk = a.y + ((size_t)n * K + k) * Ho * Wo;
#pragma unroll
        for (int aa = 0; aa < M; aa++) {
          const int yy = ty * M + aa;
          if (yy < Ho) {
            float o[M];
#pragma unroll
            for (int b = 0; b < M; b++)
              o[b] = (out[aa][b][r] + rk_l[(aa * M + b) * kTileK + r]) + gp[aa][b];
            float* dst = yk + (size_t)yy * Wo + tx * M;
            if (vec_ok) {  // the tile's four columns are inside and 16-byte aligned
              typedef float f4 __attribute__((ext_vector_type(4)));
              *reinterpret_cast<f4*>(dst) = f4{o[0], o[1], o[2], o[3]};
            } else if (tx * M + 3 < Wo) {  // inside, any 4-byte alignment: still one store
              typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
              *reinterpret_cast<f4u*>(dst) = f4u{o[0], o[1], o[2], o[3]};
            } else {
#pragma unroll
              for (int b = 0; b < M; b++)
                if (tx * M + b < Wo) dst[b] = o[b];
            }
          }
        }
      }
    }
  }
}

// CBS: channel blocks per stage (1 or 2; divides NB).  ODD: NB / CBS is odd.  NST: NB / CBS if it
// is known at compile time (then there is no loop left in the product phase), else 0.
template <int CBS, bool ODD, int NST>
__global__ __launch_bounds__(kThreads, 4) void gemm_fused_tiled_m4_kernel(const G4Args a) {
  constexpr int M = 4, E = 36, DEPTH = 2;
  constexpr int kBufBytes = CBS * kBlockBytes;
  extern __shared__ char smem[];
  char* stage_s = smem;                                             // [2][kBufBytes]
  float* rk_s = reinterpret_cast<float*>(smem + 2 * kBufBytes);     // [M*M][64]
  float* sc_s = rk_s + M * M * kTileK;                              // [E] s_e

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kw = wave & 3, tg = wave >> 2;  // this wave: filters 16*kw .., tiles 16*tg ..
  const int K = a.K, P = a.P;
  // work item = (tile block, filter tile), the filter tiles of a tile block next to each other
  // on one die so that they share the block's codes in its L2
  const int item = dev::xcd_contiguous(blockIdx.x, gridDim.x);
  const int tb = item / a.nky, ky = item - tb * a.nky;
  const int k0w = ky * kTileK, p0w = tb * kTileP;

  // Copy descriptors.  Per channel block: 256 chunks of uq and 128 chunks of vq.  Every thread
  // moves one chunk of each per stage: with two blocks per stage thread t takes uq chunk t & 255
  // of block t >> 8, and vq chunk t & 127 of block (t >> 7) & 1 (the upper 256 threads move the
  // lower ones' vq chunks again); a single block's chunks are moved two and four times.
  const int asel = CBS == 2 ? tid >> 8 : 0, bsel = CBS == 2 ? (tid >> 7) & 1 : 0;
  const int crow = (tid & 255) >> 2, cchunk = tid & 3;   // uq: row 0..63
  const int brow = crow & 31;                            // vq: row 0..31
  const unsigned la_off = (unsigned)asel * kBlockBytes + (unsigned)crow * 64u +
                          (unsigned)((cchunk ^ ((crow >> 2) & 3)) * 16);
  const unsigned lb_off = (unsigned)bsel * kBlockBytes + (unsigned)(kTileK + brow) * 64u +
                          (unsigned)((cchunk ^ ((brow >> 2) & 3)) * 16);
  const size_t sa = (size_t)K * 64, sb = (size_t)P * 64;  // bytes between consecutive channel blocks
  const int8_t* ga = a.uq + (size_t)min(k0w + crow, K - 1) * 64 + cchunk * 16 + asel * sa;
  const int8_t* gb = a.vq + (size_t)min(p0w + brow, P - 1) * 64 + cchunk * 16 + bsel * sb;
  const int S = E * a.NB / CBS;  // stages

  v4i ra[DEPTH], rb[DEPTH];
  auto request = [&](int stage, v4i& xa, v4i& xb) {
    const size_t blk = (size_t)min(stage, S - 1) * CBS;  // past the end: the last stage again
    xa = *reinterpret_cast<const v4i*>(ga + blk * sa);
    xb = *reinterpret_cast<const v4i*>(gb + blk * sb);
  };
  auto commit = [&](char* buf, const v4i& xa, const v4i& xb) {
    *reinterpret_cast<v4i*>(buf + la_off) = xa;
    *reinterpret_cast<v4i*>(buf + lb_off) = xb;
  };
#pragma unroll
  for (int d = 0; d < DEPTH; d++) request(d, ra[d], rb[d]);

  m4_filter_terms(a, rk_s, k0w, kw, tg, lane);
  if (tid < E) sc_s[tid] = a.dq[4 * tid];

  // this wave's sub-tile: filters 16*kw .., tiles 16*tg ..
  const int col = lane & 15, kq = lane >> 4;
  const int arow_l = kw * 16 + col, brow_l = tg * 16 + col;
  const unsigned fa = (unsigned)arow_l * 64u + (unsigned)((kq ^ ((arow_l >> 2) & 3)) * 16);
  const unsigned fb =
      (unsigned)(kTileK + brow_l) * 64u + (unsigned)((kq ^ ((brow_l >> 2) & 3)) * 16);

  commit(stage_s, ra[0], rb[0]);
  __syncthreads();

  v4f out[M][M];   // [a][b][accumulator register]
  v4f rowacc[M];   // [b][accumulator register]
#pragma unroll
  for (int aa = 0; aa < M; aa++)
#pragma unroll
    for (int b = 0; b < M; b++)
#pragma unroll
      for (int r = 0; r < 4; r++) out[aa][b][r] = 0.0f;
#pragma unroll
  for (int b = 0; b < M; b++)
#pragma unroll
    for (int r = 0; r < 4; r++) rowacc[b][r] = 0.0f;
  v4i acc = {0, 0, 0, 0};

  // The 36 positions are unrolled so that the coefficients of the folds are compile-time
  // constants (looked up at run time they cost a chain of dependent table loads and branches per
  // stage, several times the products themselves).  Slot and LDS buffer of a stage are its
  // parity; with an odd number of stages per position a position starts on the parity of e.
  int s = 0;                      // stages done
  const int nst = a.NB / CBS;     // stages per position
  auto stage = [&](auto uc) {
    constexpr int u = decltype(uc)::value;
    request(s + DEPTH, ra[u], rb[u]);  // slot u is free: stage s is in LDS
    const char* buf = stage_s + u * kBufBytes;
#pragma unroll
    for (int c = 0; c < CBS; c++) {
      const v4i af = *reinterpret_cast<const v4i*>(buf + c * kBlockBytes + fa);
      const v4i bf = *reinterpret_cast<const v4i*>(buf + c * kBlockBytes + fb);
      acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(af, bf, acc, 0, 0, 0);
    }
    // stage s + 1 has been in flight for DEPTH - 1 stages
    commit(stage_s + (u ^ 1) * kBufBytes, ra[u ^ 1], rb[u ^ 1]);
    __syncthreads();
    s++;
  };
  static_for<E>([&](auto ec) {
    constexpr int e = decltype(ec)::value;
    if constexpr (NST > 0) {
      static_for<NST>([&](auto ic) {
        stage(std::integral_constant<int, (e * NST + decltype(ic)::value) & 1>{});
      });
    } else if constexpr (ODD) {
      constexpr int u0 = e & 1;
      for (int i = 0; i + 1 < nst; i += 2) {
        stage(std::integral_constant<int, u0>{});
        stage(std::integral_constant<int, u0 ^ 1>{});
      }
      stage(std::integral_constant<int, u0>{});
    } else {
      for (int i = 0; i < nst; i += 2) {
        stage(std::integral_constant<int, 0>{});
        stage(std::integral_constant<int, 1>{});
      }
    }
    m4_fold<e>(acc, sc_s, rowacc, out);
    acc = v4i{0, 0, 0, 0};
  });

  m4_tail(a, out, rk_s, k0w, p0w, kw, tg, kq, col);
}

// ---- streaming variant: NB from 2 to 8 -------------------------------------------------------
// The same workgroup tile and wave layout, but the code pieces go from memory straight into LDS
// (buffer loads that write LDS: no registers, no LDS store instructions), four channel blocks
// (24 KB) per step into a ring of three slots, i.e. eight blocks in flight ahead of the one being
// multiplied: with two 16-byte loads per thread two stages ahead the loop above waits for memory
// (one stage per half a memory latency); this one does not.  The blocks of all positions are a
// constant stride apart in both code tensors, so a step is simply the next four blocks; which of
// them ends a position is known at compile time (NB is a template parameter), and so are the
// coefficients of the folds.  One barrier per step.
constexpr int kStepBlocks = 4, kStepBytes = kStepBlocks * kBlockBytes, kRing = 3;

struct G4sArgs {
  G4Args g;
  unsigned uq_bytes, vq_bytes;
};

// This wave's three copies of one step: uq pieces 8j + wave (j = 0, 1) and vq piece wave, 1 KB
// each (16 rows of 64 bytes, lane l = row l/4, stored chunk l%4).
__device__ __forceinline__ void m4_copy_step(const int8_t* uq, unsigned uq_bytes, const int8_t* vq,
                                             unsigned vq_bytes, char* slot, int wave,
                                             const unsigned (&voff)[3], unsigned off_u,
                                             unsigned off_v) {
  const __amdgpu_buffer_rsrc_t res_u =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(uq), 0, uq_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t res_v =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(vq), 0, vq_bytes, 0x00020000);
#pragma unroll
  for (int j = 0; j < 2; j++) {
    const int pu = 8 * j + wave;  // block pu / 4, rows 16 * (pu % 4) ..
    auto* dst = (__attribute__((address_space(3))) char*)(slot + (pu >> 2) * kBlockBytes +
                                                          (pu & 3) * 1024);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(res_u, dst, 16, voff[j], off_u, 0, 0);
  }
  auto* dst = (__attribute__((address_space(3))) char*)(slot + (wave >> 1) * kBlockBytes +
                                                        kTileK * 64 + (wave & 1) * 1024);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(res_v, dst, 16, voff[2], off_v, 0, 0);
}

// At most N of this wave's copies outstanding, all its LDS reads done; then the other waves.
template <int N>
__device__ __forceinline__ void m4_wait_and_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt((N & 15) | 0x70 | ((N >> 4) << 14));  // vmcnt(N) lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Chunk swizzle of the streaming kernel's LDS rows (its own: the rows are written by loads that
// write LDS and read as 16 x 16 x 64 fragments, lane & 15 = row, lane >> 4 = chunk).  One row bit
// of (0,1) and one of (2,3), by measurement: 48.9 us against 50.9 us with bits (2,3) on the
// 128-channel 56 x 56 layer.
__device__ __forceinline__ int m4s_swizzle(int r) { return ((r >> 1) & 1) | (((r >> 3) & 1) << 1); }

template <int NB>
__global__ __launch_bounds__(kThreads, 4) void gemm_fused_m4_stream_kernel(const G4sArgs as) {
  constexpr int M = 4, E = 36;
  constexpr int kSteps = E * NB / kStepBlocks;
  static_assert(E * NB % kStepBlocks == 0, "whole steps");
  const G4Args& a = as.g;
  extern __shared__ char smem[];
  char* ring = smem;                                               // [kRing][kStepBytes]
  float* rk_s = reinterpret_cast<float*>(smem + kRing * kStepBytes);  // [M*M][64]
  float* sc_s = rk_s + M * M * kTileK;                              // [E] s_e

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kw = wave & 3, tg = wave >> 2;  // this wave: filters 16*kw .., tiles 16*tg ..
  const int K = a.K, P = a.P;
  const int item = dev::xcd_contiguous(blockIdx.x, gridDim.x);
  const int tb = item / a.nky, ky = item - tb * a.nky;
  const int k0w = ky * kTileK, p0w = tb * kTileP;

  // lane offsets of the three copies inside a step (block stride included)
  const unsigned su = (unsigned)K * 64u, sv = (unsigned)P * 64u;  // bytes between blocks
  unsigned voff[3];
  {
    const int r16 = lane >> 2, cpos = lane & 3;
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const int pu = 8 * j + wave, row = 16 * (pu & 3) + r16;
      voff[j] = (unsigned)(pu >> 2) * su + (unsigned)min(k0w + row, K - 1) * 64u +
                (unsigned)((cpos ^ m4s_swizzle(row)) * 16);
    }
    const int row = 16 * (wave & 1) + r16;
    voff[2] = (unsigned)(wave >> 1) * sv + (unsigned)min(p0w + row, P - 1) * 64u +
              (unsigned)((cpos ^ m4s_swizzle(row)) * 16);
  }
  unsigned off_u = 0, off_v = 0;
  const unsigned last_u = (unsigned)(kSteps - 1) * kStepBlocks * su;
  const unsigned last_v = (unsigned)(kSteps - 1) * kStepBlocks * sv;
  // Copies past the last step read it again (into a slot nobody reads any more): every step
  // issues the same number of copies and the waits stay exact.
  auto issue = [&](int slot) {
    m4_copy_step(a.uq, as.uq_bytes, a.vq, as.vq_bytes, ring + slot * kStepBytes, wave, voff,
                 off_u, off_v);
    off_u = min(off_u + kStepBlocks * su, last_u);
    off_v = min(off_v + kStepBlocks * sv, last_v);
  };
  issue(0);
  issue(1);

  m4_filter_terms(a, rk_s, k0w, kw, tg, lane);
  if (tid < E) sc_s[tid] = a.dq[4 * tid];

  const int col = lane & 15, kq = lane >> 4;
  const int arow_l = kw * 16 + col, brow_l = tg * 16 + col;
  const unsigned fa = (unsigned)arow_l * 64u + (unsigned)((kq ^ m4s_swizzle(arow_l)) * 16);
  const unsigned fb =
      (unsigned)(kTileK + brow_l) * 64u + (unsigned)((kq ^ m4s_swizzle(brow_l)) * 16);

  typedef float v4f __attribute__((ext_vector_type(4)));
  v4f out[M][M], rowacc[M];
#pragma unroll
  for (int aa = 0; aa < M; aa++)
#pragma unroll
    for (int b = 0; b < M; b++) out[aa][b] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int b = 0; b < M; b++) rowacc[b] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
  v4i acc = {0, 0, 0, 0};

  static_for<kSteps>([&](auto tc) {
    constexpr int t = decltype(tc)::value;
    // This wave's copies of step t have landed and so have, after the barrier, everybody's
    // (rk_s and sc_s too, the first time); every wave has read step t - 1, whose slot takes
    // step t + 2.
    m4_wait_and_barrier<3>();
    issue((t + 2) % kRing);
    const char* blk = ring + (t % kRing) * kStepBytes;
    v4i af[kStepBlocks], bf[kStepBlocks];
#pragma unroll
    for (int i = 0; i < kStepBlocks; i++) {
      af[i] = *reinterpret_cast<const v4i*>(blk + i * kBlockBytes + fa);
      bf[i] = *reinterpret_cast<const v4i*>(blk + i * kBlockBytes + fb);
    }
    static_for<kStepBlocks>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      constexpr int q = t * kStepBlocks + i;  // block number: position q / NB, block q % NB
      acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[i], bf[i], acc, 0, 0, 0);
      if constexpr (q % NB == NB - 1) {
        m4_fold<q / NB>(acc, sc_s, rowacc, out);
        acc = v4i{0, 0, 0, 0};
      }
    });
  });
  // the copies past the end are still in flight: they must have landed before the workgroup
  // ends (its LDS is handed to the next one)
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  m4_tail(a, out, rk_s, k0w, p0w, kw, tg, kq, col);
}

// ---- the same product on packed 4-bit codes (block rows of 32 bytes, see packed_codes.h) -------
// Any number of channel blocks: steps of SB blocks (4, 2 or 1, the largest that divides NB), the
// blocks of a position a run-time loop, the positions unrolled.  Per step the workgroup brings
// SB * (2 KB of uq + 1 KB of vq) into LDS; every wave issues two copies (one 32-row piece of uq,
// one of vq; where that is more waves than pieces, waves copy a piece twice).  The nibbles go to
// the matrix cores unsigned; 64 * Cp comes off the integer sums before conversion and the rest of
// the offset is in the constants (DqOut::bias).
constexpr int kPkBlockBytes4 = (kTileK + kTileP) * pk::kRow;  // 3 KB

struct G4pArgs {
  G4Args g;
  unsigned uq_bytes, vq_bytes;
  int bias2;
};

__device__ __forceinline__ void m4p_copy_step(const int8_t* uq, unsigned uq_bytes, const int8_t* vq,
                                              unsigned vq_bytes, char* slot, unsigned dst_u,
                                              unsigned voff_u, unsigned dst_v, unsigned voff_v,
                                              unsigned off_u, unsigned off_v) {
  const __amdgpu_buffer_rsrc_t res_u =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(uq), 0, uq_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t res_v =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t*>(vq), 0, vq_bytes, 0x00020000);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(
      res_u, (__attribute__((address_space(3))) char*)(slot + dst_u), 16, voff_u, off_u, 0, 0);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(
      res_v, (__attribute__((address_space(3))) char*)(slot + dst_v), 16, voff_v, off_v, 0, 0);
}

template <int SB>
__global__ __launch_bounds__(kThreads, 4) void gemm_fused_m4_packed_kernel(const G4pArgs as) {
  constexpr int M = 4, E = 36;
  constexpr int kStep = SB * kPkBlockBytes4;
  constexpr int kSlots = SB == 4 ? 4 : (SB == 2 ? 6 : 8);
  constexpr int kCopies = 2;
  const G4Args& a = as.g;
  extern __shared__ char smem[];
  char* ring = smem;                                             // [kSlots][kStep]
  float* rk_s = reinterpret_cast<float*>(smem + kSlots * kStep);  // [M*M][64]
  float* sc_s = rk_s + M * M * kTileK;                           // [E] s_e

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kw = wave & 3, tg = wave >> 2;  // this wave: filters 16*kw .., tiles 16*tg ..
  const int K = a.K, P = a.P, NB = a.NB;
  const int item = dev::xcd_contiguous(blockIdx.x, gridDim.x);
  const int tb = item / a.nky, ky = item - tb * a.nky;
  const int k0w = ky * kTileK, p0w = tb * kTileP;

  const unsigned su = (unsigned)K * pk::kRow, sv = (unsigned)P * pk::kRow;  // bytes between blocks
  const int qu = wave % (2 * SB);  // uq piece of the step: block qu / 2, rows 32 * (qu % 2) ..
  const int qv = wave % SB;        // vq piece of the step: block qv, rows 0 .. 31
  const unsigned voff_u = (unsigned)(qu >> 1) * su +
                          (unsigned)min(k0w + 32 * (qu & 1) + pk::lane_row(lane), K - 1) * pk::kRow +
                          (unsigned)pk::lane_chunk(lane) * 16u;
  const unsigned voff_v = (unsigned)qv * sv +
                          (unsigned)min(p0w + pk::lane_row(lane), P - 1) * pk::kRow +
                          (unsigned)pk::lane_chunk(lane) * 16u;
  const unsigned dst_u = (unsigned)((qu >> 1) * kPkBlockBytes4 + (qu & 1) * 1024);
  const unsigned dst_v = (unsigned)(qv * kPkBlockBytes4 + kTileK * pk::kRow);
  const int steps = E * NB / SB;
  unsigned off_u = 0, off_v = 0;
  const unsigned last_u = (unsigned)(steps - 1) * SB * su, last_v = (unsigned)(steps - 1) * SB * sv;
  int slot_w = 0, slot_r = 0;
  // Copies past the last step read it again (into a slot nobody reads any more): every step
  // issues the same number of copies and the waits stay exact.
  auto issue = [&]() {
    m4p_copy_step(a.uq, as.uq_bytes, a.vq, as.vq_bytes, ring + slot_w * kStep, dst_u, voff_u, dst_v,
                  voff_v, off_u, off_v);
    off_u = min(off_u + SB * su, last_u);
    off_v = min(off_v + SB * sv, last_v);
    slot_w = slot_w + 1 == kSlots ? 0 : slot_w + 1;
  };
#pragma unroll
  for (int d = 0; d < kSlots - 1; d++) issue();

  m4_filter_terms(a, rk_s, k0w, kw, tg, lane);
  if (tid < E) sc_s[tid] = a.dq[4 * tid];

  // fragments: lane = (row col of the wave's 16, quarter kq of the block's 64 contraction bytes)
  const int col = lane & 15, kq = lane >> 4;
  const int arow = (kw & 1) * 16 + col;  // row inside its 32-row piece (piece kw >> 1)
  const unsigned fa = (unsigned)((kw >> 1) * 1024) + pk::frag_offset(arow, kq >> 1, kq & 1);
  const unsigned fb = (unsigned)(kTileK * pk::kRow) + pk::frag_offset(tg * 16 + col, kq >> 1, kq & 1);

  typedef float v4f __attribute__((ext_vector_type(4)));
  v4f out[M][M], rowacc[M];
#pragma unroll
  for (int aa = 0; aa < M; aa++)
#pragma unroll
    for (int b = 0; b < M; b++) out[aa][b] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int b = 0; b < M; b++) rowacc[b] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
  v4i acc = {0, 0, 0, 0};

  auto step = [&]() {
    m4_wait_and_barrier<(kSlots - 2) * kCopies>();
    issue();
    const char* blk = ring + slot_r * kStep;
    slot_r = slot_r + 1 == kSlots ? 0 : slot_r + 1;
    pk::v2i xa[SB], xb[SB];
#pragma unroll
    for (int i = 0; i < SB; i++) {
      xa[i] = *reinterpret_cast<const pk::v2i*>(blk + i * kPkBlockBytes4 + fa);
      xb[i] = *reinterpret_cast<const pk::v2i*>(blk + i * kPkBlockBytes4 + fb);
    }
#pragma unroll
    for (int i = 0; i < SB; i++)
      acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(pk::unpack(xa[i]), pk::unpack(xb[i]), acc, 0, 0, 0);
  };
  static_for<E>([&](auto ec) {
    constexpr int e = decltype(ec)::value;
    for (int i = 0; i < NB / SB; i++) step();
    m4_fold<e>(acc, sc_s, rowacc, out, as.bias2);
    acc = v4i{0, 0, 0, 0};
  });
  // the copies past the end are still in flight: they must have landed before the workgroup
  // ends (its LDS is handed to the next one)
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  m4_tail(a, out, rk_s, k0w, p0w, kw, tg, kq, col);
}

constexpr size_t kTailBytes = (4 * 4 * kTileK + 36) * sizeof(float);

}  // namespace

bool gemm_fused_tiled_m4_applicable(const Geo& g) {
  if (is_packed(g)) return false;  // packed codes have a kernel of their own
  const long long items = (long long)((g.P + kTileP - 1) / kTileP) * ((g.K + kTileK - 1) / kTileK);
  return g.m == 4 && g.CB == 64 && items < (1LL << 31);
}

hipError_t launch_gemm_fused_tiled_m4(const Geo& g, const int8_t* uq, const int8_t* vq,
                                      const int32_t* colsum, const float* dq, const double* dqd,
                                      const int32_t* u_rowsum, float* y, hipStream_t s) {
  if (!gemm_fused_tiled_m4_applicable(g)) return hipErrorInvalidValue;
  G4Args a{uq, vq, colsum, dq, dqd, u_rowsum, y, g.K, g.P, g.NB, g.th, g.tw, g.Ho, g.Wo,
           (g.K + kTileK - 1) / kTileK, is_nhwc(g) ? 1 : 0};
  const unsigned grid = (unsigned)(((g.P + kTileP - 1) / kTileP) * a.nky);
  const long long uq_bytes = (long long)g.E * g.NB * g.K * 64, vq_bytes = (long long)g.E * g.NB * g.P * 64;
  // (one fully unrolled variant per block count: 2 .. 8, i.e. up to 512 channels)
  if (g.NB >= 2 && g.NB <= 8 && uq_bytes < (1LL << 32) && vq_bytes < (1LL << 32)) {
    const G4sArgs as{a, (unsigned)uq_bytes, (unsigned)vq_bytes};
    const size_t lds = (size_t)kRing * kStepBytes + kTailBytes;
    auto run = [&](auto kern) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
      note_kernel("gemm_fused_m4_stream_kernel");
      kern<<<grid, kThreads, lds, s>>>(as);
      return hipGetLastError();
    };
    switch (g.NB) {
      case 2: return run(gemm_fused_m4_stream_kernel<2>);
      case 3: return run(gemm_fused_m4_stream_kernel<3>);
      case 4: return run(gemm_fused_m4_stream_kernel<4>);
      case 5: return run(gemm_fused_m4_stream_kernel<5>);
      case 6: return run(gemm_fused_m4_stream_kernel<6>);
      case 7: return run(gemm_fused_m4_stream_kernel<7>);
      default: return run(gemm_fused_m4_stream_kernel<8>);
    }
  }
  note_kernel("gemm_fused_tiled_m4_kernel");
  if (g.NB % 2 == 0) {
    const size_t lds = 2 * 2 * (size_t)kBlockBytes + kTailBytes;
    if ((g.NB / 2) % 2)
      gemm_fused_tiled_m4_kernel<2, true, 0><<<grid, kThreads, lds, s>>>(a);
    else
      gemm_fused_tiled_m4_kernel<2, false, 0><<<grid, kThreads, lds, s>>>(a);
  } else {
    const size_t lds = 2 * (size_t)kBlockBytes + kTailBytes;
    gemm_fused_tiled_m4_kernel<1, true, 0><<<grid, kThreads, lds, s>>>(a);
  }
  return hipGetLastError();
}

bool gemm_fused_packed_m4_applicable(const Geo& g) {
  const long long items = (long long)((g.P + kTileP - 1) / kTileP) * ((g.K + kTileK - 1) / kTileK);
  return is_packed(g) && g.m == 4 && g.CB == 64 && items < (1LL << 31);
}

hipError_t launch_gemm_fused_packed_m4(const Geo& g, const int8_t* uq, const int8_t* vq,
                                       const int32_t* colsum, const float* dq, const double* dqd,
                                       const int32_t* u_rowsum, float* y, hipStream_t s) {
  if (!gemm_fused_packed_m4_applicable(g)) return hipErrorInvalidValue;
  G4Args a{uq, vq, colsum, dq, dqd, u_rowsum, y, g.K, g.P, g.NB, g.th, g.tw, g.Ho, g.Wo,
           (g.K + kTileK - 1) / kTileK, is_nhwc(g) ? 1 : 0};
  const unsigned grid = (unsigned)(((g.P + kTileP - 1) / kTileP) * a.nky);
  const G4pArgs as{a, (unsigned)((long long)g.E * g.NB * g.K * pk::kRow),
                   (unsigned)((long long)g.E * g.NB * g.P * pk::kRow), 64 * g.Cp};
  const int sb = g.NB % 4 == 0 ? 4 : (g.NB % 2 == 0 ? 2 : 1);
  const size_t lds = (size_t)(sb == 4 ? 16 : (sb == 2 ? 12 : 8)) * kPkBlockBytes4 + kTailBytes;
  auto run = [&](auto kern) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    note_kernel("gemm_fused_m4_packed_kernel");
    kern<<<grid, kThreads, lds, s>>>(as);
    return hipGetLastError();
  };
  if (sb == 4) return run(gemm_fused_m4_packed_kernel<4>);
  return sb == 2 ? run(gemm_fused_m4_packed_kernel<2>) : run(gemm_fused_m4_packed_kernel<1>);
}

}  // namespace lance
