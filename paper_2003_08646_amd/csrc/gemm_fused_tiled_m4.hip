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

namespace lance {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
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
};

// CBS: channel blocks per stage (1 or 2; divides NB).
template <int CBS>
__global__ __launch_bounds__(kThreads, 2) void gemm_fused_tiled_m4_kernel(const G4Args a) {
  constexpr int M = 4, A = 6, E = 36, DEPTH = 2;
  constexpr int kBufBytes = CBS * kBlockBytes;
  extern __shared__ char smem[];
  char* stage_s = smem;                                             // [2][kBufBytes]
  float* rk_s = reinterpret_cast<float*>(smem + 2 * kBufBytes);     // [M*M][64]
  float* sc_s = rk_s + M * M * kTileK;                              // [E] s_e

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = a.K, P = a.P;
  // work item = (tile block, filter tile), the filter tiles of a tile block next to each other
  // on one die so that they share the block's codes in its L2
  const int item = dev::xcd_contiguous(blockIdx.x, gridDim.x);
  const int tb = item / a.nky, ky = item - tb * a.nky;
  const int k0w = ky * kTileK, p0w = tb * kTileP;

  // Copy descriptors.  Per channel block: 256 chunks of uq (thread t moves chunk t) and 128
  // chunks of vq.  With two blocks per stage the lower 128 threads take the first block's vq
  // chunks and the upper 128 the second one's; a single block's are moved twice, by both halves.
  const int crow = tid >> 2, cchunk = tid & 3;           // uq: row 0..63
  const int brow = crow & 31, bsel = tid >> 7;           // vq: row 0..31; which block of the pair
  const unsigned la_off = (unsigned)crow * 64u + (unsigned)((cchunk ^ ((crow >> 2) & 3)) * 16);
  const unsigned lb_off = (unsigned)(kTileK + brow) * 64u + (unsigned)((cchunk ^ ((brow >> 2) & 3)) * 16);
  const size_t sa = (size_t)K * 64, sb = (size_t)P * 64;  // bytes between consecutive channel blocks
  const int8_t* ga = a.uq + (size_t)min(k0w + crow, K - 1) * 64 + cchunk * 16;
  const int8_t* gb = a.vq + (size_t)min(p0w + brow, P - 1) * 64 + cchunk * 16;
  const int S = E * a.NB / CBS;  // stages (even: E is)

  v4i ra[DEPTH][CBS], rb[DEPTH];
  auto request = [&](int stage, v4i (&xa)[CBS], v4i& xb) {
    const size_t blk = (size_t)min(stage, S - 1) * CBS;  // past the end: the last stage again
#pragma unroll
    for (int c = 0; c < CBS; c++) xa[c] = *reinterpret_cast<const v4i*>(ga + (blk + c) * sa);
    xb = *reinterpret_cast<const v4i*>(gb + (blk + (CBS == 2 ? bsel : 0)) * sb);
  };
  auto commit = [&](char* buf, const v4i (&xa)[CBS], const v4i& xb) {
#pragma unroll
    for (int c = 0; c < CBS; c++) *reinterpret_cast<v4i*>(buf + c * kBlockBytes + la_off) = xa[c];
    *reinterpret_cast<v4i*>(buf + (CBS == 2 ? bsel : 0) * kBlockBytes + lb_off) = xb;
  };
#pragma unroll
  for (int d = 0; d < DEPTH; d++) request(d, ra[d], rb[d]);

  // filter-side terms f[e,k] = su*ov*rowsum[e][k] + C*ou*ov through A^T . A, in binary64: thread =
  // (ab quad, filter): wave w forms ab = 4w .. 4w+3 for filter kk = lane
  {
    const int kk = lane, k = min(k0w + kk, K - 1);
    double accd[4] = {0.0, 0.0, 0.0, 0.0};
    for (int e2 = 0; e2 < E; e2++) {
      const double f = a.dqd[2 * e2] * (double)a.u_rowsum[(size_t)e2 * K + k] + a.dqd[2 * e2 + 1];
      const double ci = (double)dev::at_coef(M, wave, e2 / A);  // a = wave
#pragma unroll
      for (int b = 0; b < 4; b++) accd[b] += ci * (double)dev::at_coef(M, b, e2 % A) * f;
    }
#pragma unroll
    for (int b = 0; b < 4; b++) rk_s[(wave * 4 + b) * kTileK + kk] = (float)accd[b];
  }
  if (tid < E) sc_s[tid] = a.dq[4 * tid];

  // this wave's sub-tiles: filters 16*wave .., tiles 0..15 and 16..31
  const int col = lane & 15, kq = lane >> 4;
  const int arow_l = wave * 16 + col;
  const unsigned fa = (unsigned)arow_l * 64u + (unsigned)((kq ^ ((arow_l >> 2) & 3)) * 16);
  unsigned fb[2];
#pragma unroll
  for (int t = 0; t < 2; t++) {
    const int brow_l = t * 16 + col;
    fb[t] = (unsigned)(kTileK + brow_l) * 64u + (unsigned)((kq ^ ((brow_l >> 2) & 3)) * 16);
  }

  commit(stage_s, ra[0], rb[0]);
  __syncthreads();

  float out[2][M][M][4];   // [sub-tile][a][b][accumulator register]
  float rowacc[2][M][4];   // [sub-tile][b][accumulator register]
#pragma unroll
  for (int t = 0; t < 2; t++)
#pragma unroll
    for (int aa = 0; aa < M; aa++)
#pragma unroll
      for (int b = 0; b < M; b++)
#pragma unroll
        for (int r = 0; r < 4; r++) out[t][aa][b][r] = 0.0f;
#pragma unroll
  for (int t = 0; t < 2; t++)
#pragma unroll
    for (int b = 0; b < M; b++)
#pragma unroll
      for (int r = 0; r < 4; r++) rowacc[t][b][r] = 0.0f;
  v4i acc[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}};

  int cb = 0, e = 0, gi = 0, gj = 0;  // channel blocks done of position e = (gi, gj)
  for (int s0 = 0; s0 < S; s0 += DEPTH) {
#pragma unroll
    for (int u = 0; u < DEPTH; u++) {
      const int s = s0 + u;
      request(s + DEPTH, ra[u], rb[u]);  // slot u is free: stage s is in LDS
      const char* buf = stage_s + (s & 1) * kBufBytes;
#pragma unroll
      for (int c = 0; c < CBS; c++) {
        const v4i af = *reinterpret_cast<const v4i*>(buf + c * kBlockBytes + fa);
        const v4i b0 = *reinterpret_cast<const v4i*>(buf + c * kBlockBytes + fb[0]);
        const v4i b1 = *reinterpret_cast<const v4i*>(buf + c * kBlockBytes + fb[1]);
        acc[0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af, b0, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af, b1, acc[1], 0, 0, 0);
      }
      cb += CBS;
      if (cb == a.NB) {  // position e = (gi, gj) is complete
        const float se = sc_s[e];
        float accf[2][4];
#pragma unroll
        for (int t = 0; t < 2; t++)
#pragma unroll
          for (int r = 0; r < 4; r++) accf[t][r] = (float)acc[t][r];
#pragma unroll
        for (int b = 0; b < M; b++) {
          const float cj = dev::at_coef(M, b, gj);  // wave-uniform
          if (cj != 0.0f) {
            const float cs = cj * se;
#pragma unroll
            for (int t = 0; t < 2; t++)
#pragma unroll
              for (int r = 0; r < 4; r++)
                rowacc[t][b][r] = __builtin_fmaf(cs, accf[t][r], rowacc[t][b][r]);
          }
        }
        acc[0] = v4i{0, 0, 0, 0};
        acc[1] = v4i{0, 0, 0, 0};
        cb = 0;
        e++;
        if (++gj == A) {  // end of grid row gi: out[a][b] += A^T[a][gi] * rowacc[b]
#pragma unroll
          for (int aa = 0; aa < M; aa++) {
            const float ca = dev::at_coef(M, aa, gi);  // wave-uniform
            if (ca != 0.0f) {
#pragma unroll
              for (int t = 0; t < 2; t++)
#pragma unroll
                for (int b = 0; b < M; b++)
#pragma unroll
                  for (int r = 0; r < 4; r++)
                    out[t][aa][b][r] = __builtin_fmaf(ca, rowacc[t][b][r], out[t][aa][b][r]);
            }
          }
#pragma unroll
          for (int t = 0; t < 2; t++)
#pragma unroll
            for (int b = 0; b < M; b++)
#pragma unroll
              for (int r = 0; r < 4; r++) rowacc[t][b][r] = 0.0f;
          gj = 0;
          gi++;
        }
      }
      // stage s + 1 has been in flight for DEPTH - 1 stages
      commit(stage_s + ((s + 1) & 1) * kBufBytes, ra[(u + 1) % DEPTH], rb[(u + 1) % DEPTH]);
      __syncthreads();
    }
  }

  // ---- tail: add the two separable terms, store the 4x4 patches ----
  const int k0 = k0w + wave * 16 + 4 * kq;  // this lane's four filters k0 .. k0+3
  const int Ho = a.Ho, Wo = a.Wo;
  const bool vec_ok = (Wo % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.y) & 15) == 0);
#pragma unroll
  for (int t = 0; t < 2; t++) {
    const int p = p0w + t * 16 + col;
    if (p < P && k0 < K) {
      float gp[M][M];  // input-side term of this lane's tile through A^T . A
#pragma unroll
      for (int aa = 0; aa < M; aa++)
#pragma unroll
        for (int b = 0; b < M; b++) gp[aa][b] = 0.0f;
      for (int i = 0; i < A; i++) {
        float gr[M] = {0.0f, 0.0f, 0.0f, 0.0f};  // sum_j A^T[b][j] g[(i, j)]
#pragma unroll
        for (int j = 0; j < A; j++) {
          const int e2 = i * A + j;
          const float g = a.dq[4 * e2 + 1] * (float)a.colsum[(size_t)e2 * P + p];
#pragma unroll
          for (int b = 0; b < M; b++) {
            const float coef = dev::Wino<M>::at(b, j);
            if (coef != 0.0f) gr[b] = __builtin_fmaf(coef, g, gr[b]);
          }
        }
#pragma unroll
        for (int aa = 0; aa < M; aa++) {
          const float ca = dev::at_coef(M, aa, i);
#pragma unroll
          for (int b = 0; b < M; b++) gp[aa][b] = __builtin_fmaf(ca, gr[b], gp[aa][b]);
        }
      }
      const int tx = p % a.tw, t2 = p / a.tw;
      const int ty = t2 % a.th, n = t2 / a.th;
      const float* rk_l = rk_s + wave * 16 + 4 * kq;
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
                o[b] = (out[t][aa][b][r] + rk_l[(aa * M + b) * kTileK + r]) + gp[aa][b];
              float* dst = yk + (size_t)yy * Wo + tx * M;
              if (vec_ok) {  // the tile's four columns are inside and 16-byte aligned
                typedef float f4 __attribute__((ext_vector_type(4)));
                *reinterpret_cast<f4*>(dst) = f4{o[0], o[1], o[2], o[3]};
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
}

constexpr size_t kTailBytes = (4 * 4 * kTileK + 36) * sizeof(float);

}  // namespace

bool gemm_fused_tiled_m4_applicable(const Geo& g) {
  const long long items = (long long)((g.P + kTileP - 1) / kTileP) * ((g.K + kTileK - 1) / kTileK);
  return g.m == 4 && g.CB == 64 && items < (1LL << 31);
}

hipError_t launch_gemm_fused_tiled_m4(const Geo& g, const int8_t* uq, const int8_t* vq,
                                      const int32_t* colsum, const float* dq, const double* dqd,
                                      const int32_t* u_rowsum, float* y, hipStream_t s) {
  if (!gemm_fused_tiled_m4_applicable(g)) return hipErrorInvalidValue;
  G4Args a{uq, vq, colsum, dq, dqd, u_rowsum, y, g.K, g.P, g.NB, g.th, g.tw, g.Ho, g.Wo,
           (g.K + kTileK - 1) / kTileK};
  const unsigned grid = (unsigned)(((g.P + kTileP - 1) / kTileP) * a.nky);
  if (g.NB % 2 == 0) {
    const size_t lds = 2 * 2 * (size_t)kBlockBytes + kTailBytes;
    gemm_fused_tiled_m4_kernel<2><<<grid, kThreads, lds, s>>>(a);
  } else {
    const size_t lds = 2 * (size_t)kBlockBytes + kTailBytes;
    gemm_fused_tiled_m4_kernel<1><<<grid, kThreads, lds, s>>>(a);
  }
  return hipGetLastError();
}

}  // namespace lance
