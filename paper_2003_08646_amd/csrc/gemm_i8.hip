// Stage 3 (and 3+4 fused): the low-precision product of Algorithm 1 as E integer GEMMs on the
// int8 matrix cores (Sec. 3.3), int32 accumulation.
//
// Operands are the blocked code tensors uq [E][NB][K][CB] and vq [E][NB][P][CB]: both have the
// reduction (channel) axis contiguous, so a lane's MFMA fragment is one 16-byte (or 8-byte)
// load.  The byte order inside a block is the same in both operands, so the dot product over
// a block equals the dot product over its channels.
//
// MFMA tile: 32 (filters k) x 32 (tiles p) per wave, v_mfma_i32_32x32x32_i8 (16 bytes of k per
// lane) when CB is a multiple of 32, v_mfma_i32_32x32x16_i8 (8 bytes) otherwise.
// Fragment layout used below (wave64): A/B lane l holds row/column l%32, k-chunk l/32;
// accumulator register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32.
#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;

// A^T of F(2x2,3x3) and F(4x4,3x3) for run-time row indices (Eq. 4).
__constant__ float kAt[2][4][6] = {
    {{1, 1, 1, 0, 0, 0}, {0, 1, -1, -1, 0, 0}, {0, 0, 0, 0, 0, 0}, {0, 0, 0, 0, 0, 0}},
    {{1, 1, 1, 1, 1, 0}, {0, 1, -1, 2, -2, 0}, {0, 1, 1, 4, 4, 0}, {0, 1, -1, 8, -8, 1}}};

// One 32x32 tile of sum_c uq[e,k,c]*vq[e,p,c] for position e.  arow/brow are this lane's
// (clamped) row pointers at block 0; consecutive blocks are astride/bstride bytes apart.
template <int KSTEP>
__device__ __forceinline__ v16i tile_product(const int8_t* __restrict__ arow,
                                             const int8_t* __restrict__ brow, size_t astride,
                                             size_t bstride, int NB, int CB, int half) {
  v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  for (int cb = 0; cb < NB; cb++) {
    const int8_t* ap = arow + cb * astride;
    const int8_t* bp = brow + cb * bstride;
    for (int kk = 0; kk < CB; kk += KSTEP) {
      if constexpr (KSTEP == 32) {
        const v4i a = *reinterpret_cast<const v4i*>(ap + kk + 16 * half);
        const v4i b = *reinterpret_cast<const v4i*>(bp + kk + 16 * half);
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc, 0, 0, 0);
      } else {
        const long a = *reinterpret_cast<const long*>(ap + kk + 8 * half);
        const long b = *reinterpret_cast<const long*>(bp + kk + 8 * half);
        acc = __builtin_amdgcn_mfma_i32_32x32x16_i8(a, b, acc, 0, 0, 0);
      }
    }
  }
  return acc;
}

// ---- stage 3 alone: acc[e][k][p] (int32) ---------------------------------------------------
template <int KSTEP>
__global__ __launch_bounds__(kThreads) void gemm_i8_kernel(const int8_t* __restrict__ uq,
                                                           const int8_t* __restrict__ vq,
                                                           int32_t* __restrict__ acc_out, int K,
                                                           int P, int CB, int NB) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int e = blockIdx.z;
  const int k0 = blockIdx.y * 64 + (wave >> 1) * 32;
  const int p0 = blockIdx.x * 64 + (wave & 1) * 32;
  if (k0 >= K || p0 >= P) return;
  const int col = lane & 31, half = lane >> 5;
  const int krow = min(k0 + col, K - 1), prow = min(p0 + col, P - 1);
  const size_t astride = (size_t)K * CB, bstride = (size_t)P * CB;
  const int8_t* arow = uq + ((size_t)e * NB * K + krow) * CB;
  const int8_t* brow = vq + ((size_t)e * NB * P + prow) * CB;
  const v16i acc = tile_product<KSTEP>(arow, brow, astride, bstride, NB, CB, half);
  const int p = p0 + col;
  if (p < P) {
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int k = k0 + 8 * (r / 4) + 4 * half + (r % 4);
      if (k < K) acc_out[((size_t)e * K + k) * P + p] = acc[r];
    }
  }
}

// ---- stages 3+4 fused: the accumulators never leave the registers ---------------------------
// De-quantization (Eq. 8, expanded) gives  M[e,k,p] = s_e*ACC[e,k,p] + f[e,k] + g[e,p]  and the
// output transform S = A^T M A (Eq. 9) is linear, so the three terms go through it separately:
//   * s_e*ACC: per position e = (i,j), finish the reduction over channels, then
//     rowacc[b] += (A^T[b][j]*s_e) * ACC   and, at the end of row i,  out[a][b] += A^T[a][i]*rowacc[b];
//   * f: already transformed by the range-reduction kernel into rk[a*m+b][k];
//   * g = dq[e][1]*colsum[e][p]: transformed once per lane (its tile p is fixed).
// Only m*m*16 outputs and m*16 row sums per lane live across positions, which is what lets the
// fusion work for F(4x4,3x3) as well (36 positions would need 576 accumulator registers).
template <int M, int KSTEP, int MINW>
__global__ __launch_bounds__(kThreads, MINW) void gemm_fused_kernel(
    const int8_t* __restrict__ uq, const int8_t* __restrict__ vq,
    const int32_t* __restrict__ colsum, const float* __restrict__ dq, const float* __restrict__ rk,
    float* __restrict__ y, int K, int P, int CB, int NB, int th, int tw, int Ho, int Wo, int nhwc) {
  constexpr int A = M + 2, E = A * A, MI = (M == 2 ? 0 : 1);
  __shared__ float rk_s[M * M][64];  // filter-side terms of this workgroup's 64 filters
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int kb0 = blockIdx.y * 64;
  for (int i = threadIdx.x; i < M * M * 64; i += kThreads) {
    const int ab = i >> 6, kk = i & 63;
    rk_s[ab][kk] = rk[(size_t)ab * K + min(kb0 + kk, K - 1)];
  }
  __syncthreads();
  const int k0 = kb0 + (wave >> 1) * 32;
  const int p0 = blockIdx.x * 64 + (wave & 1) * 32;
  if (k0 >= K || p0 >= P) return;
  const int col = lane & 31, half = lane >> 5;
  const int krow = min(k0 + col, K - 1), prow = min(p0 + col, P - 1);
  const size_t astride = (size_t)K * CB, bstride = (size_t)P * CB;

  // input-side term of this lane's tile, through A^T . A
  float gp[M][M];
#pragma unroll
  for (int a = 0; a < M; a++)
#pragma unroll
    for (int b = 0; b < M; b++) gp[a][b] = 0.0f;
#pragma unroll
  for (int e = 0; e < E; e++) {
    const float g = dq[4 * e + 1] * (float)colsum[(size_t)e * P + prow];
#pragma unroll
    for (int a = 0; a < M; a++)
#pragma unroll
      for (int b = 0; b < M; b++) {
        const float coef = dev::Wino<M>::at(a, e / A) * dev::Wino<M>::at(b, e % A);
        if (coef != 0.0f) gp[a][b] = __builtin_fmaf(coef, g, gp[a][b]);
      }
  }

  float out[M][M][16];
#pragma unroll
  for (int a = 0; a < M; a++)
#pragma unroll
    for (int b = 0; b < M; b++)
#pragma unroll
      for (int r = 0; r < 16; r++) out[a][b][r] = 0.0f;

#pragma nounroll
  for (int i = 0; i < A; i++) {
    float rowacc[M][16];
#pragma unroll
    for (int b = 0; b < M; b++)
#pragma unroll
      for (int r = 0; r < 16; r++) rowacc[b][r] = 0.0f;
#pragma unroll
    for (int j = 0; j < A; j++) {
      const int e = i * A + j;
      const int8_t* arow = uq + ((size_t)e * NB * K + krow) * CB;
      const int8_t* brow = vq + ((size_t)e * NB * P + prow) * CB;
      const v16i acc = tile_product<KSTEP>(arow, brow, astride, bstride, NB, CB, half);
      const float s = dq[4 * e];
#pragma unroll
      for (int b = 0; b < M; b++) {
        const float coef = dev::Wino<M>::at(b, j);  // compile-time: zero terms vanish
        if (coef != 0.0f) {
          const float cs = coef * s;
#pragma unroll
          for (int r = 0; r < 16; r++)
            rowacc[b][r] = __builtin_fmaf(cs, (float)acc[r], rowacc[b][r]);
        }
      }
    }
#pragma unroll
    for (int a = 0; a < M; a++) {
      const float ca = kAt[MI][a][i];
#pragma unroll
      for (int b = 0; b < M; b++)
#pragma unroll
        for (int r = 0; r < 16; r++) out[a][b][r] = __builtin_fmaf(ca, rowacc[b][r], out[a][b][r]);
    }
  }

  const int p = p0 + col;
  if (p < P) {
    const int tx = p % tw, t2 = p / tw;
    const int ty = t2 % th, n = t2 / th;
    const bool pair_ok = (M == 2) && (tx * M + 1 < Wo) && ((Wo & 1) == 0) && !nhwc;
    const float* rk_l = &rk_s[0][(wave >> 1) * 32 + 4 * half];
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int kk = 8 * (r / 4) + (r % 4);
      const int k = k0 + 4 * half + kk;
      if (k < K) {
        float* yk = y + ((size_t)n * K + k) * Ho * Wo;
#pragma unroll
        for (int a = 0; a < M; a++) {
          const int yy = ty * M + a;
          if (yy < Ho) {
            float o[M];
#pragma unroll
            for (int b = 0; b < M; b++)
              o[b] = (out[a][b][r] + rk_l[(a * M + b) * 64 + kk]) + gp[a][b];
            if (pair_ok) {
              *reinterpret_cast<float2*>(yk + (size_t)yy * Wo + tx * M) = make_float2(o[0], o[1]);
            } else {
#pragma unroll
              for (int b = 0; b < M; b++) {
                const int xx = tx * M + b;
                if (xx < Wo) y[dev::act_index(nhwc, n, k, yy, xx, K, Ho, Wo)] = o[b];
              }
            }
          }
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_gemm_i8(const Geo& g, const int8_t* uq, const int8_t* vq, int32_t* acc,
                          hipStream_t s) {
  if (gemm_i8_tiled_applicable(g)) return launch_gemm_i8_tiled(g, uq, vq, acc, s);
  // what is left are the 16-channel code blocks (descriptor validation keeps every tensor within
  // the 32-bit offsets of the tiled kernel)
  if (g.CB != 16) return hipErrorInvalidValue;
  dim3 grid((g.P + 63) / 64, (g.K + 63) / 64, g.E);
  gemm_i8_kernel<16><<<grid, kThreads, 0, s>>>(uq, vq, acc, g.K, g.P, g.CB, g.NB);
  return hipGetLastError();
}

bool gemm_fused_wants_rk(const Geo& g) {
  return !(is_packed(g) || gemm_fused_rows_applicable(g) || gemm_fused_tiled_applicable(g) ||
           gemm_fused_tiled_m4_applicable(g) || conv_fused_c16_applicable(g));
}

hipError_t launch_gemm_fused(const Geo& g, const int8_t* uq, const int8_t* vq,
                             const int32_t* v_colsum, const float* dq, const float* rk,
                             const double* dqd, const int32_t* u_rowsum, float* y, hipStream_t s) {
  if (is_packed(g))
    return g.m == 2 ? launch_gemm_fused_packed(g, uq, vq, v_colsum, dq, dqd, u_rowsum, y, s)
                    : launch_gemm_fused_packed_m4(g, uq, vq, v_colsum, dq, dqd, u_rowsum, y, s);
  if (gemm_fused_rows_applicable(g))
    return launch_gemm_fused_rows(g, uq, vq, v_colsum, dq, dqd, u_rowsum, y, s);
  if (gemm_fused_tiled_applicable(g))
    return launch_gemm_fused_tiled(g, uq, vq, v_colsum, dq, dqd, u_rowsum, y, s);
  if (gemm_fused_tiled_m4_applicable(g))
    return launch_gemm_fused_tiled_m4(g, uq, vq, v_colsum, dq, dqd, u_rowsum, y, s);
  if (g.CB != 16) return hipErrorInvalidValue;  // 64-channel blocks are served above
  dim3 grid((g.P + 63) / 64, (g.K + 63) / 64, 1);
#define LANCE_FUSED(MM, KS, MW)                                                                 \
  gemm_fused_kernel<MM, KS, MW><<<grid, kThreads, 0, s>>>(uq, vq, v_colsum, dq, rk, y, g.K, \
                                                          g.P, g.CB, g.NB, g.th, g.tw, g.Ho, g.Wo,     \
                                                          is_nhwc(g) ? 1 : 0)
  note_kernel("gemm_fused_kernel");
  if (g.m == 2) LANCE_FUSED(2, 16, 2); else LANCE_FUSED(4, 16, 1);
#undef LANCE_FUSED
  return hipGetLastError();
}

}  // namespace lance
