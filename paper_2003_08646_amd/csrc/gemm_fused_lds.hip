// Stages 3+4 fused, streaming variant for layers whose code rows are short (Cp = 64): the int8
// product of Algorithm 1 (Sec. 3.3) on the matrix cores with the de-quantization (Eq. 8) and the
// output transform (Eq. 9) applied to the register accumulators.
//
// Such layers have so little matrix work per byte that the kernel is a stream over vq; what
// matters is that the whole stream is in flight at once.  A workgroup owns 64 tiles (p) and all
// filters.  It copies the vq rows of its tiles into LDS in bulk -- one row of the position grid
// ((m+2) positions x NB blocks x 64 tiles x 64 bytes) per ring slot, every slot requested before
// anything is computed -- and then runs over the positions reading the B fragments from LDS.
// When the ring holds the whole grid (m = 2, Cp = 64) vq is read exactly once, also for K > 64.
// The A fragments (uq, a few hundred KB, cache resident) of the next grid row are requested
// while the current row is multiplied.
//
// LDS rows are 64 bytes; the 16-byte chunk c of row p is stored at chunk c ^ ((p >> 1) & 3), so
// that the 16-byte fragment reads of eight consecutive rows cover all 32 banks.
//
// Epilogue algebra (as in gemm_i8.hip): M[e,k,p] = s_e*ACC + f[e,k] + g[e,p]; the three terms go
// through the linear map S = A^T M A separately; f arrives pre-transformed in rk[a*m+b][k].
#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;

template <int M, int NB, int NR>
__global__ __launch_bounds__(kThreads, (M == 2 ? 2 : 1)) void gemm_fused_lds_kernel(
    const int8_t* __restrict__ uq, const int8_t* __restrict__ vq,
    const int32_t* __restrict__ colsum, const float* __restrict__ dq, const float* __restrict__ rk,
    float* __restrict__ y, int K, int P, int th, int tw, int Ho, int Wo) {
  constexpr int A = M + 2, E = A * A;
  constexpr int kPieces = A * NB;             // 4 KB pieces (64 rows x 64 B) per grid row
  constexpr int kSlotBytes = kPieces * 4096;  // one ring slot
  constexpr int kFrags = kPieces * 2;         // A fragments (16 B per lane) per grid row
  static_assert(A % NR == 0, "ring slots must divide the grid rows");
  extern __shared__ char smem[];
  char* ring = smem;                                               // [NR][kSlotBytes]
  float* rk_s = reinterpret_cast<float*>(smem + NR * kSlotBytes);  // [M*M][64], then sc_s[E]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, half = lane >> 5;
  const int p0 = blockIdx.x * 64;
  const int prow_l = (wave & 1) * 32 + col;  // this lane's tile row inside the block
  const int p = p0 + prow_l;
  const int prow = min(p, P - 1);
  const int nkb = (K + 63) / 64;
  const int total = nkb * A;  // (filter block, grid row) steps

  // copy descriptors: thread t moves chunk t%4 of row t/4 of every 4 KB piece
  const int crow = tid >> 2, cchunk = tid & 3;
  const unsigned g_off = (unsigned)min(p0 + crow, P - 1) * 64u + (unsigned)cchunk * 16u;
  const unsigned l_off = (unsigned)crow * 64u + (unsigned)((cchunk ^ ((crow >> 1) & 3)) * 16);
  const size_t piece_stride = (size_t)P * 64;  // bytes between consecutive (e, cb) planes of vq
  // fragment read offsets of this lane inside a piece (k-halves 0 and 1)
  const unsigned f_off0 = (unsigned)prow_l * 64u + (unsigned)(((0 + half) ^ ((prow_l >> 1) & 3)) * 16);
  const unsigned f_off1 = (unsigned)prow_l * 64u + (unsigned)(((2 + half) ^ ((prow_l >> 1) & 3)) * 16);

  auto load_row = [&](int i, v4i (&st)[kPieces]) {  // grid row i of vq -> registers
    const int8_t* src = vq + (size_t)i * kPieces * piece_stride;
#pragma unroll
    for (int q = 0; q < kPieces; q++)
      st[q] = *reinterpret_cast<const v4i*>(src + (size_t)q * piece_stride + g_off);
  };
  auto store_row = [&](int slot, const v4i (&st)[kPieces]) {
#pragma unroll
    for (int q = 0; q < kPieces; q++)
      *reinterpret_cast<v4i*>(ring + slot * kSlotBytes + q * 4096 + l_off) = st[q];
  };
  auto load_afrags = [&](int kb, int i, v4i (&af)[kFrags]) {  // uq fragments of grid row i
    const int krow = min(kb * 64 + (wave >> 1) * 32 + col, K - 1);
    const int8_t* src = uq + ((size_t)i * kPieces * K + krow) * 64 + 16 * half;
#pragma unroll
    for (int q = 0; q < kPieces; q++) {
      af[2 * q] = *reinterpret_cast<const v4i*>(src + (size_t)q * K * 64);
      af[2 * q + 1] = *reinterpret_cast<const v4i*>(src + (size_t)q * K * 64 + 32);
    }
  };

  // ---- prologue: request everything that can be in flight -----------------------------------
  float* sc_s = rk_s + M * M * 64;  // [E]: s_e = scale_u * scale_v per position
  if (tid < E) sc_s[tid] = dq[4 * tid];
  v4i afrag[2][kFrags];  // double buffer over grid rows
  load_afrags(0, 0, afrag[0]);
  {
    // the whole ring is requested before anything is computed
    v4i st[NR][kPieces];
#pragma unroll
    for (int i = 0; i < NR; i++) load_row(i, st[i]);
#pragma unroll
    for (int i = 0; i < NR; i++) store_row(i, st[i]);
  }
  float gp[M][M];  // input-side term of this lane's tile through A^T . A
  {
    float g[E];
#pragma unroll
    for (int e = 0; e < E; e++) g[e] = (float)colsum[(size_t)e * P + prow];
#pragma unroll
    for (int a = 0; a < M; a++)
#pragma unroll
      for (int b = 0; b < M; b++) gp[a][b] = 0.0f;
#pragma unroll
    for (int e = 0; e < E; e++) {
      const float ge = dq[4 * e + 1] * g[e];
#pragma unroll
      for (int a = 0; a < M; a++)
#pragma unroll
        for (int b = 0; b < M; b++) {
          const float coef = dev::Wino<M>::at(a, e / A) * dev::Wino<M>::at(b, e % A);
          if (coef != 0.0f) gp[a][b] = __builtin_fmaf(coef, ge, gp[a][b]);
        }
    }
  }

  // output coordinates of this lane's tile
  const int tx = prow % tw, t2 = prow / tw;
  const int ty = t2 % th, n = t2 / th;
  const bool pair_ok = (M == 2) && (tx * M + 1 < Wo) && ((Wo & 1) == 0);

  for (int kb = 0; kb < nkb; kb++) {
    const int kb0 = kb * 64;
    __syncthreads();  // the previous block's tail has read rk_s; first block: the ring is filled
    for (int i2 = tid; i2 < M * M * 64; i2 += kThreads) {
      const int ab = i2 >> 6, kk = i2 & 63;
      rk_s[i2] = rk[(size_t)ab * K + min(kb0 + kk, K - 1)];
    }

    float out[M][M][16];
#pragma unroll
    for (int a = 0; a < M; a++)
#pragma unroll
      for (int b = 0; b < M; b++)
#pragma unroll
        for (int r = 0; r < 16; r++) out[a][b][r] = 0.0f;

    // one grid row: products of its (m+2) positions from the ring slot, folded into out[][]
    auto do_row = [&](int i, const v4i (&af)[kFrags], v4i (&af_next)[kFrags]) {
      const int s = kb * A + i;  // step number
      // request the A fragments of the next step: they arrive while this row is multiplied
      {
        const int in = (i + 1 == A) ? 0 : i + 1, kbn = (i + 1 == A) ? kb + 1 : kb;
        if (s + 1 < total) load_afrags(kbn, in, af_next);
      }
      // ring refill: the slot of the previous step is free since the barrier that ended it
      v4i st[kPieces];
      const bool refill = (NR < A) && s >= 1 && (s - 1 + NR) < total;
      if (refill) load_row((i - 1 + NR + A) % A, st);

      const char* slot = ring + (i % NR) * kSlotBytes;
      float rowacc[M][16];  // sum_j A^T[b][j] * s_e * ACC[e = (i, j)]
#pragma unroll
      for (int b = 0; b < M; b++)
#pragma unroll
        for (int r = 0; r < 16; r++) rowacc[b][r] = 0.0f;
#pragma unroll
      for (int j = 0; j < A; j++) {
        v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int cb = 0; cb < NB; cb++) {
          const int q = j * NB + cb;
          const v4i b0 = *reinterpret_cast<const v4i*>(slot + q * 4096 + f_off0);
          const v4i b1 = *reinterpret_cast<const v4i*>(slot + q * 4096 + f_off1);
          acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[2 * q], b0, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[2 * q + 1], b1, acc, 0, 0, 0);
        }
        const float se = sc_s[i * A + j];
#pragma unroll
        for (int b = 0; b < M; b++) {
          const float coef = dev::Wino<M>::at(b, j);  // compile-time: zero terms vanish
          if (coef != 0.0f) {
            const float cs = coef * se;
#pragma unroll
            for (int r = 0; r < 16; r++)
              rowacc[b][r] = __builtin_fmaf(cs, (float)acc[r], rowacc[b][r]);
          }
        }
      }
      // out[a][b] += A^T[a][i] * rowacc[b]   (i is a run-time value)
#pragma unroll
      for (int a = 0; a < M; a++) {
        const float ca = dev::at_coef(M, a, i);
#pragma unroll
        for (int b = 0; b < M; b++)
#pragma unroll
          for (int r = 0; r < 16; r++) out[a][b][r] = __builtin_fmaf(ca, rowacc[b][r], out[a][b][r]);
      }
      if (NR < A) {
        if (refill) store_row((i - 1 + NR) % NR, st);
        __syncthreads();
      }
    };
#pragma nounroll
    for (int i = 0; i < A; i += 2) {  // A is even: the two fragment buffers alternate
      do_row(i, afrag[0], afrag[1]);
      do_row(i + 1, afrag[1], afrag[0]);
    }

    if (NR == A) __syncthreads();  // rk_s written (any block) -- no barrier inside the row loop
    // ---- tail of this filter block: add the two separable terms, store the m x m patches ----
    const int k0 = kb0 + (wave >> 1) * 32;
    if (p < P && k0 < K) {
      const float* rk_l = rk_s + (wave >> 1) * 32 + 4 * half;
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
                  if (xx < Wo) yk[(size_t)yy * Wo + xx] = o[b];
                }
              }
            }
          }
        }
      }
    }
  }
}

template <int M, int NB, int NR>
hipError_t launch_variant(const Geo& g, const int8_t* uq, const int8_t* vq, const int32_t* colsum,
                          const float* dq, const float* rk, float* y, hipStream_t s) {
  constexpr int A = M + 2;
  const size_t lds = (size_t)NR * A * NB * 4096 + ((size_t)M * M * 64 + A * A) * sizeof(float);
  auto kern = gemm_fused_lds_kernel<M, NB, NR>;
  if (lds > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  kern<<<(g.P + 63) / 64, kThreads, lds, s>>>(uq, vq, colsum, dq, rk, y, g.K, g.P, g.th, g.tw,
                                               g.Ho, g.Wo);
  return hipGetLastError();
}

}  // namespace

// Built for F(2x2,3x3) with one 64-channel block (the ring then holds the whole position grid in
// 64 KB and the register budget allows two workgroups per CU); other shapes use gemm_i8.hip.
bool gemm_fused_lds_applicable(const Geo& g) { return g.m == 2 && g.CB == 64 && g.NB == 1; }

hipError_t launch_gemm_fused_lds(const Geo& g, const int8_t* uq, const int8_t* vq,
                                 const int32_t* colsum, const float* dq, const float* rk, float* y,
                                 hipStream_t s) {
  return launch_variant<2, 1, 4>(g, uq, vq, colsum, dq, rk, y, s);
}

}  // namespace lance
