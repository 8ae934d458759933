// Stages 2 (second pass) + 3 + 4 in one kernel for F(2x2,3x3) layers with one 64-channel block:
// v^ = Q(B^T d B) (Algorithm 1; Eq. 7) is formed in registers and written to LDS only, the int8
// products of Sec. 3.3 run on the matrix cores from there, and the de-quantization (Eq. 8) and
// output transform (Eq. 9) are applied to the register accumulators.  The codes of V never
// touch device memory; the ranges come from the range pass and its reduction.
//
// A workgroup of four waves owns 64 consecutive tiles p and all filters.
//
// Phase T (transform + quantize into LDS): quant_phase.h.  Phase R (range reduction + constants)
// runs inside it, after the first patch loads have been requested.
//
// Phase G (products + epilogue).  Wave (w & 1) takes the tiles 32(w & 1).., wave (w >> 1) the
// filters 32(w >> 1).. of each 64-filter block; the B fragments come from LDS, the A fragments
// (uq, cache resident) from memory one grid row ahead.  Epilogue algebra:
// M[e,k,p] = s_e*ACC + f[e,k] + g[e,p]; the three terms go through the linear map S = A^T M A
// separately; f arrives pre-transformed in rk[a*m+b][k], g is formed from the column sums.
#include "lance_device.h"
#include "lance_internal.h"
#include "patch_loader.h"
#include "quant_phase.h"
#include "quant_phase_nhwc.h"

namespace lance {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;

struct CfArgs {
  const float* x;
  const int8_t* uq;
  const float* u_range;      // [E][2]
  const int32_t* u_rowsum;   // [E][K]
  const float* partial;      // [count][E][2] records of the range pass
  float* v_range;            // [E][2]: written by workgroup 0, or read when is_static
  float* y;
  int count, per_tensor, is_static;
  int N, C, H, W, K, pad, P, th, tw, Ho, Wo, bits, bits_w;
  unsigned reach;  // bytes from the plane (first image of a block, channel) that tiles of the block may read
  unsigned y_bytes;
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

// B8: 8-bit codes.  FULL: all 64 channels of the block exist.  MODE: patch load mode
// (patch_load_mode), or kModeNhwc: X is [N][H][W][C] and Y is [N][Ho][Wo][K] (C a multiple of 4).
constexpr int kModeNhwc = 3;
template <bool B8, bool FULL, int MODE>
__global__ __launch_bounds__(kThreads, 2) void conv_fused_c64_kernel(const CfArgs a) {
  constexpr int M = 2, A = 4, E = 16;
  constexpr int kFrags = A * 2;  // A fragments (16 B per lane) per grid row
  extern __shared__ char smem[];
  char* ring = smem;                                       // [E][64 rows][64 B]
  float* rk_s = reinterpret_cast<float*>(smem + E * 4096);  // [64 filters][M*M]
  float* sc_s = rk_s + M * M * 64;                          // [E] s_e = scale_u * scale_v
  int* cs_s = reinterpret_cast<int*>(sc_s + E);             // [E][64] column sums (unsigned codes)
  float* res_s = reinterpret_cast<float*>(cs_s + E * 64);   // [E][2] reduced ranges
  float* qp_s = res_s + 2 * E;                              // [E][2] = {min, inv} of Eq. 7
  float* gc_s = qp_s + 2 * E;                               // [E] scale_v * offset_u
  double* rmul_s = reinterpret_cast<double*>(gc_s + E);     // [E] scale_u * offset_v
  double* kconst_s = rmul_s + E;                            // [E] C * offset_u * offset_v

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int p0 = dev::xcd_contiguous(blockIdx.x, gridDim.x) * 64;
  const int K = a.K, P = a.P;

  // ---- phase R (runs inside phase T, after the first patch loads have been requested) ----
  // Every workgroup reduces the range pass's records for itself (64 KB from L2 at most, far
  // cheaper than a kernel of its own between the two passes) and forms the constants of Eq. 7
  // and of the expanded Eq. 8.  With ou = min_u + su*h, ov = min_v + sv*h:
  //   M[e,k,p] = su*sv*ACC + (su*ov*rowsum[e][k] + C*ou*ov) + sv*ou*colsum[e][p].
  auto rk_rows = [&](int kb, int32_t (&rs)[E]) {  // thread = (ab = wave, filter kk = lane)
    const int k = min(kb * 64 + lane, K - 1);
#pragma unroll
    for (int e = 0; e < E; e++) rs[e] = a.u_rowsum[(size_t)e * K + k];
  };
  auto rk_store = [&](auto&& rowsum_of) {  // rk_s[kk][ab] = sum_e A^T[a][i] A^T[b][j] f[e,k]
    // (a, b) from a copy of the wave number the compiler cannot see through: the 16 binary64
    // coefficients are then formed at each call instead of living in registers between calls
    int w = wave;
    asm volatile("" : "+s"(w));
    const int aa = w >> 1, b = w & 1;
    double acc = 0.0;
#pragma unroll
    for (int e = 0; e < E; e++) {
      const double coef = (double)dev::at_coef(M, aa, e / A) * (double)dev::at_coef(M, b, e % A);
      acc += coef * (rmul_s[e] * (double)rowsum_of(e) + kconst_s[e]);
    }
    rk_s[4 * lane + wave] = (float)acc;
  };

  // ============================ phase T ============================
  // (quant_phase.h; phase R runs inside it, under the latency of the first patch loads)
  {
    const dev::QuantBlockGeo qg{a.x, a.N, a.C, a.H, a.W, a.pad, a.th, a.tw, a.P, a.bits, a.reach};
    auto phase_r = [&]() {
      // filter row sums of the first filter block: each wave fetches four of the 16 positions
      // and shares them through LDS (the ring is free until phase T ends)
      int* rs_s = reinterpret_cast<int*>(ring + 4096);  // [E][64]
      int32_t rs4[4];
      {
        const int k = min(lane, K - 1);
#pragma unroll
        for (int i = 0; i < 4; i++) rs4[i] = a.u_rowsum[(size_t)(4 * wave + i) * K + k];
      }
      for (int i = tid; i < E * 64; i += kThreads) cs_s[i] = 0;
      float* red = reinterpret_cast<float*>(ring);  // [4 waves][2E], free until phase T ends
      typedef float f4 __attribute__((ext_vector_type(4)));
      f4 v = {INFINITY, -INFINITY, INFINITY, -INFINITY};  // {min, max} of positions 2*qd, 2*qd+1
      const int qd = lane & 7;                            // 16-byte piece of a 128-byte record
      if (!a.is_static) {
        // records rg, rg + 32, ...; all loads of a batch are requested before the first is used
        constexpr int kBatch = 16, kRowGroups = kThreads / 8;
        for (int row0 = tid >> 3; row0 < a.count; row0 += kBatch * kRowGroups) {
          f4 xv[kBatch];
#pragma unroll
          for (int u = 0; u < kBatch; u++) {
            const int row = row0 + u * kRowGroups;
            xv[u] = row < a.count
                        ? *reinterpret_cast<const f4*>(a.partial + (size_t)row * (2 * E) + 4 * qd)
                        : v;
          }
#pragma unroll
          for (int u = 0; u < kBatch; u++) {
            v[0] = fminf(v[0], xv[u][0]); v[1] = fmaxf(v[1], xv[u][1]);
            v[2] = fminf(v[2], xv[u][2]); v[3] = fmaxf(v[3], xv[u][3]);
          }
        }
      }
      // filter-side parameters: independent of the records, computed under the load latency
      float su = 0.0f;
      double ou = 0.0;
      if (tid < E) {
        float iu;
        dev::quant_params(a.u_range[2 * tid], a.u_range[2 * tid + 1], a.bits_w, &iu, &su);
        ou = (double)a.u_range[2 * tid] + (double)su * (double)(1 << (a.bits_w - 1));
      }
      if (a.is_static) {
        if (tid < 2 * E) res_s[tid] = a.v_range[tid];
      } else {
#pragma unroll
        for (int o = 8; o < 64; o <<= 1) {  // lanes with the same qd
          v[0] = fminf(v[0], __shfl_xor(v[0], o, 64)); v[1] = fmaxf(v[1], __shfl_xor(v[1], o, 64));
          v[2] = fminf(v[2], __shfl_xor(v[2], o, 64)); v[3] = fmaxf(v[3], __shfl_xor(v[3], o, 64));
        }
        if (lane < 8) *reinterpret_cast<f4*>(red + wave * 2 * E + 4 * lane) = v;
      }
#pragma unroll
      for (int i = 0; i < 4; i++) rs_s[(4 * wave + i) * 64 + lane] = rs4[i];
      __syncthreads();
      if (!a.is_static && tid < 2 * E) {
        const bool is_max = tid & 1;
        float r = red[tid];
#pragma unroll
        for (int w2 = 1; w2 < kThreads / 64; w2++) {
          const float x2 = red[w2 * 2 * E + tid];
          r = is_max ? fmaxf(r, x2) : fminf(r, x2);
        }
        res_s[tid] = r;
      }
      __syncthreads();
      if (tid < E) {
        float lo = res_s[2 * tid], hi = res_s[2 * tid + 1];
        if (a.per_tensor && !a.is_static) {
          for (int e = 0; e < E; e++) { lo = fminf(lo, res_s[2 * e]); hi = fmaxf(hi, res_s[2 * e + 1]); }
        }
        if (!a.is_static && blockIdx.x == 0) {
          a.v_range[2 * tid] = lo;
          a.v_range[2 * tid + 1] = hi;
        }
        float inv, sv;
        dev::quant_params(lo, hi, a.bits, &inv, &sv);
        const double ov = (double)lo + (double)sv * (double)(1 << (a.bits - 1));
        qp_s[2 * tid] = lo;
        qp_s[2 * tid + 1] = inv;
        sc_s[tid] = (float)((double)su * (double)sv);
        gc_s[tid] = (float)((double)sv * ou);
        rmul_s[tid] = (double)su * ov;
        kconst_s[tid] = (double)a.C * ou * ov;
      }
      __syncthreads();
      rk_store([&](int e) { return rs_s[e * 64 + lane]; });
    };
    auto qp = [&](int e, float* mn, float* inv) { *mn = qp_s[2 * e]; *inv = qp_s[2 * e + 1]; };
    if constexpr (MODE == kModeNhwc)
      dev::quantize_block_nhwc_to_lds<B8, 64, 1>(qg, p0, ring, cs_s, tid, phase_r, qp);
    else
      dev::quantize_block_to_lds<B8, FULL, MODE>(qg, p0, 0, ring, cs_s, lane, wave, phase_r, qp);
  }

  // ============================ phase G ============================
  // The index arithmetic of this phase starts from a lane number the compiler cannot see
  // through: otherwise it is hoisted above phase T and held in registers (or spilled) across it.
  int lane_g = lane;
  asm volatile("" : "+v"(lane_g)::"memory");
  const int col = lane_g & 31, half = lane_g >> 5;
  const int prow_l = (wave & 1) * 32 + col;  // this lane's tile row inside the block
  const int p = p0 + prow_l;
  const int prow = min(p, P - 1);
  const int nkb = (K + 63) / 64;
  const int total = nkb * A;  // (filter block, grid row) steps
  // fragment read offsets of this lane inside a 4 KB position plane (k-halves 0 and 1)
  const unsigned f_off0 = (unsigned)prow_l * 64u + (unsigned)(((0 + half) ^ dev::row_swizzle(prow_l)) * 16);
  const unsigned f_off1 = (unsigned)prow_l * 64u + (unsigned)(((2 + half) ^ dev::row_swizzle(prow_l)) * 16);

  auto load_afrags = [&](int kb, int i, v4i (&af)[kFrags]) {  // uq fragments of grid row i
    const int krow = min(kb * 64 + (wave >> 1) * 32 + col, K - 1);
    const int8_t* src = a.uq + ((size_t)i * A * K + krow) * 64 + 16 * half;
#pragma unroll
    for (int q = 0; q < A; q++) {
      af[2 * q] = *reinterpret_cast<const v4i*>(src + (size_t)q * K * 64);
      af[2 * q + 1] = *reinterpret_cast<const v4i*>(src + (size_t)q * K * 64 + 32);
    }
  };
  v4i afrag[2][kFrags];  // double buffer over grid rows
  load_afrags(0, 0, afrag[0]);
  __syncthreads();  // codes and column sums of all four waves are in LDS

  float gp[M][M];  // input-side term of this lane's tile through A^T . A
  {
    const int ch_h = a.C * (int)(1u << (a.bits - 1));  // signed code = unsigned code - h
#pragma unroll
    for (int aa = 0; aa < M; aa++)
#pragma unroll
      for (int b = 0; b < M; b++) gp[aa][b] = 0.0f;
#pragma unroll
    for (int e = 0; e < E; e++) {
      const float ge = gc_s[e] * (float)(cs_s[e * 64 + prow_l] - ch_h);
#pragma unroll
      for (int aa = 0; aa < M; aa++)
#pragma unroll
        for (int b = 0; b < M; b++) {
          const float coef = dev::Wino<M>::at(aa, e / A) * dev::Wino<M>::at(b, e % A);
          if (coef != 0.0f) gp[aa][b] = __builtin_fmaf(coef, ge, gp[aa][b]);
        }
    }
  }

  // output coordinates of this lane's tile
  const int tx = prow % a.tw, t2 = prow / a.tw;
  const int ty = t2 % a.th, n = t2 / a.th;
  const int Ho = a.Ho, Wo = a.Wo;

  for (int kb = 0; kb < nkb; kb++) {
    const int kb0 = kb * 64;
    if (kb > 0) {
      int32_t rs[E];
      rk_rows(kb, rs);
      __syncthreads();  // the previous block's tail has read rk_s
      rk_store([&](int e) { return rs[e]; });
    }

    float out[M][M][16];
#pragma unroll
    for (int aa = 0; aa < M; aa++)
#pragma unroll
      for (int b = 0; b < M; b++)
#pragma unroll
        for (int r = 0; r < 16; r++) out[aa][b][r] = 0.0f;

    // one grid row: products of its four positions, folded into out[][]
    auto do_row = [&](int i, const v4i (&af)[kFrags], v4i (&af_next)[kFrags]) {
      const int s = kb * A + i;  // step number
      {  // request the A fragments of the next step: they arrive while this row is multiplied
        const int in = (i + 1 == A) ? 0 : i + 1, kbn = (i + 1 == A) ? kb + 1 : kb;
        if (s + 1 < total) load_afrags(kbn, in, af_next);
      }
      const char* slot = ring + i * (A * 4096);
      float rowacc[M][16];  // sum_j A^T[b][j] * s_e * ACC[e = (i, j)]
#pragma unroll
      for (int b = 0; b < M; b++)
#pragma unroll
        for (int r = 0; r < 16; r++) rowacc[b][r] = 0.0f;
#pragma unroll
      for (int j = 0; j < A; j++) {
        v16i acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        const v4i b0 = *reinterpret_cast<const v4i*>(slot + j * 4096 + f_off0);
        const v4i b1 = *reinterpret_cast<const v4i*>(slot + j * 4096 + f_off1);
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[2 * j], b0, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[2 * j + 1], b1, acc, 0, 0, 0);
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
      for (int aa = 0; aa < M; aa++) {
        const float ca = dev::at_coef(M, aa, i);
#pragma unroll
        for (int b = 0; b < M; b++)
#pragma unroll
          for (int r = 0; r < 16; r++)
            out[aa][b][r] = __builtin_fmaf(ca, rowacc[b][r], out[aa][b][r]);
      }
    };
#pragma nounroll
    for (int i = 0; i < A; i += 2) {  // the two fragment buffers alternate
      do_row(i, afrag[0], afrag[1]);
      do_row(i + 1, afrag[1], afrag[0]);
    }

    __syncthreads();  // rk_s written -- no barrier inside the row loop
    // ---- tail of this filter block: add the two separable terms, store the 2x2 patches.
    // Stores that must not happen (tiles past P, filters past K, the second row or column of a
    // patch cut by an odd output size) get an offset beyond the buffer instead of a branch. ----
    {
      typedef float v4f __attribute__((ext_vector_type(4)));
      const int kfirst = kb0 + (wave >> 1) * 32 + 4 * half;  // this lane's first filter
      float o[16][M][M];
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int kk = 8 * (r / 4) + (r % 4);
        const v4f f4 = *reinterpret_cast<const v4f*>(rk_s + 4 * ((wave >> 1) * 32 + 4 * half + kk));
#pragma unroll
        for (int aa = 0; aa < M; aa++)
#pragma unroll
          for (int b = 0; b < M; b++) o[r][aa][b] = (out[aa][b][r] + f4[aa * M + b]) + gp[aa][b];
      }
      if constexpr (MODE == kModeNhwc) {
        // the lane's filters come in groups of four consecutive ones: one store per group and pixel
        const bool k4 = (K & 3) == 0;
#pragma unroll
        for (int aa = 0; aa < M; aa++)
#pragma unroll
          for (int b = 0; b < M; b++) {
            const int oy = ty * M + aa, ox = tx * M + b;
            const bool pix_ok = p < P && oy < Ho && ox < Wo;
            const unsigned pix = (((unsigned)n * (unsigned)Ho + (unsigned)oy) * (unsigned)Wo +
                                  (unsigned)ox) * (unsigned)K * 4u;
#pragma unroll
            for (int rq = 0; rq < 4; rq++)
              dev::store_nhwc_k4(a.y, a.y_bytes, pix, (unsigned)(kfirst + 8 * rq) * 4u, pix_ok,
                                 K - (kfirst + 8 * rq), k4, o[4 * rq][aa][b], o[4 * rq + 1][aa][b],
                                 o[4 * rq + 2][aa][b], o[4 * rq + 3][aa][b]);
          }
      } else {
        const unsigned Wo_u = (unsigned)Wo, plane = (unsigned)Ho * Wo_u;
        const unsigned base = (((unsigned)n * (unsigned)K + (unsigned)kfirst) * plane +
                               (unsigned)(ty * M) * Wo_u + (unsigned)(tx * M)) * 4u;
        store_patches(a.y, a.y_bytes, o, base, plane * 4u, Wo_u * 4u, K - kfirst, p < P,
                      ty * M + 1 < Ho, tx * M + 1 < Wo, (Wo & 1) == 0);
      }
    }
  }
}

constexpr size_t kLdsBytes = 16 * 4096 + (2 * 2 * 64 + 16) * sizeof(float) + 16 * 64 * sizeof(int) +
                             (32 + 32 + 16) * sizeof(float) + 2 * 16 * sizeof(double);

}  // namespace

// F(2x2,3x3), one 64-channel block, and byte offsets below 2^31 from the first image of a
// workgroup to every pixel its 64 tiles read.
static long long block_reach_bytes(const Geo& g) {
  const long long tiles = (long long)g.th * g.tw;
  const long long images = 63 / tiles + 2;  // images a block of 64 consecutive tiles can touch
  return images * g.C * g.H * g.W * 4LL;
}

bool conv_fused_c64_applicable(const Geo& g) {
  if (!(g.m == 2 && g.CB == 64 && g.NB == 1)) return false;
  if ((long long)g.N * g.K * g.Ho * g.Wo * 4 >= 0xFFFFFFF0LL) return false;  // 32-bit store offsets
  // NHWC: 16-byte pixel loads of four channels at 32-bit offsets; the caller checks X's alignment
  if (is_nhwc(g)) return g.C % 4 == 0 && (long long)g.N * g.C * g.H * g.W * 4 < 0xFFFFFFF0LL;
  return block_reach_bytes(g) < (1LL << 31);
}

template <bool B8, bool FULL, int MODE>
static hipError_t launch_variant(const CfArgs& a, unsigned grid, hipStream_t s) {
  auto kern = conv_fused_c64_kernel<B8, FULL, MODE>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes);
  if (e != hipSuccess) return e;
  note_kernel("conv_fused_c64_kernel");
  kern<<<grid, kThreads, kLdsBytes, s>>>(a);
  return hipGetLastError();
}

template <bool B8, bool FULL>
static hipError_t launch_rows(const Geo& g, const CfArgs& a, unsigned grid, hipStream_t s) {
  switch (patch_load_mode(g)) {
    case 0: return launch_variant<B8, FULL, 0>(a, grid, s);
    case 1: return launch_variant<B8, FULL, 1>(a, grid, s);
    default: return launch_variant<B8, FULL, 2>(a, grid, s);
  }
}

hipError_t launch_conv_fused_c64(const Geo& g, const float* x, const int8_t* uq,
                                 const float* u_range, const int32_t* u_rowsum,
                                 const float* partial, int count, float* v_range, float* y,
                                 hipStream_t s) {
  if (!conv_fused_c64_applicable(g)) return hipErrorInvalidValue;
  CfArgs a{x, uq, u_range, u_rowsum, partial, v_range, y, count,
           (g.flags & LANCE_RANGE_PER_TENSOR) ? 1 : 0, (g.flags & LANCE_INPUT_RANGE_STATIC) ? 1 : 0,
           g.N, g.C, g.H, g.W, g.K, g.pad, g.P, g.th, g.tw, g.Ho, g.Wo, g.bits, g.bits_w,
           is_nhwc(g) ? (unsigned)((size_t)g.N * g.C * g.H * g.W * 4) : (unsigned)block_reach_bytes(g),
           (unsigned)((size_t)g.N * g.K * g.Ho * g.Wo * 4)};
  const unsigned grid = (unsigned)((g.P + 63) / 64);
  const bool b8 = g.bits == 8, full = g.C == 64;
  if (is_nhwc(g)) {
    if ((reinterpret_cast<uintptr_t>(x) & 15) != 0) return hipErrorInvalidValue;
    return b8 ? launch_variant<true, false, kModeNhwc>(a, grid, s)
              : launch_variant<false, false, kModeNhwc>(a, grid, s);
  }
  if (b8) return full ? launch_rows<true, true>(g, a, grid, s) : launch_rows<true, false>(g, a, grid, s);
  return full ? launch_rows<false, true>(g, a, grid, s) : launch_rows<false, false>(g, a, grid, s);
}

}  // namespace lance
