// Stages 2 (second pass) + 3 + 4 in one kernel for F(4x4,3x3) layers with at most two 64-channel
// blocks (C <= 128): v^ = Q(B^T d B) (Algorithm 1; Eq. 7) is formed in registers and written to
// LDS only (36 KB of codes per channel block for 16 tiles), the int8 products of Sec. 3.3 run on
// the matrix cores from there, and the de-quantization (Eq. 8) and output transform (Eq. 9) are
// applied to the register accumulators.  The codes of V never touch device memory.  With
// caller-supplied ranges (Sec. 3.4's inference mode) this kernel is the whole call.
//
// A workgroup of four waves owns 16 consecutive tiles p and all filters; two workgroups (three
// with one channel block) share a compute unit, so that one's transform phase (vector ALUs) runs
// under the other's product phase (loads of uq, LDS reads, matrix cores).
//
// Phase T: quant_phase_m4.h, channels 0..63 then channels 64..127, each into its own code planes;
// the column sums of both add up in one table.  The Eq. 7 / Eq. 8 constants come either finished
// from the reduction kernel (qparams, dq, dqd) or are formed here from the caller's ranges or from
// a few range records (range_reduce.h), after the first patch loads have been requested.
//
// Phase G: filters in blocks of 64; wave w takes filters 16w.. of the block and all 16 tiles
// (one v_mfma_i32_16x16x64_i8 per position and channel block).  The B fragments come from LDS two
// positions ahead, the A fragments (uq, cache resident) from memory five positions ahead (a ring
// of six register buffers, buffer loads with the position's plane as scalar offset), and the
// matrix instructions of position e+1 are issued before the fold of position e; the 36 positions
// are unrolled, so the fold coefficients are compile-time constants (m4_fold.h).  Epilogue algebra:
// M[e,k,p] = s_e*ACC + f[e,k] + g[e,p]; the three terms go through the linear map S = A^T M A
// separately; f is formed here from the filter row sums (binary64), g from the column sums.
//
// Measured on the 128-channel 56 x 56 layer at N = 64 by leaving phases out: 10 us of constants and
// filter-side terms, 29 us of phase T, 43 us of phase G, and they add up (83 us): the two workgroups
// of a compute unit start together and stay in step.  Phase G is bound by instruction issue: per
// position and accumulator register one conversion and about five multiply-adds of the fold stand
// against a quarter of a matrix instruction; neither a deeper fragment ring (11 positions) nor
// the order of products and fold changed its time.  A variant with one workgroup of eight waves
// per compute unit - four waves quantizing tile block i+1 into one half of LDS while four
// multiply block i from the other half, one barrier per block - was built and passed parity, and
// was slower (107 us): a lone product wave per SIMD issues one instruction per five to six cycles,
// and every tail (filter-side terms, input-side terms, stores: 3 us per 64 filters) sits on its
// critical path.
#include "lance_device.h"
#include "lance_internal.h"
#include "m4_fold.h"
#include "patch_loader.h"
#include "quant_phase_m4.h"
#include "range_reduce.h"

namespace lance {
namespace {

using m4e::m4_fold;
using m4e::static_for;
using m4e::v4f;
typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kTiles = 16;
constexpr int kE = 36;
constexpr int kPlane = kTiles * 64;        // code plane of one position: 1 KB
constexpr int kBlockPlanes = kE * kPlane;  // code planes of one channel block: 36 KB
constexpr int kFilters = 64;               // filters per pass of phase G

struct C4Args {
  const float* x;
  const int8_t* uq;
  const int32_t* u_rowsum;  // [E][K]
  float* y;
  dev::RangeSource rs;  // merge == 0: finished qparams (then dq / dqd below are finished too)
  const float* dq;      // [E][4]  (merge == 0)
  const double* dqd;    // [E][2]  (merge == 0)
  int N, C, H, W, K, pad, P, th, tw, Ho, Wo, bits;
  unsigned reach;  // bytes from the plane (first image of a block, channel) that tiles of the block may read
};

// LDS carve-up behind the code planes
struct Lds {
  float* rk_s;       // [16 outputs][64 filters]
  int* cs_s;         // [E][16] column sums (unsigned codes)
  float* sc_s;       // [E] s_e = scale_u * scale_v
  float* gc_s;       // [E] scale_v * offset_u
  float* res_s;      // [E][2] reduced ranges
  float* qp_s;       // [E][2] = {min, inv} of Eq. 7
  double* rmul_s;    // [E] scale_u * offset_v
  double* kconst_s;  // [E] C * offset_u * offset_v
};
constexpr size_t kTailBytes = 16 * kFilters * sizeof(float) + kE * kTiles * sizeof(int) +
                              (2 + 2 + 2) * kE * sizeof(float) + 2 * kE * sizeof(double);

__device__ __forceinline__ Lds carve(char* p) {
  Lds l;
  l.rmul_s = reinterpret_cast<double*>(p);  // the doubles first: 8-byte aligned
  l.kconst_s = l.rmul_s + kE;
  l.rk_s = reinterpret_cast<float*>(l.kconst_s + kE);
  l.cs_s = reinterpret_cast<int*>(l.rk_s + 16 * kFilters);
  l.sc_s = reinterpret_cast<float*>(l.cs_s + kE * kTiles);
  l.gc_s = l.sc_s + kE;
  l.res_s = l.gc_s + kE;
  l.qp_s = l.res_s + 2 * kE;
  return l;
}

// B8: 8-bit codes.  FULL: all 64 * NB channels exist.  MODE: patch load mode (patch_load_mode).
// NB: channel blocks (1 or 2).
template <bool B8, bool FULL, int MODE, int NB>
__global__ __launch_bounds__(kThreads, 2) void conv_fused_m4_kernel(const C4Args a) {
  constexpr int M = 4, A = 6, E = kE;
  constexpr int kAhead = 5;  // positions whose A fragments are in flight ahead of the products
  static_assert(E % (kAhead + 1) == 0, "the fragment ring keeps its phase across filter blocks");
  extern __shared__ char smem[];
  char* ring = smem;  // [NB][E][16 rows][64 B]
  const Lds l = carve(smem + NB * kBlockPlanes);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int p0 = dev::xcd_contiguous(blockIdx.x, gridDim.x) * kTiles;
  const int K = a.K, P = a.P;

  // rk_s[(a*4 + b)*64 + filter] = sum_e A^T[a][i] A^T[b][j] (su*ov*rowsum[e][k] + C*ou*ov) for the
  // 64 filters of block kb, in binary64: thread = (a = wave, filter = lane), all four b
  auto rk_block = [&](int kb) {
    // a from a copy of the wave number the compiler cannot see through: the binary64
    // coefficients are then formed at each call instead of living in registers between calls
    int w = wave;
    asm volatile("" : "+s"(w));
    const int k = min(kb * kFilters + lane, K - 1);
    double ca[A], cb[M][A];
#pragma unroll
    for (int i = 0; i < A; i++) {
      ca[i] = (double)dev::at_coef(M, w, i);
#pragma unroll
      for (int b = 0; b < M; b++) cb[b][i] = (double)dev::at_coef(M, b, i);
    }
    int32_t rs[E];
#pragma unroll
    for (int e = 0; e < E; e++) rs[e] = a.u_rowsum[(size_t)e * K + k];
    double acc[M] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int e = 0; e < E; e++) {
      const double f = l.rmul_s[e] * (double)rs[e] + l.kconst_s[e];
      const double ci = ca[e / A];
#pragma unroll
      for (int b = 0; b < M; b++) acc[b] += ci * cb[b][e % A] * f;
    }
#pragma unroll
    for (int b = 0; b < M; b++) l.rk_s[(w * M + b) * kFilters + lane] = (float)acc[b];
  };

  // ============================ phase T ============================
  {
    const dev::QuantBlockGeo qg{a.x, a.N, a.C, a.H, a.W, a.pad, a.th, a.tw, a.P, a.bits, a.reach};
    auto phase_r = [&]() {
      for (int i = tid; i < E * kTiles; i += kThreads) l.cs_s[i] = 0;
      const dev::Eq8Lds lds{l.sc_s, l.gc_s, l.rmul_s, l.kconst_s};
      // the code planes are free until the first codes are written
      dev::ranges_to_lds<E>(a.rs, reinterpret_cast<float*>(ring), l.res_s, l.qp_s, tid,
                            blockIdx.x == 0, a.rs.merge ? &lds : nullptr);
      if (!a.rs.merge) {  // the reduction kernel left the constants in memory
        if (tid < E) {
          l.sc_s[tid] = a.dq[4 * tid];
          l.gc_s[tid] = a.dq[4 * tid + 1];
          l.rmul_s[tid] = a.dqd[2 * tid];
          l.kconst_s[tid] = a.dqd[2 * tid + 1];
        }
        __syncthreads();
      }
      rk_block(0);
    };
    auto nothing = []() {};
    dev::quantize_m4_block16_to_lds<B8, FULL, MODE>(qg, p0, 0, ring, l.cs_s, l.qp_s, lane, wave,
                                                    phase_r);
    if constexpr (NB == 2)
      dev::quantize_m4_block16_to_lds<B8, FULL, MODE>(qg, p0, 64, ring + kBlockPlanes, l.cs_s,
                                                      l.qp_s, lane, wave, nothing);
  }

  // ============================ phase G ============================
  // The index arithmetic of this phase starts from a lane number the compiler cannot see
  // through: otherwise it is hoisted above phase T and held in registers (or spilled) across it.
  int lane_g = lane;
  asm volatile("" : "+v"(lane_g)::"memory");
  const int col = lane_g & 15, kq = lane_g >> 4;  // fragment row; 16-byte piece of the 64 channels
  const int nkb = (K + kFilters - 1) / kFilters;
  // B fragment of this lane inside a 1 KB position plane: chunk kq of the code row of tile col
  const unsigned f_off = dev::code_row_offset(col, kq);

  // uq fragments of position e: filters 16*wave + col of block kb, one per channel block, by buffer
  // loads: the lane's row in a VGPR, the (position, channel block) plane in a scalar offset
  const __amdgpu_buffer_rsrc_t uq_res = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<int8_t*>(a.uq), 0, (unsigned)((size_t)E * NB * K * 64), 0x00020000);
  unsigned uq_plane = (unsigned)K * 64u;  // bytes of one (position, channel block) plane
  auto load_afrags = [&](int kb, int e, v4i (&af)[NB]) {
    const unsigned row = (unsigned)min(kb * kFilters + wave * 16 + col, K - 1) * 64u + 16u * (unsigned)kq;
#pragma unroll
    for (int nb = 0; nb < NB; nb++)
      af[nb] = __builtin_bit_cast(
          v4i, __builtin_amdgcn_raw_buffer_load_b128(uq_res, row, (unsigned)(e * NB + nb) * uq_plane, 0));
  };
  v4i afrag[kAhead + 1][NB];  // ring over positions (36 positions = six turns)
#pragma unroll
  for (int e = 0; e < kAhead; e++) load_afrags(0, e, afrag[e]);
  __syncthreads();  // codes and column sums of all four waves are in LDS

  // input-side term of this lane's tile through A^T . A (the same for every filter)
  const int p = p0 + col;
  float gp[M][M];
  {
    const int ch_h = a.C * (int)(1u << (a.bits - 1));  // signed code = unsigned code - h
#pragma unroll
    for (int aa = 0; aa < M; aa++)
#pragma unroll
      for (int b = 0; b < M; b++) gp[aa][b] = 0.0f;
#pragma unroll
    for (int i = 0; i < A; i++) {
      float gr[M] = {0.0f, 0.0f, 0.0f, 0.0f};  // sum_j A^T[b][j] g[(i, j)]
#pragma unroll
      for (int j = 0; j < A; j++) {
        const int e = i * A + j;
        const float ge = l.gc_s[e] * (float)(l.cs_s[e * kTiles + col] - ch_h);
#pragma unroll
        for (int b = 0; b < M; b++) {
          const float coef = dev::Wino<M>::at(b, j);
          if (coef != 0.0f) gr[b] = __builtin_fmaf(coef, ge, gr[b]);
        }
      }
#pragma unroll
      for (int aa = 0; aa < M; aa++) {
        const float ca = dev::Wino<M>::at(aa, i);
#pragma unroll
        for (int b = 0; b < M; b++) gp[aa][b] = __builtin_fmaf(ca, gr[b], gp[aa][b]);
      }
    }
  }
  const int pc = min(p, P - 1);
  const int tx = pc % a.tw, t2 = pc / a.tw;
  const int ty = t2 % a.th, n = t2 / a.th;
  const int Ho = a.Ho, Wo = a.Wo;
  const bool vec_ok = (Wo % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.y) & 15) == 0);

  for (int kb = 0; kb < nkb; kb++) {
    if (kb > 0) {
      __syncthreads();  // the previous block's tail has read rk_s
      rk_block(kb);
    }
    v4f out[M][M];  // [a][b][accumulator register]
    v4f rowacc[M];  // [b][accumulator register]
#pragma unroll
    for (int aa = 0; aa < M; aa++)
#pragma unroll
      for (int b = 0; b < M; b++) out[aa][b] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int b = 0; b < M; b++) rowacc[b] = v4f{0.0f, 0.0f, 0.0f, 0.0f};

    // (a value the compiler cannot see through: the 36 * NB plane offsets are then formed where
    // they are used instead of living in scalar registers across the loop over filter blocks)
    asm volatile("" : "+s"(uq_plane));
    // B fragments of positions e+1 and e+2 and the sums of position e+1 are on their way while
    // position e is folded
    v4i bfrag[3][NB];
    auto read_b = [&](int e, v4i (&bf)[NB]) {
#pragma unroll
      for (int nb = 0; nb < NB; nb++)
        bf[nb] = *reinterpret_cast<const v4i*>(ring + nb * kBlockPlanes + e * kPlane + f_off);
    };
    auto mma = [&](const v4i (&af)[NB], const v4i (&bf)[NB]) {
      v4i acc = {0, 0, 0, 0};
#pragma unroll
      for (int nb = 0; nb < NB; nb++)
        acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[nb], bf[nb], acc, 0, 0, 0);
      return acc;
    };
    read_b(0, bfrag[0]);
    read_b(1, bfrag[1]);
    v4i acc_next = mma(afrag[0], bfrag[0]);
    float se_next = l.sc_s[0];  // the scale s_e, read one position ahead
    static_for<E>([&](auto ec) {
      constexpr int e = decltype(ec)::value;
      {  // request the A fragments kAhead positions ahead (of the next filter block at the end)
        constexpr int en = (e + kAhead) % E;
        const int kbn = e + kAhead >= E ? kb + 1 : kb;
        if (kbn < nkb) load_afrags(kbn, en, afrag[(e + kAhead) % (kAhead + 1)]);
      }
      if constexpr (e + 2 < E) read_b(e + 2, bfrag[(e + 2) % 3]);
      const v4i acc = acc_next;
      if constexpr (e + 1 < E) acc_next = mma(afrag[(e + 1) % (kAhead + 1)], bfrag[(e + 1) % 3]);
      const float se = se_next;
      if constexpr (e + 1 < E) se_next = l.sc_s[e + 1];
      m4_fold<e>(acc, se, rowacc, out);
    });

    __syncthreads();  // rk_s written -- no barrier inside the position loop
    // ---- tail of this filter block: add the two separable terms, store the 4x4 patches.  The
    // lane holds filters k0 + r (r = accumulator register) of tile p. ----
    const int kin = wave * 16 + 4 * kq;
    const int k0 = kb * kFilters + kin;
    if (p < P && k0 < K) {
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
                o[b] = (out[aa][b][r] + l.rk_s[(aa * M + b) * kFilters + kin + r]) + gp[aa][b];
              float* dst = yk + (size_t)yy * Wo + tx * M;
              if (vec_ok) {  // the tile's four columns are inside and 16-byte aligned
                *reinterpret_cast<v4f*>(dst) = v4f{o[0], o[1], o[2], o[3]};
              } else if (tx * M + 3 < Wo) {  // inside, any 4-byte alignment: still one store
                typedef float v4fu __attribute__((ext_vector_type(4), aligned(4)));
                *reinterpret_cast<v4fu*>(dst) = v4fu{o[0], o[1], o[2], o[3]};
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

constexpr size_t lds_bytes(int nb) { return (size_t)nb * kBlockPlanes + kTailBytes; }

// Bytes from the first image of a workgroup to every pixel its 16 tiles read; the lane groups of
// the transform phase read up to three channel planes above the descriptor's.
long long block_reach_bytes(const Geo& g) {
  const long long tiles = (long long)g.th * g.tw;
  const long long images = (kTiles - 1) / tiles + 2;  // images a block of consecutive tiles can touch
  return images * g.C * g.H * g.W * 4LL + 3LL * g.H * g.W * 4LL;
}

template <bool B8, bool FULL, int MODE, int NB>
hipError_t launch_variant(const C4Args& a, unsigned grid, hipStream_t s) {
  auto kern = conv_fused_m4_kernel<B8, FULL, MODE, NB>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes(NB));
  if (e != hipSuccess) return e;
  note_kernel("conv_fused_m4_kernel");
  kern<<<grid, kThreads, lds_bytes(NB), s>>>(a);
  return hipGetLastError();
}

template <bool B8, bool FULL, int NB>
hipError_t launch_rows(const Geo& g, const C4Args& a, unsigned grid, hipStream_t s) {
  switch (patch_load_mode(g)) {
    case 0: return launch_variant<B8, FULL, 0, NB>(a, grid, s);
    case 1: return launch_variant<B8, FULL, 1, NB>(a, grid, s);
    default: return launch_variant<B8, FULL, 2, NB>(a, grid, s);
  }
}

template <int NB>
hipError_t launch_blocks(const Geo& g, const C4Args& a, unsigned grid, hipStream_t s) {
  const bool b8 = g.bits == 8, full = g.C == 64 * NB;
  if (b8) return full ? launch_rows<true, true, NB>(g, a, grid, s) : launch_rows<true, false, NB>(g, a, grid, s);
  return full ? launch_rows<false, true, NB>(g, a, grid, s) : launch_rows<false, false, NB>(g, a, grid, s);
}

}  // namespace

// F(4x4,3x3) on NCHW tensors with one or two 64-channel code blocks, unpacked codes, and byte
// offsets below 2^31 from the first image of a workgroup to every pixel its 16 tiles read.
bool conv_fused_m4_applicable(const Geo& g) {
  if (!(g.m == 4 && g.CB == 64 && g.NB <= 2) || is_nhwc(g) || is_packed(g)) return false;
  return block_reach_bytes(g) < (1LL << 31) && (long long)(g.P + kTiles - 1) / kTiles < (1LL << 31);
}

// Every workgroup reads all `count` records of the range pass: worth it while that stays a small
// part of the pass (the bound of the quantize passes that reduce for themselves).
bool conv_fused_m4_can_merge(const Geo& g, int count) {
  const long long grid = (g.P + kTiles - 1) / kTiles;
  return grid * count * (8LL * g.E) <= (32LL << 20);
}

// merge != 0: the kernel forms the Eq. 7 / Eq. 8 constants itself, from v_range (static ranges)
// or from the `count` records in `partial`, and its first workgroup writes v_range (dynamic);
// merge == 0: qparams, dq and dqd are finished (launch_range_finalize with a DqOut).
hipError_t launch_conv_fused_m4(const Geo& g, const float* x, const int8_t* uq,
                                const float* u_range, const int32_t* u_rowsum,
                                const float* partial, int count, int merge, const float* qparams,
                                const float* dq, const double* dqd, float* v_range, float* y,
                                hipStream_t s) {
  if (!conv_fused_m4_applicable(g)) return hipErrorInvalidValue;
  C4Args a{};
  a.x = x; a.uq = uq; a.u_rowsum = u_rowsum; a.y = y;
  a.rs = dev::RangeSource{qparams, partial, v_range, u_range, nullptr, nullptr, count, merge ? 1 : 0,
                          (g.flags & LANCE_INPUT_RANGE_STATIC) ? 1 : 0,
                          (g.flags & LANCE_RANGE_PER_TENSOR) ? 1 : 0, g.bits, g.C, g.bits_w, 0};
  a.dq = dq; a.dqd = dqd;
  a.N = g.N; a.C = g.C; a.H = g.H; a.W = g.W; a.K = g.K; a.pad = g.pad; a.P = g.P;
  a.th = g.th; a.tw = g.tw; a.Ho = g.Ho; a.Wo = g.Wo; a.bits = g.bits;
  a.reach = (unsigned)block_reach_bytes(g);
  const unsigned grid = (unsigned)((g.P + kTiles - 1) / kTiles);
  return g.NB == 1 ? launch_blocks<1>(g, a, grid, s) : launch_blocks<2>(g, a, grid, s);
}

}  // namespace lance
