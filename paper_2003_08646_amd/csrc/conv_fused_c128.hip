// Stages 2 (second pass) + 3 + 4 in one kernel for F(2x2,3x3) layers with two 64-channel blocks
// (65 .. 128 channels): v^ = Q(B^T d B) (Algorithm 1; Eq. 7) is formed in registers and written
// to LDS only (64 KB of codes for 32 tiles), the int8 products of Sec. 3.3 run on the matrix
// cores from there, and the de-quantization (Eq. 8) and output transform (Eq. 9) are applied to
// the register accumulators.  The codes of V never touch device memory: against the general plan
// (quantize pass to memory, product kernel reading it back) a layer moves three fifths of the
// bytes.
//
// A workgroup of four waves owns 32 consecutive tiles p and all filters; two workgroups share a
// compute unit.  The two phases of a workgroup are bound by different units (phase T by the
// vector ALUs; phase G by load/store instructions, LDS reads and the matrix cores), so two
// workgroups in different phases fill each other's gaps (a first version with 64 tiles and one
// workgroup of eight waves per compute unit spent the sum of the parts: 22 us per 64 tiles).
//
// Phase T (transform + quantize into LDS): quant_phase32.h, channels 0..63 then channels 64..127,
// each into its own code planes; the column sums of both add up in one table.  The range records
// are reduced and the Eq. 7 / Eq. 8 constants formed inside it, after the first patch loads have
// been requested (range_reduce.h).
//
// Phase G (products + epilogue).  Wave w takes the filters 32w.. of each 128-filter block (two
// groups of 16) and all 32 tiles (two groups of 16): v_mfma_i32_16x16x64_i8, the B fragments
// from LDS, the A fragments (uq, cache resident) from memory three positions ahead (a ring of
// four register buffers; the 16 positions are unrolled, so the fold coefficients are +-s_e or
// absent at compile time).  Epilogue algebra: M[e,k,p] = s_e*ACC + f[e,k] + g[e,p]; the three
// terms go through the linear map S = A^T M A separately; f is formed here from the filter row
// sums (binary64), g from the column sums.
#include "lance_device.h"
#include "lance_internal.h"
#include "patch_loader.h"
#include "quant_phase32.h"
#include "quant_phase_nhwc.h"
#include "range_reduce.h"
#include <utility>

namespace lance {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kTiles = 32;
constexpr int kPlane = kTiles * 64;          // code plane of one position: 2 KB
constexpr int kBlockPlanes = 16 * kPlane;    // code planes of one channel block: 32 KB

struct CgArgs {
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

// The tail's stores: o[r][aa] = the two pixels of row aa of the 2x2 patch of filter r (counted
// from the lane's first filter), at base + r*plane_bytes + aa*row_bytes.  kleft: filters that
// exist from the lane's first one on.  even_w (kernel-uniform): the output width is even, so a
// patch never loses its second column and the pair is stored as one 8-byte store.  Masked stores
// get an offset the buffer's range check drops.
__device__ __forceinline__ void store_patches4(float* y, unsigned y_bytes, const float (&o)[4][2][2],
                                               unsigned base, unsigned plane_bytes,
                                               unsigned row_bytes, int kleft, bool tile_ok,
                                               bool row1, bool col1, bool even_w) {
  const __amdgpu_buffer_rsrc_t res = __builtin_amdgcn_make_buffer_rsrc(y, 0, y_bytes, 0x00020000);
  typedef unsigned v2u __attribute__((ext_vector_type(2)));
  constexpr unsigned kOob = 0xFFFFFFF0u;
#pragma unroll
  for (int r = 0; r < 4; r++) {
    const bool k_ok = tile_ok && r < kleft;
#pragma unroll
    for (int aa = 0; aa < 2; aa++) {
      const unsigned off = (k_ok && (aa == 0 || row1)) ? base + (unsigned)aa * row_bytes : kOob;
      if (even_w) {
        const v2u v = {__float_as_uint(o[r][aa][0]), __float_as_uint(o[r][aa][1])};
        __builtin_amdgcn_raw_buffer_store_b64(v, res, off, (unsigned)r * plane_bytes, 0);
      } else {
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o[r][aa][0]), res, off,
                                              (unsigned)r * plane_bytes, 0);
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o[r][aa][1]), res,
                                              col1 ? off + 4u : kOob, (unsigned)r * plane_bytes, 0);
      }
    }
  }
}

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

// B8: 8-bit codes.  FULL: all 128 channels exist.  MODE: patch load mode (patch_load_mode), or
// kModeNhwc: X is [N][H][W][C] (C a multiple of 4, a.reach = its size in bytes) and Y is
// [N][Ho][Wo][K].
constexpr int kModeNhwc = 3;

template <bool B8, bool FULL, int MODE>
__global__ __launch_bounds__(kThreads, 2) void conv_fused_c128_kernel(const CgArgs a) {
  constexpr int M = 2, A = 4, E = 16, NB = 2;
  constexpr int kAhead = 3;  // positions whose A fragments are in flight ahead of the products
  extern __shared__ char smem[];
  char* ring = smem;                                                 // [NB][E][32 rows][64 B]
  float* rk_s = reinterpret_cast<float*>(smem + NB * kBlockPlanes);   // [128 filters][M*M]
  float* sc_s = rk_s + M * M * 128;                                   // [E] s_e = scale_u * scale_v
  int* cs_s = reinterpret_cast<int*>(sc_s + E);                       // [E][32] column sums (unsigned codes)
  float* res_s = reinterpret_cast<float*>(cs_s + E * kTiles);         // [E][2] reduced ranges
  float* qp_s = res_s + 2 * E;                                        // [E][2] = {min, inv} of Eq. 7
  float* gc_s = qp_s + 2 * E;                                         // [E] scale_v * offset_u
  double* rmul_s = reinterpret_cast<double*>(gc_s + E);               // [E] scale_u * offset_v
  double* kconst_s = rmul_s + E;                                      // [E] C * offset_u * offset_v

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int p0 = dev::xcd_contiguous(blockIdx.x, gridDim.x) * kTiles;
  const int K = a.K, P = a.P;

  // rk_s[4*filter + ab] = sum_e A^T[a][i] A^T[b][j] (su*ov*rowsum[e][k] + C*ou*ov) for the 128
  // filters of block kb: thread = (ab = wave, filters lane and 64 + lane)
  auto rk_block = [&](int kb) {
    // (a, b) from a copy of the wave number the compiler cannot see through: the 16 binary64
    // coefficients are then formed at each call instead of living in registers between calls
    int w = wave;
    asm volatile("" : "+s"(w));
    const int aa = w >> 1, b = w & 1;
#pragma unroll
    for (int hf = 0; hf < 2; hf++) {
      const int k = min(kb * 128 + hf * 64 + lane, K - 1);
      double acc = 0.0;
#pragma unroll
      for (int e = 0; e < E; e++) {
        const double coef = (double)dev::at_coef(M, aa, e / A) * (double)dev::at_coef(M, b, e % A);
        acc += coef * (rmul_s[e] * (double)a.u_rowsum[(size_t)e * K + k] + kconst_s[e]);
      }
      rk_s[4 * (hf * 64 + lane) + wave] = (float)acc;
    }
  };

  // ============================ phase T ============================
  {
    const dev::QuantBlockGeo qg{a.x, a.N, a.C, a.H, a.W, a.pad, a.th, a.tw, a.P, a.bits, a.reach};
    auto phase_r = [&]() {
      for (int i = tid; i < E * kTiles; i += kThreads) cs_s[i] = 0;
      const dev::RangeSource src{nullptr, a.partial, a.v_range, a.u_range, nullptr, nullptr,
                                 a.count, 1, a.is_static, a.per_tensor, a.bits, a.C, a.bits_w, 0};
      const dev::Eq8Lds lds{sc_s, gc_s, rmul_s, kconst_s};
      // the code planes are free until the first codes are written
      dev::ranges_to_lds<E>(src, reinterpret_cast<float*>(ring), res_s, qp_s, tid, blockIdx.x == 0,
                            &lds);
      rk_block(0);
    };
    auto nothing = []() {};
    auto qp = [&](int e, float* mn, float* inv) { *mn = qp_s[2 * e]; *inv = qp_s[2 * e + 1]; };
    if constexpr (MODE == kModeNhwc) {
      dev::quantize_block_nhwc_to_lds<B8, kTiles, NB>(qg, p0, ring, cs_s, tid, phase_r, qp);
    } else {
      dev::quantize_half_block_to_lds<B8, FULL, MODE, 3>(qg, p0, 0, ring, cs_s, lane, wave, phase_r, qp);
      dev::quantize_half_block_to_lds<B8, FULL, MODE, 3>(qg, p0, 64, ring + kBlockPlanes, cs_s, lane,
                                                      wave, nothing, qp);
    }
  }

  // ============================ phase G ============================
  // The index arithmetic of this phase starts from a lane number the compiler cannot see
  // through: otherwise it is hoisted above phase T and held in registers (or spilled) across it.
  int lane_g = lane;
  asm volatile("" : "+v"(lane_g)::"memory");
  const int col = lane_g & 15, kq = lane_g >> 4;  // fragment row; 16-byte piece of the 64 channels
  const int nkb = (K + 127) / 128;
  // B fragment offsets of this lane inside a 2 KB position plane, one per group of 16 tiles
  unsigned f_off[2];
#pragma unroll
  for (int t = 0; t < 2; t++) {
    const int row = 16 * t + col;
    f_off[t] = (unsigned)row * 64u + (unsigned)((kq ^ dev::row_swizzle(row)) * 16);
  }

  // uq fragments of position e: [filter group][channel block]
  auto load_afrags = [&](int kb, int e, v4i (&af)[2][NB]) {
#pragma unroll
    for (int mt = 0; mt < 2; mt++) {
      const int krow = min(kb * 128 + wave * 32 + mt * 16 + col, K - 1);
      const int8_t* src = a.uq + ((size_t)e * NB * K + krow) * 64 + 16 * kq;
#pragma unroll
      for (int nb = 0; nb < NB; nb++)
        af[mt][nb] = *reinterpret_cast<const v4i*>(src + (size_t)nb * K * 64);
    }
  };
  v4i afrag[kAhead + 1][2][NB];  // ring over positions (16 positions = four turns)
#pragma unroll
  for (int e = 0; e < kAhead; e++) load_afrags(0, e, afrag[e]);
  __syncthreads();  // codes and column sums of all four waves are in LDS

  typedef float v4f __attribute__((ext_vector_type(4)));
  for (int kb = 0; kb < nkb; kb++) {
    if (kb > 0) {
      __syncthreads();  // the previous block's tail has read rk_s
      rk_block(kb);
    }

    v4f out[2][2][M * M];  // [filter group][tile group][ab][accumulator register]
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int t = 0; t < 2; t++)
#pragma unroll
        for (int ab = 0; ab < M * M; ab++) out[mt][t][ab] = v4f{0.0f, 0.0f, 0.0f, 0.0f};

    static_for<E>([&](auto ec) {
      constexpr int e = decltype(ec)::value;
      {  // request the A fragments kAhead positions ahead (of the next filter block at the end)
        constexpr int en = (e + kAhead) % E;
        const int kbn = e + kAhead >= E ? kb + 1 : kb;
        if (kbn < nkb) load_afrags(kbn, en, afrag[(e + kAhead) % (kAhead + 1)]);
      }
      const v4i(&af)[2][NB] = afrag[e % (kAhead + 1)];
      const char* plane = ring + e * kPlane;
      v4i acc[2][2];
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int t = 0; t < 2; t++) acc[mt][t] = v4i{0, 0, 0, 0};
#pragma unroll
      for (int nb = 0; nb < NB; nb++)
#pragma unroll
        for (int t = 0; t < 2; t++) {
          const v4i bf = *reinterpret_cast<const v4i*>(plane + nb * kBlockPlanes + f_off[t]);
#pragma unroll
          for (int mt = 0; mt < 2; mt++)
            acc[mt][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[mt][nb], bf, acc[mt][t], 0, 0, 0);
        }
      // Position e is complete: out[ab] += A^T[a][i] A^T[b][j] s_e ACC (coefficients +-1 or 0).
      // The empty statements tie the sums to their position (the compiler would otherwise sink
      // the folds of all positions to the first use of the outputs and keep every accumulator
      // until then).
      constexpr int gi = e / A, gj = e % A;
      const float se = sc_s[e];
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int t = 0; t < 2; t++) {
          v4f accf;
#pragma unroll
          for (int r = 0; r < 4; r++) accf[r] = (float)acc[mt][t][r];
          static_for<4>([&](auto abc) {
            constexpr int ab = decltype(abc)::value;
            constexpr float coef = kAt2[ab >> 1][gi] * kAt2[ab & 1][gj];
            if constexpr (coef != 0.0f) {
              const float c = coef * se;
#pragma unroll
              for (int r = 0; r < 4; r++)
                out[mt][t][ab][r] = __builtin_fmaf(c, accf[r], out[mt][t][ab][r]);
              asm volatile("" : "+v"(out[mt][t][ab]));
            }
          });
        }
    });

    __syncthreads();  // rk_s written -- no barrier inside the position loop
    // ---- tail of this filter block: add the two separable terms, store the 2x2 patches.  The
    // lane holds filters kfirst + r (r = accumulator register) of the tiles 16t + col.  Stores
    // that must not happen (tiles past P, filters past K, the second row or column of a patch cut
    // by an odd output size) get an offset beyond the buffer instead of a branch. ----
    {
      const int ch_h = a.C * (int)(1u << (a.bits - 1));  // signed code = unsigned code - h
      const unsigned Wo_u = (unsigned)a.Wo, plane_px = (unsigned)a.Ho * Wo_u;
#pragma unroll
      for (int t = 0; t < 2; t++) {
        const int prow_l = 16 * t + col;
        const int p = p0 + prow_l;
        const int prow = min(p, P - 1);
        float gp[M * M] = {0.0f, 0.0f, 0.0f, 0.0f};  // input-side term of the tile through A^T . A
#pragma unroll
        for (int e = 0; e < E; e++) {
          const float ge = gc_s[e] * (float)(cs_s[e * kTiles + prow_l] - ch_h);
#pragma unroll
          for (int ab = 0; ab < M * M; ab++) {
            const float coef = kAt2[ab >> 1][e / A] * kAt2[ab & 1][e % A];
            if (coef != 0.0f) gp[ab] = __builtin_fmaf(coef, ge, gp[ab]);
          }
        }
        const int tx = prow % a.tw, t2 = prow / a.tw;
        const int ty = t2 % a.th, n = t2 / a.th;
#pragma unroll
        for (int mt = 0; mt < 2; mt++) {
          const int kin = wave * 32 + mt * 16 + 4 * kq;  // first of the lane's four filters in the block
          const int kfirst = kb * 128 + kin;
          const unsigned base = (((unsigned)n * (unsigned)K + (unsigned)kfirst) * plane_px +
                                 (unsigned)(ty * M) * Wo_u + (unsigned)(tx * M)) * 4u;
          float o[4][M][M];
#pragma unroll
          for (int r = 0; r < 4; r++) {
            const v4f f4 = *reinterpret_cast<const v4f*>(rk_s + 4 * (kin + r));
#pragma unroll
            for (int ab = 0; ab < M * M; ab++)
              o[r][ab >> 1][ab & 1] = (out[mt][t][ab][r] + f4[ab]) + gp[ab];
          }
          if constexpr (MODE == kModeNhwc) {
            // the lane's four filters are consecutive: one store per output pixel
#pragma unroll
            for (int aa = 0; aa < M; aa++)
#pragma unroll
              for (int b = 0; b < M; b++) {
                const int oy = ty * M + aa, ox = tx * M + b;
                const unsigned pix = (((unsigned)n * (unsigned)a.Ho + (unsigned)oy) * Wo_u +
                                      (unsigned)ox) * (unsigned)K * 4u;
                dev::store_nhwc_k4(a.y, a.y_bytes, pix, (unsigned)kfirst * 4u,
                                   p < P && oy < a.Ho && ox < a.Wo, K - kfirst, (K & 3) == 0,
                                   o[0][aa][b], o[1][aa][b], o[2][aa][b], o[3][aa][b]);
              }
          } else {
            store_patches4(a.y, a.y_bytes, o, base, plane_px * 4u, Wo_u * 4u, K - kfirst, p < P,
                           ty * M + 1 < a.Ho, tx * M + 1 < a.Wo, (a.Wo & 1) == 0);
          }
        }
      }
    }
  }
}

constexpr size_t kLdsBytes = 2 * (size_t)kBlockPlanes + (2 * 2 * 128 + 16) * sizeof(float) +
                             16 * kTiles * sizeof(int) + (32 + 32 + 16) * sizeof(float) +
                             2 * 16 * sizeof(double);

}  // namespace

// F(2x2,3x3), two 64-channel blocks, and byte offsets below 2^31 from the first image of a
// workgroup to every pixel its 32 tiles read (the upper lane half reads two channel planes above
// the descriptor's).
static long long block_reach_bytes(const Geo& g) {
  const long long tiles = (long long)g.th * g.tw;
  const long long images = (kTiles - 1) / tiles + 2;  // images a block of consecutive tiles can touch
  return images * g.C * g.H * g.W * 4LL + 2LL * g.H * g.W * 4LL;
}

bool conv_fused_c128_applicable(const Geo& g) {
  if (!(g.m == 2 && g.CB == 64 && g.NB == 2)) return false;
  if ((long long)g.N * g.K * g.Ho * g.Wo * 4 >= 0xFFFFFFF0LL) return false;  // 32-bit store offsets
  // NHWC: 16-byte pixel loads of four channels at 32-bit offsets; the caller checks X's alignment
  if (is_nhwc(g)) return g.C % 4 == 0 && (long long)g.N * g.C * g.H * g.W * 4 < 0xFFFFFFF0LL;
  return block_reach_bytes(g) < (1LL << 31);
}

template <bool B8, bool FULL, int MODE>
static hipError_t launch_variant(const CgArgs& a, unsigned grid, hipStream_t s) {
  auto kern = conv_fused_c128_kernel<B8, FULL, MODE>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes);
  if (e != hipSuccess) return e;
  note_kernel("conv_fused_c128_kernel");
  kern<<<grid, kThreads, kLdsBytes, s>>>(a);
  return hipGetLastError();
}

template <bool B8, bool FULL>
static hipError_t launch_rows(const Geo& g, const CgArgs& a, unsigned grid, hipStream_t s) {
  switch (patch_load_mode(g)) {
    case 0: return launch_variant<B8, FULL, 0>(a, grid, s);
    case 1: return launch_variant<B8, FULL, 1>(a, grid, s);
    default: return launch_variant<B8, FULL, 2>(a, grid, s);
  }
}

hipError_t launch_conv_fused_c128(const Geo& g, const float* x, const int8_t* uq,
                                  const float* u_range, const int32_t* u_rowsum,
                                  const float* partial, int count, float* v_range, float* y,
                                  hipStream_t s) {
  if (!conv_fused_c128_applicable(g)) return hipErrorInvalidValue;
  CgArgs a{x, uq, u_range, u_rowsum, partial, v_range, y, count,
           (g.flags & LANCE_RANGE_PER_TENSOR) ? 1 : 0, (g.flags & LANCE_INPUT_RANGE_STATIC) ? 1 : 0,
           g.N, g.C, g.H, g.W, g.K, g.pad, g.P, g.th, g.tw, g.Ho, g.Wo, g.bits, g.bits_w,
           is_nhwc(g) ? (unsigned)((size_t)g.N * g.C * g.H * g.W * 4) : (unsigned)block_reach_bytes(g),
           (unsigned)((size_t)g.N * g.K * g.Ho * g.Wo * 4)};
  const unsigned grid = (unsigned)((g.P + kTiles - 1) / kTiles);
  const bool b8 = g.bits == 8, full = g.C == 128;
  if (is_nhwc(g)) {
    if ((reinterpret_cast<uintptr_t>(x) & 15) != 0) return hipErrorInvalidValue;
    return b8 ? launch_variant<true, false, kModeNhwc>(a, grid, s)
              : launch_variant<false, false, kModeNhwc>(a, grid, s);
  }
  if (b8) return full ? launch_rows<true, true>(g, a, grid, s) : launch_rows<true, false>(g, a, grid, s);
  return full ? launch_rows<false, true>(g, a, grid, s) : launch_rows<false, false>(g, a, grid, s);
}

}  // namespace lance
