// Quantize pass, products and epilogue in one kernel for F(2x2,3x3) layers with at most 16
// channels (one 16-channel code block; e.g. the 3-channel first layer of an image network):
// v^ = Q(B^T d B), m^ = sum_c u^ . v^, Eq. 8 and S = A^T m A (Algorithm 1, Eq. 7-9) with the
// codes of V, their column sums and the accumulators never leaving registers.
//
// With so few channels the layer is a stream: per tile it reads 4*C*4 bytes and writes 4*K*4, the
// products are a 16-deep contraction.  Every wave works alone on 64 consecutive tiles, lane =
// tile:
//   T  the lane loads the 4x4 patch of each channel (patch_loader.h), transforms and quantizes
//      it and packs the codes of its tile: 16 bytes per position (the blocked channel order of
//      the code layout), i.e. four registers per position; column sums by v_sad_u8.
//   X  v_mfma_i32_32x32x16_i8 wants the codes of 32 tiles, the lower lanes holding contraction
//      bytes 0-7 and the upper lanes bytes 8-15.  Two v_permlane32_swap per position turn the
//      lane-per-tile registers into exactly that, for both groups of 32 tiles at once.
//   G  per filter tile (32 filters) and tile group: 16 matrix instructions, one per position,
//      each folded at once into the four outputs of the 2x2 patch with the (compile-time sparse)
//      coefficients A^T[a][i] A^T[b][j] s_e; then the two separable terms of the expanded Eq. 8
//      are added and the patches stored.
// The ranges come from the range pass and its reduction kernel (Eq. 7 parameters, s_e and the
// constants of the filter-side terms), so this kernel has no reduction of its own.  With
// caller-supplied ranges (Sec. 3.4's inference mode) there is no other kernel at all: every
// workgroup forms the 16 parameter sets from the two range tables itself.
#include "lance_device.h"
#include "lance_internal.h"
#include "nhwc_window.h"
#include "patch_loader.h"

namespace lance {
namespace {

typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kMaxK = 1024;  // filters whose rk terms fit the LDS table

struct CsArgs {
  const float* x;
  const int8_t* uq;     // [E][K][16]
  const float* qparams; // [E][2] = {min, inv}
  const float* dq;      // [E][4] = {su*sv, sv*ou, -, -}
  const double* dqd;    // [E][2] = {su*ov, C*ou*ov}
  const int32_t* u_rowsum;  // [E][K]
  float* y;
  int N, C, H, W, K, pad, P, th, tw, Ho, Wo, bits;
  unsigned reach, y_bytes;
  // caller-supplied ranges (LANCE_INPUT_RANGE_STATIC): the kernel forms the parameters and
  // constants itself from v_range and u_range; qparams, dq and dqd are not read
  const float* v_range;  // [E][2], or nullptr: dynamic ranges, tables from the reduction kernel
  const float* u_range;  // [E][2]
  int bits_w;
};

// lanes 0-31 keep `own`, lanes 32-63 receive the value of lane - 32 (*g0); lanes 0-31 receive
// the value of lane + 32, lanes 32-63 keep `own` (*g1): what the two tile groups' columns need.
__device__ __forceinline__ void spread(unsigned own, unsigned* g0, unsigned* g1) {
  const v2u s = __builtin_amdgcn_permlane32_swap(own, own, false, false);
  *g0 = s[0];
  *g1 = s[1];
}

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

// MODE: patch load mode (0 or 2, patch_load_mode), or kModeNhwc: X is [N][H][W][C] (a.reach =
// its size in bytes) and Y is [N][Ho][Wo][K]; the codes then keep the channels in natural order.
constexpr int kModeNhwc = 3;

template <bool B8, int MODE>
__global__ __launch_bounds__(kThreads, 2) void conv_fused_c16_kernel(const CsArgs a) {
  constexpr int M = 2, A = 4, E = 16;
  constexpr bool kNhwc = MODE == kModeNhwc;
  extern __shared__ float rk_s[];  // [K][M*M]
  __shared__ float qp_s[2 * E], dq_s[2 * E];  // {min, inv}, {su*sv, sv*ou} per position
  __shared__ double dqd_s[2 * E];             // {su*ov, C*ou*ov}
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int K = a.K, P = a.P, C = a.C;

  // Eq. 7 parameters and Eq. 8 constants: from the reduction kernel's tables, or (calibrated
  // ranges) formed here exactly as that kernel forms them
  if (tid < E) {
    if (a.v_range) {
      float inv, sv, iu, su;
      const float lo = a.v_range[2 * tid], hi = a.v_range[2 * tid + 1];
      dev::quant_params(lo, hi, a.bits, &inv, &sv);
      dev::quant_params(a.u_range[2 * tid], a.u_range[2 * tid + 1], a.bits_w, &iu, &su);
      const double ou = (double)a.u_range[2 * tid] + (double)su * (double)(1 << (a.bits_w - 1));
      const double ov = (double)lo + (double)sv * (double)(1 << (a.bits - 1));
      qp_s[2 * tid] = lo;
      qp_s[2 * tid + 1] = inv;
      dq_s[2 * tid] = (float)((double)su * (double)sv);
      dq_s[2 * tid + 1] = (float)((double)sv * ou);
      dqd_s[2 * tid] = (double)su * ov;
      dqd_s[2 * tid + 1] = (double)C * ou * ov;
    } else {
      qp_s[2 * tid] = a.qparams[2 * tid];
      qp_s[2 * tid + 1] = a.qparams[2 * tid + 1];
      dq_s[2 * tid] = a.dq[4 * tid];
      dq_s[2 * tid + 1] = a.dq[4 * tid + 1];
      dqd_s[2 * tid] = a.dqd[2 * tid];
      dqd_s[2 * tid + 1] = a.dqd[2 * tid + 1];
    }
  }
  __syncthreads();

  // filter-side terms f[e,k] = su*ov*rowsum[e][k] + C*ou*ov through A^T . A, in binary64
  // (thread = filter)
  for (int k = tid; k < K; k += kThreads) {
    double f[E];
#pragma unroll
    for (int e = 0; e < E; e++)
      f[e] = dqd_s[2 * e] * (double)a.u_rowsum[(size_t)e * K + k] + dqd_s[2 * e + 1];
    v4f r4;
#pragma unroll
    for (int ab = 0; ab < M * M; ab++) {
      double accd = 0.0;
#pragma unroll
      for (int e = 0; e < E; e++) {
        const float coef = dev::Wino<M>::at(ab >> 1, e / A) * dev::Wino<M>::at(ab & 1, e % A);
        if (coef != 0.0f) accd += (double)coef * f[e];
      }
      r4[ab] = (float)accd;
    }
    *reinterpret_cast<v4f*>(rk_s + 4 * k) = r4;
  }
  __syncthreads();
  const int p0 = (dev::xcd_contiguous(blockIdx.x, gridDim.x) * 4 + wave) * 64;
  if (p0 >= P) return;  // (no barrier below)

  // Eq. 7 parameters and the scales of the expanded Eq. 8, wave-uniform
  float qmn[E], qinv[E], sc[E], gc[E];
#pragma unroll
  for (int e = 0; e < E; e++) {
    qmn[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(qp_s[2 * e])));
    qinv[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(qp_s[2 * e + 1])));
    sc[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(dq_s[2 * e])));
    gc[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(dq_s[2 * e + 1])));
  }

  // ============================ T: transform + quantize ============================
  const bool valid = p0 + lane < P;
  const int pt = min(p0 + lane, P - 1);
  const int tx = pt % a.tw, t2 = pt / a.tw;
  const int ty = t2 % a.th, n = t2 / a.th;
  const unsigned HW = (unsigned)a.H * (unsigned)a.W;
  const int n0 = p0 / (a.th * a.tw);  // image of the block's first tile (wave-uniform)
  dev::PatchLoader<M> pl;
  unsigned pixoff[A * A];  // NHWC: byte offsets of the window's pixels
  if constexpr (kNhwc)
    dev::window_offsets_nhwc<M>(n, ty * M - a.pad, tx * M - a.pad, a.H, a.W, C, pixoff);
  else
    pl.setup((unsigned)(n - n0) * (unsigned)C * HW, n0, n, a.N, ty, tx, a.pad, a.H, a.W);
  const char* xb = reinterpret_cast<const char*>(a.x + (size_t)n0 * C * HW);
  constexpr bool kRows = MODE == 2;
  constexpr int kAhead = 2, kBuf = kAhead + 1;
  float buf[kBuf][E];
  auto issue = [&](int c) {
    const char* plane = xb + (size_t)c * HW * 4;
    if constexpr (kNhwc)
      dev::load_channel_nhwc<M>(a.x, a.reach, pixoff, c, buf[c % kBuf]);
    else if constexpr (kRows)
      pl.issue_rows_shifted(plane, a.reach, pl.first_image && c == 0, pl.last_image && c == C - 1,
                            buf[c % kBuf]);
    else
      pl.template issue<false>(plane, a.reach, buf[c % kBuf]);
  };
  // NHWC layers with at most four channels (an RGB image): a pixel is one load
  const bool pix = kNhwc && C <= 4;  // kernel-uniform
  float px[A * A][4];
  if (pix) {
    dev::load_pixels_nhwc<M>(a.x, a.reach, pixoff, C, px);
  } else {
#pragma unroll
    for (int c = 0; c < kAhead; c++)
      if (c < C) issue(c);
  }

  // codes[e][d]: channel c sits in dword c % 4, byte c / 4 (the blocked order of the code layout)
  unsigned codes[E][4];
#pragma unroll
  for (int e = 0; e < E; e++)
#pragma unroll
    for (int d = 0; d < 4; d++) codes[e][d] = 0u;
  const float L = (float)((1 << a.bits) - 1);
#pragma unroll
  for (int c = 0; c < 16; c++) {
    if (c < C) {  // wave-uniform
      if (!pix && c + kAhead < C) issue(c + kAhead);
      float d[A][A];
#pragma unroll
      for (int r = 0; r < A; r++)
#pragma unroll
        for (int q = 0; q < A; q++)
          d[r][q] = (kNhwc && pix) ? px[r * A + q][c & 3] : buf[c % kBuf][r * A + q];
      if constexpr (kRows) {
        pl.unshift(pl.first_image && c == 0, pl.last_image && c == C - 1, d);
        pl.template fix<true>(d);
      }
      dev::input_tile_transform<M>(d);
#pragma unroll
      for (int e = 0; e < E; e++) {
        // clamp(rne((x - min) * inv), 0, L): v_cvt_pk_u8_f32 rounds to nearest even and
        // saturates to [0, 255]; only the upper clamp of narrower codes needs an instruction
        float tq = (d[e / A][e % A] - qmn[e]) * qinv[e];
        if constexpr (!B8) tq = fminf(tq, L);
        constexpr int dw = kNhwc ? 0 : 1;  // natural order: dword c / 4, byte c % 4
        const int cd = dw ? c % 4 : c / 4, cbyte = dw ? c / 4 : c % 4;
        codes[e][cd] = __builtin_amdgcn_cvt_pk_u8_f32(tq, cbyte, codes[e][cd]);
      }
#pragma unroll
      for (int e = 0; e < E; e++) asm volatile("" : "+v"(codes[e][kNhwc ? c / 4 : c % 4]));
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // column sums -> the input-side term g[e,p] = sv*ou*colsum through A^T . A; unsigned -> signed
  // codes (bytes of channels that do not exist stay 0)
  float gp[M][M];
#pragma unroll
  for (int aa = 0; aa < M; aa++)
#pragma unroll
    for (int b = 0; b < M; b++) gp[aa][b] = 0.0f;
  unsigned realmask[4];
#pragma unroll
  for (int d = 0; d < 4; d++) {
    realmask[d] = 0;
#pragma unroll
    for (int i = 0; i < 4; i++)
      if ((kNhwc ? 4 * d + i : d + 4 * i) < C) realmask[d] |= 0xFFu << (8 * i);
  }
  const unsigned h = 1u << (a.bits - 1);
  const unsigned H8 = 0x80808080u, hh = h * 0x01010101u;
#pragma unroll
  for (int e = 0; e < E; e++) {
    unsigned cs = 0;
#pragma unroll
    for (int d = 0; d < 4; d++) {
      const unsigned u = codes[e][d];
      cs = __builtin_amdgcn_sad_u8(u, 0u, cs);
      unsigned v;
      if constexpr (B8)
        v = u ^ H8;
      else
        v = ((u | H8) - (hh & ~H8)) ^ ((u ^ ~hh) & H8);
      codes[e][d] = v & realmask[d];
    }
    const float g = gc[e] * (float)((int)cs - C * (int)h);  // column sum of the signed codes
#pragma unroll
    for (int aa = 0; aa < M; aa++)
#pragma unroll
      for (int b = 0; b < M; b++) {
        const float coef = dev::Wino<M>::at(aa, e / A) * dev::Wino<M>::at(b, e % A);
        if (coef != 0.0f) gp[aa][b] = __builtin_fmaf(coef, g, gp[aa][b]);
      }
  }

  // ============================ X: lane-per-tile -> matrix operands ============================
  // After the swaps (codes[e][0], codes[e][1]) is the operand of tile group 0 and
  // (codes[e][2], codes[e][3]) that of tile group 1, in every lane.
#pragma unroll
  for (int e = 0; e < E; e++)
#pragma unroll
    for (int d = 0; d < 2; d++) {
      const v2u s = __builtin_amdgcn_permlane32_swap(codes[e][d], codes[e][d + 2], false, false);
      codes[e][d] = s[0];
      codes[e][d + 2] = s[1];
    }
  // what a lane must know of the tile of its column in each group: validity, the element offset
  // of the patch's first pixel in plane 0 of its image, edge flags, the input-side term
  const int Ho = a.Ho, Wo = a.Wo;
  const unsigned plane = (unsigned)Ho * (unsigned)Wo;
  // (NHWC: the pixel index of the patch's first pixel)
  const unsigned own_off = kNhwc ? ((unsigned)n * (unsigned)Ho + (unsigned)(ty * M)) * (unsigned)Wo +
                                       (unsigned)(tx * M)
                                 : (unsigned)n * (unsigned)K * plane +
                                       (unsigned)(ty * M) * (unsigned)Wo + (unsigned)(tx * M);
  const unsigned own_flags = (valid ? 1u : 0u) | ((ty * M + 1 < Ho) ? 2u : 0u) |
                             ((tx * M + 1 < Wo) ? 4u : 0u);
  unsigned off_g[2], flags_g[2], gp_g[2][M * M];
  spread(own_off, &off_g[0], &off_g[1]);
  spread(own_flags, &flags_g[0], &flags_g[1]);
#pragma unroll
  for (int ab = 0; ab < M * M; ab++)
    spread(__float_as_uint(gp[ab >> 1][ab & 1]), &gp_g[0][ab], &gp_g[1][ab]);

  // ============================ G: products + epilogue ============================
  const int col = lane & 31, half = lane >> 5;
  const bool even_w = (Wo & 1) == 0;
  const int nkt = (K + 31) / 32;
  for (int kt = 0; kt < nkt; kt++) {
    // filter operands of this tile: row = filter, bytes 8*half .. 8*half+7 of its 16
    long af[E];
    {
      const int krow = min(kt * 32 + col, K - 1);
      const int8_t* src = a.uq + (size_t)krow * 16 + 8 * half;
#pragma unroll
      for (int e = 0; e < E; e++)
        af[e] = *reinterpret_cast<const long*>(src + (size_t)e * K * 16);
    }
#pragma unroll
    for (int g = 0; g < 2; g++) {
      v16f out[M * M];
#pragma unroll
      for (int ab = 0; ab < M * M; ab++)
#pragma unroll
        for (int r = 0; r < 16; r++) out[ab][r] = 0.0f;
#pragma unroll
      for (int e = 0; e < E; e++) {
        const long bf = (long)(((unsigned long long)codes[e][2 * g + 1] << 32) | codes[e][2 * g]);
        const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        const v16i acc = __builtin_amdgcn_mfma_i32_32x32x16_i8(af[e], bf, zero, 0, 0, 0);
#pragma unroll
        for (int ab = 0; ab < M * M; ab++) {
          const float coef = dev::Wino<M>::at(ab >> 1, e / A) * dev::Wino<M>::at(ab & 1, e % A);
          if (coef != 0.0f) {
            const float c = coef * sc[e];
#pragma unroll
            for (int r = 0; r < 16; r++) out[ab][r] = __builtin_fmaf(c, (float)acc[r], out[ab][r]);
          }
        }
        // One position at a time: left alone, the compiler issues all 16 matrix instructions
        // first and holds 256 accumulator registers.  The empty statements tie the folded
        // outputs to this point.
#pragma unroll
        for (int ab = 0; ab < M * M; ab++) asm volatile("" : "+v"(out[ab]));
        __builtin_amdgcn_sched_barrier(0);
      }
      // tail of this (filter tile, tile group): add the two separable terms, store the patches;
      // stores that must not happen get an offset the buffer's range check drops
      {
        const int kfirst = kt * 32 + 4 * half;  // this lane's first filter
        if constexpr (kNhwc) {
          // the lane's filters come in groups of four consecutive ones: one store per group and
          // pixel, formed group by group (no table of all 64 outputs)
          const bool k4 = (K & 3) == 0;
#pragma unroll
          for (int rq = 0; rq < 4; rq++) {
            v4f f4[4];
#pragma unroll
            for (int q = 0; q < 4; q++)
              f4[q] = *reinterpret_cast<const v4f*>(rk_s + 4 * min(kfirst + 8 * rq + q, K - 1));
#pragma unroll
            for (int aa = 0; aa < M; aa++)
#pragma unroll
              for (int b = 0; b < M; b++) {
                const bool pix_ok = (flags_g[g] & 1u) && (aa == 0 || (flags_g[g] & 2u)) &&
                                    (b == 0 || (flags_g[g] & 4u));
                const unsigned pix = (off_g[g] + (unsigned)(aa * Wo + b)) * (unsigned)K * 4u;
                const int ab = aa * M + b;
                const float gpv = __uint_as_float(gp_g[g][ab]);
                dev::store_nhwc_k4(a.y, a.y_bytes, pix, (unsigned)(kfirst + 8 * rq) * 4u, pix_ok,
                                   K - (kfirst + 8 * rq), k4,
                                   (out[ab][4 * rq + 0] + f4[0][ab]) + gpv,
                                   (out[ab][4 * rq + 1] + f4[1][ab]) + gpv,
                                   (out[ab][4 * rq + 2] + f4[2][ab]) + gpv,
                                   (out[ab][4 * rq + 3] + f4[3][ab]) + gpv);
              }
          }
        } else {
          float o[16][M][M];
#pragma unroll
          for (int r = 0; r < 16; r++) {
            const int k = min(kfirst + 8 * (r / 4) + (r % 4), K - 1);
            const v4f f4 = *reinterpret_cast<const v4f*>(rk_s + 4 * k);
#pragma unroll
            for (int aa = 0; aa < M; aa++)
#pragma unroll
              for (int b = 0; b < M; b++)
                o[r][aa][b] = (out[aa * M + b][r] + f4[aa * M + b]) + __uint_as_float(gp_g[g][aa * M + b]);
          }
          store_patches(a.y, a.y_bytes, o, (off_g[g] + (unsigned)kfirst * plane) * 4u, plane * 4u,
                        (unsigned)Wo * 4u, K - kfirst, flags_g[g] & 1u, flags_g[g] & 2u,
                        flags_g[g] & 4u, even_w);
        }
      }
    }
  }
}

}  // namespace

// F(2x2,3x3), one 16-channel block, byte offsets below 2^31 from the first image of a wave's 64
// tiles to every pixel they read, output bytes addressed with 32 bits, rk table in LDS.
bool conv_fused_c16_applicable(const Geo& g) {
  if (!(g.m == 2 && g.CB == 16 && g.NB == 1 && g.K <= kMaxK)) return false;
  if (is_nhwc(g))  // the whole of X and of Y addressed with 32-bit offsets
    return (long long)g.N * g.C * g.H * g.W * 4 < 0xFFFFFFF0LL &&
           (long long)g.N * g.K * g.Ho * g.Wo * 4 < 0xFFFFFFF0LL;
  const long long tiles = (long long)g.th * g.tw;
  const long long images = 63 / tiles + 2;  // images a block of 64 consecutive tiles can touch
  const long long reach = images * g.C * g.H * g.W * 4LL;
  const long long y_elems = (long long)g.N * g.K * g.Ho * g.Wo;
  return reach < (1LL << 31) && y_elems * 4 < 0xFFFFFFF0LL;  // 32-bit store offsets
}

hipError_t launch_conv_fused_c16(const Geo& g, const float* x, const int8_t* uq,
                                 const float* qparams, const float* dq, const double* dqd,
                                 const int32_t* u_rowsum, float* y, const float* static_v_range,
                                 const float* u_range, hipStream_t s) {
  if (!conv_fused_c16_applicable(g)) return hipErrorInvalidValue;
  const long long tiles = (long long)g.th * g.tw;
  const long long images = 63 / tiles + 2;
  CsArgs a{x, uq, qparams, dq, dqd, u_rowsum, y, g.N, g.C, g.H, g.W, g.K, g.pad, g.P, g.th, g.tw, g.Ho, g.Wo,
           g.bits,
           is_nhwc(g) ? (unsigned)((long long)g.N * g.C * g.H * g.W * 4) : (unsigned)(images * g.C * g.H * g.W * 4LL),
           (unsigned)((size_t)g.N * g.K * g.Ho * g.Wo * 4), static_v_range, u_range, g.bits_w};
  const unsigned grid = (unsigned)((g.P + 255) / 256);
  const size_t lds = (size_t)4 * g.K * sizeof(float);
  const bool rows = patch_load_mode(g) == 2;
  note_kernel("conv_fused_c16_kernel");
#define LANCE_C16(B8, MODE) conv_fused_c16_kernel<B8, MODE><<<grid, kThreads, lds, s>>>(a)
  if (is_nhwc(g)) {
    if (g.bits == 8) LANCE_C16(true, kModeNhwc); else LANCE_C16(false, kModeNhwc);
  } else if (g.bits == 8) {
    if (rows) LANCE_C16(true, 2); else LANCE_C16(true, 0);
  } else {
    if (rows) LANCE_C16(false, 2); else LANCE_C16(false, 0);
  }
#undef LANCE_C16
  return hipGetLastError();
}

}  // namespace lance
