// Stage 2: v^ = Q(B^T d B) for every input patch (Algorithm 1; Eq. 7), NCHW fp32 in, blocked
// int8 codes out.  Two passes over X (the range of a position is only known after the whole
// tensor has been seen), one write of the codes; fp32 V is never stored.
//
// Both passes share one structure.  A workgroup (256 lanes) takes a region of TR x TC tiles of
// one image and one block of CB <= 64 channels, stages the (TR*m+2)-row pixel window of every
// channel in LDS (zero outside the image), then transforms from LDS.
//
// Staging: a staged row is cut into groups of VW floats aligned to VW in the image (W % VW == 0
// and a VW*4-byte aligned base make every group lie entirely inside or entirely outside the
// image).  Lane l of a wave owns the same (row, group) of the window for every channel and
// every work item, so its descriptors are computed once; waves take channels round robin and
// issue eight independent loads before storing them.
//
// Compute: 16 lanes per tile, lane cl handles the channels cl, cl+Q, cl+2Q, cl+3Q of the block,
// so its four codes form one dword of the blocked layout (byte 4*cl+i holds channel cl+i*Q) and
// a half-wave (two vertically adjacent tiles) writes two full 64-byte rows.  LDS is laid out
// [channel][row][col] with an odd channel stride and a row pitch Wp with m*Wp = 16 (mod 32):
// the 32 lanes of a half-wave then hit 32 different banks.
//
//   range pass : per-lane running (min,max) per position -> one partial record per workgroup
//   quant pass : codes + column sums (16-lane DPP reduction; atomic add when the channel axis
//                spans several blocks)
#include <limits.h>

#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

constexpr int kThreads = 256;
constexpr int kRangeGroups = kMaxRangeGroups;  // persistent range-pass grid: 2 groups per CU

struct InArgs {
  const float* x;
  int8_t* vq;
  int32_t* colsum;
  float* partial;        // range pass: [gridDim.x][E][2]
  const float* qparams;  // quant pass: [E][2] = {min, inv}
  int N, C, H, W, pad, th, tw, P, CB, NB, Q, bits;
  int TR, TC, Wp, R, Wc, CS;  // region geometry (tiles, LDS pitch, rows, cols, channel stride)
  int nry, nrx, items;        // regions per image, work items = NB*N*nry*nrx
  int ng;                     // vector groups per staged row
  int RG, CPW;                // groups per channel window; channels per wave load (RG <= 64)
  unsigned magicTC;           // ceil(2^32 / TC)
  int zero_colsum;            // range pass, NB > 1: channel block 0 clears the column sums
};

template <int M, bool QUANT, int VW>
__global__ __launch_bounds__(kThreads) void input_kernel(const InArgs a) {
  constexpr int A = M + 2, E = A * A;
  constexpr int NSLOT = 4 / VW;  // a channel window has at most 64*NSLOT groups
  constexpr int kUnroll = 8;
  typedef float vec __attribute__((ext_vector_type(VW)));
  extern __shared__ float lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cl = lane & 15, sub = (lane >> 4) & 1, hw = lane >> 5;
  const bool lane_on = cl < a.Q;
  const int HW = a.H * a.W;

  // staging descriptors of this lane (the same for every channel and work item)
  int s_goff[NSLOT], s_lds[NSLOT], s_r[NSLOT], s_gx[NSLOT], s_lc[NSLOT];
  bool s_on[NSLOT];
#pragma unroll
  for (int s = 0; s < NSLOT; s++) {
    const int q = lane + 64 * s;
    const int lc = a.CPW > 1 ? q / a.RG : 0;
    const int qq = a.CPW > 1 ? q - lc * a.RG : q;
    s_on[s] = a.CPW > 1 ? (lc < a.CPW) : (q < a.RG);
    const int r = qq / a.ng, g = qq - r * a.ng;
    s_lc[s] = lc;
    s_r[s] = r;
    s_gx[s] = g * VW;
    s_goff[s] = lc * HW + r * a.W + g * VW;
    s_lds[s] = lc * a.CS + r * a.Wp + g * VW;
  }

  float mn[QUANT ? 1 : E], mx[QUANT ? 1 : E];
  if constexpr (!QUANT) {
#pragma unroll
    for (int e = 0; e < E; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }
  }
  const float L = (float)((1 << a.bits) - 1);
  const unsigned h = 1u << (a.bits - 1);
  const size_t estride = (size_t)a.NB * a.P * a.CB;  // bytes between positions in vq

  for (int item = blockIdx.x; item < a.items; item += gridDim.x) {
    int t = item;
    const int rx = t % a.nrx; t /= a.nrx;
    const int ry = t % a.nry; t /= a.nry;
    const int n = t % a.N;
    const int cb = t / a.N;
    const int y0 = ry * a.TR * M - a.pad, x0 = rx * a.TC * M - a.pad;
    const int cbn = min(a.CB, a.C - cb * a.CB);  // real channels in this block
    // the staged row starts at the aligned column at or left of x0
    const int xa = (x0 >= 0 ? x0 / VW : -((-x0 + VW - 1) / VW)) * VW;
    const int shift = x0 - xa;

    __syncthreads();  // the previous item's compute phase has finished with LDS
    {
      // element index of window pixel (row 0, column xa) of the block's first channel; may
      // point outside the tensor, it is only used where the pixel is inside the image
      const long long ibase =
          (((long long)n * a.C + (long long)cb * a.CB) * a.H + y0) * (long long)a.W + xa;
      bool ok[NSLOT];
#pragma unroll
      for (int s = 0; s < NSLOT; s++) {
        const int gy = y0 + s_r[s], gx = xa + s_gx[s];
        ok[s] = s_on[s] && gy >= 0 && gy < a.H && gx >= 0 && gx < a.W;
      }
      const int ngroups = (cbn + a.CPW - 1) / a.CPW;
      for (int cg0 = wave; cg0 < ngroups; cg0 += 4 * kUnroll) {
        vec v[kUnroll][NSLOT];
#pragma unroll
        for (int u = 0; u < kUnroll; u++) {
          const int c0 = (cg0 + 4 * u) * a.CPW;
#pragma unroll
          for (int s = 0; s < NSLOT; s++) {
#pragma unroll
            for (int i = 0; i < VW; i++) v[u][s][i] = 0.0f;
            if (ok[s] && c0 + s_lc[s] < cbn)
              v[u][s] = *reinterpret_cast<const vec*>(a.x + ibase + (long long)c0 * HW + s_goff[s]);
          }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; u++) {
          const int c0 = (cg0 + 4 * u) * a.CPW;
#pragma unroll
          for (int s = 0; s < NSLOT; s++) {
            if (s_on[s] && c0 + s_lc[s] < cbn) {
              float* dst = lds + c0 * a.CS + s_lds[s];
#pragma unroll
              for (int i = 0; i < VW; i++) dst[i] = v[u][s][i];
            }
          }
        }
      }
    }
    __syncthreads();

    // this lane's four channels cl + i*Q: which of them are real
    unsigned realmask = 0;
    int nreal = 0;
#pragma unroll
    for (int i = 0; i < 4; i++)
      if (lane_on && cl + a.Q * i < cbn) { realmask |= 0xFFu << (8 * i); nreal++; }

    const int npairs = (a.TR / 2) * a.TC;
    for (int u = wave * 2 + hw; u < npairs; u += 8) {
      const int typ = (int)__umulhi((unsigned)u, a.magicTC), txl = u - typ * a.TC;
      const int tyl = 2 * typ + sub;
      const int ty = ry * a.TR + tyl, tx = rx * a.TC + txl;
      const bool valid = ty < a.th && tx < a.tw;
      const int p = (n * a.th + ty) * a.tw + tx;
      const float* tile0 = lds + cl * a.CS + tyl * M * a.Wp + txl * M + shift;

      if constexpr (QUANT) {
        unsigned pk[E];  // unsigned codes of Eq. 7, byte i = channel cl + i*Q
#pragma unroll
        for (int e = 0; e < E; e++) pk[e] = 0;
#pragma unroll
        for (int i = 0; i < 4; i++) {
          if ((realmask >> (8 * i)) & 1) {
            float d[A][A];
            const float* src = tile0 + a.Q * i * a.CS;
#pragma unroll
            for (int r = 0; r < A; r++)
#pragma unroll
              for (int s = 0; s < A; s++) d[r][s] = src[r * a.Wp + s];
            dev::input_tile_transform<M>(d);
#pragma unroll
            for (int e = 0; e < E; e++) {
              // clamp(rne((x - min) * inv), 0, L); the float already holds an integer in
              // [0, 255], so the conversion to a byte is exact
              const float tq = (d[e / A][e % A] - a.qparams[2 * e]) * a.qparams[2 * e + 1];
              const float rq = __builtin_amdgcn_fmed3f(rintf(tq), 0.0f, L);
              pk[e] = __builtin_amdgcn_cvt_pk_u8_f32(rq, i, pk[e]);
            }
          }
        }
        int* dst = reinterpret_cast<int*>(a.vq + ((size_t)cb * a.P + p) * a.CB) + cl;
        const unsigned H8 = 0x80808080u, hh = h * 0x01010101u;
#pragma unroll
        for (int e = 0; e < E; e++) {
          // column sum of the signed codes: (sum of the unsigned bytes) - nreal*h
          const int part = (int)__builtin_amdgcn_sad_u8(pk[e], 0u, 0u) - nreal * (int)h;
          const int tot = dev::row16_sum(part);
          // per-byte (code - h) mod 256 without borrows between bytes, padding lanes -> 0
          const unsigned sg = (((pk[e] | H8) - (hh & ~H8)) ^ ((pk[e] ^ ~hh) & H8)) & realmask;
          if (valid && lane_on)
            *reinterpret_cast<int*>(reinterpret_cast<char*>(dst) + e * estride) = (int)sg;
          if (valid && cl == 0) {
            if (a.NB > 1)
              atomicAdd(a.colsum + (size_t)e * a.P + p, tot);
            else
              a.colsum[(size_t)e * a.P + p] = tot;
          }
        }
      } else {
        // two channels at a time, so that min/max fold into three-operand instructions
#pragma unroll
        for (int i = 0; i < 4; i += 2) {
          const bool r0 = (realmask >> (8 * i)) & 1, r1 = (realmask >> (8 * i + 8)) & 1;
          if (valid && (r0 || r1)) {
            float d0[A][A], d1[A][A];
            const float* src0 = tile0 + a.Q * (r0 ? i : i + 1) * a.CS;
            const float* src1 = tile0 + a.Q * (r1 ? i + 1 : i) * a.CS;
#pragma unroll
            for (int r = 0; r < A; r++)
#pragma unroll
              for (int s = 0; s < A; s++) {
                d0[r][s] = src0[r * a.Wp + s];
                d1[r][s] = src1[r * a.Wp + s];
              }
            dev::input_tile_transform<M>(d0);
            dev::input_tile_transform<M>(d1);
#pragma unroll
            for (int e = 0; e < E; e++) {
              mn[e] = fminf(fminf(mn[e], d0[e / A][e % A]), d1[e / A][e % A]);
              mx[e] = fmaxf(fmaxf(mx[e], d0[e / A][e % A]), d1[e / A][e % A]);
            }
          }
        }
        if (a.zero_colsum && cb == 0 && valid && cl == 0) {
#pragma unroll
          for (int e = 0; e < E; e++) a.colsum[(size_t)e * a.P + p] = 0;
        }
      }
    }
  }

  if constexpr (!QUANT) {
    __syncthreads();
    float* red = lds;  // [4 waves][E][2]
#pragma unroll
    for (int e = 0; e < E; e++) {
      const float lo = dev::wave_min(mn[e]), hi = dev::wave_max(mx[e]);
      if (lane == 0) { red[(wave * E + e) * 2] = lo; red[(wave * E + e) * 2 + 1] = hi; }
    }
    __syncthreads();
    if (tid < E) {
      float lo = red[tid * 2], hi = red[tid * 2 + 1];
      for (int wv = 1; wv < kThreads / 64; wv++) {
        lo = fminf(lo, red[(wv * E + tid) * 2]);
        hi = fmaxf(hi, red[(wv * E + tid) * 2 + 1]);
      }
      a.partial[((size_t)blockIdx.x * E + tid) * 2 + 0] = lo;
      a.partial[((size_t)blockIdx.x * E + tid) * 2 + 1] = hi;
    }
  }
}

// Region geometry.  Constraints: the LDS pitch satisfies m*Wp = 16 (mod 32) and holds every
// vector group that can overlap a staged row; a channel window has at most 64*(4/vw) groups;
// the window of all CB channels fits the LDS budget.  Among those pick the shape that stages
// the fewest pixels per image (least halo, fewest out-of-range tiles, fewest idle lane slots).
bool choose_region(const Geo& g, int vw, InArgs* a) {
  const int M = g.m;
  const int mod = 32 / M, want = 16 / M;  // Wp = want (mod mod)
  // m = 2: aim at four resident workgroups per CU; m = 4 windows are larger, allow two
  const long long budget = (M == 2 ? 40 : 80) * 1024;
  long long best_cost = -1;
  for (int TC = 1; TC <= g.tw && TC <= 64; TC++) {
    const int Wc = TC * M + 2;
    const int ng = (Wc + 2 * (vw - 1)) / vw;  // groups overlapping a row, any alignment
    const int need = ng * vw;
    const int Wp = need + ((want - need % mod) % mod + mod) % mod;
    for (int TR = 2; TR <= ((g.th + 1) & ~1) && TR <= 32; TR += 2) {
      const int R = TR * M + 2;
      const long long lds = (long long)g.CB * (R * Wp + 1) * 4;
      if (lds > budget || R * ng > 64 * (4 / vw)) break;
      const int nry = (g.th + TR - 1) / TR, nrx = (g.tw + TC - 1) / TC;
      const int pairs = (TR / 2) * TC;
      const long long cost =
          (long long)nry * nrx * ((long long)R * Wc + 4LL * ((pairs + 7) / 8 * 8 - pairs));
      if (best_cost < 0 || cost < best_cost) {
        best_cost = cost;
        a->TR = TR; a->TC = TC; a->Wp = Wp; a->R = R; a->Wc = Wc; a->CS = R * Wp + 1;
        a->nry = nry; a->nrx = nrx; a->ng = ng;
      }
    }
  }
  return best_cost >= 0;
}

template <bool QUANT>
hipError_t launch_pass(const Geo& g, const InArgs& a, int vw, int grid, size_t lds,
                       hipStream_t s) {
#define LANCE_IN(MM, VV) input_kernel<MM, QUANT, VV><<<grid, kThreads, lds, s>>>(a)
  if (g.m == 2) {
    if (vw == 4) LANCE_IN(2, 4); else if (vw == 2) LANCE_IN(2, 2); else LANCE_IN(2, 1);
  } else {
    if (vw == 4) LANCE_IN(4, 4); else if (vw == 2) LANCE_IN(4, 2); else LANCE_IN(4, 1);
  }
#undef LANCE_IN
  return hipGetLastError();
}

}  // namespace

hipError_t launch_input_transform(const Geo& g, const float* x, int8_t* vq, float* v_range,
                                  int32_t* v_colsum, char* ws, const Workspace& wl,
                                  hipStream_t s, const DqOut* dqo, hipEvent_t* ev) {
  InArgs a{};
  a.x = x; a.vq = vq; a.colsum = v_colsum;
  a.partial = reinterpret_cast<float*>(ws + wl.off_partial);
  float* qparams = reinterpret_cast<float*>(ws + wl.off_qparams);
  a.qparams = qparams;
  a.N = g.N; a.C = g.C; a.H = g.H; a.W = g.W; a.pad = g.pad; a.th = g.th; a.tw = g.tw;
  a.P = g.P; a.CB = g.CB; a.NB = g.NB; a.Q = g.Q; a.bits = g.bits;
  // widest vector the row pitch and the base address allow
  int vw = 1;
  if (g.W % 4 == 0 && ((uintptr_t)x & 15) == 0) vw = 4;
  else if (g.W % 2 == 0 && ((uintptr_t)x & 7) == 0) vw = 2;
  if (!choose_region(g, vw, &a)) return hipErrorInvalidValue;
  a.RG = a.R * a.ng;
  a.CPW = a.RG <= 64 ? 64 / a.RG : 1;
  a.magicTC = (unsigned)(((1ULL << 32) + a.TC - 1) / a.TC);
  const long long items = (long long)g.NB * g.N * a.nry * a.nrx;
  if (items > INT_MAX) return hipErrorInvalidValue;
  a.items = (int)items;
  size_t lds = (size_t)g.CB * a.CS * sizeof(float);
  const size_t red = (size_t)(kThreads / 64) * g.E * 2 * sizeof(float);
  if (lds < red) lds = red;

  const bool is_static = (g.flags & LANCE_INPUT_RANGE_STATIC) != 0;
  const int per_tensor = (g.flags & LANCE_RANGE_PER_TENSOR) ? 1 : 0;
  hipError_t e;
  int range_groups = 0;
  if (ev && (e = hipEventRecord(ev[0], s)) != hipSuccess) return e;
  if (!is_static) {
    range_groups = a.items < kRangeGroups ? a.items : kRangeGroups;
    a.zero_colsum = g.NB > 1;
    e = launch_pass<false>(g, a, vw, range_groups, lds, s);
    if (e != hipSuccess) return e;
  } else if (g.NB > 1) {
    e = launch_fill_zero(v_colsum, (size_t)g.E * g.P, s);
    if (e != hipSuccess) return e;
  }
  if (ev && (e = hipEventRecord(ev[1], s)) != hipSuccess) return e;
  e = launch_range_finalize(a.partial, range_groups, g.E, per_tensor, is_static, g.bits, v_range,
                            qparams, dqo, s);
  if (e != hipSuccess) return e;
  if (ev && (e = hipEventRecord(ev[2], s)) != hipSuccess) return e;
  a.zero_colsum = 0;
  e = launch_pass<true>(g, a, vw, a.items, lds, s);
  if (e != hipSuccess) return e;
  if (ev && (e = hipEventRecord(ev[3], s)) != hipSuccess) return e;
  return hipSuccess;
}

}  // namespace lance
