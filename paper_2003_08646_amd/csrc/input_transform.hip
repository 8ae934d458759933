// Stage 2: v^ = Q(B^T d B) for every input patch (Algorithm 1; Eq. 7), NCHW fp32 in, blocked
// int8 codes out.  HBM-bound: two passes over X (the range of a position is only known after
// the whole tensor has been seen), one write of the codes; fp32 V is never stored.
//
// Both passes share one structure.  A workgroup (256 lanes) takes a region of TR x TC tiles of
// one image and one block of CB <= 64 channels, stages the (TR*m+2) x (TC*m+2) pixel window of
// every channel in LDS with coalesced row reads (zero outside the image), then transforms from
// LDS.  Lane mapping in the compute phase: 16 lanes per tile, lane cl handles the channels
// cl, cl+Q, cl+2Q, cl+3Q of the block, so its four codes form one dword of the blocked layout
// (byte 4*cl+i holds channel cl+i*Q) and a half-wave (two vertically adjacent tiles) writes
// two full 64-byte rows.  LDS is laid out [channel][row][col] with an odd channel stride and a
// row pitch Wp chosen so that m*Wp = 16 (mod 32): the 32 lanes of a half-wave then hit 32
// different banks.
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
constexpr int kLdsBudget = 64 * 1024;  // two workgroups per CU

struct InArgs {
  const float* x;
  int8_t* vq;
  int32_t* colsum;
  float* partial;        // range pass: [gridDim.x][E][2]
  const float* qparams;  // quant pass: [E][2] = {min, inv}
  int N, C, H, W, pad, th, tw, P, CB, NB, Q, bits;
  int TR, TC, Wp, R, Wc, CS;  // region geometry (tiles, LDS pitch, rows, cols, channel stride)
  int nry, nrx, items;        // regions per image, work items = NB*N*nry*nrx
  unsigned magicR;            // ceil(2^32 / R): rowid / R == umulhi(rowid, magicR)
  int stepq, stepr;           // 256 / Wc, 256 % Wc
  int zero_colsum;            // range pass, NB > 1: channel block 0 clears the column sums
};

template <int M, bool QUANT>
__global__ __launch_bounds__(kThreads) void input_kernel(const InArgs a) {
  constexpr int A = M + 2, E = A * A;
  extern __shared__ float lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cl = lane & 15, sub = (lane >> 4) & 1, hw = lane >> 5;
  const bool lane_on = cl < a.Q;

  float mn[QUANT ? 1 : E], mx[QUANT ? 1 : E];
  if constexpr (!QUANT) {
#pragma unroll
    for (int e = 0; e < E; e++) { mn[e] = INFINITY; mx[e] = -INFINITY; }
  }
  const float L = (float)((1 << a.bits) - 1);
  const int h = 1 << (a.bits - 1);
  const size_t estride = (size_t)a.NB * a.P * a.CB;  // bytes between positions in vq

  for (int item = blockIdx.x; item < a.items; item += gridDim.x) {
    int t = item;
    const int rx = t % a.nrx; t /= a.nrx;
    const int ry = t % a.nry; t /= a.nry;
    const int n = t % a.N;
    const int cb = t / a.N;
    const int y0 = ry * a.TR * M - a.pad, x0 = rx * a.TC * M - a.pad;
    const int cbn = min(a.CB, a.C - cb * a.CB);  // real channels in this block

    __syncthreads();  // the previous item's compute phase has finished with LDS
    {
      const int nrows = cbn * a.R;
      int rowid = tid / a.Wc;
      int xx = tid - rowid * a.Wc;
      const float* xn = a.x + ((size_t)n * a.C + (size_t)cb * a.CB) * a.H * a.W;
#pragma unroll 4
      while (rowid < nrows) {
        const int c = (int)__umulhi((unsigned)rowid, a.magicR);
        const int r = rowid - c * a.R;
        const int gy = y0 + r, gx = x0 + xx;
        float v = 0.0f;
        if (gy >= 0 && gy < a.H && gx >= 0 && gx < a.W)
          v = xn[((size_t)c * a.H + gy) * a.W + gx];
        lds[c * a.CS + r * a.Wp + xx] = v;
        xx += a.stepr;
        rowid += a.stepq;
        if (xx >= a.Wc) { xx -= a.Wc; rowid++; }
      }
    }
    __syncthreads();

    const int npairs = (a.TR / 2) * a.TC;
    for (int u = wave * 2 + hw; u < npairs; u += 8) {
      const int typ = u / a.TC, txl = u - typ * a.TC;
      const int tyl = 2 * typ + sub;
      const int ty = ry * a.TR + tyl, tx = rx * a.TC + txl;
      const bool valid = ty < a.th && tx < a.tw;
      const int p = (n * a.th + ty) * a.tw + tx;

      int pk[QUANT ? E : 1], cs[QUANT ? E : 1];
      if constexpr (QUANT) {
#pragma unroll
        for (int e = 0; e < E; e++) { pk[e] = 0; cs[e] = 0; }
      }
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int c = cl + a.Q * i;
        const bool real = lane_on && (cb * a.CB + c < a.C);
        if (real) {
          float d[A][A];
          const float* src = lds + c * a.CS + tyl * M * a.Wp + txl * M;
#pragma unroll
          for (int r = 0; r < A; r++)
#pragma unroll
            for (int s = 0; s < A; s++) d[r][s] = src[r * a.Wp + s];
          dev::input_tile_transform<M>(d);
          if constexpr (QUANT) {
#pragma unroll
            for (int e = 0; e < E; e++) {
              const int q = dev::quantize_code(d[e / A][e % A], a.qparams[2 * e],
                                               a.qparams[2 * e + 1], L, h);
              pk[e] |= (q & 0xFF) << (8 * i);
              cs[e] += q;
            }
          } else if (valid) {
#pragma unroll
            for (int e = 0; e < E; e++) {
              mn[e] = fminf(mn[e], d[e / A][e % A]);
              mx[e] = fmaxf(mx[e], d[e / A][e % A]);
            }
          }
        }
      }
      if constexpr (QUANT) {
        int* dst = reinterpret_cast<int*>(a.vq + ((size_t)cb * a.P + p) * a.CB) + cl;
#pragma unroll
        for (int e = 0; e < E; e++) {
          const int tot = dev::row16_sum(cs[e]);
          if (valid && lane_on)
            *reinterpret_cast<int*>(reinterpret_cast<char*>(dst) + e * estride) = pk[e];
          if (valid && cl == 0) {
            if (a.NB > 1)
              atomicAdd(a.colsum + (size_t)e * a.P + p, tot);
            else
              a.colsum[(size_t)e * a.P + p] = tot;
          }
        }
      } else if (a.zero_colsum && cb == 0 && valid && cl == 0) {
#pragma unroll
        for (int e = 0; e < E; e++) a.colsum[(size_t)e * a.P + p] = 0;
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

// Region geometry: the LDS pitch must satisfy m*Wp = 16 (mod 32); among the shapes that fit
// the LDS budget pick the one that loads the fewest pixels per image (least halo, least
// out-of-range tiles).
void choose_region(const Geo& g, InArgs* a) {
  const int M = g.m;
  const int mod = 32 / M, want = 16 / M;  // Wp = want (mod mod)
  long long best_cost = -1;
  for (int TC = 1; TC <= g.tw && TC <= 64; TC++) {
    const int Wc = TC * M + 2;
    int Wp = Wc + ((want - Wc % mod) % mod + mod) % mod;
    for (int TR = 2; TR <= ((g.th + 1) & ~1) && TR <= 32; TR += 2) {
      const int R = TR * M + 2;
      const long long lds = (long long)g.CB * (R * Wp + 1) * 4;
      if (lds > kLdsBudget) break;
      const int nry = (g.th + TR - 1) / TR, nrx = (g.tw + TC - 1) / TC;
      // cost: pixels staged per image and channel, plus a term for idle half-wave slots
      const int pairs = (TR / 2) * TC;
      const long long cost =
          (long long)nry * nrx * ((long long)R * Wc + 4LL * ((pairs + 7) / 8 * 8 - pairs));
      if (best_cost < 0 || cost < best_cost) {
        best_cost = cost;
        a->TR = TR; a->TC = TC; a->Wp = Wp; a->R = R; a->Wc = Wc; a->CS = R * Wp + 1;
        a->nry = nry; a->nrx = nrx;
      }
    }
  }
}

template <bool QUANT>
hipError_t launch_pass(const Geo& g, const InArgs& a, int grid, size_t lds, hipStream_t s) {
  if (g.m == 2)
    input_kernel<2, QUANT><<<grid, kThreads, lds, s>>>(a);
  else
    input_kernel<4, QUANT><<<grid, kThreads, lds, s>>>(a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_input_transform(const Geo& g, const float* x, int8_t* vq, float* v_range,
                                  int32_t* v_colsum, char* ws, const Workspace& wl,
                                  hipStream_t s, hipEvent_t* ev) {
  InArgs a{};
  a.x = x; a.vq = vq; a.colsum = v_colsum;
  a.partial = reinterpret_cast<float*>(ws + wl.off_partial);
  float* qparams = reinterpret_cast<float*>(ws + wl.off_qparams);
  a.qparams = qparams;
  a.N = g.N; a.C = g.C; a.H = g.H; a.W = g.W; a.pad = g.pad; a.th = g.th; a.tw = g.tw;
  a.P = g.P; a.CB = g.CB; a.NB = g.NB; a.Q = g.Q; a.bits = g.bits;
  choose_region(g, &a);
  a.magicR = (unsigned)(((1ULL << 32) + a.R - 1) / a.R);
  a.stepq = kThreads / a.Wc; a.stepr = kThreads % a.Wc;
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
    range_groups = a.items < kMaxRangeGroups ? a.items : kMaxRangeGroups;
    a.zero_colsum = g.NB > 1;
    e = launch_pass<false>(g, a, range_groups, lds, s);
    if (e != hipSuccess) return e;
  } else if (g.NB > 1) {
    e = launch_fill_zero(v_colsum, (size_t)g.E * g.P, s);
    if (e != hipSuccess) return e;
  }
  if (ev && (e = hipEventRecord(ev[1], s)) != hipSuccess) return e;
  e = launch_range_finalize(a.partial, range_groups, g.E, per_tensor, is_static, g.bits, v_range,
                            qparams, s);
  if (e != hipSuccess) return e;
  if (ev && (e = hipEventRecord(ev[2], s)) != hipSuccess) return e;
  a.zero_colsum = 0;
  e = launch_pass<true>(g, a, a.items, lds, s);
  if (e != hipSuccess) return e;
  if (ev && (e = hipEventRecord(ev[3], s)) != hipSuccess) return e;
  return hipSuccess;
}

}  // namespace lance
