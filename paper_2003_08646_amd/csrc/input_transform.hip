// Stage 2, second pass for layers with code blocks of fewer than 64 channels (today: at most 16
// channels, one block of 16): v^ = Q(B^T d B) for every input patch (Algorithm 1; Eq. 7), NCHW fp32 in, blocked
// int8 codes out.  Layers with 64-channel code blocks take input_quant.hip instead.  The ranges
// come from the first pass (input_range.hip); fp32 V is never stored.  This file also holds the
// driver of the whole input transform (range pass, reduction, quantize pass).
//
// A (persistent) workgroup of 256 lanes takes a region of TR x TC tiles of
// one image and one block of CB <= 64 channels, stages the (TR*m+2)-row pixel window of every
// channel in LDS (zero outside the image), then transforms from LDS.
//
// Staging: lane q of a wave owns the LDS words q, q+64, q+128, q+192 of a channel window (the
// window is a [rows][Wp] array of at most 256 words), i.e. the same pixels of the window for
// every channel and every work item, so its descriptors are computed once.  Waves take the
// channels round robin; a wave's loads of one channel are plain dword loads of consecutive
// pixels (coalesced rows) and its LDS stores hit consecutive banks.  All loads of an item are
// issued before any is stored, and the loads of the next item are in flight while the current
// one is transformed (the workgroups are persistent).
//
// Compute: 16 lanes per tile, lane cl handles the channels cl, cl+Q, cl+2Q, cl+3Q of the block,
// so its four codes form one dword of the blocked layout (byte 4*cl+i holds channel cl+i*Q) and
// a half-wave (two vertically adjacent tiles) writes two full 64-byte rows.  LDS is laid out
// [channel][row][col] with an odd channel stride and a row pitch Wp with m*Wp = 16 (mod 32):
// the 32 lanes of a half-wave then hit 32 different banks.
//
// Column sums of the codes: 16-lane DPP reduction; atomic add when the channel axis spans
// several blocks.
#include <limits.h>

#include "lance_device.h"
#include "lance_internal.h"

namespace lance {
namespace {

constexpr int kThreads = 256;
constexpr int kGroups = 512;  // persistent grid: two workgroups per CU

struct InArgs {
  const float* x;
  int8_t* vq;
  int32_t* colsum;
  const float* qparams;  // quant pass: [E][2] = {min, inv}
  int N, C, H, W, pad, th, tw, P, CB, NB, Q, bits;
  int TR, TC, Wp, R, Wc, CS;  // region geometry (tiles, LDS pitch, rows, cols, channel stride)
  int nry, nrx, items;        // regions per image, work items = NB*N*nry*nrx
  int win;                    // words of a channel window that are staged: R*Wp (<= 256)
  unsigned magicTC;           // dev::fast_div magic of TC
};

// Geometry of one work item (all values are wave-uniform).
struct Item {
  int rx, ry, n, cb;  // region column / row, image, channel block
  int y0, x0;         // window origin in the image (may be negative: zero padding)
  int cbn;            // real channels in the block
};

template <int M>
__device__ __forceinline__ Item decode_item(const InArgs& a, int item) {
  Item it;
  int t = item;
  it.rx = t % a.nrx; t /= a.nrx;
  it.ry = t % a.nry; t /= a.nry;
  it.n = t % a.N;
  it.cb = t / a.N;
  it.y0 = it.ry * a.TR * M - a.pad;
  it.x0 = it.rx * a.TC * M - a.pad;
  it.cbn = min(a.CB, a.C - it.cb * a.CB);
  return it;
}

// B8: the code width is 8 bits.
template <int M, bool B8>
__global__ __launch_bounds__(kThreads) void input_kernel(const InArgs a) {
  constexpr int A = M + 2, E = A * A;
  constexpr int kSlots = 4;   // a channel window has at most 64*kSlots words
  constexpr int kChan = 16;   // channels a wave stages per item: CB/4 <= 16
  extern __shared__ float lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept scalar
  const int cl = lane & 15, sub = (lane >> 4) & 1, hw = lane >> 5;
  const bool lane_on = cl < a.Q;
  const unsigned HW = (unsigned)a.H * (unsigned)a.W;

  // staging descriptors of this lane (the same for every channel and work item)
  unsigned s_goff[kSlots];
  int s_r[kSlots], s_x[kSlots];
  bool s_on[kSlots];
#pragma unroll
  for (int k = 0; k < kSlots; k++) {
    const int q = lane + 64 * k;
    const int r = q / a.Wp, xx = q - r * a.Wp;
    s_on[k] = q < a.win && xx < a.Wc;
    s_r[k] = r;
    s_x[k] = xx;
    s_goff[k] = (unsigned)(r * a.W + xx);
  }

  // Eq. 7 parameters as wave-uniform scalars (quantize pass)
  float qmn[E], qinv[E];
  {
#pragma unroll
    for (int e = 0; e < E; e++) {
      qmn[e] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a.qparams[2 * e])));
      qinv[e] =
          __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a.qparams[2 * e + 1])));
    }
  }
  const float L = (float)((1 << a.bits) - 1);
  const unsigned h = 1u << (a.bits - 1);
  const unsigned estride = (unsigned)a.NB * (unsigned)a.P * (unsigned)a.CB;  // bytes per position

  // Software pipeline over the items of this (persistent) workgroup: the loads of the next
  // item's window are in flight while the current one is transformed.
  float v[kChan][kSlots];
  auto issue_loads = [&](const Item& it) {
    // window pixel (row 0, column 0) of the block's first channel; may point outside the
    // tensor, it is only dereferenced where the pixel is inside the image
    const float* base =
        a.x + ((((long long)it.n * a.C + (long long)it.cb * a.CB) * a.H + it.y0) * (long long)a.W +
               it.x0);
    bool ok[kSlots];
#pragma unroll
    for (int k = 0; k < kSlots; k++) {
      const int gy = it.y0 + s_r[k], gx = it.x0 + s_x[k];
      ok[k] = s_on[k] && gy >= 0 && gy < a.H && gx >= 0 && gx < a.W;
    }
#pragma unroll
    for (int u = 0; u < kChan; u++) {
      const int c = wave + 4 * u;
      const float* cbase = base + (size_t)c * HW;  // wave-uniform
#pragma unroll
      for (int k = 0; k < kSlots; k++) {
        v[u][k] = 0.0f;
        if (ok[k] && c < it.cbn) v[u][k] = cbase[s_goff[k]];
      }
    }
  };
  auto commit_loads = [&](const Item& it) {
#pragma unroll
    for (int u = 0; u < kChan; u++) {
      const int c = wave + 4 * u;
      if (c < it.cbn) {
        float* dst = lds + c * a.CS + lane;
#pragma unroll
        for (int k = 0; k < kSlots; k++)
          if (lane + 64 * k < a.win) dst[64 * k] = v[u][k];
      }
    }
  };

  int item = blockIdx.x;
  if (item < a.items) issue_loads(decode_item<M>(a, item));
  while (item < a.items) {
    const Item it = decode_item<M>(a, item);
    __syncthreads();  // the previous item's compute phase has finished with LDS
    commit_loads(it);
    __syncthreads();
    const int next = item + gridDim.x;
    if (next < a.items) issue_loads(decode_item<M>(a, next));

    // this lane's four channels cl + i*Q: which of them are real
    unsigned realmask = 0;
    int nreal = 0;
#pragma unroll
    for (int i = 0; i < 4; i++)
      if (lane_on && cl + a.Q * i < it.cbn) { realmask |= 0xFFu << (8 * i); nreal++; }

    const int npairs = (a.TR / 2) * a.TC;
    for (int u = wave * 2 + hw; u < npairs; u += 8) {
      const int typ = dev::fast_div(u, a.magicTC), txl = u - typ * a.TC;
      const int tyl = 2 * typ + sub;
      const int ty = it.ry * a.TR + tyl, tx = it.rx * a.TC + txl;
      const bool valid = ty < a.th && tx < a.tw;
      const int p = (it.n * a.th + ty) * a.tw + tx;
      const float* tile0 = lds + cl * a.CS + tyl * M * a.Wp + txl * M;

      {
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
              // clamp(rne((x - min) * inv), 0, L): v_cvt_pk_u8_f32 rounds to nearest even and
              // saturates to [0, 255] (checked by the tie and clamp parity tests), so only the
              // upper clamp of narrower codes needs an instruction of its own
              float tq = (d[e / A][e % A] - qmn[e]) * qinv[e];
              if constexpr (!B8) tq = fminf(tq, L);
              pk[e] = __builtin_amdgcn_cvt_pk_u8_f32(tq, i, pk[e]);
            }
          }
        }
        const unsigned H8 = 0x80808080u, hh = h * 0x01010101u;
        int tot[E];
#pragma unroll
        for (int e = 0; e < E; e++) {
          // column sum of the signed codes: (sum of the unsigned bytes) - nreal*h
          tot[e] = dev::row16_sum((int)__builtin_amdgcn_sad_u8(pk[e], 0u, 0u) - nreal * (int)h);
          // per-byte (code - h) mod 256 without borrows between bytes (for h = 128 that is a
          // flip of the top bit), padding lanes -> 0
          if constexpr (B8)
            pk[e] = (pk[e] ^ H8) & realmask;
          else
            pk[e] = (((pk[e] | H8) - (hh & ~H8)) ^ ((pk[e] ^ ~hh) & H8)) & realmask;
        }
        // 32-bit byte offsets from the tensor bases (the descriptor check keeps them in range)
        const unsigned voff = ((unsigned)it.cb * (unsigned)a.P + (unsigned)p) * (unsigned)a.CB + 4u * cl;
        if (valid && lane_on) {
#pragma unroll
          for (int e = 0; e < E; e++)
            *reinterpret_cast<unsigned*>(reinterpret_cast<char*>(a.vq) + (voff + e * estride)) = pk[e];
        }
        if (valid && cl == 0) {
          const unsigned coff = (unsigned)p;
          if (a.NB > 1) {
#pragma unroll
            for (int e = 0; e < E; e++) atomicAdd(a.colsum + (coff + (unsigned)e * a.P), tot[e]);
          } else {
#pragma unroll
            for (int e = 0; e < E; e++) a.colsum[coff + (unsigned)e * a.P] = tot[e];
          }
        }
      }
    }
    item = next;
  }
}

// Region geometry.  Constraints: the LDS pitch satisfies m*Wp = 16 (mod 32); a channel window
// has at most 256 words; the window of all CB channels fits the LDS budget (two resident
// workgroups per CU).  Among those pick the shape that stages the fewest pixels per image (least
// halo, fewest out-of-range tiles, fewest idle lane slots).
bool choose_region(const Geo& g, InArgs* a) {
  const int M = g.m;
  const int mod = 32 / M, want = 16 / M;  // Wp = want (mod mod)
  const long long budget = 72 * 1024;
  long long best_cost = -1;
  for (int TC = 1; TC <= g.tw && TC <= 64; TC++) {
    const int Wc = TC * M + 2;
    const int Wp = Wc + ((want - Wc % mod) % mod + mod) % mod;
    for (int TR = 2; TR <= ((g.th + 1) & ~1) && TR <= 32; TR += 2) {
      const int R = TR * M + 2;
      const long long lds = (long long)g.CB * (R * Wp + 1) * 4;
      if (lds > budget || R * Wp > 256) break;
      const int nry = (g.th + TR - 1) / TR, nrx = (g.tw + TC - 1) / TC;
      const int pairs = (TR / 2) * TC;
      const long long cost =
          (long long)nry * nrx * ((long long)R * Wc + 4LL * ((pairs + 7) / 8 * 8 - pairs));
      if (best_cost < 0 || cost < best_cost) {
        best_cost = cost;
        a->TR = TR; a->TC = TC; a->Wp = Wp; a->R = R; a->Wc = Wc; a->CS = R * Wp + 1;
        a->nry = nry; a->nrx = nrx; a->win = R * Wp;
      }
    }
  }
  return best_cost >= 0;
}

hipError_t launch_quant_pass(const Geo& g, const InArgs& a, int grid, size_t lds, hipStream_t s) {
  const bool b8 = g.bits == 8;
  note_kernel("input_kernel");
  if (g.m == 2) {
    if (b8) input_kernel<2, true><<<grid, kThreads, lds, s>>>(a);
    else input_kernel<2, false><<<grid, kThreads, lds, s>>>(a);
  } else {
    if (b8) input_kernel<4, true><<<grid, kThreads, lds, s>>>(a);
    else input_kernel<4, false><<<grid, kThreads, lds, s>>>(a);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_input_transform(const Geo& g, const float* x, int8_t* vq, float* v_range,
                                  int32_t* v_colsum, char* ws, const Workspace& wl,
                                  hipStream_t s, const DqOut* dqo, hipEvent_t* ev) {
  InArgs a{};
  a.x = x; a.vq = vq; a.colsum = v_colsum;
  float* partial = reinterpret_cast<float*>(ws + wl.off_partial);
  float* qparams = reinterpret_cast<float*>(ws + wl.off_qparams);
  a.qparams = qparams;
  a.N = g.N; a.C = g.C; a.H = g.H; a.W = g.W; a.pad = g.pad; a.th = g.th; a.tw = g.tw;
  a.P = g.P; a.CB = g.CB; a.NB = g.NB; a.Q = g.Q; a.bits = g.bits;
  const bool nhwc = is_nhwc(g);  // takes the kernels of input_nhwc.hip: no LDS regions
  if (!nhwc && !choose_region(g, &a)) return hipErrorInvalidValue;
  a.magicTC = div_magic(a.TC);
  const long long items = (long long)g.NB * g.N * a.nry * a.nrx;
  if (items > INT_MAX) return hipErrorInvalidValue;
  a.items = (int)items;
  const size_t lds = (size_t)g.CB * a.CS * sizeof(float);

  const bool is_static = (g.flags & LANCE_INPUT_RANGE_STATIC) != 0;
  const int per_tensor = (g.flags & LANCE_RANGE_PER_TENSOR) ? 1 : 0;
  hipError_t e;
  int range_groups = 0;
  // column sums that are added to with atomics start at zero
  const bool need_zero = nhwc ? input_nhwc_adds_colsum_atomically(g) : g.NB > 1;
  if (ev && (e = hipEventRecord(ev[0], s)) != hipSuccess) return e;
  note_slot(0);
  if (!is_static) {
    e = launch_input_range(g, x, partial, v_colsum, need_zero, &range_groups, s);
    if (e != hipSuccess) return e;
  } else if (need_zero) {
    e = launch_fill_zero(v_colsum, (size_t)g.E * g.P, s);
    if (e != hipSuccess) return e;
  }
  if (ev && (e = hipEventRecord(ev[1], s)) != hipSuccess) return e;
  note_slot(1);
  // The quantize pass of 64-channel code blocks can reduce the records itself (no kernel between
  // the passes) unless somebody needs rk, which only the reduction kernel forms.
  const bool merge = input_quant_applicable(g) && !(dqo && dqo->want_rk) &&
                     input_quant_can_merge(g, range_groups);
  if (!merge) {
    e = launch_range_finalize(partial, range_groups, g.E, per_tensor, is_static, g.bits, v_range,
                              qparams, dqo, s);
    if (e != hipSuccess) return e;
  }
  if (ev && (e = hipEventRecord(ev[2], s)) != hipSuccess) return e;
  note_slot(2);
  if (nhwc) {
    e = launch_input_nhwc_quant(g, x, qparams, vq, v_colsum, s);
  } else if (input_quant_applicable(g)) {
    const QuantSource src{qparams, partial, range_groups, merge ? 1 : 0, v_range, dqo};
    e = launch_input_quant(g, x, src, vq, v_colsum, s);
  } else {
    if (is_packed(g)) return hipErrorInvalidValue;  // only the pass above packs its codes
    e = launch_quant_pass(g, a, a.items < kGroups ? a.items : kGroups, lds, s);
  }
  if (e != hipSuccess) return e;
  if (ev && (e = hipEventRecord(ev[3], s)) != hipSuccess) return e;
  note_slot(3);
  return hipSuccess;
}

}  // namespace lance
