// Reduction of the range pass's records and the constants of Eq. 7 and of the expanded Eq. 8,
// done by a 256-thread workgroup for itself at the start of a quantize pass: the records are a
// few tens of KB in L2, and a one-workgroup kernel between the two passes costs its run time plus
// a launch gap on the critical path of every layer.
//
// With ou = min_u + su*h, ov = min_v + sv*h (h = 2^(b-1), the shift of the stored codes):
//   M[e,k,p] = su*sv*ACC + (su*ov*rowsum[e][k] + C*ou*ov) + sv*ou*colsum[e][p]
// dq[e] = {su*sv, sv*ou, 0, 0} (binary32) and dqd[e] = {su*ov, C*ou*ov} (binary64) are what the
// product kernels read.
#pragma once
#include "lance_device.h"

namespace lance {
namespace dev {

// Where a workgroup wants the Eq. 8 constants in LDS (any pointer may be null: not wanted).
struct Eq8Lds {
  float* sc_s;       // [E] su*sv
  float* gc_s;       // [E] sv*ou
  double* rmul_s;    // [E] su*ov
  double* kconst_s;  // [E] C*ou*ov
};

struct RangeSource {
  const float* qparams;   // finished Eq. 7 parameters [E][2] = {min, inv}; used when !merge
  const float* partial;   // records [count][E][2] of the range pass (merge, dynamic ranges)
  float* v_range;         // [E][2]: written by the publishing workgroup (dynamic), read (static)
  const float* u_range;   // filter ranges [E][2], or nullptr: no Eq. 8 constants wanted
  float* dq;              // [E][4], written by the publishing workgroup
  double* dqd;            // [E][2], written by the publishing workgroup
  int count, merge, is_static, per_tensor, bits, C;  // bits: width of the input codes
  int bits_w;                                         // width of the filter codes
  int bias;  // the product kernel multiplies (code + bias): dq[1] and dqd[0] lose bias*su*sv
};

// LDS floats needed beyond `red`: res_s[2E] and qp_s[2E].
template <int E>
constexpr int range_reduce_lds_floats() { return 4 * E; }

// Called by all 256 threads.  red: LDS scratch of at least 4 KB that nobody else touches until
// this returns.  On return (after a barrier) qp_s[2e] = min, qp_s[2e+1] = inv of position e.
// publish: this workgroup also writes v_range (dynamic ranges), dq and dqd to memory.
// Threads beyond 256 may call too (they only meet the barriers).  lds (optional): also leave the
// Eq. 8 constants in LDS (needs r.u_range).
template <int E>
__device__ __forceinline__ void ranges_to_lds(const RangeSource& r, float* red, float* res_s,
                                              float* qp_s, int tid, bool publish,
                                              const Eq8Lds* lds = nullptr) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  constexpr int kThreads = 256;
  constexpr int kPieces = E / 2;               // 16-byte pieces of a record: two positions each
  constexpr int kGroups = kThreads / kPieces;  // records in flight side by side
  static_assert(kGroups * 2 * E * sizeof(float) <= 4096, "red holds one partial row per group");
  if (!r.merge) {
    if (tid < 2 * E) qp_s[tid] = r.qparams[tid];
    __syncthreads();
    return;
  }
  const int piece = tid % kPieces, grp = tid / kPieces;
  f4 v = {INFINITY, -INFINITY, INFINITY, -INFINITY};  // {min, max} of positions 2*piece, +1
  if (!r.is_static && grp < kGroups) {
    // all loads of a batch are requested before the first is used
    constexpr int kBatch = 16;
    for (int row0 = grp; row0 < r.count; row0 += kBatch * kGroups) {
      f4 xv[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; u++) {
        const int row = row0 + u * kGroups;
        xv[u] = row < r.count
                    ? *reinterpret_cast<const f4*>(r.partial + (size_t)row * (2 * E) + 4 * piece)
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
  if (r.u_range && tid < E) {
    float iu;
    quant_params(r.u_range[2 * tid], r.u_range[2 * tid + 1], r.bits_w, &iu, &su);
    ou = (double)r.u_range[2 * tid] + (double)su * (double)(1 << (r.bits_w - 1));
  }
  if (r.is_static) {
    if (tid < 2 * E) res_s[tid] = r.v_range[tid];
  } else {
    if (grp < kGroups) *reinterpret_cast<f4*>(red + grp * 2 * E + 4 * piece) = v;
    __syncthreads();
    // column = (position, min|max): kGroups partial rows -> kFan -> 1
    constexpr int kFan = kThreads / (2 * E), kPer = (kGroups + kFan - 1) / kFan;
    float x = 0.0f;
    const int col = tid % (2 * E), part = tid / (2 * E);
    const bool is_max = col & 1;
    const bool active = part < kFan;
    if (active) {
      x = is_max ? -INFINITY : INFINITY;
#pragma unroll
      for (int i = 0; i < kPer; i++) {
        const int g2 = part * kPer + i;
        if (g2 < kGroups) {
          const float y = red[g2 * 2 * E + col];
          x = is_max ? fmaxf(x, y) : fminf(x, y);
        }
      }
    }
    __syncthreads();
    if (active) red[part * 2 * E + col] = x;
    __syncthreads();
    if (tid < 2 * E) {
      float y = red[tid];
#pragma unroll
      for (int i = 1; i < kFan; i++) y = is_max ? fmaxf(y, red[i * 2 * E + tid]) : fminf(y, red[i * 2 * E + tid]);
      res_s[tid] = y;
    }
  }
  __syncthreads();
  if (tid < E) {
    float lo = res_s[2 * tid], hi = res_s[2 * tid + 1];
    if (r.per_tensor && !r.is_static) {
      for (int e = 0; e < E; e++) { lo = fminf(lo, res_s[2 * e]); hi = fmaxf(hi, res_s[2 * e + 1]); }
    }
    float inv, sv;
    quant_params(lo, hi, r.bits, &inv, &sv);
    qp_s[2 * tid] = lo;
    qp_s[2 * tid + 1] = inv;
    if (lds) {
      const double ov = (double)lo + (double)sv * (double)(1 << (r.bits - 1));
      const double sb = (double)r.bias * ((double)su * (double)sv);
      if (lds->sc_s) lds->sc_s[tid] = (float)((double)su * (double)sv);
      if (lds->gc_s) lds->gc_s[tid] = (float)((double)sv * ou - sb);
      if (lds->rmul_s) lds->rmul_s[tid] = (double)su * ov - sb;
      if (lds->kconst_s) lds->kconst_s[tid] = (double)r.C * ou * ov;
    }
    if (publish) {
      if (!r.is_static) {
        r.v_range[2 * tid] = lo;
        r.v_range[2 * tid + 1] = hi;
      }
      if (r.u_range && r.dq) {
        const double ov = (double)lo + (double)sv * (double)(1 << (r.bits - 1));
        const double sb = (double)r.bias * ((double)su * (double)sv);
        r.dq[4 * tid + 0] = (float)((double)su * (double)sv);
        r.dq[4 * tid + 1] = (float)((double)sv * ou - sb);
        r.dq[4 * tid + 2] = 0.0f;
        r.dq[4 * tid + 3] = 0.0f;
        r.dqd[2 * tid + 0] = (double)su * ov - sb;
        r.dqd[2 * tid + 1] = (double)r.C * ou * ov;
      }
    }
  }
  __syncthreads();
}

}  // namespace dev
}  // namespace lance
