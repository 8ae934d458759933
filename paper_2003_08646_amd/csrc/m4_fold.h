// The fold of F(4x4,3x3)'s 36 positions into the 16 outputs of a tile and filter (Eq. 9 applied to
// the first term of the expanded Eq. 8), on the accumulator registers of v_mfma_i32_16x16x64_i8,
// with compile-time positions.  Shared by the kernels that multiply F(4x4,3x3) codes.
#pragma once
#include "lance_device.h"
#include <utility>

namespace lance {
namespace m4e {

typedef int v4i __attribute__((ext_vector_type(4)));

// A^T of F(4x4,3x3) (points 0, 1, -1, 2, -2, inf), for compile-time indices.
constexpr float kAt[4][6] = {
    {1, 1, 1, 1, 1, 0}, {0, 1, -1, 2, -2, 0}, {0, 1, 1, 4, 4, 0}, {0, 1, -1, 8, -8, 1}};

template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{})
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

typedef float v4f __attribute__((ext_vector_type(4)));

// Position e = (gi, gj) is complete: rowacc[b] += A^T[b][gj] s_e ACC, and at the end of grid row
// gi out[a][b] += A^T[a][gi] rowacc[b]; zero coefficients cost nothing (e is a compile-time
// constant).
// bias2: what every integer sum carries beyond the product of the stored codes (0, or 64 * Cp for
// packed codes, which are multiplied as code + 8).
// se: the scale s_e = scale_u * scale_v of position e.
template <int e>
__device__ __forceinline__ void m4_fold(const v4i& acc, const float se, v4f (&rowacc)[4],
                                        v4f (&out)[4][4], const int bias2 = 0) {
  constexpr int M = 4, A = 6, gi = e / A, gj = e % A;
  // The sums are first read in the tail, in another basic block: left alone the compiler sinks
  // the folds of all positions down there and keeps every position's accumulators (in scratch
  // memory) until then.  The empty statements tie them to their position.
  auto pin = [](v4f& x) { asm volatile("" : "+v"(x)); };
  __builtin_amdgcn_sched_barrier(0);
  float accf[4];
#pragma unroll
  for (int r = 0; r < 4; r++) accf[r] = (float)(acc[r] - bias2);
  static_for<M>([&](auto bc) {
    constexpr int b = decltype(bc)::value;
    constexpr float cj = kAt[b][gj];
    if constexpr (cj != 0.0f) {
      const float cs = cj * se;
#pragma unroll
      for (int r = 0; r < 4; r++) rowacc[b][r] = __builtin_fmaf(cs, accf[r], rowacc[b][r]);
      pin(rowacc[b]);
    }
  });
  if constexpr (gj == A - 1) {
    static_for<M>([&](auto ac) {
      constexpr int aa = decltype(ac)::value;
      constexpr float ca = kAt[aa][gi];
      if constexpr (ca != 0.0f) {
#pragma unroll
        for (int b = 0; b < M; b++)
#pragma unroll
          for (int r = 0; r < 4; r++)
            out[aa][b][r] = __builtin_fmaf(ca, rowacc[b][r], out[aa][b][r]);
#pragma unroll
        for (int b = 0; b < M; b++) pin(out[aa][b]);
      }
    });
#pragma unroll
    for (int b = 0; b < M; b++) rowacc[b] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
  }
  __builtin_amdgcn_sched_barrier(0);
}
// ... with the scales in a table (LDS): the read happens after the scheduling barrier.
template <int e>
__device__ __forceinline__ void m4_fold(const v4i& acc, const float* sc_s, v4f (&rowacc)[4],
                                        v4f (&out)[4][4], const int bias2 = 0) {
  __builtin_amdgcn_sched_barrier(0);
  m4_fold<e>(acc, sc_s[e], rowacc, out, bias2);
}

}  // namespace m4e
}  // namespace lance
