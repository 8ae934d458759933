// Stage 2, second pass for F(2x2,3x3) layers of any channel count: v^ = Q(B^T d B) for every
// input patch (Algorithm 1; Eq. 7), NCHW fp32 in, blocked int8 codes and their column sums out.
// The ranges come from the first pass (input_range.hip) and its reduction.
//
// A workgroup takes 64 consecutive tiles and one block of 64 channels, transforms and quantizes
// them into LDS code rows (quant_phase.h: lane = tile, no pixel staging), then copies the 16
// position planes of 64 rows x 64 bytes to vq with fully coalesced 16-byte stores (the rows of
// consecutive tiles are contiguous in vq).  Each XCD takes a contiguous range of tile blocks.
#include "lance_device.h"
#include "lance_internal.h"
#include "quant_phase.h"

namespace lance {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

struct QArgs {
  dev::QuantBlockGeo g;
  int8_t* vq;             // [E][NB][P][64]
  int32_t* colsum;        // [E][P]
  const float* qparams;   // [E][2] = {min, inv}
  int NB, TB;             // channel blocks, tile blocks
};

template <bool B8, bool FULL, int MODE>
__global__ __launch_bounds__(kThreads, 2) void input_quant_m2_kernel(const QArgs a) {
  constexpr int E = 16;
  extern __shared__ char smem[];
  char* ring = smem;                                    // [E][64 rows][64 B]
  int* cs_s = reinterpret_cast<int*>(smem + E * 4096);  // [E][64]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // work item = (channel block, tile block); tile blocks of one channel block are consecutive
  const int item = dev::xcd_contiguous(blockIdx.x, gridDim.x);
  const int cb = item / a.TB, tb = item - cb * a.TB;
  const int p0 = tb * 64;
  const int P = a.g.P;

  for (int i = tid; i < E * 64; i += kThreads) cs_s[i] = 0;
  auto mid = [&]() { __syncthreads(); };  // the column sums start at zero
  auto qp = [&](int e, float* mn, float* inv) { *mn = a.qparams[2 * e]; *inv = a.qparams[2 * e + 1]; };
  dev::quantize_block_to_lds<B8, FULL, MODE>(a.g, p0, cb * 64, ring, cs_s, lane, wave, mid, qp);
  __syncthreads();

  // copy-out: thread = (row, chunk) of a plane; 256 threads move one 4 KB plane per pass
  const int row = tid >> 2, chunk = tid & 3;
  if (p0 + row < P) {
    const unsigned src = dev::code_row_offset(row, chunk);
    int8_t* dst = a.vq + ((size_t)cb * P + p0 + row) * 64 + chunk * 16;
    const size_t plane = (size_t)a.NB * P * 64;  // bytes per position
    v4i v[E];
#pragma unroll
    for (int e = 0; e < E; e++) v[e] = *reinterpret_cast<const v4i*>(ring + e * 4096 + src);
#pragma unroll
    for (int e = 0; e < E; e++) *reinterpret_cast<v4i*>(dst + (size_t)e * plane) = v[e];
  }
  // column sums of the signed codes: (sum of the unsigned bytes) - h * (channels of the block)
  const int cbn = min(64, a.g.C - cb * 64);
  const int hsum = cbn * (1 << (a.g.bits - 1));
  for (int i = tid; i < E * 64; i += kThreads) {
    const int e = i >> 6, t = i & 63;
    if (p0 + t < P) {
      const int v = cs_s[i] - hsum;
      if (a.NB > 1)
        atomicAdd(a.colsum + (size_t)e * P + p0 + t, v);
      else
        a.colsum[(size_t)e * P + p0 + t] = v;
    }
  }
}

constexpr size_t kLdsBytes = 16 * 4096 + 16 * 64 * sizeof(int);

template <bool B8, bool FULL, int MODE>
hipError_t launch_variant(const QArgs& a, unsigned grid, hipStream_t s) {
  auto kern = input_quant_m2_kernel<B8, FULL, MODE>;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes);
  if (e != hipSuccess) return e;
  kern<<<grid, kThreads, kLdsBytes, s>>>(a);
  return hipGetLastError();
}

template <bool B8, bool FULL>
hipError_t launch_rows(const Geo& g, const QArgs& a, unsigned grid, hipStream_t s) {
  switch (patch_load_mode(g)) {
    case 0: return launch_variant<B8, FULL, 0>(a, grid, s);
    case 1: return launch_variant<B8, FULL, 1>(a, grid, s);
    default: return launch_variant<B8, FULL, 2>(a, grid, s);
  }
}

long long block_reach_bytes(const Geo& g) {
  const long long tiles = (long long)g.th * g.tw;
  const long long images = 63 / tiles + 2;  // images a block of 64 consecutive tiles can touch
  return images * g.C * g.H * g.W * 4LL;
}

}  // namespace

// F(2x2,3x3), 64-channel code blocks, and byte offsets below 2^31 from the first image of a
// 64-tile block to every pixel it reads.
bool input_quant_m2_applicable(const Geo& g) {
  return g.m == 2 && g.CB == 64 && block_reach_bytes(g) < (1LL << 31) &&
         (long long)g.NB * ((g.P + 63) / 64) < (1LL << 31);
}

// colsum must have been cleared when NB > 1 (the range pass does it).
hipError_t launch_input_quant_m2(const Geo& g, const float* x, const float* qparams, int8_t* vq,
                                 int32_t* colsum, hipStream_t s) {
  if (!input_quant_m2_applicable(g)) return hipErrorInvalidValue;
  QArgs a{};
  a.g = dev::QuantBlockGeo{x, g.N, g.C, g.H, g.W, g.pad, g.th, g.tw, g.P, g.bits,
                           (unsigned)block_reach_bytes(g)};
  a.vq = vq; a.colsum = colsum; a.qparams = qparams;
  a.NB = g.NB; a.TB = (g.P + 63) / 64;
  const unsigned grid = (unsigned)(a.NB * a.TB);
  const bool b8 = g.bits == 8, full = g.C % 64 == 0;
  if (b8) return full ? launch_rows<true, true>(g, a, grid, s) : launch_rows<true, false>(g, a, grid, s);
  return full ? launch_rows<false, true>(g, a, grid, s) : launch_rows<false, false>(g, a, grid, s);
}

}  // namespace lance
