// Internal declarations shared by the liblance translation units (host side + launchers).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "lance.h"

namespace lance {

// Layer geometry derived from a validated descriptor (Sec. 2.3: tiling into (m+2)^2 patches).
struct Geo {
  int N, C, H, W, K, pad, m, bits;  // bits: width of the input codes
  int bits_w;                       // width of the filter codes
  unsigned flags;
  int alpha, E;      // m+2, (m+2)^2
  int Ho, Wo, th, tw;
  int P;             // N*th*tw
  int Cp, CB, NB, Q; // padded channels, channel block, blocks, dwords per block row
};

// Fills g; returns LANCE_OK or the validation error.  Touches no HIP API.
int make_geo(const lance_conv_desc* d, Geo* g);

inline bool is_nhwc(const Geo& g) { return (g.flags & LANCE_LAYOUT_NHWC) != 0; }
// Two 4-bit codes per byte in uq and vq (block rows of 32 bytes).
inline bool is_packed(const Geo& g) { return (g.flags & LANCE_CODES_PACKED4) != 0; }
// Bytes of one block row of the code tensors.
inline int code_row_bytes(const Geo& g) { return is_packed(g) ? g.CB / 2 : g.CB; }
// What the matrix cores are fed instead of the stored code: stored code + code_bias(g) (packed
// codes go in as their unsigned nibbles; Eq. 8's constants absorb the difference).
inline int code_bias(const Geo& g) { return is_packed(g) ? 8 : 0; }

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Host side of dev::fast_div: ceil(2^32 / d), with 0 standing for d == 1.
inline unsigned div_magic(int d) { return d <= 1 ? 0u : (unsigned)(((1ULL << 32) + d - 1) / d); }

// Largest number of range-pass workgroups (each writes one partial (min,max) per position).
constexpr int kMaxRangeGroups = 1024;

// Workspace carve-up for the input transform / the fused convolution.
struct Workspace {
  size_t off_partial;  // float [kMaxRangeGroups][E][2]
  size_t off_qparams;  // float [E][2] = {min, inv}
  size_t off_dq;       // float [E][4] (a = su*sv, sv*ou, spare, spare)
  size_t off_rk;       // float [m*m][K]: filter-side de-quantization terms after A^T . A
  size_t off_dqd;      // double [E][2] = {su*ov, C*ou*ov}: what rk is formed from
  size_t off_vrange;   // float [E][2] (when the caller passes none)
  size_t off_colsum;   // int32 [E][P]   (fused conv only)
  size_t off_vq;       // int8  vq       (fused conv only)
  size_t input_bytes, conv_bytes;
};
Workspace make_workspace(const Geo& g);

// Which kernel ran in which slot of the timing twin of the fused call.  Only that twin installs a
// sink (per thread); everywhere else both functions do nothing.
struct KernelNotes {
  const char* name[LANCE_PROFILE_KERNELS];
  int slot;
};
extern thread_local KernelNotes* g_kernel_notes;
inline void note_slot(int slot) { if (g_kernel_notes) g_kernel_notes->slot = slot; }
inline void note_kernel(const char* name) {
  if (g_kernel_notes && g_kernel_notes->slot >= 0 && g_kernel_notes->slot < LANCE_PROFILE_KERNELS)
    g_kernel_notes->name[g_kernel_notes->slot] = name;
}

// Kernel launchers (each enqueues on `s` and returns the launch status).
// Where the constants of the expanded Eq. 8 go (fused convolution only).
struct DqOut {
  const float* u_range;
  const int32_t* u_rowsum;
  float* dq;    // [E][4]
  float* rk;    // [m*m][K]; written only if want_rk
  double* dqd;  // [E][2] = {su*ov, C*ou*ov}
  int K, C;
  int want_rk;  // 0: the product kernel forms its own rk from dqd and the filter row sums
  int bits_w;   // width of the filter codes (u_range belongs to them)
  int bias;     // code_bias(): the product kernel multiplies (code + bias); with s = su*sv the
                // constants become dq[1] = sv*ou - bias*s and dqd[0] = su*ov - bias*s (the term
                // bias^2 * Cp is taken off the integer sums by the product kernel itself)
};
// Reduces `count` partial records [count][E][2] into range[E][2] (skipped when is_static: the
// caller's range is used as is); if qparams != nullptr writes qparams[E][2] = {min, inv}; if
// dqo != nullptr also writes the de-quantization constants.
hipError_t launch_range_finalize(const float* partial, int count, int E, int per_tensor,
                                 int is_static, int bits, float* range, float* qparams,
                                 const DqOut* dqo, hipStream_t s);
hipError_t launch_fill_zero(int32_t* p, size_t n, hipStream_t s);
// Quantize, multiply and transform back in one kernel for F(4x4,3x3) layers of at most 128
// channels (conv_fused_m4.hip).  merge != 0: the kernel forms the Eq. 7 / Eq. 8 constants itself
// from v_range (static ranges) or the `count` records in `partial`; merge == 0: qparams, dq and dqd
// are finished (launch_range_finalize with a DqOut).
bool conv_fused_m4_applicable(const Geo& g);
bool conv_fused_m4_can_merge(const Geo& g, int count);
hipError_t launch_conv_fused_m4(const Geo& g, const float* x, const int8_t* uq,
                                const float* u_range, const int32_t* u_rowsum,
                                const float* partial, int count, int merge, const float* qparams,
                                const float* dq, const double* dqd, float* v_range, float* y,
                                hipStream_t s);
// Range pass over X: writes *groups_out partial records [groups][E][2] (groups <= kMaxRangeGroups);
// clears colsum[E][P] first if zero_colsum.
hipError_t launch_input_range(const Geo& g, const float* x, float* partial, int32_t* colsum,
                              int zero_colsum, int* groups_out, hipStream_t s);
// Stage 2 on NHWC activations (input_nhwc.hip): the range pass (used by launch_input_range) and
// the quantize pass with finished Eq. 7 parameters qparams [E][2] = {min, inv}.
hipError_t launch_input_nhwc_range(const Geo& g, const float* x, float* partial, int32_t* colsum,
                                   int zero_colsum, int* groups_out, hipStream_t s);
// True if the quantize pass adds to the column sums with atomics (they must be zero before it).
bool input_nhwc_adds_colsum_atomically(const Geo& g);
hipError_t launch_input_nhwc_quant(const Geo& g, const float* x, const float* qparams, int8_t* vq,
                                   int32_t* colsum, hipStream_t s);
// The same pass with every pixel loaded once per strip of tile rows (input_range_strip.hip);
// used by launch_input_range when applicable.
bool input_range_strip_applicable(const Geo& g, const float* x);
hipError_t launch_input_range_strip(const Geo& g, const float* x, float* partial, int32_t* colsum,
                                    int zero_colsum, int* groups_out, hipStream_t s);
// Blocks of 64 tiles whose pixels are addressed by 32-bit offsets (see input_range.hip).
unsigned tile_block_reach(const Geo& g, int* bpi, int* blocks);
// Patch rows may be loaded with one wide load each (see patch_loader.h).
inline bool patch_rows_allowed(const Geo& g) {
  return g.pad <= 1 && g.W >= g.m + 2 && (long long)g.H * g.W >= 8;
}
// With pad = 1 and a width that is a multiple of m, only the first and the last column of a
// patch can lie outside the image.
inline bool patch_edge_cols_only(const Geo& g) { return g.pad == 1 && g.W % g.m == 0; }
// Load mode of the kernels built on patch_loader.h: 0 = pixel by pixel, 1 = by rows, any column
// may be outside, 2 = by rows, only edge columns may be outside.
inline int patch_load_mode(const Geo& g) {
  return !patch_rows_allowed(g) ? 0 : (patch_edge_cols_only(g) ? 2 : 1);
}
hipError_t launch_filter_transform(const Geo& g, const float* w, int8_t* uq, float* u_range,
                                   int32_t* u_rowsum, hipStream_t s);
// ev (optional, 4 events): recorded before the range pass and after the range pass, the range
// reduction and the quantize pass.  dqo (optional): see launch_range_finalize.
hipError_t launch_input_transform(const Geo& g, const float* x, int8_t* vq, float* v_range,
                                  int32_t* v_colsum, char* ws, const Workspace& wl,
                                  hipStream_t s, const DqOut* dqo = nullptr,
                                  hipEvent_t* ev = nullptr);
// Quantize pass of layers with 64-channel code blocks (see input_quant.hip); used by
// launch_input_transform when applicable.
bool input_quant_applicable(const Geo& g);
// Where the quantize pass takes its Eq. 7 parameters from.  merge == 0: qparams [E][2], finished
// by launch_range_finalize.  merge == 1: every workgroup reduces the `count` records in
// `partial` (or, with static ranges, reads v_range) and forms the parameters itself; the first
// workgroup writes v_range (dynamic ranges) and, when dqo is given, dq and dqd (never rk).
struct QuantSource {
  const float* qparams;
  const float* partial;
  int count;
  int merge;
  float* v_range;
  const DqOut* dqo;
};
bool input_quant_can_merge(const Geo& g, int count);
hipError_t launch_input_quant(const Geo& g, const float* x, const QuantSource& src, int8_t* vq,
                              int32_t* colsum, hipStream_t s);
hipError_t launch_gemm_i8(const Geo& g, const int8_t* uq, const int8_t* vq, int32_t* acc,
                          hipStream_t s);
// LDS-tiled stage 3 for 64-channel code blocks (gemm_i8_tiled.hip); used by launch_gemm_i8.
bool gemm_i8_tiled_applicable(const Geo& g);
hipError_t launch_gemm_i8_tiled(const Geo& g, const int8_t* uq, const int8_t* vq, int32_t* acc,
                                hipStream_t s);
hipError_t launch_output_transform(const Geo& g, const int32_t* acc, const float* u_range,
                                   const int32_t* u_rowsum, const float* v_range,
                                   const int32_t* v_colsum, float* y, hipStream_t s);
// True if launch_gemm_fused reads rk (else it forms the terms itself from dqd and u_rowsum).
bool gemm_fused_wants_rk(const Geo& g);
hipError_t launch_gemm_fused(const Geo& g, const int8_t* uq, const int8_t* vq,
                             const int32_t* v_colsum, const float* dq, const float* rk,
                             const double* dqd, const int32_t* u_rowsum, float* y, hipStream_t s);
// Range reduction, quantize pass, products and epilogue in one kernel (see conv_fused_c64.hip).
// partial/count: the records of launch_input_range (unused with static input ranges, which are
// read from v_range; otherwise v_range receives the reduced ranges).
bool conv_fused_c64_applicable(const Geo& g);
hipError_t launch_conv_fused_c64(const Geo& g, const float* x, const int8_t* uq,
                                 const float* u_range, const int32_t* u_rowsum,
                                 const float* partial, int count, float* v_range, float* y,
                                 hipStream_t s);
// The same for layers with two 64-channel blocks (see conv_fused_c128.hip).
bool conv_fused_c128_applicable(const Geo& g);
hipError_t launch_conv_fused_c128(const Geo& g, const float* x, const int8_t* uq,
                                  const float* u_range, const int32_t* u_rowsum,
                                  const float* partial, int count, float* v_range, float* y,
                                  hipStream_t s);
// Quantize pass, products and epilogue in one kernel for F(2x2,3x3) layers with at most 16
// channels (see conv_fused_c16.hip); qparams, dq and dqd come from launch_range_finalize.
bool conv_fused_c16_applicable(const Geo& g);
// static_v_range != nullptr (caller-supplied ranges): the kernel forms parameters and constants
// itself from it and u_range, and qparams, dq, dqd are not read.
hipError_t launch_conv_fused_c16(const Geo& g, const float* x, const int8_t* uq,
                                 const float* qparams, const float* dq, const double* dqd,
                                 const int32_t* u_rowsum, float* y, const float* static_v_range,
                                 const float* u_range, hipStream_t s);
// LDS-tiled fused GEMM for F(2x2,3x3) layers with several channel blocks (gemm_fused_tiled.hip).
bool gemm_fused_tiled_applicable(const Geo& g);
hipError_t launch_gemm_fused_tiled(const Geo& g, const int8_t* uq, const int8_t* vq,
                                   const int32_t* v_colsum, const float* dq, const double* dqd,
                                   const int32_t* u_rowsum, float* y, hipStream_t s);
// True when launch_gemm_fused_tiled would run its streaming kernel and that is the fastest plan.
bool gemm_fused_stream_m2_preferred(const Geo& g);
// Fused GEMM for F(2x2,3x3) layers with several channel blocks and small grids: one wave per
// row of the position grid, no barrier in the product loop (gemm_fused_rows.hip).
bool gemm_fused_rows_applicable(const Geo& g);
hipError_t launch_gemm_fused_rows(const Geo& g, const int8_t* uq, const int8_t* vq,
                                  const int32_t* v_colsum, const float* dq, const double* dqd,
                                  const int32_t* u_rowsum, float* y, hipStream_t s);
// LDS-tiled fused GEMM for F(4x4,3x3) layers with 64-channel code blocks (gemm_fused_tiled_m4.hip).
bool gemm_fused_tiled_m4_applicable(const Geo& g);
// Fused GEMM on packed 4-bit codes, F(2x2,3x3) (gemm_fused_packed.hip).
bool gemm_fused_packed_applicable(const Geo& g);
hipError_t launch_gemm_fused_packed(const Geo& g, const int8_t* uq, const int8_t* vq,
                                    const int32_t* v_colsum, const float* dq, const double* dqd,
                                    const int32_t* u_rowsum, float* y, hipStream_t s);
// The same for F(4x4,3x3) (gemm_fused_tiled_m4.hip).
bool gemm_fused_packed_m4_applicable(const Geo& g);
hipError_t launch_gemm_fused_packed_m4(const Geo& g, const int8_t* uq, const int8_t* vq,
                                       const int32_t* v_colsum, const float* dq, const double* dqd,
                                       const int32_t* u_rowsum, float* y, hipStream_t s);
hipError_t launch_gemm_fused_tiled_m4(const Geo& g, const int8_t* uq, const int8_t* vq,
                                      const int32_t* v_colsum, const float* dq, const double* dqd,
                                      const int32_t* u_rowsum, float* y, hipStream_t s);
// Algorithm 1 with per-matrix ranges and a binary32 channel sum (alg1_literal.hip).
hipError_t launch_alg1_literal(const Geo& g, const float* x, const float* w, float* y,
                               hipStream_t s);
// Weight-only quantization: de-quantized filter codes times the unquantized transformed input in
// binary32 (weight_only.hip).
hipError_t launch_weight_only(const Geo& g, const float* x, const int8_t* uq, const float* u_range,
                              float* y, hipStream_t s);
hipError_t launch_direct_conv(const Geo& g, const float* x, const float* w, float* y,
                              hipStream_t s);

}  // namespace lance
