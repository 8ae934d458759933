// liblance host side: descriptor validation, size queries and the C-ABI entry points.
// Every entry point validates before the first HIP call, so argument errors are reported on a
// machine without a GPU.
#include <limits.h>

#include "lance_internal.h"
#include <atomic>
#include <cstdlib>

namespace lance {

thread_local KernelNotes* g_kernel_notes = nullptr;

int make_geo(const lance_conv_desc* d, Geo* g) {
  if (!d || !g) return LANCE_ERR_INVALID_ARG;
  if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->K <= 0 || d->pad < 0)
    return LANCE_ERR_INVALID_ARG;
  if (d->m != 2 && d->m != 4) return LANCE_ERR_UNSUPPORTED;
  if (d->bits < 2 || d->bits > 8) return LANCE_ERR_UNSUPPORTED;
  if (d->flags & ~(uint32_t)(LANCE_RANGE_PER_TENSOR | LANCE_INPUT_RANGE_STATIC | LANCE_PLAN_WIDE_TILES |
                             LANCE_LAYOUT_NHWC | LANCE_CODES_PACKED4 | LANCE_FILTER_BITS_MASK))
    return LANCE_ERR_UNSUPPORTED;
  const int bits_w_field = (int)((d->flags & LANCE_FILTER_BITS_MASK) >> LANCE_FILTER_BITS_SHIFT);
  if (bits_w_field != 0 && (bits_w_field < 2 || bits_w_field > 8)) return LANCE_ERR_UNSUPPORTED;
  long long Ho = (long long)d->H + 2LL * d->pad - 2, Wo = (long long)d->W + 2LL * d->pad - 2;
  if (Ho <= 0 || Wo <= 0) return LANCE_ERR_INVALID_ARG;  // empty output
  if (d->pad > 1 << 20 || Ho > INT_MAX / 4 || Wo > INT_MAX / 4) return LANCE_ERR_UNSUPPORTED;
  g->N = d->N; g->C = d->C; g->H = d->H; g->W = d->W; g->K = d->K; g->pad = d->pad;
  g->m = d->m; g->bits = d->bits; g->flags = d->flags;
  g->bits_w = bits_w_field ? bits_w_field : d->bits;
  if ((d->flags & LANCE_CODES_PACKED4) &&
      (d->bits > 4 || g->bits_w > 4 || d->C <= 16))
    return LANCE_ERR_UNSUPPORTED;
  g->alpha = d->m + 2; g->E = g->alpha * g->alpha;
  g->Ho = (int)Ho; g->Wo = (int)Wo;
  g->th = (g->Ho + g->m - 1) / g->m; g->tw = (g->Wo + g->m - 1) / g->m;
  long long P = (long long)d->N * g->th * g->tw;
  // one 16-channel block for the narrowest layers, 64-channel blocks for all others (the fast
  // kernels work on 64-byte code rows; padding lanes hold code 0 and cost matrix-unit time only)
  g->Cp = d->C <= 16 ? 16 : (d->C + 63) / 64 * 64;
  g->CB = g->Cp < 64 ? g->Cp : 64;
  g->NB = g->Cp / g->CB;
  g->Q = g->CB / 4;
  // Kernel index arithmetic is 32-bit: every tensor stays below 4 GiB, a dimension that becomes
  // a grid's y or z extent below 65536, and the pixels that 64 consecutive tiles read within
  // 2^31 bytes of the first of their images (far beyond any of the paper's layer shapes).
  const long long lim = 1LL << 31, lim_bytes = 0xFFFFFFF0LL;
  if (d->K > 65535 || d->N > 65535) return LANCE_ERR_UNSUPPORTED;
  const long long tiles_per_image = (long long)g->th * g->tw;
  const long long images_per_block = 63 / tiles_per_image + 2;
  if (P >= lim || (long long)d->N * d->C * d->H * d->W * 4 >= lim_bytes ||
      (long long)d->N * d->K * Ho * Wo * 4 >= lim_bytes ||
      (long long)g->E * P * g->Cp >= lim_bytes || (long long)g->E * d->K * g->Cp >= lim_bytes ||
      (long long)g->E * P >= lim / 2 ||
      (images_per_block * d->C + 2) * d->H * d->W * 4 >= lim ||
      d->C > (1 << 17) /* int32 accumulator: C * 2^14 < 2^31 */)
    return LANCE_ERR_UNSUPPORTED;
  g->P = (int)P;
  return LANCE_OK;
}

Workspace make_workspace(const Geo& g) {
  Workspace w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  w.off_partial = take((size_t)kMaxRangeGroups * g.E * 2 * sizeof(float));
  w.off_qparams = take((size_t)g.E * 2 * sizeof(float));
  w.input_bytes = off;
  w.off_dq = take((size_t)g.E * 4 * sizeof(float));
  w.off_rk = take((size_t)g.E * g.K * sizeof(float));
  w.off_dqd = take((size_t)g.E * 2 * sizeof(double));
  w.off_vrange = take((size_t)g.E * 2 * sizeof(float));
  w.off_colsum = take((size_t)g.E * g.P * sizeof(int32_t));
  w.off_vq = take((size_t)g.E * g.P * g.NB * code_row_bytes(g));
  w.conv_bytes = off;
  return w;
}

}  // namespace lance

using namespace lance;

extern "C" {

int lance_query_sizes(const lance_conv_desc* desc, lance_sizes* out) {
  if (!out) return LANCE_ERR_INVALID_ARG;
  Geo g;
  int rc = make_geo(desc, &g);
  if (rc != LANCE_OK) return rc;
  Workspace w = make_workspace(g);
  out->Ho = g.Ho; out->Wo = g.Wo; out->tiles_h = g.th; out->tiles_w = g.tw; out->P = g.P;
  out->E = g.E; out->Cp = g.Cp; out->CB = g.CB; out->NB = g.NB;
  out->uq_bytes = (size_t)g.E * g.K * g.NB * code_row_bytes(g);
  out->u_range_bytes = (size_t)g.E * 2 * sizeof(float);
  out->u_rowsum_bytes = (size_t)g.E * g.K * sizeof(int32_t);
  out->vq_bytes = (size_t)g.E * g.P * g.NB * code_row_bytes(g);
  out->v_range_bytes = (size_t)g.E * 2 * sizeof(float);
  out->v_colsum_bytes = (size_t)g.E * g.P * sizeof(int32_t);
  out->acc_bytes = (size_t)g.E * g.K * g.P * sizeof(int32_t);
  out->y_bytes = (size_t)g.N * g.K * g.Ho * g.Wo * sizeof(float);
  out->input_workspace_bytes = w.input_bytes;
  out->conv_workspace_bytes = w.conv_bytes;
  return LANCE_OK;
}

size_t lance_code_offset(const lance_conv_desc* desc, int64_t rows, int32_t e, int64_t row,
                         int32_t c) {
  Geo g;
  if (make_geo(desc, &g) != LANCE_OK) return (size_t)-1;
  if (rows <= 0 || e < 0 || e >= g.E || row < 0 || row >= rows || c < 0 || c >= g.Cp)
    return (size_t)-1;
  int b = c / g.CB, r = c % g.CB;
  int pos = is_nhwc(g) ? r : 4 * (r % g.Q) + r / g.Q;
  const int rb = code_row_bytes(g);
  return (((size_t)e * g.NB + b) * (size_t)rows + (size_t)row) * rb + pos % rb;
}

int lance_code_shift(const lance_conv_desc* desc, int32_t c) {
  Geo g;
  if (make_geo(desc, &g) != LANCE_OK || c < 0 || c >= g.Cp) return -1;
  if (!is_packed(g)) return 0;
  const int r = c % g.CB;
  const int pos = is_nhwc(g) ? r : 4 * (r % g.Q) + r / g.Q;
  return pos >= g.CB / 2 ? 4 : 0;
}

static thread_local const char* g_detail = "";

static int hip_rc(hipError_t e) {
  if (e == hipSuccess) return LANCE_OK;
  g_detail = hipGetErrorString(e);
  return LANCE_ERR_HIP;
}

// The staged entry points address the int32 accumulators [E][K][P] with 32-bit byte offsets.
static bool acc_addressable(const Geo& g) {
  return (long long)g.E * g.K * g.P * 4 < 0xFFFFFFF0LL;
}

// Launch status is read with hipGetLastError(), which also reports errors left behind by
// earlier, unrelated runtime calls of this thread; drop those before the first launch.
static void clear_stale_error() { (void)hipGetLastError(); }

int lance_filter_transform_q8(const lance_conv_desc* desc, const float* w_dev, int8_t* uq_dev,
                              float* u_range_dev, int32_t* u_rowsum_dev, void* stream) {
  Geo g;
  int rc = make_geo(desc, &g);
  if (rc != LANCE_OK) return rc;
  if (!w_dev || !uq_dev || !u_range_dev || !u_rowsum_dev) return LANCE_ERR_INVALID_ARG;
  clear_stale_error();
  return hip_rc(launch_filter_transform(g, w_dev, uq_dev, u_range_dev, u_rowsum_dev,
                                        (hipStream_t)stream));
}

int lance_input_transform_q8(const lance_conv_desc* desc, const float* x_dev, int8_t* vq_dev,
                             float* v_range_dev, int32_t* v_colsum_dev, void* workspace_dev,
                             size_t workspace_bytes, void* stream) {
  Geo g;
  int rc = make_geo(desc, &g);
  if (rc != LANCE_OK) return rc;
  if (!x_dev || !vq_dev || !v_range_dev || !v_colsum_dev) return LANCE_ERR_INVALID_ARG;
  Workspace wl = make_workspace(g);
  if (!workspace_dev || workspace_bytes < wl.input_bytes || ((uintptr_t)workspace_dev & 255))
    return LANCE_ERR_WORKSPACE;
  clear_stale_error();
  return hip_rc(launch_input_transform(g, x_dev, vq_dev, v_range_dev, v_colsum_dev,
                                       (char*)workspace_dev, wl, (hipStream_t)stream));
}

int lance_winograd_gemm_i8(const lance_conv_desc* desc, const int8_t* uq_dev,
                           const int8_t* vq_dev, int32_t* acc_dev, void* stream) {
  Geo g;
  int rc = make_geo(desc, &g);
  if (rc != LANCE_OK) return rc;
  if (!uq_dev || !vq_dev || !acc_dev) return LANCE_ERR_INVALID_ARG;
  if (!acc_addressable(g)) return LANCE_ERR_UNSUPPORTED;
  clear_stale_error();
  return hip_rc(launch_gemm_i8(g, uq_dev, vq_dev, acc_dev, (hipStream_t)stream));
}

int lance_output_transform_dq(const lance_conv_desc* desc, const int32_t* acc_dev,
                              const float* u_range_dev, const int32_t* u_rowsum_dev,
                              const float* v_range_dev, const int32_t* v_colsum_dev,
                              float* y_dev, void* stream) {
  Geo g;
  int rc = make_geo(desc, &g);
  if (rc != LANCE_OK) return rc;
  if (!acc_dev || !u_range_dev || !u_rowsum_dev || !v_range_dev || !v_colsum_dev || !y_dev)
    return LANCE_ERR_INVALID_ARG;
  if (!acc_addressable(g)) return LANCE_ERR_UNSUPPORTED;
  clear_stale_error();
  return hip_rc(launch_output_transform(g, acc_dev, u_range_dev, u_rowsum_dev, v_range_dev,
                                        v_colsum_dev, y_dev, (hipStream_t)stream));
}

// Everything the fused call checks before its first HIP call.
static int conv_check_args(const lance_conv_desc* desc, const float* x_dev, const int8_t* uq_dev,
                           const float* u_range_dev, const int32_t* u_rowsum_dev,
                           const float* v_range_dev, const float* y_dev, const void* workspace_dev,
                           size_t workspace_bytes, Geo* g, Workspace* wl) {
  const int rc = make_geo(desc, g);
  if (rc != LANCE_OK) return rc;
  if (!x_dev || !uq_dev || !u_range_dev || !u_rowsum_dev || !y_dev) return LANCE_ERR_INVALID_ARG;
  if ((g->flags & LANCE_INPUT_RANGE_STATIC) && !v_range_dev) return LANCE_ERR_INVALID_ARG;
  *wl = make_workspace(*g);
  if (!workspace_dev || workspace_bytes < wl->conv_bytes || ((uintptr_t)workspace_dev & 255))
    return LANCE_ERR_WORKSPACE;
  return LANCE_OK;
}

// ev: nullptr, or LANCE_PROFILE_KERNELS + 1 created events that are recorded between the kernels
// (nothing waits for them here); *plan_out tells which of them were recorded.
// (kPlanThreeKernels: range pass, reduction kernel, one kernel for everything else)
enum ConvPlan { kPlanGeneral = 0, kPlanTwoKernels = 1, kPlanThreeKernels = 2 };

// Layers with one 64-channel block (m = 2) run as two kernels: the range pass, then one kernel
// that reduces the ranges, quantizes, multiplies and transforms back (V's codes stay on chip).
// Layers with two blocks (m = 2) take the same two-kernel form (128 KB of codes in LDS) unless
// the descriptor asks for the general plan's wide tiles.  Layers of at most 16 channels (m = 2)
// and F(4x4,3x3) layers of at most 128 channels: range pass, reduction kernel, one kernel for the
// rest (the reduction kernel drops out where the last kernel can reduce for itself).
struct PlanChoice {
  bool fuse_q1, fuse_q2, fuse_s, fuse_m4;
  ConvPlan plan() const {
    return (fuse_q1 || fuse_q2) ? kPlanTwoKernels
                                : ((fuse_s || fuse_m4) ? kPlanThreeKernels : kPlanGeneral);
  }
};

static PlanChoice choose_plan(const Geo& g, const float* x_dev) {
  PlanChoice c{};
  if (is_packed(g)) return c;  // packed codes: the general plan (quantize pass, product kernel)
  const bool x_ok = !is_nhwc(g) || (reinterpret_cast<uintptr_t>(x_dev) & 15) == 0;
  c.fuse_q1 = conv_fused_c64_applicable(g) && x_ok;
  c.fuse_q2 = !c.fuse_q1 && conv_fused_c128_applicable(g) && !(g.flags & LANCE_PLAN_WIDE_TILES) && x_ok;
  c.fuse_s = !c.fuse_q1 && !c.fuse_q2 && conv_fused_c16_applicable(g);
  c.fuse_m4 = !c.fuse_q1 && !c.fuse_q2 && !c.fuse_s && conv_fused_m4_applicable(g);
  return c;
}

// Bytes of the workspace carve-up that the chosen plan really touches: the plans that keep V's
// codes on chip use nothing from the column sums on.
static size_t plan_scratch_bytes(const PlanChoice& c, const Workspace& wl) {
  return c.plan() == kPlanGeneral ? wl.conv_bytes : wl.off_colsum;
}

// The launches of the fused call on validated arguments.
static int conv_launch(const Geo& g, const Workspace& wl, const float* x_dev, const int8_t* uq_dev,
                       const float* u_range_dev, const int32_t* u_rowsum_dev, float* v_range_dev,
                       float* y_dev, char* ws, void* stream, hipEvent_t* ev, int* plan_out) {
  hipStream_t s = (hipStream_t)stream;
  float* v_range = v_range_dev ? v_range_dev : (float*)(ws + wl.off_vrange);
  int8_t* vq = (int8_t*)(ws + wl.off_vq);
  int32_t* colsum = (int32_t*)(ws + wl.off_colsum);
  float* dq = (float*)(ws + wl.off_dq);
  float* rk = (float*)(ws + wl.off_rk);
  clear_stale_error();
  hipError_t e = hipSuccess;
  double* dqd = (double*)(ws + wl.off_dqd);
  const DqOut dqo{u_range_dev, u_rowsum_dev, dq, rk, dqd, g.K, g.C, gemm_fused_wants_rk(g) ? 1 : 0,
                  g.bits_w, code_bias(g)};
  const PlanChoice pc = choose_plan(g, x_dev);
  const bool fuse_q1 = pc.fuse_q1, fuse_q = pc.fuse_q1 || pc.fuse_q2, fuse_s = pc.fuse_s;
  if (plan_out) *plan_out = pc.plan();
  if (fuse_q) {
    const bool is_static = (g.flags & LANCE_INPUT_RANGE_STATIC) != 0;
    float* partial = (float*)(ws + wl.off_partial);
    int groups = 0;
    if (e == hipSuccess && ev) e = hipEventRecord(ev[0], s);
    note_slot(0);
    if (e == hipSuccess && !is_static) e = launch_input_range(g, x_dev, partial, colsum, 0, &groups, s);
    if (e == hipSuccess && ev) e = hipEventRecord(ev[1], s);
    note_slot(3);
    if (e == hipSuccess)
      e = fuse_q1 ? launch_conv_fused_c64(g, x_dev, uq_dev, u_range_dev, u_rowsum_dev, partial,
                                          groups, v_range, y_dev, s)
                  : launch_conv_fused_c128(g, x_dev, uq_dev, u_range_dev, u_rowsum_dev, partial,
                                           groups, v_range, y_dev, s);
  } else if (fuse_s) {
    // Layers with at most 16 channels (m = 2): range pass, reduction kernel, then one kernel
    // that quantizes, multiplies and transforms back.
    const bool is_static = (g.flags & LANCE_INPUT_RANGE_STATIC) != 0;
    float* partial = (float*)(ws + wl.off_partial);
    float* qparams = (float*)(ws + wl.off_qparams);
    int groups = 0;
    if (e == hipSuccess && ev) e = hipEventRecord(ev[0], s);
    note_slot(0);
    if (e == hipSuccess && !is_static) e = launch_input_range(g, x_dev, partial, colsum, 0, &groups, s);
    if (e == hipSuccess && ev) e = hipEventRecord(ev[1], s);
    note_slot(1);
    // (with caller-supplied ranges the product kernel needs no reduction kernel before it)
    if (e == hipSuccess && !is_static)
      e = launch_range_finalize(partial, groups, g.E, (g.flags & LANCE_RANGE_PER_TENSOR) ? 1 : 0,
                                0, g.bits, v_range, qparams, &dqo, s);
    if (e == hipSuccess && ev) e = hipEventRecord(ev[2], s);
    note_slot(3);
    if (e == hipSuccess)
      e = launch_conv_fused_c16(g, x_dev, uq_dev, qparams, dq, dqd, u_rowsum_dev, y_dev,
                                is_static ? v_range : nullptr, u_range_dev, s);
  } else if (pc.fuse_m4) {
    // F(4x4,3x3) layers of at most 128 channels: range pass, reduction kernel (unless the last
    // kernel reduces for itself: caller-supplied ranges, or few records), then one kernel that
    // quantizes, multiplies and transforms back.
    const bool is_static = (g.flags & LANCE_INPUT_RANGE_STATIC) != 0;
    float* partial = (float*)(ws + wl.off_partial);
    float* qparams = (float*)(ws + wl.off_qparams);
    int groups = 0;
    if (e == hipSuccess && ev) e = hipEventRecord(ev[0], s);
    note_slot(0);
    if (e == hipSuccess && !is_static) e = launch_input_range(g, x_dev, partial, colsum, 0, &groups, s);
    if (e == hipSuccess && ev) e = hipEventRecord(ev[1], s);
    note_slot(1);
    const bool merge = is_static || conv_fused_m4_can_merge(g, groups);
    DqOut dqo4 = dqo;
    dqo4.want_rk = 0;  // the kernel forms the filter-side terms from dqd and the row sums
    if (e == hipSuccess && !merge)
      e = launch_range_finalize(partial, groups, g.E, (g.flags & LANCE_RANGE_PER_TENSOR) ? 1 : 0,
                                0, g.bits, v_range, qparams, &dqo4, s);
    if (e == hipSuccess && ev) e = hipEventRecord(ev[2], s);
    note_slot(3);
    if (e == hipSuccess)
      e = launch_conv_fused_m4(g, x_dev, uq_dev, u_range_dev, u_rowsum_dev, partial, groups,
                               merge ? 1 : 0, qparams, dq, dqd, v_range, y_dev, s);
  } else {
    if (e == hipSuccess)
      e = launch_input_transform(g, x_dev, vq, v_range, colsum, ws, wl, s, &dqo, ev);
    if (e == hipSuccess)
      e = launch_gemm_fused(g, uq_dev, vq, colsum, dq, rk, dqd, u_rowsum_dev, y_dev, s);
  }
  if (e == hipSuccess && ev) e = hipEventRecord(ev[LANCE_PROFILE_KERNELS], s);
  return hip_rc(e);
}

static int conv_impl(const lance_conv_desc* desc, const float* x_dev, const int8_t* uq_dev,
                     const float* u_range_dev, const int32_t* u_rowsum_dev, float* v_range_dev,
                     float* y_dev, void* workspace_dev, size_t workspace_bytes, void* stream,
                     hipEvent_t* ev, int* plan_out) {
  Geo g;
  Workspace wl;
  int rc = conv_check_args(desc, x_dev, uq_dev, u_range_dev, u_rowsum_dev, v_range_dev, y_dev,
                           workspace_dev, workspace_bytes, &g, &wl);
  if (rc != LANCE_OK) return rc;
  return conv_launch(g, wl, x_dev, uq_dev, u_range_dev, u_rowsum_dev, v_range_dev, y_dev,
                     (char*)workspace_dev, stream, ev, plan_out);
}

int lance_conv3x3_winograd_q8(const lance_conv_desc* desc, const float* x_dev,
                              const int8_t* uq_dev, const float* u_range_dev,
                              const int32_t* u_rowsum_dev, float* v_range_dev, float* y_dev,
                              void* workspace_dev, size_t workspace_bytes, void* stream) {
  return conv_impl(desc, x_dev, uq_dev, u_range_dev, u_rowsum_dev, v_range_dev, y_dev,
                   workspace_dev, workspace_bytes, stream, nullptr, nullptr);
}

// ---- the fused call for callers that cannot allocate ------------------------------------------
// Scratch memory of lance_conv3x3_winograd_q8_noalloc: one array per GPU, held by every device
// the library is loaded on until the process ends.  In host code `noalloc_scratch` is only a
// handle for hipGetSymbolAddress; the device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char noalloc_scratch[LANCE_NOALLOC_SCRATCH_BYTES];

static hipError_t noalloc_scratch_ptr(char** out) {
  constexpr int kMaxDevices = 64;
  static std::atomic<char*> ptr_of_device[kMaxDevices];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  char* p = ptr_of_device[dev].load(std::memory_order_acquire);
  if (!p) {
    // each device has its own copy of the array at its own address; the current device is `dev`
    void* sym = nullptr;
    e = hipGetSymbolAddress(&sym, HIP_SYMBOL(noalloc_scratch));
    if (e != hipSuccess) return e;
    if (!sym || (reinterpret_cast<uintptr_t>(sym) & 255)) return hipErrorInvalidSymbol;
    p = static_cast<char*>(sym);
    ptr_of_device[dev].store(p, std::memory_order_release);  // racing callers store the same value
  }
  *out = p;
  return hipSuccess;
}

int lance_conv3x3_winograd_q8_noalloc(const lance_conv_desc* desc, const float* x_dev,
                                      const int8_t* uq_dev, const float* u_range_dev,
                                      const int32_t* u_rowsum_dev, float* v_range_dev,
                                      float* y_dev, void* stream) {
  Geo g;
  const int rc = make_geo(desc, &g);
  if (rc != LANCE_OK) return rc;
  if (!x_dev || !uq_dev || !u_range_dev || !u_rowsum_dev || !y_dev) return LANCE_ERR_INVALID_ARG;
  if ((g.flags & LANCE_INPUT_RANGE_STATIC) && !v_range_dev) return LANCE_ERR_INVALID_ARG;
  const Workspace wl = make_workspace(g);
  if (plan_scratch_bytes(choose_plan(g, x_dev), wl) > (size_t)LANCE_NOALLOC_SCRATCH_BYTES) {
    g_detail = "layer needs more scratch memory than LANCE_NOALLOC_SCRATCH_BYTES";
    return LANCE_ERR_WORKSPACE;
  }
  char* ws = nullptr;
  const hipError_t e = noalloc_scratch_ptr(&ws);
  if (e != hipSuccess) return hip_rc(e);
  return conv_launch(g, wl, x_dev, uq_dev, u_range_dev, u_rowsum_dev, v_range_dev, y_dev, ws,
                     stream, nullptr, nullptr);
}

// Names of the kernels the calling thread's last timing-twin call launched, by slot.
static thread_local KernelNotes g_profile_notes = {{nullptr, nullptr, nullptr, nullptr}, -1};

const char* lance_profile_kernel_name(int slot) {
  if (slot < 0 || slot >= LANCE_PROFILE_KERNELS || !g_profile_notes.name[slot]) return "";
  return g_profile_notes.name[slot];
}

static int profile_impl(const lance_conv_desc* desc, const float* const* x_devs,
                        float* const* y_devs, int pairs, const int8_t* uq_dev,
                        const float* u_range_dev, const int32_t* u_rowsum_dev, float* v_range_dev,
                        void* workspace_dev, size_t workspace_bytes, void* stream, int repeats,
                        float* kernel_ms_host) {
  constexpr int kEv = LANCE_PROFILE_KERNELS + 1;
  if (!kernel_ms_host || repeats < 1 || repeats > LANCE_PROFILE_MAX_REPEATS || !x_devs || !y_devs ||
      pairs < 1 || pairs > LANCE_PROFILE_MAX_REPEATS)
    return LANCE_ERR_INVALID_ARG;
  for (int i = 0; i < pairs; i++) {  // argument errors are reported before the first HIP call
    Geo g;
    Workspace wl;
    const int rc = conv_check_args(desc, x_devs[i], uq_dev, u_range_dev, u_rowsum_dev, v_range_dev,
                                   y_devs[i], workspace_dev, workspace_bytes, &g, &wl);
    if (rc != LANCE_OK) return rc;
  }
  hipEvent_t* ev = (hipEvent_t*)calloc((size_t)repeats * kEv, sizeof(hipEvent_t));
  if (!ev) return LANCE_ERR_INVALID_ARG;
  hipError_t e = hipSuccess;
  int made = 0;
  for (; made < repeats * kEv && e == hipSuccess; made++) e = hipEventCreate(&ev[made]);
  if (e != hipSuccess) made--;
  int rc = hip_rc(e), plan = kPlanGeneral, done = 0;
  g_profile_notes = KernelNotes{{nullptr, nullptr, nullptr, nullptr}, -1};
  g_kernel_notes = &g_profile_notes;
  for (; done < repeats && rc == LANCE_OK; done++)
    rc = conv_impl(desc, x_devs[done % pairs], uq_dev, u_range_dev, u_rowsum_dev, v_range_dev,
                   y_devs[done % pairs], workspace_dev, workspace_bytes, stream,
                   ev + (size_t)done * kEv, &plan);
  g_kernel_notes = nullptr;
  if (rc == LANCE_OK) rc = hip_rc(hipEventSynchronize(ev[(size_t)repeats * kEv - 1]));
  if (rc == LANCE_OK) {
    // recorded events per plan: general 0..4; two kernels 0, 1, 4; small channels 0, 1, 2, 4
    double sum[LANCE_PROFILE_KERNELS] = {0.0, 0.0, 0.0, 0.0};
    for (int r = 0; r < repeats && e == hipSuccess; r++) {
      hipEvent_t* v = ev + (size_t)r * kEv;
      const int from[LANCE_PROFILE_KERNELS] = {0, 1, 2, plan == kPlanTwoKernels ? 1 : (plan == kPlanThreeKernels ? 2 : 3)};
      const int to[LANCE_PROFILE_KERNELS] = {1, 2, 3, 4};
      for (int i = 0; i < LANCE_PROFILE_KERNELS && e == hipSuccess; i++) {
        const bool skipped = (plan == kPlanTwoKernels && (i == 1 || i == 2)) ||
                             (plan == kPlanThreeKernels && i == 2);
        if (skipped) continue;
        float ms = 0.0f;
        e = hipEventElapsedTime(&ms, v[from[i]], v[to[i]]);
        sum[i] += ms;
      }
    }
    rc = hip_rc(e);
    for (int i = 0; i < LANCE_PROFILE_KERNELS; i++) kernel_ms_host[i] = (float)(sum[i] / repeats);
  } else if (done > 0) {
    (void)hipStreamSynchronize((hipStream_t)stream);  // events in flight must not be destroyed
  }
  for (int i = 0; i < made; i++) (void)hipEventDestroy(ev[i]);
  free(ev);
  return rc;
}

int lance_conv3x3_winograd_q8_profile(const lance_conv_desc* desc, const float* x_dev,
                                      const int8_t* uq_dev, const float* u_range_dev,
                                      const int32_t* u_rowsum_dev, float* v_range_dev,
                                      float* y_dev, void* workspace_dev, size_t workspace_bytes,
                                      void* stream, int repeats, float* kernel_ms_host) {
  return profile_impl(desc, &x_dev, &y_dev, 1, uq_dev, u_range_dev, u_rowsum_dev, v_range_dev,
                      workspace_dev, workspace_bytes, stream, repeats, kernel_ms_host);
}

int lance_conv3x3_winograd_q8_profile_rotating(const lance_conv_desc* desc,
                                               const float* const* x_devs_host,
                                               float* const* y_devs_host, int pairs,
                                               const int8_t* uq_dev, const float* u_range_dev,
                                               const int32_t* u_rowsum_dev, float* v_range_dev,
                                               void* workspace_dev, size_t workspace_bytes,
                                               void* stream, int repeats, float* kernel_ms_host) {
  return profile_impl(desc, x_devs_host, y_devs_host, pairs, uq_dev, u_range_dev, u_rowsum_dev,
                      v_range_dev, workspace_dev, workspace_bytes, stream, repeats, kernel_ms_host);
}

int lance_direct_conv3x3_f32(const lance_conv_desc* desc, const float* x_dev,
                             const float* w_dev, float* y_dev, void* stream) {
  lance_conv_desc d2;
  if (!desc) return LANCE_ERR_INVALID_ARG;
  d2 = *desc;
  d2.m = 2; d2.bits = 8;
  d2.flags = desc->flags & LANCE_LAYOUT_NHWC;  // only N,C,H,W,K,pad and the layout matter here
  Geo g;
  int rc = make_geo(&d2, &g);
  if (rc != LANCE_OK) return rc;
  if (!x_dev || !w_dev || !y_dev) return LANCE_ERR_INVALID_ARG;
  clear_stale_error();
  return hip_rc(launch_direct_conv(g, x_dev, w_dev, y_dev, (hipStream_t)stream));
}

int lance_alg1_literal_f32(const lance_conv_desc* desc, const float* x_dev, const float* w_dev,
                           float* y_dev, void* stream) {
  Geo g;
  int rc = make_geo(desc, &g);
  if (rc != LANCE_OK) return rc;
  // the ranges are those of the single matrices: the range flags have no meaning here
  if (g.flags & (LANCE_RANGE_PER_TENSOR | LANCE_INPUT_RANGE_STATIC | LANCE_PLAN_WIDE_TILES |
                 LANCE_CODES_PACKED4))
    return LANCE_ERR_UNSUPPORTED;
  if (!x_dev || !w_dev || !y_dev) return LANCE_ERR_INVALID_ARG;
  clear_stale_error();
  return hip_rc(launch_alg1_literal(g, x_dev, w_dev, y_dev, (hipStream_t)stream));
}

int lance_conv3x3_winograd_wq_f32(const lance_conv_desc* desc, const float* x_dev,
                                  const int8_t* uq_dev, const float* u_range_dev, float* y_dev,
                                  void* stream) {
  Geo g;
  int rc = make_geo(desc, &g);
  if (rc != LANCE_OK) return rc;
  // the input is not quantized: input ranges and the plans of the integer path mean nothing here
  if (g.flags & (LANCE_INPUT_RANGE_STATIC | LANCE_PLAN_WIDE_TILES | LANCE_CODES_PACKED4))
    return LANCE_ERR_UNSUPPORTED;
  if (!x_dev || !uq_dev || !u_range_dev || !y_dev) return LANCE_ERR_INVALID_ARG;
  clear_stale_error();
  return hip_rc(launch_weight_only(g, x_dev, uq_dev, u_range_dev, y_dev, (hipStream_t)stream));
}

const char* lance_status_string(int status) {
  switch (status) {
    case LANCE_OK: return "ok";
    case LANCE_ERR_INVALID_ARG: return "invalid argument";
    case LANCE_ERR_UNSUPPORTED: return "unsupported configuration";
    case LANCE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case LANCE_ERR_HIP: return "HIP call or kernel launch failed";
    default: return "unknown status";
  }
}

const char* lance_last_error_detail(void) { return g_detail; }

int lance_version(void) { return 100; }

}  // extern "C"
