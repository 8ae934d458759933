/*
 * lance.h -- C ABI of liblance: quantized Winograd 3x3 convolution F(m x m, 3 x 3), m in {2,4},
 * with linear quantization inside the Winograd domain (LANCE, arXiv 2003.08646), for AMD
 * MI355X (gfx950).  C99; no C++ or framework types cross this boundary.
 *
 * What is computed (paper, Sec. 3.2, Eq. 9 and Algorithm 1, with the Hadamard product done as
 * one integer GEMM per Winograd-domain position, Sec. 3.3):
 *
 *   U[e,k,c] = (G g_{k,c} G^T)[e]           filter transform          e = i*(m+2)+j, E=(m+2)^2
 *   V[e,p,c] = (B^T d_{p,c} B)[e]           input-patch transform     p = (n*th+ty)*tw+tx
 *   qu, qv   = Q(U), Q(V)                   Eq. 7, one (min,max) per position e
 *   ACC[e,k,p] = sum_c qu[e,k,c]*qv[e,p,c]  int8 x int8 -> int32, exact
 *   M = Q'(ACC)                             Eq. 8 applied to both operands (see below)
 *   Y tile = A^T M A                        output transform, tiles merged and cropped
 *
 * Conventions common to every call
 *   - Pointers named *_dev are DEVICE pointers owned by the caller (any allocator).  The
 *     library allocates no device memory and frees none.  The only state it keeps between calls:
 *     per device, the number of resident workgroups of a few kernels (a constant of kernel and
 *     chip, asked of the runtime on first use), and per thread the text of the last HIP error.
 *     Calls are thread-safe as long as they do not share output or workspace buffers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it; no call synchronizes.  Outputs are valid once the stream has drained.
 *   - Return value: LANCE_OK or a negative lance_status.  Descriptor validation happens
 *     before the first HIP call, so argument errors are reported on a machine with no GPU.
 *     Nothing is thrown or aborted across the ABI.
 *   - NaN or infinite inputs are not supported (ranges and codes are then unspecified).
 *   - Size limits (LANCE_ERR_UNSUPPORTED beyond them; kernel offsets are 32-bit): each of x, y,
 *     uq and vq below 4 GiB (for the staged calls also acc), N and K at most 65535, C at most
 *     2^17, and the pixels of any 64 consecutive tiles within 2 GiB of their first image.
 *
 * Tensors and layouts
 *   x       fp32 [N][C][H][W]                        (NCHW)
 *   w       fp32 [K][C][3][3]                        (KCRS), stride 1, dilation 1
 *   y       fp32 [N][K][Ho][Wo], Ho = H+2*pad-2, Wo = W+2*pad-2
 *   (with LANCE_LAYOUT_NHWC: x fp32 [N][H][W][C], y fp32 [N][Ho][Wo][K])
 *   Tiles: th = ceil(Ho/m), tw = ceil(Wo/m), P = N*th*tw.  Tile (n,ty,tx) reads the
 *   (m+2)x(m+2) window whose top-left input pixel is (ty*m-pad, tx*m-pad); pixels outside
 *   the image read as 0 (zero padding and ragged last tiles alike).
 *
 *   Codes are signed: stored code = Eq. 7's code - 2^(bits-1), in [-2^(bits-1), 2^(bits-1)-1],
 *   one per int8.  The reduction axis is padded to Cp and cut into blocks of CB channels:
 *       Cp = 16 if C <= 16, else C rounded up to a multiple of 64
 *       CB = min(Cp, 64),  NB = Cp / CB,  Q = CB / 4
 *   uq      int8 [E][NB][K][CB]
 *   vq      int8 [E][NB][P][CB]
 *   Within a block, channel c = b*CB + r is stored at byte  4*(r mod Q) + r/Q  (the same
 *   permutation in uq and vq, so the product over the block is unchanged); with
 *   LANCE_LAYOUT_NHWC at byte r (the channels of a pixel are contiguous in X already).  Channels
 *   c >= C hold code 0.  lance_code_offset() returns the byte offset of (e,row,c).
 *   (A plain [E][rows][Cp] layout would do for the method; the blocks make a 32-row matrix-core
 *   fragment one contiguous 2 KB piece and the permutation lets a lane of the quantize pass own
 *   one aligned dword of four channels.  Tests go through lance_code_offset().)
 *   With LANCE_CODES_PACKED4 a block row is 32 bytes: uq int8 [E][NB][K][32], vq
 *   int8 [E][NB][P][32].  The code whose unpacked position is byte q of its 64-byte row sits in
 *   byte q mod 32, in the low four bits if q < 32 and in the high four bits otherwise, as the
 *   unsigned value  stored code + 8  (so a padding channel reads 8).  lance_code_offset() gives
 *   the byte, lance_code_shift() the bit position (0 or 4).
 *   u_range, v_range   fp32 [E][2] = {min, max} of U[e,.,.] resp. V[e,.,.] over real channels
 *   u_rowsum int32 [E][K] = sum_{c<C} qu[e,k,c];  v_colsum int32 [E][P] = sum_{c<C} qv[e,p,c]
 *   acc     int32 [E][K][P]
 *
 * Quantizer (Eq. 7; choices the paper leaves open are marked *):
 *   L = 2^bits-1;  inv = (float)(L/((double)max-(double)min));  scale = (float)(((double)max-min)/L)
 *   max == min, or inv not finite: inv = 0 (every code is 0)
 *   code = clamp(round_half_even*((x - min)*inv), 0, L)      -- two binary32 operations
 *   * Eq. 7's T (the matrix a value belongs to) is read as the GEMM operand of position e: one
 *     range per e.  LANCE_RANGE_PER_TENSOR uses one range for all e.
 * De-quantizer (Eq. 8 on both operands, products expanded), with h = 2^(bits-1),
 *   ou = min_u + scale_u*h, ov = min_v + scale_v*h:
 *   M[e,k,p] = su*sv*ACC + su*ov*u_rowsum[e,k] + sv*ou*v_colsum[e,p] + C*ou*ov
 */
#ifndef LANCE_H
#define LANCE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum lance_status {
  LANCE_OK = 0,
  LANCE_ERR_INVALID_ARG = -1, /* null pointer, non-positive dimension, empty output        */
  LANCE_ERR_UNSUPPORTED = -2, /* m not in {2,4}, bits not in [2,8], unknown flag, too large */
  LANCE_ERR_WORKSPACE = -3,   /* workspace missing or smaller than lance_query_sizes says   */
  LANCE_ERR_HIP = -4          /* a HIP call or kernel launch failed                         */
} lance_status;

enum {
  LANCE_RANGE_PER_POSITION = 0u,  /* default: one (min,max) per Winograd-domain position   */
  LANCE_RANGE_PER_TENSOR = 1u,    /* one (min,max) for the whole transformed tensor        */
  LANCE_INPUT_RANGE_STATIC = 2u,  /* v_range is given by the caller (calibrated ranges);
                                     values outside it are clamped to the end codes        */
  LANCE_PLAN_WIDE_TILES = 4u,     /* tuning: the fused convolution of F(2x2,3x3) layers with
                                     C > 64 multiplies with 128 x 64 workgroup tiles whatever
                                     the layer size (by default only large layers do); the
                                     codes are the same, Y may differ in fp32 rounding order */
  LANCE_LAYOUT_NHWC = 8u,         /* X is [N][H][W][C] and Y is [N][Ho][Wo][K] (the layout of
                                     Sec. 3.3); W stays [K][C][3][3]; codes, sums and ranges are
                                     those of the NCHW call on the transposed tensors, with the
                                     channels of a code block in their natural order           */
  LANCE_CODES_PACKED4 = 16u       /* codes of at most 4 bits (Sec. 4's 4-4 rows) stored two to a
                                     byte: uq and vq take half the bytes (layout below).  Needs
                                     bits <= 4, filter bits <= 4 and C > 16, else
                                     LANCE_ERR_UNSUPPORTED.  Same codes, sums and ranges; Y may
                                     differ from the unpacked call in fp32 rounding.  Served
                                     by every entry point that takes or gives codes, in both
                                     activation layouts and for both tile sizes; the staged
                                     lance_winograd_gemm_i8 gives the exact int32 products of
                                     the codes as with unpacked rows.                          */
};
/* Filter codes of another width than the input codes (Sec. 4 evaluates weights and inputs at
 * different widths): OR LANCE_FILTER_BITS(bw), bw in [2,8], into flags.  Absent (field 0): the
 * filters use `bits` too.  Every entry point of one layer must get the same descriptor. */
#define LANCE_FILTER_BITS_SHIFT 8
#define LANCE_FILTER_BITS_MASK 0x00000F00u
#define LANCE_FILTER_BITS(bw) ((uint32_t)(bw) << LANCE_FILTER_BITS_SHIFT) /* a width outside
                                     [2,8] lands outside the field or on a bad value: rejected */

typedef struct lance_conv_desc {
  int32_t N, C, H, W; /* input dimensions (NCHW order unless LANCE_LAYOUT_NHWC) */
  int32_t K;          /* number of 3x3 filters                        */
  int32_t pad;        /* symmetric zero padding >= 0                  */
  int32_t m;          /* output tile edge: 2 or 4                     */
  int32_t bits;       /* code width b in [2,8] (always stored in int8): of the input codes,
                         and of the filter codes unless flags carries LANCE_FILTER_BITS */
  uint32_t flags;     /* LANCE_RANGE_* | LANCE_INPUT_RANGE_STATIC | LANCE_PLAN_* |
                         LANCE_LAYOUT_NHWC | LANCE_CODES_PACKED4 | LANCE_FILTER_BITS(bw) */
} lance_conv_desc;

typedef struct lance_sizes {
  int32_t Ho, Wo, tiles_h, tiles_w, P, E, Cp, CB, NB;
  size_t uq_bytes, u_range_bytes, u_rowsum_bytes;
  size_t vq_bytes, v_range_bytes, v_colsum_bytes;
  size_t acc_bytes, y_bytes;
  size_t input_workspace_bytes; /* for lance_input_transform_q8  */
  size_t conv_workspace_bytes;  /* for lance_conv3x3_winograd_q8 */
} lance_sizes;

/* Geometry and buffer sizes of a layer.  Host only; needs no GPU.  (Sec. 2.3: tiling.) */
int lance_query_sizes(const lance_conv_desc *desc, lance_sizes *out);

/* Byte offset of channel c of row `row` (k for uq, p for vq; `rows` = K resp. P) at
 * position e inside uq / vq.  Host only.  Returns (size_t)-1 on a bad argument. */
size_t lance_code_offset(const lance_conv_desc *desc, int64_t rows, int32_t e, int64_t row,
                         int32_t c);

/* Bit position (0 or 4) of channel c's code inside the byte lance_code_offset() names; 0 for
 * unpacked codes.  Host only.  Returns -1 on a bad argument. */
int lance_code_shift(const lance_conv_desc *desc, int32_t c);

/* Stage 1 -- Algorithm 1, u^ = Q(G g G^T) for every (k,c); Eq. 7.  Run once per set of
 * weights (Sec. 3.4: the filters are transformed and quantized off-line, a single time).
 *   in : w_dev fp32 [K][C][3][3]
 *   out: uq_dev, u_range_dev, u_rowsum_dev (layouts above; every byte of uq is written). */
int lance_filter_transform_q8(const lance_conv_desc *desc, const float *w_dev, int8_t *uq_dev,
                              float *u_range_dev, int32_t *u_rowsum_dev, void *stream);

/* Stage 2 -- Algorithm 1, D <- patches with padding, v^ = Q(B^T d B); Eq. 7.
 *   in : x_dev fp32 NCHW
 *   out: vq_dev, v_colsum_dev; v_range_dev is an output, or an INPUT when
 *        LANCE_INPUT_RANGE_STATIC is set.
 *   workspace_dev: >= input_workspace_bytes, 256-byte aligned; contents undefined after. */
int lance_input_transform_q8(const lance_conv_desc *desc, const float *x_dev, int8_t *vq_dev,
                             float *v_range_dev, int32_t *v_colsum_dev, void *workspace_dev,
                             size_t workspace_bytes, void *stream);

/* Stage 3 -- Algorithm 1, m^ = u^ .* v^ summed over channels, as E integer GEMMs (Sec. 3.3):
 *   acc[e][k][p] = sum_c uq[e,k,c] * vq[e,p,c], exact in int32 (|acc| <= C*2^14). */
int lance_winograd_gemm_i8(const lance_conv_desc *desc, const int8_t *uq_dev,
                           const int8_t *vq_dev, int32_t *acc_dev, void *stream);

/* Stage 4 -- Algorithm 1, m~ = Q'(m^) (Eq. 8), S = A^T m A, Y_{p,k} <- S (Eq. 9).
 * Arithmetic in binary32; the per-position constants are formed in binary64. */
int lance_output_transform_dq(const lance_conv_desc *desc, const int32_t *acc_dev,
                              const float *u_range_dev, const int32_t *u_rowsum_dev,
                              const float *v_range_dev, const int32_t *v_colsum_dev,
                              float *y_dev, void *stream);

/* Stages 2-4 in one call -- Eq. 9 as a whole, Y = LANCE(X, W) of Algorithm 1 with the
 * filters prepared by lance_filter_transform_q8.  The int32 accumulators stay on chip
 * (stage 3 and 4 are one kernel; with at most two 64-channel blocks so do the codes of V, for
 * m = 4 on NCHW tensors).  v_range_dev is an argument the method's statement does not have: with
 * LANCE_INPUT_RANGE_STATIC it supplies the calibrated ranges (Sec. 3.4's inference mode);
 * otherwise pass NULL, or a buffer of v_range_bytes to receive the ranges Eq. 7 found.
 *   workspace_dev: >= conv_workspace_bytes, 256-byte aligned. */
int lance_conv3x3_winograd_q8(const lance_conv_desc *desc, const float *x_dev,
                              const int8_t *uq_dev, const float *u_range_dev,
                              const int32_t *u_rowsum_dev, float *v_range_dev, float *y_dev,
                              void *workspace_dev, size_t workspace_bytes, void *stream);

/* lance_conv3x3_winograd_q8 for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments without the workspace, same kernels, same result bits.  Its
 * scratch memory is a fixed array of LANCE_NOALLOC_SCRATCH_BYTES inside the library's device
 * image, which every GPU the library runs on holds until the process ends; the call itself
 * allocates and frees nothing.
 *   - A layer whose plan needs more scratch than that returns LANCE_ERR_WORKSPACE before any
 *     HIP call (lance_last_error_detail() says why).  Needed: about 4 KB * (m+2)^2 for m = 2
 *     layers of at most 128 channels, else vq_bytes + v_colsum_bytes + the same
 *     (lance_query_sizes); every configuration of the paper's benchmark shapes at batch 16-128
 *     fits.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two threads) race.  Serialize them, or use lance_conv3x3_winograd_q8 with a
 *     workspace per stream.  Nothing in the array has to survive between calls, and every call
 *     clears what it needs cleared with its own kernels.
 *   - The first call on a device looks up the array's address there (hipGetSymbolAddress, no
 *     allocation); make that first call outside a graph capture. */
#define LANCE_NOALLOC_SCRATCH_BYTES (64u << 20)
int lance_conv3x3_winograd_q8_noalloc(const lance_conv_desc *desc, const float *x_dev,
                                      const int8_t *uq_dev, const float *u_range_dev,
                                      const int32_t *u_rowsum_dev, float *v_range_dev,
                                      float *y_dev, void *stream);

/* Diagnostic twin of lance_conv3x3_winograd_q8 for roofline accounting: `repeats` passes of
 * the same launches, enqueued back to back on the same stream with a HIP event recorded between
 * the kernels, one wait for the stream at the end (the GPU stays busy between the passes, as it
 * does in a timed loop of lance_conv3x3_winograd_q8).  Creates and destroys its events and
 * returns each kernel's duration, averaged over the passes, in milliseconds in
 * kernel_ms_host[LANCE_PROFILE_KERNELS] (HOST memory): [0] range pass over X, [1] range
 * reduction + quantizer/de-quantizer constants, [2] transform+quantize pass,
 * [3] GEMM+epilogue.  Layers with one 64-channel block and m = 2 run as two kernels (V's codes
 * never leave the chip): then [1] and [2] are exactly 0 and [3] covers range reduction,
 * transform+quantize, GEMM and epilogue.  Where the quantize pass reduces the range records
 * itself [1] is the time between two adjacent events.  A duration includes the launch gap in
 * front of its kernel.  repeats: 1 .. LANCE_PROFILE_MAX_REPEATS, else LANCE_ERR_INVALID_ARG.
 * (Times the kernels of Algorithm 1's steps; defines no operation of its own.) */
#define LANCE_PROFILE_KERNELS 4
#define LANCE_PROFILE_MAX_REPEATS 4096
int lance_conv3x3_winograd_q8_profile(const lance_conv_desc *desc, const float *x_dev,
                                      const int8_t *uq_dev, const float *u_range_dev,
                                      const int32_t *u_rowsum_dev, float *v_range_dev,
                                      float *y_dev, void *workspace_dev, size_t workspace_bytes,
                                      void *stream, int repeats, float *kernel_ms_host);

/* The same twin over `pairs` (input, output) buffer pairs, pass r using pair r % pairs: with a
 * total footprint beyond the last-level cache every pass reads its input from HBM, as a layer in
 * the middle of a network does.  x_devs_host / y_devs_host: HOST arrays of `pairs` device
 * pointers (1 <= pairs <= LANCE_PROFILE_MAX_REPEATS). */
int lance_conv3x3_winograd_q8_profile_rotating(const lance_conv_desc *desc,
                                               const float *const *x_devs_host,
                                               float *const *y_devs_host, int pairs,
                                               const int8_t *uq_dev, const float *u_range_dev,
                                               const int32_t *u_rowsum_dev, float *v_range_dev,
                                               void *workspace_dev, size_t workspace_bytes,
                                               void *stream, int repeats, float *kernel_ms_host);

/* Name (function name without template arguments) of the kernel that the calling thread's most
 * recent lance_conv3x3_winograd_q8_profile(_rotating) call launched in slot 0..LANCE_PROFILE_KERNELS-1, ""
 * for a slot that launched nothing.  Host only; lets a profile be matched with the slots.
 * (Like the twin itself: measurement support, defines no operation.) */
const char *lance_profile_kernel_name(int slot);

/* Full-precision comparator -- Eq. 1 evaluated directly in binary32 (the unquantized
 * convolution that the speedups of Sec. 4 are measured against).  Uses desc N,C,H,W,K,pad and the
 * LANCE_LAYOUT_NHWC flag only. */
int lance_direct_conv3x3_f32(const lance_conv_desc *desc, const float *x_dev,
                             const float *w_dev, float *y_dev, void *stream);

/* Accuracy ablation -- Algorithm 1 taken literally (loops k, p, c): the transformed filter and
 * the transformed patch of every channel are quantized with the range of their own
 * (m+2)x(m+2) matrix (Eq. 7 with T = that matrix), de-quantized (Eq. 8), multiplied, and the
 * products summed over the channels in binary32; then A^T m A (Eq. 9).  The forward pass of a
 * simulated quantization in the Winograd domain: no integer product, no matrix cores, slow.
 * x, w, y as for lance_conv3x3_winograd_q8 (w fp32 [K][C][3][3], not codes); uses N,C,H,W,K,
 * pad,m,bits, LANCE_FILTER_BITS and LANCE_LAYOUT_NHWC; the range and plan flags give
 * LANCE_ERR_UNSUPPORTED.  Needs no workspace. */
int lance_alg1_literal_f32(const lance_conv_desc *desc, const float *x_dev, const float *w_dev,
                           float *y_dev, void *stream);

/* Weight-only quantization -- the rows of Sec. 4 (Table 2) that quantize the weights and keep
 * full-precision inputs: Algorithm 1 with v^ replaced by the unquantized B^T d B,
 *   M[e,k,p] = sum_c Q'(u^[e,k,c]) * V[e,p,c] (Eq. 8 on the filter codes), Y tile = A^T M A,
 * evaluated in binary32 on the vector ALUs (no integer product exists for this mode).
 *   in : x as for lance_conv3x3_winograd_q8; uq_dev, u_range_dev from
 *        lance_filter_transform_q8 with the same descriptor (filter width = LANCE_FILTER_BITS,
 *        else bits; LANCE_RANGE_PER_TENSOR as there; LANCE_LAYOUT_NHWC honoured)
 *   out: y.  LANCE_INPUT_RANGE_STATIC and LANCE_PLAN_* give LANCE_ERR_UNSUPPORTED.  No workspace. */
int lance_conv3x3_winograd_wq_f32(const lance_conv_desc *desc, const float *x_dev,
                                  const int8_t *uq_dev, const float *u_range_dev, float *y_dev,
                                  void *stream);

const char *lance_status_string(int status);
/* Text of the HIP error behind the calling thread's most recent LANCE_ERR_HIP, or the reason of
 * its most recent LANCE_ERR_WORKSPACE from lance_conv3x3_winograd_q8_noalloc ("" if none).
 * The only per-thread state the library keeps; diagnostic only. */
const char *lance_last_error_detail(void);
int lance_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LANCE_H */
