/*
 * lance_oracle.c -- CPU oracle for the quantized Winograd 3x3 convolution of LANCE.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, loop-by-loop
 * statement of what the method computes, written from the paper so that a reader can
 * check it by eye.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.  It shares no code, header, table or constant with the HIP library.
 *
 * Two parts:
 *   Part 1  direct 3x3 correlation in fp64                       (Sec. 2.1, Eq. 1 / Eq. 2)
 *   Part 2  the quantized Winograd convolution, step by step      (Sec. 2.3 Eq. 4, Sec. 3.2
 *           Eq. 7, Eq. 8, Eq. 9, Algorithm 1; GEMM form of the Hadamard product, Sec. 3.3)
 *           plus two variants: Algorithm 1 with per-matrix ranges, and weight-only
 *           quantization (Sec. 4, Table 2's 4-32 row)
 *
 * Parity status of the choices the paper leaves open (see the function headers):
 *   - rounding tie rule of Eq. 7's `round` (half-to-even here)      : parity unpinned by the paper
 *   - granularity of T in Eq. 7 (one range per Winograd position)   : parity unpinned by the paper
 *   Everything else is pinned by tests that do not go through this file's own formulas
 *   (direct-convolution identity, values printed in Eq. 6, integer matmul, closed forms).
 *
 * Build: gcc -O2 -std=c99 -fopenmp -ffp-contract=off -fno-fast-math -shared -fPIC
 * Precision: the transforms, ranges, scales and codes are IEEE binary32 with one rounding
 * per written operation (no fused multiply-add), because the codes are integers decided by
 * floating point and both sides of a parity test must take that decision the same way.
 * The integer product is exact.  De-quantization and the output transform are fp64.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------------------ */
/* Transform matrices for F(m x m, 3 x 3)  (Sec. 2.3, Eq. 4).                            */
/* The paper prints only B^T for m = 2 (Eq. 6) and defers to Lavin & Gray for the rest; */
/* these are the standard matrices for interpolation points {0, 1, -1, inf} (m = 2) and */
/* {0, 1, -1, 2, -2, inf} (m = 4).  A test checks Eq. 4 == Eq. 1 with them.             */
/* ------------------------------------------------------------------------------------ */
static const double BT2[4][4] = {
    {1, 0, -1, 0}, {0, 1, 1, 0}, {0, -1, 1, 0}, {0, 1, 0, -1}};
static const double G2[4][3] = {
    {1, 0, 0}, {0.5, 0.5, 0.5}, {0.5, -0.5, 0.5}, {0, 0, 1}};
static const double AT2[2][4] = {{1, 1, 1, 0}, {0, 1, -1, -1}};

static const double BT4[6][6] = {
    {4, 0, -5, 0, 1, 0},  {0, -4, -4, 1, 1, 0}, {0, 4, -4, -1, 1, 0},
    {0, -2, -1, 2, 1, 0}, {0, 2, -1, -2, 1, 0}, {0, 4, 0, -5, 0, 1}};
static const double G4[6][3] = {
    {1.0 / 4, 0, 0},
    {-1.0 / 6, -1.0 / 6, -1.0 / 6},
    {-1.0 / 6, 1.0 / 6, -1.0 / 6},
    {1.0 / 24, 1.0 / 12, 1.0 / 6},
    {1.0 / 24, -1.0 / 12, 1.0 / 6},
    {0, 0, 1}};
static const double AT4[4][6] = {
    {1, 1, 1, 1, 1, 0}, {0, 1, -1, 2, -2, 0}, {0, 1, 1, 4, 4, 0}, {0, 1, -1, 8, -8, 1}};

static double bt_at(int m, int i, int j) { return m == 2 ? BT2[i][j] : BT4[i][j]; }
static double g_at(int m, int i, int j) { return m == 2 ? G2[i][j] : G4[i][j]; }
static double at_at(int m, int i, int j) { return m == 2 ? AT2[i][j] : AT4[i][j]; }

/* Copies the matrices out so a test can check the values the paper prints (Eq. 6). */
void lance_oracle_matrices(int m, double *bt /*a*a*/, double *g /*a*3*/, double *at /*m*a*/) {
  int a = m + 2;
  for (int i = 0; i < a; i++)
    for (int j = 0; j < a; j++) bt[i * a + j] = bt_at(m, i, j);
  for (int i = 0; i < a; i++)
    for (int j = 0; j < 3; j++) g[i * 3 + j] = g_at(m, i, j);
  for (int i = 0; i < m; i++)
    for (int j = 0; j < a; j++) at[i * a + j] = at_at(m, i, j);
}

/* Geometry shared by every step: output size, tile counts (Sec. 2.3: the image is cut   */
/* into overlapping (m+2)x(m+2) patches, one per m x m output patch; stride 1).          */
static int out_dim(int in, int pad) { return in + 2 * pad - 2; }
static int n_tiles(int out, int m) { return (out + m - 1) / m; }

/* Zero-padded read of X[n][c][y][x] (the paper's "patches ... with padding"). */
static float x_at(const float *X, int C, int H, int W, int n, int c, int y, int x) {
  if (y < 0 || y >= H || x < 0 || x >= W) return 0.0f;
  return X[(((size_t)n * C + c) * H + y) * W + x];
}

/* ==================================================================================== */
/* Part 1: direct correlation, Eq. 1 (stride 1, symmetric zero padding), fp64.          */
/*   Y[n,k,i,j] = sum_c sum_r sum_s X[n,c,i+r-pad,j+s-pad] * W[k,c,r,s]                 */
/* ==================================================================================== */
void lance_oracle_direct_conv_f64(const float *X, const float *Wt, double *Y, int N, int C,
                                  int H, int W, int K, int pad) {
  int Ho = out_dim(H, pad), Wo = out_dim(W, pad);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; n++)
    for (int k = 0; k < K; k++)
      for (int i = 0; i < Ho; i++)
        for (int j = 0; j < Wo; j++) {
          double acc = 0.0;
          for (int c = 0; c < C; c++)
            for (int r = 0; r < 3; r++)
              for (int s = 0; s < 3; s++)
                acc += (double)x_at(X, C, H, W, n, c, i + r - pad, j + s - pad) *
                       (double)Wt[(((size_t)k * C + c) * 3 + r) * 3 + s];
          Y[(((size_t)n * K + k) * Ho + i) * Wo + j] = acc;
        }
}

/* ==================================================================================== */
/* Unquantized Winograd convolution, Eq. 4, in fp64 by plain matrix products.           */
/*   S = A^T [ (G g G^T) .* (B^T d B) ] A, summed over channels before A^T . A          */
/* Exists so a test can check the matrices, the tiling, the padding, the merge and the  */
/* crop against Part 1.                                                                  */
/* ==================================================================================== */
void lance_oracle_winograd_conv_f64(const float *X, const float *Wt, double *Y, int N, int C,
                                    int H, int W, int K, int pad, int m) {
  int a = m + 2;
  int Ho = out_dim(H, pad), Wo = out_dim(W, pad);
  int th = n_tiles(Ho, m), tw = n_tiles(Wo, m);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; n++)
    for (int k = 0; k < K; k++)
      for (int ty = 0; ty < th; ty++)
        for (int tx = 0; tx < tw; tx++) {
          double Msum[6][6];
          memset(Msum, 0, sizeof Msum);
          for (int c = 0; c < C; c++) {
            double d[6][6], g[3][3], tmp[6][6], U[6][6], V[6][6];
            for (int i = 0; i < a; i++)
              for (int j = 0; j < a; j++)
                d[i][j] = x_at(X, C, H, W, n, c, ty * m - pad + i, tx * m - pad + j);
            for (int r = 0; r < 3; r++)
              for (int s = 0; s < 3; s++) g[r][s] = Wt[(((size_t)k * C + c) * 3 + r) * 3 + s];
            /* V = B^T d B */
            for (int i = 0; i < a; i++)
              for (int j = 0; j < a; j++) {
                double t = 0;
                for (int q = 0; q < a; q++) t += bt_at(m, i, q) * d[q][j];
                tmp[i][j] = t;
              }
            for (int i = 0; i < a; i++)
              for (int j = 0; j < a; j++) {
                double t = 0;
                for (int q = 0; q < a; q++) t += tmp[i][q] * bt_at(m, j, q); /* B[q][j]=BT[j][q] */
                V[i][j] = t;
              }
            /* U = G g G^T */
            for (int i = 0; i < a; i++)
              for (int s = 0; s < 3; s++) {
                double t = 0;
                for (int r = 0; r < 3; r++) t += g_at(m, i, r) * g[r][s];
                tmp[i][s] = t;
              }
            for (int i = 0; i < a; i++)
              for (int j = 0; j < a; j++) {
                double t = 0;
                for (int s = 0; s < 3; s++) t += tmp[i][s] * g_at(m, j, s);
                U[i][j] = t;
              }
            for (int i = 0; i < a; i++)
              for (int j = 0; j < a; j++) Msum[i][j] += U[i][j] * V[i][j];
          }
          /* S = A^T M A, cropped into Y */
          for (int oi = 0; oi < m; oi++)
            for (int oj = 0; oj < m; oj++) {
              int y = ty * m + oi, x = tx * m + oj;
              if (y >= Ho || x >= Wo) continue;
              double s = 0;
              for (int i = 0; i < a; i++)
                for (int j = 0; j < a; j++) s += at_at(m, oi, i) * Msum[i][j] * at_at(m, oj, j);
              Y[(((size_t)n * K + k) * Ho + y) * Wo + x] = s;
            }
        }
}

/* ==================================================================================== */
/* Part 2, steps 1-3: the transforms in binary32 with a fixed operation order.          */
/* The paper does not say how G g G^T and B^T d B are evaluated; any order is a valid   */
/* reading, but codes are only comparable if one order is fixed.  Chosen here:          */
/*   2-D transform = the 1-D transform applied to every column (left multiplication),   */
/*   then to every row of the result (right multiplication); each 1-D transform is the  */
/*   expression below, every + - * being one rounded binary32 operation.                */
/* ==================================================================================== */

/* t = B^T d for one column/row of length 4 (m = 2). */
static void in1d_m2(const float d[4], float t[4]) {
  t[0] = d[0] - d[2];
  t[1] = d[1] + d[2];
  t[2] = d[2] - d[1];
  t[3] = d[1] - d[3];
}
/* t = B^T d, length 6 (m = 4). */
static void in1d_m4(const float d[6], float t[6]) {
  float p, q, r, s;
  t[0] = (4.0f * d[0] - 5.0f * d[2]) + d[4];
  p = d[4] - 4.0f * d[2];
  q = d[3] - 4.0f * d[1];
  t[1] = p + q;
  t[2] = p - q;
  r = d[4] - d[2];
  s = 2.0f * (d[3] - d[1]);
  t[3] = r + s;
  t[4] = r - s;
  t[5] = (4.0f * d[1] - 5.0f * d[3]) + d[5];
}
/* u = G g for one column/row of length 3 -> 4 (m = 2). */
static void flt1d_m2(const float g[3], float u[4]) {
  float e = g[0] + g[2];
  u[0] = g[0];
  u[1] = (e + g[1]) * 0.5f;
  u[2] = (e - g[1]) * 0.5f;
  u[3] = g[2];
}
/* u = G g, 3 -> 6 (m = 4). */
static void flt1d_m4(const float g[3], float u[6]) {
  const float c6 = (float)(1.0 / 6.0), c24 = (float)(1.0 / 24.0);
  float e = g[0] + g[2];
  float a = g[0] + 4.0f * g[2];
  float b = 2.0f * g[1];
  u[0] = 0.25f * g[0];
  u[1] = (e + g[1]) * (-c6);
  u[2] = (e - g[1]) * (-c6);
  u[3] = (a + b) * c24;
  u[4] = (a - b) * c24;
  u[5] = g[2];
}

/* V = B^T d B for one a x a patch (binary32). */
static void input_tile_transform_f32(int m, const float d[6][6], float V[6][6]) {
  int a = m + 2;
  float T[6][6];
  for (int j = 0; j < a; j++) { /* columns: T = B^T d */
    float col[6], out[6];
    for (int i = 0; i < a; i++) col[i] = d[i][j];
    if (m == 2) in1d_m2(col, out); else in1d_m4(col, out);
    for (int i = 0; i < a; i++) T[i][j] = out[i];
  }
  for (int i = 0; i < a; i++) { /* rows: V = T B, i.e. V[i,:] = B^T T[i,:]^T */
    float out[6];
    if (m == 2) in1d_m2(T[i], out); else in1d_m4(T[i], out);
    for (int j = 0; j < a; j++) V[i][j] = out[j];
  }
}

/* U = G g G^T for one 3 x 3 filter (binary32). */
static void filter_transform_f32(int m, const float g[3][3], float U[6][6]) {
  int a = m + 2;
  float T[6][3];
  for (int s = 0; s < 3; s++) { /* columns: T = G g */
    float col[3], out[6];
    for (int r = 0; r < 3; r++) col[r] = g[r][s];
    if (m == 2) flt1d_m2(col, out); else flt1d_m4(col, out);
    for (int i = 0; i < a; i++) T[i][s] = out[i];
  }
  for (int i = 0; i < a; i++) { /* rows: U = T G^T */
    float out[6];
    if (m == 2) flt1d_m2(T[i], out); else flt1d_m4(T[i], out);
    for (int j = 0; j < a; j++) U[i][j] = out[j];
  }
}

/* Exposed single-tile transforms (tests pin them against printed values / fp64 products). */
void lance_oracle_input_tile_f32(int m, const float *d /*a*a*/, float *v /*a*a*/) {
  int a = m + 2;
  float D[6][6], V[6][6];
  for (int i = 0; i < a; i++)
    for (int j = 0; j < a; j++) D[i][j] = d[i * a + j];
  input_tile_transform_f32(m, D, V);
  for (int i = 0; i < a; i++)
    for (int j = 0; j < a; j++) v[i * a + j] = V[i][j];
}
void lance_oracle_filter_tile_f32(int m, const float *g /*3*3*/, float *u /*a*a*/) {
  int a = m + 2;
  float Gm[3][3], U[6][6];
  for (int i = 0; i < 3; i++)
    for (int j = 0; j < 3; j++) Gm[i][j] = g[i * 3 + j];
  filter_transform_f32(m, Gm, U);
  for (int i = 0; i < a; i++)
    for (int j = 0; j < a; j++) u[i * a + j] = U[i][j];
}

/* U[e][k][c] for all filters (Algorithm 1: g <- W_{k,c}; G g G^T).  e = i*a + j. */
void lance_oracle_filter_transform_f32(const float *Wt, float *U, int K, int C, int m) {
  int a = m + 2;
#pragma omp parallel for schedule(static)
  for (int k = 0; k < K; k++)
    for (int c = 0; c < C; c++) {
      float g[3][3], Um[6][6];
      for (int r = 0; r < 3; r++)
        for (int s = 0; s < 3; s++) g[r][s] = Wt[(((size_t)k * C + c) * 3 + r) * 3 + s];
      filter_transform_f32(m, g, Um);
      for (int i = 0; i < a; i++)
        for (int j = 0; j < a; j++) U[((size_t)(i * a + j) * K + k) * C + c] = Um[i][j];
    }
}

/* V[e][p][c] for all patches (Algorithm 1: D <- patches of X with padding; B^T d B).  */
/* Patch p = (n*th + ty)*tw + tx covers input rows ty*m-pad .. ty*m-pad+a-1; reads      */
/* outside the image are 0 (also for the ragged last tile when m does not divide Ho).   */
void lance_oracle_input_transform_f32(const float *X, float *V, int N, int C, int H, int W,
                                      int pad, int m) {
  int a = m + 2;
  int Ho = out_dim(H, pad), Wo = out_dim(W, pad);
  int th = n_tiles(Ho, m), tw = n_tiles(Wo, m);
  size_t P = (size_t)N * th * tw;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; n++)
    for (int ty = 0; ty < th; ty++)
      for (int tx = 0; tx < tw; tx++) {
        size_t p = ((size_t)n * th + ty) * tw + tx;
        for (int c = 0; c < C; c++) {
          float d[6][6], Vm[6][6];
          for (int i = 0; i < a; i++)
            for (int j = 0; j < a; j++)
              d[i][j] = x_at(X, C, H, W, n, c, ty * m - pad + i, tx * m - pad + j);
          input_tile_transform_f32(m, d, Vm);
          for (int i = 0; i < a; i++)
            for (int j = 0; j < a; j++) V[((size_t)(i * a + j) * P + p) * C + c] = Vm[i][j];
        }
      }
}

/* ==================================================================================== */
/* Part 2, step 4: ranges.  Eq. 7 takes min(T), max(T) over the matrix T that holds x.   */
/* Reading used (parity unpinned by the paper): with the Hadamard product computed as   */
/* one GEMM per Winograd position e (Sec. 3.3), the matrix is that GEMM's operand, so   */
/* there is one (min,max) per position e: over all (k,c) for U, over all (p,c) for V.   */
/* per_tensor != 0 collapses the E ranges into one.  T is [E][count].                   */
/* ==================================================================================== */
void lance_oracle_ranges(const float *T, int E, size_t count, int per_tensor,
                         float *range /*[E][2] = min,max*/) {
  for (int e = 0; e < E; e++) {
    float mn = T[(size_t)e * count], mx = mn;
    for (size_t i = 1; i < count; i++) {
      float x = T[(size_t)e * count + i];
      if (x < mn) mn = x;
      if (x > mx) mx = x;
    }
    range[2 * e] = mn;
    range[2 * e + 1] = mx;
  }
  if (per_tensor) {
    float mn = range[0], mx = range[1];
    for (int e = 1; e < E; e++) {
      if (range[2 * e] < mn) mn = range[2 * e];
      if (range[2 * e + 1] > mx) mx = range[2 * e + 1];
    }
    for (int e = 0; e < E; e++) {
      range[2 * e] = mn;
      range[2 * e + 1] = mx;
    }
  }
}

/* ==================================================================================== */
/* Part 2, steps 5-6: the quantizer Q of Eq. 7.                                          */
/*   levels L = 2^b - 1;   inv = (float)(L / (max - min))  [quotient taken in fp64],     */
/*   scale = (float)((max - min) / L);   a constant matrix (max == min), or a range so   */
/*   small that inv is not finite, gives inv = 0: every code is 0 and Q' returns min.    */
/*   code = round_half_even( (x - min) * inv ), clamped to [0, L]   (two binary32 ops).  */
/* Stored code: code - 2^(b-1), a signed value in [-2^(b-1), 2^(b-1)-1], because signed  */
/* 8-bit multipliers are what the product step uses; Eq. 8 absorbs the shift (below).    */
/* ==================================================================================== */
void lance_oracle_quant_params(float mn, float mx, int bits, float *inv, float *scale) {
  double L = (double)((1 << bits) - 1);
  double range = (double)mx - (double)mn;
  if (range == 0.0) {
    *inv = 0.0f;
    *scale = 0.0f;
    return;
  }
  *inv = (float)(L / range);
  *scale = (float)(range / L);
  if (!isfinite(*inv)) *inv = 0.0f;
}

/* Unsigned code of Eq. 7 in [0, L]. */
int lance_oracle_quantize_value(float x, float mn, float inv, int bits) {
  float L = (float)((1 << bits) - 1);
  float t = (x - mn) * inv;
  float r = rintf(t); /* default rounding mode: to nearest, ties to even */
  if (r < 0.0f) r = 0.0f;
  if (r > L) r = L;
  return (int)r;
}

/* Q' of Eq. 8 on an unsigned code. */
double lance_oracle_dequantize_value(int code, float mn, float scale) {
  return (double)code * (double)scale + (double)mn;
}

/* Quantize T[E][rows][C] (binary32) with range[e] into signed codes [E][rows][Cp];      */
/* lanes c in [C, Cp) hold signed code 0 (they add nothing to the integer product).      */
/* sums[e][row] = sum over c < C of the signed codes (needed by de-quantization).        */
void lance_oracle_quantize(const float *T, const float *range, int bits, int E, size_t rows,
                           int C, int Cp, int8_t *codes, int32_t *sums) {
  int h = 1 << (bits - 1);
  for (int e = 0; e < E; e++) {
    float inv, scale;
    lance_oracle_quant_params(range[2 * e], range[2 * e + 1], bits, &inv, &scale);
#pragma omp parallel for schedule(static)
    for (size_t r = 0; r < rows; r++) {
      int32_t s = 0;
      for (int c = 0; c < C; c++) {
        int q = lance_oracle_quantize_value(T[((size_t)e * rows + r) * C + c], range[2 * e], inv,
                                            bits) - h;
        codes[((size_t)e * rows + r) * Cp + c] = (int8_t)q;
        s += q;
      }
      for (int c = C; c < Cp; c++) codes[((size_t)e * rows + r) * Cp + c] = 0;
      sums[(size_t)e * rows + r] = s;
    }
  }
}

/* ==================================================================================== */
/* Part 2, step 7: the low-precision product.  Algorithm 1 multiplies the codes          */
/* element-wise and sums over channels; over all (k,p) that is, per position e, the      */
/* integer matrix product  ACC_e[k][p] = sum_c qu[e][k][c] * qv[e][p][c]   (Sec. 3.3).   */
/* Exact: int64 accumulation, checked to fit int32.  Returns 0, or 1 on overflow.        */
/* ==================================================================================== */
int lance_oracle_gemm_i8(const int8_t *Uq, const int8_t *Vq, int32_t *ACC, int E, int K,
                         size_t P, int Cp) {
  int overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : overflow)
  for (int e = 0; e < E; e++)
    for (int k = 0; k < K; k++) {
      const int8_t *u = Uq + ((size_t)e * K + k) * Cp;
      for (size_t p = 0; p < P; p++) {
        const int8_t *v = Vq + ((size_t)e * P + p) * Cp;
        int64_t acc = 0;
        for (int c = 0; c < Cp; c++) acc += (int64_t)u[c] * (int64_t)v[c];
        if (acc > INT32_MAX || acc < INT32_MIN) overflow = 1;
        ACC[((size_t)e * K + k) * P + p] = (int32_t)acc;
      }
    }
  return overflow;
}

/* The same product at a list of sampled (e,k,p) triples (for full-size parity checks). */
void lance_oracle_gemm_i8_sampled(const int8_t *Uq, const int8_t *Vq, int K, size_t P, int Cp,
                                  const int64_t *ekp /*[n][3]*/, size_t n, int32_t *out) {
  for (size_t i = 0; i < n; i++) {
    int64_t e = ekp[3 * i], k = ekp[3 * i + 1], p = ekp[3 * i + 2];
    const int8_t *u = Uq + ((size_t)e * K + k) * Cp;
    const int8_t *v = Vq + ((size_t)e * P + p) * Cp;
    int64_t acc = 0;
    for (int c = 0; c < Cp; c++) acc += (int64_t)u[c] * (int64_t)v[c];
    out[i] = (int32_t)acc;
  }
}

/* ==================================================================================== */
/* Part 2, steps 8-9: de-quantize (Eq. 8) and output transform (Eq. 9, Algorithm 1).     */
/* Q' of a product of two codes is read as the product of the two de-quantized values.   */
/* With the stored signed code q' = code - h:   u~ = su*q'u + ou,  ou = min_u + su*h     */
/* (Eq. 8 exactly), likewise v~.  Summing u~ * v~ over the C real channels gives          */
/*   M[e][k][p] = su*sv*ACC + su*ov*RU[e][k] + sv*ou*CV[e][p] + C*ou*ov                  */
/* with RU, CV the code sums.  Then S = A^T M A per (k,p), written into Y (NKHW), rows   */
/* and columns beyond Ho, Wo cropped.  All in fp64.                                      */
/* ==================================================================================== */
void lance_oracle_dequant_output_f64(const int32_t *ACC, const float *u_range,
                                     const int32_t *u_rowsum, const float *v_range,
                                     const int32_t *v_colsum, double *Y, int N, int C, int H,
                                     int W, int K, int pad, int m, int bits_w, int bits_x) {
  /* bits_w, bits_x: bit widths of the filter and of the input codes (Sec. 4 evaluates weights */
  /* and inputs at different widths); each operand's stored code is shifted by its own 2^(b-1). */
  int a = m + 2, E = a * a;
  int Ho = out_dim(H, pad), Wo = out_dim(W, pad);
  int th = n_tiles(Ho, m), tw = n_tiles(Wo, m);
  size_t P = (size_t)N * th * tw;
  double hu = (double)(1 << (bits_w - 1)), hv = (double)(1 << (bits_x - 1));
  double su[36], sv[36], ou[36], ov[36];
  for (int e = 0; e < E; e++) {
    float inv, sc;
    lance_oracle_quant_params(u_range[2 * e], u_range[2 * e + 1], bits_w, &inv, &sc);
    su[e] = sc;
    ou[e] = (double)u_range[2 * e] + su[e] * hu;
    lance_oracle_quant_params(v_range[2 * e], v_range[2 * e + 1], bits_x, &inv, &sc);
    sv[e] = sc;
    ov[e] = (double)v_range[2 * e] + sv[e] * hv;
  }
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; n++)
    for (int k = 0; k < K; k++)
      for (int ty = 0; ty < th; ty++)
        for (int tx = 0; tx < tw; tx++) {
          size_t p = ((size_t)n * th + ty) * tw + tx;
          double M[6][6];
          for (int e = 0; e < E; e++) {
            double acc = ACC[((size_t)e * K + k) * P + p];
            double ru = u_rowsum[(size_t)e * K + k];
            double cv = v_colsum[(size_t)e * P + p];
            M[e / a][e % a] = su[e] * sv[e] * acc + su[e] * ov[e] * ru + sv[e] * ou[e] * cv +
                              (double)C * ou[e] * ov[e];
          }
          for (int oi = 0; oi < m; oi++)
            for (int oj = 0; oj < m; oj++) {
              int y = ty * m + oi, x = tx * m + oj;
              if (y >= Ho || x >= Wo) continue;
              double s = 0;
              for (int i = 0; i < a; i++)
                for (int j = 0; j < a; j++) s += at_at(m, oi, i) * M[i][j] * at_at(m, oj, j);
              Y[(((size_t)n * K + k) * Ho + y) * Wo + x] = s;
            }
        }
}

/* ==================================================================================== */
/* Algorithm 1 taken literally: loops k, p, c; every patch and every filter is           */
/* transformed, quantized (Eq. 7), multiplied code by code, de-quantized (Eq. 8) and     */
/* summed over channels in full precision; then A^T m A.                                  */
/* bits_w, bits_x: widths of the filter and of the input codes (Sec. 4's width grid).    */
/* range_mode 0: T is the (m+2)x(m+2) matrix itself (its own min and max).               */
/* range_mode 1: the ranges are given per position (u_range[e], v_range[e]); then the    */
/*               result must equal the GEMM form above -- a test checks that.            */
/* O(K*P*C) transforms: tiny inputs only.                                                 */
/* ==================================================================================== */
void lance_oracle_alg1_literal_f64(const float *X, const float *Wt, double *Y, int N, int C,
                                   int H, int W, int K, int pad, int m, int bits_w, int bits_x,
                                   int range_mode, const float *u_range, const float *v_range) {
  int a = m + 2;
  int Ho = out_dim(H, pad), Wo = out_dim(W, pad);
  int th = n_tiles(Ho, m), tw = n_tiles(Wo, m);
  for (int k = 0; k < K; k++)
    for (int n = 0; n < N; n++)
      for (int ty = 0; ty < th; ty++)
        for (int tx = 0; tx < tw; tx++) {
          double msum[6][6];
          memset(msum, 0, sizeof msum);
          for (int c = 0; c < C; c++) {
            float g[3][3], d[6][6], U[6][6], V[6][6];
            for (int r = 0; r < 3; r++)
              for (int s = 0; s < 3; s++) g[r][s] = Wt[(((size_t)k * C + c) * 3 + r) * 3 + s];
            for (int i = 0; i < a; i++)
              for (int j = 0; j < a; j++)
                d[i][j] = x_at(X, C, H, W, n, c, ty * m - pad + i, tx * m - pad + j);
            filter_transform_f32(m, g, U);
            input_tile_transform_f32(m, d, V);
            float umn = U[0][0], umx = U[0][0], vmn = V[0][0], vmx = V[0][0];
            for (int i = 0; i < a; i++)
              for (int j = 0; j < a; j++) {
                if (U[i][j] < umn) umn = U[i][j];
                if (U[i][j] > umx) umx = U[i][j];
                if (V[i][j] < vmn) vmn = V[i][j];
                if (V[i][j] > vmx) vmx = V[i][j];
              }
            for (int i = 0; i < a; i++)
              for (int j = 0; j < a; j++) {
                int e = i * a + j;
                float un = umn, ux = umx, vn = vmn, vx = vmx, uinv, us, vinv, vs;
                if (range_mode == 1) {
                  un = u_range[2 * e]; ux = u_range[2 * e + 1];
                  vn = v_range[2 * e]; vx = v_range[2 * e + 1];
                }
                lance_oracle_quant_params(un, ux, bits_w, &uinv, &us);
                lance_oracle_quant_params(vn, vx, bits_x, &vinv, &vs);
                int uh = lance_oracle_quantize_value(U[i][j], un, uinv, bits_w); /* u^ */
                int vh = lance_oracle_quantize_value(V[i][j], vn, vinv, bits_x); /* v^ */
                /* m~ = Q'(u^ .* v^): product of the two de-quantized operands */
                msum[i][j] += lance_oracle_dequantize_value(uh, un, us) *
                              lance_oracle_dequantize_value(vh, vn, vs);
              }
          }
          for (int oi = 0; oi < m; oi++)
            for (int oj = 0; oj < m; oj++) {
              int y = ty * m + oi, x = tx * m + oj;
              if (y >= Ho || x >= Wo) continue;
              double s = 0;
              for (int i = 0; i < a; i++)
                for (int j = 0; j < a; j++) s += at_at(m, oi, i) * msum[i][j] * at_at(m, oj, j);
              Y[(((size_t)n * K + k) * Ho + y) * Wo + x] = s;
            }
        }
}

/* ==================================================================================== */
/* Weight-only quantization (the W-I "4-32" rows of Sec. 4, Table 2): the filters are    */
/* transformed and quantized as above (Eq. 7, one range per position), the input is      */
/* transformed but NOT quantized.  Algorithm 1 with v^ replaced by v = B^T d B:          */
/*   M[e][k][p] = sum_c Q'(u^[e][k][c]) * v[e][p][c],   S = A^T M A.                    */
/* Uq: signed stored codes [E][K][Cc] (Cc >= C, lanes >= C unused); Q' is Eq. 8 on the   */
/* unsigned code (stored code + 2^(bits_w-1)).  v is the binary32 transform; the         */
/* products and sums are fp64.                                                            */
/* ==================================================================================== */
void lance_oracle_weight_only_f64(const float *X, const int8_t *Uq, const float *u_range,
                                  double *Y, int N, int C, int Cc, int H, int W, int K, int pad,
                                  int m, int bits_w) {
  int a = m + 2, E = a * a;
  int Ho = out_dim(H, pad), Wo = out_dim(W, pad);
  int th = n_tiles(Ho, m), tw = n_tiles(Wo, m);
  int hu = 1 << (bits_w - 1);
  float su[36];
  for (int e = 0; e < E; e++) {
    float inv;
    lance_oracle_quant_params(u_range[2 * e], u_range[2 * e + 1], bits_w, &inv, &su[e]);
  }
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; n++)
    for (int ty = 0; ty < th; ty++)
      for (int tx = 0; tx < tw; tx++) {
        for (int k = 0; k < K; k++) {
          double M[6][6];
          memset(M, 0, sizeof M);
          for (int c = 0; c < C; c++) {
            float d[6][6], V[6][6];
            for (int i = 0; i < a; i++)
              for (int j = 0; j < a; j++)
                d[i][j] = x_at(X, C, H, W, n, c, ty * m - pad + i, tx * m - pad + j);
            input_tile_transform_f32(m, d, V);
            for (int i = 0; i < a; i++)
              for (int j = 0; j < a; j++) {
                int e = i * a + j;
                int code = (int)Uq[((size_t)e * K + k) * Cc + c] + hu; /* unsigned code of Eq. 7 */
                M[i][j] += lance_oracle_dequantize_value(code, u_range[2 * e], su[e]) * (double)V[i][j];
              }
          }
          for (int oi = 0; oi < m; oi++)
            for (int oj = 0; oj < m; oj++) {
              int y = ty * m + oi, x = tx * m + oj;
              if (y >= Ho || x >= Wo) continue;
              double s = 0;
              for (int i = 0; i < a; i++)
                for (int j = 0; j < a; j++) s += at_at(m, oi, i) * M[i][j] * at_at(m, oj, j);
              Y[(((size_t)n * K + k) * Ho + y) * Wo + x] = s;
            }
        }
      }
}

/* Number of OpenMP threads the parallel loops above will use. */
#ifdef _OPENMP
#include <omp.h>
int lance_oracle_threads(void) { return omp_get_max_threads(); }
#else
int lance_oracle_threads(void) { return 1; }
#endif
