/* CPU oracle for a chain of local operators executed on row bands.
 *
 * TEST INFRASTRUCTURE ONLY. This file is the slow, plain definition the GPU
 * library is checked against; the product never calls it. It shares no code
 * with the HIP path.
 *
 * What it computes: the paper's block-wise local operators (Sec. IV-A:
 * convolution and max pooling, whose input block follows from kernel size,
 * padding and dilation) and element-wise local operators (Sec. IV-A: ReLU and
 * the like), each evaluated on a contiguous interval of output rows (the
 * "operation batching" interval of Sec. IV-C, Computational Efficiency) of a
 * tensor that is held as a *row slab*: rows [row0, row0+rows) of an image whose
 * true height is H. A slab with row0 = 0 and rows = H is the whole tensor, so
 * the same functions give the unpartitioned result.
 *
 * Layout: activations NCHW, weights OIHW (depthwise: C x 1 x kh x kw), all
 * stored as float. bf16 tensors are floats whose values are bf16-representable.
 *
 * Arithmetic: every output element is accumulated in double in the fixed order
 * ci -> kh -> kw, taps that fall outside the image [0,H) x [0,W) are skipped
 * (zero padding for convolution, -inf padding for max pooling), then bias,
 * residual and activation are applied in double and the result is rounded
 * ONCE to the storage type (float, or bfloat16 with round-to-nearest-even).
 * A tap inside the image but outside the slab is a planner error: the function
 * returns ORACLE_ERR_SLAB and the output is not to be trusted.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_SLAB (-1)
#define ORACLE_ERR_ARG (-2)

enum { ORACLE_ACT_NONE = 0, ORACLE_ACT_RELU = 1, ORACLE_ACT_RELU6 = 2 };
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* Threads the parallel loops below will use (for reporting next to timings). */
int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Round a double to the nearest bfloat16 value (8 significant bits, float32
 * exponent range), ties to even; the result is returned as a double that is
 * exactly representable in bfloat16. nearbyint() rounds ties to even in the
 * default rounding mode. */
double oracle_round_bf16(double v) {
  if (v == 0.0 || isnan(v) || isinf(v)) return v;
  int e;
  (void)frexp(v, &e);            /* |v| = m * 2^e, m in [0.5, 1) */
  int q = e - 8;                 /* quantum 2^q keeps 8 significant bits */
  if (q < -133) q = -133;        /* bf16 subnormals: multiples of 2^-133 */
  double r = ldexp(nearbyint(ldexp(v, -q)), q);
  if (fabs(r) >= ldexp(1.0, 128)) r = v > 0 ? INFINITY : -INFINITY;
  return r;
}

static inline float store(double v, int dtype) {
  if (dtype == ORACLE_BF16) v = oracle_round_bf16(v);
  return (float)v;
}

static inline double activate(double v, int act) {
  if (act == ORACLE_ACT_RELU) return v > 0.0 ? v : 0.0;
  if (act == ORACLE_ACT_RELU6) return v < 0.0 ? 0.0 : (v > 6.0 ? 6.0 : v);
  return v;
}

/* Output height/width of a windowed operator (floor mode). */
int oracle_out_size(int in, int k, int s, int p, int d) {
  int span = in + 2 * p - d * (k - 1) - 1;
  if (span < 0) return 0;
  return span / s + 1;
}

/* Convolution (cross-correlation, no kernel flip) with `groups` channel groups.
 *
 * x    : [N][C_in][x_rows][W]   rows x_row0 .. x_row0+x_rows of an image of height H
 * w    : [C_out][C_in/groups][kh][kw]
 * bias : [C_out] or NULL
 * res  : [N][C_out][r_rows][W_out] rows r_row0.. of the H_out-row residual, or NULL
 * y    : [N][C_out][y_rows][W_out] rows y_row0.. ; ALL y_rows rows are computed.
 */
int oracle_conv2d(const float* x, int x_row0, int x_rows, int N, int C_in, int H, int W,
                  const float* w, const float* bias, int C_out, int groups,
                  int kh, int kw, int sh, int sw, int ph, int pw, int dh, int dw,
                  const float* res, int r_row0, int r_rows, int act, int dtype,
                  float* y, int y_row0, int y_rows) {
  if (groups < 1 || C_in % groups || C_out % groups) return ORACLE_ERR_ARG;
  const int H_out = oracle_out_size(H, kh, sh, ph, dh);
  const int W_out = oracle_out_size(W, kw, sw, pw, dw);
  if (y_row0 < 0 || y_row0 + y_rows > H_out) return ORACLE_ERR_ARG;
  const int cig = C_in / groups, cog = C_out / groups;
  int bad = 0;
#pragma omp parallel for collapse(3) schedule(static) reduction(| : bad)
  for (int n = 0; n < N; ++n)
    for (int co = 0; co < C_out; ++co)
      for (int yr = 0; yr < y_rows; ++yr) {
        const int oh = y_row0 + yr;
        const int g = co / cog;
        for (int ow = 0; ow < W_out; ++ow) {
          double acc = 0.0;
          for (int cl = 0; cl < cig; ++cl) {
            const int ci = g * cig + cl;
            for (int a = 0; a < kh; ++a) {
              const int ih = oh * sh - ph + a * dh;
              if (ih < 0 || ih >= H) continue;               /* zero padding */
              if (ih < x_row0 || ih >= x_row0 + x_rows) { bad = 1; continue; }
              for (int b = 0; b < kw; ++b) {
                const int iw = ow * sw - pw + b * dw;
                if (iw < 0 || iw >= W) continue;             /* zero padding */
                const double xv =
                    x[(((size_t)n * C_in + ci) * x_rows + (ih - x_row0)) * W + iw];
                const double wv = w[(((size_t)co * cig + cl) * kh + a) * kw + b];
                acc += xv * wv;
              }
            }
          }
          if (bias) acc += (double)bias[co];
          if (res) {
            if (oh < r_row0 || oh >= r_row0 + r_rows) { bad = 1; }
            else acc += (double)res[(((size_t)n * C_out + co) * r_rows + (oh - r_row0)) * W_out + ow];
          }
          y[(((size_t)n * C_out + co) * y_rows + yr) * W_out + ow] = store(activate(acc, act), dtype);
        }
      }
  return bad ? ORACLE_ERR_SLAB : ORACLE_OK;
}

/* Max pooling, floor mode; taps outside the image are skipped (-inf padding).
 * A window with no tap inside the image cannot occur when p < k. */
int oracle_maxpool2d(const float* x, int x_row0, int x_rows, int N, int C, int H, int W,
                     int kh, int kw, int sh, int sw, int ph, int pw,
                     float* y, int y_row0, int y_rows) {
  const int H_out = oracle_out_size(H, kh, sh, ph, 1);
  const int W_out = oracle_out_size(W, kw, sw, pw, 1);
  if (y_row0 < 0 || y_row0 + y_rows > H_out) return ORACLE_ERR_ARG;
  int bad = 0;
#pragma omp parallel for collapse(3) schedule(static) reduction(| : bad)
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < C; ++c)
      for (int yr = 0; yr < y_rows; ++yr) {
        const int oh = y_row0 + yr;
        for (int ow = 0; ow < W_out; ++ow) {
          double m = -INFINITY;
          for (int a = 0; a < kh; ++a) {
            const int ih = oh * sh - ph + a;
            if (ih < 0 || ih >= H) continue;
            if (ih < x_row0 || ih >= x_row0 + x_rows) { bad = 1; continue; }
            for (int b = 0; b < kw; ++b) {
              const int iw = ow * sw - pw + b;
              if (iw < 0 || iw >= W) continue;
              const double v = x[(((size_t)n * C + c) * x_rows + (ih - x_row0)) * W + iw];
              if (v > m) m = v;
            }
          }
          y[(((size_t)n * C + c) * y_rows + yr) * W_out + ow] = (float)m;
        }
      }
  return bad ? ORACLE_ERR_SLAB : ORACLE_OK;
}

/* Stand-alone element-wise operator: y = act(x + bias[c] + res). */
int oracle_eltwise(const float* x, int x_row0, int x_rows, int N, int C, int H, int W,
                   const float* bias, const float* res, int r_row0, int r_rows,
                   int act, int dtype, float* y, int y_row0, int y_rows) {
  if (y_row0 < 0 || y_row0 + y_rows > H) return ORACLE_ERR_ARG;
  int bad = 0;
#pragma omp parallel for collapse(3) schedule(static) reduction(| : bad)
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < C; ++c)
      for (int yr = 0; yr < y_rows; ++yr) {
        const int oh = y_row0 + yr;
        if (oh < x_row0 || oh >= x_row0 + x_rows) { bad = 1; continue; }
        if (res && (oh < r_row0 || oh >= r_row0 + r_rows)) { bad = 1; continue; }
        for (int ow = 0; ow < W; ++ow) {
          double v = x[(((size_t)n * C + c) * x_rows + (oh - x_row0)) * W + ow];
          if (bias) v += (double)bias[c];
          if (res) v += (double)res[(((size_t)n * C + c) * r_rows + (oh - r_row0)) * W + ow];
          y[(((size_t)n * C + c) * y_rows + yr) * W + ow] = store(activate(v, act), dtype);
        }
      }
  return bad ? ORACLE_ERR_SLAB : ORACLE_OK;
}

/* Row-wise local operator (Intra-DP Sec. IV-A, Eq. 1): rows [row0, row0 + rows) of
 * y = act(x * W^T + bias + res) for a matrix x of m rows and k columns (row-major) and a
 * parameter matrix W of n rows and k columns (one row per output column) that every row of x
 * meets whole. x, res and y are full matrices; only the named rows of y are written, each from
 * the same row of x (and of res) alone. Accumulation in double over j = 0..k-1, one rounding. */
int oracle_rowwise(const float* x, int m, int k, const float* w, int n, const float* bias,
                   const float* res, int act, int dtype, float* y, int row0, int rows) {
  if (row0 < 0 || rows < 0 || row0 + rows > m) return ORACLE_ERR_ARG;
#pragma omp parallel for collapse(2) schedule(static)
  for (int i = row0; i < row0 + rows; ++i)
    for (int c = 0; c < n; ++c) {
      double acc = 0.0;
      for (int j = 0; j < k; ++j) acc += (double)x[(size_t)i * k + j] * (double)w[(size_t)c * k + j];
      if (bias) acc += (double)bias[c];
      if (res) acc += (double)res[(size_t)i * n + c];
      y[(size_t)i * n + c] = store(activate(acc, act), dtype);
    }
  return ORACLE_OK;
}
