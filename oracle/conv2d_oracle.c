/*
 * conv2d_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, direct CPU forward 2-D convolution: the definition written
 * out as seven nested loops (batch, output row, output column, window row,
 * window column, input channel, output feature), accumulating in fp64 and
 * rounding once on store.  It is the reference the GPU library is compared
 * against, and it shares no code, header or table with that library.  Only
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What it follows.  The paper (section 3, "SYCL-DNN") names the forward
 * convolution as the routine to accelerate and describes its simplest kernel
 * as a naive one that computes each output directly; the caption of Figure 1
 * gives the parameter tuple (window, stride, image rows, image columns,
 * input features, output features) plus a batch size.  The paper prints no
 * formula, layout, padding rule or data type, so the readings below are
 * conventions fixed by this build (each is restated where it is used):
 *   - cross-correlation (no filter flip);
 *   - input  in[n][h][w][c]   (NHWC, dense),
 *     filter f[r][s][c][k]    (HWCF, dense),
 *     output out[n][p][q][k]  (NHWC, dense);
 *   - VALID: P = ceil((H-R+1)/sr), no padding;
 *     SAME : P = ceil(H/sr), total padding max((P-1)*sr + R - H, 0), the
 *            smaller half before (top/left), the larger after (bottom/right);
 *   - a tap outside the image contributes nothing (it is skipped, not
 *     multiplied by zero);
 *   - dilation 1, one group, no bias, no activation.
 *
 *   out[n,p,q,k] = sum_{r,s,c} X(n, p*sr + r - pt, q*sc + s - pl, c) * f[r,s,c,k]
 *   X = in inside the image, 0 outside.
 *
 * Pins (tests/test_oracle_pins.py): all-ones closed form (count of valid taps
 * times C), hand-worked 4x4 examples, identity/delta filters, linearity,
 * translation equivariance, 1x1 == matmul, full-window VALID == dot product,
 * brute-force im2col + naive matmul on tiny random shapes.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_PAD_VALID = 0, ORACLE_PAD_SAME = 1 };

typedef struct {
  int32_t batch, in_rows, in_cols, channels, features;
  int32_t window_rows, window_cols, stride_rows, stride_cols;
  int32_t padding; /* ORACLE_PAD_VALID or ORACLE_PAD_SAME */
} conv2d_oracle_params;

typedef struct {
  int32_t out_rows, out_cols, pad_top, pad_bottom, pad_left, pad_right;
} conv2d_oracle_geometry;

/* ceil(a / b) for b > 0 and any sign of a. */
static int64_t ceil_div(int64_t a, int64_t b) {
  int64_t q = a / b;
  if ((a % b != 0) && ((a < 0) == (b < 0))) q += 1;
  return q;
}

/* One spatial axis: output extent and the padding before/after it. */
static int axis_geometry(int32_t padding, int64_t extent, int64_t window, int64_t stride,
                         int32_t* out_extent, int32_t* pad_before, int32_t* pad_after) {
  int64_t o, total;
  if (padding == ORACLE_PAD_VALID) {
    o = ceil_div(extent - window + 1, stride);
    total = 0;
  } else if (padding == ORACLE_PAD_SAME) {
    o = ceil_div(extent, stride);
    total = (o - 1) * stride + window - extent;
    if (total < 0) total = 0;
  } else {
    return -1;
  }
  if (o <= 0) return -1;
  *out_extent = (int32_t)o;
  *pad_before = (int32_t)(total / 2);          /* smaller half first  */
  *pad_after = (int32_t)(total - total / 2);   /* larger half last    */
  return 0;
}

static int params_ok(const conv2d_oracle_params* p) {
  return p && p->batch >= 0 && p->in_rows > 0 && p->in_cols > 0 && p->channels > 0 &&
         p->features > 0 && p->window_rows > 0 && p->window_cols > 0 && p->stride_rows > 0 &&
         p->stride_cols > 0;
}

/* Output size and padding for a parameter tuple.  Returns 0, or -1 for a
 * tuple with no valid output (non-positive sizes, VALID window larger than
 * the image, unknown padding mode). */
int conv2d_oracle_get_geometry(const conv2d_oracle_params* p, conv2d_oracle_geometry* g) {
  if (!params_ok(p) || !g) return -1;
  if (axis_geometry(p->padding, p->in_rows, p->window_rows, p->stride_rows, &g->out_rows,
                    &g->pad_top, &g->pad_bottom))
    return -1;
  if (axis_geometry(p->padding, p->in_cols, p->window_cols, p->stride_cols, &g->out_cols,
                    &g->pad_left, &g->pad_right))
    return -1;
  return 0;
}

int conv2d_oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Forward convolution, fp32 data, fp64 accumulation, one rounding to fp32.
 * All pointers are host memory.  num_threads <= 0 means "all cores".
 * Loop nest: n, p, q outermost (shared over threads), then r, s with the
 * bounds test, then c, and innermost k over a per-pixel fp64 accumulator
 * row (the filter row f[r][s][c][:] is contiguous). */
int conv2d_oracle_forward_f32(const conv2d_oracle_params* p, const float* in, const float* filt,
                              float* out, int num_threads) {
  conv2d_oracle_geometry g;
  if (conv2d_oracle_get_geometry(p, &g)) return -1;
  if (p->batch == 0) return 0;
  if (!in || !filt || !out) return -1;
  const int64_t N = p->batch, H = p->in_rows, W = p->in_cols, C = p->channels, K = p->features;
  const int64_t R = p->window_rows, S = p->window_cols, sr = p->stride_rows, sc = p->stride_cols;
  const int64_t P = g.out_rows, Q = g.out_cols, pt = g.pad_top, pl = g.pad_left;
  int nt = num_threads > 0 ? num_threads : conv2d_oracle_max_threads();
  int failed = 0;
#pragma omp parallel num_threads(nt)
  {
    double* acc = (double*)malloc((size_t)K * sizeof(double));
    if (!acc) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp for collapse(2) schedule(dynamic, 1)
    for (int64_t n = 0; n < N; ++n) {
      for (int64_t op = 0; op < P; ++op) {
        if (!acc) continue;
        for (int64_t oq = 0; oq < Q; ++oq) {
          for (int64_t k = 0; k < K; ++k) acc[k] = 0.0;
          for (int64_t r = 0; r < R; ++r) {
            const int64_t h = op * sr + r - pt;
            if (h < 0 || h >= H) continue;
            for (int64_t s = 0; s < S; ++s) {
              const int64_t w = oq * sc + s - pl;
              if (w < 0 || w >= W) continue;
              const float* x = in + ((n * H + h) * W + w) * C;
              const float* f = filt + ((r * S + s) * C) * K;
              for (int64_t c = 0; c < C; ++c) {
                const double xv = (double)x[c];
                const float* fk = f + c * K;
                for (int64_t k = 0; k < K; ++k) acc[k] += xv * (double)fk[k];
              }
            }
          }
          float* o = out + ((n * P + op) * Q + oq) * K;
          for (int64_t k = 0; k < K; ++k) o[k] = (float)acc[k];
        }
      }
    }
    free(acc);
  }
  return failed ? -2 : 0;
}

/* Same definition on fp64 data with fp64 output (used by the pin tests so
 * that exact identities can be checked without the final fp32 rounding). */
int conv2d_oracle_forward_f64(const conv2d_oracle_params* p, const double* in,
                              const double* filt, double* out, int num_threads) {
  conv2d_oracle_geometry g;
  if (conv2d_oracle_get_geometry(p, &g)) return -1;
  if (p->batch == 0) return 0;
  if (!in || !filt || !out) return -1;
  const int64_t N = p->batch, H = p->in_rows, W = p->in_cols, C = p->channels, K = p->features;
  const int64_t R = p->window_rows, S = p->window_cols, sr = p->stride_rows, sc = p->stride_cols;
  const int64_t P = g.out_rows, Q = g.out_cols, pt = g.pad_top, pl = g.pad_left;
  int nt = num_threads > 0 ? num_threads : conv2d_oracle_max_threads();
#pragma omp parallel for collapse(2) schedule(dynamic, 1) num_threads(nt)
  for (int64_t n = 0; n < N; ++n) {
    for (int64_t op = 0; op < P; ++op) {
      for (int64_t oq = 0; oq < Q; ++oq) {
        for (int64_t k = 0; k < K; ++k) {
          double acc = 0.0;
          for (int64_t r = 0; r < R; ++r) {
            const int64_t h = op * sr + r - pt;
            if (h < 0 || h >= H) continue;
            for (int64_t s = 0; s < S; ++s) {
              const int64_t w = oq * sc + s - pl;
              if (w < 0 || w >= W) continue;
              for (int64_t c = 0; c < C; ++c)
                acc += in[((n * H + h) * W + w) * C + c] * filt[((r * S + s) * C + c) * K + k];
            }
          }
          out[((n * P + op) * Q + oq) * K + k] = acc;
        }
      }
    }
  }
  return 0;
}

/* Selected outputs only: out_vals[i] = the fp64 sum (not rounded) at the flat
 * NHWC output index flat_index[i].  Lets a test check sampled elements of a
 * layer that is too large to convolve whole on the CPU in seconds. */
int conv2d_oracle_points_f32(const conv2d_oracle_params* p, const float* in, const float* filt,
                             const int64_t* flat_index, int64_t count, double* out_vals,
                             int num_threads) {
  conv2d_oracle_geometry g;
  if (conv2d_oracle_get_geometry(p, &g)) return -1;
  if (count == 0) return 0;
  if (!in || !filt || !flat_index || !out_vals || count < 0) return -1;
  const int64_t N = p->batch, H = p->in_rows, W = p->in_cols, C = p->channels, K = p->features;
  const int64_t R = p->window_rows, S = p->window_cols, sr = p->stride_rows, sc = p->stride_cols;
  const int64_t P = g.out_rows, Q = g.out_cols, pt = g.pad_top, pl = g.pad_left;
  const int64_t total = N * P * Q * K;
  for (int64_t i = 0; i < count; ++i)
    if (flat_index[i] < 0 || flat_index[i] >= total) return -1;
  int nt = num_threads > 0 ? num_threads : conv2d_oracle_max_threads();
#pragma omp parallel for schedule(dynamic, 16) num_threads(nt)
  for (int64_t i = 0; i < count; ++i) {
    int64_t idx = flat_index[i];
    const int64_t k = idx % K; idx /= K;
    const int64_t oq = idx % Q; idx /= Q;
    const int64_t op = idx % P; idx /= P;
    const int64_t n = idx;
    double acc = 0.0;
    for (int64_t r = 0; r < R; ++r) {
      const int64_t h = op * sr + r - pt;
      if (h < 0 || h >= H) continue;
      for (int64_t s = 0; s < S; ++s) {
        const int64_t w = oq * sc + s - pl;
        if (w < 0 || w >= W) continue;
        for (int64_t c = 0; c < C; ++c)
          acc += (double)in[((n * H + h) * W + w) * C + c] *
                 (double)filt[((r * S + s) * C + c) * K + k];
      }
    }
    out_vals[i] = acc;
  }
  return 0;
}
