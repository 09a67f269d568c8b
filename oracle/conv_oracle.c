/*
 * CPU oracle for the lowering-based convolutional layer.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file;
 * it exists so that the HIP kernels can be checked against a plain, slow,
 * obviously correct implementation.  It shares no code with the GPU path.
 *
 * Part A (direct definition).  The lowering method reaches exactly the result
 * of the direct convolution (the three lowerings only regroup the sum of
 * eq. (1), Sec. 2.1 "Lowering Strategies"), so the oracle for the layer is
 * eq. (1) itself written as nested loops, extended with stride, zero padding,
 * channel groups and bias in the way Caffe defines them (the paper claims
 * layer-by-layer agreement with Caffe, Sec. 1 / Sec. 3.2):
 *
 *   y[n,o,r,c] = bias[o] + sum_{ci<Cg} sum_{i<K} sum_{j<K}
 *                x[n, (o / Og)*Cg + ci, r*s + i - p, c*s + j - p] * w[o,ci,i,j]
 *
 * with out-of-range rows/columns contributing zero, Cg = C/groups,
 * Og = O/groups, Hout = floor((H + 2p - K)/s) + 1.  No kernel flip
 * (cross-correlation), as eq. (1) prints D[r+r', c+c'] * K[r', c'].
 *
 * The paper does not describe the backward passes.  They are defined here as
 * the adjoints of the forward map with respect to x and to w (the gradient of
 * <dy, y>), plus dbias = plain sum of dy over n, r, c.
 *
 * Part B (the paper's three lowerings, Sec. 2.1, Type 1 / Type 2 / Type 3),
 * written step by step (lower, multiply, lift) in the paper's order with the
 * same generalisation to stride / pad / groups / batch.  Used for the
 * bit-exact check of the GPU lowering maps and as a second route to y.
 *
 * Floating point: inputs are fp32 (the bytes the GPU sees); every product and
 * sum is fp64 (a product of two fp32 values is exact in fp64); outputs fp64.
 *
 * Threading: OpenMP over independent output elements only.  No blocking, no
 * reordering of the reduction: each output is one sequential fp64 sum in the
 * loop order written here.
 *
 * Pins (tests/test_oracle_pins.py): hand-computed tiny case, 1x1 conv ==
 * matrix product, delta kernel, all-ones closed form, pad/stride/group
 * structural identities, scipy/torch library convolutions, the paper's
 * printed index formulas for Types 1-3 written out in Python, adjoint
 * identities and finite differences for the backward passes.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int N, C, H, W, O, K, stride, pad, groups;
} oracle_dims_t;

static int out_dim(int in, int K, int s, int p) {
  int t = in + 2 * p - K;
  if (t < 0) return 0;
  return t / s + 1;
}

static int dims_ok(const oracle_dims_t* d) {
  if (!d) return 0;
  if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->O <= 0 || d->K <= 0) return 0;
  if (d->stride < 1 || d->pad < 0 || d->groups < 1) return 0;
  if (d->C % d->groups || d->O % d->groups) return 0;
  if (d->H + 2 * d->pad < d->K || d->W + 2 * d->pad < d->K) return 0;
  return 1;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

int oracle_output_dims(const oracle_dims_t* d, int* Hout, int* Wout) {
  if (!dims_ok(d)) return -1;
  *Hout = out_dim(d->H, d->K, d->stride, d->pad);
  *Wout = out_dim(d->W, d->K, d->stride, d->pad);
  return 0;
}

/* ------------------------------------------------------------------ */
/* Part A: direct definition                                           */
/* ------------------------------------------------------------------ */

/* One output element of the forward map (eq. (1) + stride/pad/groups/bias). */
static double fwd_elem(const oracle_dims_t* d, const float* x, const float* w, const float* bias,
                       int n, int o, int r, int c) {
  const int Cg = d->C / d->groups, Og = d->O / d->groups, K = d->K;
  const int q = o / Og;
  double acc = bias ? (double)bias[o] : 0.0;
  for (int ci = 0; ci < Cg; ++ci) {
    const float* xp = x + ((int64_t)n * d->C + (int64_t)q * Cg + ci) * d->H * d->W;
    const float* wp = w + ((int64_t)o * Cg + ci) * K * K;
    for (int i = 0; i < K; ++i) {
      const int h = r * d->stride + i - d->pad;
      if (h < 0 || h >= d->H) continue;
      for (int j = 0; j < K; ++j) {
        const int ww = c * d->stride + j - d->pad;
        if (ww < 0 || ww >= d->W) continue;
        acc += (double)xp[(int64_t)h * d->W + ww] * (double)wp[i * K + j];
      }
    }
  }
  return acc;
}

int oracle_conv_forward(const oracle_dims_t* d, const float* x, const float* w, const float* bias,
                        double* y) {
  if (!dims_ok(d) || !x || !w || !y) return -1;
  const int Hout = out_dim(d->H, d->K, d->stride, d->pad);
  const int Wout = out_dim(d->W, d->K, d->stride, d->pad);
  const int64_t planes = (int64_t)d->N * d->O;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t t = 0; t < planes; ++t) {
    const int n = (int)(t / d->O), o = (int)(t % d->O);
    double* yp = y + t * Hout * Wout;
    for (int r = 0; r < Hout; ++r)
      for (int c = 0; c < Wout; ++c) yp[(int64_t)r * Wout + c] = fwd_elem(d, x, w, bias, n, o, r, c);
  }
  return 0;
}

/* Forward at sampled linear indices of y (N x O x Hout x Wout order). */
int oracle_conv_forward_at(const oracle_dims_t* d, const float* x, const float* w, const float* bias,
                           const int64_t* idx, int64_t nidx, double* out) {
  if (!dims_ok(d) || !x || !w || !idx || !out) return -1;
  const int Hout = out_dim(d->H, d->K, d->stride, d->pad);
  const int Wout = out_dim(d->W, d->K, d->stride, d->pad);
  const int64_t total = (int64_t)d->N * d->O * Hout * Wout;
  for (int64_t t = 0; t < nidx; ++t)
    if (idx[t] < 0 || idx[t] >= total) return -2;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t t = 0; t < nidx; ++t) {
    int64_t v = idx[t];
    const int c = (int)(v % Wout); v /= Wout;
    const int r = (int)(v % Hout); v /= Hout;
    const int o = (int)(v % d->O); v /= d->O;
    out[t] = fwd_elem(d, x, w, bias, (int)v, o, r, c);
  }
  return 0;
}

/* One element of dx: the adjoint of the forward map in x.
 * dx[n, q*Cg+ci, h, w] = sum over o in group q and over (i,j) such that
 * h = r*s + i - p and w = c*s + j - p for an output position (r,c). */
static double bwd_data_elem(const oracle_dims_t* d, const float* w, const float* dy, int Hout,
                            int Wout, int n, int cglob, int h, int ww) {
  const int Cg = d->C / d->groups, Og = d->O / d->groups, K = d->K, s = d->stride;
  const int q = cglob / Cg, ci = cglob % Cg;
  double acc = 0.0;
  for (int oo = 0; oo < Og; ++oo) {
    const int o = q * Og + oo;
    const float* dyp = dy + ((int64_t)n * d->O + o) * Hout * Wout;
    const float* wp = w + ((int64_t)o * Cg + ci) * K * K;
    for (int i = 0; i < K; ++i) {
      const int hr = h + d->pad - i;
      if (hr < 0 || hr % s) continue;
      const int r = hr / s;
      if (r >= Hout) continue;
      for (int j = 0; j < K; ++j) {
        const int wc = ww + d->pad - j;
        if (wc < 0 || wc % s) continue;
        const int c = wc / s;
        if (c >= Wout) continue;
        acc += (double)dyp[(int64_t)r * Wout + c] * (double)wp[i * K + j];
      }
    }
  }
  return acc;
}

int oracle_conv_backward_data(const oracle_dims_t* d, const float* w, const float* dy, double* dx) {
  if (!dims_ok(d) || !w || !dy || !dx) return -1;
  const int Hout = out_dim(d->H, d->K, d->stride, d->pad);
  const int Wout = out_dim(d->W, d->K, d->stride, d->pad);
  const int64_t planes = (int64_t)d->N * d->C;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t t = 0; t < planes; ++t) {
    const int n = (int)(t / d->C), cg = (int)(t % d->C);
    double* dxp = dx + t * d->H * d->W;
    for (int h = 0; h < d->H; ++h)
      for (int ww = 0; ww < d->W; ++ww)
        dxp[(int64_t)h * d->W + ww] = bwd_data_elem(d, w, dy, Hout, Wout, n, cg, h, ww);
  }
  return 0;
}

int oracle_conv_backward_data_at(const oracle_dims_t* d, const float* w, const float* dy,
                                 const int64_t* idx, int64_t nidx, double* out) {
  if (!dims_ok(d) || !w || !dy || !idx || !out) return -1;
  const int Hout = out_dim(d->H, d->K, d->stride, d->pad);
  const int Wout = out_dim(d->W, d->K, d->stride, d->pad);
  const int64_t total = (int64_t)d->N * d->C * d->H * d->W;
  for (int64_t t = 0; t < nidx; ++t)
    if (idx[t] < 0 || idx[t] >= total) return -2;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t t = 0; t < nidx; ++t) {
    int64_t v = idx[t];
    const int ww = (int)(v % d->W); v /= d->W;
    const int h = (int)(v % d->H); v /= d->H;
    const int cg = (int)(v % d->C); v /= d->C;
    out[t] = bwd_data_elem(d, w, dy, Hout, Wout, (int)v, cg, h, ww);
  }
  return 0;
}

/* One element of dw: the adjoint of the forward map in w.
 * dw[o,ci,i,j] = sum_n sum_r sum_c dy[n,o,r,c] * x[n, q*Cg+ci, r*s+i-p, c*s+j-p]. */
static double bwd_weights_elem(const oracle_dims_t* d, const float* x, const float* dy, int Hout,
                               int Wout, int o, int ci, int i, int j) {
  const int Cg = d->C / d->groups, Og = d->O / d->groups;
  const int q = o / Og;
  double acc = 0.0;
  for (int n = 0; n < d->N; ++n) {
    const float* xp = x + ((int64_t)n * d->C + (int64_t)q * Cg + ci) * d->H * d->W;
    const float* dyp = dy + ((int64_t)n * d->O + o) * Hout * Wout;
    for (int r = 0; r < Hout; ++r) {
      const int h = r * d->stride + i - d->pad;
      if (h < 0 || h >= d->H) continue;
      for (int c = 0; c < Wout; ++c) {
        const int ww = c * d->stride + j - d->pad;
        if (ww < 0 || ww >= d->W) continue;
        acc += (double)dyp[(int64_t)r * Wout + c] * (double)xp[(int64_t)h * d->W + ww];
      }
    }
  }
  return acc;
}

/* dbias may be NULL. */
int oracle_conv_backward_weights(const oracle_dims_t* d, const float* x, const float* dy, double* dw,
                                 double* dbias) {
  if (!dims_ok(d) || !x || !dy || !dw) return -1;
  const int Hout = out_dim(d->H, d->K, d->stride, d->pad);
  const int Wout = out_dim(d->W, d->K, d->stride, d->pad);
  const int Cg = d->C / d->groups, K = d->K;
  const int64_t total = (int64_t)d->O * Cg * K * K;
#pragma omp parallel for schedule(dynamic, 4)
  for (int64_t t = 0; t < total; ++t) {
    int64_t v = t;
    const int j = (int)(v % K); v /= K;
    const int i = (int)(v % K); v /= K;
    const int ci = (int)(v % Cg); v /= Cg;
    dw[t] = bwd_weights_elem(d, x, dy, Hout, Wout, (int)v, ci, i, j);
  }
  if (dbias) {
#pragma omp parallel for schedule(static)
    for (int o = 0; o < d->O; ++o) {
      double acc = 0.0;
      for (int n = 0; n < d->N; ++n) {
        const float* dyp = dy + ((int64_t)n * d->O + o) * Hout * Wout;
        for (int64_t t = 0; t < (int64_t)Hout * Wout; ++t) acc += (double)dyp[t];
      }
      dbias[o] = acc;
    }
  }
  return 0;
}

int oracle_conv_backward_weights_at(const oracle_dims_t* d, const float* x, const float* dy,
                                    const int64_t* idx, int64_t nidx, double* out) {
  if (!dims_ok(d) || !x || !dy || !idx || !out) return -1;
  const int Hout = out_dim(d->H, d->K, d->stride, d->pad);
  const int Wout = out_dim(d->W, d->K, d->stride, d->pad);
  const int Cg = d->C / d->groups, K = d->K;
  const int64_t total = (int64_t)d->O * Cg * K * K;
  for (int64_t t = 0; t < nidx; ++t)
    if (idx[t] < 0 || idx[t] >= total) return -2;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t t = 0; t < nidx; ++t) {
    int64_t v = idx[t];
    const int j = (int)(v % K); v /= K;
    const int i = (int)(v % K); v /= K;
    const int ci = (int)(v % Cg); v /= Cg;
    out[t] = bwd_weights_elem(d, x, dy, Hout, Wout, (int)v, ci, i, j);
  }
  return 0;
}

/* ------------------------------------------------------------------ */
/* Part B: the three lowerings of Sec. 2.1                             */
/* ------------------------------------------------------------------ */
/*
 * Conventions (the paper's flattening formula is garbled and its tensors are
 * channel-last; the lowered matrix is internal to the method, so any
 * flattening used consistently for the columns of D^ and the rows of K^
 * gives the same product).  Per group q:
 *
 *   Type 1  rows (n, r, c) over OUTPUT positions,    cols (ci, i, j)
 *           D^[(n,r,c),(ci,i,j)] = x[n, q*Cg+ci, r*s+i-p, c*s+j-p]  (0 outside)
 *           K^[(ci,i,j), o]      = w[o,ci,i,j]
 *           R^[(n,r,c), o]       -> y[n,o,r,c] = R^ + bias            (trivial lift)
 *
 *   Type 2  rows (n, h, c): every INPUT row h, output column c;  cols (ci, j)
 *           D^[(n,h,c),(ci,j)]   = x[n, q*Cg+ci, h, c*s+j-p]         (0 outside)
 *           K^[(ci,j),(o,i)]     = w[o,ci,i,j]
 *           y[n,o,r,c] = bias + sum_i R^[(n, r*s+i-p, c),(o,i)]      (rows in range)
 *
 *   Type 3  rows (n, h, w) over INPUT positions,      cols (ci)
 *           D^[(n,h,w), ci]      = x[n, q*Cg+ci, h, w]
 *           K^[ci,(o,i,j)]       = w[o,ci,i,j]
 *           y[n,o,r,c] = bias + sum_{i,j} R^[(n, r*s+i-p, c*s+j-p),(o,i,j)]
 *
 * The matrices of all groups are stored one after another (group-major).
 */

int oracle_lowered_shape(const oracle_dims_t* d, int type, int64_t* rows, int64_t* cols,
                         int64_t* rcols) {
  if (!dims_ok(d) || type < 1 || type > 3) return -1;
  const int Hout = out_dim(d->H, d->K, d->stride, d->pad);
  const int Wout = out_dim(d->W, d->K, d->stride, d->pad);
  const int Cg = d->C / d->groups, Og = d->O / d->groups, K = d->K;
  if (type == 1) { *rows = (int64_t)d->N * Hout * Wout; *cols = (int64_t)Cg * K * K; *rcols = Og; }
  if (type == 2) { *rows = (int64_t)d->N * d->H * Wout; *cols = (int64_t)Cg * K;     *rcols = (int64_t)Og * K; }
  if (type == 3) { *rows = (int64_t)d->N * d->H * d->W; *cols = Cg;                  *rcols = (int64_t)Og * K * K; }
  return 0;
}

static float x_or_zero(const oracle_dims_t* d, const float* x, int n, int cglob, int h, int w) {
  if (h < 0 || h >= d->H || w < 0 || w >= d->W) return 0.0f;
  return x[(((int64_t)n * d->C + cglob) * d->H + h) * d->W + w];
}

/* Lowering phase for the data: dhat has groups * rows * cols floats. */
int oracle_lower_data(const oracle_dims_t* d, int type, const float* x, float* dhat) {
  int64_t rows, cols, rcols;
  if (oracle_lowered_shape(d, type, &rows, &cols, &rcols) || !x || !dhat) return -1;
  const int Hout = out_dim(d->H, d->K, d->stride, d->pad);
  const int Wout = out_dim(d->W, d->K, d->stride, d->pad);
  const int Cg = d->C / d->groups, K = d->K, s = d->stride, p = d->pad;
  for (int q = 0; q < d->groups; ++q) {
    float* m = dhat + (int64_t)q * rows * cols;
    if (type == 1) {
      for (int n = 0; n < d->N; ++n)
        for (int r = 0; r < Hout; ++r)
          for (int c = 0; c < Wout; ++c) {
            float* row = m + (((int64_t)n * Hout + r) * Wout + c) * cols;
            for (int ci = 0; ci < Cg; ++ci)
              for (int i = 0; i < K; ++i)
                for (int j = 0; j < K; ++j)
                  row[((int64_t)ci * K + i) * K + j] =
                      x_or_zero(d, x, n, q * Cg + ci, r * s + i - p, c * s + j - p);
          }
    } else if (type == 2) {
      for (int n = 0; n < d->N; ++n)
        for (int h = 0; h < d->H; ++h)
          for (int c = 0; c < Wout; ++c) {
            float* row = m + (((int64_t)n * d->H + h) * Wout + c) * cols;
            for (int ci = 0; ci < Cg; ++ci)
              for (int j = 0; j < K; ++j)
                row[(int64_t)ci * K + j] = x_or_zero(d, x, n, q * Cg + ci, h, c * s + j - p);
          }
    } else {
      for (int n = 0; n < d->N; ++n)
        for (int h = 0; h < d->H; ++h)
          for (int w = 0; w < d->W; ++w) {
            float* row = m + (((int64_t)n * d->H + h) * d->W + w) * cols;
            for (int ci = 0; ci < Cg; ++ci) row[ci] = x_or_zero(d, x, n, q * Cg + ci, h, w);
          }
    }
  }
  return 0;
}

/* Lowering phase for the kernels: khat has groups * cols * rcols floats. */
int oracle_lower_kernel(const oracle_dims_t* d, int type, const float* w, float* khat) {
  int64_t rows, cols, rcols;
  if (oracle_lowered_shape(d, type, &rows, &cols, &rcols) || !w || !khat) return -1;
  const int Cg = d->C / d->groups, Og = d->O / d->groups, K = d->K;
  for (int q = 0; q < d->groups; ++q) {
    float* m = khat + (int64_t)q * cols * rcols;
    for (int oo = 0; oo < Og; ++oo)
      for (int ci = 0; ci < Cg; ++ci)
        for (int i = 0; i < K; ++i)
          for (int j = 0; j < K; ++j) {
            const float v = w[((((int64_t)q * Og + oo) * Cg + ci) * K + i) * K + j];
            int64_t kr, kc;
            if (type == 1)      { kr = ((int64_t)ci * K + i) * K + j; kc = oo; }
            else if (type == 2) { kr = (int64_t)ci * K + j;           kc = (int64_t)oo * K + i; }
            else                { kr = ci;                            kc = ((int64_t)oo * K + i) * K + j; }
            m[kr * rcols + kc] = v;
          }
  }
  return 0;
}

/* Multiply phase: rhat[q] = dhat[q] (rows x cols) * khat[q] (cols x rcols), fp64. */
int oracle_multiply(const oracle_dims_t* d, int type, const float* dhat, const float* khat,
                    double* rhat) {
  int64_t rows, cols, rcols;
  if (oracle_lowered_shape(d, type, &rows, &cols, &rcols) || !dhat || !khat || !rhat) return -1;
  for (int q = 0; q < d->groups; ++q) {
    const float* A = dhat + (int64_t)q * rows * cols;
    const float* B = khat + (int64_t)q * cols * rcols;
    double* R = rhat + (int64_t)q * rows * rcols;
#pragma omp parallel for schedule(static)
    for (int64_t a = 0; a < rows; ++a)
      for (int64_t b = 0; b < rcols; ++b) {
        double acc = 0.0;
        for (int64_t t = 0; t < cols; ++t) acc += (double)A[a * cols + t] * (double)B[t * rcols + b];
        R[a * rcols + b] = acc;
      }
  }
  return 0;
}

/* Lifting phase (+ bias): rhat -> y (N x O x Hout x Wout, fp64). */
int oracle_lift(const oracle_dims_t* d, int type, const double* rhat, const float* bias, double* y) {
  int64_t rows, cols, rcols;
  if (oracle_lowered_shape(d, type, &rows, &cols, &rcols) || !rhat || !y) return -1;
  const int Hout = out_dim(d->H, d->K, d->stride, d->pad);
  const int Wout = out_dim(d->W, d->K, d->stride, d->pad);
  const int Og = d->O / d->groups, K = d->K, s = d->stride, p = d->pad;
  for (int n = 0; n < d->N; ++n)
    for (int o = 0; o < d->O; ++o) {
      const int q = o / Og, oo = o % Og;
      const double* R = rhat + (int64_t)q * rows * rcols;
      for (int r = 0; r < Hout; ++r)
        for (int c = 0; c < Wout; ++c) {
          double acc = bias ? (double)bias[o] : 0.0;
          if (type == 1) {
            acc += R[(((int64_t)n * Hout + r) * Wout + c) * rcols + oo];
          } else if (type == 2) {
            for (int i = 0; i < K; ++i) {
              const int h = r * s + i - p;
              if (h < 0 || h >= d->H) continue;
              acc += R[(((int64_t)n * d->H + h) * Wout + c) * rcols + (int64_t)oo * K + i];
            }
          } else {
            for (int i = 0; i < K; ++i) {
              const int h = r * s + i - p;
              if (h < 0 || h >= d->H) continue;
              for (int j = 0; j < K; ++j) {
                const int w = c * s + j - p;
                if (w < 0 || w >= d->W) continue;
                acc += R[(((int64_t)n * d->H + h) * d->W + w) * rcols + ((int64_t)oo * K + i) * K + j];
              }
            }
          }
          y[(((int64_t)n * d->O + o) * Hout + r) * Wout + c] = acc;
        }
    }
  return 0;
}
