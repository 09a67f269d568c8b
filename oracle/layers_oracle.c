/*
 * CPU oracle for the layers of CaffeNet other than the convolutions: the rectified linear unit,
 * max pooling, local response normalisation, dropout and the softmax loss.  TEST INFRASTRUCTURE ONLY: nothing in the product path may call
 * this file, and it shares no code with the GPU path.
 *
 * The paper names these layers only collectively (Sec. 1: all layers are optimised with the
 * same techniques, and every layer's output matches Caffe's); their definitions are Caffe's:
 *
 *   ReLU      y = max(x, 0);   dx = dy where x > 0, else 0  (the test on x and on y agree).
 *   max pool  y[n,c,r,q] = max over the K x K window whose top-left corner is
 *             (r*s - p, q*s - p), clipped to the image; output size
 *             ceil((H + 2p - K)/s) + 1, minus one if the last window would start beyond the
 *             image (only possible with padding).  The position of the maximum is the FIRST one
 *             in row-major scan order of the window (strict > when scanning); the backward pass
 *             routes dy[n,c,r,q] to that position and sums where windows overlap.
 *
 *   LRN       local response normalisation across channels (the layer after pool1 and pool2):
 *             scale[n,c,h,w] = k + (alpha/size) * sum of x[n,c',h,w]^2 over the `size` channels
 *             centred on c (size odd; channels outside [0,C) contribute nothing),
 *             y = x * scale^(-beta).  Backward is the exact derivative of that map:
 *             dx[c] = dy[c]*scale[c]^(-beta)
 *                     - (2*alpha*beta/size) * x[c] * sum over c' with |c'-c| <= (size-1)/2 of
 *                       dy[c'] * x[c'] * scale[c']^(-beta-1).
 *
 *   dropout   (after fc6 and fc7 while training) y = x * mask * scale, mask in {0, 1} per element and
 *             scale = 1 / (1 - ratio); backward dx = dy * mask * scale.  The random draw is the
 *             caller's: the mask is an input, so both sides of a parity test see the same one.
 *
 *   softmax loss  (the last layer) over the C scores of each of N images:
 *             prob[n,c] = exp(x[n,c] - max_c x[n,:]) / sum_c exp(x[n,c] - max_c x[n,:]),
 *             loss = -(1/N) * sum_n log prob[n, label[n]]   (taken as x[l] - max - log(sum), so a
 *             probability that underflows does not turn the loss into infinity),
 *             backward dx[n,c] = (prob[n,c] - [c == label[n]]) / N, from the fp32 prob the forward
 *             pass produced.
 *
 * Plain loops, one output at a time, exact (comparisons and copies of fp32 values; the backward
 * sum of the few overlapping windows is done in fp64); LRN, dropout's product and the softmax are
 * computed in fp64 and rounded once.
 *
 * Pins (tests/test_oracle_pins.py): values worked out by hand, the output-size law at CaffeNet's
 * 55 -> 27 and 27 -> 13, torch's CPU max_pool2d (ceil mode) and its autograd on tie-free data,
 * the tie rule on a constant image; for LRN a hand-worked three-channel case, the closed form on a
 * constant tensor (edge channels see fewer neighbours), size 1 = a pointwise power law, torch's CPU
 * local_response_norm and its autograd, and a finite-difference check of the backward pass; for
 * dropout the identity and zero masks, torch's CPU dropout (its output fixes the mask and the scale)
 * and the exact adjoint identity on dyadic data; for the softmax loss a hand-worked two-class case,
 * uniform scores (prob = 1/C, loss = log C), shift invariance, torch's CPU softmax / cross_entropy
 * and its autograd, and finite differences of the loss.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>

typedef struct {
  int N, C, H, W, K, stride, pad;
} oracle_pool_t;

static int pool_ok(const oracle_pool_t* d) {
  return d && d->N > 0 && d->C > 0 && d->H > 0 && d->W > 0 && d->K > 0 && d->stride > 0 &&
         d->pad >= 0 && d->pad < d->K;
}

static int pool_out(int in, int K, int s, int p) {
  int t = in + 2 * p - K;
  int o;
  if (t < 0) t = 0;
  o = (t + s - 1) / s + 1;
  if (p > 0 && (o - 1) * s >= in + p) --o;
  return o;
}

int oracle_pool_output_dims(const oracle_pool_t* d, int* Hout, int* Wout) {
  if (!pool_ok(d) || !Hout || !Wout) return -1;
  *Hout = pool_out(d->H, d->K, d->stride, d->pad);
  *Wout = pool_out(d->W, d->K, d->stride, d->pad);
  return 0;
}

int oracle_relu_forward(const float* x, float* y, int64_t n) {
  if (!x || !y || n < 0) return -1;
  for (int64_t i = 0; i < n; ++i) y[i] = x[i] > 0.0f ? x[i] : 0.0f;
  return 0;
}

int oracle_relu_backward(const float* x, const float* dy, float* dx, int64_t n) {
  if (!x || !dy || !dx || n < 0) return -1;
  for (int64_t i = 0; i < n; ++i) dx[i] = x[i] > 0.0f ? dy[i] : 0.0f;
  return 0;
}

/* y: N*C*Hout*Wout floats; argmax (nullable): index h*W + w of the chosen pixel in its plane. */
int oracle_maxpool_forward(const oracle_pool_t* d, const float* x, float* y, int32_t* argmax) {
  int Ho, Wo;
  if (oracle_pool_output_dims(d, &Ho, &Wo) || !x || !y) return -1;
  for (int64_t pl = 0; pl < (int64_t)d->N * d->C; ++pl) {
    const float* xp = x + pl * d->H * d->W;
    for (int r = 0; r < Ho; ++r)
      for (int q = 0; q < Wo; ++q) {
        int h0 = r * d->stride - d->pad, w0 = q * d->stride - d->pad;
        int h1 = h0 + d->K, w1 = w0 + d->K;
        int best = -1;
        float bv = 0.0f;
        if (h0 < 0) h0 = 0;
        if (w0 < 0) w0 = 0;
        if (h1 > d->H) h1 = d->H;
        if (w1 > d->W) w1 = d->W;
        for (int h = h0; h < h1; ++h)
          for (int w = w0; w < w1; ++w) {
            const float v = xp[h * d->W + w];
            if (best < 0 || v > bv) {
              bv = v;
              best = h * d->W + w;
            }
          }
        y[(pl * Ho + r) * Wo + q] = bv;
        if (argmax) argmax[(pl * Ho + r) * Wo + q] = best;
      }
  }
  return 0;
}

/* dx[n,c,h,w] = sum of dy over the windows whose argmax is (h,w): every window adds its dy to
 * the pixel it chose (fp64 accumulator per pixel, windows visited in row-major order). */
int oracle_maxpool_backward(const oracle_pool_t* d, const float* dy, const int32_t* argmax, float* dx) {
  int Ho, Wo;
  double* acc;
  if (oracle_pool_output_dims(d, &Ho, &Wo) || !dy || !argmax || !dx) return -1;
  acc = (double*)malloc(sizeof(double) * (size_t)d->H * d->W);
  if (!acc) return -1;
  for (int64_t pl = 0; pl < (int64_t)d->N * d->C; ++pl) {
    for (int t = 0; t < d->H * d->W; ++t) acc[t] = 0.0;
    for (int r = 0; r < Ho; ++r)
      for (int q = 0; q < Wo; ++q) {
        const int32_t a = argmax[(pl * Ho + r) * Wo + q];
        if (a < 0 || a >= d->H * d->W) {
          free(acc);
          return -1;
        }
        acc[a] += (double)dy[(pl * Ho + r) * Wo + q];
      }
    for (int t = 0; t < d->H * d->W; ++t) dx[pl * d->H * d->W + t] = (float)acc[t];
  }
  free(acc);
  return 0;
}

/* ---- local response normalisation across channels -------------------------------------- */
typedef struct {
  int N, C, H, W, size;
  double alpha, beta, k;
} oracle_lrn_t;

static int lrn_ok(const oracle_lrn_t* d) {
  return d && d->N > 0 && d->C > 0 && d->H > 0 && d->W > 0 && d->size > 0 && (d->size & 1) &&
         d->k > 0.0 && d->alpha >= 0.0;
}

static double lrn_scale(const oracle_lrn_t* d, const float* xp, int64_t hw, int c) {
  const int half = (d->size - 1) / 2;
  double s = 0.0;
  for (int cc = c - half; cc <= c + half; ++cc)
    if (cc >= 0 && cc < d->C) s += (double)xp[cc * hw] * (double)xp[cc * hw];
  return d->k + d->alpha / d->size * s;
}

int oracle_lrn_forward(const oracle_lrn_t* d, const float* x, float* y) {
  if (!lrn_ok(d) || !x || !y) return -1;
  const int64_t hw = (int64_t)d->H * d->W;
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < (int64_t)d->N * hw; ++t) {
    const int64_t n = t / hw, pix = t % hw;
    const float* xp = x + n * d->C * hw + pix; /* channel c of this pixel is xp[c*hw] */
    float* yp = y + n * d->C * hw + pix;
    for (int c = 0; c < d->C; ++c)
      yp[c * hw] = (float)((double)xp[c * hw] * pow(lrn_scale(d, xp, hw, c), -d->beta));
  }
  return 0;
}

int oracle_lrn_backward(const oracle_lrn_t* d, const float* x, const float* dy, float* dx) {
  if (!lrn_ok(d) || !x || !dy || !dx) return -1;
  const int64_t hw = (int64_t)d->H * d->W;
  const int half = (d->size - 1) / 2;
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < (int64_t)d->N * hw; ++t) {
    const int64_t n = t / hw, pix = t % hw;
    const float* xp = x + n * d->C * hw + pix;
    const float* gp = dy + n * d->C * hw + pix;
    float* op = dx + n * d->C * hw + pix;
    for (int c = 0; c < d->C; ++c) {
      double cross = 0.0;
      for (int cc = c - half; cc <= c + half; ++cc)
        if (cc >= 0 && cc < d->C)
          cross += (double)gp[cc * hw] * (double)xp[cc * hw] *
                   pow(lrn_scale(d, xp, hw, cc), -d->beta - 1.0);
      op[c * hw] = (float)((double)gp[c * hw] * pow(lrn_scale(d, xp, hw, c), -d->beta) -
                           2.0 * d->alpha * d->beta / d->size * (double)xp[c * hw] * cross);
    }
  }
  return 0;
}

int oracle_dropout(const float* x, const uint8_t* mask, double scale, float* y, int64_t n) {
  if (!x || !mask || !y || n < 0 || !(scale > 0.0)) return -1;
  for (int64_t i = 0; i < n; ++i) y[i] = mask[i] ? (float)((double)x[i] * scale) : 0.0f;
  return 0;
}

static int labels_ok(int N, int C, const int32_t* label) {
  for (int n = 0; n < N; ++n)
    if (label[n] < 0 || label[n] >= C) return 0;
  return 1;
}

int oracle_softmax_loss_forward(int N, int C, const float* x, const int32_t* label, float* prob,
                                double* loss) {
  if (N <= 0 || C <= 0 || !x || !label || !prob || !loss || !labels_ok(N, C, label)) return -1;
  double total = 0.0;
  for (int n = 0; n < N; ++n) {
    const float* xr = x + (int64_t)n * C;
    double mx = xr[0], sum = 0.0;
    for (int c = 1; c < C; ++c)
      if (xr[c] > mx) mx = xr[c];
    for (int c = 0; c < C; ++c) sum += exp((double)xr[c] - mx);
    for (int c = 0; c < C; ++c) prob[(int64_t)n * C + c] = (float)(exp((double)xr[c] - mx) / sum);
    total -= (double)xr[label[n]] - mx - log(sum);
  }
  *loss = total / N;
  return 0;
}

int oracle_softmax_loss_backward(int N, int C, const float* prob, const int32_t* label, float* dx) {
  if (N <= 0 || C <= 0 || !prob || !label || !dx || !labels_ok(N, C, label)) return -1;
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < C; ++c) {
      const int64_t i = (int64_t)n * C + c;
      dx[i] = (float)(((double)prob[i] - (c == label[n] ? 1.0 : 0.0)) / N);
    }
  return 0;
}
