// The layers between CaffeNet's convolutional layers, as library entry points: the rectified
// linear unit, max pooling and local response normalisation, forward and backward (Sec. 1: the other layers are built with the
// same techniques as the convolution and match Caffe layer by layer; Sec. 2.2: processing the
// whole batch at once applies to every layer).  All are pure streaming kernels: every element of
// the input is read once and every element of the output written once, the whole batch in one
// launch.  Semantics are Caffe's:
//   ReLU      y = max(x, 0);  dx = dy where x > 0, else 0.
//   LRN       across channels: scale = k + (alpha/size) * sum of x^2 over the `size` channels
//             centred on the channel (zero padded), y = x * scale^(-beta); backward is the exact
//             derivative.  A thread owns one pixel of one image and walks a segment of its
//             channels (all of them when the batch has enough pixels to fill the chip), keeping
//             the window in registers: x (and dy) are read once, apart from the few channels
//             around a segment's ends, and y (dx) is written once.
//   dropout   y = x * scale where the caller's mask is set, else 0 (both directions).
//   softmax loss  softmax over the classes of each image, mean negative log-likelihood of the
//             labels; backward (prob - onehot) / N.  One workgroup per image, fixed-order sums.
//   max pool  K x K windows with stride s and padding p, clipped to the image, output size
//             ceil((H + 2p - K)/s) + 1 (minus one if the last window would start beyond the
//             image); the FIRST maximum in row-major order of the window is the one that
//             receives the gradient.  The backward pass is a gather (no atomics): a pixel sums
//             dy over the at most ceil(K/s)^2 windows that contain it and chose it.
#include "cct_internal.h"
#include "index_common.h"

namespace cct {
namespace {


__global__ __launch_bounds__(TPB) void relu_forward_kernel(const float* __restrict__ x,
                                                           float* __restrict__ y, long long n4,
                                                           long long n) {
  const long long stride = (long long)gridDim.x * TPB;
  for (long long i = (long long)blockIdx.x * TPB + threadIdx.x; i < n4; i += stride) {
    float4 v = reinterpret_cast<const float4*>(x)[i];
    v.x = v.x > 0.f ? v.x : 0.f;
    v.y = v.y > 0.f ? v.y : 0.f;
    v.z = v.z > 0.f ? v.z : 0.f;
    v.w = v.w > 0.f ? v.w : 0.f;
    reinterpret_cast<float4*>(y)[i] = v;
  }
  // tail (and everything, when the pointers are not 16-byte aligned: then n4 == 0)
  for (long long i = n4 * 4 + (long long)blockIdx.x * TPB + threadIdx.x; i < n; i += stride) {
    const float v = x[i];
    y[i] = v > 0.f ? v : 0.f;
  }
}

__global__ __launch_bounds__(TPB) void relu_backward_kernel(const float* __restrict__ x,
                                                            const float* __restrict__ dy,
                                                            float* __restrict__ dx, long long n4,
                                                            long long n) {
  const long long stride = (long long)gridDim.x * TPB;
  for (long long i = (long long)blockIdx.x * TPB + threadIdx.x; i < n4; i += stride) {
    const float4 v = reinterpret_cast<const float4*>(x)[i];
    float4 g = reinterpret_cast<const float4*>(dy)[i];
    g.x = v.x > 0.f ? g.x : 0.f;
    g.y = v.y > 0.f ? g.y : 0.f;
    g.z = v.z > 0.f ? g.z : 0.f;
    g.w = v.w > 0.f ? g.w : 0.f;
    reinterpret_cast<float4*>(dx)[i] = g;
  }
  for (long long i = n4 * 4 + (long long)blockIdx.x * TPB + threadIdx.x; i < n; i += stride)
    dx[i] = x[i] > 0.f ? dy[i] : 0.f;
}

struct PoolGeom {
  int H, W, K, s, p, Ho, Wo;
};

// one thread per output element, consecutive threads along the output row
__global__ __launch_bounds__(TPB) void maxpool_forward_kernel(const float* __restrict__ x,
                                                              float* __restrict__ y,
                                                              int* __restrict__ argmax,
                                                              long long total, PoolGeom g) {
  const long long t = (long long)blockIdx.x * TPB + threadIdx.x;
  if (t >= total) return;
  const int q = (int)(t % g.Wo);
  const long long u = t / g.Wo;
  const int r = (int)(u % g.Ho);
  const long long plane = u / g.Ho;
  const float* __restrict__ xp = x + plane * g.H * g.W;
  const int h0 = max(r * g.s - g.p, 0), w0 = max(q * g.s - g.p, 0);
  const int h1 = min(r * g.s - g.p + g.K, g.H), w1 = min(q * g.s - g.p + g.K, g.W);
  int best = -1;
  float bv = 0.f;
  for (int h = h0; h < h1; ++h)
    for (int w = w0; w < w1; ++w) {
      const float v = xp[h * g.W + w];
      if (best < 0 || v > bv) {
        bv = v;
        best = h * g.W + w;
      }
    }
  y[t] = bv;
  if (argmax) argmax[t] = best;
}

// one thread per input pixel: windows (r, q) with r*s - p <= h < r*s - p + K (same for w)
__global__ __launch_bounds__(TPB) void maxpool_backward_kernel(const float* __restrict__ dy,
                                                               const int* __restrict__ argmax,
                                                               float* __restrict__ dx,
                                                               long long total, PoolGeom g) {
  const long long t = (long long)blockIdx.x * TPB + threadIdx.x;
  if (t >= total) return;
  const int w = (int)(t % g.W);
  const long long u = t / g.W;
  const int h = (int)(u % g.H);
  const long long plane = u / g.H;
  const int me = h * g.W + w;
  const int rlo = h + g.p - g.K + 1 <= 0 ? 0 : (h + g.p - g.K + g.s) / g.s;   // ceil((h+p-K+1)/s)
  const int qlo = w + g.p - g.K + 1 <= 0 ? 0 : (w + g.p - g.K + g.s) / g.s;
  const int rhi = min((h + g.p) / g.s, g.Ho - 1), qhi = min((w + g.p) / g.s, g.Wo - 1);
  const long long base = plane * g.Ho * g.Wo;
  float acc = 0.f;
  for (int r = rlo; r <= rhi; ++r)
    for (int q = qlo; q <= qhi; ++q) {
      const long long o = base + (long long)r * g.Wo + q;
      if (argmax[o] == me) acc += dy[o];
    }
  dx[t] = acc;
}

// The same gather with the output planes staged in LDS: a workgroup owns `np` consecutive
// (image, channel) planes, copies their dy and argmax (np*Ho*Wo values each, contiguous in memory)
// into LDS with coalesced loads and then walks the np*H*W input pixels, which gather from LDS in
// the same window order.  dy and argmax are read from memory once, and all index arithmetic is
// 32-bit with multiplicative division.
__global__ __launch_bounds__(TPB) void maxpool_backward_lds_kernel(
    const float* __restrict__ dy, const int* __restrict__ argmax, float* __restrict__ dx,
    long long planes, int np, PoolGeom g, FastDiv divP, FastDiv divW, FastDiv divS) {
  extern __shared__ float pool_smem[];
  const int Po = g.Ho * g.Wo, P = g.H * g.W;
  const long long pl0 = (long long)blockIdx.x * np;
  const int n_here = (int)min((long long)np, planes - pl0);
  float* sdy = pool_smem;
  int* sarg = reinterpret_cast<int*>(pool_smem + np * Po);
  const float* __restrict__ dyp = dy + pl0 * Po;
  const int* __restrict__ ap = argmax + pl0 * Po;
  for (int i = threadIdx.x; i < n_here * Po; i += TPB) {
    sdy[i] = dyp[i];
    sarg[i] = ap[i];
  }
  __syncthreads();
  float* __restrict__ dxp = dx + pl0 * P;
  for (int i = threadIdx.x; i < n_here * P; i += TPB) {
    const int pl = fdiv(i, divP), me = i - pl * P;
    const int h = fdiv(me, divW), w = me - h * g.W;
    const int rlo = h + g.p - g.K + 1 <= 0 ? 0 : fdiv(h + g.p - g.K + g.s, divS);
    const int qlo = w + g.p - g.K + 1 <= 0 ? 0 : fdiv(w + g.p - g.K + g.s, divS);
    const int rhi = min(fdiv(h + g.p, divS), g.Ho - 1), qhi = min(fdiv(w + g.p, divS), g.Wo - 1);
    const int ob = pl * Po;
    float acc = 0.f;
    for (int r = rlo; r <= rhi; ++r)
      for (int q = qlo; q <= qhi; ++q) {
        const int o = ob + r * g.Wo + q;
        if (sarg[o] == me) acc += sdy[o];
      }
    dxp[i] = acc;
  }
}

bool pool_geom(const cct_pool_desc_t* d, PoolGeom* g) {
  if (!d || d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->K <= 0 || d->stride <= 0 ||
      d->pad < 0 || d->pad >= d->K)
    return false;
  auto out = [&](int in) {
    const long long t = std::max<long long>((long long)in + 2LL * d->pad - d->K, 0);
    long long o = (t + d->stride - 1) / d->stride + 1;
    if (d->pad > 0 && (o - 1) * d->stride >= (long long)in + d->pad) --o;
    return o;
  };
  const long long ho = out(d->H), wo = out(d->W);
  if ((long long)d->H * d->W >= 2147483647LL || ho >= 2147483647LL || wo >= 2147483647LL) return false;
  *g = PoolGeom{d->H, d->W, d->K, d->stride, d->pad, (int)ho, (int)wo};
  return true;
}

inline long long vec4_count(const void* a, const void* b, const void* c, long long n) {
  const uintptr_t bits = reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) |
                         reinterpret_cast<uintptr_t>(c);
  return bits % 16 == 0 ? n / 4 : 0;
}

inline unsigned stream_blocks(long long work_items) {
  // enough workgroups to fill the chip several times over; the kernels loop (ReLU) or are
  // launched with one thread per element (pooling)
  const long long want = (work_items + TPB - 1) / TPB;
  return (unsigned)std::max<long long>(1, std::min<long long>(want, 256LL * 64));
}


// ---- local response normalisation -------------------------------------------------------------
struct LrnGeom {
  int C;
  int cs;  // channels per thread: blockIdx.y selects the segment [y*cs, min(C, (y+1)*cs))
  long long hw, pixels;  // H*W, N*H*W
  float a, beta, k, coef;  // alpha/size; 2*alpha*beta/size
};

constexpr long long kLrnThreads = 1 << 20;
constexpr int kLrnMinSeg = 8;

template <int SIZE>
__global__ __launch_bounds__(TPB) void lrn_forward_kernel(const float* __restrict__ x,
                                                          float* __restrict__ y, LrnGeom g) {
  constexpr int HALF = (SIZE - 1) / 2;
  const long long t = (long long)blockIdx.x * TPB + threadIdx.x;
  if (t >= g.pixels) return;
  const long long n = t / g.hw, pix = t - n * g.hw;
  const float* xp = x + n * g.C * g.hw + pix;  // channel c of this pixel is xp[c*hw]
  float* yp = y + n * g.C * g.hw + pix;
  const int c0 = blockIdx.y * g.cs, c1 = min(g.C, c0 + g.cs);
  float xs[SIZE];  // x of channels c-HALF .. c+HALF
#pragma unroll
  for (int i = 0; i < SIZE; ++i) {
    const int ch = c0 + i - HALF;
    xs[i] = (ch >= 0 && ch < g.C) ? xp[ch * g.hw] : 0.f;
  }
  for (int c = c0; c < c1; ++c) {
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < SIZE; ++i) sum += xs[i] * xs[i];
    yp[c * g.hw] = xs[HALF] * powf(g.k + g.a * sum, -g.beta);
#pragma unroll
    for (int i = 0; i + 1 < SIZE; ++i) xs[i] = xs[i + 1];
    const int nx = c + HALF + 1;
    xs[SIZE - 1] = nx < g.C ? xp[nx * g.hw] : 0.f;
  }
}

// dx[c] = dy[c]*scale[c]^-beta - coef * x[c] * sum_{|c'-c| <= HALF} dy[c'] x[c'] scale[c']^(-beta-1).
// Iteration j computes the terms of channel j and emits channel j - HALF, whose window is then
// complete; a thread that owns channels c0 .. c1-1 therefore runs j over c0-HALF .. c1-1+HALF.
template <int SIZE>
__global__ __launch_bounds__(TPB) void lrn_backward_kernel(const float* __restrict__ x,
                                                           const float* __restrict__ dy,
                                                           float* __restrict__ dx, LrnGeom g) {
  constexpr int HALF = (SIZE - 1) / 2;
  const long long t = (long long)blockIdx.x * TPB + threadIdx.x;
  if (t >= g.pixels) return;
  const long long n = t / g.hw, pix = t - n * g.hw;
  const float* xp = x + n * g.C * g.hw + pix;
  const float* gp = dy + n * g.C * g.hw + pix;
  float* op = dx + n * g.C * g.hw + pix;
  const int c0 = blockIdx.y * g.cs, c1 = min(g.C, c0 + g.cs);
  float xs[SIZE];      // x of channels j-HALF .. j+HALF
  float tr[SIZE];      // cross terms of channels j-SIZE+1 .. j
  float ur[HALF + 1];  // direct terms dy*scale^-beta of channels j-HALF .. j
#pragma unroll
  for (int i = 0; i < SIZE; ++i) {
    const int ch = c0 - HALF + i - HALF;
    xs[i] = (ch >= 0 && ch < g.C) ? xp[ch * g.hw] : 0.f;
    tr[i] = 0.f;
  }
#pragma unroll
  for (int i = 0; i <= HALF; ++i) ur[i] = 0.f;
  for (int j = c0 - HALF; j < c1 + HALF; ++j) {
    // shift the term windows and append channel j
#pragma unroll
    for (int i = 0; i + 1 < SIZE; ++i) tr[i] = tr[i + 1];
#pragma unroll
    for (int i = 0; i < HALF; ++i) ur[i] = ur[i + 1];
    float tj = 0.f, uj = 0.f;
    if (j >= 0 && j < g.C) {
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < SIZE; ++i) sum += xs[i] * xs[i];
      const float scale = g.k + g.a * sum;
      const float pw = powf(scale, -g.beta);
      const float gj = gp[j * g.hw];
      uj = gj * pw;
      tj = gj * xs[HALF] * pw / scale;
    }
    tr[SIZE - 1] = tj;
    ur[HALF] = uj;
    const int c = j - HALF;
    if (c >= c0) {
      float cross = 0.f;
#pragma unroll
      for (int i = 0; i < SIZE; ++i) cross += tr[i];
      op[c * g.hw] = ur[0] - g.coef * xs[0] * cross;  // xs[0] = x of channel j - HALF
    }
#pragma unroll
    for (int i = 0; i + 1 < SIZE; ++i) xs[i] = xs[i + 1];
    const int nx = j + HALF + 1;
    xs[SIZE - 1] = (nx >= 0 && nx < g.C) ? xp[nx * g.hw] : 0.f;
  }
}

bool lrn_geom(const cct_lrn_desc_t* d, LrnGeom* g) {
  if (!d || d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0) return false;
  if (d->size < 1 || !(d->size & 1) || !(d->k > 0.f) || !(d->alpha >= 0.f)) return false;
  g->C = d->C;
  g->hw = (long long)d->H * d->W;
  g->pixels = g->hw * d->N;
  g->a = d->alpha / (float)d->size;
  g->beta = d->beta;
  g->k = d->k;
  g->coef = 2.0f * d->alpha * d->beta / (float)d->size;
  return true;
}

template <int SIZE>
void launch_lrn(bool backward, const float* x, const float* dy, float* out, const LrnGeom& g,
                dim3 grid, hipStream_t st) {
  if (backward)
    hipLaunchKernelGGL(lrn_backward_kernel<SIZE>, grid, dim3(TPB), 0, st, x, dy, out, g);
  else
    hipLaunchKernelGGL(lrn_forward_kernel<SIZE>, grid, dim3(TPB), 0, st, x, out, g);
}

int run_lrn(const cct_lrn_desc_t* desc, bool backward, const float* x, const float* dy, float* out,
            hipStream_t st) {
  LrnGeom g;
  if (!lrn_geom(desc, &g) || !x || !out || (backward && !dy)) return CCT_EINVAL;
  const long long blocks = (g.pixels + TPB - 1) / TPB;
  if (blocks >= 2147483647LL) return CCT_EUNSUPPORTED;
  const double elems = (double)g.pixels * g.C;
  ProfScope ps(backward ? "lrn_backward_kernel" : "lrn_forward_kernel", 0.0,
               (backward ? 12.0 : 8.0) * elems, st);
  // A thread walks a segment of the channels of its pixel.  With few pixels (CaffeNet's norm2 has
  // 43 264 at batch 256) one thread per pixel leaves most of the chip idle, so the channels are cut
  // into segments of at least kLrnMinSeg until about kLrnThreads threads exist; a segment re-reads
  // the size-1 (backward: 2*(size-1)) neighbouring channels of its ends.
  const long long want = (kLrnThreads + g.pixels - 1) / g.pixels;
  const long long nseg0 = std::max<long long>(1, std::min<long long>(want, g.C / kLrnMinSeg));
  g.cs = (int)((g.C + nseg0 - 1) / nseg0);
  const unsigned nseg = (unsigned)((g.C + g.cs - 1) / g.cs);
  if (nseg > 65535) return CCT_EUNSUPPORTED;
  const dim3 grid((unsigned)blocks, nseg);
  switch (desc->size) {
    case 1: launch_lrn<1>(backward, x, dy, out, g, grid, st); break;
    case 3: launch_lrn<3>(backward, x, dy, out, g, grid, st); break;
    case 5: launch_lrn<5>(backward, x, dy, out, g, grid, st); break;
    case 7: launch_lrn<7>(backward, x, dy, out, g, grid, st); break;
    case 9: launch_lrn<9>(backward, x, dy, out, g, grid, st); break;
    default: return CCT_EUNSUPPORTED;  // window sizes are compiled in: 1, 3, 5, 7, 9
  }
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

// Dropout with the caller's mask: y = x * scale where mask != 0, else 0 (both directions).
__global__ __launch_bounds__(TPB) void dropout_kernel(const float* __restrict__ x,
                                                      const unsigned char* __restrict__ mask,
                                                      float scale, float* __restrict__ y,
                                                      long long n) {
  const long long stride = (long long)gridDim.x * TPB;
  for (long long i = (long long)blockIdx.x * TPB + threadIdx.x; i < n; i += stride)
    y[i] = mask[i] ? x[i] * scale : 0.f;
}

// Combines one value per thread over the workgroup, always in the same order: lanes by
// shuffles, the four waves through LDS.  Every thread gets the result.
template <bool MAX>
__device__ __forceinline__ float block_combine(float v, float* red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float o = __shfl_xor(v, off, 64);
    v = MAX ? fmaxf(v, o) : v + o;
  }
  __syncthreads();   // red may still be read from an earlier call
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  const float a = red[0], b = red[1], c = red[2], d = red[3];
  return MAX ? fmaxf(fmaxf(a, b), fmaxf(c, d)) : (a + b) + (c + d);
}

// Softmax over the C scores of image blockIdx.x and its loss term
// -(x[label] - max - log(sum exp(x - max))); NaN for a label outside [0, C).
__global__ __launch_bounds__(TPB) void softmax_loss_forward_kernel(const float* __restrict__ x,
                                                                   const int* __restrict__ label,
                                                                   float* __restrict__ prob,
                                                                   float* __restrict__ image_loss,
                                                                   int C) {
  __shared__ float red[4];
  const float* xr = x + (long long)blockIdx.x * C;
  float* pr = prob + (long long)blockIdx.x * C;
  float mx = -__builtin_inff();
  for (int c = threadIdx.x; c < C; c += TPB) mx = fmaxf(mx, xr[c]);
  mx = block_combine<true>(mx, red);
  float sum = 0.f;
  for (int c = threadIdx.x; c < C; c += TPB) sum += expf(xr[c] - mx);
  sum = block_combine<false>(sum, red);
  const float inv = 1.0f / sum;
  for (int c = threadIdx.x; c < C; c += TPB) pr[c] = expf(xr[c] - mx) * inv;
  if (threadIdx.x == 0) {
    const int l = label[blockIdx.x];
    image_loss[blockIdx.x] =
        (l >= 0 && l < C) ? -(xr[l] - mx - logf(sum)) : __builtin_nanf("");
  }
}

// loss = (1/N) * sum of the per-image terms, added in a fixed order by one workgroup.
__global__ __launch_bounds__(TPB) void mean_kernel(const float* __restrict__ v,
                                                   float* __restrict__ out, int N) {
  __shared__ float red[4];
  float acc = 0.f;
  for (int i = threadIdx.x; i < N; i += TPB) acc += v[i];
  acc = block_combine<false>(acc, red);
  if (threadIdx.x == 0) out[0] = acc / (float)N;
}

__global__ __launch_bounds__(TPB) void softmax_loss_backward_kernel(const float* __restrict__ prob,
                                                                    const int* __restrict__ label,
                                                                    float* __restrict__ dx,
                                                                    long long total, FastDiv divC,
                                                                    float inv_n) {
  const long long t = (long long)blockIdx.x * TPB + threadIdx.x;
  if (t >= total) return;
  const int n = fdiv((int)t, divC), c = (int)t - n * divC.d;
  dx[t] = (prob[t] - (c == label[n] ? 1.f : 0.f)) * inv_n;
}

int run_dropout(const float* x, const unsigned char* mask, float scale, float* y, long long n,
                hipStream_t st) {
  if (!x || !mask || !y || n < 0 || !(scale > 0.f)) return CCT_EINVAL;
  if (n == 0) return CCT_OK;
  const long long blocks = std::min<long long>((n + TPB - 1) / TPB, 1 << 16);
  ProfScope ps("dropout_kernel", 0.0, 9.0 * (double)n, st);
  hipLaunchKernelGGL(dropout_kernel, dim3((unsigned)blocks), dim3(TPB), 0, st, x, mask, scale, y, n);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

}  // namespace
}  // namespace cct

using namespace cct;

extern "C" {

int cct_relu_forward(const float* x, float* y, int64_t n, void* hip_stream) {
  if (!x || !y || n < 0) return CCT_EINVAL;
  if (n == 0) return CCT_OK;
  hipStream_t st = (hipStream_t)hip_stream;
  const long long n4 = vec4_count(x, y, nullptr, n);
  ProfScope ps("relu_forward_kernel", 0.0, 8.0 * (double)n, st);
  hipLaunchKernelGGL(relu_forward_kernel, dim3(stream_blocks(n4 ? n4 : n)), dim3(TPB), 0, st, x, y,
                     n4, (long long)n);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int cct_relu_backward(const float* x, const float* dy, float* dx, int64_t n, void* hip_stream) {
  if (!x || !dy || !dx || n < 0) return CCT_EINVAL;
  if (n == 0) return CCT_OK;
  hipStream_t st = (hipStream_t)hip_stream;
  const long long n4 = vec4_count(x, dy, dx, n);
  ProfScope ps("relu_backward_kernel", 0.0, 12.0 * (double)n, st);
  hipLaunchKernelGGL(relu_backward_kernel, dim3(stream_blocks(n4 ? n4 : n)), dim3(TPB), 0, st, x,
                     dy, dx, n4, (long long)n);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int cct_pool_output_dims(const cct_pool_desc_t* desc, int32_t* Hout, int32_t* Wout) {
  PoolGeom g;
  if (!Hout || !Wout || !pool_geom(desc, &g)) return CCT_EINVAL;
  *Hout = g.Ho;
  *Wout = g.Wo;
  return CCT_OK;
}

int cct_maxpool_forward(const cct_pool_desc_t* desc, const float* x, float* y, int32_t* argmax,
                        void* hip_stream) {
  PoolGeom g;
  if (!pool_geom(desc, &g) || !x || !y) return CCT_EINVAL;
  const long long total = (long long)desc->N * desc->C * g.Ho * g.Wo;
  const long long blocks = (total + TPB - 1) / TPB;
  if (blocks >= 2147483647LL) return CCT_EUNSUPPORTED;
  hipStream_t st = (hipStream_t)hip_stream;
  ProfScope ps("maxpool_forward_kernel", 0.0,
               4.0 * (double)desc->N * desc->C * g.H * g.W + (argmax ? 8.0 : 4.0) * (double)total, st);
  hipLaunchKernelGGL(maxpool_forward_kernel, dim3((unsigned)blocks), dim3(TPB), 0, st, x, y, argmax,
                     total, g);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int cct_maxpool_backward(const cct_pool_desc_t* desc, const float* dy, const int32_t* argmax,
                         float* dx, void* hip_stream) {
  PoolGeom g;
  if (!pool_geom(desc, &g) || !dy || !argmax || !dx) return CCT_EINVAL;
  const long long total = (long long)desc->N * desc->C * g.H * g.W;
  const long long blocks = (total + TPB - 1) / TPB;
  if (blocks >= 2147483647LL) return CCT_EUNSUPPORTED;
  hipStream_t st = (hipStream_t)hip_stream;
  ProfScope ps("maxpool_backward_kernel", 0.0,
               4.0 * (double)total + 8.0 * (double)desc->N * desc->C * g.Ho * g.Wo, st);
  // planes whose dy and argmax fit 64 KiB of LDS: about 4096 input pixels per workgroup
  const long long P = (long long)g.H * g.W, Po = (long long)g.Ho * g.Wo;
  const long long planes = (long long)desc->N * desc->C;
  if (Po * 8 <= 65536 && P <= 65536) {
    long long np = std::max<long long>(1, 4096 / P);
    np = std::min({np, 65536 / (Po * 8), planes});
    const long long wgs = (planes + np - 1) / np;
    if (wgs >= 2147483647LL) return CCT_EUNSUPPORTED;
    hipLaunchKernelGGL(maxpool_backward_lds_kernel, dim3((unsigned)wgs), dim3(TPB),
                       (size_t)(np * Po * 8), st, dy, argmax, dx, planes, (int)np, g,
                       make_fastdiv((int)P), make_fastdiv(g.W), make_fastdiv(g.s));
    CCT_CHECK_LAUNCH();
    return CCT_OK;
  }
  hipLaunchKernelGGL(maxpool_backward_kernel, dim3((unsigned)blocks), dim3(TPB), 0, st, dy, argmax,
                     dx, total, g);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int cct_lrn_forward(const cct_lrn_desc_t* desc, const float* x, float* y, void* hip_stream) {
  return run_lrn(desc, false, x, nullptr, y, (hipStream_t)hip_stream);
}

int cct_lrn_backward(const cct_lrn_desc_t* desc, const float* x, const float* dy, float* dx,
                     void* hip_stream) {
  return run_lrn(desc, true, x, dy, dx, (hipStream_t)hip_stream);
}

int cct_dropout_forward(const float* x, const uint8_t* mask, float scale, float* y, int64_t n,
                        void* hip_stream) {
  return run_dropout(x, mask, scale, y, n, (hipStream_t)hip_stream);
}

int cct_dropout_backward(const float* dy, const uint8_t* mask, float scale, float* dx, int64_t n,
                         void* hip_stream) {
  return run_dropout(dy, mask, scale, dx, n, (hipStream_t)hip_stream);
}

int cct_softmax_loss_forward(int32_t N, int32_t C, const float* x, const int32_t* label, float* prob,
                             float* image_loss, float* loss, void* hip_stream) {
  if (N <= 0 || C <= 0 || !x || !label || !prob || !image_loss || !loss) return CCT_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  ProfScope ps("softmax_loss_forward_kernel", 0.0, 8.0 * (double)N * C, st);
  hipLaunchKernelGGL(softmax_loss_forward_kernel, dim3((unsigned)N), dim3(TPB), 0, st, x, label, prob,
                     image_loss, C);
  CCT_CHECK_LAUNCH();
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(TPB), 0, st, image_loss, loss, N);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int cct_softmax_loss_backward(int32_t N, int32_t C, const float* prob, const int32_t* label,
                              float* dx, void* hip_stream) {
  if (N <= 0 || C <= 0 || !prob || !label || !dx) return CCT_EINVAL;
  const long long total = (long long)N * C;
  if (total >= 2147483647LL) return CCT_EUNSUPPORTED;
  hipStream_t st = (hipStream_t)hip_stream;
  ProfScope ps("softmax_loss_backward_kernel", 0.0, 8.0 * (double)total, st);
  hipLaunchKernelGGL(softmax_loss_backward_kernel, dim3((unsigned)((total + TPB - 1) / TPB)), dim3(TPB),
                     0, st, prob, label, dx, total, make_fastdiv(C), 1.0f / (float)N);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

}  // extern "C"
