// The two layers between CaffeNet's convolutional layers, as library entry points: the rectified
// linear unit and max pooling, forward and backward (Sec. 1: the other layers are built with the
// same techniques as the convolution and match Caffe layer by layer; Sec. 2.2: processing the
// whole batch at once applies to every layer).  Both are pure streaming kernels: every element of
// the input is read once and every element of the output written once, the whole batch in one
// launch.  Semantics are Caffe's:
//   ReLU      y = max(x, 0);  dx = dy where x > 0, else 0.
//   max pool  K x K windows with stride s and padding p, clipped to the image, output size
//             ceil((H + 2p - K)/s) + 1 (minus one if the last window would start beyond the
//             image); the FIRST maximum in row-major order of the window is the one that
//             receives the gradient.  The backward pass is a gather (no atomics): a pixel sums
//             dy over the at most ceil(K/s)^2 windows that contain it and chose it.
#include "cct_internal.h"

namespace cct {
namespace {

constexpr int TPB = 256;

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
  hipLaunchKernelGGL(maxpool_backward_kernel, dim3((unsigned)blocks), dim3(TPB), 0, st, dy, argmax,
                     dx, total, g);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

}  // extern "C"
