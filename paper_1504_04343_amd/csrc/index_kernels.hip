// The lowered-kernel pack (K^, Sec. 2.1) and the small reductions of the backward-weights
// pass (split-K partial sums -> dw, dbias).
#include "cct_internal.h"
#include "index_common.h"

namespace cct {

static thread_local int g_last_hip_error = 0;
void set_hip_error(hipError_t e) { g_last_hip_error = (int)e; }
int last_hip_error_value() { return g_last_hip_error; }

namespace {

// ---------------------------------------------------------------------------------------
// Lowered kernel matrix K^ (Sec. 2.1), zero padded to the GEMM tile, optionally transposed.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ long long weight_index(const PackDesc& d, int q, int rho, int delta) {
  const int jR = rho % d.RKj;
  const int iR = (rho / d.RKj) % d.RKi;
  const int oo = rho / (d.RKj * d.RKi);
  const int jD = delta % d.DKj;
  const int iD = (delta / d.DKj) % d.DKi;
  const int ci = delta / (d.DKj * d.DKi);
  const int i = d.RKi > 1 ? iR : iD;
  const int j = d.RKj > 1 ? jR : jD;
  return ((((long long)q * d.Og + oo) * d.Cg + ci) * d.K + i) * d.K + j;
}

template <bool BF16>
__global__ __launch_bounds__(TPB) void pack_kernel(const float* __restrict__ w, void* __restrict__ pack,
                                                   PackDesc d) {
  const long long per_group = (long long)d.Mpad * d.Kpad;
  const long long t = (long long)blockIdx.x * TPB + threadIdx.x;
  if (t >= per_group * d.G) return;
  const int q = (int)(t / per_group);
  const long long e = t - q * per_group;
  const int k = (int)(e / d.Mpad), mm = (int)(e % d.Mpad);
  const int nrho = d.Og * d.RKi * d.RKj, ndelta = d.Cg * d.DKi * d.DKj;
  const int rho = d.transposed ? k : mm;
  const int delta = d.transposed ? mm : k;
  float v = 0.0f;
  if (rho < nrho && delta < ndelta) v = w[weight_index(d, q, rho, delta)];
  store_elem<BF16>(pack, t, v);
}

// Kernel matrix of the fused backward-data pass: the backward-data map of a stride-1 convolution
// is itself a convolution of dy with the kernels flipped in both axes and the channel roles
// swapped: pack[q][k = (oo, i', j')][m = ci] = w[q*Og + oo, ci, K-1-i', K-1-j'], zero padded.
__global__ __launch_bounds__(TPB) void pack_flipped_kernel(const float* __restrict__ w,
                                                           float* __restrict__ pack, int G, int Og,
                                                           int Cg, int K, int Mpad, int Kpad) {
  const long long per_group = (long long)Mpad * Kpad;
  const long long t = (long long)blockIdx.x * TPB + threadIdx.x;
  if (t >= per_group * G) return;
  const int q = (int)(t / per_group);
  const long long e = t - q * per_group;
  const int k = (int)(e / Mpad), ci = (int)(e % Mpad);
  float v = 0.0f;
  if (k < Og * K * K && ci < Cg) {
    const int j = k % K, i = (k / K) % K, oo = k / (K * K);
    v = w[((((long long)q * Og + oo) * Cg + ci) * K + (K - 1 - i)) * K + (K - 1 - j)];
  }
  pack[t] = v;
}

// Kernel matrix of the Type-2 backward-data pass when the GEMM gathers dR^ from dy itself:
// rows k = i'*Opad + oo (vertical tap i' = K-1-i first, so that a K tile has one tap), columns
// m = ci*K + j.
__global__ __launch_bounds__(TPB) void pack_type2_bwd_kernel(const float* __restrict__ w,
                                                             float* __restrict__ pack, int G, int Og,
                                                             int Cg, int K, int Opad, int Mpad) {
  const long long per_group = (long long)Mpad * K * Opad;
  const long long t = (long long)blockIdx.x * TPB + threadIdx.x;
  if (t >= per_group * G) return;
  const int q = (int)(t / per_group);
  const long long e = t - q * per_group;
  const int k = (int)(e / Mpad), m = (int)(e % Mpad);
  const int ip = k / Opad, oo = k - ip * Opad;
  const int ci = m / K, j = m - ci * K;
  float v = 0.0f;
  if (oo < Og && ci < Cg)
    v = w[((((long long)q * Og + oo) * Cg + ci) * K + (K - 1 - ip)) * K + j];
  pack[t] = v;
}

// dw = sum over split-K partials, mapped back to O x Cg x K x K.  A workgroup owns 64 outputs;
// its 4 thread groups each add up a quarter of the splits (in split order), and the four
// quarter sums are combined in a fixed order: the result is bit-reproducible run to run.
__global__ __launch_bounds__(TPB) void reduce_dw_kernel(const float* __restrict__ part,
                                                        float* __restrict__ dw, int S, PackDesc d,
                                                        int accumulate) {
  __shared__ float red[4][64];
  const int nrho = d.Og * d.RKi * d.RKj, ndelta = d.Cg * d.DKi * d.DKj;
  const long long per_group = (long long)nrho * ndelta;
  const long long total = per_group * d.G;
  const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const long long t = (long long)blockIdx.x * 64 + lane;
  const int per = (S + 3) / 4;
  const int s0 = slice * per, s1 = min(S, s0 + per);
  float acc = 0.0f;
  if (t < total) {
    const float* src = part + t;
    int sidx = s0;
    for (; sidx + 8 <= s1; sidx += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = src[(long long)(sidx + u) * total];
#pragma unroll
      for (int u = 0; u < 8; ++u) acc += v[u];
    }
    for (; sidx < s1; ++sidx) acc += src[(long long)sidx * total];
  }
  red[slice][lane] = acc;
  __syncthreads();
  if (slice == 0 && t < total) {
    const float sum = ((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane];
    const int q = (int)(t / per_group);
    const long long e = t - q * per_group;
    const int rho = (int)(e / ndelta), delta = (int)(e % ndelta);
    const long long wi = weight_index(d, q, rho, delta);
    dw[wi] = accumulate ? dw[wi] + sum : sum;
  }
}

// dbias, stage 1: block (o, blk) sums the planes dy[n, o, :, :] of the images n = blk, blk+nblk, ...
// Its threads walk the (image, pixel) pairs of those planes as one flat range, four independent
// partial sums per thread (loads of four iterations in flight), then combine: lanes by shuffles,
// the four waves through LDS, always in the same order.
__global__ __launch_bounds__(TPB) void dbias_stage1(const float* __restrict__ dy,
                                                    float* __restrict__ scratch, int N, int O, int P,
                                                    int nblk, FastDiv divP) {
  __shared__ float red[TPB / 64];
  const int o = blockIdx.x / nblk, blk = blockIdx.x % nblk;
  const int nimg = (N - blk + nblk - 1) / nblk;          // images of this block
  const long long total = (long long)nimg * P;
  const long long img_stride = (long long)nblk * O * P;
  const float* base = dy + ((long long)blk * O + o) * P;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  long long t = threadIdx.x;
  for (; t + 3 * TPB < total; t += 4 * TPB) {
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int e = (int)(t + u * TPB);
      const int i = fdiv(e, divP);
      v[u] = base[i * img_stride + (e - i * P)];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) acc[u] += v[u];
  }
  for (; t < total; t += TPB) {
    const int e = (int)t;
    const int i = fdiv(e, divP);
    acc[0] += base[i * img_stride + (e - i * P)];
  }
  float sum = (acc[0] + acc[1]) + (acc[2] + acc[3]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_down(sum, off, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
  __syncthreads();
  if (threadIdx.x == 0) scratch[blockIdx.x] = ((red[0] + red[1]) + red[2]) + red[3];
}

__global__ void dbias_stage2(const float* __restrict__ scratch, float* __restrict__ dbias, int O,
                             int nblk) {
  const int o = blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= O) return;
  float acc = 0.0f;
  for (int b = 0; b < nblk; ++b) acc += scratch[o * nblk + b];
  dbias[o] = acc;
}

}  // namespace

int launch_pack_kernel_matrix(const float* w, void* pack, const PackDesc& d, hipStream_t st) {
  const long long total = (long long)d.Mpad * d.Kpad * d.G;
  const long long blocks = (total + TPB - 1) / TPB;
  if (!grid_ok(blocks)) return CCT_EUNSUPPORTED;
  ProfScope ps("pack_kernel", 0.0,
               4.0 * d.G * d.Og * d.Cg * d.K * d.K + (d.bf16 ? 2.0 : 4.0) * total, st);
  if (d.bf16)
    hipLaunchKernelGGL(pack_kernel<true>, dim3((unsigned)blocks), dim3(TPB), 0, st, w, pack, d);
  else
    hipLaunchKernelGGL(pack_kernel<false>, dim3((unsigned)blocks), dim3(TPB), 0, st, w, pack, d);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int launch_pack_flipped(const float* w, float* pack, int G, int Og, int Cg, int K, int Mpad,
                        int Kpad, hipStream_t st) {
  const long long total = (long long)Mpad * Kpad * G;
  const long long blocks = (total + TPB - 1) / TPB;
  if (!grid_ok(blocks)) return CCT_EUNSUPPORTED;
  ProfScope ps("pack_flipped_kernel", 0.0, 4.0 * G * Og * Cg * K * K + 4.0 * total, st);
  hipLaunchKernelGGL(pack_flipped_kernel, dim3((unsigned)blocks), dim3(TPB), 0, st, w, pack, G, Og,
                     Cg, K, Mpad, Kpad);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int launch_pack_type2_bwd(const float* w, float* pack, int G, int Og, int Cg, int K, int Opad,
                          int Mpad, hipStream_t st) {
  const long long total = (long long)Mpad * K * Opad * G;
  const long long blocks = (total + TPB - 1) / TPB;
  if (!grid_ok(blocks)) return CCT_EUNSUPPORTED;
  ProfScope ps("pack_type2_bwd_kernel", 0.0, 4.0 * G * Og * Cg * K * K + 4.0 * total, st);
  hipLaunchKernelGGL(pack_type2_bwd_kernel, dim3((unsigned)blocks), dim3(TPB), 0, st, w, pack, G, Og,
                     Cg, K, Opad, Mpad);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int launch_reduce_dw(const float* part, float* dw, int S, const PackDesc& d, int accumulate,
                     hipStream_t st) {
  const long long total = (long long)d.Og * d.RKi * d.RKj * d.Cg * d.DKi * d.DKj * d.G;
  const long long blocks = (total + 63) / 64;
  if (!grid_ok(blocks)) return CCT_EUNSUPPORTED;
  ProfScope ps("reduce_dw_kernel", 0.0, 4.0 * total * (S + 1), st);
  hipLaunchKernelGGL(reduce_dw_kernel, dim3((unsigned)blocks), dim3(TPB), 0, st, part, dw, S, d,
                     accumulate);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int launch_dbias(const float* dy, float* dbias, float* scratch, int N, int O, int P, int nblk,
                 hipStream_t st) {
  if (!grid_ok((long long)O * nblk)) return CCT_EUNSUPPORTED;
  ProfScope ps("dbias_stage1+2", 0.0, 4.0 * N * O * P, st);
  hipLaunchKernelGGL(dbias_stage1, dim3((unsigned)(O * nblk)), dim3(TPB), 0, st, dy, scratch, N, O,
                     P, nblk, make_fastdiv(P));
  CCT_CHECK_LAUNCH();
  hipLaunchKernelGGL(dbias_stage2, dim3((unsigned)((O + 63) / 64)), dim3(64), 0, st, scratch, dbias,
                     O, nblk);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

}  // namespace cct
