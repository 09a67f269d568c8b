// Lowering / lifting phases (Sec. 2.1) and their adjoints, the lowered-kernel pack, and the
// small reductions of the backward-weights pass.  All of these are pure index maps or short
// sums: HBM-bound, one coalesced stream in, one coalesced stream out.
#include "cct_internal.h"

namespace cct {

static thread_local int g_last_hip_error = 0;
void set_hip_error(hipError_t e) { g_last_hip_error = (int)e; }
int last_hip_error_value() { return g_last_hip_error; }

namespace {

constexpr int TPB = 256;

// fp32 -> bf16, round to nearest even (NaN stays NaN).
__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f) {
  unsigned int u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}

template <bool BF16>
__device__ __forceinline__ void store_elem(void* base, long long idx, float v) {
  if (BF16)
    reinterpret_cast<unsigned short*>(base)[idx] = f32_to_bf16_rne(v);
  else
    reinterpret_cast<float*>(base)[idx] = v;
}

// ---------------------------------------------------------------------------------------
// Lowering phase.  One workgroup = one matrix row (channel, tap i, tap j) x 256 consecutive
// matrix columns, so stores are one contiguous run; loads are contiguous for stride 1 and
// every s-th float otherwise (the re-reads of x by the other taps hit in L2).
// ---------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(TPB) void lower_kernel(const float* __restrict__ x, void* __restrict__ dt,
                                                    long long ld, int ncols, int nblk_col, int C,
                                                    WinMap m) {
  const int row = blockIdx.x / nblk_col;
  const int col = (blockIdx.x % nblk_col) * TPB + threadIdx.x;
  if (col >= ncols) return;
  const int j = row % m.Kj;
  const int i = (row / m.Kj) % m.Ki;
  const int ch = row / (m.Kj * m.Ki);
  const int Pc = m.Ha * m.Wb;
  const int n = col / Pc;
  const int rem = col - n * Pc;
  const int a = rem / m.Wb;
  const int b = rem - a * m.Wb;
  const int h = a * m.sh + i - m.ph;
  const int w = b * m.sw + j - m.pw;
  float v = 0.0f;
  if (h >= 0 && h < m.Ht && w >= 0 && w < m.Wt)
    v = x[(((long long)n * C + ch) * m.Ht + h) * m.Wt + w];
  store_elem<BF16>(dt, (long long)row * ld + col, v);
}

// Adjoint of the lifting phase: spreads dy over the rows (o, tap i, tap j) of the lowered
// gradient matrix.  Same store pattern as lower_kernel.
template <bool BF16>
__global__ __launch_bounds__(TPB) void inv_lift_kernel(const float* __restrict__ dy,
                                                       void* __restrict__ drt, long long ld,
                                                       int ncols, int nblk_col, int O, WinMap m) {
  const int row = blockIdx.x / nblk_col;
  const int col = (blockIdx.x % nblk_col) * TPB + threadIdx.x;
  if (col >= ncols) return;
  const int j = row % m.Kj;
  const int i = (row / m.Kj) % m.Ki;
  const int o = row / (m.Kj * m.Ki);
  const int Pc = m.Ha * m.Wb;
  const int n = col / Pc;
  const int rem = col - n * Pc;
  const int a = rem / m.Wb;
  const int b = rem - a * m.Wb;
  // a = r*sh + i - ph, b = c*sw + j - pw
  const int hr = a + m.ph - i;
  const int wc = b + m.pw - j;
  float v = 0.0f;
  if (hr >= 0 && wc >= 0) {
    const int r = hr / m.sh, c = wc / m.sw;
    if (r * m.sh == hr && c * m.sw == wc && r < m.Ht && c < m.Wt)
      v = dy[(((long long)n * O + o) * m.Ht + r) * m.Wt + c];
  }
  store_elem<BF16>(drt, (long long)row * ld + col, v);
}

// ---------------------------------------------------------------------------------------
// Lifting phase fused with the bias add.  One thread per output element; for a fixed tap the
// threads of a wave read consecutive (stride sw) columns of one R^ row.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(TPB) void lift_kernel(const float* __restrict__ rt, long long ld,
                                                   float* __restrict__ y,
                                                   const float* __restrict__ bias, long long total,
                                                   int O, WinMap m) {
  const long long t = (long long)blockIdx.x * TPB + threadIdx.x;
  if (t >= total) return;
  const int c = (int)(t % m.Wt);
  long long v = t / m.Wt;
  const int r = (int)(v % m.Ht);
  v /= m.Ht;
  const int o = (int)(v % O);
  const int n = (int)(v / O);
  const long long colbase = (long long)n * m.Ha * m.Wb;
  float acc = bias ? bias[o] : 0.0f;
  for (int i = 0; i < m.Ki; ++i) {
    const int a = r * m.sh + i - m.ph;
    if (a < 0 || a >= m.Ha) continue;
    for (int j = 0; j < m.Kj; ++j) {
      const int b = c * m.sw + j - m.pw;
      if (b < 0 || b >= m.Wb) continue;
      const long long row = ((long long)o * m.Ki + i) * m.Kj + j;
      acc += rt[row * ld + colbase + (long long)a * m.Wb + b];
    }
  }
  y[t] = acc;
}

// Adjoint of the lowering phase as a gather (no atomics): every dx pixel sums the entries of
// the lowered gradient that were copied from it.
__global__ __launch_bounds__(TPB) void inv_lower_kernel(const float* __restrict__ ddt, long long ld,
                                                        float* __restrict__ dx, long long total,
                                                        int C, WinMap m) {
  const long long t = (long long)blockIdx.x * TPB + threadIdx.x;
  if (t >= total) return;
  const int w = (int)(t % m.Wt);
  long long v = t / m.Wt;
  const int h = (int)(v % m.Ht);
  v /= m.Ht;
  const int ch = (int)(v % C);
  const int n = (int)(v / C);
  const long long colbase = (long long)n * m.Ha * m.Wb;
  float acc = 0.0f;
  for (int i = 0; i < m.Ki; ++i) {
    const int hr = h + m.ph - i;
    if (hr < 0) break;
    const int a = hr / m.sh;
    if (a * m.sh != hr || a >= m.Ha) continue;
    for (int j = 0; j < m.Kj; ++j) {
      const int wc = w + m.pw - j;
      if (wc < 0) break;
      const int b = wc / m.sw;
      if (b * m.sw != wc || b >= m.Wb) continue;
      const long long row = ((long long)ch * m.Ki + i) * m.Kj + j;
      acc += ddt[row * ld + colbase + (long long)a * m.Wb + b];
    }
  }
  dx[t] = acc;
}

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

// dw = sum over split-K partials, in split order (deterministic), mapped back to O x Cg x K x K.
__global__ __launch_bounds__(TPB) void reduce_dw_kernel(const float* __restrict__ part,
                                                        float* __restrict__ dw, int S, PackDesc d,
                                                        int accumulate) {
  const int nrho = d.Og * d.RKi * d.RKj, ndelta = d.Cg * d.DKi * d.DKj;
  const long long per_group = (long long)nrho * ndelta;
  const long long total = per_group * d.G;
  const long long t = (long long)blockIdx.x * TPB + threadIdx.x;
  if (t >= total) return;
  const int q = (int)(t / per_group);
  const long long e = t - q * per_group;
  const int rho = (int)(e / ndelta), delta = (int)(e % ndelta);
  float acc = 0.0f;
  for (int s = 0; s < S; ++s) acc += part[(long long)s * total + t];
  const long long wi = weight_index(d, q, rho, delta);
  dw[wi] = accumulate ? dw[wi] + acc : acc;
}

// dbias, stage 1: block (o, blk) sums a slice of the N*P values of channel o.
__global__ __launch_bounds__(TPB) void dbias_stage1(const float* __restrict__ dy,
                                                    float* __restrict__ scratch, int N, int O, int P,
                                                    int nblk) {
  __shared__ float red[TPB];
  const int o = blockIdx.x / nblk, blk = blockIdx.x % nblk;
  const long long total = (long long)N * P;
  float acc = 0.0f;
  for (long long t = (long long)blk * TPB + threadIdx.x; t < total; t += (long long)nblk * TPB) {
    const long long n = t / P;
    const int pix = (int)(t - n * P);
    acc += dy[(n * O + o) * P + pix];
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = TPB / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) scratch[blockIdx.x] = red[0];
}

__global__ void dbias_stage2(const float* __restrict__ scratch, float* __restrict__ dbias, int O,
                             int nblk) {
  const int o = blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= O) return;
  float acc = 0.0f;
  for (int b = 0; b < nblk; ++b) acc += scratch[o * nblk + b];
  dbias[o] = acc;
}

inline bool grid_ok(long long blocks) { return blocks > 0 && blocks < 2147483647LL; }

}  // namespace

int launch_lower(const float* x, void* dt, long long ld, int nimg, int C, const WinMap& m, int bf16,
                 hipStream_t st) {
  const long long ncols = (long long)nimg * m.Ha * m.Wb;
  const long long rows = (long long)C * m.Ki * m.Kj;
  const long long nblk_col = (ncols + TPB - 1) / TPB;
  if (ncols >= 2147483647LL || !grid_ok(rows * nblk_col)) return CCT_EUNSUPPORTED;
  dim3 grid((unsigned)(rows * nblk_col));
  ProfScope ps(bf16 ? "lower_kernel<true>" : "lower_kernel<false>", 0.0,
               4.0 * nimg * C * m.Ht * m.Wt + (bf16 ? 2.0 : 4.0) * rows * ncols, st);
  if (bf16)
    hipLaunchKernelGGL(lower_kernel<true>, grid, dim3(TPB), 0, st, x, dt, ld, (int)ncols,
                       (int)nblk_col, C, m);
  else
    hipLaunchKernelGGL(lower_kernel<false>, grid, dim3(TPB), 0, st, x, dt, ld, (int)ncols,
                       (int)nblk_col, C, m);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int launch_inv_lift(const float* dy, void* drt, long long ld, int nimg, int O, const WinMap& m,
                    int bf16, hipStream_t st) {
  const long long ncols = (long long)nimg * m.Ha * m.Wb;
  const long long rows = (long long)O * m.Ki * m.Kj;
  const long long nblk_col = (ncols + TPB - 1) / TPB;
  if (ncols >= 2147483647LL || !grid_ok(rows * nblk_col)) return CCT_EUNSUPPORTED;
  dim3 grid((unsigned)(rows * nblk_col));
  ProfScope ps(bf16 ? "inv_lift_kernel<true>" : "inv_lift_kernel<false>", 0.0,
               4.0 * nimg * O * m.Ht * m.Wt + (bf16 ? 2.0 : 4.0) * rows * ncols, st);
  if (bf16)
    hipLaunchKernelGGL(inv_lift_kernel<true>, grid, dim3(TPB), 0, st, dy, drt, ld, (int)ncols,
                       (int)nblk_col, O, m);
  else
    hipLaunchKernelGGL(inv_lift_kernel<false>, grid, dim3(TPB), 0, st, dy, drt, ld, (int)ncols,
                       (int)nblk_col, O, m);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int launch_lift(const float* rt, long long ld, float* y, const float* bias, int nimg, int O,
                const WinMap& m, hipStream_t st) {
  const long long total = (long long)nimg * O * m.Ht * m.Wt;
  const long long blocks = (total + TPB - 1) / TPB;
  if (!grid_ok(blocks)) return CCT_EUNSUPPORTED;
  ProfScope ps("lift_kernel", 0.0,
               4.0 * total + 4.0 * O * m.Ki * m.Kj * (double)nimg * m.Ha * m.Wb, st);
  hipLaunchKernelGGL(lift_kernel, dim3((unsigned)blocks), dim3(TPB), 0, st, rt, ld, y, bias, total, O,
                     m);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int launch_inv_lower(const float* ddt, long long ld, float* dx, int nimg, int C, const WinMap& m,
                     hipStream_t st) {
  const long long total = (long long)nimg * C * m.Ht * m.Wt;
  const long long blocks = (total + TPB - 1) / TPB;
  if (!grid_ok(blocks)) return CCT_EUNSUPPORTED;
  ProfScope ps("inv_lower_kernel", 0.0,
               4.0 * total + 4.0 * C * m.Ki * m.Kj * (double)nimg * m.Ha * m.Wb, st);
  hipLaunchKernelGGL(inv_lower_kernel, dim3((unsigned)blocks), dim3(TPB), 0, st, ddt, ld, dx, total,
                     C, m);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

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

int launch_reduce_dw(const float* part, float* dw, int S, const PackDesc& d, int accumulate,
                     hipStream_t st) {
  const long long total = (long long)d.Og * d.RKi * d.RKj * d.Cg * d.DKi * d.DKj * d.G;
  const long long blocks = (total + TPB - 1) / TPB;
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
                     P, nblk);
  CCT_CHECK_LAUNCH();
  hipLaunchKernelGGL(dbias_stage2, dim3((unsigned)((O + 63) / 64)), dim3(64), 0, st, scratch, dbias,
                     O, nblk);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

}  // namespace cct
