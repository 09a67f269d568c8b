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

// Division by a run-time constant without the hardware's ~40-instruction integer divide:
// for n < 2^31, n / d == (n * M) >> sh with M = ceil(2^sh / d), sh = 31 + ceil(log2 d).
struct FastDiv {
  unsigned M;
  int sh;
  int d;
};
inline FastDiv make_fastdiv(int d) {
  FastDiv f;
  int s = 0;
  while ((1LL << s) < d) ++s;
  f.sh = 31 + s;
  f.M = (unsigned)(((1ULL << f.sh) + (unsigned long long)d - 1) / (unsigned long long)d);
  f.d = d;
  return f;
}
__device__ __forceinline__ int fdiv(int n, const FastDiv& f) {
  return (int)(((unsigned long long)(unsigned)n * f.M) >> f.sh);
}

constexpr int VEC = 4;  // matrix columns (or tensor elements) per thread; stores are 16 bytes

template <bool BF16>
__device__ __forceinline__ void store_vec(void* base, long long idx, const float (&v)[VEC]) {
  if (BF16) {
    uint2 pk;
    pk.x = (unsigned)f32_to_bf16_rne(v[0]) | ((unsigned)f32_to_bf16_rne(v[1]) << 16);
    pk.y = (unsigned)f32_to_bf16_rne(v[2]) | ((unsigned)f32_to_bf16_rne(v[3]) << 16);
    *reinterpret_cast<uint2*>(reinterpret_cast<unsigned short*>(base) + idx) = pk;
  } else {
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(base) + idx) =
        make_float4(v[0], v[1], v[2], v[3]);
  }
}

// ---------------------------------------------------------------------------------------
// Lowering phase.  grid.y/z = matrix row (channel, tap i, tap j); each thread produces VEC
// consecutive matrix columns and writes them with one 16-byte store, so the write stream
// (the k^2-times larger side) is fully coalesced.  The reads are contiguous for stride 1 and
// every s-th float otherwise; the re-reads of x by the other taps hit in L2 / Infinity Cache.
// Columns in [ncols, ld) are padding and receive zeros.
// ---------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(TPB) void lower_kernel(const float* __restrict__ x, void* __restrict__ dt,
                                                    long long ld, int ncols, int rows, int C,
                                                    WinMap m, FastDiv divP, FastDiv divW) {
  const int row = blockIdx.z * 32768 + blockIdx.y;
  const int col0 = (blockIdx.x * TPB + threadIdx.x) * VEC;
  if (row >= rows || col0 >= ld) return;
  const int j = row % m.Kj;                 // uniform over the workgroup
  const int i = (row / m.Kj) % m.Ki;
  const int ch = row / (m.Kj * m.Ki);
  const int Pc = m.Ha * m.Wb;
  int n = fdiv(col0, divP);
  const int rem = col0 - n * Pc;
  int a = fdiv(rem, divW);
  int b = rem - a * m.Wb;
  float v[VEC];
  const float* rowp = nullptr;              // x row (n, ch, h) or null when h is in the padding
  bool fresh = true;
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    if (fresh) {
      const int h = a * m.sh + i - m.ph;
      rowp = (h >= 0 && h < m.Ht) ? x + (((long long)n * C + ch) * m.Ht + h) * m.Wt : nullptr;
      fresh = false;
    }
    const int w = b * m.sw + j - m.pw;
    float val = 0.0f;
    if (col0 + e < ncols && rowp && w >= 0 && w < m.Wt) val = rowp[w];
    v[e] = val;
    if (++b == m.Wb) {
      b = 0;
      fresh = true;
      if (++a == m.Ha) {
        a = 0;
        ++n;
      }
    }
  }
  store_vec<BF16>(dt, (long long)row * ld + col0, v);
}

// Adjoint of the lifting phase: spreads dy over the rows (o, tap i, tap j) of the lowered
// gradient matrix.  Same structure as lower_kernel.
template <bool BF16>
__global__ __launch_bounds__(TPB) void inv_lift_kernel(const float* __restrict__ dy,
                                                       void* __restrict__ drt, long long ld,
                                                       int ncols, int rows, int O, WinMap m,
                                                       FastDiv divP, FastDiv divW, FastDiv divSh,
                                                       FastDiv divSw) {
  const int row = blockIdx.z * 32768 + blockIdx.y;
  const int col0 = (blockIdx.x * TPB + threadIdx.x) * VEC;
  if (row >= rows || col0 >= ld) return;
  const int j = row % m.Kj;
  const int i = (row / m.Kj) % m.Ki;
  const int o = row / (m.Kj * m.Ki);
  const int Pc = m.Ha * m.Wb;
  int n = fdiv(col0, divP);
  const int rem = col0 - n * Pc;
  int a = fdiv(rem, divW);
  int b = rem - a * m.Wb;
  float v[VEC];
  const float* rowp = nullptr;              // dy row (n, o, r) or null when no r maps to a
  bool fresh = true;
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    if (fresh) {
      // a = r*sh + i - ph
      const int hr = a + m.ph - i;
      rowp = nullptr;
      if (hr >= 0) {
        const int r = fdiv(hr, divSh);
        if (r * m.sh == hr && r < m.Ht) rowp = dy + (((long long)n * O + o) * m.Ht + r) * m.Wt;
      }
      fresh = false;
    }
    // b = c*sw + j - pw
    const int wc = b + m.pw - j;
    float val = 0.0f;
    if (col0 + e < ncols && rowp && wc >= 0) {
      const int c = fdiv(wc, divSw);
      if (c * m.sw == wc && c < m.Wt) val = rowp[c];
    }
    v[e] = val;
    if (++b == m.Wb) {
      b = 0;
      fresh = true;
      if (++a == m.Ha) {
        a = 0;
        ++n;
      }
    }
  }
  store_vec<BF16>(drt, (long long)row * ld + col0, v);
}

// ---------------------------------------------------------------------------------------
// Lifting phase fused with the bias add.  One thread per output element; for a fixed tap the
// lanes of a wave read consecutive (stride sw) columns of one R^ row, and every R^ entry is
// read exactly once.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(TPB) void lift_kernel(const float* __restrict__ rt, long long ld,
                                                   float* __restrict__ y,
                                                   const float* __restrict__ bias, long long total,
                                                   int O, WinMap m, FastDiv divWt, FastDiv divPl,
                                                   FastDiv divO) {
  const int t = blockIdx.x * TPB + threadIdx.x;   // total < 2^31 is checked by the launcher
  if (t >= total) return;
  const int plane = fdiv(t, divPl);               // n*O + o
  const int pix = t - plane * (m.Ht * m.Wt);
  const int r = fdiv(pix, divWt);
  const int c = pix - r * m.Wt;
  const int n = fdiv(plane, divO);
  const int o = plane - n * O;
  const float* base = rt + (long long)o * m.Ki * m.Kj * ld + (long long)n * m.Ha * m.Wb;
  float acc = bias ? bias[o] : 0.0f;
  for (int i = 0; i < m.Ki; ++i) {
    const int a = r * m.sh + i - m.ph;
    if (a < 0 || a >= m.Ha) continue;
    const float* rp = base + (long long)i * m.Kj * ld + (long long)a * m.Wb;
    for (int j = 0; j < m.Kj; ++j) {
      const int b = c * m.sw + j - m.pw;
      if (b >= 0 && b < m.Wb) acc += rp[(long long)j * ld + b];
    }
  }
  y[t] = acc;
}

// Adjoint of the lowering phase as a gather (no atomics): every dx pixel sums the entries of
// the lowered gradient that were copied from it.  Only taps i = (h+ph) mod sh, +sh, +2sh, ...
// (and likewise j) can have come from pixel (h, w), so the loops step by the stride.
__global__ __launch_bounds__(TPB) void inv_lower_kernel(const float* __restrict__ ddt, long long ld,
                                                        float* __restrict__ dx, long long total,
                                                        int C, WinMap m, FastDiv divWt, FastDiv divPl,
                                                        FastDiv divC, FastDiv divSh, FastDiv divSw) {
  const int t = blockIdx.x * TPB + threadIdx.x;   // total < 2^31 is checked by the launcher
  if (t >= total) return;
  const int plane = fdiv(t, divPl);               // n*C + ch
  const int pix = t - plane * (m.Ht * m.Wt);
  const int h = fdiv(pix, divWt);
  const int w = pix - h * m.Wt;
  const int n = fdiv(plane, divC);
  const int ch = plane - n * C;
  const float* base = ddt + (long long)ch * m.Ki * m.Kj * ld + (long long)n * m.Ha * m.Wb;
  // first admissible taps and the grid coordinates they map to
  const int a0 = fdiv(h + m.ph, divSh), i0 = h + m.ph - a0 * m.sh;
  const int b0 = fdiv(w + m.pw, divSw), j0 = w + m.pw - b0 * m.sw;
  float acc = 0.0f;
  int a = a0;
  for (int i = i0; i < m.Ki && a >= 0; i += m.sh, --a) {
    if (a >= m.Ha) continue;
    const float* rp = base + (long long)i * m.Kj * ld + (long long)a * m.Wb;
    int b = b0;
    for (int j = j0; j < m.Kj && b >= 0; j += m.sw, --b) {
      if (b < m.Wb) acc += rp[(long long)j * ld + b];
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

namespace {
inline bool row_grid(long long rows, long long ld, dim3* grid) {
  const long long xblocks = (ld / VEC + TPB - 1) / TPB;
  if (rows <= 0 || xblocks <= 0 || xblocks >= 2147483647LL) return false;
  const long long gy = rows < 32768 ? rows : 32768;
  const long long gz = (rows + 32767) / 32768;
  if (gz > 65535) return false;
  *grid = dim3((unsigned)xblocks, (unsigned)gy, (unsigned)gz);
  return true;
}
}  // namespace

int launch_lower(const float* x, void* dt, long long ld, int nimg, int C, const WinMap& m, int bf16,
                 hipStream_t st) {
  const long long ncols = (long long)nimg * m.Ha * m.Wb;
  const long long rows = (long long)C * m.Ki * m.Kj;
  dim3 grid;
  if (ncols >= 2147483647LL - 256 || ld % 64 || ld < ncols || rows >= 2147483647LL ||
      !row_grid(rows, ld, &grid))
    return CCT_EUNSUPPORTED;
  const FastDiv divP = make_fastdiv(m.Ha * m.Wb), divW = make_fastdiv(m.Wb);
  ProfScope ps(bf16 ? "lower_kernel<true>" : "lower_kernel<false>", 0.0,
               4.0 * nimg * C * m.Ht * m.Wt + (bf16 ? 2.0 : 4.0) * rows * ncols, st);
  if (bf16)
    hipLaunchKernelGGL(lower_kernel<true>, grid, dim3(TPB), 0, st, x, dt, ld, (int)ncols, (int)rows,
                       C, m, divP, divW);
  else
    hipLaunchKernelGGL(lower_kernel<false>, grid, dim3(TPB), 0, st, x, dt, ld, (int)ncols, (int)rows,
                       C, m, divP, divW);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int launch_inv_lift(const float* dy, void* drt, long long ld, int nimg, int O, const WinMap& m,
                    int bf16, hipStream_t st) {
  const long long ncols = (long long)nimg * m.Ha * m.Wb;
  const long long rows = (long long)O * m.Ki * m.Kj;
  dim3 grid;
  if (ncols >= 2147483647LL - 256 || ld % 64 || ld < ncols || rows >= 2147483647LL ||
      !row_grid(rows, ld, &grid))
    return CCT_EUNSUPPORTED;
  const FastDiv divP = make_fastdiv(m.Ha * m.Wb), divW = make_fastdiv(m.Wb);
  const FastDiv divSh = make_fastdiv(m.sh), divSw = make_fastdiv(m.sw);
  ProfScope ps(bf16 ? "inv_lift_kernel<true>" : "inv_lift_kernel<false>", 0.0,
               4.0 * nimg * O * m.Ht * m.Wt + (bf16 ? 2.0 : 4.0) * rows * ncols, st);
  if (bf16)
    hipLaunchKernelGGL(inv_lift_kernel<true>, grid, dim3(TPB), 0, st, dy, drt, ld, (int)ncols,
                       (int)rows, O, m, divP, divW, divSh, divSw);
  else
    hipLaunchKernelGGL(inv_lift_kernel<false>, grid, dim3(TPB), 0, st, dy, drt, ld, (int)ncols,
                       (int)rows, O, m, divP, divW, divSh, divSw);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int launch_lift(const float* rt, long long ld, float* y, const float* bias, int nimg, int O,
                const WinMap& m, hipStream_t st) {
  const long long total = (long long)nimg * O * m.Ht * m.Wt;
  const long long blocks = (total + TPB - 1) / TPB;
  if (!grid_ok(blocks) || total >= 2147483647LL - TPB) return CCT_EUNSUPPORTED;
  ProfScope ps("lift_kernel", 0.0,
               4.0 * total + 4.0 * O * m.Ki * m.Kj * (double)nimg * m.Ha * m.Wb, st);
  hipLaunchKernelGGL(lift_kernel, dim3((unsigned)blocks), dim3(TPB), 0, st, rt, ld, y, bias, total, O,
                     m, make_fastdiv(m.Wt), make_fastdiv(m.Ht * m.Wt), make_fastdiv(O));
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int launch_inv_lower(const float* ddt, long long ld, float* dx, int nimg, int C, const WinMap& m,
                     hipStream_t st) {
  const long long total = (long long)nimg * C * m.Ht * m.Wt;
  const long long blocks = (total + TPB - 1) / TPB;
  if (!grid_ok(blocks) || total >= 2147483647LL - TPB) return CCT_EUNSUPPORTED;
  ProfScope ps("inv_lower_kernel", 0.0,
               4.0 * total + 4.0 * C * m.Ki * m.Kj * (double)nimg * m.Ha * m.Wb, st);
  hipLaunchKernelGGL(inv_lower_kernel, dim3((unsigned)blocks), dim3(TPB), 0, st, ddt, ld, dx, total,
                     C, m, make_fastdiv(m.Wt), make_fastdiv(m.Ht * m.Wt), make_fastdiv(C),
                     make_fastdiv(m.sh), make_fastdiv(m.sw));
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
