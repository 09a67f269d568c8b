// Lowering phase (Sec. 2.1) and the adjoint of the lifting phase: the two kernels that WRITE
// a lowered matrix (k or k^2 times larger than the tensor they read).  HBM-bound on the
// write stream.
//
// One workgroup owns one channel and an aligned run of NCB matrix columns (positions of the
// chunk's images, side by side as in Sec. 2.2) and produces ALL tap rows (i, j) of that
// channel for those columns:
//   1. the input rows that these columns can touch are staged in LDS with coalesced loads,
//      so every tensor element is fetched from HBM/L2 once per workgroup instead of once per tap;
//   2. every thread decodes its VEC consecutive columns once, then for each tap reads VEC
//      values from LDS and writes them with one 16-byte store.  Per row the workgroup's stores
//      are one contiguous, aligned run.
#include "cct_internal.h"
#include "index_common.h"

namespace cct {
namespace {

// Staging layout shared by both kernels.  The columns [cb, ce) of a workgroup cover images
// n_first..n_last; of image n they cover grid rows a_lo(n)..a_hi(n), which is the whole image
// except for the first and the last one.  For each image the tensor rows [t_lo, t_hi] that can
// be referenced from those grid rows are copied to LDS back to back.
struct Span {
  int n_first, n_last, a_first, a_last;
};

__device__ __forceinline__ Span block_span(int cb, int ce, int Pc, const FastDiv& divP,
                                           const FastDiv& divW) {
  Span s;
  s.n_first = fdiv(cb, divP);
  s.a_first = fdiv(cb - s.n_first * Pc, divW);
  s.n_last = fdiv(ce - 1, divP);
  s.a_last = fdiv(ce - 1 - s.n_last * Pc, divW);
  return s;
}

// lowering: grid row a reads tensor rows a*sh - ph .. a*sh - ph + Ki - 1
__device__ __forceinline__ void lower_rows(const WinMap& m, int a_lo, int a_hi, int* t_lo, int* t_hi) {
  *t_lo = max(0, a_lo * m.sh - m.ph);
  *t_hi = min(m.Ht - 1, a_hi * m.sh - m.ph + m.Ki - 1);
}
// adjoint of lifting: grid row a receives from tensor rows r with a = r*sh + i - ph
__device__ __forceinline__ void inv_lift_rows(const WinMap& m, const FastDiv& divSh, int a_lo,
                                              int a_hi, int* t_lo, int* t_hi) {
  const int t = a_lo + m.ph - (m.Ki - 1);
  *t_lo = t <= 0 ? 0 : fdiv(t + m.sh - 1, divSh);
  *t_hi = min(m.Ht - 1, fdiv(a_hi + m.ph, divSh));
}

template <bool BF16, int NTH>
__global__ __launch_bounds__(NTH) void lower_kernel(const float* __restrict__ x, void* __restrict__ dt,
                                                    long long ld, int ncols, int C, WinMap m,
                                                    FastDiv divP, FastDiv divW) {
  extern __shared__ float tile[];
  constexpr int NCB = NTH * VEC;
  const int tid = threadIdx.x;
  const int ch = blockIdx.z * 32768 + blockIdx.y;
  const int cb = blockIdx.x * NCB;
  const int ce = min(cb + NCB, ncols);
  const int Pc = m.Ha * m.Wb;
  const int col0 = cb + tid * VEC;

  int len_first = 0, len_full = 0, tlo_first = 0;
  Span sp = {0, -1, 0, 0};
  if (ce > cb) {
    sp = block_span(cb, ce, Pc, divP, divW);
    int off = 0;
    for (int n = sp.n_first; n <= sp.n_last; ++n) {
      const int a_lo = n == sp.n_first ? sp.a_first : 0;
      const int a_hi = n == sp.n_last ? sp.a_last : m.Ha - 1;
      int t_lo, t_hi;
      lower_rows(m, a_lo, a_hi, &t_lo, &t_hi);
      const int len = max(0, t_hi - t_lo + 1) * m.Wt;
      const float* src = x + (((long long)n * C + ch) * m.Ht + t_lo) * m.Wt;
      for (int t = tid; t < len; t += NTH) tile[off + t] = src[t];
      if (n == sp.n_first) {
        len_first = len;
        tlo_first = t_lo;
      }
      off += len;
    }
    int t_lo, t_hi;
    lower_rows(m, 0, m.Ha - 1, &t_lo, &t_hi);
    len_full = max(0, t_hi - t_lo + 1) * m.Wt;
  }
  __syncthreads();
  if (col0 >= ld) return;

  // decode this thread's VEC columns once
  int base[VEC], hh[VEC], ww[VEC];
  {
    int n = fdiv(col0, divP);
    const int rem = col0 - n * Pc;
    int a = fdiv(rem, divW);
    int b = rem - a * m.Wb;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const bool first = n == sp.n_first;
      const int seg = first ? 0 : len_first + (n - sp.n_first - 1) * len_full;
      const int t_lo = first ? tlo_first : 0;
      hh[e] = a * m.sh - m.ph;
      ww[e] = b * m.sw - m.pw;
      base[e] = seg + (hh[e] - t_lo) * m.Wt + ww[e];
      if (col0 + e >= ce) hh[e] = -(1 << 30);  // padding column: every tap is out of range
      if (++b == m.Wb) {
        b = 0;
        if (++a == m.Ha) {
          a = 0;
          ++n;
        }
      }
    }
  }
  const long long row0 = (long long)ch * m.Ki * m.Kj;
  for (int i = 0; i < m.Ki; ++i) {
    for (int j = 0; j < m.Kj; ++j) {
      float v[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const bool ok = (unsigned)(hh[e] + i) < (unsigned)m.Ht && (unsigned)(ww[e] + j) < (unsigned)m.Wt;
        const float t = tile[ok ? base[e] + i * m.Wt + j : 0];
        v[e] = ok ? t : 0.0f;
      }
      store_vec<BF16>(dt, (row0 + i * m.Kj + j) * ld + col0, v);
    }
  }
}

template <bool BF16, int NTH>
__global__ __launch_bounds__(NTH) void inv_lift_kernel(const float* __restrict__ dy,
                                                       void* __restrict__ drt, long long ld,
                                                       int ncols, int O, WinMap m, FastDiv divP,
                                                       FastDiv divW, FastDiv divSh, FastDiv divSw) {
  extern __shared__ float tile[];
  constexpr int NCB = NTH * VEC;
  const int tid = threadIdx.x;
  const int o = blockIdx.z * 32768 + blockIdx.y;
  const int cb = blockIdx.x * NCB;
  const int ce = min(cb + NCB, ncols);
  const int Pc = m.Ha * m.Wb;
  const int col0 = cb + tid * VEC;

  int len_first = 0, len_full = 0, tlo_first = 0, tlo_full = 0;
  Span sp = {0, -1, 0, 0};
  if (ce > cb) {
    sp = block_span(cb, ce, Pc, divP, divW);
    int off = 0;
    for (int n = sp.n_first; n <= sp.n_last; ++n) {
      const int a_lo = n == sp.n_first ? sp.a_first : 0;
      const int a_hi = n == sp.n_last ? sp.a_last : m.Ha - 1;
      int t_lo, t_hi;
      inv_lift_rows(m, divSh, a_lo, a_hi, &t_lo, &t_hi);
      const int len = max(0, t_hi - t_lo + 1) * m.Wt;
      const float* src = dy + (((long long)n * O + o) * m.Ht + t_lo) * m.Wt;
      for (int t = tid; t < len; t += NTH) tile[off + t] = src[t];
      if (n == sp.n_first) {
        len_first = len;
        tlo_first = t_lo;
      }
      off += len;
    }
    int t_hi;
    inv_lift_rows(m, divSh, 0, m.Ha - 1, &tlo_full, &t_hi);
    len_full = max(0, t_hi - tlo_full + 1) * m.Wt;
  }
  __syncthreads();
  if (col0 >= ld) return;

  int seg[VEC], ha[VEC], wb[VEC];  // ha = a + ph, wb = b + pw; seg already has -t_lo*Wt folded in
  {
    int n = fdiv(col0, divP);
    const int rem = col0 - n * Pc;
    int a = fdiv(rem, divW);
    int b = rem - a * m.Wb;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const bool first = n == sp.n_first;
      seg[e] = (first ? 0 : len_first + (n - sp.n_first - 1) * len_full) -
               (first ? tlo_first : tlo_full) * m.Wt;
      ha[e] = a + m.ph;
      wb[e] = b + m.pw;
      if (col0 + e >= ce) ha[e] = -1;  // padding column
      if (++b == m.Wb) {
        b = 0;
        if (++a == m.Ha) {
          a = 0;
          ++n;
        }
      }
    }
  }
  const long long row0 = (long long)o * m.Ki * m.Kj;
  for (int i = 0; i < m.Ki; ++i) {
    for (int j = 0; j < m.Kj; ++j) {
      float v[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        // a = r*sh + i - ph,  b = c*sw + j - pw
        const int hr = ha[e] - i, wc = wb[e] - j;
        const int r = fdiv(max(hr, 0), divSh), c = fdiv(max(wc, 0), divSw);
        const bool ok = hr >= 0 && wc >= 0 && r * m.sh == hr && c * m.sw == wc && r < m.Ht && c < m.Wt;
        const float t = tile[ok ? seg[e] + r * m.Wt + c : 0];
        v[e] = ok ? t : 0.0f;
      }
      store_vec<BF16>(drt, (row0 + i * m.Kj + j) * ld + col0, v);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Lowering phase, direct form (fallback for shapes whose input window does not fit in LDS).
// grid.y/z = matrix row (channel, tap i, tap j); each thread produces VEC
// consecutive matrix columns and writes them with one 16-byte store, so the write stream
// (the k^2-times larger side) is fully coalesced.  The reads are contiguous for stride 1 and
// every s-th float otherwise; the re-reads of x by the other taps hit in L2 / Infinity Cache.
// Columns in [ncols, ld) are padding and receive zeros.
// ---------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(TPB) void lower_direct_kernel(const float* __restrict__ x, void* __restrict__ dt,
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
__global__ __launch_bounds__(TPB) void inv_lift_direct_kernel(const float* __restrict__ dy,
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


// Upper bound (floats) of the LDS staging area of a workgroup that owns ncb columns.
// images touched T <= (ncb-1)/Pc + 2; grid rows touched A <= (ncb-1)/Wb + 2 (A >= T).
inline long long lower_lds_floats(const WinMap& m, int ncb) {
  const long long Pc = (long long)m.Ha * m.Wb;
  const long long T = (ncb - 1) / Pc + 2, A = (ncb - 1) / m.Wb + 2;
  const long long full = (long long)m.Ht * m.Wt;
  // a run of A_t grid rows inside one image needs (A_t - 1)*sh + Ki tensor rows; with the A rows
  // split over t <= T images that is (A - t)*sh + t*Ki, largest at t = 1 or t = T
  const long long r1 = (A - 1) * m.sh + m.Ki;
  const long long rT = (A > T ? A - T : 0) * m.sh + T * m.Ki;
  const long long by_rows = (r1 > rT ? r1 : rT) * m.Wt;
  return T * full < by_rows ? T * full : by_rows;
}
inline long long inv_lift_lds_floats(const WinMap& m, int ncb) {
  const long long Pc = (long long)m.Ha * m.Wb;
  const long long T = (ncb - 1) / Pc + 2, A = (ncb - 1) / m.Wb + 2;
  const long long full = (long long)m.Ht * m.Wt;
  const long long by_rows = ((A + T * (m.Ki - 1)) / m.sh + 2 * T) * m.Wt;
  return T * full < by_rows ? T * full : by_rows;
}
// Threads per workgroup for the staged kernels: prefer 256 with <= 32 KiB of LDS (keeps several
// workgroups per CU), then smaller groups, then anything up to 64 KiB; 0 = does not fit.
template <typename F>
inline int pick_threads(const WinMap& m, F lds_floats, long long* lds_bytes) {
  const int cand[3] = {256, 128, 64};
  for (long long cap : {32768LL, 65536LL})
    for (int nth : cand) {
      const long long b = lds_floats(m, nth * VEC) * 4;
      if (b <= cap) {
        *lds_bytes = b;
        return nth;
      }
    }
  return 0;
}

inline bool chan_grid(long long chans, long long ld, int ncb, dim3* grid) {
  const long long xblocks = (ld + ncb - 1) / ncb;
  if (chans <= 0 || xblocks <= 0 || xblocks >= 2147483647LL) return false;
  const long long gy = chans < 32768 ? chans : 32768;
  const long long gz = (chans + 32767) / 32768;
  if (gz > 65535) return false;
  *grid = dim3((unsigned)xblocks, (unsigned)gy, (unsigned)gz);
  return true;
}

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
  const double bytes = 4.0 * nimg * C * m.Ht * m.Wt + (bf16 ? 2.0 : 4.0) * rows * ncols;
  long long lds = 0;
  const int nth = pick_threads(m, lower_lds_floats, &lds);
  dim3 sgrid;
  if (nth && chan_grid(C, ld, nth * VEC, &sgrid)) {
    ProfScope ps(bf16 ? "lower_kernel<true>" : "lower_kernel<false>", 0.0, bytes, st);
#define CCT_LAUNCH_LOWER(BF, NTH)                                                              \
  hipLaunchKernelGGL((lower_kernel<BF, NTH>), sgrid, dim3(NTH), (size_t)lds, st, x, dt, ld,     \
                     (int)ncols, C, m, divP, divW)
    if (bf16) {
      if (nth == 256) CCT_LAUNCH_LOWER(true, 256);
      else if (nth == 128) CCT_LAUNCH_LOWER(true, 128);
      else CCT_LAUNCH_LOWER(true, 64);
    } else {
      if (nth == 256) CCT_LAUNCH_LOWER(false, 256);
      else if (nth == 128) CCT_LAUNCH_LOWER(false, 128);
      else CCT_LAUNCH_LOWER(false, 64);
    }
#undef CCT_LAUNCH_LOWER
    CCT_CHECK_LAUNCH();
    return CCT_OK;
  }
  ProfScope ps(bf16 ? "lower_direct_kernel<true>" : "lower_direct_kernel<false>", 0.0, bytes, st);
  if (bf16)
    hipLaunchKernelGGL(lower_direct_kernel<true>, grid, dim3(TPB), 0, st, x, dt, ld, (int)ncols,
                       (int)rows, C, m, divP, divW);
  else
    hipLaunchKernelGGL(lower_direct_kernel<false>, grid, dim3(TPB), 0, st, x, dt, ld, (int)ncols,
                       (int)rows, C, m, divP, divW);
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
  const double bytes = 4.0 * nimg * O * m.Ht * m.Wt + (bf16 ? 2.0 : 4.0) * rows * ncols;
  long long lds = 0;
  const int nth = pick_threads(m, inv_lift_lds_floats, &lds);
  dim3 sgrid;
  if (nth && chan_grid(O, ld, nth * VEC, &sgrid)) {
    ProfScope ps(bf16 ? "inv_lift_kernel<true>" : "inv_lift_kernel<false>", 0.0, bytes, st);
#define CCT_LAUNCH_INV_LIFT(BF, NTH)                                                           \
  hipLaunchKernelGGL((inv_lift_kernel<BF, NTH>), sgrid, dim3(NTH), (size_t)lds, st, dy, drt, ld, \
                     (int)ncols, O, m, divP, divW, divSh, divSw)
    if (bf16) {
      if (nth == 256) CCT_LAUNCH_INV_LIFT(true, 256);
      else if (nth == 128) CCT_LAUNCH_INV_LIFT(true, 128);
      else CCT_LAUNCH_INV_LIFT(true, 64);
    } else {
      if (nth == 256) CCT_LAUNCH_INV_LIFT(false, 256);
      else if (nth == 128) CCT_LAUNCH_INV_LIFT(false, 128);
      else CCT_LAUNCH_INV_LIFT(false, 64);
    }
#undef CCT_LAUNCH_INV_LIFT
    CCT_CHECK_LAUNCH();
    return CCT_OK;
  }
  ProfScope ps(bf16 ? "inv_lift_direct_kernel<true>" : "inv_lift_direct_kernel<false>", 0.0, bytes,
               st);
  if (bf16)
    hipLaunchKernelGGL(inv_lift_direct_kernel<true>, grid, dim3(TPB), 0, st, dy, drt, ld, (int)ncols,
                       (int)rows, O, m, divP, divW, divSh, divSw);
  else
    hipLaunchKernelGGL(inv_lift_direct_kernel<false>, grid, dim3(TPB), 0, st, dy, drt, ld,
                       (int)ncols, (int)rows, O, m, divP, divW, divSh, divSw);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

}  // namespace cct
