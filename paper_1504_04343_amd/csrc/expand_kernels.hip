// Lowering phase (Sec. 2.1) and the adjoint of the lifting phase: the two kernels that WRITE
// a lowered matrix (k or k^2 times larger than the tensor they read).  HBM-bound on the
// write stream.
//
// One workgroup owns one channel and an aligned run of NCB matrix columns (positions of the
// chunk's images, side by side as in Sec. 2.2) and produces ALL tap rows (i, j) of that
// channel for those columns:
//   1. the input rows that these columns can touch are staged in LDS with coalesced loads,
//      so every tensor element is fetched from HBM/L2 once per workgroup instead of once per tap;
//   2. every thread decodes its VEC columns once (consecutive lanes own consecutive columns),
//      then for each tap reads VEC values from LDS and stores them: per tap row every wave
//      writes contiguous 256-byte runs.
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

// Column assignment inside a workgroup: a lane owns CPT consecutive columns and consecutive lanes
// own consecutive groups, so the global stores of a wave are one contiguous run (4, or with the
// four-column fp32 form of lower_kernel 16, bytes per lane).  The LDS reads of that form hit the
// banks four at a time, which does not matter for a kernel bound by its HBM write stream.
template <bool BF16, int CPT>
__device__ __forceinline__ void store_run(void* base, long long idx, const float* v) {
  if (BF16) {
    reinterpret_cast<unsigned*>(reinterpret_cast<unsigned short*>(base) + idx)[0] =
        (unsigned)f32_to_bf16_rne(v[0]) | ((unsigned)f32_to_bf16_rne(v[1]) << 16);
  } else if (CPT == 4) {
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(base) + idx) = make_float4(v[0], v[1], v[2], v[3]);
  } else {
    reinterpret_cast<float*>(base)[idx] = v[0];
  }
}

template <bool BF16, int VC>
__global__ __launch_bounds__(TPB) void lower_kernel(const float* __restrict__ x, void* __restrict__ dt,
                                                    long long ld, int ncols, int C, WinMap m,
                                                    FastDiv divP, FastDiv divW, FastDiv divWt,
                                                    FastDiv divSw) {
  extern __shared__ float tile[];
  constexpr int NTH = TPB;
  constexpr int NCB = NTH * VC;        // columns per workgroup
  // consecutive columns per lane: 4 (one 16-byte store per tap row) when a thread has 4 columns,
  // 2 in bf16 mode (one 4-byte store); else 1
  constexpr int CPT = BF16 ? 2 : (VC == 4 ? 4 : 1);
  constexpr int EG = VC / CPT;         // column groups per thread
  static_assert(VC % CPT == 0, "columns per thread");
  const int tid = threadIdx.x;
  const int ch = blockIdx.z * 32768 + blockIdx.y;
  const int cb = blockIdx.x * NCB;
  const int ce = min(cb + NCB, ncols);
  const int Pc = m.Ha * m.Wb;
  // LDS row layout: for stride sw > 1 a tensor row is stored de-interleaved by w mod sw
  // (residue r at [r*Wq, (r+1)*Wq)), so that the columns b, b+1, ... of one tap, which are sw
  // pixels apart, sit in consecutive LDS words.
  const int Wq = (m.Wt + m.sw - 1) / m.sw;
  const int Wrow = Wq * m.sw;

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
      const int nrows = max(0, t_hi - t_lo + 1);
      const float* src = x + (((long long)n * C + ch) * m.Ht + t_lo) * m.Wt;
      // 8 independent loads per thread in flight, then the LDS stores
      const int len = nrows * m.Wt;
      for (int t0 = tid; t0 < len; t0 += NTH * 8) {
        float rv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int t = t0 + u * NTH;
          rv[u] = t < len ? src[t] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int t = t0 + u * NTH;
          if (t < len) {
            if (m.sw == 1) {
              tile[off + t] = rv[u];
            } else {
              const int r = fdiv(t, divWt), w = t - r * m.Wt;
              const int wq = fdiv(w, divSw), wr = w - wq * m.sw;
              tile[off + r * Wrow + wr * Wq + wq] = rv[u];
            }
          }
        }
      }
      if (n == sp.n_first) {
        len_first = nrows * Wrow;
        tlo_first = t_lo;
      }
      off += nrows * Wrow;
    }
    int t_lo, t_hi;
    lower_rows(m, 0, m.Ha - 1, &t_lo, &t_hi);
    len_full = max(0, t_hi - t_lo + 1) * Wrow;
  }
  __syncthreads();

  // decode this thread's columns once
  int base[VC], hh[VC], bb[VC];
#pragma unroll
  for (int e = 0; e < EG; ++e) {
    const int c0 = cb + (e * NTH + tid) * CPT;
    int n = fdiv(c0, divP);
    const int rem = c0 - n * Pc;
    int a = fdiv(rem, divW);
    int b = rem - a * m.Wb;
#pragma unroll
    for (int u = 0; u < CPT; ++u) {
      const int q = e * CPT + u;
      const bool first = n == sp.n_first;
      const int seg = first ? 0 : len_first + (n - sp.n_first - 1) * len_full;
      const int t_lo = first ? tlo_first : 0;
      hh[q] = a * m.sh - m.ph;
      bb[q] = b;
      base[q] = seg + (hh[q] - t_lo) * Wrow + b;
      if (c0 + u >= ce) hh[q] = -(1 << 30);  // padding column: every tap is out of range
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
  for (int j = 0; j < m.Kj; ++j) {
    // w = b*sw + (j - pw) = (b + qj)*sw + rj with 0 <= rj < sw
    const int jj = j - m.pw;
    const int qj = jj >= 0 ? fdiv(jj, divSw) : -fdiv(-jj + m.sw - 1, divSw);
    const int rj = jj - qj * m.sw;
    const int joff = rj * Wq + qj;
    for (int i = 0; i < m.Ki; ++i) {
      float v[VC];
#pragma unroll
      for (int q = 0; q < VC; ++q) {
        const bool ok = (unsigned)(hh[q] + i) < (unsigned)m.Ht &&
                        (unsigned)(bb[q] * m.sw + jj) < (unsigned)m.Wt;
        const float t = tile[ok ? base[q] + i * Wrow + joff : 0];
        v[q] = ok ? t : 0.0f;
      }
      const long long rbase = (row0 + i * m.Kj + j) * ld;
#pragma unroll
      for (int e = 0; e < EG; ++e) {
        const int c0 = cb + (e * NTH + tid) * CPT;
        if (c0 < ld) store_run<BF16, CPT>(dt, rbase + c0, &v[e * CPT]);
      }
    }
  }
}

template <bool BF16, int VC>
__global__ __launch_bounds__(TPB) void inv_lift_kernel(const float* __restrict__ dy,
                                                       void* __restrict__ drt, long long ld,
                                                       int ncols, int O, WinMap m, FastDiv divP,
                                                       FastDiv divW, FastDiv divSh, FastDiv divSw) {
  extern __shared__ float tile[];
  constexpr int NTH = TPB;
  constexpr int NCB = NTH * VC;
  constexpr int CPT = BF16 ? 2 : 1;
  constexpr int EG = VC / CPT;
  static_assert(VC % CPT == 0, "columns per thread");
  const int tid = threadIdx.x;
  const int o = blockIdx.z * 32768 + blockIdx.y;
  const int cb = blockIdx.x * NCB;
  const int ce = min(cb + NCB, ncols);
  const int Pc = m.Ha * m.Wb;

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
      for (int t0 = tid; t0 < len; t0 += NTH * 8) {
        float rv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int t = t0 + u * NTH;
          rv[u] = t < len ? src[t] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int t = t0 + u * NTH;
          if (t < len) tile[off + t] = rv[u];
        }
      }
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

  int seg[VC], ha[VC], wb[VC];  // ha = a + ph, wb = b + pw; seg already has -t_lo*Wt folded in
#pragma unroll
  for (int e = 0; e < EG; ++e) {
    const int c0 = cb + (e * NTH + tid) * CPT;
    int n = fdiv(c0, divP);
    const int rem = c0 - n * Pc;
    int a = fdiv(rem, divW);
    int b = rem - a * m.Wb;
#pragma unroll
    for (int u = 0; u < CPT; ++u) {
      const int q = e * CPT + u;
      const bool first = n == sp.n_first;
      seg[q] = (first ? 0 : len_first + (n - sp.n_first - 1) * len_full) -
               (first ? tlo_first : tlo_full) * m.Wt;
      ha[q] = a + m.ph;
      wb[q] = b + m.pw;
      if (c0 + u >= ce) ha[q] = -1;  // padding column
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
      float v[VC];
#pragma unroll
      for (int q = 0; q < VC; ++q) {
        // a = r*sh + i - ph,  b = c*sw + j - pw
        const int hr = ha[q] - i, wc = wb[q] - j;
        const int r = fdiv(max(hr, 0), divSh), c = fdiv(max(wc, 0), divSw);
        const bool ok = hr >= 0 && wc >= 0 && r * m.sh == hr && c * m.sw == wc && r < m.Ht && c < m.Wt;
        const float t = tile[ok ? seg[q] + r * m.Wt + c : 0];
        v[q] = ok ? t : 0.0f;
      }
      const long long rbase = (row0 + i * m.Kj + j) * ld;
#pragma unroll
      for (int e = 0; e < EG; ++e) {
        const int c0 = cb + (e * NTH + tid) * CPT;
        if (c0 < ld) store_run<BF16, CPT>(drt, rbase + c0, &v[e * CPT]);
      }
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
  const long long Wrow = (long long)((m.Wt + m.sw - 1) / m.sw) * m.sw;  // de-interleaved LDS row
  const long long full = (long long)m.Ht * Wrow;
  // a run of A_t grid rows inside one image needs (A_t - 1)*sh + Ki tensor rows; with the A rows
  // split over t <= T images that is (A - t)*sh + t*Ki, largest at t = 1 or t = T
  const long long r1 = (A - 1) * m.sh + m.Ki;
  const long long rT = (A > T ? A - T : 0) * m.sh + T * m.Ki;
  const long long by_rows = (r1 > rT ? r1 : rT) * Wrow;
  return T * full < by_rows ? T * full : by_rows;
}
inline long long inv_lift_lds_floats(const WinMap& m, int ncb) {
  const long long Pc = (long long)m.Ha * m.Wb;
  const long long T = (ncb - 1) / Pc + 2, A = (ncb - 1) / m.Wb + 2;
  const long long full = (long long)m.Ht * m.Wt;
  const long long by_rows = ((A + T * (m.Ki - 1)) / m.sh + 2 * T) * m.Wt;
  return T * full < by_rows ? T * full : by_rows;
}
// Columns per thread (workgroups are 256 threads) for the staged kernels: the most columns
// whose staging area fits 32 KiB (several workgroups per CU), else the most that fit 64 KiB;
// 0 = does not fit.  bf16 output packs two columns per lane, so it needs an even count.
template <typename F>
inline int pick_cols(const WinMap& m, F lds_floats, int bf16, long long* lds_bytes) {
  const int cand[3] = {4, 2, 1};
  for (long long cap : {32768LL, 65536LL})
    for (int vc : cand) {
      if (bf16 && vc < 2) continue;
      const long long b = lds_floats(m, TPB * vc) * 4;
      if (b <= cap) {
        *lds_bytes = b;
        return vc;
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
  const int vc = pick_cols(m, lower_lds_floats, bf16, &lds);
  dim3 sgrid;
  if (vc && chan_grid(C, ld, TPB * vc, &sgrid)) {
    ProfScope ps(bf16 ? "lower_kernel<true>" : "lower_kernel<false>", 0.0, bytes, st);
#define CCT_LAUNCH_LOWER(BF, VC)                                                               \
  hipLaunchKernelGGL((lower_kernel<BF, VC>), sgrid, dim3(TPB), (size_t)lds, st, x, dt, ld,      \
                     (int)ncols, C, m, divP, divW, make_fastdiv(m.Wt), make_fastdiv(m.sw))
    if (bf16) {
      if (vc == 4) CCT_LAUNCH_LOWER(true, 4);
      else CCT_LAUNCH_LOWER(true, 2);
    } else {
      if (vc == 4) CCT_LAUNCH_LOWER(false, 4);
      else if (vc == 2) CCT_LAUNCH_LOWER(false, 2);
      else CCT_LAUNCH_LOWER(false, 1);
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
  const int vc = pick_cols(m, inv_lift_lds_floats, bf16, &lds);
  dim3 sgrid;
  if (vc && chan_grid(O, ld, TPB * vc, &sgrid)) {
    ProfScope ps(bf16 ? "inv_lift_kernel<true>" : "inv_lift_kernel<false>", 0.0, bytes, st);
#define CCT_LAUNCH_INV_LIFT(BF, VC)                                                            \
  hipLaunchKernelGGL((inv_lift_kernel<BF, VC>), sgrid, dim3(TPB), (size_t)lds, st, dy, drt, ld,  \
                     (int)ncols, O, m, divP, divW, divSh, divSw)
    if (bf16) {
      if (vc == 4) CCT_LAUNCH_INV_LIFT(true, 4);
      else CCT_LAUNCH_INV_LIFT(true, 2);
    } else {
      if (vc == 4) CCT_LAUNCH_INV_LIFT(false, 4);
      else if (vc == 2) CCT_LAUNCH_INV_LIFT(false, 2);
      else CCT_LAUNCH_INV_LIFT(false, 1);
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
