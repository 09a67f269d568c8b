// Lifting phase (Sec. 2.1, fused with the bias add) and the adjoint of the lowering phase:
// the two kernels that READ a lowered matrix once and write the (k or k^2 times smaller)
// tensor.  HBM-bound on the read stream.
#include "cct_internal.h"
#include "index_common.h"

namespace cct {
namespace {

// Consecutive workgroup ids are dealt round-robin to the 8 XCDs, each with an L2 of its own.
// Neighbouring runs of output elements read neighbouring (often line-sharing) stretches of the
// matrix rows, so the kernels below renumber their workgroups: every XCD gets one contiguous
// range of runs and walks it in order, and a cache line that two neighbouring runs share is
// fetched from HBM once instead of once per XCD.
__device__ __forceinline__ int xcd_contiguous_block() {
  const int total = gridDim.x;
  const int per = total >> 3, rem = total & 7;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  return xcd * per + min(xcd, rem) + slot;
}

// ---------------------------------------------------------------------------------------
// Lifting phase fused with the bias add.  Each thread produces VEC consecutive output
// elements (one 16-byte store); for a fixed tap the lanes of a wave read consecutive
// (stride sw) columns of one R^ row, every R^ entry is read exactly once, and the VEC loads of
// a tap are independent, which keeps enough reads in flight to stream from HBM.
// ---------------------------------------------------------------------------------------
template <bool VSTORE>
__global__ __launch_bounds__(TPB) void lift_kernel(const float* __restrict__ rt, long long ld,
                                                   float* __restrict__ y,
                                                   const float* __restrict__ bias, int total, int O,
                                                   WinMap m, FastDiv divWt, FastDiv divPl,
                                                   FastDiv divO) {
  const int t0 = (xcd_contiguous_block() * TPB + threadIdx.x) * VEC;   // total < 2^31 checked by the launcher
  if (t0 >= total) return;
  const long long kk = (long long)m.Ki * m.Kj;
  const int PcG = m.Ha * m.Wb;
  long long base[VEC];
  int ra[VEC], cb[VEC];
  float acc[VEC];
  {
    int plane = fdiv(t0, divPl);               // n*O + o
    const int pix = t0 - plane * (m.Ht * m.Wt);
    int r = fdiv(pix, divWt);
    int c = pix - r * m.Wt;
    int n = fdiv(plane, divO);
    int o = plane - n * O;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const bool live = t0 + e < total;
      base[e] = (long long)o * kk * ld + (long long)n * PcG;
      ra[e] = live ? r * m.sh - m.ph : -(1 << 30);
      cb[e] = c * m.sw - m.pw;
      acc[e] = (bias && live) ? bias[o] : 0.0f;
      if (++c == m.Wt) {
        c = 0;
        if (++r == m.Ht) {
          r = 0;
          if (++o == O) {
            o = 0;
            ++n;
          }
        }
      }
    }
  }
  for (int i = 0; i < m.Ki; ++i) {
    for (int j = 0; j < m.Kj; ++j) {
      const long long tap = (long long)(i * m.Kj + j) * ld;
      float v[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const int a = ra[e] + i, b = cb[e] + j;
        const bool ok = (unsigned)a < (unsigned)m.Ha && (unsigned)b < (unsigned)m.Wb;
        const float t = rt[ok ? base[e] + tap + a * m.Wb + b : 0];
        v[e] = ok ? t : 0.0f;
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] += v[e];
    }
  }
  if (VSTORE && t0 + VEC <= total) {
    *reinterpret_cast<float4*>(y + t0) = make_float4(acc[0], acc[1], acc[2], acc[3]);
  } else {
#pragma unroll
    for (int e = 0; e < VEC; ++e)
      if (t0 + e < total) y[t0 + e] = acc[e];
  }
}

// Adjoint of the lowering phase as a gather (no atomics): every dx pixel sums the entries of
// the lowered gradient that were copied from it.  Only taps i = (h+ph) mod sh, +sh, +2sh, ...
// (and likewise j) can have come from pixel (h, w), so the tap loops step by the stride.
template <bool VSTORE>
__global__ __launch_bounds__(TPB) void inv_lower_kernel(const float* __restrict__ ddt, long long ld,
                                                        float* __restrict__ dx, int total, int C,
                                                        WinMap m, FastDiv divWt, FastDiv divPl,
                                                        FastDiv divC, FastDiv divSh, FastDiv divSw) {
  const int t0 = (xcd_contiguous_block() * TPB + threadIdx.x) * VEC;
  if (t0 >= total) return;
  const long long kk = (long long)m.Ki * m.Kj;
  const int PcG = m.Ha * m.Wb;
  long long base[VEC];
  int i0[VEC], a0[VEC], j0[VEC], b0[VEC];
  float acc[VEC];
  {
    int plane = fdiv(t0, divPl);               // n*C + ch
    const int pix = t0 - plane * (m.Ht * m.Wt);
    int h = fdiv(pix, divWt);
    int w = pix - h * m.Wt;
    int n = fdiv(plane, divC);
    int ch = plane - n * C;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const bool live = t0 + e < total;
      base[e] = (long long)ch * kk * ld + (long long)n * PcG;
      // first admissible taps and the grid coordinates they map to
      a0[e] = fdiv(h + m.ph, divSh);
      i0[e] = live ? h + m.ph - a0[e] * m.sh : (1 << 30);
      b0[e] = fdiv(w + m.pw, divSw);
      j0[e] = w + m.pw - b0[e] * m.sw;
      acc[e] = 0.0f;
      if (++w == m.Wt) {
        w = 0;
        if (++h == m.Ht) {
          h = 0;
          if (++ch == C) {
            ch = 0;
            ++n;
          }
        }
      }
    }
  }
  const int nti = (m.Ki + m.sh - 1) / m.sh, ntj = (m.Kj + m.sw - 1) / m.sw;
  for (int ti = 0; ti < nti; ++ti) {
    for (int tj = 0; tj < ntj; ++tj) {
      float v[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const int i = i0[e] + ti * m.sh, a = a0[e] - ti;
        const int j = j0[e] + tj * m.sw, b = b0[e] - tj;
        const bool ok = i < m.Ki && j < m.Kj && (unsigned)a < (unsigned)m.Ha &&
                        (unsigned)b < (unsigned)m.Wb;
        const float t = ddt[ok ? base[e] + (long long)(i * m.Kj + j) * ld + a * m.Wb + b : 0];
        v[e] = ok ? t : 0.0f;
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] += v[e];
    }
  }
  if (VSTORE && t0 + VEC <= total) {
    *reinterpret_cast<float4*>(dx + t0) = make_float4(acc[0], acc[1], acc[2], acc[3]);
  } else {
#pragma unroll
    for (int e = 0; e < VEC; ++e)
      if (t0 + e < total) dx[t0 + e] = acc[e];
  }
}

}  // namespace

int launch_lift(const float* rt, long long ld, float* y, const float* bias, int nimg, int O,
                const WinMap& m, hipStream_t st) {
  const long long total = (long long)nimg * O * m.Ht * m.Wt;
  const long long blocks = (total + TPB * VEC - 1) / (TPB * VEC);
  if (!grid_ok(blocks) || total >= 2147483647LL - TPB * VEC) return CCT_EUNSUPPORTED;
  ProfScope ps("lift_kernel", 0.0,
               4.0 * total + 4.0 * O * m.Ki * m.Kj * (double)nimg * m.Ha * m.Wb, st);
  if (reinterpret_cast<uintptr_t>(y) % 16 == 0)
    hipLaunchKernelGGL(lift_kernel<true>, dim3((unsigned)blocks), dim3(TPB), 0, st, rt, ld, y, bias,
                       (int)total, O, m, make_fastdiv(m.Wt), make_fastdiv(m.Ht * m.Wt),
                       make_fastdiv(O));
  else
    hipLaunchKernelGGL(lift_kernel<false>, dim3((unsigned)blocks), dim3(TPB), 0, st, rt, ld, y, bias,
                       (int)total, O, m, make_fastdiv(m.Wt), make_fastdiv(m.Ht * m.Wt),
                       make_fastdiv(O));
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int launch_inv_lower(const float* ddt, long long ld, float* dx, int nimg, int C, const WinMap& m,
                     hipStream_t st) {
  const long long total = (long long)nimg * C * m.Ht * m.Wt;
  const long long blocks = (total + TPB * VEC - 1) / (TPB * VEC);
  if (!grid_ok(blocks) || total >= 2147483647LL - TPB * VEC) return CCT_EUNSUPPORTED;
  ProfScope ps("inv_lower_kernel", 0.0,
               4.0 * total + 4.0 * C * m.Ki * m.Kj * (double)nimg * m.Ha * m.Wb, st);
  if (reinterpret_cast<uintptr_t>(dx) % 16 == 0)
    hipLaunchKernelGGL(inv_lower_kernel<true>, dim3((unsigned)blocks), dim3(TPB), 0, st, ddt, ld, dx,
                       (int)total, C, m, make_fastdiv(m.Wt), make_fastdiv(m.Ht * m.Wt),
                       make_fastdiv(C), make_fastdiv(m.sh), make_fastdiv(m.sw));
  else
    hipLaunchKernelGGL(inv_lower_kernel<false>, dim3((unsigned)blocks), dim3(TPB), 0, st, ddt, ld, dx,
                       (int)total, C, m, make_fastdiv(m.Wt), make_fastdiv(m.Ht * m.Wt),
                       make_fastdiv(C), make_fastdiv(m.sh), make_fastdiv(m.sw));
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

}  // namespace cct
