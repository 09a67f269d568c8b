// Pieces shared by the two GEMM kernels (gemm_tn.hip, gemm_nt.hip).
#pragma once

#include "cct_internal.h"

namespace cct {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
// explicit global address space, so that loads are global_load (vmcnt only), not flat_load
typedef const float __attribute__((address_space(1)))* gptr_f32;
typedef const f32x4 __attribute__((address_space(1)))* gptr_f32x4;

// n / d for n < 2^31 with M = ceil(2^sh / d), sh = 31 + ceil(log2 d) (see make_fastdiv_parts)
__device__ __forceinline__ int fdiv_u(int n, unsigned M, int sh) {
  return (int)(((unsigned long long)(unsigned)n * M) >> sh);
}

__device__ __forceinline__ long long col_offset(const ColMap& cm, int col) {
  const int n = fdiv_u(col, cm.divM, cm.divsh);
  return (long long)n * cm.img_stride + (col - n * cm.P);
}

// One K-step of the wave tile: operands come from LDS ([k][row] layout), lanes 0..31 supply k,
// lanes 32..63 supply k+1 of their row/column.  The LDS reads of step s+1 are issued before the
// MFMAs of step s.
template <int BK, int LDA, int LDB, int WM, int WN>
__device__ __forceinline__ void mma_stage(const float* __restrict__ as, const float* __restrict__ bs,
                                          floatx16 (&acc)[WM][WN]) {
  float a[2][WM], b[2][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i) a[0][i] = as[i * 32];
#pragma unroll
  for (int j = 0; j < WN; ++j) b[0][j] = bs[j * 32];
#pragma unroll
  for (int s = 0; s < BK / 2; ++s) {
    const int cur = s & 1, nxt = cur ^ 1;
    if (s + 1 < BK / 2) {
#pragma unroll
      for (int i = 0; i < WM; ++i) a[nxt][i] = as[(s + 1) * 2 * LDA + i * 32];
#pragma unroll
      for (int j = 0; j < WN; ++j) b[nxt][j] = bs[(s + 1) * 2 * LDB + j * 32];
    }
    __builtin_amdgcn_sched_barrier(0);  // keep the next step's LDS reads ahead of these MFMAs
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int j = 0; j < WN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
}

}  // namespace
}  // namespace cct
