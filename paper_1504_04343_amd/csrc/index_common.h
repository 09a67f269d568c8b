// Helpers shared by the index-map kernels (lowering / lifting and their adjoints).
#pragma once

#include "cct_internal.h"

namespace cct {
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

inline bool grid_ok(long long blocks) { return blocks > 0 && blocks < 2147483647LL; }

}  // namespace
}  // namespace cct
