// Multiply phase of the backward-weights pass: dK^ = D^T dR^, i.e.
//     Cpart[s][m][n] = sum_{col in split s} A(m, col) * B(n, col)
// where the reduction runs over the columns of the transposed lowered matrices (all
// positions of all images of the chunk: 43 264 .. 774 400 terms for CaffeNet at batch 256)
// and the output is tiny.  The column range is therefore split over many workgroups
// (split-K); the partial products are summed afterwards in split order, which keeps the
// result bit-reproducible (no atomics).
//
// Both operands are contiguous along the reduction dimension.  Tiles are transposed on their
// way into LDS ([k][row] with an odd row stride, so both the transposing stores and the MFMA
// operand loads stay nearly conflict free).
#include <stdio.h>

#include "cct_internal.h"
#include "gemm_common.h"

namespace cct {
namespace {

constexpr int NT = 256;

template <int BM, int BN, int BK, int WM, int WN>
__global__ __launch_bounds__(NT) void gemm_nt_f32(GemmNT p, int tiles_m, int tiles_n) {
  constexpr int WAVES_N = BN / (32 * WN);
  constexpr int WAVES_M = BM / (32 * WM);
  static_assert(WAVES_M * WAVES_N == 4, "4 waves per workgroup");
  static_assert(NT % BK == 0, "BK divides 256");
  constexpr int ROWS_PER_PASS = NT / BK;
  static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "tile rows");
  constexpr int A_IT = BM / ROWS_PER_PASS;
  constexpr int B_IT = BN / ROWS_PER_PASS;
  constexpr int LDA = BM + 1, LDB = BN + 1;

  __shared__ float As[2][BK * LDA];
  __shared__ float Bs[2][BK * LDB];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;

  const int tile = blockIdx.x;
  const int tile_m = tile / tiles_n, tile_n = tile - tile_m * tiles_n;
  const int s = blockIdx.y;
  const int g = blockIdx.z;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int col_begin = s * p.split_len;
  const int col_end = min(p.Ncols, col_begin + p.split_len);

  gptr_f32 A = (gptr_f32)(p.A) + (long long)g * p.a_gs;
  gptr_f32 B = (gptr_f32)(p.B) + (long long)g * p.b_gs;

  const int tk = tid % BK;  // this thread's position along the reduction dimension
  const int tr = tid / BK;  // first tile row it copies

  float ra[A_IT], rb[B_IT];
  auto load_tile = [&](int c0) {
    const int col = c0 + tk;
    const bool ok = col < col_end;
    const long long aoff = ok ? col_offset(p.amap, col) : 0;
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
      const int m = m0 + tr + it * ROWS_PER_PASS;
      ra[it] = (ok && m < p.M) ? A[(long long)m * p.a_ms + aoff] : 0.f;
    }
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
      const int n = n0 + tr + it * ROWS_PER_PASS;
      rb[it] = (ok && n < p.N) ? B[(long long)n * p.b_ns + col] : 0.f;
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int it = 0; it < A_IT; ++it) As[buf][tk * LDA + tr + it * ROWS_PER_PASS] = ra[it];
#pragma unroll
    for (int it = 0; it < B_IT; ++it) Bs[buf][tk * LDB + tr + it * ROWS_PER_PASS] = rb[it];
  };

  floatx16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int lane_lo = lane & 31, lane_hi = lane >> 5;
  const int am = wave_m * WM * 32 + lane_lo;
  const int bn = wave_n * WN * 32 + lane_lo;

  const int ktiles = (col_end - col_begin + BK - 1) / BK;  // <= 0 for an empty split
  if (ktiles > 0) {
    load_tile(col_begin);
    store_tile(0);
  }
  __syncthreads();
  for (int t = 0; t < ktiles; ++t) {
    const int buf = t & 1;
    if (t + 1 < ktiles) load_tile(col_begin + (t + 1) * BK);
    mma_stage<BK, LDA, LDB, WM, WN>(&As[buf][lane_hi * LDA + am], &Bs[buf][lane_hi * LDB + bn], acc);
    if (t + 1 < ktiles) store_tile(buf ^ 1);
    __syncthreads();
  }

  float* __restrict__ C = p.Cpart + ((long long)s * p.G + g) * p.M * p.N;
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    const int n = n0 + bn + j * 32;
    if (n >= p.N) continue;
#pragma unroll
    for (int i = 0; i < WM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wave_m * WM * 32 + i * 32 + (r >> 2) * 8 + lane_hi * 4 + (r & 3);
        if (m < p.M) C[(long long)m * p.N + n] = acc[i][j][r];
      }
    }
  }
}

template <int BM, int BN, int BK, int WM, int WN>
int launch_f32(const GemmNT& p, hipStream_t st) {
  const int tiles_m = (p.M + BM - 1) / BM;
  const int tiles_n = (p.N + BN - 1) / BN;
  const long long tiles = (long long)tiles_m * tiles_n;
  if (tiles <= 0 || tiles >= 2147483647LL || p.S < 1 || p.S > 65535 || p.G > 65535)
    return CCT_EUNSUPPORTED;
  if (p.split_len % BK) return CCT_EINVAL;
  dim3 grid((unsigned)tiles, (unsigned)p.S, (unsigned)p.G);
  char name[96];
  snprintf(name, sizeof(name), "gemm_nt_f32<%d, %d, %d, %d, %d>", BM, BN, BK, WM, WN);
  ProfScope ps(name, 2.0 * p.M * p.N * p.Ncols * p.G,
               4.0 * ((double)p.M * p.Ncols + (double)p.N * p.Ncols + (double)p.M * p.N * p.S) * p.G,
               st);
  hipLaunchKernelGGL((gemm_nt_f32<BM, BN, BK, WM, WN>), grid, dim3(NT), 0, st, p, tiles_m, tiles_n);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

}  // namespace

void gemm_nt_tile(int M, int /*N*/, int* BM, int* BN, int* BK) {
  *BN = 128;
  *BK = 16;
  if (M <= 64)
    *BM = 64;
  else if (M % 128 != 0 && M % 96 == 0)
    *BM = 96;
  else
    *BM = 128;
}

int launch_gemm_nt(const GemmNT& p, hipStream_t st) {
  if (p.bf16) return CCT_EUNSUPPORTED;
  int BM, BN, BK;
  gemm_nt_tile(p.M, p.N, &BM, &BN, &BK);
  if (BM == 64) return launch_f32<64, 128, 16, 1, 2>(p, st);
  if (BM == 96) return launch_f32<96, 128, 16, 3, 1>(p, st);
  return launch_f32<128, 128, 16, 2, 2>(p, st);
}

}  // namespace cct
