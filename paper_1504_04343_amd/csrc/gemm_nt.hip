// Multiply phase of the backward-weights pass: dK^ = D^T dR^, i.e.
//     Cpart[s][m][n] = sum_{col in split s} A(m, col) * B(n, col)
// where the reduction runs over the columns of the transposed lowered matrices (all
// positions of all images of the chunk: 43 264 .. 774 400 terms for CaffeNet at batch 256)
// and the output is tiny.  The column range is therefore split over many workgroups
// (split-K); the partial products are summed afterwards in split order, which keeps the
// result bit-reproducible (no atomics).
//
// Both operands are contiguous along the reduction dimension, and they stay that way in LDS
// ([row][k], rows padded by 4 floats): no transposition anywhere, 16-byte global loads, LDS
// writes and LDS reads.
#include <stdio.h>

#include "cct_internal.h"
#include "gemm_common.h"

namespace cct {
namespace {

constexpr int NT = 256;

// K-step over 8 reduction indices with operands stored [row][k] in LDS: every lane fetches
// 4 consecutive k of its row with one 16-byte LDS read (lanes 0..31 take k = 8q..8q+3, lanes
// 32..63 take k = 8q+4..8q+7) and MFMA e of the group consumes component e.  Any assignment of
// reduction indices to (lane half, component) is valid as long as A and B use the same one.
template <int BK, int LDK, int WM, int WN>
__device__ __forceinline__ void mma_stage_kcontig(const float* __restrict__ as,
                                                  const float* __restrict__ bs,
                                                  floatx16 (&acc)[WM][WN]) {
  f32x4 a[2][WM], b[2][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i) a[0][i] = *reinterpret_cast<const f32x4*>(as + i * 32 * LDK);
#pragma unroll
  for (int j = 0; j < WN; ++j) b[0][j] = *reinterpret_cast<const f32x4*>(bs + j * 32 * LDK);
#pragma unroll
  for (int q = 0; q < BK / 8; ++q) {
    const int cur = q & 1, nxt = cur ^ 1;
    if (q + 1 < BK / 8) {
#pragma unroll
      for (int i = 0; i < WM; ++i)
        a[nxt][i] = *reinterpret_cast<const f32x4*>(as + i * 32 * LDK + (q + 1) * 8);
#pragma unroll
      for (int j = 0; j < WN; ++j)
        b[nxt][j] = *reinterpret_cast<const f32x4*>(bs + j * 32 * LDK + (q + 1) * 8);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
          acc[i][j] =
              __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][i][e], b[cur][j][e], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Fast division constants of the gather mode (see make_fastdiv_parts).
struct NtGather {
  unsigned mP, mWout, mKK, mK;
  int sP, sWout, sKK, sK;
};

// AVEC: A rows are plain 16-byte aligned matrix rows (inverse-lifted dy of Types 2/3);
// otherwise A is dy read in place through the NCHW column map (Type 1), 4-byte loads.
// BG (with !AVEC): B is not a lowered matrix but the tensor x of an unpadded layer, and row
// n = (ci, i, j) of the Type-1 lowering is gathered while the tile is loaded.  Both operands then
// go through buffer loads: a thread's rows give fixed byte offsets, the column of the tile adds
// one offset per tile, columns past the end of the split fail the range check and load as zero.
template <int BM, int BN, int BK, int WM, int WN, bool AVEC, bool BG>
__global__ __launch_bounds__(NT) void gemm_nt_f32(GemmNT p, NtGather ng, int tiles_m, int tiles_n) {
  static_assert(!(AVEC && BG), "the gather mode reads dy in place");
  constexpr int WAVES_N = BN / (32 * WN);
  constexpr int WAVES_M = BM / (32 * WM);
  static_assert(WAVES_M * WAVES_N == 4, "4 waves per workgroup");
  static_assert(BK % 8 == 0 && NT % BK == 0, "BK");
  constexpr int LDK = BK + 4;            // 16-byte aligned rows, conflict-free 16-byte reads
  constexpr int KQ = BK / 4;             // 16-byte vectors per tile row
  constexpr int AV_IT = BM * KQ / NT;    // vector loads per thread (A, vector path)
  constexpr int BV_IT = BN * KQ / NT;
  constexpr int AS_IT = BM * BK / NT;    // scalar loads per thread (A, scalar path)
  constexpr int AS_ROWS = NT / BK;       // tile rows covered per scalar pass
  constexpr int BS_IT = BN * BK / NT;    // scalar loads per thread (B, gather mode)
  static_assert((BM * KQ) % NT == 0 && (BN * KQ) % NT == 0, "tile/thread split");

  __shared__ __attribute__((aligned(16))) float As[2][BM * LDK];
  __shared__ __attribute__((aligned(16))) float Bs[2][BN * LDK];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;

  // Workgroup order: consecutive ids go round-robin over the 8 XCDs, so give every XCD a
  // contiguous run of (split, tile) pairs with the tile index fastest: all tiles of one split
  // read the same column range of A and B and then share it through that XCD's L2.
  int bid = blockIdx.x;
  {
    const int total = tiles_m * tiles_n * p.S;
    const int per = total >> 3, rem = total & 7;
    const int xcd = bid & 7, slot = bid >> 3;
    bid = xcd * per + min(xcd, rem) + slot;
  }
  const int ntiles = tiles_m * tiles_n;
  const int s = bid / ntiles;
  const int tile = bid - s * ntiles;
  const int tile_m = tile / tiles_n, tile_n = tile - tile_m * tiles_n;
  const int g = blockIdx.y;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int col_begin = s * p.split_len;
  const int col_end = min(p.Ncols, col_begin + p.split_len);

  gptr_f32 A = (gptr_f32)(p.A) + (long long)g * p.a_gs;
  gptr_f32 B = (gptr_f32)(p.B) + (long long)g * p.b_gs;

  // Rows beyond M / N are clamped to the last valid row: their products land in rows/columns of
  // the tile that are never stored.  Columns beyond Ncols inside a plain lowered matrix are zero
  // padding written by the lowering kernels, so plain rows need no column guard.
  gptr_f32 b_src[BG ? 1 : BV_IT];
  int b_dst[BG ? 1 : BV_IT];
  if (!BG) {
#pragma unroll
    for (int it = 0; it < BV_IT; ++it) {
      const int v = tid + it * NT;
      const int row = v / KQ, kq = v % KQ;
      b_src[it] = B + (long long)min(n0 + row, p.N - 1) * p.b_ns + col_begin + kq * 4;
      b_dst[it] = row * LDK + kq * 4;
    }
  }
  gptr_f32 av_src[AVEC ? AV_IT : 1];
  int av_dst[AVEC ? AV_IT : 1];
  const int as_k = tid % BK, as_r0 = tid / BK;
  // gather mode: fixed byte offsets of this thread's dy rows and of its taps (ci, i, j) in x
  unsigned g_arow[BG ? AS_IT : 1], g_btap[BG ? BS_IT : 1];
  const int gP = p.gHout * p.gWout, gHW = p.gH * p.gW;
  const long long gCHW = (long long)p.gC * gHW;
  if (BG) {
#pragma unroll
    for (int it = 0; it < AS_IT; ++it)
      g_arow[it] = (unsigned)(min(m0 + as_r0 + it * AS_ROWS, p.M - 1) * (int)p.a_ms) * 4u;
#pragma unroll
    for (int it = 0; it < BS_IT; ++it) {
      const int n = min(n0 + as_r0 + it * AS_ROWS, p.N - 1);
      const int ci = fdiv_u(n, ng.mKK, ng.sKK), t = n - ci * p.gK * p.gK;
      const int ti = fdiv_u(t, ng.mK, ng.sK), tj = t - ti * p.gK;
      g_btap[it] = (unsigned)(ci * gHW + ti * p.gW + tj) * 4u;
    }
  }
  if (AVEC) {
#pragma unroll
    for (int it = 0; it < AV_IT; ++it) {
      const int v = tid + it * NT;
      const int row = v / KQ, kq = v % KQ;
      av_src[it] = A + (long long)min(m0 + row, p.M - 1) * p.a_ms + col_begin + kq * 4;
      av_dst[it] = row * LDK + kq * 4;
    }
  }

  f32x4 rb[BG ? 1 : BV_IT];
  f32x4 rav[AVEC ? AV_IT : 1];
  float ras[AVEC ? 1 : AS_IT];
  float rbs[BG ? BS_IT : 1];

#define CCT_NT_LOAD(C0)                                                                   \
  {                                                                                       \
  if (BG) {                                                                               \
    const int c0_ = (C0);                                                                 \
    const int n_f = fdiv_u(c0_, ng.mP, ng.sP);   /* first image of the tile (uniform) */  \
    const int col = c0_ + as_k;                                                           \
    const bool ok = col < col_end;                                                        \
    const int cc = ok ? col : c0_;                                                        \
    const int n = fdiv_u(cc, ng.mP, ng.sP), pix = cc - n * gP;                            \
    const int r = fdiv_u(pix, ng.mWout, ng.sWout), c = pix - r * p.gWout;                 \
    const unsigned aoff =                                                                 \
        ok ? ((unsigned)(n - n_f) * (unsigned)p.amap.img_stride + (unsigned)pix) * 4u     \
           : 0x80000000u;                                                                 \
    const unsigned boff =                                                                 \
        ok ? ((unsigned)(n - n_f) * (unsigned)gCHW + (unsigned)((r * p.gW + c) * p.gs)) * 4u \
           : 0x80000000u;                                                                 \
    const __amdgpu_buffer_rsrc_t rsa = __builtin_amdgcn_make_buffer_rsrc(                 \
        const_cast<float*>(reinterpret_cast<const float*>(p.A) + (long long)g * p.a_gs +  \
                           (long long)n_f * p.amap.img_stride),                           \
        0, 0x7fffffff, 0x00020000);                                                       \
    const __amdgpu_buffer_rsrc_t rsb = __builtin_amdgcn_make_buffer_rsrc(                 \
        const_cast<float*>(reinterpret_cast<const float*>(p.B) + (long long)g * p.b_gs +  \
                           (long long)n_f * gCHW),                                        \
        0, 0x7fffffff, 0x00020000);                                                       \
    _Pragma("unroll") for (int it = 0; it < AS_IT; ++it)                                  \
      ras[it] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(           \
                                              rsa, (int)(g_arow[it] + aoff), 0, 0));      \
    _Pragma("unroll") for (int it = 0; it < BS_IT; ++it)                                  \
      rbs[it] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(           \
                                              rsb, (int)(g_btap[it] + boff), 0, 0));      \
  } else {                                                                                \
    _Pragma("unroll") for (int it = 0; it < BV_IT; ++it) {                                \
      rb[it] = *(gptr_f32x4)(b_src[it]);                                                  \
      b_src[it] += BK;                                                                    \
    }                                                                                     \
    if (AVEC) {                                                                           \
      _Pragma("unroll") for (int it = 0; it < AV_IT; ++it) {                              \
        rav[it] = *(gptr_f32x4)(av_src[it]);                                              \
        av_src[it] += BK;                                                                 \
      }                                                                                   \
    } else {                                                                              \
      const int col = (C0) + as_k;                                                        \
      const bool ok = col < col_end;                                                      \
      const long long aoff = ok ? col_offset(p.amap, col) : 0;                            \
      _Pragma("unroll") for (int it = 0; it < AS_IT; ++it) {                              \
        const int m = min(m0 + as_r0 + it * AS_ROWS, p.M - 1);                            \
        const float val = A[(long long)m * p.a_ms + aoff];                                \
        ras[it] = ok ? val : 0.f;                                                         \
      }                                                                                   \
    }                                                                                     \
  }                                                                                       \
  }
#define CCT_NT_STORE(BUF)                                                                 \
  {                                                                                       \
    if (BG) {                                                                             \
      _Pragma("unroll") for (int it = 0; it < BS_IT; ++it)                                \
        Bs[BUF][(as_r0 + it * AS_ROWS) * LDK + as_k] = rbs[it];                           \
    } else {                                                                              \
      _Pragma("unroll") for (int it = 0; it < BV_IT; ++it)                                \
        *reinterpret_cast<f32x4*>(&Bs[BUF][b_dst[it]]) = rb[it];                          \
    }                                                                                     \
    if (AVEC) {                                                                           \
      _Pragma("unroll") for (int it = 0; it < AV_IT; ++it)                                \
        *reinterpret_cast<f32x4*>(&As[BUF][av_dst[it]]) = rav[it];                        \
    } else {                                                                              \
      _Pragma("unroll") for (int it = 0; it < AS_IT; ++it)                                \
        As[BUF][(as_r0 + it * AS_ROWS) * LDK + as_k] = ras[it];                           \
    }                                                                                     \
  }

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
  const int a_lds = am * LDK + lane_hi * 4;
  const int b_lds = bn * LDK + lane_hi * 4;

  // Main loop: same software pipeline as the forward GEMM (operand reads one step ahead, the
  // next tile's LDS writes in the middle of the current tile, the barrier before the last step).
  const int ktiles = (col_end - col_begin + BK - 1) / BK;  // <= 0 for an empty split
  constexpr int QS = BK / 8;
  f32x4 a[2][WM], b[2][WN];
  if (ktiles > 0) {
    CCT_NT_LOAD(col_begin);
    CCT_NT_STORE(0);
  }
  __syncthreads();
  if (ktiles > 1) CCT_NT_LOAD(col_begin + BK);
  if (ktiles > 0) {
#pragma unroll
    for (int i = 0; i < WM; ++i) a[0][i] = *reinterpret_cast<const f32x4*>(&As[0][a_lds + i * 32 * LDK]);
#pragma unroll
    for (int j = 0; j < WN; ++j) b[0][j] = *reinterpret_cast<const f32x4*>(&Bs[0][b_lds + j * 32 * LDK]);
  }
  for (int t = 0; t < ktiles; ++t) {
    const int buf = t & 1;
    const bool more = t + 1 < ktiles;
    const float* as = &As[buf][a_lds];
    const float* bs = &Bs[buf][b_lds];
#pragma unroll
    for (int q = 0; q < QS; ++q) {
      const int cur = q & 1, nxt = cur ^ 1;
      if (q + 1 < QS) {
#pragma unroll
        for (int i = 0; i < WM; ++i)
          a[nxt][i] = *reinterpret_cast<const f32x4*>(as + i * 32 * LDK + (q + 1) * 8);
#pragma unroll
        for (int j = 0; j < WN; ++j)
          b[nxt][j] = *reinterpret_cast<const f32x4*>(bs + j * 32 * LDK + (q + 1) * 8);
      } else {
        __syncthreads();
        if (more) {
#pragma unroll
          for (int i = 0; i < WM; ++i)
            a[nxt][i] = *reinterpret_cast<const f32x4*>(&As[buf ^ 1][a_lds + i * 32 * LDK]);
#pragma unroll
          for (int j = 0; j < WN; ++j)
            b[nxt][j] = *reinterpret_cast<const f32x4*>(&Bs[buf ^ 1][b_lds + j * 32 * LDK]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
          for (int j = 0; j < WN; ++j)
            acc[i][j] =
                __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][i][e], b[cur][j][e], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (q == QS / 2 - 1 && more) {
        CCT_NT_STORE(buf ^ 1);
        if (t + 2 < ktiles) CCT_NT_LOAD(col_begin + (t + 2) * BK);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
#undef CCT_NT_LOAD
#undef CCT_NT_STORE

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

// bf16 operands (both plain lowered matrices written in bf16 by the lowering kernels), fp32
// accumulate.  Same structure as the fp32 kernel; a lane feeds v_mfma_f32_32x32x8_bf16_1k with 4
// consecutive reduction indices of its row, i.e. one 8-byte LDS read (lanes 32..63 take the
// next 4), and LDS rows hold BK + 8 bf16 so that 16-byte writes stay aligned.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef const u32x4 __attribute__((address_space(1)))* gptr_u32x4;
template <int BM, int BN, int BK, int WM, int WN>
__global__ __launch_bounds__(NT) void gemm_nt_bf16(GemmNT p, int tiles_m, int tiles_n) {
  constexpr int WAVES_N = BN / (32 * WN);
  constexpr int WAVES_M = BM / (32 * WM);
  static_assert(WAVES_M * WAVES_N == 4, "4 waves per workgroup");
  static_assert(BK % 8 == 0, "BK");
  constexpr int LDK = BK + 8;            // bf16 elements per LDS row
  constexpr int KV = BK / 8;             // 16-byte vectors per tile row
  constexpr int AV_IT = (BM * KV + NT - 1) / NT;
  constexpr int BV_IT = (BN * KV + NT - 1) / NT;

  __shared__ __attribute__((aligned(16))) unsigned short As[2][BM * LDK];
  __shared__ __attribute__((aligned(16))) unsigned short Bs[2][BN * LDK];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
  int bid = blockIdx.x;
  {
    const int total = tiles_m * tiles_n * p.S;
    const int per = total >> 3, rem = total & 7;
    const int xcd = bid & 7, slot = bid >> 3;
    bid = xcd * per + min(xcd, rem) + slot;
  }
  const int ntiles = tiles_m * tiles_n;
  const int s = bid / ntiles;
  const int tile = bid - s * ntiles;
  const int tile_m = tile / tiles_n, tile_n = tile - tile_m * tiles_n;
  const int g = blockIdx.y;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int col_begin = s * p.split_len;
  const int col_end = min(p.Ncols, col_begin + p.split_len);

  const unsigned short* A = reinterpret_cast<const unsigned short*>(p.A) + (long long)g * p.a_gs;
  const unsigned short* B = reinterpret_cast<const unsigned short*>(p.B) + (long long)g * p.b_gs;
  const unsigned short* a_src[AV_IT];
  const unsigned short* b_src[BV_IT];
  int a_dst[AV_IT], b_dst[BV_IT];
#pragma unroll
  for (int it = 0; it < AV_IT; ++it) {
    const int v = min(tid + it * NT, BM * KV - 1);
    const int row = v / KV, kv = v % KV;
    a_src[it] = A + (long long)min(m0 + row, p.M - 1) * p.a_ms + col_begin + kv * 8;
    a_dst[it] = row * LDK + kv * 8;
  }
#pragma unroll
  for (int it = 0; it < BV_IT; ++it) {
    const int v = min(tid + it * NT, BN * KV - 1);
    const int row = v / KV, kv = v % KV;
    b_src[it] = B + (long long)min(n0 + row, p.N - 1) * p.b_ns + col_begin + kv * 8;
    b_dst[it] = row * LDK + kv * 8;
  }
  u32x4 ra[AV_IT], rb[BV_IT];

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
  const int a_lds = am * LDK + lane_hi * 4;
  const int b_lds = bn * LDK + lane_hi * 4;

  const int ktiles = (col_end - col_begin + BK - 1) / BK;
  for (int t = 0; t < ktiles; ++t) {
#pragma unroll
    for (int it = 0; it < AV_IT; ++it) {
      ra[it] = *(gptr_u32x4)(a_src[it]);
      a_src[it] += BK;
    }
#pragma unroll
    for (int it = 0; it < BV_IT; ++it) {
      rb[it] = *(gptr_u32x4)(b_src[it]);
      b_src[it] += BK;
    }
    const int buf = t & 1;
#pragma unroll
    for (int it = 0; it < AV_IT; ++it) *reinterpret_cast<u32x4*>(&As[buf][a_dst[it]]) = ra[it];
#pragma unroll
    for (int it = 0; it < BV_IT; ++it) *reinterpret_cast<u32x4*>(&Bs[buf][b_dst[it]]) = rb[it];
    __syncthreads();  // two buffers: the next iteration writes the other one
#pragma unroll
    for (int q = 0; q < BK / 8; ++q) {
      shortx4 a[WM], b[WN];
#pragma unroll
      for (int i = 0; i < WM; ++i)
        a[i] = *reinterpret_cast<const shortx4*>(&As[buf][a_lds + i * 32 * LDK + q * 8]);
#pragma unroll
      for (int j = 0; j < WN; ++j)
        b[j] = *reinterpret_cast<const shortx4*>(&Bs[buf][b_lds + j * 32 * LDK + q * 8]);
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a[i], b[j], acc[i][j], 0, 0, 0);
    }
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
int launch_bf16(const GemmNT& p, hipStream_t st) {
  const int tiles_m = (p.M + BM - 1) / BM;
  const int tiles_n = (p.N + BN - 1) / BN;
  const long long tiles = (long long)tiles_m * tiles_n;
  if (tiles <= 0 || p.S < 1 || tiles * p.S >= 2147483647LL || p.G > 65535) return CCT_EUNSUPPORTED;
  if (p.split_len % BK) return CCT_EINVAL;
  // both operands must be plain bf16 lowered matrices with 16-byte aligned rows
  if (p.amap.P != 2147483647 || p.a_ms % 8 || p.a_gs % 8 || p.b_ns % 8 || p.b_gs % 8 ||
      reinterpret_cast<uintptr_t>(p.A) % 16 || reinterpret_cast<uintptr_t>(p.B) % 16)
    return CCT_EINVAL;
  dim3 grid((unsigned)(tiles * p.S), (unsigned)p.G);
  char name[96];
  snprintf(name, sizeof(name), "gemm_nt_bf16<%d, %d, %d, %d, %d>", BM, BN, BK, WM, WN);
  ProfScope ps(name, 2.0 * p.M * p.N * p.Ncols * p.G,
               (2.0 * ((double)p.M * p.Ncols + (double)p.N * p.Ncols) + 4.0 * (double)p.M * p.N * p.S) *
                   p.G,
               st);
  hipLaunchKernelGGL((gemm_nt_bf16<BM, BN, BK, WM, WN>), grid, dim3(NT), 0, st, p, tiles_m, tiles_n);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

template <int BM, int BN, int BK, int WM, int WN>
int launch_f32(const GemmNT& p, hipStream_t st) {
  const int tiles_m = (p.M + BM - 1) / BM;
  const int tiles_n = (p.N + BN - 1) / BN;
  const long long tiles = (long long)tiles_m * tiles_n;
  if (tiles <= 0 || p.S < 1 || tiles * p.S >= 2147483647LL || p.G > 65535) return CCT_EUNSUPPORTED;
  if (p.split_len % BK) return CCT_EINVAL;
  dim3 grid((unsigned)(tiles * p.S), (unsigned)p.G);
  char name[96];
  NtGather ng;
  memset(&ng, 0, sizeof(ng));
  if (p.gather) {
    // fused lowering: dy in place, x gathered; 32-bit byte offsets from the tile's first image
    const long long P = (long long)p.gHout * p.gWout;
    const long long T = (BK - 1) / P + 2;   // images a tile of BK positions can span
    if (p.amap.P != P || p.a_ms != P || p.gK < 1 ||
        (T + 1) * p.amap.img_stride >= (1LL << 29) ||
        (T + 1) * (long long)p.gC * p.gH * p.gW >= (1LL << 29))
      return CCT_EUNSUPPORTED;
    make_fastdiv_parts((int)P, &ng.mP, &ng.sP);
    make_fastdiv_parts(p.gWout, &ng.mWout, &ng.sWout);
    make_fastdiv_parts(p.gK * p.gK, &ng.mKK, &ng.sKK);
    make_fastdiv_parts(p.gK, &ng.mK, &ng.sK);
    snprintf(name, sizeof(name), "gemm_nt_f32<%d, %d, %d, %d, %d, gather>", BM, BN, BK, WM, WN);
    const double x_bytes = 4.0 * ((double)p.Ncols / P) * p.gC * p.gH * p.gW;
    ProfScope ps(name, 2.0 * p.M * p.N * p.Ncols * p.G,
                 x_bytes + 4.0 * ((double)p.M * p.Ncols + (double)p.M * p.N * p.S) * p.G, st);
    hipLaunchKernelGGL((gemm_nt_f32<BM, BN, BK, WM, WN, false, true>), grid, dim3(NT), 0, st, p, ng,
                       tiles_m, tiles_n);
    CCT_CHECK_LAUNCH();
    return CCT_OK;
  }
  // B must be a plain lowered matrix with 16-byte aligned rows (the lowering kernels write it so)
  if (p.b_ns % 4 || p.b_gs % 4 || reinterpret_cast<uintptr_t>(p.B) % 16) return CCT_EINVAL;
  const bool avec = p.amap.P == 2147483647 && p.a_ms % 4 == 0 && p.a_gs % 4 == 0 &&
                    reinterpret_cast<uintptr_t>(p.A) % 16 == 0;
  snprintf(name, sizeof(name), "gemm_nt_f32<%d, %d, %d, %d, %d, %s>", BM, BN, BK, WM, WN,
           avec ? "true" : "false");
  ProfScope ps(name, 2.0 * p.M * p.N * p.Ncols * p.G,
               4.0 * ((double)p.M * p.Ncols + (double)p.N * p.Ncols + (double)p.M * p.N * p.S) * p.G,
               st);
  if (avec)
    hipLaunchKernelGGL((gemm_nt_f32<BM, BN, BK, WM, WN, true, false>), grid, dim3(NT), 0, st, p, ng,
                       tiles_m, tiles_n);
  else
    hipLaunchKernelGGL((gemm_nt_f32<BM, BN, BK, WM, WN, false, false>), grid, dim3(NT), 0, st, p,
                       ng, tiles_m, tiles_n);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

}  // namespace

void gemm_nt_tile(int M, int /*N*/, int* BM, int* BN, int* BK) {
  *BN = 128;
  *BK = 32;
  if (M <= 64)
    *BM = 64;
  else if (M % 128 != 0 && M % 96 == 0)
    *BM = 96;
  else
    *BM = 128;
}

bool gemm_nt_gather_fits(int C, int H, int W, int O, int Hout, int Wout) {
  int BM, BN, BK;
  gemm_nt_tile(1, 1, &BM, &BN, &BK);
  const long long P = (long long)Hout * Wout;
  const long long T = (BK - 1) / P + 2;
  return (T + 1) * O * P < (1LL << 29) && (T + 1) * (long long)C * H * W < (1LL << 29);
}

int launch_gemm_nt(const GemmNT& p0, hipStream_t st) {
  GemmNT p = p0;
  colmap_prepare(&p.amap);
  int BM, BN, BK;
  gemm_nt_tile(p.M, p.N, &BM, &BN, &BK);
  if (p.gather && p.bf16) return CCT_EUNSUPPORTED;
  if (p.bf16) {
    if (BM == 64) return launch_bf16<64, 128, 32, 1, 2>(p, st);
    if (BM == 96) return launch_bf16<96, 128, 32, 3, 1>(p, st);
    return launch_bf16<128, 128, 32, 2, 2>(p, st);
  }
  if (BM == 64) return launch_f32<64, 128, 32, 1, 2>(p, st);
  if (BM == 96) return launch_f32<96, 128, 32, 3, 1>(p, st);
  return launch_f32<128, 128, 32, 2, 2>(p, st);
}

}  // namespace cct
