// Fused backward-weights pass: the Type-1 product dK^ = dR^T D^ (Sec. 2.1 read backwards)
//     Cpart[s][q][oo][(ci,i,j)] = sum_{pos in split s} dy[n, q*Og+oo, r, c] * xpad[n, q*Cg+ci, r*s+i, c*s+j]
// without a lowered matrix in HBM.  The reduction runs over positions pos = (n, r, c); it is cut
// into splits (one per workgroup, summed afterwards in split order) and every split into chunks
// of 32 positions.  Per chunk a workgroup stages in LDS
//   - the dy tile [BM kernels][32 positions] (positions contiguous, as in the plain
//     backward-weights GEMM), and
//   - the zero-padded input rows that the 32 positions can reach, for the input channels its 128
//     lowered rows (ci,i,j) touch: staged row u holds the plane [channel][padded column] of one
//     input row, ROWP floats apart,
// and a lane gets its MFMA B operand for lowered row (ci,i,j) and position k with one LDS read at
//     (i*ROWP + ci*Wp + j)  +  posoff[k],      posoff[k] = staged row of r(k) * ROWP + c(k)*stride,
// a per-lane constant plus a per-position offset from a 32-entry table in LDS.
//
// Vector-ALU instructions are not hidden behind MFMAs on this chip (each costs about 1/16 of a
// 32x32x2 MFMA), scalar-ALU and LDS instructions are.  The staging therefore keeps everything that
// changes from chunk to chunk uniform: a thread owns fixed cells of the plane and fixed dy rows,
// its byte offsets never change, and the chunk's row / image / position enters through the base
// and the scalar offset of buffer loads, whose range check also supplies the zeros of the padding.
#include <stdio.h>

#include "cct_internal.h"
#include "gemm_common.h"

namespace cct {
namespace {

constexpr int NT = 256;
constexpr int BN = 128;
constexpr int BK = 32;          // positions per chunk
constexpr int LDK = BK + 4;     // dy tile rows in LDS
constexpr int QS = BK / 8;
constexpr int kMaxLds = 80 * 1024;  // two workgroups per CU
constexpr unsigned kRsrcFlags = 0x00020000u;  // raw buffer, 32-bit elements
constexpr unsigned kDead = 0x80000000u;       // byte offset beyond every buffer range used here

struct BwdwGeom {
  int Wp;         // padded row width
  int nch;        // channels staged per chunk
  int plane;      // nch * Wp cells per staged row
  int V, XR;      // cells per thread and row (plane <= V*256); staged rows
  int KK, P, M, N, ncols;
  int rows_full;  // staged rows of a whole image: (Hout-1)*stride + K
  unsigned mP, mWout, mWp, mKK, mK;
  int sP, sWout, sWp, sKK, sK;
};

typedef int i32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float buf_load(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
  return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0));
}

template <int BM, int WM, int WN, int V, int XR>
__global__ __launch_bounds__(NT, 3) void conv_bwdw_fused_f32(ConvBwdW p, BwdwGeom fg, int tiles_m,
                                                             int tiles_n) {
  constexpr int WAVES_N = BN / (32 * WN);
  constexpr int WAVES_M = BM / (32 * WM);
  static_assert(WAVES_M * WAVES_N == 4, "4 waves per workgroup");
  constexpr int AS_IT = BM * BK / NT;
  constexpr int AS_ROWS = NT / BK;
  constexpr int ROWP = V * NT + 8;   // floats between staged rows (the 8 spreads taps over banks)
  constexpr int XS = XR * ROWP;      // floats per staging buffer

  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* As = smem;                                   // [2][BM*LDK]
  float* Xs = smem + 2 * BM * LDK;                    // [2][XS]
  int* tabs = reinterpret_cast<int*>(Xs + 2 * XS);    // [3][BK]: chunk t uses slot t % 3

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
  const int lane_lo = lane & 31, lane_hi = lane >> 5;

  // consecutive workgroup ids go round-robin over the 8 XCDs: give every XCD a contiguous run of
  // (split, tile) pairs, tile fastest, so that the tiles of one split share dy and x through L2
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
  const int col_end = min(fg.ncols, col_begin + p.split_len);

  const int HW = p.H * p.W;
  const long long CHW = (long long)p.C * HW;
  const int ci0 = fdiv_u(n0, fg.mKK, fg.sKK);   // first channel this tile's rows touch
  const float* Ag = p.dy + (long long)g * p.Og * fg.P;
  const float* Xg = p.x + ((long long)g * p.Cg + ci0) * HW;
  const long long dy_img = (long long)p.O * fg.P;

  // Fixed cells of the staged plane: cell = tid + v*256 is channel cc = cell / Wp, padded column
  // cell % Wp.  Its byte offset inside (image, first staged channel, input row) never changes;
  // padding columns and channels past the group get an offset that fails every range check.
  unsigned xvoff[V];
#pragma unroll
  for (int v = 0; v < V; ++v) {
    const int cell = tid + v * NT;
    const int cc = fdiv_u(cell, fg.mWp, fg.sWp);
    const int w = cell - cc * fg.Wp - p.p;
    const bool live = cell < fg.plane && ci0 + cc < p.Cg && w >= 0 && w < p.W;
    xvoff[v] = live ? (unsigned)(cc * HW + w) * 4u : kDead;
  }
  // Fixed dy rows: byte offset of (kernel row, position as_k of the chunk) relative to the chunk's
  // first position; rows past the last kernel are clamped (their products are never stored).
  const int as_k = tid % BK, as_r0 = tid / BK;
  unsigned rowoff[AS_IT];
#pragma unroll
  for (int it = 0; it < AS_IT; ++it)
    rowoff[it] = (unsigned)(min(m0 + as_r0 + it * AS_ROWS, fg.M - 1) * fg.P + as_k) * 4u;

  float ras[AS_IT];
  float rx[XR * V] = {};   // rows a chunk does not need keep their previous contents

  // Global loads of one chunk (dy tile, input rows) and its position table.
#define CCT_BW_LOAD(C0, TSLOT)                                                                  \
  {                                                                                             \
    const int c0_ = (C0);                                                                       \
    const int ce_ = min(c0_ + BK, col_end);                                                     \
    const int n_f = fdiv_u(c0_, fg.mP, fg.sP);                                                  \
    const int pix_f = c0_ - n_f * fg.P;                                                         \
    const int a_f = fdiv_u(pix_f, fg.mWout, fg.sWout);                                          \
    const int n_l = fdiv_u(ce_ - 1, fg.mP, fg.sP);                                              \
    const int a_l = fdiv_u(ce_ - 1 - n_l * fg.P, fg.mWout, fg.sWout);                           \
    const int rows_first = ((n_f == n_l ? a_l : p.Hout - 1) - a_f) * p.s + p.K;                 \
    const int rows_total =                                                                      \
        n_f == n_l ? rows_first                                                                 \
                   : rows_first + (n_l - n_f - 1) * fg.rows_full + a_l * p.s + p.K;             \
    /* dy tile */                                                                               \
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(                        \
        const_cast<float*>(Ag + (long long)n_f * dy_img), 0, 0x7fffffff, kRsrcFlags);           \
    if (n_f == n_l && ce_ - c0_ == BK) {                                                        \
      /* 32 positions of one image: uniform offset, nothing per thread */                       \
      _Pragma("unroll") for (int it = 0; it < AS_IT; ++it)                                      \
        ras[it] = buf_load(ra, rowoff[it], (unsigned)pix_f * 4u);                               \
    } else {                                                                                    \
      const int col = c0_ + as_k;                                                               \
      const int n = fdiv_u(min(col, ce_ - 1), fg.mP, fg.sP);                                    \
      const unsigned aoff =                                                                     \
          col < ce_ ? ((unsigned)(n - n_f) * (unsigned)dy_img + (unsigned)(col - n * fg.P) -    \
                       (unsigned)as_k) * 4u                                                     \
                    : kDead;                                                                    \
      _Pragma("unroll") for (int it = 0; it < AS_IT; ++it)                                      \
        ras[it] = buf_load(ra, rowoff[it] + aoff, 0u);                                          \
    }                                                                                           \
    /* position table: staged row of the position's first tap row, times ROWP, plus its column; \
       positions past the end of the split repeat the last one (their dy is zero) */            \
    if (wave == 0) {                                                                            \
      const int pos = min(c0_ + as_k, ce_ - 1);                                                 \
      const int n = fdiv_u(pos, fg.mP, fg.sP), pix = pos - n * fg.P;                            \
      const int r = fdiv_u(pix, fg.mWout, fg.sWout), c = pix - r * p.Wout;                      \
      const int srow = n == n_f ? (r - a_f) * p.s                                               \
                                : rows_first + (n - n_f - 1) * fg.rows_full + r * p.s;          \
      tabs[(TSLOT) * BK + as_k] = srow * ROWP + c * p.s;                                        \
    }                                                                                           \
    /* input rows: a scalar walk over the staged rows (rest of the first image, whole images,   \
       the first rows of the last image).  The row pointer advances by one input row per staged \
       row and jumps at an image boundary; rows outside the image get an empty range, rows     \
       past the last needed one are not loaded at all (nothing reads them). */                  \
    {                                                                                           \
      int h = a_f * p.s - p.p, left = rows_first;                                               \
      const float* rowp = Xg + (long long)n_f * CHW + (long long)h * p.W;                       \
      _Pragma("unroll") for (int u = 0; u < XR; ++u) {                                          \
        if (u < rows_total) {                                                                   \
          const bool valid = h >= 0 && h < p.H;                                                 \
          const __amdgpu_buffer_rsrc_t rxs = __builtin_amdgcn_make_buffer_rsrc(                 \
              const_cast<float*>(rowp), 0, valid ? 0x7fffffff : 0, kRsrcFlags);                 \
          _Pragma("unroll") for (int v = 0; v < V; ++v)                                         \
            rx[u * V + v] = buf_load(rxs, xvoff[v], 0u);                                        \
          ++h;                                                                                  \
          rowp += p.W;                                                                          \
          if (--left == 0) { /* next image: its staged rows start at input row -pad */          \
            rowp += CHW - (long long)(h + p.p) * p.W;                                           \
            h = -p.p;                                                                           \
            left = fg.rows_full;                                                                \
          }                                                                                     \
        }                                                                                       \
      }                                                                                         \
    }                                                                                           \
  }
#define CCT_BW_STORE(BUF)                                                                       \
  {                                                                                             \
    _Pragma("unroll") for (int it = 0; it < AS_IT; ++it)                                        \
      As[(BUF) * BM * LDK + (as_r0 + it * AS_ROWS) * LDK + as_k] = ras[it];                     \
    _Pragma("unroll") for (int u = 0; u < XR; ++u)                                              \
      _Pragma("unroll") for (int v = 0; v < V; ++v)                                             \
        Xs[(BUF) * XS + u * ROWP + v * NT + tid] = rx[u * V + v];                               \
  }

  floatx16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int am = wave_m * WM * 32 + lane_lo;
  const int bn = wave_n * WN * 32 + lane_lo;
  const int a_lds = am * LDK + lane_hi * 4;
  // lowered row n = (ci, i, j) -> offset of tap (i, j) of channel ci inside the staged rows
  int laneoff[WN];
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    const int n = min(n0 + bn + j * 32, fg.N - 1);
    const int ci = fdiv_u(n, fg.mKK, fg.sKK), t = n - ci * fg.KK;
    const int ti = fdiv_u(t, fg.mK, fg.sK), tj = t - ti * p.K;
    laneoff[j] = ti * ROWP + (ci - ci0) * fg.Wp + tj;
  }

  const int ktiles = (col_end - col_begin + BK - 1) / BK;  // <= 0 for an empty split
  if (ktiles > 0) {
    CCT_BW_LOAD(col_begin, 0);
    CCT_BW_STORE(0);
  }
  if (ktiles > 1) CCT_BW_LOAD(col_begin + BK, 1);
  __syncthreads();

  // Position offsets run two steps ahead of the MFMAs: pa holds those of the step whose operands
  // are read next, pb those of the step after it (being fetched from the table).
  int pa[4], pb[4];
  f32x4 a[2][WM];
  float b[2][WN][4];
#pragma unroll
  for (int e = 0; e < 4; ++e) pa[e] = pb[e] = 0;
  if (ktiles > 0) {
    const i32x4 v0 = *reinterpret_cast<const i32x4*>(tabs + lane_hi * 4);
    const i32x4 v1 = *reinterpret_cast<const i32x4*>(tabs + 8 + lane_hi * 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      pa[e] = v1[e];
      pb[e] = v0[e];   // only used for the first reads below
    }
#pragma unroll
    for (int i = 0; i < WM; ++i) a[0][i] = *reinterpret_cast<const f32x4*>(&As[a_lds + i * 32 * LDK]);
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) b[0][j][e] = Xs[pb[e] + laneoff[j]];
  }

  // Main loop: the pipeline of the plain backward-weights GEMM.  Operand reads run one step (8
  // positions) ahead and their position offsets one step further; in the middle of chunk t the
  // values loaded for chunk t+1 go to LDS and the loads of chunk t+2 are issued; the barrier sits
  // before the last step.  The position table of chunk t+2 is written during chunk t into the
  // third slot, which no wave reads any more: the tables of chunks t and t+1 are still in use.
  int ts0 = 0, ts1 = 1, ts2 = 2;  // table slots of chunks t, t+1, t+2
  for (int t = 0; t < ktiles; ++t) {
    const int buf = t & 1;
    const bool more = t + 1 < ktiles;
    const float* as = As + buf * BM * LDK + a_lds;
    const float* xs = Xs + buf * XS;
    const float* xs_n = Xs + (buf ^ 1) * XS;
#pragma unroll
    for (int q = 0; q < QS; ++q) {
      const int cur = q & 1, nxt = cur ^ 1;
      // on entry pa = offsets of step q+1 (of the next chunk when q = 3)
      if (q + 1 < QS) {
#pragma unroll
        for (int i = 0; i < WM; ++i)
          a[nxt][i] = *reinterpret_cast<const f32x4*>(as + i * 32 * LDK + (q + 1) * 8);
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e) b[nxt][j][e] = xs[pa[e] + laneoff[j]];
      } else {
        __syncthreads();
        if (more) {
#pragma unroll
          for (int i = 0; i < WM; ++i)
            a[nxt][i] = *reinterpret_cast<const f32x4*>(&As[(buf ^ 1) * BM * LDK + a_lds + i * 32 * LDK]);
#pragma unroll
          for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) b[nxt][j][e] = xs_n[pa[e] + laneoff[j]];
        }
      }
      // fetch the offsets of step q+2: same chunk for q < 2, else steps 0 / 1 of the next chunk
      if (q + 2 < QS || more) {
        const int slot = q + 2 < QS ? ts0 : ts1;
        const i32x4 v =
            *reinterpret_cast<const i32x4*>(tabs + slot * BK + ((q + 2) % QS) * 8 + lane_hi * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) pb[e] = v[e];
      }
      // In the step that also moves the next chunk, the LDS stores and the global loads are
      // issued between the MFMA groups (a wave issues in order: what follows an MFMA goes out
      // while that MFMA occupies the matrix pipe), not after all sixteen.
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
          for (int j = 0; j < WN; ++j)
            acc[i][j] =
                __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][i][e], b[cur][j][e], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (q == QS / 2 - 1 && more) {
          if (e == 0) CCT_BW_STORE(buf ^ 1);
          if (e == 1 && t + 2 < ktiles) CCT_BW_LOAD(col_begin + (t + 2) * BK, ts2);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int e = 0; e < 4; ++e) pa[e] = pb[e];
    }
    const int ts = ts0;
    ts0 = ts1;
    ts1 = ts2;
    ts2 = ts;
  }
#undef CCT_BW_LOAD
#undef CCT_BW_STORE

  float* __restrict__ C = p.Cpart + ((long long)s * p.G + g) * fg.M * fg.N;
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    const int n = n0 + bn + j * 32;
    if (n >= fg.N) continue;
#pragma unroll
    for (int i = 0; i < WM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wave_m * WM * 32 + i * 32 + (r >> 2) * 8 + lane_hi * 4 + (r & 3);
        if (m < fg.M) C[(long long)m * fg.N + n] = acc[i][j][r];
      }
    }
  }
}

// Staging geometry; false = the shape does not fit the kernel (use a materialised layout).
bool make_geom(int C, int H, int W, int K, int s, int pad, int Hout, int Wout, int Cg, int O,
               int BM, BwdwGeom* fg, size_t* lds) {
  if (K < 2) return false;
  const long long P = (long long)Hout * Wout;
  const long long Wp = (long long)W + 2 * pad;
  const long long KK = (long long)K * K;
  // rows of padded input that 32 consecutive positions can touch: they cover at most A output rows
  // spread over at most T images; t images need (A - t)*stride + t*K rows, largest at t = 1 or T
  const long long A = (BK - 1) / Wout + 2, T = (BK - 1) / P + 2;
  const long long r1 = (A - 1) * s + K;
  const long long rT = (A > T ? A - T : 0) * s + T * K;
  const long long rows = r1 > rT ? r1 : rT;
  long long nch = (BN - 1) / KK + 2;
  if (nch > Cg) nch = Cg;
  const long long plane = nch * Wp;
  int V, XR;
  if (plane <= NT) {
    V = 1;
    XR = rows <= 8 ? 8 : (rows <= 12 ? 12 : (rows <= 16 ? 16 : 24));
  } else {
    V = 2;
    XR = 8;
  }
  if (plane > (long long)V * NT || rows > XR) return false;
  // 32-bit byte offsets: dy relative to the chunk's first image, x inside one image
  if ((T + 1) * O * P >= (1LL << 29) || (long long)C * H * W >= (1LL << 29)) return false;
  if ((long long)Cg * KK >= (1LL << 30) || P >= (1LL << 24)) return false;
  fg->Wp = (int)Wp;
  fg->nch = (int)nch;
  fg->plane = (int)plane;
  fg->V = V;
  fg->XR = XR;
  fg->KK = (int)KK;
  fg->P = (int)P;
  fg->rows_full = (Hout - 1) * s + K;
  make_fastdiv_parts((int)P, &fg->mP, &fg->sP);
  make_fastdiv_parts(Wout, &fg->mWout, &fg->sWout);
  make_fastdiv_parts((int)Wp, &fg->mWp, &fg->sWp);
  make_fastdiv_parts((int)KK, &fg->mKK, &fg->sKK);
  make_fastdiv_parts(K, &fg->mK, &fg->sK);
  *lds = 4ull * (2ull * BM * LDK + 2ull * XR * (V * NT + 8) + 3ull * BK);
  return *lds <= (size_t)kMaxLds;
}

template <int BM, int WM, int WN, int V, int XR>
int launch_kernel(const ConvBwdW& p, const BwdwGeom& fg, size_t lds, dim3 grid, int tiles_m,
                  int tiles_n, hipStream_t st) {
  constexpr auto kern = conv_bwdw_fused_f32<BM, WM, WN, V, XR>;
  if (const int rc = ensure_dynamic_lds<kern>(kMaxLds)) return rc;
  hipLaunchKernelGGL(kern, grid, dim3(NT), lds, st, p, fg, tiles_m, tiles_n);
  return CCT_OK;
}

template <int BM, int WM, int WN>
int launch_variant(const ConvBwdW& p, BwdwGeom fg, size_t lds, hipStream_t st) {
  const int tiles_m = (fg.M + BM - 1) / BM;
  const int tiles_n = (fg.N + BN - 1) / BN;
  const long long tiles = (long long)tiles_m * tiles_n;
  if (tiles <= 0 || p.S < 1 || tiles * p.S >= 2147483647LL || p.G > 65535) return CCT_EUNSUPPORTED;
  if (p.split_len % BK) return CCT_EINVAL;
  dim3 grid((unsigned)(tiles * p.S), (unsigned)p.G);
  char name[96];
  snprintf(name, sizeof(name), "conv_bwdw_fused_f32<%d, %d, %d, %d, %d>", BM, WM, WN, fg.V, fg.XR);
  ProfScope ps(name, 2.0 * fg.M * fg.N * (double)fg.ncols * p.G,
               4.0 * ((double)p.nimg * p.C * p.H * p.W + (double)p.nimg * p.O * fg.P +
                      (double)fg.M * fg.N * p.S * p.G),
               st);
  int rc;
  if (fg.V == 2)
    rc = launch_kernel<BM, WM, WN, 2, 8>(p, fg, lds, grid, tiles_m, tiles_n, st);
  else if (fg.XR == 8)
    rc = launch_kernel<BM, WM, WN, 1, 8>(p, fg, lds, grid, tiles_m, tiles_n, st);
  else if (fg.XR == 12)
    rc = launch_kernel<BM, WM, WN, 1, 12>(p, fg, lds, grid, tiles_m, tiles_n, st);
  else if (fg.XR == 16)
    rc = launch_kernel<BM, WM, WN, 1, 16>(p, fg, lds, grid, tiles_m, tiles_n, st);
  else
    rc = launch_kernel<BM, WM, WN, 1, 24>(p, fg, lds, grid, tiles_m, tiles_n, st);
  if (rc) return rc;
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

}  // namespace

bool conv_bwdw_fused_fits(int C, int H, int W, int K, int s, int pad, int Hout, int Wout, int Cg,
                          int Og, int O) {
  int BM, BNt, BKt;
  gemm_nt_tile(Og, Cg * K * K, &BM, &BNt, &BKt);
  BwdwGeom fg;
  size_t lds;
  return BNt == BN && BKt == BK &&
         make_geom(C, H, W, K, s, pad, Hout, Wout, Cg, O, BM, &fg, &lds);
}

int launch_conv_bwdw_fused(const ConvBwdW& p, hipStream_t st) {
  int BM, BNt, BKt;
  gemm_nt_tile(p.Og, p.Cg * p.K * p.K, &BM, &BNt, &BKt);
  BwdwGeom fg;
  size_t lds;
  if (BNt != BN || BKt != BK ||
      !make_geom(p.C, p.H, p.W, p.K, p.s, p.p, p.Hout, p.Wout, p.Cg, p.O, BM, &fg, &lds))
    return CCT_EUNSUPPORTED;
  const long long ncols = (long long)p.nimg * fg.P;
  if (ncols <= 0 || ncols >= 2147483647LL - 256) return CCT_EUNSUPPORTED;
  fg.ncols = (int)ncols;
  fg.M = p.Og;
  fg.N = p.Cg * p.K * p.K;
  if (BM == 64) return launch_variant<64, 1, 2>(p, fg, lds, st);
  if (BM == 96) return launch_variant<96, 3, 1>(p, fg, lds, st);
  return launch_variant<128, 2, 2>(p, fg, lds, st);
}

}  // namespace cct
