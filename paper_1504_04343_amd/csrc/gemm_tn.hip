// Multiply phase (Sec. 2.1): R^ = D^ K^ on the gfx950 matrix cores.
//
// The library keeps D^ transposed ("K-major": one row per patch element, one column per
// position of the whole chunk of images), so the product is computed as
//     C[m][col] = sum_k Apack[k][m] * B[k][col]          (m: kernels, col: positions)
// with both operands K-major.  C columns (and, for the backward-data pass, B columns) can be
// mapped straight onto an NCHW tensor through a ColMap, which turns the Type-1 lifting
// phase + bias add into the GEMM epilogue.
//
// Tiling: 256 threads = 4 waves; the workgroup owns a BM x BN tile of C, each wave a
// (32*WM) x (32*WN) sub-tile built from v_mfma_f32_32x32x2_f32 (fp32) or
// v_mfma_f32_32x32x8_bf16_1k (bf16 operands) with fp32 accumulators.  K is walked in steps
// of BK through a double-buffered LDS stage; the global loads of step t+1 are issued before
// the MFMAs of step t.
#include <stdio.h>

#include "cct_internal.h"
#include "gemm_common.h"

namespace cct {
namespace {


constexpr int NT = 256;

// fp32 kernel.  BMODE 0: B rows are plain, 16-byte aligned rows -> 16-byte loads.
// BMODE 1: B columns go through a column map (an NCHW tensor read in place), 4-byte loads.
// BMODE 2: fused lowering, B tiles are gathered from x (see GemmTN::gather), 4-byte loads; the
//          (ci, i, j) -> offset table of all K rows is built once per workgroup in LDS.
// BMODE 3: same, but the taps are decoded arithmetically (for K too long for the LDS table).
// BMODE 4: gather with the K dimension ordered tap-major, k = tap*Cpad + channel with Cpad a
// multiple of BK and taps on a tKi x tKj grid (pads tph, tpw, stride 1): all rows of a K tile share
// one tap, so a thread (which owns one position) needs one byte offset per tap - position + tap,
// or an offset the buffer range check rejects when the tap falls into the padding - kept in an
// LDS table [tap][position of the tile]; the channel of each row enters through the scalar offset
// of the buffer load.  A tile's gather then costs no vector-ALU work at all.  Used for the
// inverse lifting of the Type-2 backward-data pass: dR^[(o,i)][(n,a,b)] = dy[n,o,a+p-i,b] is a
// gather from dy with K vertical taps.
template <int BM, int BN, int BK, int WM, int WN, int BMODE>
__global__ __launch_bounds__(NT) void gemm_tn_f32(GemmTN p, int tiles_m, int tiles_n, int fast) {
  constexpr bool BVEC = BMODE == 0;
  constexpr bool GATHER = BMODE >= 2;
  constexpr bool TAPS_LDS = BMODE == 2;
  constexpr bool TAPMAJOR = BMODE == 4;
  extern __shared__ int2 tap_tab[];  // BMODE 2: {(ci*H + i)*W + j, (i << 16) | j} per row k
  constexpr int WAVES_N = BN / (32 * WN);
  constexpr int WAVES_M = BM / (32 * WM);
  static_assert(WAVES_M * WAVES_N == 4, "4 waves per workgroup");
  constexpr int A_VECS = BK * BM / 4;
  constexpr int A_IT = (A_VECS + NT - 1) / NT;
  constexpr int B_VECS = BK * BN / 4;
  constexpr int B_IT = (B_VECS + NT - 1) / NT;
  constexpr int B_SC_IT = BK * BN / NT;  // scalar path: loads per thread
  constexpr int B_KSTEP = NT / BN;       // scalar path: k rows covered per pass
  static_assert(NT % BN == 0 || BVEC, "scalar B path needs BN | 256");
  static_assert(B_VECS % NT == 0, "B tile is a whole number of 16-byte loads per thread");

  __shared__ __attribute__((aligned(16))) float As[2][BK * BM];
  __shared__ __attribute__((aligned(16))) float Bs[2][BK * BN];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;

  // Tile order: consecutive workgroup ids go round-robin over the 8 XCDs, so give each XCD a
  // contiguous run of column tiles and let the M tiles of one column tile follow each other on
  // the same XCD: the B tile they share is then fetched from HBM once per XCD L2.
  int bid = blockIdx.x;
  {
    const int total = tiles_m * tiles_n;
    const int per = total >> 3, rem = total & 7;
    const int xcd = bid & 7, slot = bid >> 3;
    bid = xcd * per + min(xcd, rem) + slot;  // XCD x owns per + (x < rem) consecutive tiles
  }
  const int tile_n = bid / tiles_m;
  const int tile_m = bid - tile_n * tiles_m;
  const int g = blockIdx.y;
  const int m0 = tile_m * BM;
  const int n0 = tile_n * BN;

  // ---- global -> register staging: fixed per-thread coordinates, pointers advance by BK rows
  gptr_f32 Ag = (gptr_f32)(p.A) + (long long)g * p.a_gs + m0;
  gptr_f32 Bg = (gptr_f32)(p.B) + (long long)g * p.b_gs;
  gptr_f32 a_src[A_IT];
  int a_dst[A_IT];
#pragma unroll
  for (int it = 0; it < A_IT; ++it) {
    const int v = tid + it * NT;
    const int k = v / (BM / 4), m4 = v % (BM / 4);
    a_src[it] = Ag + (long long)k * p.Mpad + m4 * 4;
    a_dst[it] = k * BM + m4 * 4;
  }
  const long long a_step = (long long)BK * p.Mpad;
  const long long b_step = (long long)BK * p.b_ks;

  // vector path: per-thread (row, 16-byte column group) of each 256-thread slab of the tile.
  // Columns need no guard: rows of a lowered matrix are padded to a multiple of 256 columns.
  gptr_f32 b_src[BVEC ? B_IT : 1];
  int b_dst[BVEC ? B_IT : 1];
  int b_k[BVEC ? B_IT : 1];
  if (BVEC) {
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
      const int v = tid + it * NT;
      const int k = v / (BN / 4), n4 = v % (BN / 4);
      b_k[it] = k;
      b_src[it] = Bg + (long long)k * p.b_ks + n0 + n4 * 4;
      b_dst[it] = k * BN + n4 * 4;
    }
  }
  gptr_f32 bs_src = nullptr;  // scalar path
  bool bs_ok = false;
  int bs_k0 = 0, bs_n = 0;
  int g_hh = 0, g_ww = 0;  // gather: top-left tensor pixel of this thread's column
  unsigned g_voff = 0, b_voff = 0;
  const bool g_nopad = GATHER && (fast & 1);
  const bool b_fast = BMODE == 1 && (fast & 2);
  if (!BVEC) {
    bs_n = tid % BN;
    bs_k0 = tid / BN;
    const int col = n0 + bs_n;
    bs_ok = col < p.Ncols;
    if (GATHER) {
      const int P = p.gHout * p.gWout;
      const int cc = bs_ok ? col : 0;
      const int n = cc / P, pix = cc - n * P;
      const int r = pix / p.gWout, c = pix - r * p.gWout;
      g_hh = r * p.gs - (TAPMAJOR ? p.tph : p.gp);
      g_ww = c * p.gs - (TAPMAJOR ? p.tpw : p.gp);
      bs_src = (gptr_f32)(p.B) + (((long long)n * p.gC + (long long)g * p.gCg) * p.gH + g_hh) * p.gW + g_ww;
      // unpadded layer: every tap of a valid position is inside the image, so the gather needs
      // no bounds checks; the position then is a fixed 32-bit byte offset from the tensor's start
      // (columns past the end get one that fails the buffer range check and load as zero)
      g_voff = bs_ok ? (unsigned)((((long long)n * p.gC + (long long)g * p.gCg) * p.gH + g_hh) * p.gW + g_ww) * 4u
                     : 0x80000000u;
    } else {
      bs_src = Bg + (bs_ok ? col_offset(p.bmap, col) : 0) + (long long)bs_k0 * p.b_ks;
      b_voff = bs_ok ? (unsigned)(col_offset(p.bmap, col) + (long long)bs_k0 * p.b_ks) * 4u
                     : 0x80000000u;
    }
  }

  unsigned* tap_voff = reinterpret_cast<unsigned*>(tap_tab);  // BMODE 4: [tap][BN positions]
  if (TAPMAJOR) {
    // the two threads that share a position (bs_k0 = 0, 1) fill alternate taps
    const long long chan0 = (long long)g * p.gCg * p.gH * p.gW;  // the group's first channel
    const int P = p.gHout * p.gWout;
    const int cc = bs_ok ? n0 + bs_n : 0;
    const long long img = (long long)(cc / P) * p.gC * p.gH * p.gW;
    for (int t = bs_k0; t < p.tKi * p.tKj; t += NT / BN) {
      const int ti = t / p.tKj, tj = t - ti * p.tKj;
      const int h = g_hh + ti, w = g_ww + tj;
      const bool ok = bs_ok && (unsigned)h < (unsigned)p.gH && (unsigned)w < (unsigned)p.gW;
      tap_voff[t * BN + bs_n] =
          ok ? (unsigned)(img + chan0 + (long long)h * p.gW + w) * 4u : 0x80000000u;
    }
    __syncthreads();
  }
  if (TAPS_LDS) {
    for (int k = tid; k < p.Kpad; k += NT) {
      const int ci = k / p.gKK, rem = k - ci * p.gKK;
      const int ti = rem / p.gK, tj = rem - ti * p.gK;
      // rows >= Kdim get a row offset that fails every bounds check
      tap_tab[k] = k < p.Kdim ? make_int2((ci * p.gH + ti) * p.gW + tj, (ti << 16) | tj)
                              : make_int2(0, 0x7fff << 16);
    }
    __syncthreads();
  }

  f32x4 ra[A_IT];
  f32x4 rbv[BVEC ? B_IT : 1];
  float rbs[BVEC ? 1 : B_SC_IT];

#define CCT_LOAD_TILE(K0)                                                                   \
  {                                                                                         \
    _Pragma("unroll") for (int it = 0; it < A_IT; ++it) {                                   \
      if (A_VECS % NT == 0 || tid + it * NT < A_VECS)                                       \
        ra[it] = *(gptr_f32x4)(a_src[it]);                                                  \
      a_src[it] += a_step;                                                                  \
    }                                                                                       \
    if (BVEC) {                                                                             \
      _Pragma("unroll") for (int it = 0; it < B_IT; ++it) {                                 \
        f32x4 val = {0.f, 0.f, 0.f, 0.f};                                                   \
        if ((K0) + b_k[it] < p.Kdim) val = *(gptr_f32x4)(b_src[it]);                        \
        rbv[it] = val;                                                                      \
        b_src[it] += b_step;                                                                \
      }                                                                                     \
    } else if (TAPMAJOR) {                                                                  \
      const int k0_ = (K0);                                                                 \
      const int t_ = fdiv_u(k0_, p.g_divKK_M, p.g_divKK_sh);  /* divides by gCpad here */    \
      const int c0_ = k0_ - t_ * p.gCpad + __builtin_amdgcn_readfirstlane(bs_k0);           \
      const unsigned vo = tap_voff[t_ * BN + bs_n];                                         \
      const __amdgpu_buffer_rsrc_t rsx = __builtin_amdgcn_make_buffer_rsrc(                 \
          const_cast<void*>(p.B), 0, 0x7fffffff, 0x00020000);                               \
      _Pragma("unroll") for (int it = 0; it < B_SC_IT; ++it) {                              \
        const int ci = min(c0_ + it * B_KSTEP, p.gCg - 1);  /* padded rows: A is zero */     \
        rbs[it] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(           \
                                                rsx, (int)vo,                               \
                                                (int)((unsigned)ci * (unsigned)(p.gH * p.gW) * 4u), 0)); \
      }                                                                                     \
    } else if (TAPS_LDS && g_nopad) {                                                       \
      const __amdgpu_buffer_rsrc_t rsx = __builtin_amdgcn_make_buffer_rsrc(                 \
          const_cast<void*>(p.B), 0, 0x7fffffff, 0x00020000);                               \
      _Pragma("unroll") for (int it = 0; it < B_SC_IT; ++it) {                              \
        const int2 tp = tap_tab[(K0) + bs_k0 + it * B_KSTEP];                               \
        rbs[it] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(           \
                                                rsx, (int)(g_voff + (unsigned)tp.x * 4u), 0, 0)); \
      }                                                                                     \
    } else if (TAPS_LDS) {                                                                  \
      _Pragma("unroll") for (int it = 0; it < B_SC_IT; ++it) {                              \
        const int2 tp = tap_tab[(K0) + bs_k0 + it * B_KSTEP];                               \
        float val = 0.f;                                                                    \
        if (bs_ok && (unsigned)(g_hh + (tp.y >> 16)) < (unsigned)p.gH &&                    \
            (unsigned)(g_ww + (tp.y & 0xffff)) < (unsigned)p.gW)                            \
          val = bs_src[tp.x];                                                               \
        rbs[it] = val;                                                                      \
      }                                                                                     \
    } else if (GATHER) {                                                                    \
      _Pragma("unroll") for (int it = 0; it < B_SC_IT; ++it) {                              \
        /* row k of the Type-1 lowered matrix = tap (ci, i, j); decoded arithmetically */   \
        const int k = (K0) + bs_k0 + it * B_KSTEP;                                          \
        const int ci = fdiv_u(k, p.g_divKK_M, p.g_divKK_sh);                                \
        const int rem = k - ci * p.gKK;                                                     \
        const int ti = fdiv_u(rem, p.g_divK_M, p.g_divK_sh);                                \
        const int tj = rem - ti * p.gK;                                                     \
        float val = 0.f;                                                                    \
        if (bs_ok && k < p.Kdim && (unsigned)(g_hh + ti) < (unsigned)p.gH &&                \
            (unsigned)(g_ww + tj) < (unsigned)p.gW)                                         \
          val = bs_src[(ci * p.gH + ti) * p.gW + tj];                                       \
        rbs[it] = val;                                                                      \
      }                                                                                     \
    } else if (b_fast) {                                                                    \
      /* column map within 2 GiB: fixed byte offset per thread, the K row in the scalar     \
         offset (rows of the zero-padded K tail re-read the last rows: A is zero there) */  \
      const __amdgpu_buffer_rsrc_t rsb = __builtin_amdgcn_make_buffer_rsrc(                 \
          const_cast<float*>(reinterpret_cast<const float*>(p.B) + (long long)g * p.b_gs),  \
          0, 0x7fffffff, 0x00020000);                                                       \
      _Pragma("unroll") for (int it = 0; it < B_SC_IT; ++it) {                              \
        const int kk = min((K0) + it * B_KSTEP, p.Kdim - B_KSTEP);                          \
        rbs[it] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(           \
                                                rsb, (int)b_voff,                           \
                                                (int)((unsigned)kk * (unsigned)p.b_ks * 4u), 0)); \
      }                                                                                     \
    } else {                                                                                \
      _Pragma("unroll") for (int it = 0; it < B_SC_IT; ++it) {                              \
        float val = 0.f;                                                                    \
        if (bs_ok && (K0) + bs_k0 + it * B_KSTEP < p.Kdim)                                  \
          val = bs_src[(long long)it * B_KSTEP * p.b_ks];                                   \
        rbs[it] = val;                                                                      \
      }                                                                                     \
      bs_src += b_step;                                                                     \
    }                                                                                       \
  }

#define CCT_STORE_TILE(BUF)                                                                 \
  {                                                                                         \
    _Pragma("unroll") for (int it = 0; it < A_IT; ++it) {                                   \
      if (A_VECS % NT == 0 || tid + it * NT < A_VECS)                                       \
        *reinterpret_cast<f32x4*>(&As[BUF][a_dst[it]]) = ra[it];                            \
    }                                                                                       \
    if (BVEC) {                                                                             \
      _Pragma("unroll") for (int it = 0; it < B_IT; ++it)                                   \
        *reinterpret_cast<f32x4*>(&Bs[BUF][b_dst[it]]) = rbv[it];                           \
    } else {                                                                                \
      _Pragma("unroll") for (int it = 0; it < B_SC_IT; ++it)                                \
        Bs[BUF][(bs_k0 + it * B_KSTEP) * BN + bs_n] = rbs[it];                              \
    }                                                                                       \
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
  const int a_lds = lane_hi * BM + am;
  const int b_lds = lane_hi * BN + bn;

  // Main loop, software pipelined so that no wave waits with an empty MFMA queue:
  //  - the LDS operands of K-step s+1 are read before the MFMAs of step s are issued;
  //  - the next tile's registers are written to the other LDS buffer in the middle of the
  //    current tile (their global loads were issued half a tile earlier), and the loads of the
  //    tile after that are issued right behind;
  //  - the barrier that publishes the next tile sits before the LAST K-step, so that this step's
  //    MFMAs cover the barrier skew and the latency of the next tile's first operand reads.
  const int ktiles = p.Kpad / BK;
  CCT_LOAD_TILE(0);
  CCT_STORE_TILE(0);
  __syncthreads();
  if (ktiles > 1) CCT_LOAD_TILE(BK);
  constexpr int KS = BK / 2;
  float a[2][WM], b[2][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i) a[0][i] = As[0][a_lds + i * 32];
#pragma unroll
  for (int j = 0; j < WN; ++j) b[0][j] = Bs[0][b_lds + j * 32];
  for (int t = 0; t < ktiles; ++t) {
    const int buf = t & 1;
    const bool more = t + 1 < ktiles;
    const float* as = &As[buf][a_lds];
    const float* bs = &Bs[buf][b_lds];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int cur = s & 1, nxt = cur ^ 1;
      if (s + 1 < KS) {
#pragma unroll
        for (int i = 0; i < WM; ++i) a[nxt][i] = as[(s + 1) * 2 * BM + i * 32];
#pragma unroll
        for (int j = 0; j < WN; ++j) b[nxt][j] = bs[(s + 1) * 2 * BN + j * 32];
      } else {
        __syncthreads();
        if (more) {
#pragma unroll
          for (int i = 0; i < WM; ++i) a[nxt][i] = As[buf ^ 1][a_lds + i * 32];
#pragma unroll
          for (int j = 0; j < WN; ++j) b[nxt][j] = Bs[buf ^ 1][b_lds + j * 32];
        }
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (s == KS / 2 - 1 && more) {
        CCT_STORE_TILE(buf ^ 1);
        if (t + 2 < ktiles) CCT_LOAD_TILE((t + 2) * BK);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
#undef CCT_LOAD_TILE
#undef CCT_STORE_TILE

  // Epilogue: lifting (Type 1) / plain store, + bias.  In the 32x32 accumulator lane l holds
  // column l%32 and rows 8*(r/4) + 4*(l/32) + r%4 for r = 0..15.
  float* __restrict__ C = p.C + (long long)g * p.c_gs;
  const float* bias = p.bias ? p.bias + (long long)g * p.bias_gs : nullptr;
  // A lane's column and its lane half's 4 rows give one 64-bit base per column block; the row
  // of each accumulator register is a uniform multiple of the row stride on top of it.  Tiles that
  // lie completely inside M (all but the last row of tiles) need no per-lane row check.
  const int mw = m0 + wave_m * WM * 32;
  const bool full_m = m0 + BM <= p.M;
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    const int col = n0 + bn + j * 32;
    if (col >= p.Ncols) continue;
    float* __restrict__ cl = C + col_offset(p.cmap, col) + (long long)(mw + lane_hi * 4) * p.c_ms;
    const float* bl = bias ? bias + mw + lane_hi * 4 : nullptr;
#pragma unroll
    for (int i = 0; i < WM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = i * 32 + (r >> 2) * 8 + (r & 3);   // relative to mw + 4*lane_hi
        if (full_m || mw + row + lane_hi * 4 < p.M) {
          float v = acc[i][j][r];
          if (bl) v += bl[row];
          cl[(long long)row * p.c_ms] = v;
        }
      }
    }
  }
}

// bf16 operands (A packed bf16, B plain bf16 rows), fp32 accumulate.
// v_mfma_f32_32x32x8_bf16_1k: each lane supplies 4 consecutive k of its row/column; lanes
// 32..63 supply k+4..k+7.
template <int BM, int BN, int BK, int WM, int WN>
__global__ __launch_bounds__(NT) void gemm_tn_bf16(GemmTN p, int tiles_m, int tiles_n) {
  constexpr int WAVES_N = BN / (32 * WN);
  constexpr int WAVES_M = BM / (32 * WM);
  static_assert(WAVES_M * WAVES_N == 4, "4 waves per workgroup");
  static_assert(BK % 8 == 0, "BK multiple of 8");
  // 8 bf16 = 16 bytes per vector load
  constexpr int A_VECS = BK * BM / 8;
  constexpr int A_IT = (A_VECS + NT - 1) / NT;
  constexpr int B_VECS = BK * BN / 8;
  constexpr int B_IT = (B_VECS + NT - 1) / NT;

  __shared__ __attribute__((aligned(16))) unsigned short As[2][BK][BM];
  __shared__ __attribute__((aligned(16))) unsigned short Bs[2][BK][BN];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
  const int bid = blockIdx.x;
  const int tile_n = bid / tiles_m;
  const int tile_m = bid - tile_n * tiles_m;
  const int g = blockIdx.y;
  const int m0 = tile_m * BM;
  const int n0 = tile_n * BN;

  const unsigned short* __restrict__ A =
      reinterpret_cast<const unsigned short*>(p.A) + (long long)g * p.a_gs + m0;
  const unsigned short* __restrict__ B =
      reinterpret_cast<const unsigned short*>(p.B) + (long long)g * p.b_gs;

  uint4 ra[A_IT], rb[B_IT];
  auto load_tile = [&](int k0) {
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
      const int v = tid + it * NT;
      if (A_VECS % NT == 0 || v < A_VECS) {
        const int k = v / (BM / 8), m8 = v % (BM / 8);
        ra[it] = *reinterpret_cast<const uint4*>(A + (long long)(k0 + k) * p.Mpad + m8 * 8);
      }
    }
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
      const int v = tid + it * NT;
      const int k = v / (BN / 8), n8 = v % (BN / 8);
      const int col = n0 + n8 * 8;
      uint4 val = make_uint4(0, 0, 0, 0);
      if ((B_VECS % NT == 0 || v < B_VECS) && (k0 + k) < p.Kdim && col < p.b_ld_guard)
        val = *reinterpret_cast<const uint4*>(B + (long long)(k0 + k) * p.b_ks + col);
      rb[it] = val;
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
      const int v = tid + it * NT;
      if (A_VECS % NT == 0 || v < A_VECS) {
        const int k = v / (BM / 8), m8 = v % (BM / 8);
        *reinterpret_cast<uint4*>(&As[buf][k][m8 * 8]) = ra[it];
      }
    }
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
      const int v = tid + it * NT;
      if (B_VECS % NT == 0 || v < B_VECS) {
        const int k = v / (BN / 8), n8 = v % (BN / 8);
        *reinterpret_cast<uint4*>(&Bs[buf][k][n8 * 8]) = rb[it];
      }
    }
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

  const int ktiles = p.Kpad / BK;
  load_tile(0);
  store_tile(0);
  __syncthreads();
  for (int t = 0; t < ktiles; ++t) {
    const int buf = t & 1;
    if (t + 1 < ktiles) load_tile((t + 1) * BK);
#pragma unroll
    for (int kk = 0; kk < BK; kk += 8) {
      shortx4 a[WM], b[WN];
      const int kb = kk + lane_hi * 4;
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) a[i][e] = (short)As[buf][kb + e][am + i * 32];
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) b[j][e] = (short)Bs[buf][kb + e][bn + j * 32];
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (t + 1 < ktiles) store_tile(buf ^ 1);
    __syncthreads();
  }

  float* __restrict__ C = p.C + (long long)g * p.c_gs;
  const float* bias = p.bias ? p.bias + (long long)g * p.bias_gs : nullptr;
  // A lane's column and its lane half's 4 rows give one 64-bit base per column block; the row
  // of each accumulator register is a uniform multiple of the row stride on top of it.  Tiles that
  // lie completely inside M (all but the last row of tiles) need no per-lane row check.
  const int mw = m0 + wave_m * WM * 32;
  const bool full_m = m0 + BM <= p.M;
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    const int col = n0 + bn + j * 32;
    if (col >= p.Ncols) continue;
    float* __restrict__ cl = C + col_offset(p.cmap, col) + (long long)(mw + lane_hi * 4) * p.c_ms;
    const float* bl = bias ? bias + mw + lane_hi * 4 : nullptr;
#pragma unroll
    for (int i = 0; i < WM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = i * 32 + (r >> 2) * 8 + (r & 3);   // relative to mw + 4*lane_hi
        if (full_m || mw + row + lane_hi * 4 < p.M) {
          float v = acc[i][j][r];
          if (bl) v += bl[row];
          cl[(long long)row * p.c_ms] = v;
        }
      }
    }
  }
}

template <int BM, int BN, int BK, int WM, int WN>
int launch_f32(const GemmTN& p, hipStream_t st) {
  const int tiles_m = p.Mpad / BM;
  const int tiles_n = (p.Ncols + BN - 1) / BN;
  const long long blocks = (long long)tiles_m * tiles_n;
  if (blocks <= 0 || blocks >= 2147483647LL || p.G > 65535) return CCT_EUNSUPPORTED;
  const bool plainB = p.bmap.P == 2147483647;
  // vector path: plain 16-byte aligned rows, padded so that a whole column tile can be read
  const bool vec = plainB && (p.b_ks % 4 == 0) && (p.b_gs % 4 == 0) &&
                   (reinterpret_cast<uintptr_t>(p.B) % 16 == 0) && p.b_ld_guard % BN == 0 &&
                   p.b_ld_guard >= p.Ncols && p.b_ks >= p.b_ld_guard;
  dim3 grid((unsigned)blocks, (unsigned)p.G);
  char name[96];
  // fused lowering: tap table in LDS when it fits 24 KiB (and the kernel size fits 15 bits)
  const size_t tab_bytes = (size_t)p.Kpad * sizeof(int2);
  const bool tab_ok = tab_bytes <= 24576 && p.gK < 32768;
  const int bmode = p.gather ? (p.tapmajor ? 4 : (tab_ok ? 2 : 3)) : (vec ? 0 : 1);
  // unpadded gather through buffer loads: the whole tensor within 2 GiB
  int gather_fast =
      p.gather && p.gp == 0 &&
      ((double)p.Ncols / (p.gHout * p.gWout)) * p.gC * p.gH * p.gW * 4.0 < 2147483648.0;
  // column-mapped B (a tensor read in place) through buffer loads: one group's operand within
  // 2 GiB and an even number of K rows (two rows are loaded per instruction)
  if (bmode == 1 && p.Kdim % 2 == 0 && p.Kdim >= 2) {
    const long long max_col = (long long)((p.Ncols - 1) / p.bmap.P) * p.bmap.img_stride +
                              (p.Ncols - 1) % p.bmap.P;
    if ((max_col + (long long)(p.Kdim + 1) * p.b_ks) * 4 < (1LL << 31)) gather_fast |= 2;
  }
  snprintf(name, sizeof(name), "gemm_tn_f32<%d, %d, %d, %d, %d, %d>", BM, BN, BK, WM, WN, bmode);
  // algorithmic bytes: operands once + result once (fused lowering: the tensor x, not D^)
  const double b_bytes = p.gather ? 4.0 * ((double)p.Ncols / (p.gHout * p.gWout)) * p.gC * p.gH * p.gW
                                  : 4.0 * (double)p.Kdim * p.Ncols * p.G;
  ProfScope ps(name, 2.0 * p.M * p.Ncols * p.Kdim * p.G,
               b_bytes + 4.0 * ((double)p.M * p.Ncols + (double)p.M * p.Kdim) * p.G, st);
  if (bmode == 4) {
    const long long taps = (long long)p.tKi * p.tKj;
    if (p.gCpad % BK || p.Kpad != taps * p.gCpad || taps * BN * 4 > 32768 || p.gs != 1 ||
        ((double)p.Ncols / (p.gHout * p.gWout)) * p.gC * p.gH * p.gW * 4.0 >= 2147483648.0)
      return CCT_EINVAL;
    hipLaunchKernelGGL((gemm_tn_f32<BM, BN, BK, WM, WN, 4>), grid, dim3(NT),
                       (size_t)taps * BN * sizeof(unsigned), st, p, tiles_m, tiles_n, gather_fast);
  } else if (bmode == 2)
    hipLaunchKernelGGL((gemm_tn_f32<BM, BN, BK, WM, WN, 2>), grid, dim3(NT), tab_bytes, st, p,
                       tiles_m, tiles_n, gather_fast);
  else if (bmode == 3)
    hipLaunchKernelGGL((gemm_tn_f32<BM, BN, BK, WM, WN, 3>), grid, dim3(NT), 0, st, p, tiles_m,
                       tiles_n, gather_fast);
  else if (bmode == 0)
    hipLaunchKernelGGL((gemm_tn_f32<BM, BN, BK, WM, WN, 0>), grid, dim3(NT), 0, st, p, tiles_m,
                       tiles_n, gather_fast);
  else
    hipLaunchKernelGGL((gemm_tn_f32<BM, BN, BK, WM, WN, 1>), grid, dim3(NT), 0, st, p, tiles_m,
                       tiles_n, gather_fast);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

template <int BM, int BN, int BK, int WM, int WN>
int launch_bf16(const GemmTN& p, hipStream_t st) {
  const int tiles_m = p.Mpad / BM;
  const int tiles_n = (p.Ncols + BN - 1) / BN;
  const long long blocks = (long long)tiles_m * tiles_n;
  if (blocks <= 0 || blocks >= 2147483647LL || p.G > 65535) return CCT_EUNSUPPORTED;
  const bool plainB = p.bmap.P == 2147483647;
  if (!plainB || p.b_ks % 8 || p.b_gs % 8 || reinterpret_cast<uintptr_t>(p.B) % 16)
    return CCT_EUNSUPPORTED;
  dim3 grid((unsigned)blocks, (unsigned)p.G);
  char name[96];
  snprintf(name, sizeof(name), "gemm_tn_bf16<%d, %d, %d, %d, %d>", BM, BN, BK, WM, WN);
  ProfScope ps(name, 2.0 * p.M * p.Ncols * p.Kdim * p.G,
               ((double)p.Kdim * p.Ncols * 2.0 + (double)p.M * p.Ncols * 4.0 + (double)p.M * p.Kdim * 2.0) * p.G,
               st);
  hipLaunchKernelGGL((gemm_tn_bf16<BM, BN, BK, WM, WN>), grid, dim3(NT), 0, st, p, tiles_m, tiles_n);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

}  // namespace

// One tile family for now: M tiles of 64, 96 or 128 rows by 128 columns.
// Tile family: M tiles of 64, 96 or 128 rows by 128 columns.  (256-column tiles were measured
// and bring nothing at the register budget they need.)
void gemm_tn_tile(int M, int /*Ncols*/, int* BM, int* BN, int* BK) {
  *BK = 16;
  *BN = 128;
  if (M <= 64)
    *BM = 64;
  else if (M % 128 != 0 && M % 96 == 0)
    *BM = 96;
  else
    *BM = 128;
}

int launch_gemm_tn(const GemmTN& p0, hipStream_t st) {
  GemmTN p = p0;
  colmap_prepare(&p.bmap);
  colmap_prepare(&p.cmap);
  int BM, BN, BK;
  gemm_tn_tile(p.M, p.Ncols, &BM, &BN, &BK);
  if (p.force_bm == 64 || p.force_bm == 96 || p.force_bm == 128) BM = p.force_bm;
  if (p.Mpad % BM || p.Kpad % BK || p.Mpad < p.M || p.Kpad < p.Kdim) return CCT_EINVAL;
  if (p.bf16) {
    if (BM == 64) return launch_bf16<64, 128, 16, 1, 2>(p, st);
    if (BM == 96) return launch_bf16<96, 128, 16, 3, 1>(p, st);
    return launch_bf16<128, 128, 16, 2, 2>(p, st);
  }
  if (BM == 64) return launch_f32<64, 128, 16, 1, 2>(p, st);
  if (BM == 96) return launch_f32<96, 128, 16, 3, 1>(p, st);
  return launch_f32<128, 128, 16, 2, 2>(p, st);
}

}  // namespace cct
