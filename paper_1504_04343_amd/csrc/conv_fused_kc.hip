// Fused forward / backward-data pass (the "Fusion" of Sec. 2.1) with channel-contiguous operands:
// the reduction index is ordered (channel group of 16, tap, channel), so that a lane fetches four
// reduction indices of its row / position with ONE 16-byte access.
//
// Why: on gfx950 the rate of an LDS-fed v_mfma_f32_32x32x2_f32 loop depends on how many LDS
// instructions accompany each MFMA.  With 4-byte operand reads (one LDS instruction per MFMA)
// a 64x64 wave tile tops out near 134 TFLOP/s; with 16-byte reads that cover four K-steps
// (0.25 LDS instructions per MFMA) the same loop reaches 150.  The first form of this kernel
// (conv_fused.hip) reads its B operand element by element from per-channel regions; this form
// transposes the staged input to [cell][channel] while writing it to LDS, which costs nothing:
// a thread already holds the 16 channels of its cells in registers and writes them as four
// 16-byte stores instead of sixteen 4-byte ones.
//
// Product: C[o][pos] = sum_{grp, tap, c} K^[grp][tap][o][c] * xpad[n, grp*16 + c, r*s + i, c*s + j]
//   - a workgroup owns BM kernels x 128 consecutive positions (output pixels of the chunk);
//   - per channel group it stages the zero-padded input rows those positions can touch as cells
//     (row, column) of 16 channels each, 20 floats apart (the 4 spare floats spread consecutive
//     cells over all LDS banks for 16-byte accesses), in a two-slot ring: the global loads of
//     group g+1 are in flight while group g is multiplied;
//   - one K tile = one tap of one channel group = 16 reduction indices.  The B operand of a lane
//     is the 16 channels of cell  base(position) + tap offset;
//   - the kernel matrix comes packed as [group][tap][kernel][16 channels] (pack_fused_kc_kernel)
//     and never passes through LDS: a K tile of the pack is Mpad rows of 64 bytes, a lane needs 16
//     of them per block (twice per tile on 32 x 32 blocks), and it loads them straight from the
//     pack with 16-byte buffer loads issued two (four) tiles ahead, the tile in the scalar offset.
//     The loads cost no address arithmetic and their latency (an L2 hit) is covered by whole
//     tiles of MFMAs.  Against staging the kernel tile through LDS this takes 6 of 11 LDS
//     instructions per tile, the tap-table read and the workgroup barrier per tile out of the
//     loop: the workgroup meets once per channel group, when the next group's cells are published;
//   - reduction index q*8 + half*4 + e goes to MFMA (q, e), lane half `half`, on both sides;
//   - epilogue = Type-1 lifting + bias, as in the plain GEMM, or the depth-to-space store of a
//     strided backward-data pass.
#include <stdio.h>

#include <algorithm>

#include "cct_internal.h"
#include "conv_fused_kc_common.h"
#include "gemm_common.h"
#include "index_common.h"

namespace cct {
namespace {

using namespace kc;
constexpr int CS = CG + 4;  // floats between cells in LDS
typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));  // 16 bytes, dword aligned

template <int BM, int WM, int WN>
__global__ __launch_bounds__(NT) void conv_fused_kc_f32(GemmTN p, KcGeom fg, int tiles_m,
                                                         int tiles_n) {
  // BM == 48: at most 48 rows (kernels, or sub-pixel channels of a strided backward-data pass),
  // computed with v_mfma_f32_16x16x4_f32 on 16 x 16 blocks so that no MFMA works on padding rows:
  // WM = 3 row blocks, WN = 2 column blocks per wave, all four waves side by side along the
  // positions.  A lane quarter (lane / 16) then supplies four of a tile's 16 reduction indices,
  // so ONE 16-byte load / read per block covers the whole tile.
  constexpr bool M16 = BM == 48;
  constexpr int MB = M16 ? 16 : 32;  // block edge
  constexpr int WAVES_N = BN / (MB * WN);
  constexpr int WAVES_M = BM / (MB * WM);
  static_assert(WAVES_M * WAVES_N == 4, "4 waves per workgroup");

  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* Xs = smem;  // [2][R][CS]
  const int slot_h = fg.R * CS;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
  const int lane_lo = M16 ? (lane & 15) : (lane & 31);  // row / column inside a block
  const int lane_hi = M16 ? (lane >> 4) : (lane >> 5);  // which reduction indices the lane supplies

  // consecutive workgroup ids go round-robin over the 8 XCDs: give every XCD a contiguous run of
  // column tiles with the M tiles of one column tile next to each other (they share x through L2)
  int bid = blockIdx.x;
  {
    const int total = tiles_m * tiles_n;
    const int per = total >> 3, rem = total & 7;
    const int xcd = bid & 7, idx = bid >> 3;
    bid = xcd * per + min(xcd, rem) + idx;
  }
  const int tile_n = bid / tiles_m;
  const int tile_m = bid - tile_n * tiles_m;
  const int g = blockIdx.y;
  const int m0 = tile_m * BM;

  // ---- which positions, images and output rows does this workgroup cover ---------------------
  const int P = p.gHout * p.gWout;
  int n0, ce;  // positions [n0, ce) of the chunk
  if (fg.tpi > 0) {
    const int img = tile_n / fg.tpi;
    n0 = img * P + (tile_n - img * fg.tpi) * BN;
    ce = min(n0 + BN, (img + 1) * P);
  } else {
    n0 = tile_n * BN;
    ce = min(n0 + BN, p.Ncols);
  }
  const int n_f = n0 / P;
  const int a_f = (n0 - n_f * P) / p.gWout;
  const int n_l = (ce - 1) / P;
  const int a_l = ((ce - 1) - n_l * P) / p.gWout;
  const int rows_first = ((n_f == n_l ? a_l : p.gHout - 1) - a_f) * p.gs + p.gK;
  const int len_first = rows_first * fg.Wp;
  const int len_full = ((p.gHout - 1) * p.gs + p.gK) * fg.Wp;
  const int rows_last = n_l == n_f ? rows_first : a_l * p.gs + p.gK;
  const int r_actual = (n_l == n_f ? 0 : len_first + (n_l - n_f - 1) * len_full) + rows_last * fg.Wp;

  // cell q -> offset of its pixel inside x, relative to (first image, first channel of the
  // group), or -1 for padding / cells past the rows this workgroup needs
  auto src_of = [&](int q) -> long long {
    if (q >= r_actual) return -1;
    int seg = 0, rem = q, a_lo = a_f;
    if (q >= len_first) {
      const int qq = q - len_first;
      seg = 1 + qq / len_full;
      rem = qq - (seg - 1) * len_full;
      a_lo = 0;
    }
    const int row = rem / fg.Wp, wp = rem - row * fg.Wp;
    const int h = a_lo * p.gs + row - p.gp, w = wp - p.gp;
    if (h < 0 || h >= p.gH || w < 0 || w >= p.gW) return -1;
    return ((long long)seg * p.gC * p.gH + h) * p.gW + w;
  };
  const long long chan_stride = (long long)p.gH * p.gW;

  // ---- staging: a thread owns cells tid + u*256 of every group.  The cell's byte offset inside
  // the tensor never changes; dead cells get an offset that fails the buffer range check and load
  // as zero; the channel enters through the scalar offset of the buffer load, channels past the
  // group's last one through an empty range.
  unsigned stg_voff[QU];
  float stg[QU * CG];
  const float* Xb = reinterpret_cast<const float*>(p.B) +
                    ((long long)n_f * p.gC + (long long)g * p.gCg) * chan_stride;
#pragma unroll
  for (int u = 0; u < QU; ++u) {
    const long long src = src_of(tid + u * NT);
    stg_voff[u] = src >= 0 ? (unsigned)src * 4u : 0x80000000u;
  }
#define CCT_STAGE_LOAD(GIDX)                                                                \
  {                                                                                         \
    _Pragma("unroll") for (int u = 0; u < QU; ++u) {                                        \
      if (tid + u * NT < fg.R) { /* whole waves: R is a multiple of 64 */                   \
        _Pragma("unroll") for (int cc = 0; cc < CG; ++cc) {                                 \
          const int ch = (GIDX) * CG + cc;                                                  \
          const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(              \
              const_cast<float*>(Xb), 0, ch < p.gCg ? 0x7fffffff : 0, 0x00020000);          \
          stg[u * CG + cc] = __builtin_bit_cast(                                            \
              float, __builtin_amdgcn_raw_buffer_load_b32(                                  \
                         rs, (int)stg_voff[u], (int)((unsigned)ch * (unsigned)chan_stride * 4u), 0)); \
        }                                                                                   \
      }                                                                                     \
    }                                                                                       \
  }
#define CCT_STAGE_STORE(SLOT)                                                               \
  {                                                                                         \
    _Pragma("unroll") for (int u = 0; u < QU; ++u) {                                        \
      const int q = tid + u * NT;                                                           \
      if (q < fg.R) {                                                                       \
        _Pragma("unroll") for (int v = 0; v < CG / 4; ++v) {                                \
          f32x4 val;                                                                        \
          _Pragma("unroll") for (int e = 0; e < 4; ++e) val[e] = stg[u * CG + v * 4 + e];   \
          *reinterpret_cast<f32x4*>(&Xs[(SLOT) * slot_h + q * CS + v * 4]) = val;           \
        }                                                                                   \
      }                                                                                     \
    }                                                                                       \
  }
  CCT_STAGE_LOAD(0);
  CCT_STAGE_STORE(0);
  if (fg.ngroups > 1) CCT_STAGE_LOAD(1);

  // ---- kernel-matrix operands come straight from the pack (L2) into registers, AD tiles ahead.
  // Tiles are taken AD at a time: the pack carries zero tiles up to a multiple of four, whose
  // B operands are cells of the last group again (finite data times zero).  The 16 x 16 form has
  // shorter tiles (24 MFMAs of 8 passes against 32 of 16), so it looks further ahead.
  constexpr int AD = M16 ? 4 : 2;
  constexpr int NQ = M16 ? 1 : 2;  // 16-byte loads per block and tile
  const int ktiles = (fg.ngroups * fg.KK + AD - 1) / AD * AD;
  const float* Abase = reinterpret_cast<const float*>(p.A) + ((long long)g * p.a_gs + (long long)m0 * CG);
  const __amdgpu_buffer_rsrc_t a_rs =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(Abase), 0, 0x7fffffff, 0x00020000);
  const int a_voff = ((wave_m * WM * MB + lane_lo) * CG + lane_hi * 4) * 4;  // bytes inside a tile
  const unsigned a_tile_bytes = (unsigned)p.Mpad * CG * 4u;
  // [tile mod AD][block][q]: reduction indices 8q + 4*half + e (32 x 32), 4*quarter + e (16 x 16)
  f32x4 ra[AD][WM][NQ];
#define CCT_LOAD_A(SET, T)                                                                  \
  {                                                                                         \
    _Pragma("unroll") for (int i = 0; i < WM; ++i)                                          \
      _Pragma("unroll") for (int q = 0; q < NQ; ++q)                                        \
        ra[SET][i][q] = __builtin_bit_cast(                                                 \
            f32x4, __builtin_amdgcn_raw_buffer_load_b128(a_rs, a_voff + (i * MB * CG + q * 8) * 4, \
                                                         (int)((unsigned)(T) * a_tile_bytes), 0)); \
  }

  constexpr int AR = M16 ? 4 : 16;  // accumulator registers per block
  typedef float acc_t __attribute__((ext_vector_type(AR)));
  acc_t acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < AR; ++r) acc[i][j][r] = 0.f;

  // per-lane base of each owned position's cell (element offsets)
  const int bn = wave_n * WN * MB + lane_lo;
  int bbase[WN];
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    const int col = n0 + bn + j * MB;
    int cb = 0;
    if (col < ce) {
      const int n = col / P, pix = col - n * P;
      const int r = pix / p.gWout, c = pix - r * p.gWout;
      const int seg = n == n_f ? 0 : len_first + (n - n_f - 1) * len_full;
      const int a_lo = n == n_f ? a_f : 0;
      cb = seg + (r - a_lo) * p.gs * fg.Wp + c * p.gs;
    }
    bbase[j] = cb * CS + lane_hi * 4;
  }

#pragma unroll
  for (int e = 0; e < AD; ++e) CCT_LOAD_A(e, e);  // ktiles >= AD
  __syncthreads();                                  // slot 0 is visible

  f32x4 b[2][WN];              // [q][block]
  int tt = 0, ti = 0, tj = 0;  // tap inside the current channel group, and its (row, column)
  int grp = 0;                 // current channel group
  int slot = 0;                // ring slot of the current group
#pragma unroll
  for (int j = 0; j < WN; ++j) b[0][j] = *reinterpret_cast<const f32x4*>(&Xs[bbase[j]]);

  if constexpr (M16) {
    // One tile: the B operands of the next tap are read before this tile's MFMAs, which cover the
    // read; the registers of this tile's A operand are reloaded with tile t + AD right after them.
    // At a group's last tap: publish the next group's cells, barrier, first read from the new slot.
#define CCT_TILE16(SET, CUR, NXT)                                                           \
  {                                                                                         \
    const bool last_tap = tt == fg.KK - 1;                                                  \
    int tj_n = tj + 1, ti_n = ti;                                                           \
    if (tj_n == p.gK) {                                                                     \
      tj_n = 0;                                                                             \
      ti_n = ti + 1;                                                                        \
    }                                                                                       \
    if (!last_tap) {                                                                        \
      const int tapo = (ti_n * fg.Wp + tj_n) * CS + slot * slot_h;                          \
      _Pragma("unroll") for (int j = 0; j < WN; ++j) b[NXT][j] =                            \
          *reinterpret_cast<const f32x4*>(&Xs[bbase[j] + tapo]);                            \
    }                                                                                       \
    _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                         \
      __builtin_amdgcn_sched_barrier(0);                                                    \
      _Pragma("unroll") for (int i = 0; i < WM; ++i)                                        \
        _Pragma("unroll") for (int j = 0; j < WN; ++j)                                      \
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(ra[SET][i][0][e], b[CUR][j][e],  \
                                                           acc[i][j], 0, 0, 0);             \
      __builtin_amdgcn_sched_barrier(0);                                                    \
    }                                                                                       \
    if (t + AD < ktiles) CCT_LOAD_A(SET, t + AD);                                           \
    if (last_tap) {                                                                         \
      const bool more_groups = grp + 1 < fg.ngroups; /* false inside the zero tiles too */  \
      if (more_groups) CCT_STAGE_STORE(slot ^ 1);                                           \
      __syncthreads();                                                                      \
      if (more_groups) slot ^= 1;                                                           \
      ++grp;                                                                                \
      if (grp + 1 < fg.ngroups) CCT_STAGE_LOAD(grp + 1);                                    \
      tt = 0;                                                                               \
      ti = 0;                                                                               \
      tj = 0;                                                                               \
      const int tapo = slot * slot_h;                                                       \
      _Pragma("unroll") for (int j = 0; j < WN; ++j) b[NXT][j] =                            \
          *reinterpret_cast<const f32x4*>(&Xs[bbase[j] + tapo]);                            \
    } else {                                                                                \
      ++tt;                                                                                 \
      ti = ti_n;                                                                            \
      tj = tj_n;                                                                            \
    }                                                                                       \
    ++t;                                                                                    \
  }
    static_assert(AD == 4 || !M16, "the loop below is unrolled by AD");
    int t = 0;
    while (t < ktiles) {  // one exit: ktiles is a multiple of AD
      CCT_TILE16(0, 0, 1);
      CCT_TILE16(1, 1, 0);
      CCT_TILE16(2, 0, 1);
      CCT_TILE16(3, 1, 0);
    }
#undef CCT_TILE16
  } else {
  // One tile = 16 reduction indices = two halves (q) of four MFMA groups (e) each.  The second
  // half's B operands are read before the first half's MFMAs and the next tile's first half behind
  // them, so every LDS read is covered by sixteen MFMAs; the registers of this tile's A operand are
  // reloaded with tile t + AD at its end.  The workgroup meets once per channel group: in the middle
  // of a group's last tap every thread publishes its cells of the next group (loaded while this
  // group was multiplied), the barrier makes them visible and frees the other slot, and the loads of
  // the group after start.
#define CCT_MFMA_GROUP(SET, Q, E)                                                           \
  {                                                                                         \
    __builtin_amdgcn_sched_barrier(0);                                                      \
    _Pragma("unroll") for (int i = 0; i < WM; ++i)                                          \
      _Pragma("unroll") for (int j = 0; j < WN; ++j)                                        \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(ra[SET][i][Q][E], b[Q][j][E],      \
                                                         acc[i][j], 0, 0, 0);               \
    __builtin_amdgcn_sched_barrier(0);                                                      \
  }
#define CCT_TILE(SET)                                                                       \
  {                                                                                         \
    const bool last_tap = tt == fg.KK - 1;                                                  \
    {                                                                                       \
      const int cur = (ti * fg.Wp + tj) * CS + slot * slot_h + 8;                           \
      _Pragma("unroll") for (int j = 0; j < WN; ++j) b[1][j] =                              \
          *reinterpret_cast<const f32x4*>(&Xs[bbase[j] + cur]);                             \
    }                                                                                       \
    CCT_MFMA_GROUP(SET, 0, 0);                                                              \
    CCT_MFMA_GROUP(SET, 0, 1);                                                              \
    CCT_MFMA_GROUP(SET, 0, 2);                                                              \
    CCT_MFMA_GROUP(SET, 0, 3);                                                              \
    if (last_tap) {                                                                         \
      const bool more_groups = grp + 1 < fg.ngroups; /* false inside the zero tile too */   \
      if (more_groups) CCT_STAGE_STORE(slot ^ 1);                                           \
      __syncthreads();                                                                      \
      if (more_groups) slot ^= 1;                                                           \
      ++grp;                                                                                \
      if (grp + 1 < fg.ngroups) CCT_STAGE_LOAD(grp + 1);                                    \
      tt = 0;                                                                               \
      ti = 0;                                                                               \
      tj = 0;                                                                               \
    } else {                                                                                \
      ++tt;                                                                                 \
      if (++tj == p.gK) {                                                                   \
        tj = 0;                                                                             \
        ++ti;                                                                               \
      }                                                                                     \
    }                                                                                       \
    {                                                                                       \
      const int nxt = (ti * fg.Wp + tj) * CS + slot * slot_h;                               \
      _Pragma("unroll") for (int j = 0; j < WN; ++j) b[0][j] =                              \
          *reinterpret_cast<const f32x4*>(&Xs[bbase[j] + nxt]);                             \
    }                                                                                       \
    CCT_MFMA_GROUP(SET, 1, 0);                                                              \
    CCT_MFMA_GROUP(SET, 1, 1);                                                              \
    CCT_MFMA_GROUP(SET, 1, 2);                                                              \
    CCT_MFMA_GROUP(SET, 1, 3);                                                              \
    if (t + AD < ktiles) CCT_LOAD_A(SET, t + AD);                                           \
    ++t;                                                                                    \
  }
    static_assert(AD == 2 || M16, "the loop below is unrolled by AD");
    int t = 0;
    while (t < ktiles) {  // one exit: ktiles is a multiple of AD
      CCT_TILE(0);
      CCT_TILE(1);
    }
#undef CCT_MFMA_GROUP
  }
#undef CCT_TILE
#undef CCT_LOAD_A
#undef CCT_STAGE_LOAD
#undef CCT_STAGE_STORE

  // ---- epilogue: Type-1 lifting + bias.  Accumulator register r of block row i is row
  // i*32 + 8*(r/4) + 4*(lane/32) + r%4 of the wave's rows (32 x 32 blocks), or
  // i*16 + 4*(lane/16) + r (16 x 16 blocks): four consecutive rows per lane either way.
  const int mw = m0 + wave_m * WM * MB;
  if (p.d2s) {
    // depth-to-space: a lane's four consecutive rows are four sub-pixels of its grid position
    float* __restrict__ D = p.C;
    const int ss = p.dS * p.dS;
#pragma unroll
    for (int j = 0; j < WN; ++j) {
      const int col = n0 + bn + j * MB;
      if (col >= ce) continue;
      const int n = col / P, pix = col - n * P;
      const int ga = pix / p.gWout, gb = pix - ga * p.gWout;
      const long long img = ((long long)n * p.dCtot + (long long)g * p.dCg) * p.dH;
#pragma unroll
      for (int i = 0; i < WM; ++i) {
#pragma unroll
        for (int r4 = 0; r4 < AR; r4 += 4) {
          // the lane's four consecutive rows m .. m+3 (m a multiple of 4)
          const int m = mw + (M16 ? i * 16 : i * 32 + (r4 >> 2) * 8) + lane_hi * 4;
          if (m >= p.M) continue;
          const int ci = fdiv_u(m, p.d_divSS_M, p.d_divSS_sh), rem = m - ci * ss;
          const int rh = fdiv_u(rem, p.d_divS_M, p.d_divS_sh), rw = rem - rh * p.dS;
          const int h = ga * p.dS + rh - p.dP, w = gb * p.dS + rw - p.dP;
          float* dst = D + ((img + (long long)ci * p.dH) + h) * p.dW + w;
          if ((p.dS & 3) == 0) {
            // stride a multiple of 4: the four rows are four consecutive pixels of one row of dx
            if ((unsigned)h >= (unsigned)p.dH) continue;
            if (w >= 0 && w + 3 < p.dW && m + 3 < p.M) {
              f32x4u v = {acc[i][j][r4], acc[i][j][r4 + 1], acc[i][j][r4 + 2], acc[i][j][r4 + 3]};
              *reinterpret_cast<f32x4u*>(dst) = v;  // 4-byte aligned
            } else {
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (m + e < p.M && (unsigned)(w + e) < (unsigned)p.dW) dst[e] = acc[i][j][r4 + e];
            }
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int me = m + e;
              if (me < p.M) {
                const int cie = fdiv_u(me, p.d_divSS_M, p.d_divSS_sh), reme = me - cie * ss;
                const int rhe = fdiv_u(reme, p.d_divS_M, p.d_divS_sh), rwe = reme - rhe * p.dS;
                const int he = ga * p.dS + rhe - p.dP, we = gb * p.dS + rwe - p.dP;
                if ((unsigned)he < (unsigned)p.dH && (unsigned)we < (unsigned)p.dW)
                  D[((img + (long long)cie * p.dH) + he) * p.dW + we] = acc[i][j][r4 + e];
              }
            }
          }
        }
      }
    }
    return;
  }
  float* __restrict__ C = p.C + (long long)g * p.c_gs;
  const float* bias = p.bias ? p.bias + (long long)g * p.bias_gs : nullptr;
  const bool full_m = m0 + BM <= p.M;
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    const int col = n0 + bn + j * MB;
    if (col >= ce) continue;
    float* __restrict__ cl = C + col_offset(p.cmap, col) + (long long)(mw + lane_hi * 4) * p.c_ms;
    const float* bl = bias ? bias + mw + lane_hi * 4 : nullptr;
#pragma unroll
    for (int i = 0; i < WM; ++i) {
#pragma unroll
      for (int r = 0; r < AR; ++r) {
        const int row = M16 ? i * 16 + r : i * 32 + (r >> 2) * 8 + (r & 3);  // relative to mw + 4*lane_hi
        if (full_m || mw + row + lane_hi * 4 < p.M) {
          float v = acc[i][j][r];
          if (bl) v += bl[row];
          cl[(long long)row * p.c_ms] = v;
        }
      }
    }
  }
}

// Geometry and LDS need; false = this form cannot run the shape.  No kernel tiles live in LDS
// (row count 0); the pack of one group is addressed with 32-bit byte offsets.
// The 16 x 16 block form has short tiles and gains from a third workgroup per CU (measured on
// conv2's backward-data pass: 131 against 124 TFLOP/s), so it first tries the geometry that fits
// a third of the LDS; the 32 x 32 forms do not (their tiles cut per image waste more than the third
// workgroup brings).
bool make_kc_geom(const GemmTN& p, int BM, KcGeom* fg, size_t* lds) {
  if (p.bf16 || (long long)p.Mpad * p.Kpad * 4 >= (1LL << 31)) return false;
  if (BM == 48 && kc::make_geom(p, 0, CS * 4, fg, lds, kLdsCap3)) return true;
  return kc::make_geom(p, 0, CS * 4, fg, lds);
}

template <int BM, int WM, int WN>
int launch_variant(const GemmTN& p, const KcGeom& fg, size_t lds, hipStream_t st) {
  const int tiles_m = BM == 48 ? 1 : p.Mpad / BM;
  const long long tn = fg.tpi > 0 ? (long long)fg.tpi * (p.Ncols / (p.gHout * p.gWout))
                                  : ((long long)p.Ncols + BN - 1) / BN;
  const long long blocks = (long long)tiles_m * tn;
  if (blocks <= 0 || blocks >= 2147483647LL || p.G > 65535) return CCT_EUNSUPPORTED;
  const int tiles_n = (int)tn;
  dim3 grid((unsigned)blocks, (unsigned)p.G);
  char name[96];
  snprintf(name, sizeof(name), "conv_fused_kc_f32<%d, %d, %d>%s", BM, WM, WN, p.d2s ? " strided" : "");
  const double nimg = (double)p.Ncols / (p.gHout * p.gWout);
  const double x_bytes = 4.0 * nimg * p.gC * p.gH * p.gW;
  const double y_bytes = p.d2s ? 4.0 * nimg * p.dCtot * p.dH * p.dW : 4.0 * (double)p.M * p.Ncols * p.G;
  ProfScope ps(name, p.prof_flops > 0 ? p.prof_flops : 2.0 * p.M * p.Ncols * p.Kdim * p.G,
               x_bytes + y_bytes + 4.0 * (double)p.M * p.Kdim * p.G, st);
  constexpr auto kern = conv_fused_kc_f32<BM, WM, WN>;
  if (const int rc = ensure_dynamic_lds<kern>(kLdsCap)) return rc;
  hipLaunchKernelGGL(kern, grid, dim3(NT), lds, st, p, fg, tiles_m, tiles_n);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

// pack[q][grp][tap][m][c] (c < 16), zero padded in m (to Mpad) and c (to whole groups).
//   forward (flipped == 0): m = kernel oo < Og,  channel = input channel ci < Cg,
//                           value w[q*Og + m, grp*16 + c, i, j],            tap = i*K + j
//   backward-data (flipped): m = input channel ci < Cg, channel = kernel oo < Og,
//                           value w[q*Og + grp*16 + c, m, K-1-i, K-1-j],    tap = i*K + j
// BF16: the pack holds bf16 values (rounded to nearest even) instead of fp32.
template <bool BF16>
__global__ __launch_bounds__(256) void pack_fused_kc_kernel(const float* __restrict__ w,
                                                            void* __restrict__ pack, int G, int Og,
                                                            int Cg, int K, int Mpad, int ktiles,
                                                            int flipped) {
  // ktiles >= groups of 16 channels x taps; tiles beyond that product decode to channels past the
  // last one and are written as zeros
  const int KK = K * K;
  const long long per_group = (long long)ktiles * Mpad * CG;
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= per_group * G) return;
  const int q = (int)(t / per_group);
  long long e = t - q * per_group;
  const int c = (int)(e % CG);
  e /= CG;
  const int m = (int)(e % Mpad);
  e /= Mpad;
  const int tap = (int)(e % KK), grp = (int)(e / KK);
  const int i = tap / K, j = tap - i * K;
  const int ch = grp * CG + c;
  float v = 0.0f;
  if (!flipped) {
    if (m < Og && ch < Cg) v = w[((((long long)q * Og + m) * Cg + ch) * K + i) * K + j];
  } else {
    if (m < Cg && ch < Og)
      v = w[((((long long)q * Og + ch) * Cg + m) * K + (K - 1 - i)) * K + (K - 1 - j)];
  }
  store_elem<BF16>(pack, t, v);
}

// Kernel pack of the strided backward-data pass (see launch_pack_fused_kc_strided).
template <bool BF16>
__global__ __launch_bounds__(256) void pack_fused_kc_strided_kernel(const float* __restrict__ w,
                                                                    void* __restrict__ pack, int G,
                                                                    int Og, int Cg, int K, int s, int U,
                                                                    int Mpad, int ktiles) {
  const int UU = U * U;
  const long long per_group = (long long)ktiles * Mpad * CG;
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= per_group * G) return;
  const int q = (int)(t / per_group);
  long long e = t - q * per_group;
  const int c = (int)(e % CG);
  e /= CG;
  const int m = (int)(e % Mpad);
  e /= Mpad;
  const int tap = (int)(e % UU), grp = (int)(e / UU);
  const int up = tap / U, vp = tap - up * U;
  const int oo = grp * CG + c;
  float v = 0.0f;
  if (m < Cg * s * s && oo < Og) {
    const int ci = m / (s * s), rem = m - ci * s * s;
    const int rh = rem / s, rw = rem - rh * s;
    const int i = rh + s * (U - 1 - up), j = rw + s * (U - 1 - vp);
    if (i < K && j < K) v = w[((((long long)q * Og + oo) * Cg + ci) * K + i) * K + j];
  }
  store_elem<BF16>(pack, t, v);
}

}  // namespace

// Row tile of this kernel: the GEMM family's choice (64 / 96 / 128), with two exceptions.
static int kc_row_tile(const GemmTN& p, int* BNt) {
  int BM, BKt;
  gemm_tn_tile(p.M, p.Ncols, &BM, BNt, &BKt);
  // Rows that are not a multiple of 128: tiles of 64 rows (4 workgroups per CU, and three times
  // as many tiles to spread over the chip) beat 96 x 64 wave tiles (measured: 128 against 116
  // TFLOP/s on conv4's 192 rows)
  if (BM == 96 && p.Mpad % 192 == 0) BM = 64;
  if (p.M <= 48) BM = 48;  // 16 x 16 MFMA blocks: no work on padding rows beyond the 48th
  return BM;
}

bool conv_fused_kc_fits(const GemmTN& p) {
  int BNt;
  const int BM = kc_row_tile(p, &BNt);
  KcGeom fg;
  size_t lds;
  return BNt == BN && make_kc_geom(p, BM, &fg, &lds);
}

long long conv_fused_kc_kpad(int channels_per_group, int K, int bf16) {
  const long long ktiles = (long long)((channels_per_group + CG - 1) / CG) * K * K;
  return (bf16 ? (ktiles + 7) / 8 * 8 : (ktiles + 3) / 4 * 4) * CG;
}

int launch_pack_fused_kc(const float* w, void* pack, int G, int Og, int Cg, int K, int Mpad,
                         int flipped, int bf16, hipStream_t st) {
  const long long kt = conv_fused_kc_kpad(flipped ? Og : Cg, K, bf16) / CG;
  if (kt >= 2147483647LL) return CCT_EUNSUPPORTED;
  const int ktiles = (int)kt;
  const long long total = (long long)G * ktiles * Mpad * CG;
  const long long blocks = (total + 255) / 256;
  if (blocks <= 0 || blocks >= 2147483647LL) return CCT_EUNSUPPORTED;
  ProfScope ps("pack_fused_kc_kernel", 0.0, 4.0 * G * Og * Cg * K * K + (bf16 ? 2.0 : 4.0) * total, st);
  if (bf16)
    hipLaunchKernelGGL(pack_fused_kc_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, st, w, pack, G,
                       Og, Cg, K, Mpad, ktiles, flipped);
  else
    hipLaunchKernelGGL(pack_fused_kc_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, st, w, pack, G,
                       Og, Cg, K, Mpad, ktiles, flipped);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int launch_pack_fused_kc_strided(const float* w, void* pack, int G, int Og, int Cg, int K, int s,
                                 int Mpad, int bf16, hipStream_t st) {
  const int U = (K + s - 1) / s;
  const long long kt = conv_fused_kc_kpad(Og, U, bf16) / CG;
  if (kt >= 2147483647LL) return CCT_EUNSUPPORTED;
  const int ktiles = (int)kt;
  const long long total = (long long)G * ktiles * Mpad * CG;
  const long long blocks = (total + 255) / 256;
  if (blocks <= 0 || blocks >= 2147483647LL) return CCT_EUNSUPPORTED;
  ProfScope ps("pack_fused_kc_strided_kernel", 0.0,
               4.0 * G * Og * Cg * K * K + (bf16 ? 2.0 : 4.0) * total, st);
  if (bf16)
    hipLaunchKernelGGL(pack_fused_kc_strided_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, st, w,
                       pack, G, Og, Cg, K, s, U, Mpad, ktiles);
  else
    hipLaunchKernelGGL(pack_fused_kc_strided_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, st, w,
                       pack, G, Og, Cg, K, s, U, Mpad, ktiles);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

// p.A must have been written by launch_pack_fused_kc; p.Kpad = conv_fused_kc_kpad(...).
int launch_conv_fused_kc(const GemmTN& p0, hipStream_t st) {
  GemmTN p = p0;
  colmap_prepare(&p.bmap);
  colmap_prepare(&p.cmap);
  if (p.d2s) {
    if (p.dS < 1 || p.M != p.dCg * p.dS * p.dS) return CCT_EINVAL;
    make_fastdiv_parts(p.dS * p.dS, &p.d_divSS_M, &p.d_divSS_sh);
    make_fastdiv_parts(p.dS, &p.d_divS_M, &p.d_divS_sh);
  }
  int BNt;
  const int BM = kc_row_tile(p, &BNt);
  KcGeom fg;
  size_t lds;
  if (BNt != BN || (BM == 48 ? p.Mpad < 48 : p.Mpad % BM != 0) || !make_kc_geom(p, BM, &fg, &lds))
    return CCT_EUNSUPPORTED;
  if (p.Kpad != conv_fused_kc_kpad(p.gCg, p.gK, 0)) return CCT_EINVAL;
  if (BM == 48) return launch_variant<48, 3, 2>(p, fg, lds, st);
  if (BM == 64) return launch_variant<64, 1, 2>(p, fg, lds, st);
  if (BM == 96) return launch_variant<96, 3, 1>(p, fg, lds, st);
  return launch_variant<128, 2, 2>(p, fg, lds, st);
}

}  // namespace cct
