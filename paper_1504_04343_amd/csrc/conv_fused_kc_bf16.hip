// The channel-contiguous fused kernel (conv_fused_kc.hip) for bf16 operands with fp32 accumulation:
// forward and backward-data passes without a lowered matrix in the reduced-precision variant.
//
// x (or dy) stays fp32 in HBM; a thread that stages a cell rounds its 16 channels to bf16
// (v_cvt_pk_bf16_f32: round to nearest even) and writes them as two 16-byte LDS stores, so a cell
// is 32 bytes, kept 48 bytes apart (consecutive cells then cover all 32 banks once per 8 lanes of
// a 16-byte access).  The kernel matrix comes packed in bf16 as [group][tap][kernel][16 channels].
// One K tile = one tap of one channel group = 16 reduction indices = ONE
// v_mfma_f32_32x32x16_bf16 per 32 x 32 block: lane half h supplies channels 8h..8h+7 of its row
// (A) and of its position (B).
//
// The matrix cores are sixteen times faster than in fp32 while staging costs the same, so the loop
// is organised around latency and issue slots, not MFMAs: the A operand never passes through LDS
// (a lane loads the 16 bytes of its row straight from the pack, eight tiles ahead, with the tile
// in the scalar offset of a buffer load), the B operand is one 16-byte LDS read per block and tap,
// and the workgroup synchronises once per channel group (when the next group's cells are
// published), not once per tile.
#include <stdio.h>

#include <algorithm>

#include "cct_internal.h"
#include "conv_fused_kc_common.h"
#include "gemm_common.h"

namespace cct {
namespace {

using namespace kc;
constexpr int CSH = 24;  // bf16 elements between cells / kernel rows in LDS (48 bytes)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef const u32x4 __attribute__((address_space(1)))* gptr_u32x4;

__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

template <int BM, int WM, int WN>
__global__ __launch_bounds__(NT) void conv_fused_kc_bf16(GemmTN p, KcGeom fg, int tiles_m,
                                                         int tiles_n) {
  constexpr int MB = 32;
  constexpr int WAVES_N = BN / (MB * WN);
  constexpr int WAVES_M = BM / (MB * WM);
  static_assert(WAVES_M * WAVES_N == 4, "4 waves per workgroup");

  extern __shared__ __attribute__((aligned(16))) unsigned short smem_h[];
  unsigned short* Xs = smem_h;  // [2][R][CSH]
  const int slot_h = fg.R * CSH;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
  const int lane_lo = lane & 31;  // row / column inside a block
  const int lane_hi = lane >> 5;  // which half of the 16 channels the lane supplies

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
        _Pragma("unroll") for (int v = 0; v < 2; ++v) {                                     \
          u32x4 val;                                                                        \
          _Pragma("unroll") for (int e = 0; e < 4; ++e)                                     \
            val[e] = pack_bf16(stg[u * CG + v * 8 + 2 * e], stg[u * CG + v * 8 + 2 * e + 1]); \
          *reinterpret_cast<u32x4*>(&Xs[(SLOT) * slot_h + q * CSH + v * 8]) = val;          \
        }                                                                                   \
      }                                                                                     \
    }                                                                                       \
  }
  CCT_STAGE_LOAD(0);
  CCT_STAGE_STORE(0);
  if (fg.ngroups > 1) CCT_STAGE_LOAD(1);

  // ---- kernel-matrix operands come straight from the pack (L2) into registers, AD tiles ahead:
  // a K tile of the pack is Mpad rows of 32 bytes, and a lane needs the 16 bytes of its row and
  // channel half, so one 16-byte buffer load per block fetches an operand with 1 KiB of contiguous
  // addresses per block.  The tile enters through the scalar offset: no address arithmetic.
  // Tiles are taken AD at a time: the pack carries zero tiles up to the next multiple of AD, whose
  // B operands are cells of the last group again (finite data times zero).
  constexpr int AD = 8;
  const int ktiles = (fg.ngroups * fg.KK + AD - 1) / AD * AD;
  const unsigned short* Abase =
      reinterpret_cast<const unsigned short*>(p.A) + ((long long)g * p.a_gs + (long long)m0 * CG);
  const __amdgpu_buffer_rsrc_t a_rs = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<unsigned short*>(Abase), 0, 0x7fffffff, 0x00020000);
  const int a_voff = ((wave_m * WM * MB + lane_lo) * CG + lane_hi * 8) * 2;  // bytes inside a tile
  const unsigned a_tile_bytes = (unsigned)p.Mpad * CG * 2u;
  u32x4 ra[AD][WM];
#define CCT_LOAD_A(SET, T)                                                                  \
  {                                                                                         \
    _Pragma("unroll") for (int i = 0; i < WM; ++i)                                          \
      ra[SET][i] = __builtin_bit_cast(                                                      \
          u32x4, __builtin_amdgcn_raw_buffer_load_b128(a_rs, a_voff + i * MB * CG * 2,      \
                                                       (int)((unsigned)(T) * a_tile_bytes), 0)); \
  }

  floatx16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

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
    bbase[j] = cb * CSH + lane_hi * 8;
  }

#pragma unroll
  for (int e = 0; e < AD; ++e) CCT_LOAD_A(e, e);  // ktiles >= AD
  __syncthreads();                                  // slot 0 is visible

  u32x4 b[2][WN];
  int tt = 0, ti = 0, tj = 0;  // tap inside the current channel group, and its (row, column)
  int grp = 0;                 // current channel group
  int slot = 0;                // ring slot of the current group
#pragma unroll
  for (int j = 0; j < WN; ++j) b[0][j] = *reinterpret_cast<const u32x4*>(&Xs[bbase[j]]);

  // One tile.  The B operands of the next tap are read before this tile's MFMAs, which cover the
  // read; the registers of this tile's A operand are reloaded with tile t + AD right after them.
  // The workgroup meets once per channel group: behind the MFMAs of a group's last tap every
  // thread publishes its cells of the next group (loaded while this group was multiplied), the
  // barrier makes them visible and frees the other slot, and the loads of the group after start.
#define CCT_TILE(SET, CUR, NXT)                                                             \
  {                                                                                         \
    const bool last_tap = tt == fg.KK - 1;                                                  \
    int tj_n = tj + 1, ti_n = ti;                                                           \
    if (tj_n == p.gK) {                                                                     \
      tj_n = 0;                                                                             \
      ti_n = ti + 1;                                                                        \
    }                                                                                       \
    if (!last_tap) {                                                                        \
      const int tapo = (ti_n * fg.Wp + tj_n) * CSH + slot * slot_h;                         \
      _Pragma("unroll") for (int j = 0; j < WN; ++j) b[NXT][j] =                            \
          *reinterpret_cast<const u32x4*>(&Xs[bbase[j] + tapo]);                            \
    }                                                                                       \
    __builtin_amdgcn_sched_barrier(0);                                                      \
    _Pragma("unroll") for (int i = 0; i < WM; ++i)                                          \
      _Pragma("unroll") for (int j = 0; j < WN; ++j)                                        \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                \
            __builtin_bit_cast(bf16x8, ra[SET][i]), __builtin_bit_cast(bf16x8, b[CUR][j]),  \
            acc[i][j], 0, 0, 0);                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                      \
    if (t + AD < ktiles) CCT_LOAD_A(SET, t + AD);                                           \
    if (last_tap) {                                                                         \
      const bool more_groups = grp + 1 < fg.ngroups;  /* false inside the zero tiles too */ \
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
          *reinterpret_cast<const u32x4*>(&Xs[bbase[j] + tapo]);                            \
    } else {                                                                                \
      ++tt;                                                                                 \
      ti = ti_n;                                                                            \
      tj = tj_n;                                                                            \
    }                                                                                       \
    ++t;                                                                                    \
  }
  {
    static_assert(AD == 8, "the loop below is unrolled by AD");
    int t = 0;
    while (t < ktiles) {  // one exit: ktiles is a multiple of AD
      CCT_TILE(0, 0, 1);
      CCT_TILE(1, 1, 0);
      CCT_TILE(2, 0, 1);
      CCT_TILE(3, 1, 0);
      CCT_TILE(4, 0, 1);
      CCT_TILE(5, 1, 0);
      CCT_TILE(6, 0, 1);
      CCT_TILE(7, 1, 0);
    }
  }
#undef CCT_TILE
#undef CCT_LOAD_A
#undef CCT_STAGE_LOAD
#undef CCT_STAGE_STORE

  // ---- epilogue: Type-1 lifting + bias.  Accumulator register r of block row i is row
  // i*32 + 8*(r/4) + 4*(lane/32) + r%4 of the wave's rows: four consecutive rows per lane.
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
        for (int r = 0; r < 16; ++r) {
          const int m = mw + i * 32 + (r >> 2) * 8 + (r & 3) + lane_hi * 4;
          if (m < p.M) {
            const int ci = fdiv_u(m, p.d_divSS_M, p.d_divSS_sh), rem = m - ci * ss;
            const int rh = fdiv_u(rem, p.d_divS_M, p.d_divS_sh), rw = rem - rh * p.dS;
            const int h = ga * p.dS + rh - p.dP, w = gb * p.dS + rw - p.dP;
            if ((unsigned)h < (unsigned)p.dH && (unsigned)w < (unsigned)p.dW)
              D[((img + (long long)ci * p.dH) + h) * p.dW + w] = acc[i][j][r];
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
      for (int r = 0; r < 16; ++r) {
        const int row = i * 32 + (r >> 2) * 8 + (r & 3);  // relative to mw + 4*lane_hi
        if (full_m || mw + row + lane_hi * 4 < p.M) {
          float v = acc[i][j][r];
          if (bl) v += bl[row];
          cl[(long long)row * p.c_ms] = v;
        }
      }
    }
  }
}

template <int BM, int WM, int WN>
int launch_variant(const GemmTN& p, const KcGeom& fg, size_t lds, hipStream_t st) {
  const int tiles_m = p.Mpad / BM;
  const long long tn = fg.tpi > 0 ? (long long)fg.tpi * (p.Ncols / (p.gHout * p.gWout))
                                  : ((long long)p.Ncols + BN - 1) / BN;
  const long long blocks = (long long)tiles_m * tn;
  if (blocks <= 0 || blocks >= 2147483647LL || p.G > 65535) return CCT_EUNSUPPORTED;
  const int tiles_n = (int)tn;
  dim3 grid((unsigned)blocks, (unsigned)p.G);
  char name[96];
  snprintf(name, sizeof(name), "conv_fused_kc_bf16<%d, %d, %d>%s", BM, WM, WN, p.d2s ? " strided" : "");
  const double nimg = (double)p.Ncols / (p.gHout * p.gWout);
  const double x_bytes = 4.0 * nimg * p.gC * p.gH * p.gW;
  const double y_bytes = p.d2s ? 4.0 * nimg * p.dCtot * p.dH * p.dW : 4.0 * (double)p.M * p.Ncols * p.G;
  ProfScope ps(name, p.prof_flops > 0 ? p.prof_flops : 2.0 * p.M * p.Ncols * p.Kdim * p.G,
               x_bytes + y_bytes + 2.0 * (double)p.M * p.Kdim * p.G, st);
  constexpr auto kern = conv_fused_kc_bf16<BM, WM, WN>;
  if (const int rc = ensure_dynamic_lds<kern>(kLdsCap)) return rc;
  hipLaunchKernelGGL(kern, grid, dim3(NT), lds, st, p, fg, tiles_m, tiles_n);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

}  // namespace

// Row tile of the bf16 form: 64 rows up to 64, else 128; the pack is padded to whole tiles.
int conv_fused_kc_bf16_mpad(int M) { return M <= 64 ? 64 : (M + 127) / 128 * 128; }

bool conv_fused_kc_bf16_fits(const GemmTN& p) {
  KcGeom fg;
  size_t lds;
  // the pack of one group is addressed with 32-bit byte offsets
  return p.bf16 && (long long)p.Mpad * p.Kpad * 2 < (1LL << 31) && kc::make_geom(p, 0, CSH * 2, &fg, &lds);
}

// p.A must have been written by launch_pack_fused_kc* with bf16 output and
// Mpad = conv_fused_kc_bf16_mpad(M); p.Kpad = conv_fused_kc_kpad(..., 1).
int launch_conv_fused_kc_bf16(const GemmTN& p0, hipStream_t st) {
  GemmTN p = p0;
  colmap_prepare(&p.bmap);
  colmap_prepare(&p.cmap);
  if (p.d2s) {
    if (p.dS < 1 || p.M != p.dCg * p.dS * p.dS) return CCT_EINVAL;
    make_fastdiv_parts(p.dS * p.dS, &p.d_divSS_M, &p.d_divSS_sh);
    make_fastdiv_parts(p.dS, &p.d_divS_M, &p.d_divS_sh);
  }
  const int BM = p.M <= 64 ? 64 : 128;
  KcGeom fg;
  size_t lds;
  if (!p.bf16 || p.Mpad != conv_fused_kc_bf16_mpad(p.M) || (long long)p.Mpad * p.Kpad * 2 >= (1LL << 31) ||
      !kc::make_geom(p, 0, CSH * 2, &fg, &lds))  // no kernel tiles in LDS: row count 0
    return CCT_EUNSUPPORTED;
  if (p.Kpad != ((long long)fg.ngroups * fg.KK + 7) / 8 * 8 * CG) return CCT_EINVAL;
  if (BM == 64) return launch_variant<64, 1, 2>(p, fg, lds, st);
  return launch_variant<128, 2, 2>(p, fg, lds, st);
}

}  // namespace cct
