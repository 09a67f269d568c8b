// Fused forward pass (the "Fusion" of Sec. 2.1): lowering, multiply and lifting in one kernel,
// with the lowering done through LDS instead of HBM.
//
// The product is the Type-1 one, C[o][pos] = sum_{(ci,i,j)} K^[(ci,i,j)][o] * D^[(ci,i,j)][pos],
// but D^ is never built, not even as an LDS tile: a workgroup that owns 128 consecutive
// positions (output pixels of the chunk, possibly of several images) stages, per input channel,
// the zero-padded input rows those positions can touch ("region", R floats), and every lane reads
// its MFMA B operand straight from the region at
//        region(ci) + (i*Wp + j) + base(position),     base = row offset * Wp + c*stride,
// i.e. one LDS read with a per-lane base and a per-K-row offset that comes from a small table.
// Padding is materialised as zeros in the region, so the inner loop has no bounds checks.
// Channels are staged 16 at a time into a two-slot ring (global loads of the next 16 channels
// are in flight while the current 16 are multiplied); when all channels of a group number 16 or
// fewer they are staged once.  The kernel matrix K^ goes through the same double-buffered LDS
// tiles as in the plain GEMM, and the epilogue is the Type-1 lifting + bias add.
#include <stdio.h>

#include "cct_internal.h"
#include "gemm_common.h"

namespace cct {
namespace {

constexpr int NT = 256;
constexpr int BN = 128;
constexpr int BK = 16;
constexpr int CGRP = 16;  // channels per ring slot
constexpr int QU = 2;     // region floats per thread and channel in ring mode (R <= QU*256)

struct FusedGeom {
  int Wp;         // padded row width W + 2*pad
  int R;          // floats reserved per channel region (multiple of 4, >= any workgroup's need)
  int ngroups;    // ring mode: channel groups of 16; 1 = all channels staged once
  int cg;         // channels per staged group
  int KK;         // K*K
  int tab_tiles;  // K-tiles covered by the tap table (ring: one group = KK tiles; else all)
};

typedef int i32x4 __attribute__((ext_vector_type(4)));

template <int BM, int WM, int WN, bool RING>
__global__ __launch_bounds__(NT) void conv_fused_f32(GemmTN p, FusedGeom fg, int tiles_m,
                                                     int tiles_n) {
  constexpr int WAVES_N = BN / (32 * WN);
  constexpr int WAVES_M = BM / (32 * WM);
  static_assert(WAVES_M * WAVES_N == 4, "4 waves per workgroup");
  constexpr int A_VECS = BK * BM / 4;
  constexpr int A_IT = (A_VECS + NT - 1) / NT;
  constexpr int KS = BK / 2;

  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* As = smem;                                  // [2][BK*BM]
  float* Xs = smem + 2 * BK * BM;                    // [slots][cg][R]
  const int slot_floats = fg.cg * fg.R;
  const int* tab = reinterpret_cast<const int*>(Xs + (RING ? 2 : 1) * slot_floats);
  int* tab_w = reinterpret_cast<int*>(Xs + (RING ? 2 : 1) * slot_floats);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
  const int lane_lo = lane & 31, lane_hi = lane >> 5;

  int bid = blockIdx.x;
  {
    const int total = tiles_m * tiles_n;
    const int per = total >> 3, rem = total & 7;
    const int xcd = bid & 7, slot = bid >> 3;
    bid = xcd * per + min(xcd, rem) + slot;
  }
  const int tile_n = bid / tiles_m;
  const int tile_m = bid - tile_n * tiles_m;
  const int g = blockIdx.y;
  const int m0 = tile_m * BM;
  const int n0 = tile_n * BN;

  // ---- which images / output rows do this workgroup's positions cover -----------------------
  const int P = p.gHout * p.gWout;
  const int ce = min(n0 + BN, p.Ncols);
  const int n_f = n0 / P;
  const int a_f = (n0 - n_f * P) / p.gWout;
  const int n_l = (ce - 1) / P;
  const int a_l = ((ce - 1) - n_l * P) / p.gWout;
  const int rows_first = ((n_f == n_l ? a_l : p.gHout - 1) - a_f) * p.gs + p.gK;
  const int len_first = rows_first * fg.Wp;
  const int len_full = ((p.gHout - 1) * p.gs + p.gK) * fg.Wp;
  const int rows_last = n_l == n_f ? rows_first : a_l * p.gs + p.gK;
  const int r_actual = (n_l == n_f ? 0 : len_first + (n_l - n_f - 1) * len_full) + rows_last * fg.Wp;

  // region float q -> source offset inside x (relative to channel 0 of this group) or -1
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
    return (((long long)(n_f + seg) * p.gC + (long long)g * p.gCg) * p.gH + h) * p.gW + w;
  };
  const long long chan_stride = (long long)p.gH * p.gW;
  gptr_f32 X = (gptr_f32)(p.B);

  // ---- tap table: entry [tile][lane half][step] = offset of K row 16*tile + 2*step + half ----
  for (int e = tid; e < fg.tab_tiles * BK; e += NT) {
    const int tile = e >> 4, kh = (e >> 3) & 1, s = e & 7;
    const int k = tile * BK + 2 * s + kh;
    const int c = k / fg.KK, t = k - c * fg.KK;
    const int ti = t / p.gK, tj = t - ti * p.gK;
    tab_w[e] = (RING || k < p.Kdim) ? c * fg.R + ti * fg.Wp + tj : 0;
  }

  // ---- staging ---------------------------------------------------------------------------------
  // Ring mode: a thread owns region cells q = tid + u*256 of every channel.  The cell's byte
  // offset inside the tensor (relative to the first image and the group's first channel) is fixed,
  // dead cells (zero padding, cells past the rows this workgroup needs) get an offset that fails
  // the buffer range check and load as zero, and the channel enters through the scalar offset of
  // the buffer load: staging 16 channels costs no vector-ALU work besides the LDS addresses.
  unsigned stg_voff[RING ? QU : 1];
  float stg[RING ? CGRP * QU : 1];
  const float* Xb = p.B ? reinterpret_cast<const float*>(p.B) +
                              ((long long)n_f * p.gC + (long long)g * p.gCg) * chan_stride
                        : nullptr;
  if (RING) {
    const long long rel0 = ((long long)n_f * p.gC + (long long)g * p.gCg) * chan_stride;
#pragma unroll
    for (int u = 0; u < QU; ++u) {
      const long long src = src_of(tid + u * NT);
      stg_voff[u] = src >= 0 ? (unsigned)(src - rel0) * 4u : 0x80000000u;
    }
  }
#define CCT_STAGE_LOAD(GIDX)                                                                \
  {                                                                                         \
    _Pragma("unroll") for (int u = 0; u < QU; ++u) {                                        \
      if (tid + u * NT < fg.R) { /* whole waves: R is a multiple of 64 */                   \
        _Pragma("unroll") for (int cc = 0; cc < CGRP; ++cc) {                               \
          const int ch = (GIDX) * CGRP + cc;                                                \
          const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(              \
              const_cast<float*>(Xb), 0, ch < p.gCg ? 0x7fffffff : 0, 0x00020000);          \
          stg[cc * QU + u] = __builtin_bit_cast(                                            \
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
        _Pragma("unroll") for (int cc = 0; cc < CGRP; ++cc)                                 \
          Xs[(SLOT) * slot_floats + cc * fg.R + q] = stg[cc * QU + u];                      \
      }                                                                                     \
    }                                                                                       \
  }
  if (RING) {
    CCT_STAGE_LOAD(0);
    CCT_STAGE_STORE(0);
    if (fg.ngroups > 1) CCT_STAGE_LOAD(1);
  } else {
    // 4 region floats per thread and pass, so that several loads are in flight per thread
    for (int q0 = tid; q0 < fg.R; q0 += 4 * NT) {
      long long src[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) src[u] = q0 + u * NT < fg.R ? src_of(q0 + u * NT) : -1;
      for (int cc = 0; cc < fg.cg; ++cc) {
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = src[u] >= 0 ? X[src[u] + cc * chan_stride] : 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (q0 + u * NT < fg.R) Xs[cc * fg.R + q0 + u * NT] = v[u];
      }
    }
  }

  // ---- kernel-matrix tiles: global -> registers -> LDS, as in the plain GEMM ------------------
  gptr_f32 Ag = (gptr_f32)(p.A) + (long long)g * p.a_gs + m0;
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
  f32x4 ra[A_IT];
#define CCT_LOAD_A()                                                                        \
  {                                                                                         \
    _Pragma("unroll") for (int it = 0; it < A_IT; ++it) {                                   \
      if (A_VECS % NT == 0 || tid + it * NT < A_VECS) ra[it] = *(gptr_f32x4)(a_src[it]);    \
      a_src[it] += a_step;                                                                  \
    }                                                                                       \
  }
#define CCT_STORE_A(BUF)                                                                    \
  {                                                                                         \
    _Pragma("unroll") for (int it = 0; it < A_IT; ++it) {                                   \
      if (A_VECS % NT == 0 || tid + it * NT < A_VECS)                                       \
        *reinterpret_cast<f32x4*>(&As[(BUF) * BK * BM + a_dst[it]]) = ra[it];               \
    }                                                                                       \
  }

  floatx16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // per-lane base of each owned position inside a channel region
  const int am = wave_m * WM * 32 + lane_lo;
  const int bn = wave_n * WN * 32 + lane_lo;
  const int a_lds = lane_hi * BM + am;
  int colbase[WN];
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    const int col = n0 + bn + j * 32;
    int cb = 0;
    if (col < p.Ncols) {
      const int n = col / P, pix = col - n * P;
      const int r = pix / p.gWout, c = pix - r * p.gWout;
      const int seg = n == n_f ? 0 : len_first + (n - n_f - 1) * len_full;
      const int a_lo = n == n_f ? a_f : 0;
      cb = seg + (r - a_lo) * p.gs * fg.Wp + c * p.gs;
    }
    colbase[j] = cb;
  }

  const int ktiles = p.Kpad / BK;
  CCT_LOAD_A();
  CCT_STORE_A(0);
  __syncthreads();  // tap table, slot 0 and the first A tile are visible
  if (ktiles > 1) CCT_LOAD_A();

  // tap offsets of the current tile (this lane half): 8 ints
  int off[KS], offn[KS];
  {
    const i32x4 t0 = *reinterpret_cast<const i32x4*>(tab + lane_hi * KS);
    const i32x4 t1 = *reinterpret_cast<const i32x4*>(tab + lane_hi * KS + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      off[e] = t0[e];
      off[4 + e] = t1[e];
    }
  }
  float a[2][WM], b[2][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i) a[0][i] = As[a_lds + i * 32];
#pragma unroll
  for (int j = 0; j < WN; ++j) b[0][j] = Xs[off[0] + colbase[j]];

  int tt = 0;      // tile index inside the current channel group (ring mode) / overall
  int grp = 0;     // current channel group
  int slot = 0;    // ring slot of the current group
  for (int t = 0; t < ktiles; ++t) {
    const int buf = t & 1;
    const bool more = t + 1 < ktiles;
    // where does the next tile live?
    int tt_n = tt + 1, grp_n = grp, slot_n = slot;
    if (RING && tt_n == fg.KK) {
      tt_n = 0;
      grp_n = grp + 1;
      slot_n = slot ^ 1;
    }
    const float* as = As + buf * BK * BM + a_lds;
    const float* xs = Xs + slot * slot_floats;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int cur = s & 1, nxt = cur ^ 1;
      if (s + 1 < KS) {
#pragma unroll
        for (int i = 0; i < WM; ++i) a[nxt][i] = as[(s + 1) * 2 * BM + i * 32];
#pragma unroll
        for (int j = 0; j < WN; ++j) b[nxt][j] = xs[off[s + 1] + colbase[j]];
      } else {
        __syncthreads();
        if (more) {
#pragma unroll
          for (int i = 0; i < WM; ++i) a[nxt][i] = As[(buf ^ 1) * BK * BM + a_lds + i * 32];
#pragma unroll
          for (int j = 0; j < WN; ++j) b[nxt][j] = Xs[slot_n * slot_floats + offn[0] + colbase[j]];
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
        CCT_STORE_A(buf ^ 1);
        if (t + 2 < ktiles) CCT_LOAD_A();
        if (RING) {
          // last tile of a group: publish the next group's regions (their loads were issued at
          // the group's first tile); first tile of a group: start loading the group after it
          if (tt == fg.KK - 1 && grp + 1 < fg.ngroups) CCT_STAGE_STORE(slot ^ 1);
          if (tt == 0 && t > 0 && grp + 1 < fg.ngroups) CCT_STAGE_LOAD(grp + 1);
        }
        // tap offsets of the next tile
        const int tb = (RING ? tt_n : t + 1) * BK + lane_hi * KS;
        const i32x4 t0 = *reinterpret_cast<const i32x4*>(tab + tb);
        const i32x4 t1 = *reinterpret_cast<const i32x4*>(tab + tb + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          offn[e] = t0[e];
          offn[4 + e] = t1[e];
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int e = 0; e < KS; ++e) off[e] = offn[e];
    tt = tt_n;
    grp = grp_n;
    slot = slot_n;
  }
#undef CCT_LOAD_A
#undef CCT_STORE_A
#undef CCT_STAGE_LOAD
#undef CCT_STAGE_STORE

  // ---- epilogue: Type-1 lifting + bias (same accumulator layout as the plain GEMM) -------------
  float* __restrict__ C = p.C + (long long)g * p.c_gs;
  const float* bias = p.bias ? p.bias + (long long)g * p.bias_gs : nullptr;
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    const int col = n0 + bn + j * 32;
    if (col >= p.Ncols) continue;
    const long long coff = col_offset(p.cmap, col);
#pragma unroll
    for (int i = 0; i < WM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wave_m * WM * 32 + i * 32 + (r >> 2) * 8 + lane_hi * 4 + (r & 3);
        if (m < p.M) {
          float v = acc[i][j][r];
          if (bias) v += bias[m];
          C[(long long)m * p.c_ms + coff] = v;
        }
      }
    }
  }
}

template <int BM, int WM, int WN>
int launch_variant(const GemmTN& p, const FusedGeom& fg, bool ring, size_t lds, hipStream_t st) {
  const int tiles_m = p.Mpad / BM;
  const int tiles_n = (p.Ncols + BN - 1) / BN;
  const long long blocks = (long long)tiles_m * tiles_n;
  if (blocks <= 0 || blocks >= 2147483647LL || p.G > 65535) return CCT_EUNSUPPORTED;
  dim3 grid((unsigned)blocks, (unsigned)p.G);
  char name[96];
  snprintf(name, sizeof(name), "conv_fused_f32<%d, %d, %d, %s>", BM, WM, WN, ring ? "true" : "false");
  const double x_bytes = 4.0 * ((double)p.Ncols / (p.gHout * p.gWout)) * p.gC * p.gH * p.gW;
  ProfScope ps(name, 2.0 * p.M * p.Ncols * p.Kdim * p.G,
               x_bytes + 4.0 * ((double)p.M * p.Ncols + (double)p.M * p.Kdim) * p.G, st);
  constexpr int kLdsCap = 80 * 1024;  // what launch_conv_fused admits
  if (ring) {
    constexpr auto kern = conv_fused_f32<BM, WM, WN, true>;
    if (const int rc = ensure_dynamic_lds<kern>(kLdsCap)) return rc;
    hipLaunchKernelGGL(kern, grid, dim3(NT), lds, st, p, fg, tiles_m, tiles_n);
  } else {
    constexpr auto kern = conv_fused_f32<BM, WM, WN, false>;
    if (const int rc = ensure_dynamic_lds<kern>(kLdsCap)) return rc;
    hipLaunchKernelGGL(kern, grid, dim3(NT), lds, st, p, fg, tiles_m, tiles_n);
  }
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

}  // namespace

// Returns CCT_EUNSUPPORTED (nothing launched) when the shape does not fit this kernel's LDS
// staging; the caller then uses the gather-fed GEMM.
int launch_conv_fused(const GemmTN& p0, hipStream_t st) {
  GemmTN p = p0;
  colmap_prepare(&p.bmap);
  colmap_prepare(&p.cmap);
  if (!p.gather || p.bf16 || p.gK < 2) return CCT_EUNSUPPORTED;
  int BM, BNt, BKt;
  gemm_tn_tile(p.M, p.Ncols, &BM, &BNt, &BKt);
  if (BNt != BN || BKt != BK || p.Mpad % BM || p.Kpad % BK) return CCT_EUNSUPPORTED;
  FusedGeom fg;
  fg.KK = p.gK * p.gK;
  fg.Wp = p.gW + 2 * p.gp;
  const long long P = (long long)p.gHout * p.gWout;
  // rows of padded input that 128 consecutive positions can touch: they cover at most A output
  // rows spread over at most T images; t images need (A - t)*stride + t*K rows, largest at t = 1
  // or t = T
  const long long A = (BN - 1) / p.gWout + 2, T = (BN - 1) / P + 2;
  const long long r1 = (A - 1) * p.gs + p.gK;
  const long long rT = (A > T ? A - T : 0) * p.gs + T * p.gK;
  const long long R = ((r1 > rT ? r1 : rT) * fg.Wp + 3) / 4 * 4;
  if (R > (1 << 20)) return CCT_EUNSUPPORTED;
  fg.R = (int)R;
  bool ring;
  if (p.gCg <= CGRP) {
    ring = false;
    fg.ngroups = 1;
    fg.cg = p.gCg;
    fg.tab_tiles = p.Kpad / BK;
  } else {
    ring = true;
    fg.R = (int)((R + 63) / 64 * 64);  // whole waves own the cells of a region
    // staged cells are addressed with 32-bit byte offsets from the workgroup's first image
    if ((T + 1) * p.gC * p.gH * p.gW >= (1LL << 29)) return CCT_EUNSUPPORTED;
    if (fg.R > QU * NT || fg.KK < 4) return CCT_EUNSUPPORTED;
    fg.ngroups = (p.gCg + CGRP - 1) / CGRP;
    fg.cg = CGRP;
    fg.tab_tiles = fg.KK;
    if ((long long)fg.ngroups * fg.KK < p.Kpad / BK) return CCT_EUNSUPPORTED;
  }
  const long long lds =
      4LL * (2 * BK * BM + (long long)(ring ? 2 : 1) * fg.cg * fg.R + (long long)fg.tab_tiles * BK);
  if (lds > 80 * 1024) return CCT_EUNSUPPORTED;  // keep two workgroups per CU (160 KiB of LDS)
  if (BM == 64) return launch_variant<64, 1, 2>(p, fg, ring, (size_t)lds, st);
  if (BM == 96) return launch_variant<96, 3, 1>(p, fg, ring, (size_t)lds, st);
  return launch_variant<128, 2, 2>(p, fg, ring, (size_t)lds, st);
}

}  // namespace cct
