// Host side of libcct.so: argument validation, the per-call plan (lowering geometry,
// workspace layout, batch chunking), the automatic lowering optimizer and the C ABI entry
// points.  No device memory is allocated here and nothing synchronises.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "cct_internal.h"

namespace cct {
int last_hip_error_value();

namespace {

constexpr long long kAlign = 256;
// Rows of the lowered matrices are padded to a multiple of this many columns (zero filled), so
// that the GEMM can read whole 128- or 256-column tiles without guards.
constexpr long long kLdAlign = 256;
constexpr int kIntMax = 2147483647;
// Default chunk budget for the lowered buffers of one chunk (the caller can pass a larger or
// smaller workspace to change it).
constexpr long long kDefaultChunkBytes = 2LL << 30;
// A layout whose buffers for ONE image exceed this is treated as infeasible.
constexpr long long kMaxOneImageBytes = 16LL << 30;

inline long long align_up(long long v, long long a) { return (v + a - 1) / a * a; }

bool desc_ok(const cct_conv_desc_t* d) {
  if (!d) return false;
  if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->O <= 0 || d->K <= 0) return false;
  if (d->stride < 1 || d->pad < 0 || d->groups < 1) return false;
  if (d->C % d->groups || d->O % d->groups) return false;
  if ((long long)d->H + 2LL * d->pad < d->K || (long long)d->W + 2LL * d->pad < d->K) return false;
  if (d->lowering < CCT_LOWER_AUTO || d->lowering > CCT_LOWER_FUSED) return false;
  if (d->precision != CCT_PREC_F32 && d->precision != CCT_PREC_BF16_IN_F32_ACC) return false;
  return true;
}

// Geometry of one lowering layout for one descriptor.
struct Geom {
  int Hout, Wout, Cg, Og;
  WinMap lower;  // x  <-> D^   (tensor plane H x W)
  WinMap lift;   // R^ <-> y    (tensor plane Hout x Wout)
  int RKi, RKj, DKi, DKj;
  long long Pc;  // matrix columns (positions) per image
  int Mr;        // rows of R^T per group  = Og*RKi*RKj
  int Kd;        // rows of D^T per group  = Cg*DKi*DKj
};

Geom make_geom(const cct_conv_desc_t& d, int type) {
  Geom g;
  g.Hout = (d.H + 2 * d.pad - d.K) / d.stride + 1;
  g.Wout = (d.W + 2 * d.pad - d.K) / d.stride + 1;
  g.Cg = d.C / d.groups;
  g.Og = d.O / d.groups;
  const int K = d.K, s = d.stride, p = d.pad;
  if (type == CCT_LOWER_TYPE1 || type == CCT_LOWER_FUSED) {
    g.lower = WinMap{K, K, s, p, s, p, g.Hout, g.Wout, d.H, d.W};
    g.lift = WinMap{1, 1, 1, 0, 1, 0, g.Hout, g.Wout, g.Hout, g.Wout};
    g.RKi = 1; g.RKj = 1; g.DKi = K; g.DKj = K;
  } else if (type == CCT_LOWER_TYPE2) {
    g.lower = WinMap{1, K, 1, 0, s, p, d.H, g.Wout, d.H, d.W};
    g.lift = WinMap{K, 1, s, p, 1, 0, d.H, g.Wout, g.Hout, g.Wout};
    g.RKi = K; g.RKj = 1; g.DKi = 1; g.DKj = K;
  } else {
    g.lower = WinMap{1, 1, 1, 0, 1, 0, d.H, d.W, d.H, d.W};
    g.lift = WinMap{K, K, s, p, s, p, d.H, d.W, g.Hout, g.Wout};
    g.RKi = K; g.RKj = K; g.DKi = 1; g.DKj = 1;
  }
  g.Pc = (long long)g.lower.Ha * g.lower.Wb;
  g.Mr = g.Og * g.RKi * g.RKj;
  g.Kd = g.Cg * g.DKi * g.DKj;
  return g;
}

// Backward-data of a strided layer as ONE stride-1 convolution of dy (Sec. 2.1 "Fusion" applied to
// the adjoint): with h + p = s*a + rh, a pixel (h, w) only receives taps i = rh + s*u, so each of
// the s*s residue classes (rh, rw) is a convolution of dy with a sub-kernel of U x U taps,
// U = ceil(K/s), on the grid (a, b) of Ah x Aw cells; the s*s*Cg results of a cell are the pixels of
// its s x s block (depth-to-space).  Taps whose index reaches K are zero: the kernel does
// (U*s/K)^2 times the useful work.
struct StridedBwd {
  int U, Ah, Aw, M;
};
inline StridedBwd strided_bwd(const cct_conv_desc_t& d, const Geom& g) {
  StridedBwd sb;
  sb.U = (d.K + d.stride - 1) / d.stride;
  sb.Ah = (d.H - 1 + d.pad) / d.stride + 1;
  sb.Aw = (d.W - 1 + d.pad) / d.stride + 1;
  sb.M = g.Cg * d.stride * d.stride;
  return sb;
}
// The operand description of one chunk of `ni` images (pack at `pack`, or null for a fit check).
GemmTN strided_bwd_problem(const cct_conv_desc_t& d, const Geom& g, const void* pack, int Mpad,
                           int Kpad_kc, const float* dyc, float* dxc, long long ni) {
  const StridedBwd sb = strided_bwd(d, g);
  GemmTN p;
  std::memset(&p, 0, sizeof(p));
  p.A = pack;
  p.Mpad = Mpad;
  p.Kpad = Kpad_kc;
  p.a_gs = (long long)Mpad * Kpad_kc;
  p.B = dyc;
  p.bmap = ColMap{1, 0};
  p.gather = 1;
  p.gC = d.O; p.gH = g.Hout; p.gW = g.Wout; p.gHout = sb.Ah; p.gWout = sb.Aw;
  p.gs = 1; p.gp = sb.U - 1; p.gCg = g.Og; p.gK = sb.U; p.gKK = sb.U * sb.U;
  p.M = sb.M; p.Ncols = (int)(ni * sb.Ah * sb.Aw); p.Kdim = g.Og * sb.U * sb.U; p.G = d.groups;
  p.C = dxc;
  p.cmap = ColMap{1, 0};
  p.d2s = 1; p.dS = d.stride; p.dP = d.pad; p.dH = d.H; p.dW = d.W; p.dCg = g.Cg; p.dCtot = d.C;
  p.bf16 = d.precision == CCT_PREC_BF16_IN_F32_ACC;
  p.prof_flops = 2.0 * (double)ni * d.O * g.Hout * g.Wout * g.Cg * d.K * d.K;
  return p;
}

// Fused forward pass over `ni` images: Type-1 arithmetic, the B operand gathered from x.
GemmTN fused_fwd_problem(const cct_conv_desc_t& d, const Geom& g, const void* pack, int Mpad, int Kpad,
                         const float* xc, float* yc, const float* bias, long long ni) {
  const long long P = (long long)g.Hout * g.Wout;
  GemmTN p;
  std::memset(&p, 0, sizeof(p));
  p.A = pack;
  p.Mpad = Mpad;
  p.Kpad = Kpad;
  p.a_gs = (long long)Mpad * Kpad;
  p.B = xc;
  p.bmap = ColMap{1, 0};  // not a plain matrix
  p.gather = 1;
  p.gC = d.C; p.gH = d.H; p.gW = d.W; p.gHout = g.Hout; p.gWout = g.Wout;
  p.gs = d.stride; p.gp = d.pad; p.gCg = g.Cg; p.gK = d.K; p.gKK = d.K * d.K;
  make_fastdiv_parts(p.gKK, &p.g_divKK_M, &p.g_divKK_sh);
  make_fastdiv_parts(p.gK, &p.g_divK_M, &p.g_divK_sh);
  p.M = g.Mr; p.Ncols = (int)(ni * g.Pc); p.Kdim = g.Kd; p.G = d.groups;
  p.C = yc;
  p.c_ms = P; p.c_gs = (long long)g.Og * P;
  p.cmap = ColMap{(int)P, (long long)d.O * P};
  p.bias = bias; p.bias_gs = g.Og;
  p.bf16 = d.precision == CCT_PREC_BF16_IN_F32_ACC;
  return p;
}

// Fused backward-data pass of a stride-1 layer over `ni` images: dx = convolution of dy (O channels,
// Hout x Wout) with the flipped kernels, stride 1, pad K-1-p.
GemmTN fused_bwd_problem(const cct_conv_desc_t& d, const Geom& g, const void* pack, int Mpad, int Kpad,
                         const float* dyc, float* dxc, long long ni) {
  const long long HW = (long long)d.H * d.W;
  GemmTN p;
  std::memset(&p, 0, sizeof(p));
  p.A = pack;
  p.Mpad = Mpad;
  p.Kpad = Kpad;
  p.a_gs = (long long)Mpad * Kpad;
  p.B = dyc;
  p.bmap = ColMap{1, 0};
  p.gather = 1;
  p.gC = d.O; p.gH = g.Hout; p.gW = g.Wout; p.gHout = d.H; p.gWout = d.W;
  p.gs = 1; p.gp = d.K - 1 - d.pad; p.gCg = g.Og; p.gK = d.K; p.gKK = d.K * d.K;
  make_fastdiv_parts(p.gKK, &p.g_divKK_M, &p.g_divKK_sh);
  make_fastdiv_parts(p.gK, &p.g_divK_M, &p.g_divK_sh);
  // the layout accepted this chunk size only if ni*H*W fits 31 bits
  p.M = g.Cg; p.Ncols = (int)(ni * HW); p.Kdim = g.Og * d.K * d.K; p.G = d.groups;
  p.C = dxc;
  p.c_ms = HW; p.c_gs = (long long)g.Cg * HW;
  p.cmap = ColMap{(int)HW, (long long)d.C * HW};
  p.bf16 = d.precision == CCT_PREC_BF16_IN_F32_ACC;
  return p;
}

inline int esize(const cct_conv_desc_t& d) { return d.precision == CCT_PREC_BF16_IN_F32_ACC ? 2 : 4; }

// Workspace layout of one pass for a given chunk size.
struct Layout {
  long long pack_off = 0, pack_bytes = 0;
  long long dt_off = 0, dt_bytes = 0;    // D^T (or dD^T)
  long long rt_off = 0, rt_bytes = 0;    // R^T (or dR^T)
  long long part_off = 0, part_bytes = 0;
  long long scratch_off = 0, scratch_bytes = 0;
  long long total = 0;
  long long ld = 0;
  int Mpad = 0, Kpad = 0;  // pack padding (TN GEMM)
  int Kpad_kc = 0;         // fused passes: K padding of the channel-contiguous pack
  int S = 1, split_len = 0;  // NT GEMM
  int t2_opad = 0;  // Type-2 backward-data with the inverse lifting gathered by the GEMM: padded Og
};

constexpr int kDbiasBlocks = 64;

bool make_layout(const cct_conv_desc_t& d, int pass, int type, const Geom& g, long long nc,
                 Layout* L) {
  const long long ncols = nc * g.Pc;
  if (ncols <= 0 || ncols >= kIntMax - 256) return false;
  if ((long long)d.C * g.DKi * g.DKj >= kIntMax || (long long)d.O * g.RKi * g.RKj >= kIntMax)
    return false;
  const int es = esize(d);
  L->ld = align_up(ncols, kLdAlign);
  long long off = 0;
  auto take = [&](long long bytes, long long* o, long long* b) {
    *o = off;
    *b = bytes;
    off += align_up(bytes, kAlign);
  };
  const long long dt_rows = (long long)d.C * g.DKi * g.DKj;
  const long long rt_rows = (long long)d.O * g.RKi * g.RKj;
  if (pass == CCT_PASS_FORWARD) {
    int BM, BN, BK;
    gemm_tn_tile(g.Mr, (int)ncols, &BM, &BN, &BK);
    L->Mpad = (int)align_up(g.Mr, BM);
    L->Kpad = (int)align_up(g.Kd, BK);
    long long kp = L->Kpad;
    if (type == CCT_LOWER_FUSED) {
      const long long kc = conv_fused_kc_kpad(g.Cg, d.K, es == 2);
      if (kc >= kIntMax) return false;
      L->Kpad_kc = (int)kc;
      kp = std::max(kp, kc);
      if (es == 2) L->Mpad = conv_fused_kc_bf16_mpad(g.Mr);  // the bf16 form has its own row tiles
    }
    take((long long)d.groups * L->Mpad * kp * es, &L->pack_off, &L->pack_bytes);
    if (type != CCT_LOWER_FUSED) {  // the fused layout has no D^T
      take(dt_rows * L->ld * es, &L->dt_off, &L->dt_bytes);
      if (type != CCT_LOWER_TYPE1) take(rt_rows * L->ld * 4, &L->rt_off, &L->rt_bytes);
    }
  } else if (pass == CCT_PASS_BACKWARD_DATA && type == CCT_LOWER_FUSED && d.stride > 1) {
    // a stride-1 convolution of dy with s*s sub-kernels of U x U taps: M = Cg*s*s, K dim = Og*U*U
    const StridedBwd sb = strided_bwd(d, g);
    if (nc * sb.Ah * sb.Aw >= kIntMax - 256 || (long long)g.Cg * d.stride * d.stride >= kIntMax)
      return false;
    int BM, BN, BK;
    gemm_tn_tile(sb.M, (int)(nc * sb.Ah * sb.Aw), &BM, &BN, &BK);
    L->Mpad = es == 2 ? conv_fused_kc_bf16_mpad(sb.M) : (int)align_up(sb.M, BM);
    const long long kc = conv_fused_kc_kpad(g.Og, sb.U, es == 2);
    if (kc >= kIntMax) return false;
    L->Kpad = L->Kpad_kc = (int)kc;
    take((long long)d.groups * L->Mpad * kc * 4, &L->pack_off, &L->pack_bytes);
  } else if (pass == CCT_PASS_BACKWARD_DATA && type == CCT_LOWER_FUSED) {
    // a stride-1 convolution of dy with the flipped kernels: M = Cg, K dim = Og*K*K
    if (nc * d.H * d.W >= kIntMax - 256) return false;
    int BM, BN, BK;
    gemm_tn_tile(g.Cg, (int)(nc * d.H * d.W), &BM, &BN, &BK);
    L->Mpad = es == 2 ? conv_fused_kc_bf16_mpad(g.Cg) : (int)align_up(g.Cg, BM);
    L->Kpad = (int)align_up((long long)g.Og * d.K * d.K, BK);
    const long long kc = conv_fused_kc_kpad(g.Og, d.K, es == 2);
    if (kc >= kIntMax) return false;
    L->Kpad_kc = (int)kc;
    take((long long)d.groups * L->Mpad * std::max<long long>(L->Kpad, kc) * 4, &L->pack_off,
         &L->pack_bytes);
  } else if (pass == CCT_PASS_BACKWARD_DATA) {
    int BM, BN, BK;
    gemm_tn_tile(g.Kd, (int)ncols, &BM, &BN, &BK);
    L->Mpad = (int)align_up(g.Kd, BM);
    L->Kpad = (int)align_up(g.Mr, BK);
    // Type 2 at stride 1 in fp32: dR^T is never built, the GEMM gathers it from dy (K vertical
    // taps per kernel) when dy can be addressed with 32-bit byte offsets
    if (type == CCT_LOWER_TYPE2 && es == 4 && d.stride == 1 && d.K > 1 && d.K <= 64 &&
        nc * d.O * g.Hout * g.Wout < (1LL << 29)) {
      L->t2_opad = (int)align_up(g.Og, BK);
      L->Kpad = d.K * L->t2_opad;
    }
    take((long long)d.groups * L->Mpad * L->Kpad * es, &L->pack_off, &L->pack_bytes);
    if ((type != CCT_LOWER_TYPE1 || es == 2) && !L->t2_opad)
      take(rt_rows * L->ld * es, &L->rt_off, &L->rt_bytes);
    if (type != CCT_LOWER_TYPE3) take(dt_rows * L->ld * 4, &L->dt_off, &L->dt_bytes);
  } else {
    int BM, BN, BK;
    gemm_nt_tile(g.Mr, g.Kd, &BM, &BN, &BK);
    if (type != CCT_LOWER_FUSED) {  // the fused layout has neither D^T nor dR^T
      take(dt_rows * L->ld * es, &L->dt_off, &L->dt_bytes);
      if (type != CCT_LOWER_TYPE1 || es == 2) take(rt_rows * L->ld * es, &L->rt_off, &L->rt_bytes);
    }
    // split the reduction so that about 1024 workgroups exist, partials capped at 256 MiB
    const long long tiles = (long long)((g.Mr + BM - 1) / BM) * ((g.Kd + BN - 1) / BN) * d.groups;
    long long S = std::max(1LL, 1024 / std::max(1LL, tiles));
    const long long out_bytes = (long long)d.groups * g.Mr * g.Kd * 4;
    S = std::min(S, std::max(1LL, (256LL << 20) / std::max(1LL, out_bytes)));
    S = std::min(S, (ncols + 4 * BK - 1) / (4 * BK));  // at least 4 k-steps per split
    S = std::max(1LL, S);
    long long split_len = align_up((ncols + S - 1) / S, BK);
    S = (ncols + split_len - 1) / split_len;
    L->S = (int)S;
    L->split_len = (int)split_len;
    take(S * out_bytes, &L->part_off, &L->part_bytes);
    take((long long)d.O * kDbiasBlocks * 4, &L->scratch_off, &L->scratch_bytes);
  }
  L->total = off;
  return true;
}

bool type_supported(const cct_conv_desc_t& d, int pass, int type) {
  if (type < CCT_LOWER_TYPE1 || type > CCT_LOWER_FUSED) return false;
  if (d.groups > 65535) return false;  // groups are the second grid dimension of every GEMM launch
  if (type == CCT_LOWER_FUSED) {
    const bool bf16 = d.precision == CCT_PREC_BF16_IN_F32_ACC;
    const Geom gg = make_geom(d, CCT_LOWER_FUSED);
    // backward-weights: the input rows of 32 positions must fit in LDS; an unpadded layer can
    // also gather its lowered rows inside the split-K GEMM (fp32 operands only)
    if (pass == CCT_PASS_BACKWARD_WEIGHTS) {
      if (bf16) return false;
      if (!conv_bwdw_fused_fits(d.C, d.H, d.W, d.K, d.stride, d.pad, gg.Hout, gg.Wout, gg.Cg, gg.Og,
                                d.O) &&
          !(d.pad == 0 && gemm_nt_gather_fits(d.C, d.H, d.W, d.O, gg.Hout, gg.Wout)))
        return false;
    }
    // with bf16 operands only the channel-contiguous kernel exists (fp32 falls back to the other
    // fused forms when it cannot stage a shape)
    if (pass == CCT_PASS_FORWARD && bf16) {
      const long long kc = conv_fused_kc_kpad(gg.Cg, d.K, bf16);
      if (kc >= kIntMax || (long long)gg.Pc >= kIntMax ||
          !conv_fused_kc_bf16_fits(fused_fwd_problem(d, gg, nullptr, conv_fused_kc_bf16_mpad(gg.Mr),
                                                     (int)kc, nullptr, nullptr, nullptr, 1)))
        return false;
    }
    // backward-data is fused as a convolution of dy with the flipped kernels (stride 1), or with
    // the s*s sub-kernels of a strided layer when the channel-contiguous kernel can stage it
    if (pass == CCT_PASS_BACKWARD_DATA && d.stride == 1 && d.pad > d.K - 1) return false;
    if (pass == CCT_PASS_BACKWARD_DATA && d.stride == 1 && bf16) {
      const long long kc = conv_fused_kc_kpad(gg.Og, d.K, bf16);
      if (kc >= kIntMax || (long long)d.H * d.W >= kIntMax ||
          !conv_fused_kc_bf16_fits(fused_bwd_problem(d, gg, nullptr, conv_fused_kc_bf16_mpad(gg.Cg),
                                                     (int)kc, nullptr, nullptr, 1)))
        return false;
    }
    if (pass == CCT_PASS_BACKWARD_DATA && d.stride > 1) {
      const StridedBwd sb = strided_bwd(d, gg);
      if ((long long)gg.Cg * d.stride * d.stride >= kIntMax || (long long)sb.Ah * sb.Aw >= kIntMax)
        return false;
      int BM, BN, BK;
      gemm_tn_tile(sb.M, sb.Ah * sb.Aw, &BM, &BN, &BK);
      const long long kc = conv_fused_kc_kpad(gg.Og, sb.U, bf16);
      if (kc >= kIntMax) return false;
      const int mpad = bf16 ? conv_fused_kc_bf16_mpad(sb.M) : (int)align_up(sb.M, BM);
      const GemmTN p = strided_bwd_problem(d, gg, nullptr, mpad, (int)kc, nullptr, nullptr, 1);
      if (!(bf16 ? conv_fused_kc_bf16_fits(p) : conv_fused_kc_fits(p))) return false;
    }
    if ((long long)d.C * d.H * d.W >= kIntMax) return false;  // 32-bit offsets inside one image
  }
  const Geom g = make_geom(d, type);
  Layout L;
  if (!make_layout(d, pass, type, g, 1, &L)) return false;
  return L.total <= kMaxOneImageBytes;
}

// ---------------------------------------------------------------------------------------
// Cost model of the automatic optimizer (Appendix A).  All three layouts do the same useful
// flops at stride 1; they differ in the bytes the lowering and lifting phases move (the k^2
// blow-up sits on the d-channel side for Type 1 and on the o-channel side for Type 3) and,
// at stride > 1, in the extra GEMM work of Types 2/3.  Rates are MI355X measurements of
// this library's own kernels (sustained streaming rate of the index-map kernels, sustained
// fp32 MFMA rate of the GEMM at large tiles).
// ---------------------------------------------------------------------------------------
constexpr double kStreamBytesPerSec = 4.0e12;   // index-map kernels (lower, lift and adjoints)
constexpr double kGemmBytesPerSec = 5.0e12;     // operand / result streaming inside a GEMM
constexpr double kGemmFlopsPerSec = 110.0e12;
constexpr double kLaunchSec = 4.0e-6;
constexpr double kFusedGemmFactor = 0.95; // fused kernels vs the GEMM on a materialised matrix

// time = sum over index-map kernels of bytes / stream rate
//      + max(t_mfma, t_mem) + 0.3 * min(t_mfma, t_mem),  t_mfma = GEMM flops / MFMA rate,
//        t_mem = GEMM bytes / GEMM stream rate              (loads mostly overlap the MFMAs)
//      + launches * launch latency
double model_cost(const cct_conv_desc_t& d, int pass, int type) {
  const Geom g = make_geom(d, type);
  const double es = esize(d);
  const double N = d.N;
  const double cols = N * (double)g.Pc;
  const double x_bytes = 4.0 * N * d.C * d.H * d.W;
  const double y_bytes = 4.0 * N * d.O * g.Hout * g.Wout;
  const double dt_elems = (double)d.C * g.DKi * g.DKj * cols;
  const double rt_elems = (double)d.O * g.RKi * g.RKj * cols;
  double gemm_flops = 2.0 * cols * (double)g.Mr * (double)g.Kd * d.groups;
  // Row-tile efficiency of the GEMM family: the launchers cut the rows into tiles of 64 (up to
  // 64 rows), 96 (multiples of 96 that are not multiples of 128) or 128; rows beyond the true
  // count are wasted work, and the 96-row tile (waves of 96 x 32) runs its MFMAs a little below
  // the other two (measured: about 0.95).
  auto eff = [](double dim) {
    const long long m = (long long)dim;
    const double tile = m <= 64 ? 64.0 : ((m % 128 != 0 && m % 96 == 0) ? 96.0 : 128.0);
    const double speed = tile == 96.0 ? 0.95 : 1.0;
    return dim / (std::ceil(dim / tile) * tile) * speed;
  };
  // the fused kernels have a 48-row form on 16 x 16 MFMA blocks: no padding rows up to 48
  auto eff_fused = [&](double dim) { return dim <= 48.0 ? dim / 48.0 * 0.97 : eff(dim); };
  auto short_k = [](double k) { return std::min(1.0, std::max(0.25, k / 64.0)); };
  // a GEMM with fewer than ~2 workgroups (128 x 128 tiles) per CU cannot fill the chip
  auto fill = [&](double rows, double ncols) {
    const double tiles = std::ceil(rows / 128.0) * std::ceil(ncols / 128.0) * d.groups;
    return std::min(1.0, tiles / 512.0);
  };
  double index_bytes = 0.0, gemm_bytes = 0.0, launches = 2.0, rate = kGemmFlopsPerSec;
  if (pass == CCT_PASS_FORWARD && type == CCT_LOWER_FUSED) {
    // no lowered matrix at all; building the operand in the kernel costs the GEMM some of its rate
    gemm_bytes = x_bytes + y_bytes;
    rate *= kFusedGemmFactor * eff_fused(g.Mr) * fill(g.Mr, cols) * short_k(g.Kd);
  } else if (pass == CCT_PASS_FORWARD) {
    index_bytes += x_bytes + dt_elems * es;      // lowering: read x, write D^T
    gemm_bytes += dt_elems * es;                 // GEMM reads D^T
    if (type == CCT_LOWER_TYPE1) {
      gemm_bytes += y_bytes;                     // epilogue writes y
    } else {
      gemm_bytes += rt_elems * 4.0;              // GEMM writes R^T
      index_bytes += rt_elems * 4.0 + y_bytes;   // lifting reads it, writes y
      launches += 1.0;
    }
    rate *= eff(g.Mr) * fill(g.Mr, cols) * short_k(g.Kd);
  } else if (pass == CCT_PASS_BACKWARD_DATA && type == CCT_LOWER_FUSED && d.stride > 1) {
    // a convolution of dy with s*s sub-kernels of U x U taps: the zero taps are executed too
    const StridedBwd sb = strided_bwd(d, g);
    const double pos = N * sb.Ah * sb.Aw;
    gemm_bytes = x_bytes + y_bytes;
    gemm_flops = 2.0 * pos * (double)sb.M * (double)g.Og * sb.U * sb.U * d.groups;
    rate *= kFusedGemmFactor * eff_fused(sb.M) * fill(sb.M, pos);
  } else if (pass == CCT_PASS_BACKWARD_DATA && type == CCT_LOWER_FUSED) {
    // a convolution of dy with the flipped kernels: Cg output rows per group, one column per pixel
    const double pos = N * d.H * d.W;
    gemm_bytes = x_bytes + y_bytes;
    gemm_flops = 2.0 * pos * (double)g.Cg * (double)g.Og * d.K * d.K * d.groups;
    rate *= kFusedGemmFactor * eff_fused(g.Cg) * fill(g.Cg, pos);
  } else if (pass == CCT_PASS_BACKWARD_DATA) {
    if (type == CCT_LOWER_TYPE1 || (type == CCT_LOWER_TYPE2 && d.stride == 1 && es == 4.0)) {
      gemm_bytes += y_bytes;                     // GEMM reads (Type 2: gathers) dy in place
    } else {
      index_bytes += y_bytes + rt_elems * es;    // inverse lifting writes dR^T
      gemm_bytes += rt_elems * es;               // GEMM reads it
      launches += 1.0;
    }
    if (type == CCT_LOWER_TYPE3) {
      gemm_bytes += x_bytes;                     // epilogue writes dx
    } else {
      gemm_bytes += dt_elems * 4.0;              // GEMM writes dD^T
      index_bytes += dt_elems * 4.0 + x_bytes;   // inverse lowering reads it, writes dx
      launches += 1.0;
    }
    rate *= eff(g.Kd) * fill(g.Kd, cols) * short_k(g.Mr);
  } else if (type == CCT_LOWER_FUSED) {
    // split partial products straight from x and dy; the tiles of one split re-read both through L2
    gemm_bytes = x_bytes + y_bytes;
    launches += 1.0;
    rate *= kFusedGemmFactor * eff(g.Mr) * eff(g.Kd);
  } else {
    index_bytes += x_bytes + dt_elems * es;      // lowering
    gemm_bytes += dt_elems * es;
    if (type == CCT_LOWER_TYPE1) {
      gemm_bytes += y_bytes;
    } else {
      index_bytes += y_bytes + rt_elems * es;    // inverse lifting
      gemm_bytes += rt_elems * es;
    }
    launches += 2.0;
    rate *= eff(g.Mr) * eff(g.Kd);
  }
  // the GEMM's operand / result streams overlap its MFMAs, but not completely: a GEMM that is
  // heavy on both (conv1's backward-data pass writes 1.1 GB of lowered gradient) takes about the
  // longer of the two plus a third of the shorter
  const double t_mfma = gemm_flops / rate, t_mem = gemm_bytes / kGemmBytesPerSec;
  return index_bytes / kStreamBytesPerSec + std::max(t_mfma, t_mem) + 0.3 * std::min(t_mfma, t_mem) +
         launches * kLaunchSec;
}

int pick(const cct_conv_desc_t& d, int pass) {
  if (d.K == 1 && d.stride == 1 && d.pad == 0 && type_supported(d, pass, CCT_LOWER_TYPE1))
    return CCT_LOWER_TYPE1;
  // one output pixel per image (a fully connected layer): every lowering is a reshape of x, and
  // AUTO / TYPE1 run it as plain matrix products (fully_connected.hip)
  if (d.K == d.H && d.K == d.W && d.pad == 0 && d.groups == 1 && d.precision == CCT_PREC_F32 &&
      type_supported(d, pass, CCT_LOWER_TYPE1))
    return CCT_LOWER_TYPE1;
  int best = 0;
  double best_cost = 0.0;
  for (int t = CCT_LOWER_TYPE1; t <= CCT_LOWER_FUSED; ++t) {
    if (!type_supported(d, pass, t)) continue;
    const double c = model_cost(d, pass, t);
    if (!best || c < best_cost) {
      best = t;
      best_cost = c;
    }
  }
  return best;
}

// Resolve descriptor -> (type, geometry); returns a CCT_* code.
int resolve(const cct_conv_desc_t* desc, int pass, int* type, Geom* g) {
  if (!desc_ok(desc)) return CCT_EINVAL;
  if (pass < CCT_PASS_FORWARD || pass > CCT_PASS_BACKWARD_WEIGHTS) return CCT_EINVAL;
  int t = desc->lowering;
  if (t == CCT_LOWER_AUTO) {
    t = pick(*desc, pass);
    if (!t) return CCT_EUNSUPPORTED;
  } else if (!type_supported(*desc, pass, t)) {
    return CCT_EUNSUPPORTED;
  }
  *type = t;
  *g = make_geom(*desc, t);
  return CCT_OK;
}

long long default_chunk(const cct_conv_desc_t& d, int pass, int type, const Geom& g) {
  // largest nc <= N whose per-chunk buffers stay within the default budget
  long long lo = 1, hi = d.N;
  Layout L;
  auto fits = [&](long long nc) {
    return make_layout(d, pass, type, g, nc, &L) && L.total <= kDefaultChunkBytes;
  };
  if (fits(hi)) return hi;
  while (lo < hi) {
    const long long mid = (lo + hi + 1) / 2;
    if (fits(mid)) lo = mid; else hi = mid - 1;
  }
  return lo;
}

// Largest chunk whose layout fits `bytes`; 0 if not even one image fits.
long long chunk_for_workspace(const cct_conv_desc_t& d, int pass, int type, const Geom& g,
                              size_t bytes, Layout* L) {
  auto fits = [&](long long nc) {
    return make_layout(d, pass, type, g, nc, L) && (unsigned long long)L->total <= bytes;
  };
  if (!fits(1)) return 0;
  long long lo = 1, hi = d.N;
  if (fits(hi)) return hi;
  while (lo < hi) {
    const long long mid = (lo + hi + 1) / 2;
    if (fits(mid)) lo = mid; else hi = mid - 1;
  }
  fits(lo);
  return lo;
}

PackDesc make_pack(const cct_conv_desc_t& d, const Geom& g, const Layout& L, int transposed) {
  PackDesc pd;
  pd.G = d.groups; pd.Og = g.Og; pd.Cg = g.Cg; pd.K = d.K;
  pd.RKi = g.RKi; pd.RKj = g.RKj; pd.DKi = g.DKi; pd.DKj = g.DKj;
  pd.Mpad = L.Mpad; pd.Kpad = L.Kpad;
  pd.transposed = transposed;
  pd.bf16 = d.precision == CCT_PREC_BF16_IN_F32_ACC;
  return pd;
}

const ColMap kPlain = {kIntMax, 0};

// a workspace size as the byte limit of a plan
inline long long ws_cap(size_t bytes) {
  return (long long)std::min<unsigned long long>(bytes, 1ULL << 62);
}

}  // namespace
}  // namespace cct

using namespace cct;

extern "C" {

const char* cct_strerror(int code) {
  switch (code) {
    case CCT_OK: return "ok";
    case CCT_EINVAL: return "invalid argument";
    case CCT_EWORKSPACE: return "workspace too small for one image";
    case CCT_EUNSUPPORTED: return "unsupported combination or size";
    case CCT_EHIP: return "HIP launch failed";
    case CCT_ESCRATCH: return "one image needs more than the library's static scratch array";
    default: return "unknown error code";
  }
}

int cct_last_hip_error(void) { return last_hip_error_value(); }

int cct_conv_output_dims(const cct_conv_desc_t* desc, int32_t* Hout, int32_t* Wout) {
  if (!desc_ok(desc) || !Hout || !Wout) return CCT_EINVAL;
  *Hout = (desc->H + 2 * desc->pad - desc->K) / desc->stride + 1;
  *Wout = (desc->W + 2 * desc->pad - desc->K) / desc->stride + 1;
  return CCT_OK;
}

int cct_lowered_shape(const cct_conv_desc_t* desc, cct_lowering_t lowering, int64_t* rows,
                      int64_t* cols, int64_t* rcols) {
  if (!desc_ok(desc) || !rows || !cols || !rcols) return CCT_EINVAL;
  if (lowering < CCT_LOWER_TYPE1 || lowering > CCT_LOWER_TYPE3) return CCT_EINVAL;
  const Geom g = make_geom(*desc, lowering);
  *rows = (int64_t)desc->N * g.Pc;
  *cols = g.Kd;
  *rcols = g.Mr;
  return CCT_OK;
}

int cct_lowered_ld(const cct_conv_desc_t* desc, cct_lowering_t lowering, int64_t* ld) {
  if (!desc_ok(desc) || !ld) return CCT_EINVAL;
  if (lowering < CCT_LOWER_TYPE1 || lowering > CCT_LOWER_TYPE3) return CCT_EINVAL;
  const Geom g = make_geom(*desc, lowering);
  const long long ncols = (long long)desc->N * g.Pc;
  if (ncols >= kIntMax - 256) return CCT_EUNSUPPORTED;
  *ld = align_up(ncols, kLdAlign);
  return CCT_OK;
}

int cct_pick_lowering(const cct_conv_desc_t* desc, cct_pass_t pass, cct_lowering_t* picked) {
  if (!desc_ok(desc) || !picked) return CCT_EINVAL;
  if (pass < CCT_PASS_FORWARD || pass > CCT_PASS_BACKWARD_WEIGHTS) return CCT_EINVAL;
  const int t = pick(*desc, pass);
  if (!t) return CCT_EUNSUPPORTED;
  *picked = (cct_lowering_t)t;
  return CCT_OK;
}

int cct_lowering_cost(const cct_conv_desc_t* desc, cct_pass_t pass, cct_lowering_t lowering,
                      double* seconds) {
  if (!desc_ok(desc) || !seconds) return CCT_EINVAL;
  if (pass < CCT_PASS_FORWARD || pass > CCT_PASS_BACKWARD_WEIGHTS) return CCT_EINVAL;
  if (lowering < CCT_LOWER_TYPE1 || lowering > CCT_LOWER_FUSED) return CCT_EINVAL;
  if (!type_supported(*desc, pass, lowering)) return CCT_EUNSUPPORTED;
  *seconds = model_cost(*desc, pass, lowering);
  return CCT_OK;
}

int cct_conv_workspace_bytes_for_chunk(const cct_conv_desc_t* desc, cct_pass_t pass,
                                       int32_t images_per_chunk, size_t* bytes) {
  int type;
  Geom g;
  if (!bytes) return CCT_EINVAL;
  const int rc = resolve(desc, pass, &type, &g);
  if (rc) return rc;
  if (images_per_chunk < 1 || images_per_chunk > desc->N) return CCT_EINVAL;
  FcPlan fp;
  if (images_per_chunk == desc->N && fc_plan(*desc, pass, -1, &fp)) {
    *bytes = (size_t)fp.total;
    return CCT_OK;
  }
  Layout L;
  if (!make_layout(*desc, pass, type, g, images_per_chunk, &L)) return CCT_EUNSUPPORTED;
  *bytes = (size_t)L.total;
  return CCT_OK;
}

int cct_conv_workspace_bytes(const cct_conv_desc_t* desc, cct_pass_t pass, size_t* bytes) {
  int type;
  Geom g;
  if (!bytes) return CCT_EINVAL;
  const int rc = resolve(desc, pass, &type, &g);
  if (rc) return rc;
  FcPlan fp;
  if (fc_plan(*desc, pass, -1, &fp)) {   // fully connected layers are never chunked
    *bytes = (size_t)fp.total;
    return CCT_OK;
  }
  const long long nc = default_chunk(*desc, pass, type, g);
  Layout L;
  if (!make_layout(*desc, pass, type, g, nc, &L)) return CCT_EUNSUPPORTED;
  *bytes = (size_t)L.total;
  return CCT_OK;
}

int cct_lower(const cct_conv_desc_t* desc, cct_lowering_t lowering, const float* x, float* dhat,
              void* hip_stream) {
  if (!desc_ok(desc) || !x || !dhat) return CCT_EINVAL;
  if (lowering < CCT_LOWER_TYPE1 || lowering > CCT_LOWER_TYPE3) return CCT_EINVAL;
  const Geom g = make_geom(*desc, lowering);
  const long long ncols = (long long)desc->N * g.Pc;
  if (ncols >= kIntMax - 256) return CCT_EUNSUPPORTED;
  return launch_lower(x, dhat, align_up(ncols, kLdAlign), desc->N, desc->C, g.lower, 0,
                      (hipStream_t)hip_stream);
}

}  // extern "C"

// Memory of cct_conv_forward_static: one array per GPU, part of the library's code object, so it
// exists from the moment the library is loaded on a device until the process ends.  Host code
// must not use this name as an address; scratch_address() asks the runtime where the current
// device's copy lives.
static __device__ __align__(256) unsigned char scratch[CCT_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, filled on first use

// Device address of the current device's scratch array (looked up once per device).
int scratch_address(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) {
    set_hip_error(e);
    return CCT_EHIP;
  }
  if (dev < 0 || dev >= kMaxDevices) return CCT_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      set_hip_error(e);
      return CCT_EHIP;
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return CCT_OK;
}

// The forward pass.  static_scratch: the workspace is the library's scratch array, whose address
// is looked up only after every argument and size check has passed.
int forward_on_workspace(const cct_conv_desc_t* desc, const float* x, const float* w,
                         const float* bias, float* y, void* workspace, size_t workspace_bytes,
                         bool static_scratch, void* hip_stream) {
  int type;
  Geom g;
  int rc = resolve(desc, CCT_PASS_FORWARD, &type, &g);
  if (rc) return rc;
  if (!x || !w || !y || (!static_scratch && !workspace)) return CCT_EINVAL;
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return CCT_EINVAL;
  const cct_conv_desc_t& d = *desc;
  // a fully connected layer whose plan fits the workspace: plain matrix products on x and w
  FcPlan fp;
  const bool fc = fc_plan(d, CCT_PASS_FORWARD, ws_cap(workspace_bytes), &fp);
  Layout L;
  const long long nc =
      fc ? d.N : chunk_for_workspace(d, CCT_PASS_FORWARD, type, g, workspace_bytes, &L);
  if (nc < 1) return static_scratch ? CCT_ESCRATCH : CCT_EWORKSPACE;
  if (static_scratch) {
    rc = scratch_address(&workspace);
    if (rc) return rc;
  }
  if (fc)
    return fc_forward(d, fp, x, w, bias, y, static_cast<char*>(workspace), (hipStream_t)hip_stream);
  hipStream_t st = (hipStream_t)hip_stream;
  char* ws = static_cast<char*>(workspace);
  const int bf16 = d.precision == CCT_PREC_BF16_IN_F32_ACC;
  const int es = esize(d);
  const long long P = (long long)g.Hout * g.Wout;

  // the fused pass: the operand description of one chunk (lowering, multiply and lifting in one
  // kernel: the GEMM gathers its B tiles from x)
  auto fused_chunk = [&](const float* xc, float* yc, long long ni, bool kc) {
    return fused_fwd_problem(d, g, ws + L.pack_off, L.Mpad, kc ? L.Kpad_kc : L.Kpad, xc, yc, bias, ni);
  };
  // channel-contiguous form of the fused kernel when the shape allows it (it has its own pack)
  const bool kc = type == CCT_LOWER_FUSED &&
                  (bf16 ? conv_fused_kc_bf16_fits(fused_chunk(x, y, nc, true))
                        : conv_fused_kc_fits(fused_chunk(x, y, nc, true)));
  if (type == CCT_LOWER_FUSED && bf16 && !kc) return CCT_EUNSUPPORTED;
  if (kc)
    rc = launch_pack_fused_kc(w, ws + L.pack_off, d.groups, g.Og, g.Cg, d.K, L.Mpad, 0, bf16, st);
  else
    rc = launch_pack_kernel_matrix(w, ws + L.pack_off, make_pack(d, g, L, 0), st);
  if (rc) return rc;
  for (long long n0 = 0; n0 < d.N; n0 += nc) {
    const int ni = (int)std::min<long long>(nc, d.N - n0);
    const long long ncols = (long long)ni * g.Pc;
    const float* xc = x + n0 * d.C * d.H * d.W;
    float* yc = y + n0 * d.O * P;
    if (type == CCT_LOWER_FUSED) {
      const GemmTN p = fused_chunk(xc, yc, ni, kc);
      if (kc) {
        rc = bf16 ? launch_conv_fused_kc_bf16(p, st) : launch_conv_fused_kc(p, st);
      } else {
        rc = launch_conv_fused(p, st);                            // LDS-staged lowering
        if (rc == CCT_EUNSUPPORTED) rc = launch_gemm_tn(p, st);  // else gather-fed GEMM
      }
      if (rc) return rc;
      continue;
    }
    // 1x1 kernel, stride 1, no padding: all three lowerings are the identity (D^ = x, R^ = y as
    // matrices), so the GEMM reads x and writes y in place through column maps
    const bool ident = d.K == 1 && d.stride == 1 && d.pad == 0 && !bf16;
    GemmTN p;
    std::memset(&p, 0, sizeof(p));
    p.A = ws + L.pack_off;
    p.a_gs = (long long)L.Mpad * L.Kpad;
    p.Mpad = L.Mpad; p.Kpad = L.Kpad;
    if (ident) {
      const long long HW = (long long)d.H * d.W;
      p.B = xc;
      p.b_ks = HW; p.b_gs = (long long)g.Cg * HW;
      p.bmap = ColMap{(int)HW, (long long)d.C * HW};
      p.b_ld_guard = 0;
    } else {
      rc = launch_lower(xc, ws + L.dt_off, L.ld, ni, d.C, g.lower, bf16, st);
      if (rc) return rc;
      p.B = ws + L.dt_off;
      p.b_ks = L.ld; p.b_gs = (long long)g.Kd * L.ld;
      p.bmap = kPlain;
      p.b_ld_guard = (int)L.ld;
    }
    p.M = g.Mr; p.Ncols = (int)ncols; p.Kdim = g.Kd; p.G = d.groups; p.bf16 = bf16;
    if (type == CCT_LOWER_TYPE1 || ident) {
      // lifting phase of Type 1 (a reshape) + bias fused into the GEMM epilogue
      p.C = yc;
      p.c_ms = P; p.c_gs = (long long)g.Og * P;
      p.cmap = ColMap{(int)P, (long long)d.O * P};
      p.bias = bias; p.bias_gs = g.Og;
      rc = launch_gemm_tn(p, st);
      if (rc) return rc;
    } else {
      p.C = reinterpret_cast<float*>(ws + L.rt_off);
      p.c_ms = L.ld; p.c_gs = (long long)g.Mr * L.ld;
      p.cmap = kPlain;
      p.bias = nullptr; p.bias_gs = 0;
      rc = launch_gemm_tn(p, st);
      if (rc) return rc;
      rc = launch_lift(reinterpret_cast<const float*>(ws + L.rt_off), L.ld, yc, bias, ni, d.O,
                       g.lift, st);
      if (rc) return rc;
    }
  }
  (void)es;
  return CCT_OK;
}

}  // namespace

extern "C" {

int cct_conv_forward(const cct_conv_desc_t* desc, const float* x, const float* w, const float* bias,
                     float* y, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return forward_on_workspace(desc, x, w, bias, y, workspace, workspace_bytes, false, hip_stream);
}

int cct_conv_forward_static(const cct_conv_desc_t* desc, const float* x, const float* w,
                            const float* bias, float* y, void* hip_stream) {
  return forward_on_workspace(desc, x, w, bias, y, nullptr, CCT_STATIC_SCRATCH_BYTES, true,
                              hip_stream);
}

int cct_conv_backward_data(const cct_conv_desc_t* desc, const float* w, const float* dy, float* dx,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  int type;
  Geom g;
  int rc = resolve(desc, CCT_PASS_BACKWARD_DATA, &type, &g);
  if (rc) return rc;
  if (!w || !dy || !dx || !workspace) return CCT_EINVAL;
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return CCT_EINVAL;
  const cct_conv_desc_t& d = *desc;
  FcPlan fp;
  if (fc_plan(d, CCT_PASS_BACKWARD_DATA, ws_cap(workspace_bytes), &fp))
    return fc_backward_data(d, fp, w, dy, dx, static_cast<char*>(workspace), (hipStream_t)hip_stream);
  Layout L;
  const long long nc = chunk_for_workspace(d, CCT_PASS_BACKWARD_DATA, type, g, workspace_bytes, &L);
  if (nc < 1) return CCT_EWORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  char* ws = static_cast<char*>(workspace);
  const int bf16 = d.precision == CCT_PREC_BF16_IN_F32_ACC;
  const long long P = (long long)g.Hout * g.Wout;
  const long long HW = (long long)d.H * d.W;

  if (type == CCT_LOWER_FUSED && d.stride > 1) {
    // one kernel per chunk: the s*s residue classes of dx as one stride-1 convolution of dy
    void* pack = ws + L.pack_off;
    rc = launch_pack_fused_kc_strided(w, pack, d.groups, g.Og, g.Cg, d.K, d.stride, L.Mpad, bf16, st);
    if (rc) return rc;
    for (long long n0 = 0; n0 < d.N; n0 += nc) {
      const long long ni = std::min<long long>(nc, d.N - n0);
      const GemmTN p = strided_bwd_problem(d, g, pack, L.Mpad, L.Kpad_kc, dy + n0 * d.O * P,
                                           dx + n0 * d.C * HW, ni);
      rc = bf16 ? launch_conv_fused_kc_bf16(p, st) : launch_conv_fused_kc(p, st);
      if (rc) return rc;
    }
    return CCT_OK;
  }
  if (type == CCT_LOWER_FUSED) {
    // one kernel per chunk: dx = convolution of dy (O channels, Hout x Wout) with the flipped
    // kernels, stride 1, pad K-1-p; lowering of dy happens in LDS (or as a gather), never in HBM
    auto fused_chunk = [&](const float* dyc, float* dxc, long long ni, bool kc) {
      return fused_bwd_problem(d, g, ws + L.pack_off, L.Mpad, kc ? L.Kpad_kc : L.Kpad, dyc, dxc, ni);
    };
    const bool kc = bf16 ? conv_fused_kc_bf16_fits(fused_chunk(dy, dx, nc, true))
                         : conv_fused_kc_fits(fused_chunk(dy, dx, nc, true));
    if (bf16 && !kc) return CCT_EUNSUPPORTED;
    if (kc)
      rc = launch_pack_fused_kc(w, ws + L.pack_off, d.groups, g.Og, g.Cg, d.K, L.Mpad, 1, bf16, st);
    else
      rc = launch_pack_flipped(w, reinterpret_cast<float*>(ws + L.pack_off), d.groups, g.Og, g.Cg,
                               d.K, L.Mpad, L.Kpad, st);
    if (rc) return rc;
    for (long long n0 = 0; n0 < d.N; n0 += nc) {
      const long long ni = std::min<long long>(nc, d.N - n0);
      const GemmTN p = fused_chunk(dy + n0 * d.O * P, dx + n0 * d.C * HW, ni, kc);
      if (kc) {
        rc = bf16 ? launch_conv_fused_kc_bf16(p, st) : launch_conv_fused_kc(p, st);
      } else {
        rc = launch_conv_fused(p, st);
        if (rc == CCT_EUNSUPPORTED) rc = launch_gemm_tn(p, st);
      }
      if (rc) return rc;
    }
    return CCT_OK;
  }
  if (L.t2_opad)
    rc = launch_pack_type2_bwd(w, reinterpret_cast<float*>(ws + L.pack_off), d.groups, g.Og, g.Cg,
                               d.K, L.t2_opad, L.Mpad, st);
  else
    rc = launch_pack_kernel_matrix(w, ws + L.pack_off, make_pack(d, g, L, 1), st);
  if (rc) return rc;
  for (long long n0 = 0; n0 < d.N; n0 += nc) {
    const int ni = (int)std::min<long long>(nc, d.N - n0);
    const long long ncols = (long long)ni * g.Pc;
    const float* dyc = dy + n0 * d.O * P;
    float* dxc = dx + n0 * d.C * HW;
    GemmTN p;
    std::memset(&p, 0, sizeof(p));
    p.A = ws + L.pack_off;
    p.a_gs = (long long)L.Mpad * L.Kpad;
    p.Mpad = L.Mpad; p.Kpad = L.Kpad;
    p.M = g.Kd; p.Ncols = (int)ncols; p.Kdim = g.Mr; p.G = d.groups; p.bf16 = bf16;
    const bool ident = d.K == 1 && d.stride == 1 && d.pad == 0 && !bf16;
    if (L.t2_opad && !ident) {
      // Type 2, stride 1: dR^T[(o,i)][(n,a,b)] = dy[n,o,a+p-i,b] gathered by the GEMM, rows
      // ordered (K-1-i, o): a convolution-like gather with K vertical taps, pad K-1-p
      p.B = dyc;
      p.bmap = ColMap{1, 0};
      p.gather = 1; p.tapmajor = 1;
      p.gC = d.O; p.gCg = g.Og; p.gH = g.Hout; p.gW = g.Wout;
      p.gHout = d.H; p.gWout = g.Wout;   // the grid of D^ columns: every input row, output columns
      p.gs = 1; p.gK = d.K; p.gKK = d.K * d.K;
      p.tKi = d.K; p.tKj = 1; p.tph = d.K - 1 - d.pad; p.tpw = 0;
      p.gCpad = L.t2_opad;
      make_fastdiv_parts(p.gCpad, &p.g_divKK_M, &p.g_divKK_sh);
      p.Kdim = L.Kpad;
    } else if (L.rt_bytes && !ident) {
      // inverse lifting: spread dy over the rows of dR^T (a copy for Type 1 in bf16 mode)
      rc = launch_inv_lift(dyc, ws + L.rt_off, L.ld, ni, d.O, g.lift, bf16, st);
      if (rc) return rc;
      p.B = ws + L.rt_off;
      p.b_ks = L.ld; p.b_gs = (long long)g.Mr * L.ld;
      p.bmap = kPlain;
      p.b_ld_guard = (int)L.ld;
    } else {
      // Type 1: dR^T is dy itself, read in place through the NCHW column map
      p.B = dyc;
      p.b_ks = P; p.b_gs = (long long)g.Og * P;
      p.bmap = ColMap{(int)P, (long long)d.O * P};
      p.b_ld_guard = 0;
    }
    if (type == CCT_LOWER_TYPE3 || ident) {
      // inverse lowering of Type 3 (and of any 1x1 layer) is a reshape: the epilogue writes dx in place
      p.C = dxc;
      p.c_ms = HW; p.c_gs = (long long)g.Cg * HW;
      p.cmap = ColMap{(int)HW, (long long)d.C * HW};
      rc = launch_gemm_tn(p, st);
      if (rc) return rc;
    } else {
      p.C = reinterpret_cast<float*>(ws + L.dt_off);
      p.c_ms = L.ld; p.c_gs = (long long)g.Kd * L.ld;
      p.cmap = kPlain;
      rc = launch_gemm_tn(p, st);
      if (rc) return rc;
      rc = launch_inv_lower(reinterpret_cast<const float*>(ws + L.dt_off), L.ld, dxc, ni, d.C,
                            g.lower, st);
      if (rc) return rc;
    }
  }
  return CCT_OK;
}

int cct_conv_backward_weights(const cct_conv_desc_t* desc, const float* x, const float* dy, float* dw,
                              float* dbias, void* workspace, size_t workspace_bytes,
                              void* hip_stream) {
  int type;
  Geom g;
  int rc = resolve(desc, CCT_PASS_BACKWARD_WEIGHTS, &type, &g);
  if (rc) return rc;
  if (!x || !dy || !dw || !workspace) return CCT_EINVAL;
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return CCT_EINVAL;
  const cct_conv_desc_t& d = *desc;
  FcPlan fp;
  if (fc_plan(d, CCT_PASS_BACKWARD_WEIGHTS, ws_cap(workspace_bytes), &fp))
    return fc_backward_weights(d, fp, x, dy, dw, dbias, static_cast<char*>(workspace),
                               (hipStream_t)hip_stream);
  Layout L;
  const long long nc =
      chunk_for_workspace(d, CCT_PASS_BACKWARD_WEIGHTS, type, g, workspace_bytes, &L);
  if (nc < 1) return CCT_EWORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  char* ws = static_cast<char*>(workspace);
  const int bf16 = d.precision == CCT_PREC_BF16_IN_F32_ACC;
  const long long P = (long long)g.Hout * g.Wout;
  const PackDesc pd = make_pack(d, g, L, 0);

  int chunk = 0;
  for (long long n0 = 0; n0 < d.N; n0 += nc, ++chunk) {
    const int ni = (int)std::min<long long>(nc, d.N - n0);
    const long long ncols = (long long)ni * g.Pc;
    const float* xc = x + n0 * d.C * d.H * d.W;
    const float* dyc = dy + n0 * d.O * P;
    if (type == CCT_LOWER_FUSED) {
      ConvBwdW f;
      std::memset(&f, 0, sizeof(f));
      f.x = xc; f.dy = dyc;
      f.Cpart = reinterpret_cast<float*>(ws + L.part_off);
      f.C = d.C; f.H = d.H; f.W = d.W; f.O = d.O; f.Hout = g.Hout; f.Wout = g.Wout;
      f.s = d.stride; f.p = d.pad; f.Cg = g.Cg; f.Og = g.Og; f.K = d.K;
      f.nimg = ni; f.G = d.groups; f.S = L.S; f.split_len = L.split_len;
      rc = launch_conv_bwdw_fused(f, st);
      if (rc == CCT_EUNSUPPORTED && d.pad == 0) {
        // the rows do not fit in LDS: split-K GEMM that gathers the lowered rows from x
        GemmNT q;
        std::memset(&q, 0, sizeof(q));
        q.A = dyc; q.a_ms = P; q.a_gs = (long long)g.Og * P;
        q.amap = ColMap{(int)P, (long long)d.O * P};
        q.B = xc; q.b_gs = (long long)g.Cg * d.H * d.W;
        q.Cpart = f.Cpart;
        q.M = g.Mr; q.N = g.Kd; q.Ncols = (int)ncols;
        q.G = d.groups; q.S = L.S; q.split_len = L.split_len;
        q.gather = 1; q.gC = d.C; q.gH = d.H; q.gW = d.W; q.gHout = g.Hout; q.gWout = g.Wout;
        q.gs = d.stride; q.gCg = g.Cg; q.gK = d.K;
        rc = launch_gemm_nt(q, st);
      }
      if (rc) return rc;
      rc = launch_reduce_dw(f.Cpart, dw, L.S, pd, chunk > 0, st);
      if (rc) return rc;
      continue;
    }
    rc = launch_lower(xc, ws + L.dt_off, L.ld, ni, d.C, g.lower, bf16, st);
    if (rc) return rc;
    GemmNT p;
    std::memset(&p, 0, sizeof(p));
    if (L.rt_bytes) {
      rc = launch_inv_lift(dyc, ws + L.rt_off, L.ld, ni, d.O, g.lift, bf16, st);
      if (rc) return rc;
      p.A = ws + L.rt_off;
      p.a_ms = L.ld; p.a_gs = (long long)g.Mr * L.ld;
      p.amap = kPlain;
    } else {
      p.A = dyc;
      p.a_ms = P; p.a_gs = (long long)g.Og * P;
      p.amap = ColMap{(int)P, (long long)d.O * P};
    }
    p.B = ws + L.dt_off;
    p.b_ns = L.ld; p.b_gs = (long long)g.Kd * L.ld;
    p.Cpart = reinterpret_cast<float*>(ws + L.part_off);
    p.M = g.Mr; p.N = g.Kd; p.Ncols = (int)ncols;
    p.G = d.groups; p.S = L.S; p.split_len = L.split_len; p.bf16 = bf16;
    rc = launch_gemm_nt(p, st);
    if (rc) return rc;
    rc = launch_reduce_dw(p.Cpart, dw, L.S, pd, chunk > 0, st);
    if (rc) return rc;
  }
  if (dbias) {
    // about 2048 workgroups: each sums the planes of every nblk-th image of one kernel
    const int nblk = std::max(1, std::min({d.N, kDbiasBlocks, (2048 + d.O - 1) / d.O}));
    rc = launch_dbias(dy, dbias, reinterpret_cast<float*>(ws + L.scratch_off), d.N, d.O, (int)P,
                      nblk, st);
    if (rc) return rc;
  }
  return CCT_OK;
}

}  // extern "C"
