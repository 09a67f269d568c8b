// Fully connected layers through the convolution entry points.
//
// A layer whose kernel covers its whole unpadded input (K = H = W, one output pixel per image)
// is the m = 1 case of the lowering of Sec. 2.1: the lowered matrix D^ is the batch itself viewed
// as [N][F], F = C*K*K, the kernel matrix K^ is w viewed as [O][F] and lifting is a reshape, so
// the three passes are the plain matrix products
//     y = D^ K^T + b          (contract over F: both operands are F-contiguous in place)
//     dD^ = dy K^             (contract over O: w is read in place, dy^T is packed: N*O values)
//     dK^ = dy^T D^           (contract over N: x is read in place, dy is packed)
// with no lowered copy, no kernel-matrix pack and no chunking.  The forward product has only
// N*O outputs (few tiles) and a long contraction, so it is split over F into partial products
// that a second kernel sums in split order together with the bias (bit-reproducible, no atomics).
// The backward-data product has N*F outputs, still too few tiles at CaffeNet's batch, and is split
// over O the same way when O has a suitable divisor (the splits run as the groups of one launch).
#include <algorithm>
#include <cstring>

#include "cct_internal.h"
#include "index_common.h"

namespace cct {
namespace {

constexpr long long kAlign = 256;
constexpr int kIntMax = 2147483647;
constexpr int kDbiasBlocks = 64;
// workgroups the split forward product aims for, and the shortest split worth a workgroup
constexpr int kFcTargetBlocks = 1024;
constexpr int kFcMinSplit = 256;
constexpr long long kFcMaxPartBytes = 256LL << 20;
// backward-data: workgroups that fill the chip, and the fewest kernels a split may hold
constexpr int kFcFillBlocks = 1024;
constexpr int kFcMinSplitRows = 128;

inline long long align_up(long long v, long long a) { return (v + a - 1) / a * a; }

// pack[r][m] (Kpad x Mpad, zero padded) = transposed ? src[m][k] : src[k][m], src compact, where
// row r = g*Kpad_s + kk stands for k = g*Ks + kk (kk < Ks; the other rows of a split are zero):
// the K indices are cut into splits of Ks, each padded to Kpad_s rows.  32 x 32 tiles through LDS
// so that reads and writes are both row-contiguous.
__global__ __launch_bounds__(TPB) void fc_pack_kernel(const float* __restrict__ src,
                                                      float* __restrict__ pack, int K, int M,
                                                      int Kpad, int Mpad, int transposed, int Ks,
                                                      int Kpad_s) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int r0 = blockIdx.y * 32, m0 = blockIdx.x * 32;
  if (transposed) {
    const int r = r0 + tx, g = r / Kpad_s, kk = r - g * Kpad_s, k = g * Ks + kk;
    const bool kok = r < Kpad && kk < Ks && k < K;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty + j * 8;
      tile[ty + j * 8][tx] = (m < M && kok) ? src[(long long)m * K + k] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int rr = r0 + ty + j * 8, m = m0 + tx;
      if (rr < Kpad && m < Mpad) pack[(long long)rr * Mpad + m] = tile[tx][ty + j * 8];
    }
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int r = r0 + ty + j * 8, m = m0 + tx;
      const int g = r / Kpad_s, kk = r - g * Kpad_s, k = g * Ks + kk;
      if (r < Kpad && m < Mpad)
        pack[(long long)r * Mpad + m] = (kk < Ks && k < K && m < M) ? src[(long long)k * M + m] : 0.0f;
    }
  }
}

// y[n][o] = sum_s part[s][n][o] + bias[o], splits added in order.
__global__ __launch_bounds__(TPB) void fc_sum_splits_kernel(const float* __restrict__ part,
                                                            float* __restrict__ y, int S,
                                                            long long total, FastDiv divO,
                                                            const float* __restrict__ bias) {
  const long long t = (long long)blockIdx.x * TPB + threadIdx.x;
  if (t >= total) return;
  const float* src = part + t;
  float acc = 0.0f;
  int s = 0;
  for (; s + 4 <= S; s += 4) {
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = src[(long long)(s + u) * total];
#pragma unroll
    for (int u = 0; u < 4; ++u) acc += v[u];
  }
  for (; s < S; ++s) acc += src[(long long)s * total];
  if (bias) {
    const int n = fdiv((int)t, divO);
    acc += bias[(int)t - n * divO.d];
  }
  y[t] = acc;
}

// Kpad = total rows of the pack = splits * Kpad_s
int launch_fc_pack(const float* src, float* pack, int K, int M, int Kpad, int Mpad, int transposed,
                   int Ks, int Kpad_s, hipStream_t st) {
  dim3 grid((unsigned)((Mpad + 31) / 32), (unsigned)((Kpad + 31) / 32));
  if (grid.y > 65535) return CCT_EUNSUPPORTED;
  ProfScope ps("fc_pack_kernel", 0.0, 4.0 * ((double)K * M + (double)Kpad * Mpad), st);
  hipLaunchKernelGGL(fc_pack_kernel, grid, dim3(TPB), 0, st, src, pack, K, M, Kpad, Mpad, transposed,
                     Ks, Kpad_s);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int launch_fc_sum_splits(const float* part, float* out, int S, long long total, int O,
                         const float* bias, hipStream_t st) {
  const long long blocks = (total + TPB - 1) / TPB;
  if (!grid_ok(blocks) || (bias && total >= kIntMax)) return CCT_EUNSUPPORTED;
  ProfScope ps("fc_sum_splits_kernel", 0.0, 4.0 * total * (S + 1), st);
  hipLaunchKernelGGL(fc_sum_splits_kernel, dim3((unsigned)blocks), dim3(TPB), 0, st, part, out, S,
                     total, make_fastdiv(O), bias);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

}  // namespace

bool fc_plan(const cct_conv_desc_t& d, int pass, long long max_bytes, FcPlan* P) {
  if (d.K != d.H || d.K != d.W || d.pad != 0 || d.groups != 1) return false;
  if (d.precision != CCT_PREC_F32) return false;
  if (d.lowering != CCT_LOWER_AUTO && d.lowering != CCT_LOWER_TYPE1) return false;
  const long long F = (long long)d.C * d.K * d.K;
  if (F >= kIntMax - 256 || (long long)d.N * d.O >= kIntMax || (long long)d.N * F >= (1LL << 40) ||
      (long long)d.O * F >= (1LL << 40))
    return false;
  std::memset(P, 0, sizeof(*P));
  P->F = (int)F;
  long long off = 0;
  auto take = [&](long long bytes, long long* o) {
    *o = off;
    off += align_up(bytes, kAlign);
  };
  int BM, BN, BK;
  if (pass == CCT_PASS_FORWARD) {
    // the split product reads whole K tiles of both operands without column guards
    gemm_nt_tile(d.N, d.O, &BM, &BN, &BK);
    if (F % BK) return false;
    const long long tiles = (long long)((d.N + BM - 1) / BM) * ((d.O + BN - 1) / BN);
    long long S = std::max<long long>(1, std::min<long long>((kFcTargetBlocks + tiles - 1) / tiles,
                                                             F / kFcMinSplit));
    // fewer, longer splits when the partial products would not fit
    const long long cap = max_bytes < 0 ? kFcMaxPartBytes : std::min(kFcMaxPartBytes, max_bytes);
    long long smax = cap / (4LL * d.N * d.O);
    while (smax > 1 && align_up(4LL * smax * d.N * d.O, kAlign) > cap) --smax;
    S = std::min(S, std::max<long long>(1, smax));
    P->split_len = (int)align_up((F + S - 1) / S, BK);
    P->S = (int)((F + P->split_len - 1) / P->split_len);
    take(4LL * P->S * d.N * d.O, &P->part_off);
  } else if (pass == CCT_PASS_BACKWARD_DATA) {
    // rows = images.  Too few tiles to fill the chip: 64-row tiles, and the contraction split into
    // S equal parts (the smallest divisor S of O that gives kFcFillBlocks workgroups, else the
    // largest one with parts of at least kFcMinSplitRows kernels) whose partial products are summed
    // afterwards.  Measured on fc6 at batch 256 (19.3 GFLOP): unsplit 0.33 ms, 4 splits of 128-row
    // tiles 0.24 ms, 4 splits of 64-row tiles 0.22 ms.
    gemm_tn_tile(d.N, (int)F, &BM, &BN, &BK);
    if (BM == 128 && d.N % 64 == 0 && (long long)((d.N + 127) / 128) * ((F + BN - 1) / BN) < 512) BM = 64;
    const long long tiles = (long long)((d.N + BM - 1) / BM) * ((F + BN - 1) / BN);
    const long long cap = max_bytes < 0 ? kFcMaxPartBytes : std::min(kFcMaxPartBytes, max_bytes);
    // workspace of a plan with sp splits: the packed dy and, when split, the partial products
    auto need = [&](long long sp) {
      const long long pack = 4LL * sp * align_up(d.O / sp, BK) * align_up(d.N, BM);
      return align_up(pack, kAlign) + (sp > 1 ? align_up(4LL * sp * d.N * F, kAlign) : 0);
    };
    int S = 1;
    for (int sp = 2; sp <= 64 && tiles * S < kFcFillBlocks; ++sp)
      if (d.O % sp == 0 && d.O / sp >= kFcMinSplitRows && need(sp) <= cap) S = sp;
    P->BM = BM;
    P->S = S;
    P->split_len = d.O / S;
    P->Mpad = (int)align_up(d.N, BM);
    P->Kpad = (int)align_up(P->split_len, BK);   // rows of one split
    take(4LL * S * P->Kpad * P->Mpad, &P->pack_off);
    if (S > 1) take(4LL * S * d.N * F, &P->part_off);
  } else {
    gemm_tn_tile(d.O, (int)F, &BM, &BN, &BK);
    P->BM = BM;
    P->Mpad = (int)align_up(d.O, BM);
    P->Kpad = (int)align_up(d.N, BK);
    P->S = 1;
    take(4LL * P->Kpad * P->Mpad, &P->pack_off);
    take(4LL * d.O * kDbiasBlocks, &P->scratch_off);
  }
  P->total = std::max<long long>(off, kAlign);
  return max_bytes < 0 || P->total <= max_bytes;
}

int fc_forward(const cct_conv_desc_t& d, const FcPlan& P, const float* x, const float* w,
               const float* bias, float* y, char* ws, hipStream_t st) {
  if (reinterpret_cast<uintptr_t>(w) % 16) return CCT_EINVAL;
  GemmNT q;
  std::memset(&q, 0, sizeof(q));
  q.A = x; q.a_ms = P.F;
  q.amap = ColMap{kIntMax, 0};
  q.B = w; q.b_ns = P.F;
  q.Cpart = reinterpret_cast<float*>(ws + P.part_off);
  q.M = d.N; q.N = d.O; q.Ncols = P.F;
  q.G = 1; q.S = P.S; q.split_len = P.split_len;
  int rc = launch_gemm_nt(q, st);
  if (rc) return rc;
  return launch_fc_sum_splits(q.Cpart, y, P.S, (long long)d.N * d.O, d.O, bias, st);
}

int fc_backward_data(const cct_conv_desc_t& d, const FcPlan& P, const float* w, const float* dy,
                     float* dx, char* ws, hipStream_t st) {
  float* pack = reinterpret_cast<float*>(ws + P.pack_off);
  // pack[s][oo][n] = dy[n][s*split_len + oo]
  int rc = launch_fc_pack(dy, pack, d.O, d.N, P.S * P.Kpad, P.Mpad, 1, P.split_len, P.Kpad, st);
  if (rc) return rc;
  float* part = reinterpret_cast<float*>(ws + P.part_off);
  GemmTN p;
  std::memset(&p, 0, sizeof(p));
  p.A = pack;
  p.a_gs = (long long)P.Kpad * P.Mpad;
  p.Mpad = P.Mpad; p.Kpad = P.Kpad;
  p.B = w; p.b_ks = P.F;
  p.b_gs = (long long)P.split_len * P.F;     // a split = the next split_len kernels
  p.bmap = ColMap{kIntMax, 0};
  p.b_ld_guard = P.F % 128 == 0 ? P.F : 0;   // whole column tiles can be read as vectors
  p.C = P.S > 1 ? part : dx;
  p.c_ms = P.F;
  p.c_gs = (long long)d.N * P.F;
  p.cmap = ColMap{kIntMax, 0};
  p.M = d.N; p.Ncols = P.F; p.Kdim = P.split_len; p.G = P.S;
  p.force_bm = P.BM;
  rc = launch_gemm_tn(p, st);
  if (rc || P.S == 1) return rc;
  return launch_fc_sum_splits(part, dx, P.S, (long long)d.N * P.F, 1, nullptr, st);
}

int fc_backward_weights(const cct_conv_desc_t& d, const FcPlan& P, const float* x, const float* dy,
                        float* dw, float* dbias, char* ws, hipStream_t st) {
  float* pack = reinterpret_cast<float*>(ws + P.pack_off);
  int rc = launch_fc_pack(dy, pack, d.N, d.O, P.Kpad, P.Mpad, 0, d.N, P.Kpad, st);  // pack[n][o] = dy[n][o]
  if (rc) return rc;
  GemmTN p;
  std::memset(&p, 0, sizeof(p));
  p.A = pack;
  p.Mpad = P.Mpad; p.Kpad = P.Kpad;
  p.B = x; p.b_ks = P.F;
  p.bmap = ColMap{kIntMax, 0};
  p.b_ld_guard = P.F % 128 == 0 ? P.F : 0;
  p.C = dw; p.c_ms = P.F;
  p.cmap = ColMap{kIntMax, 0};
  p.M = d.O; p.Ncols = P.F; p.Kdim = d.N; p.G = 1;
  p.force_bm = P.BM;
  rc = launch_gemm_tn(p, st);
  if (rc) return rc;
  if (dbias) {
    const int nblk = std::max(1, std::min({d.N, kDbiasBlocks, (2048 + d.O - 1) / d.O}));
    rc = launch_dbias(dy, dbias, reinterpret_cast<float*>(ws + P.scratch_off), d.N, d.O, 1, nblk, st);
  }
  return rc;
}

}  // namespace cct
