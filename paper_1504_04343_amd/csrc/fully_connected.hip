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

inline long long align_up(long long v, long long a) { return (v + a - 1) / a * a; }

// pack[k][m] (Kpad x Mpad, zero padded) = transposed ? src[m][k] : src[k][m], src compact.
// 32 x 32 tiles through LDS so that reads and writes are both row-contiguous.
__global__ __launch_bounds__(TPB) void fc_pack_kernel(const float* __restrict__ src,
                                                      float* __restrict__ pack, int K, int M,
                                                      int Kpad, int Mpad, int transposed) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int k0 = blockIdx.y * 32, m0 = blockIdx.x * 32;
  if (transposed) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty + j * 8, k = k0 + tx;
      tile[ty + j * 8][tx] = (m < M && k < K) ? src[(long long)m * K + k] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + ty + j * 8, m = m0 + tx;
      if (k < Kpad && m < Mpad) pack[(long long)k * Mpad + m] = tile[tx][ty + j * 8];
    }
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + ty + j * 8, m = m0 + tx;
      if (k < Kpad && m < Mpad)
        pack[(long long)k * Mpad + m] = (k < K && m < M) ? src[(long long)k * M + m] : 0.0f;
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

int launch_fc_pack(const float* src, float* pack, int K, int M, int Kpad, int Mpad, int transposed,
                   hipStream_t st) {
  dim3 grid((unsigned)((Mpad + 31) / 32), (unsigned)((Kpad + 31) / 32));
  if (grid.y > 65535) return CCT_EUNSUPPORTED;
  ProfScope ps("fc_pack_kernel", 0.0, 4.0 * ((double)K * M + (double)Kpad * Mpad), st);
  hipLaunchKernelGGL(fc_pack_kernel, grid, dim3(TPB), 0, st, src, pack, K, M, Kpad, Mpad, transposed);
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
    S = std::min(S, std::max<long long>(1, cap / align_up(4LL * d.N * d.O, kAlign)));
    P->split_len = (int)align_up((F + S - 1) / S, BK);
    P->S = (int)((F + P->split_len - 1) / P->split_len);
    take(4LL * P->S * d.N * d.O, &P->part_off);
  } else if (pass == CCT_PASS_BACKWARD_DATA) {
    // rows = images; 64-row tiles when that fills the chip better than 128-row ones
    gemm_tn_tile(d.N, (int)F, &BM, &BN, &BK);
    if (BM == 128 && d.N % 64 == 0 && (long long)(d.N / 128) * ((F + BN - 1) / BN) < 512) BM = 64;
    P->BM = BM;
    P->Mpad = (int)align_up(d.N, BM);
    P->Kpad = (int)align_up(d.O, BK);
    take(4LL * P->Kpad * P->Mpad, &P->pack_off);
  } else {
    gemm_tn_tile(d.O, (int)F, &BM, &BN, &BK);
    P->BM = BM;
    P->Mpad = (int)align_up(d.O, BM);
    P->Kpad = (int)align_up(d.N, BK);
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
  const long long total = (long long)d.N * d.O;
  const long long blocks = (total + TPB - 1) / TPB;
  if (!grid_ok(blocks)) return CCT_EUNSUPPORTED;
  ProfScope ps("fc_sum_splits_kernel", 0.0, 4.0 * total * (P.S + 1), st);
  hipLaunchKernelGGL(fc_sum_splits_kernel, dim3((unsigned)blocks), dim3(TPB), 0, st, q.Cpart, y, P.S,
                     total, make_fastdiv(d.O), bias);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int fc_backward_data(const cct_conv_desc_t& d, const FcPlan& P, const float* w, const float* dy,
                     float* dx, char* ws, hipStream_t st) {
  float* pack = reinterpret_cast<float*>(ws + P.pack_off);
  int rc = launch_fc_pack(dy, pack, d.O, d.N, P.Kpad, P.Mpad, 1, st);  // pack[o][n] = dy[n][o]
  if (rc) return rc;
  GemmTN p;
  std::memset(&p, 0, sizeof(p));
  p.A = pack;
  p.Mpad = P.Mpad; p.Kpad = P.Kpad;
  p.B = w; p.b_ks = P.F;
  p.bmap = ColMap{kIntMax, 0};
  p.b_ld_guard = P.F % 128 == 0 ? P.F : 0;   // whole column tiles can be read as vectors
  p.C = dx; p.c_ms = P.F;
  p.cmap = ColMap{kIntMax, 0};
  p.M = d.N; p.Ncols = P.F; p.Kdim = d.O; p.G = 1;
  p.force_bm = P.BM;
  return launch_gemm_tn(p, st);
}

int fc_backward_weights(const cct_conv_desc_t& d, const FcPlan& P, const float* x, const float* dy,
                        float* dw, float* dbias, char* ws, hipStream_t st) {
  float* pack = reinterpret_cast<float*>(ws + P.pack_off);
  int rc = launch_fc_pack(dy, pack, d.N, d.O, P.Kpad, P.Mpad, 0, st);  // pack[n][o] = dy[n][o]
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
