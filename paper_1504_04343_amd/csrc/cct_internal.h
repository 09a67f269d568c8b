// Internal declarations shared by the translation units of libcct.so.
// Nothing here is part of the C ABI (see include/cct.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <atomic>

#include "cct.h"

namespace cct {

// ---------------------------------------------------------------------------------------
// Window map.  All three lowerings (Sec. 2.1) and their liftings are the same gather with
// different parameters: a matrix column is (image n, grid row a, grid col b) over a grid
// of Ha x Wb positions per image, a matrix row is (channel, tap i < Ki, tap j < Kj), and the
// tensor pixel that belongs to them is
//        h = a*sh + i - ph,      w = b*sw + j - pw
// in a tensor of Ht x Wt pixels per (image, channel).
//   lowering of x   : Type 1 (K,K,s,p,s,p) on the Hout x Wout grid; Type 2 (1,K,1,0,s,p) on
//                     H x Wout; Type 3 (1,1,1,0,1,0) on H x W; tensor = x (H x W).
//   lifting  to y   : the same formula read the other way: the tensor is the a/b grid of R^
//                     and the "pixel" is the output position; see LiftMap.
// ---------------------------------------------------------------------------------------
struct WinMap {
  int Ki, Kj;          // taps that index matrix rows
  int sh, ph, sw, pw;  // stride / pad per axis
  int Ha, Wb;          // grid of matrix columns per image
  int Ht, Wt;          // tensor plane size
};

// n / d == (n * M) >> sh for 0 <= n < 2^31
inline void make_fastdiv_parts(int d, unsigned* M, int* sh) {
  int s = 0;
  while ((1LL << s) < d) ++s;
  *sh = 31 + s;
  *M = (unsigned)(((1ULL << *sh) + (unsigned long long)d - 1) / (unsigned long long)d);
}

// Column -> memory offset map used by the GEMM kernels so that they can read and write
// NCHW tensors in place: off(col) = (col / P) * img_stride + (col % P).
// A plain matrix row uses P = INT32_MAX, img_stride = 0.
struct ColMap {
  int P;
  long long img_stride;
  unsigned divM;  // col / P == (col * divM) >> divsh; filled by the GEMM launchers (colmap_prepare)
  int divsh;
};
inline void colmap_prepare(ColMap* c) { make_fastdiv_parts(c->P, &c->divM, &c->divsh); }

// C[m][col] = sum_k Apack[k][m] * B(k, col) (+ bias[m]); one launch covers all groups.
struct GemmTN {
  const void* A;       // packed operand [G][Kpad][Mpad], zero padded (fp32 or bf16)
  long long a_gs;      // elements between groups
  int Mpad, Kpad;
  const void* B;       // [.. k ..][cols] rows of stride b_ks (fp32 or bf16)
  long long b_ks, b_gs;
  ColMap bmap;
  int b_ld_guard;      // vector path: columns >= this are not read
  float* C;
  long long c_ms, c_gs;
  ColMap cmap;
  const float* bias;   // nullable; bias[g*bias_gs + m]
  int bias_gs;
  int M, Ncols, Kdim;  // true sizes per group
  int G;
  int bf16;            // operands are bf16 (A packed bf16, B bf16 plain rows)
  // Fused lowering (gather != 0): B is the NCHW tensor x itself and the kernel builds the Type-1
  // lowered tile on the fly: B(k, col) = x[n, q*Cg + ci, r*s + i - p, c*s + j - p] or 0, with
  // (ci, i, j) decoded from k = (ci*K + i)*K + j and (n, r, c) from col.
  int gather;
  int gC, gH, gW, gHout, gWout, gs, gp, gCg, gK, gKK;
  // tapmajor != 0 (with gather): rows are ordered k = tap*gCpad + channel, gCpad a multiple of the
  // K tile, taps on a tKi x tKj grid with pads tph / tpw and stride 1; g_divKK_* divide by gCpad;
  // the gathered tensor must lie within 2 GiB.
  int tapmajor, gCpad, tKi, tKj, tph, tpw;
  unsigned g_divKK_M, g_divK_M;  // fast division by K*K and by K
  int g_divKK_sh, g_divK_sh;
  // Depth-to-space epilogue of the channel-contiguous fused kernel (d2s != 0), used for the
  // backward-data pass of a strided layer: row m = (ci*dS + rh)*dS + rw of the product at grid
  // position (a, b) of image n is pixel (h, w) = (a*dS + rh - dP, b*dS + rw - dP) of channel
  // g*dCg + ci of the dCtot-channel, dH x dW tensor at C; pixels outside the tensor are dropped.
  int d2s, dS, dP, dH, dW, dCg, dCtot;
  int force_bm;       // row tile to use (64 / 96 / 128; Mpad a multiple of it); 0 = gemm_tn_tile's choice
  double prof_flops;  // algorithmic flops to book for the launch when they differ from 2*M*N*K*G (else 0)
  unsigned d_divSS_M, d_divS_M;  // fast division by dS*dS and by dS
  int d_divSS_sh, d_divS_sh;
};
// Cpart[s][g][m][n] = sum_{col in split s} A(m, col) * B(n, col); both operands col-contiguous.
struct GemmNT {
  const void* A;       // rows m: a_ms apart, groups a_gs apart, columns through amap
  long long a_ms, a_gs;
  ColMap amap;
  const void* B;       // plain rows n of stride b_ns, groups b_gs apart
  long long b_ns, b_gs;
  float* Cpart;        // [S][G][M][N] compact
  int M, N, Ncols;
  int G, S, split_len; // split_len is a multiple of the kernel's BK
  int bf16;
  // Fused lowering of an unpadded layer (gather != 0; fp32, A read in place): B is the NCHW
  // tensor x of the chunk and row n = (ci, i, j) of the Type-1 lowered matrix is gathered on
  // the fly, B(n, col) = x[img, q*Cg + ci, r*s + i, c*s + j] with (img, r, c) decoded from col.
  int gather;
  int gC, gH, gW, gHout, gWout, gs, gCg, gK;
};

int launch_gemm_tn(const GemmTN& p, hipStream_t st);
int launch_gemm_nt(const GemmNT& p, hipStream_t st);
// gather mode of the NT GEMM (GemmNT::gather): do its 32-bit offsets cover this geometry?
bool gemm_nt_gather_fits(int C, int H, int W, int O, int Hout, int Wout);
// Fused forward with LDS-staged lowering (p.gather must be set).  CCT_EUNSUPPORTED = the shape
// does not fit its staging area and nothing was launched: use launch_gemm_tn instead.
int launch_conv_fused(const GemmTN& p, hipStream_t st);
// The same pass with channel-contiguous operands in LDS (16-byte operand reads; see
// conv_fused_kc.hip).  It needs its own kernel pack, [group of 16 channels][tap][row][16], with
// Kpad = conv_fused_kc_kpad(channels per group, K); `flipped` selects the flipped, role-swapped
// kernels of the fused backward-data pass.  conv_fused_kc_fits: can it run this problem
// (p filled as for launch_conv_fused)?
bool conv_fused_kc_fits(const GemmTN& p);
// A pack carries zero tiles up to a multiple of four K tiles (taps x groups); the bf16 form up to a
// multiple of eight.
long long conv_fused_kc_kpad(int channels_per_group, int K, int bf16);
// `bf16`: the pack holds bf16 values (rounded to nearest even) for the bf16 form of the kernel.
int launch_pack_fused_kc(const float* w, void* pack, int G, int Og, int Cg, int K, int Mpad,
                         int flipped, int bf16, hipStream_t st);
// Kernel pack of the strided backward-data pass computed as a stride-1 convolution of dy with
// s*s sub-kernels of U x U taps, U = ceil(K/s): rows m = (ci*s + rh)*s + rw, channels = kernels oo,
// pack[q][grp][(u',v')][m][c] = w[q*Og + grp*16 + c, ci, rh + s*(U-1-u'), rw + s*(U-1-v')] (0 where
// that tap index is >= K).
int launch_pack_fused_kc_strided(const float* w, void* pack, int G, int Og, int Cg, int K, int s,
                                 int Mpad, int bf16, hipStream_t st);
int launch_conv_fused_kc(const GemmTN& p, hipStream_t st);
// The bf16-operand form (conv_fused_kc_bf16.hip): p.bf16 set, the pack in bf16 with its rows padded
// to conv_fused_kc_bf16_mpad(M); x / dy stay fp32 and are rounded while they are staged.
int conv_fused_kc_bf16_mpad(int M);
bool conv_fused_kc_bf16_fits(const GemmTN& p);
int launch_conv_fused_kc_bf16(const GemmTN& p, hipStream_t st);
// Fused backward-weights pass: split partial products of dy (NCHW, read in place) with the
// Type-1 lowering of x built in LDS.  Cpart[s][q][oo][(ci,i,j)], compact, S splits of split_len
// positions (a multiple of 32) over the nimg*Hout*Wout positions.
struct ConvBwdW {
  const float* x;
  const float* dy;
  float* Cpart;
  int C, H, W, O, Hout, Wout, s, p, Cg, Og, K;
  int nimg, G, S, split_len;
};
// false = the geometry does not fit the kernel's LDS staging (use a materialised layout)
bool conv_bwdw_fused_fits(int C, int H, int W, int K, int s, int pad, int Hout, int Wout, int Cg,
                          int Og, int O);
int launch_conv_bwdw_fused(const ConvBwdW& p, hipStream_t st);
// Tile sizes the launchers will use for a problem (so that the planner can pad the packs).
void gemm_tn_tile(int M, int Ncols, int* BM, int* BN, int* BK);
void gemm_nt_tile(int M, int N, int* BM, int* BN, int* BK);

// ---- fully connected layers (fully_connected.hip) ------------------------------------------
// Plan of one pass of a layer with K = H = W, no padding, one group, fp32 and lowering AUTO or
// TYPE1: plain matrix products over F = C*K*K features on the tensors in place.
struct FcPlan {
  int F;
  long long pack_off, part_off, scratch_off, total;  // workspace layout (bytes)
  int BM, Mpad, Kpad;   // packed dy of the two backward passes (Kpad: rows of one split)
  int S, split_len;     // splits of the contraction: forward over F, backward-data over O
};
// max_bytes < 0: the recommended plan; otherwise a plan within max_bytes of workspace (the forward
// pass then uses fewer splits).  false = the descriptor is not such a layer, the pass cannot take
// this path, or no plan fits.
bool fc_plan(const cct_conv_desc_t& d, int pass, long long max_bytes, FcPlan* P);
int fc_forward(const cct_conv_desc_t& d, const FcPlan& P, const float* x, const float* w,
               const float* bias, float* y, char* ws, hipStream_t st);
int fc_backward_data(const cct_conv_desc_t& d, const FcPlan& P, const float* w, const float* dy,
                     float* dx, char* ws, hipStream_t st);
int fc_backward_weights(const cct_conv_desc_t& d, const FcPlan& P, const float* x, const float* dy,
                        float* dw, float* dbias, char* ws, hipStream_t st);

// ---- index-map kernels (lowering / lifting and their adjoints) -----------------------------
// dt[(ch*Ki+i)*Kj+j][col] = x[n, ch, h, w] or +0; col = n*Ha*Wb + a*Wb + b, n < nimg.
int launch_lower(const float* x, void* dt, long long ld, int nimg, int C, const WinMap& m,
                 int bf16, hipStream_t st);
// y[n,o,r,c] = bias[o] + sum_{i,j} rt[(o*Ki+i)*Kj+j][n*Ha*Wb + a*Wb + b], a = r*sh+i-ph, b = c*sw+j-pw.
// Here (Ht, Wt) of the map is the output plane (Hout x Wout).
int launch_lift(const float* rt, long long ld, float* y, const float* bias, int nimg, int O,
                const WinMap& m, hipStream_t st);
// Adjoint of lift: drt[(o*Ki+i)*Kj+j][col] = dy[n,o,r,c] if a = r*sh+i-ph, b = c*sw+j-pw has a
// solution (r,c) inside the Ht x Wt plane, else +0.
int launch_inv_lift(const float* dy, void* drt, long long ld, int nimg, int O, const WinMap& m,
                    int bf16, hipStream_t st);
// Adjoint of lower: dx[n,ch,h,w] = sum_{i,j} ddt[(ch*Ki+i)*Kj+j][n*Ha*Wb + a*Wb + b] over the
// (i,j) for which h = a*sh+i-ph, w = b*sw+j-pw has a solution (a,b) inside the grid.
int launch_inv_lower(const float* ddt, long long ld, float* dx, int nimg, int C, const WinMap& m,
                     hipStream_t st);

// Lowered-kernel pack.  rho = (oo, iR, jR) indexes R^ columns, delta = (ci, iD, jD) indexes D^
// columns; K^[delta][rho] = w[q*Og+oo, ci, i, j] with (i,j) taken from whichever side carries it.
// transposed == 0: pack[q][k = delta][m = rho] (forward);  1: pack[q][k = rho][m = delta].
struct PackDesc {
  int G, Og, Cg, K;
  int RKi, RKj, DKi, DKj;  // taps carried on the R^ side / D^ side (product = K*K)
  int Mpad, Kpad;
  int transposed;
  int bf16;
};
int launch_pack_kernel_matrix(const float* w, void* pack, const PackDesc& d, hipStream_t st);
// pack[q][(oo,i',j')][ci] = w[q*Og+oo, ci, K-1-i', K-1-j'] (fp32), zero padded to Kpad x Mpad.
int launch_pack_flipped(const float* w, float* pack, int G, int Og, int Cg, int K, int Mpad,
                        int Kpad, hipStream_t st);
// Kernel matrix of the Type-2 backward-data pass with the inverse lifting done as a gather:
// pack[q][k = i'*Opad + oo][m = (ci, j)] = w[q*Og + oo, ci, K-1-i', j], zero padded.
int launch_pack_type2_bwd(const float* w, float* pack, int G, int Og, int Cg, int K, int Opad,
                          int Mpad, hipStream_t st);
// dw[o,ci,i,j] = (accumulate ? dw : 0) + sum_s part[s][q][rho][delta]
int launch_reduce_dw(const float* part, float* dw, int S, const PackDesc& d, int accumulate,
                     hipStream_t st);
// dbias[o] = sum_{n,r,c} dy[n,o,r,c]; `scratch` holds O*nblk floats.
int launch_dbias(const float* dy, float* dbias, float* scratch, int N, int O, int P, int nblk,
                 hipStream_t st);

void set_hip_error(hipError_t e);

// Times the launches issued during its lifetime when cct_profile_enable(1) is active;
// otherwise does nothing.  flops / bytes are the ALGORITHMIC work of the launch.
class ProfScope {
 public:
  ProfScope(const char* name, double flops, double bytes, hipStream_t st);
  ~ProfScope();
  ProfScope(const ProfScope&) = delete;
  ProfScope& operator=(const ProfScope&) = delete;

 private:
  hipStream_t st_;
  long long idx_;
};

// Raises the dynamic-LDS limit of kernel `Kern` to `bytes` once per device and process instead of
// on every launch.  CCT_EHIP if the runtime refuses.
template <auto Kern>
int ensure_dynamic_lds(int bytes) {
  static std::atomic<unsigned long long> done{0};  // bit d: set for device d
  int dev = 0;
  const bool known = hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64;
  if (known && (done.load(std::memory_order_acquire) >> dev) & 1ULL) return CCT_OK;
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess) {
    set_hip_error(e);
    return CCT_EHIP;
  }
  if (known) done.fetch_or(1ULL << dev, std::memory_order_release);
  return CCT_OK;
}

#define CCT_CHECK_LAUNCH()                       \
  do {                                           \
    hipError_t e__ = hipGetLastError();          \
    if (e__ != hipSuccess) {                     \
      ::cct::set_hip_error(e__);                 \
      return CCT_EHIP;                           \
    }                                            \
  } while (0)

}  // namespace cct
