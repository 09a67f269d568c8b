// What the two channel-contiguous fused kernels (fp32 operands, bf16 operands) share: the tile
// constants, the staging geometry of a launch and its LDS need.
#pragma once
#include <algorithm>

#include "cct_internal.h"

namespace cct {
namespace kc {

constexpr int NT = 256;       // threads per workgroup
constexpr int BN = 128;       // positions per workgroup
constexpr int CG = 16;        // channels per group = reduction indices per K tile
constexpr int QU = 2;         // cells per thread and slot (R <= QU*256)
constexpr int kLdsCap = 80 * 1024;   // two workgroups per CU
constexpr int kLdsCap3 = 53 * 1024;  // three

struct KcGeom {
  int Wp;       // padded row width W + 2*pad (cells per staged row)
  int R;        // cells reserved per slot (multiple of 64, >= any workgroup's need)
  int ngroups;  // channel groups of 16
  int KK;       // taps
  int tpi;      // > 0: column tiles never cross an image, tpi tiles per image (the last one
                // partly empty); used when the rows of a tile that spans two images would not
                // fit the staging area.  0: tiles are cut from the positions of the whole chunk.
};

// Geometry and LDS need (at most `lds_cap` bytes: the cap decides whether column tiles are cut per
// image) of a launch whose cells and kernel rows take `cell_bytes` bytes of LDS
// each (16 channels plus the padding that spreads 16-byte accesses over the banks); false = this
// form cannot run the shape.  LDS: kernel tiles [2][BM] | cells [2][R] | tap table [KK] ints.
inline bool make_geom(const GemmTN& p, int BM, int cell_bytes, KcGeom* fg, size_t* lds,
                      int lds_cap = kLdsCap) {
  if (!p.gather || p.tapmajor || p.gK < 2 || p.gCg < 1) return false;
  fg->KK = p.gK * p.gK;
  // staged row width: the padded input row, or what the last grid column's window reaches if the
  // caller's grid is wider than the convolution arithmetic gives (columns beyond the input load
  // as zeros like any padding)
  fg->Wp = std::max(p.gW + 2 * p.gp, (p.gWout - 1) * p.gs + p.gK);
  fg->ngroups = (p.gCg + CG - 1) / CG;
  // channels are padded to whole groups of 16: not worth it when that wastes over an eighth
  if ((long long)fg->ngroups * CG * 8 > (long long)p.gCg * 9) return false;
  const long long P = (long long)p.gHout * p.gWout;
  // rows of padded input that 128 consecutive positions can touch: at most A output rows spread
  // over at most T images; t images need (A - t)*stride + t*K rows, largest at t = 1 or t = T
  const long long A = (BN - 1) / p.gWout + 2, T = (BN - 1) / P + 2;
  const long long r1 = (A - 1) * p.gs + p.gK;
  const long long rT = (A > T ? A - T : 0) * p.gs + T * p.gK;
  auto cells = [&](long long rows) { return (rows * fg->Wp + 63) / 64 * 64; };
  auto lds_of = [&](long long R) {
    return (long long)cell_bytes * (2LL * BM + 2LL * R) + 4LL * fg->KK;
  };
  long long R = cells(r1 > rT ? r1 : rT);
  fg->tpi = 0;
  if (R > QU * NT || lds_of(R) > lds_cap) {
    // tiles cut per image need the rows of one image only; worth it while the partly empty last
    // tile of an image wastes less than a tenth of the launch
    const long long tpi = (P + BN - 1) / BN;
    const long long rows1 = (A < p.gHout ? A - 1 : p.gHout - 1) * p.gs + p.gK;
    R = cells(rows1);
    if (tpi * BN * 10 > P * 11 || tpi * ((double)p.Ncols / P) >= 2147483647.0) return false;
    fg->tpi = (int)tpi;
  }
  if (R > QU * NT) return false;
  fg->R = (int)R;
  // staged cells are addressed with 32-bit byte offsets from the workgroup's first image
  if ((T + 1) * p.gC * p.gH * p.gW >= (1LL << 29)) return false;
  const long long need = lds_of(R);
  if (need > lds_cap) return false;
  *lds = (size_t)need;
  return true;
}

}  // namespace kc
}  // namespace cct
