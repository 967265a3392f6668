// Planner for MCC_Capsule: ten dimensions (n, p, q, k, mi, mj | c, r, s, mk), the last four
// reduced with + (paper: Section "Examples", Subfigure 2; Appendix "Data Characteristics used in
// Deep Neural Networks").  `sizes` as for MCC: (N, P, Q, K, C, R, S, stride_h, stride_w); the three
// matrix dimensions are fixed at 4.
#include <string.h>

#include "mdh_internal.h"

namespace mdh {
using namespace detail;

static const int kCapMenu[][2] = {{1, 1}, {2, 1}, {4, 1}, {1, 2}, {2, 2}};  // NI, RW

static void extents(const int64_t* s, int64_t* e) {
  e[0] = s[0], e[1] = s[1], e[2] = s[2], e[3] = s[3];
  e[4] = 4, e[5] = 4;
  e[6] = s[4], e[7] = s[5], e[8] = s[6];
  e[9] = 4;
}

void params_from_plan(const int64_t* s, const CapsulePlan& pl, mdh_tile_params* p) {
  clear_params(p, 10);
  // MFMA block: (8 q x 4 mi) x (8 k x 4 mj) x 2 of mk
  p->blk[2] = 8;
  p->blk[4] = 4;
  p->blk[3] = 8;
  p->blk[5] = 4;
  p->blk[9] = 2;
  p->prt[MDH_L_WG][0] = (int32_t)(s[0] > 0 ? s[0] : 1);
  p->prt[MDH_L_WG][1] = (int32_t)cdiv(s[1], 4);
  p->prt[MDH_L_WG][2] = (int32_t)cdiv(cdiv(s[2], 8), pl.QT);
  p->prt[MDH_L_HBM][2] = pl.QT;  // column tiles walked sequentially with the filter slice resident
  p->prt[MDH_L_WG][3] = (int32_t)(s[3] > 0 ? cdiv(s[3], 8 * pl.NI) : 1);
  p->prt[MDH_L_WAVE][1] = 4;      // one output row per wavefront
  // the walk over (r, s, c) is cut into RW wavefront parts; in the table they sit on r
  p->prt[MDH_L_WAVE][7] = pl.RW;
  p->prt[MDH_L_VGPR][3] = pl.NI;  // blocks along k per wavefront
  p->prt[MDH_L_VGPR][9] = 2;      // a lane's 16-byte operand read: mk = 0..3 over two MFMA pairs
  p->prt[MDH_L_LDS][6] = (int32_t)s[4];  // c, r, s are walked inside LDS (s and c fused)
  p->prt[MDH_L_LDS][7] = (int32_t)cdiv(s[5], pl.RW);
  p->prt[MDH_L_LDS][8] = (int32_t)s[6];
  static const int dims[10] = {0, 1, 2, 3, 4, 5, 6, 7, 8, 9};
  set_order(p, dims);
  p->strided = 0;
  p->lane_fast_dim = 5;  // mj, then k: the lanes of a block column
  p->in_region[0] = MDH_MR_LDS;
  p->in_region[1] = MDH_MR_LDS;
  p->in_transposed[1] = 1;  // the filter's 4 x 4 matrices are staged transposed
  p->out_region = MDH_MR_VGPR;
  p->ragged = (uint8_t)pl.ragged;
}

static int cap_ragged(const int64_t* s, const CapsulePlan& pl) {
  return s[0] == 0 || s[3] == 0 || (s[1] % 4) || (s[2] % (8 * pl.QT)) || (s[3] % (8 * pl.NI)) || (s[5] % pl.RW);
}

static bool cap_fits(const int64_t* s, int ni, int rw = 1) {
  return capsule_lds_bytes(ni, rw, s[4], s[5], s[6], s[7], s[8]) <= 160 * 1024;
}

static CapsulePlan cap_plan(const int64_t* s, int ni, int qt, int rw) {
  const int64_t tiles = cdiv(s[2] > 0 ? s[2] : 1, 8);
  if (qt > tiles) qt = (int)tiles;
  qt = (int)cdiv(tiles, cdiv(tiles, qt));  // no workgroup without a tile
  CapsulePlan pl{ni, qt, rw, 0};
  pl.ragged = cap_ragged(s, pl);
  return pl;
}

static CapsulePlan cap_default(const int64_t* s) {
  // Measured: long walks (7x7x3 taps: 77 steps) are fastest with one block of 8 channels per
  // wavefront and the walk split over two wavefronts (2.09 ms against 2.31 ms unsplit); short ones
  // (3x3x3: 15 steps) unsplit, with four blocks per wavefront where K gives every workgroup 32
  // channels (VGG-16 shape: 1.52 ms against 1.61 ms with one block), else one block (MobileNet
  // shape, K = 32: 0.24 ms against 0.26 ms with four).  Column tiles per workgroup: as many as leave
  // one workgroup per compute unit (the filter slice is staged once per workgroup).
  const bool long_walk = s[5] * cdiv(s[6] * s[4], 2) >= 32;
  const int rw = long_walk && cap_fits(s, 1, 2) ? 2 : 1;
  const int ni = !long_walk && s[3] >= 64 && cap_fits(s, 4, 1) ? 4 : 1;
  const int64_t tiles = cdiv(s[2] > 0 ? s[2] : 1, 8);
  const int64_t other = (s[0] > 0 ? s[0] : 1) * cdiv(s[1] > 0 ? s[1] : 1, 4) * cdiv(s[3] > 0 ? s[3] : 1, 8 * ni);
  int qt = 1;
  while (qt < tiles && qt < 16 && other * cdiv(tiles, qt * 2) >= 256) qt *= 2;  // beyond ~16 tiles nothing is gained
  return cap_plan(s, ni, qt, rw);
}

int capsule_candidates(const int64_t* s, CapsulePlan* out, int cap) {
  int n = 0;
  const CapsulePlan d = cap_default(s);
  if (n < cap) out[n++] = d;
  static const int qts[] = {1, 2, 4, 7, 8, 14, 16, 28};
  for (auto& m : kCapMenu)
    for (int qt : qts) {
      if (!cap_fits(s, m[0], m[1]) || n >= cap) continue;
      const CapsulePlan pl = cap_plan(s, m[0], qt, m[1]);
      bool dup = false;
      for (int i = 0; i < n; ++i) dup = dup || (out[i].NI == pl.NI && out[i].QT == pl.QT && out[i].RW == pl.RW);
      if (!dup) out[n++] = pl;
    }
  return n;
}

mdh_status plan_capsule(const int64_t* s, const mdh_tile_params* p, CapsulePlan* out) {
  if (!p) {
    *out = cap_default(s);
    return cap_fits(s, out->NI, out->RW) ? MDH_OK : MDH_ERR_TILE_RESOURCES;
  }
  if (p->D != 10) return MDH_ERR_UNSUPPORTED;
  int64_t e[10];
  extents(s, e);
  bool ragged;
  mdh_status st = check_products(p, e, &ragged);
  if (st != MDH_OK) return st;
  if ((st = check_lanes(p)) != MDH_OK) return st;
  CapsulePlan pl{p->prt[MDH_L_VGPR][3], p->prt[MDH_L_HBM][2], p->prt[MDH_L_WAVE][7], ragged};
  // a workgroup part of q that owns no tile is not a partition of the columns
  if ((int64_t)(p->prt[MDH_L_WG][2] - 1) * pl.QT * 8 >= (s[2] > 0 ? s[2] : 1)) return MDH_ERR_TILE_NOT_DIVIDING;
  bool inst = false;
  for (auto& m : kCapMenu) inst = inst || (m[0] == pl.NI && m[1] == pl.RW);
  mdh_tile_params chk;
  params_from_plan(s, pl, &chk);
  if (!same_table(chk, *p) || !inst) return MDH_ERR_UNSUPPORTED;
  if (!cap_fits(s, pl.NI, pl.RW)) return MDH_ERR_TILE_RESOURCES;
  *out = pl;
  return MDH_OK;
}

}  // namespace mdh
