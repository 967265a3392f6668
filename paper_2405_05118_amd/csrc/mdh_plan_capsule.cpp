// Planner for MCC_Capsule: ten dimensions (n, p, q, k, mi, mj | c, r, s, mk), the last four
// reduced with + (paper: Section "Examples", Subfigure 2; Appendix "Data Characteristics used in
// Deep Neural Networks").  `sizes` as for MCC: (N, P, Q, K, C, R, S, stride_h, stride_w); the three
// matrix dimensions are fixed at 4.
#include <string.h>

#include "mdh_internal.h"

namespace mdh {
using namespace detail;

static const int kCapNI[] = {1, 2, 4};

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
  p->prt[MDH_L_WG][2] = (int32_t)cdiv(s[2], 8);
  p->prt[MDH_L_WG][3] = (int32_t)(s[3] > 0 ? cdiv(s[3], 8 * pl.NI) : 1);
  p->prt[MDH_L_WAVE][1] = 4;      // one output row per wavefront
  p->prt[MDH_L_VGPR][3] = pl.NI;  // blocks along k per wavefront
  p->prt[MDH_L_VGPR][9] = 2;      // a lane's 16-byte operand read: mk = 0..3 over two MFMA pairs
  p->prt[MDH_L_LDS][6] = (int32_t)s[4];  // c, r, s are walked inside LDS (s and c fused)
  p->prt[MDH_L_LDS][7] = (int32_t)s[5];
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
  return s[0] == 0 || s[3] == 0 || (s[1] % 4) || (s[2] % 8) || (s[3] % (8 * pl.NI));
}

static bool cap_fits(const int64_t* s, int ni) {
  return capsule_lds_bytes(ni, s[4], s[5], s[6], s[7], s[8]) <= 160 * 1024;
}

static CapsulePlan cap_default(const int64_t* s) {
  // as many channel blocks per wavefront as LDS holds (the whole filter slice is staged) and K needs
  CapsulePlan pl{1, 0};
  for (int ni : kCapNI)
    if (cap_fits(s, ni) && (ni == 1 || s[3] >= 8 * ni)) pl.NI = ni;
  pl.ragged = cap_ragged(s, pl);
  return pl;
}

int capsule_candidates(const int64_t* s, CapsulePlan* out, int cap) {
  int n = 0;
  const CapsulePlan d = cap_default(s);
  if (n < cap) out[n++] = d;
  for (int ni : kCapNI) {
    if (ni == d.NI || !cap_fits(s, ni) || n >= cap) continue;
    CapsulePlan pl{ni, 0};
    pl.ragged = cap_ragged(s, pl);
    out[n++] = pl;
  }
  return n;
}

mdh_status plan_capsule(const int64_t* s, const mdh_tile_params* p, CapsulePlan* out) {
  if (!p) {
    *out = cap_default(s);
    return cap_fits(s, out->NI) ? MDH_OK : MDH_ERR_TILE_RESOURCES;
  }
  if (p->D != 10) return MDH_ERR_UNSUPPORTED;
  int64_t e[10];
  extents(s, e);
  bool ragged;
  mdh_status st = check_products(p, e, &ragged);
  if (st != MDH_OK) return st;
  if ((st = check_lanes(p)) != MDH_OK) return st;
  CapsulePlan pl{p->prt[MDH_L_VGPR][3], ragged};
  bool inst = false;
  for (int ni : kCapNI) inst = inst || ni == pl.NI;
  mdh_tile_params chk;
  params_from_plan(s, pl, &chk);
  if (!same_table(chk, *p) || !inst) return MDH_ERR_UNSUPPORTED;
  if (!cap_fits(s, pl.NI)) return MDH_ERR_TILE_RESOURCES;
  *out = pl;
  return MDH_OK;
}

}  // namespace mdh
