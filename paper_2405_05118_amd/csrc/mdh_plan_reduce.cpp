// Planner for the pure-reduction instances Dot = md_hom(*, (+)) and MatVec = md_hom(*, (++,+)):
// tuning-parameter table <-> launch descriptor, as mdh_plan.cpp does for the other instances.
// In both, the reduction dimension k runs over the lanes (strided assignment: consecutive
// lanes own consecutive 4-element parts, the paper's "inner parallelism"), so its re-composition
// climbs the whole ladder lane -> wavefront -> workgroup -> grid.
#include <string.h>

#include "mdh_internal.h"

namespace mdh {
using namespace detail;

// =============================================================================== Dot

static const int kDotWaves[] = {4, 8, 16};

void params_from_plan(const int64_t* s, const DotPlan& pl, mdh_tile_params* p) {
  clear_params(p, 1);
  p->prt[MDH_L_WG][0] = pl.S;
  p->prt[MDH_L_WAVE][0] = pl.WAVES;
  p->prt[MDH_L_LANE][0] = 64;
  p->prt[MDH_L_VGPR][0] = 4;
  p->prt[MDH_L_HBM][0] = (int32_t)cdiv(s[0], (int64_t)pl.S * pl.WAVES * 256);
  static const int dims[1] = {0};
  set_order(p, dims);
  p->strided = (uint8_t)pl.strided;
  p->lane_fast_dim = 0;
  p->in_region[0] = MDH_MR_VGPR;  // streamed once: global memory straight to registers
  p->in_region[1] = MDH_MR_VGPR;
  // where the workgroup-layer parts are combined: device memory, by the last part to arrive (one
  // launch), or a second kernel (the first kernel's results leave from registers)
  p->out_region = (pl.S > 1 && pl.fused) ? MDH_MR_HBM : MDH_MR_VGPR;
  p->ragged = (uint8_t)pl.ragged;
}

static int dot_ragged(const int64_t* s, const DotPlan& pl) {
  return (s[0] % ((int64_t)pl.S * pl.WAVES * 256)) != 0;
}

static DotPlan dot_default(const int64_t* s) {
  // workgroups of 8 wavefronts, one per compute unit, as long as each still streams a few KiB
  // (2^28 elements: 0.300 ms with 256 such workgroups, 0.314 ms with 1024 of 4 wavefronts)
  DotPlan pl{8, 1, 0};
  int S = 1;
  while (S < 256 && s[0] / (2ll * S) >= (int64_t)pl.WAVES * 256 * 8) S *= 2;
  // a few KiB in all: one workgroup and no second pass (2^16 elements: 8.8 us against 12.3 us)
  if (s[0] <= (1 << 17)) S = 1;
  pl.S = S;
  pl.fused = S > 1;
  pl.ragged = dot_ragged(s, pl);
  return pl;
}

int dot_candidates(const int64_t* s, DotPlan* out, int cap) {
  int n = 0;
  auto push = [&](DotPlan pl) {
    if (n >= cap || pl.S < 1) return;
    if (pl.S > 1 && s[0] / pl.S < 1) return;
    pl.ragged = dot_ragged(s, pl);
    if (pl.S == 1) pl.fused = 0;
    for (int i = 0; i < n; ++i)
      if (out[i].WAVES == pl.WAVES && out[i].S == pl.S && out[i].strided == pl.strided && out[i].fused == pl.fused) return;
    out[n++] = pl;
  };
  DotPlan d = dot_default(s);
  push(d);
  for (int w : kDotWaves)
    for (int S = d.S / 4 > 0 ? d.S / 4 : 1; S <= d.S * 4 && S <= 8192; S *= 2) push(DotPlan{w, S, 0});
  // the default's tile with the second kernel instead of the one-launch combination, and with the
  // blocked lane assignment (parameter D2: every lane one contiguous part)
  DotPlan v = d;
  v.fused = 0;
  push(v);
  v = d;
  v.strided = 0;
  push(v);
  return n;
}

mdh_status plan_dot(const int64_t* s, const mdh_tile_params* p, DotPlan* out) {
  if (!p) {
    *out = dot_default(s);
    return MDH_OK;
  }
  if (p->D != 1) return MDH_ERR_UNSUPPORTED;
  bool ragged;
  mdh_status st = check_products(p, s, &ragged);
  if (st != MDH_OK) return st;
  if ((st = check_lanes(p)) != MDH_OK) return st;
  DotPlan pl{p->prt[MDH_L_WAVE][0], p->prt[MDH_L_WG][0], ragged};
  pl.strided = p->strided ? 1 : 0;
  pl.fused = (pl.S > 1 && p->out_region == MDH_MR_HBM) ? 1 : 0;
  bool inst = false;
  for (int w : kDotWaves) inst = inst || (w == pl.WAVES);
  mdh_tile_params chk;
  params_from_plan(s, pl, &chk);
  if (!same_table(chk, *p) || !inst || pl.S > 8192) return MDH_ERR_UNSUPPORTED;
  *out = pl;
  return MDH_OK;
}

// =============================================================================== MatVec

static const int kMatVecMenu[][3] = {  // RM, WM, WK
    {4, 4, 1}, {2, 4, 1}, {8, 4, 1}, {1, 4, 1}, {4, 2, 2}, {2, 2, 2}, {4, 1, 4}, {2, 1, 4}, {1, 1, 4},
    {4, 8, 1}, {1, 1, 8}, {2, 1, 8}};

static bool matvec_inst(const MatVecPlan& pl) {
  for (auto& m : kMatVecMenu)
    if (m[0] == pl.RM && m[1] == pl.WM && m[2] == pl.WK) return true;
  return false;
}

void params_from_plan(const int64_t* s, const MatVecPlan& pl, mdh_tile_params* p) {
  clear_params(p, 2);  // dims: 0 i, 1 k
  if (pl.rowlanes) {  // lanes along i: 4 wavefronts x 64 rows per workgroup, a lane walks all of k in steps of 4
    p->prt[MDH_L_WG][0] = (int32_t)cdiv(s[0], 256);
    p->prt[MDH_L_WAVE][0] = 4;
    p->prt[MDH_L_LANE][0] = 64;
    p->prt[MDH_L_VGPR][1] = 4;
    p->prt[MDH_L_HBM][1] = (int32_t)cdiv(s[1], 4);
    static const int rdims[2] = {0, 1};
    set_order(p, rdims);
    p->strided = 0;
    p->lane_fast_dim = 0;
    p->in_region[0] = MDH_MR_VGPR;
    p->in_region[1] = MDH_MR_VGPR;
    p->out_region = MDH_MR_VGPR;
    p->ragged = (uint8_t)((s[0] % 256) || (s[1] % 4));
    return;
  }
  p->prt[MDH_L_WG][0] = (int32_t)cdiv(s[0], (int64_t)pl.WM * pl.RM);
  p->prt[MDH_L_WG][1] = pl.S;
  p->prt[MDH_L_WAVE][0] = pl.WM;
  p->prt[MDH_L_WAVE][1] = pl.WK;
  p->prt[MDH_L_LANE][1] = 64;
  p->prt[MDH_L_VGPR][0] = pl.RM;
  p->prt[MDH_L_VGPR][1] = 4;
  p->prt[MDH_L_HBM][1] = (int32_t)cdiv(s[1], (int64_t)pl.S * pl.WK * 256);
  static const int dims[2] = {0, 1};
  set_order(p, dims);
  p->strided = (uint8_t)pl.strided;
  p->lane_fast_dim = 1;           // k is the contiguous dimension of A
  p->in_region[0] = MDH_MR_VGPR;  // A is read once: no staging
  p->in_region[1] = MDH_MR_VGPR;  // x is reused RM times from registers, across rows from L2
  p->out_region = MDH_MR_VGPR;
  p->ragged = (uint8_t)pl.ragged;
}

static int matvec_ragged(const int64_t* s, const MatVecPlan& pl) {
  return (s[0] % ((int64_t)pl.WM * pl.RM)) || (s[1] % ((int64_t)pl.S * pl.WK * 256));
}

static MatVecPlan matvec_default(const int64_t* s) {
  const int64_t M = s[0], K = s[1];
  // long rows: the eight wavefronts of a workgroup interleave 256-element steps of k (measured
  // 7.2 TB/s at 16384^2); short rows: one wavefront per group of rows
  MatVecPlan pl{2, 1, 8, 1, 0};
  if (K < 2048) pl = MatVecPlan{8, 4, 1, 1, 0};
  if (M < 64 && K >= 2048) pl = MatVecPlan{1, 1, 8, 1, 0};
  const int64_t wgs = cdiv(M, (int64_t)pl.WM * pl.RM);
  int S = 1;
  while (wgs * S < 1024 && S < 256 && K / (2ll * S) >= (int64_t)pl.WK * 256 * 4) S *= 2;
  pl.S = S;
  pl.ragged = matvec_ragged(s, pl);
  return pl;
}

int matvec_candidates(const int64_t* s, MatVecPlan* out, int cap) {
  int n = 0;
  auto push = [&](MatVecPlan pl) {
    if (n >= cap) return;
    if (pl.S > 1 && s[1] / pl.S < 1) return;
    pl.ragged = matvec_ragged(s, pl);
    for (int i = 0; i < n; ++i)
      if (out[i].RM == pl.RM && out[i].WM == pl.WM && out[i].WK == pl.WK && out[i].S == pl.S &&
          out[i].strided == pl.strided)
        return;
    out[n++] = pl;
  };
  MatVecPlan d = matvec_default(s);
  push(d);
  for (auto& m : kMatVecMenu)
    for (int S = d.S / 2 > 0 ? d.S / 2 : 1; S <= d.S * 2 && S <= 256; S *= 2)
      push(MatVecPlan{m[0], m[1], m[2], S, 0});
  // the default's tile with the blocked lane assignment (parameter D2: every lane one contiguous part)
  d.strided = 0;
  push(d);
  // lanes along i instead of k (the dimension that follows the fastest lane index)
  if (n < cap) {
    MatVecPlan r{1, 4, 1, 1, 0};
    r.strided = 0;
    r.rowlanes = 1;
    r.ragged = (s[0] % 256) || (s[1] % 4);
    out[n++] = r;
  }
  return n;
}

mdh_status plan_matvec(const int64_t* s, const mdh_tile_params* p, MatVecPlan* out) {
  if (!p) {
    *out = matvec_default(s);
    return MDH_OK;
  }
  if (p->D != 2) return MDH_ERR_UNSUPPORTED;
  bool ragged;
  mdh_status st = check_products(p, s, &ragged);
  if (st != MDH_OK) return st;
  if ((st = check_lanes(p)) != MDH_OK) return st;
  MatVecPlan pl{p->prt[MDH_L_VGPR][0], p->prt[MDH_L_WAVE][0], p->prt[MDH_L_WAVE][1],
                p->prt[MDH_L_WG][1], ragged};
  pl.strided = p->strided ? 1 : 0;
  mdh_tile_params chk;
  if (p->lane_fast_dim == 0) {  // lanes along i
    pl = MatVecPlan{1, 4, 1, 1, ragged};
    pl.strided = 0;
    pl.rowlanes = 1;
    params_from_plan(s, pl, &chk);
    if (!same_table(chk, *p)) return MDH_ERR_UNSUPPORTED;
    *out = pl;
    return MDH_OK;
  }
  params_from_plan(s, pl, &chk);
  if (!same_table(chk, *p) || !matvec_inst(pl) || pl.S > 256) return MDH_ERR_UNSUPPORTED;
  *out = pl;
  return MDH_OK;
}

}  // namespace mdh
