// Planner for the batched / transposed MatMul (bMatMul, MatMul^T): dims (b, i, j, k).
// The table is the one of MatMul with the batch as one more workgroup-layer concatenation
// dimension; the transposed views are carried by the layout parameters (D4/R4):
// in_transposed[0] (A), in_transposed[1] (B), out_transposed (C).
#include <string.h>

#include "mdh_internal.h"

namespace mdh {
using namespace detail;

static const int kExMenu[][5] = {  // BM, BN, BK, WM, WN
    {128, 128, 16, 64, 64}, {128, 64, 16, 64, 32}, {64, 64, 16, 32, 32}, {32, 128, 16, 32, 32}, {32, 64, 16, 32, 32}};

static bool ex_inst(const GemmPlan& g) {
  for (auto& m : kExMenu)
    if (m[0] == g.BM && m[1] == g.BN && m[2] == g.BK && m[3] == g.WM && m[4] == g.WN) return true;
  return false;
}

// sizes: batch, M, N, K, trans_a, trans_b, trans_c
void params_from_plan(const int64_t* s, const GemmExPlan& pl, mdh_tile_params* p) {
  const GemmPlan& g = pl.g;
  clear_params(p, 4);
  p->blk[1] = 32;
  p->blk[2] = 32;
  p->blk[3] = 2;
  p->prt[MDH_L_WG][0] = (int32_t)s[0];
  p->prt[MDH_L_WG][1] = (int32_t)cdiv(s[1], g.BM);
  p->prt[MDH_L_WG][2] = (int32_t)cdiv(s[2], g.BN);
  p->prt[MDH_L_WG][3] = g.S;
  p->prt[MDH_L_HBM][3] = (int32_t)cdiv(cdiv(s[3], g.S), g.BK);
  p->prt[MDH_L_WAVE][1] = g.BM / g.WM;
  p->prt[MDH_L_WAVE][2] = g.BN / g.WN;
  p->prt[MDH_L_LDS][3] = g.BK / 2;
  p->prt[MDH_L_VGPR][1] = g.WM / 32;
  p->prt[MDH_L_VGPR][2] = g.WN / 32;
  static const int dims[4] = {0, 1, 2, 3};
  set_order(p, dims);
  p->strided = 0;
  p->lane_fast_dim = pl.tc ? 1 : 2;
  p->in_region[0] = MDH_MR_LDS;
  p->in_region[1] = MDH_MR_LDS;
  p->out_region = MDH_MR_VGPR;
  p->in_transposed[0] = (uint8_t)pl.ta;
  p->in_transposed[1] = (uint8_t)pl.tb;
  p->out_transposed = (uint8_t)pl.tc;
  p->ragged = (uint8_t)g.ragged;
}

static int ex_ragged(const int64_t* s, const GemmPlan& g) {
  return (s[1] % g.BM) || (s[2] % g.BN) || (s[3] % ((int64_t)g.S * g.BK));
}

static GemmExPlan ex_default(const int64_t* s) {
  const int64_t batch = s[0], M = s[1], N = s[2], K = s[3];
  GemmPlan g{128, 128, 16, 64, 64, 1, 0};
  if (N <= 64) g = GemmPlan{128, 64, 16, 64, 32, 1, 0};
  if (M <= 64) g = GemmPlan{64, 64, 16, 32, 32, 1, 0};
  if (M <= 32) g = GemmPlan{32, 128, 16, 32, 32, 1, 0};  // small M: one block row, lanes spent on j
  if (M <= 32 && N <= 64) g = GemmPlan{32, 64, 16, 32, 32, 1, 0};
  // mid-sized problems: the largest tile that still gives every compute unit two workgroups
  if (M > 64 && N > 64 && batch * cdiv(M, 128) * cdiv(N, 128) < 512) {
    g = GemmPlan{128, 64, 16, 64, 32, 1, 0};
    if (batch * cdiv(M, 128) * cdiv(N, 64) < 512) g = GemmPlan{64, 64, 16, 32, 32, 1, 0};
  }
  // few output tiles: parallelise the reduction dimension over workgroups (the paper's point about
  // small-M deep-learning shapes)
  const int64_t tiles = batch * cdiv(M, g.BM) * cdiv(N, g.BN);
  int S = 1;
  while (tiles * S < 1024 && S < 64 && K / (S * 2) >= 4 * g.BK) S *= 2;
  g.S = S;
  g.ragged = ex_ragged(s, g);
  return GemmExPlan{g, (int)s[4], (int)s[5], (int)s[6]};
}

int matmul_ex_candidates(const int64_t* s, GemmExPlan* out, int cap) {
  int n = 0;
  auto push = [&](GemmPlan g) {
    if (n >= cap) return;
    if (g.S > 1 && s[3] / g.S < g.BK) return;
    g.ragged = ex_ragged(s, g);
    for (int i = 0; i < n; ++i)
      if (out[i].g.BM == g.BM && out[i].g.BN == g.BN && out[i].g.S == g.S) return;
    out[n++] = GemmExPlan{g, (int)s[4], (int)s[5], (int)s[6]};
  };
  push(ex_default(s).g);
  static const int splits[] = {1, 2, 4, 8, 16, 32};
  for (auto& m : kExMenu)
    for (int S : splits) {
      const int64_t tiles = s[0] * cdiv(s[1], m[0]) * cdiv(s[2], m[1]);
      if (S > 1 && tiles * (S / 2) >= 2048) continue;
      push(GemmPlan{m[0], m[1], m[2], m[3], m[4], S, 0});
    }
  return n;
}

mdh_status plan_matmul_ex(const int64_t* s, const mdh_tile_params* p, GemmExPlan* out) {
  if (!p) {
    *out = ex_default(s);
    return MDH_OK;
  }
  if (p->D != 4) return MDH_ERR_UNSUPPORTED;
  bool ragged;
  mdh_status st = check_products(p, s, &ragged);
  if (st != MDH_OK) return st;
  if ((st = check_lanes(p)) != MDH_OK) return st;
  GemmPlan g;
  g.WM = p->prt[MDH_L_VGPR][1] * 32;
  g.WN = p->prt[MDH_L_VGPR][2] * 32;
  g.BM = p->prt[MDH_L_WAVE][1] * g.WM;
  g.BN = p->prt[MDH_L_WAVE][2] * g.WN;
  g.BK = p->prt[MDH_L_LDS][3] * 2;
  g.S = p->prt[MDH_L_WG][3];
  g.ragged = ragged;
  GemmExPlan pl{g, (int)s[4], (int)s[5], (int)s[6]};
  mdh_tile_params chk;
  params_from_plan(s, pl, &chk);
  // the layout parameters of the configuration must describe the views the call passes
  if (!same_table(chk, *p) || !ex_inst(g)) return MDH_ERR_UNSUPPORTED;
  *out = pl;
  return MDH_OK;
}

}  // namespace mdh
