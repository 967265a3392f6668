// Planner for the batched / transposed MatMul (bMatMul, MatMul^T): dims (b, i, j, k).
// The table is the one of MatMul with the batch as one more workgroup-layer concatenation
// dimension; the transposed views are carried by the layout parameters (D4/R4):
// in_transposed[0] (A), in_transposed[1] (B), out_transposed (C).
#include <string.h>

#include "mdh_internal.h"

namespace mdh {
using namespace detail;

static const int kExMenu[][5] = {  // BM, BN, BK, WM, WN
    {128, 128, 32, 64, 64}, {128, 64, 32, 64, 32}, {64, 64, 32, 32, 32}, {128, 128, 16, 64, 64},
    {128, 64, 16, 64, 32},  {64, 64, 16, 32, 32},  {32, 128, 16, 32, 32}, {32, 64, 16, 32, 32}};

static bool ex_inst(const GemmPlan& g) {
  for (auto& m : kExMenu)
    if (m[0] == g.BM && m[1] == g.BN && m[2] == g.BK && m[3] == g.WM && m[4] == g.WN) return true;
  return false;
}

// Small-M kernel: wavefronts along j x wavefronts along k
static const int kSkinnyMenu[][2] = {{1, 4}, {1, 8}, {2, 2}, {4, 1}, {1, 1}};

static bool skinny_inst(int wn, int wk) {
  for (auto& m : kSkinnyMenu)
    if (m[0] == wn && m[1] == wk) return true;
  return false;
}

// Table of the small-M kernel: block 16 x 16 x 4, a wavefront owns 64 columns (4 column residues
// in registers) and walks its k part in steps of 16 (4 k per lane group in registers); A and B are
// read into registers directly.
static void skinny_params(const int64_t* s, const GemmExPlan& pl, mdh_tile_params* p) {
  const GemmPlan& g = pl.g;
  clear_params(p, 4);
  p->blk[1] = 16;
  p->blk[2] = 16;
  p->blk[3] = 4;
  const bool narrow = g.BN == 16;  // a workgroup owns one block column; rounds of 128 k per wavefront
  // k a wavefront takes per step (four 16-steps at once when B is transposed, eight with narrow strips)
  const int64_t kstep = narrow ? 128 : pl.tb ? 64 : 16;
  const int64_t kchunk = cdiv(cdiv(s[3], g.S), kstep) * kstep;
  p->prt[MDH_L_WG][0] = (int32_t)s[0];
  p->prt[MDH_L_WG][1] = (int32_t)cdiv(s[1], 16);
  p->prt[MDH_L_WG][2] = (int32_t)cdiv(s[2], g.BN);
  p->prt[MDH_L_WG][3] = g.S;
  p->prt[MDH_L_HBM][3] = (int32_t)cdiv(kchunk, kstep * pl.WK);
  p->prt[MDH_L_WAVE][2] = narrow ? 1 : g.BN / 64;
  p->prt[MDH_L_WAVE][3] = pl.WK;
  p->prt[MDH_L_VGPR][2] = narrow ? 1 : 4;
  p->prt[MDH_L_VGPR][3] = (int32_t)(kstep / 4);
  static const int dims[4] = {0, 1, 2, 3};
  set_order(p, dims);
  p->strided = 1;  // the wavefronts along k interleave their 16-row parts
  p->lane_fast_dim = 2;
  // narrow strips with B transposed: operands read straight into the MFMA layout, or staged through LDS
  p->in_region[0] = (narrow && pl.lds) ? MDH_MR_LDS : MDH_MR_VGPR;
  p->in_region[1] = (narrow && pl.lds) ? MDH_MR_LDS : MDH_MR_VGPR;
  // where the workgroup-layer parts of k are combined: in device memory by the last workgroup part of a
  // strip to arrive (one launch), or by a second kernel (results leave the first from registers)
  p->out_region = (g.S > 1 && pl.fused) ? MDH_MR_HBM : MDH_MR_VGPR;
  p->in_transposed[1] = (uint8_t)pl.tb;
  p->ragged = (uint8_t)g.ragged;
}

static int skinny_ragged(const int64_t* s, const GemmExPlan& pl) {
  const int64_t kstep = pl.g.BN == 16 ? 128 : pl.tb ? 64 : 16;
  const int64_t kchunk = cdiv(cdiv(s[3], pl.g.S), kstep) * kstep;
  return (s[1] % 16) || (s[2] % pl.g.BN) || (s[3] != (int64_t)pl.g.S * cdiv(kchunk, kstep * pl.WK) * pl.WK * kstep);
}

// strips whose arrivals the one-launch combination has to count
static int64_t skinny_strips(const int64_t* s) { return s[0] * cdiv(s[1], 16) * cdiv(s[2], 64); }

static GemmExPlan skinny_plan(const int64_t* s, int wn, int wk, int S, int fused = 1) {
  GemmExPlan pl{GemmPlan{16, 64 * wn, 16, 16, 64, S, 0}, 0, (int)s[5], 0, 1, wk};
  pl.g.ragged = skinny_ragged(s, pl);
  pl.fused = (S > 1 && fused && skinny_strips(s) <= kArrivalCounters) ? 1 : 0;
  return pl;
}

// narrow strips: 16 columns per workgroup, k over the wk wavefronts of the workgroup only
static GemmExPlan skinny_narrow_plan(const int64_t* s, int wk, int lds = 0) {
  GemmExPlan pl{GemmPlan{16, 16, 16, 16, 16, 1, 0}, 0, (int)s[5], 0, 1, wk};
  pl.lds = lds;
  pl.g.ragged = skinny_ragged(s, pl);
  return pl;
}

// plain views, or B transposed (B stored [N][K])
static bool skinny_applies(const int64_t* s) { return s[1] <= 16 && !s[4] && !s[6]; }

// sizes: batch, M, N, K, trans_a, trans_b, trans_c
void params_from_plan(const int64_t* s, const GemmExPlan& pl, mdh_tile_params* p) {
  if (pl.skinny) return skinny_params(s, pl, p);
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

static GemmExPlan ex_default_tiled(const int64_t* s);

static GemmExPlan ex_default(const int64_t* s) {
  const int64_t batch = s[0], M = s[1], N = s[2], K = s[3];
  if (skinny_applies(s)) {
    // B streams once from HBM: 8 wavefronts along k per workgroup, and k parts over workgroups until
    // 2048 wavefronts (two per SIMD) are in flight, each still walking at least one step of 16 rows: what
    // a compute unit keeps in flight is bounded (~16 KB per microsecond for cold data), so a small B is
    // read fastest when every unit reads a little, and the parts are combined by all wavefronts of the
    // last workgroup in one round of loads
    // (measured best on 16 x 1000 x 2048, 8 x 1000 x 4096, 16 x 4096 x 4096 and 16 x 4096 x 25088)
    // B transposed: a lane reads 16 bytes of its column's row whatever the strip width, so 16-column
    // strips cost nothing in coalescing and need no combination between workgroups; they win once they
    // fill the chip or a workgroup's slice of B (64 B x K) is a few rounds of requests
    // (16 x 1000 x 2048: 10.0 against 14.3 us; 16 x 4096 x 4096: 18.7 against 24.9; 16 x 1000 x 8192 and
    // 16 x 256 x 8192: the split of k over workgroups wins, 24 against 32 and 21 against 32 us)
    // B transposed: the strips' rows of B are runs of k, read as whole 512-byte runs and handed to the MFMA
    // operand layout through LDS (16 x 4096 x 25088: 73 us against 109 with one 16-byte piece per lane and
    // row; 16 x 8192 x 8192: 46 against 69; 16 x 4096 x 4096: 14.9 against 19.2; 16 x 1000 x 2048: 8.1
    // against 9.9; four wavefronts a workgroup are as fast as eight or faster)
    if (s[5] && (batch * cdiv(N, 16) >= 192 || K <= 3072)) return skinny_narrow_plan(s, 4, 1);
    // plain view: 16-column strips use half of every 128-byte line, which only pays where they fill the
    // chip and a workgroup's slice is one or two rounds (16 x 4096 x 1024: 7.9 against 9.1 us; 4 x 16 x 1000
    // x 2048: 14.8 against 17.1 us; 16 x 4096 x 4096: 23.6 against 17.3 us)
    if (!s[5] && batch * cdiv(N, 16) >= 192 && K <= 2048) return skinny_narrow_plan(s, 8);
    const int64_t strips = batch * cdiv(M, 16) * cdiv(N, 64);
    int S = 1;
    // more than 32 parts (a second round of loads in the combination) only where a part still walks four
    // steps (16 x 256 x 8192: 10.7 us with 32 parts, 14.4 with 64; 16 x 64 x 65536: 19.6 us with 64, 25.8 with 32)
    while (strips * 8 * S < 2048 && S < 64 && K / (2 * S) >= 8 * 16 && (S < 32 || K / (2 * S) >= 8 * 16 * 4)) S *= 2;
    return skinny_plan(s, 1, 8, S);
  }
  return ex_default_tiled(s);
}

static GemmExPlan ex_default_tiled(const int64_t* s) {
  const int64_t batch = s[0], M = s[1], N = s[2], K = s[3];
  // the rule of MatMul with the batch counted into the workgroups: the largest of 128x128, 128x64,
  // 64x64 that still gives two workgroups per compute unit
  GemmPlan g{128, 128, 32, 64, 64, 1, 0};
  // one tile spans a short dimension: 128 x 64 tiles only where they still give two workgroups per
  // compute unit, 64 x 64 otherwise (96 x 512 x 64 x 512: 33 us against 41 us with 128 x 64 and k split)
  if (N <= 64) g = batch * cdiv(M, 128) >= 512 ? GemmPlan{128, 64, 32, 64, 32, 1, 0} : GemmPlan{64, 64, 32, 32, 32, 1, 0};
  if (M <= 64) g = GemmPlan{64, 64, 32, 32, 32, 1, 0};
  if (M <= 32) g = GemmPlan{32, 128, 16, 32, 32, 1, 0};  // small M: one block row, lanes spent on j
  if (M <= 32 && N <= 64) g = GemmPlan{32, 64, 16, 32, 32, 1, 0};
  if (M > 64 && N > 64 && batch * cdiv(M, 128) * cdiv(N, 128) < 512) {
    g = GemmPlan{128, 64, 32, 64, 32, 1, 0};
    if (batch * cdiv(M, 128) * cdiv(N, 64) < 512) g = GemmPlan{64, 64, 32, 32, 32, 1, 0};
  } else if (M > 64 && N > 64) {
    // wave quantisation, as for MatMul: when the last round of 128 x 128 tiles (512 run at once)
    // would be mostly empty, the next smaller tile whose rounds fill (12 x 1000^3: 768 tiles of
    // 128 x 128, 0.289 ms; 1536 tiles of 128 x 64, 0.235 ms)
    auto poor = [](int64_t tiles, int64_t slots) {
      return (double)cdiv(tiles, slots) > 1.3 * (double)tiles / (double)slots;
    };
    if (poor(batch * cdiv(M, 128) * cdiv(N, 128), 512))
      g = poor(batch * cdiv(M, 128) * cdiv(N, 64), 768) ? GemmPlan{64, 64, 32, 32, 32, 1, 0}
                                                        : GemmPlan{128, 64, 32, 64, 32, 1, 0};
  }
  // few output tiles: parallelise the reduction dimension over workgroups (the paper's point about
  // small-M deep-learning shapes), every part keeping at least 8 k-tiles
  // short reductions: k-tiles of 16, so that the two-tile pipeline prologue stays a small share of the
  // walk (64 x 512^3: 0.140 against 0.162 ms with k-tiles of 32; equal at K = 1024)
  if (K < 1024 && g.BM >= 64) g.BK = 16;
  const int64_t tiles = batch * cdiv(M, g.BM) * cdiv(N, g.BN);
  const int64_t want = (M <= 64 || N <= 64) ? 512 : 256;
  int S = 1;
  while (tiles * S < want && S < 64 && K / (S * 2) >= 8 * g.BK) S *= 2;
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
      if (!out[i].skinny && out[i].g.BM == g.BM && out[i].g.BN == g.BN && out[i].g.BK == g.BK && out[i].g.S == g.S) return;
    out[n++] = GemmExPlan{g, (int)s[4], (int)s[5], (int)s[6]};
  };
  if (skinny_applies(s)) {
    const GemmExPlan d = ex_default(s);
    out[n++] = d;
    if (d.fused) out[n++] = skinny_plan(s, d.g.BN / 64, d.WK, d.g.S, 0);  // the same with the second kernel
    for (int wk : {16, 8})
      if (!(d.g.BN == 16 && d.WK == wk && !d.lds)) out[n++] = skinny_narrow_plan(s, wk);
    if (s[5])
      for (int wk : {8, 4})
        if (!(d.g.BN == 16 && d.WK == wk && d.lds)) out[n++] = skinny_narrow_plan(s, wk, 1);
    static const int sk_splits[] = {1, 2, 4, 8, 16, 32, 64};
    for (auto& m : kSkinnyMenu)
      for (int S : sk_splits) {
        if (n >= cap / 2) break;
        if ((m[0] == d.g.BN / 64 && m[1] == d.WK && S == d.g.S) || (S > 1 && s[3] / S < 16 * m[1])) continue;
        const int64_t waves = s[0] * cdiv(s[1], 16) * cdiv(s[2], 64) * m[1] * S;
        if (S > 1 && waves / 2 >= 16384) continue;
        out[n++] = skinny_plan(s, m[0], m[1], S);
      }
  }
  push(ex_default_tiled(s).g);
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
  if (p->blk[1] == 16) {  // the small-M kernel
    const int wn = p->prt[MDH_L_WAVE][2], wk = p->prt[MDH_L_WAVE][3];
    const bool narrow = p->prt[MDH_L_VGPR][2] == 1;
    if (s[4] || s[6] || (narrow && s[1] > 16)) return MDH_ERR_UNSUPPORTED;
    const int lds = p->in_region[1] == MDH_MR_LDS;  // narrow strips, B transposed: operands staged through LDS
    if (lds && (!narrow || !s[5] || (wk != 4 && wk != 8))) return MDH_ERR_UNSUPPORTED;
    if (narrow ? (wn != 1 || (!lds && wk != 8 && wk != 16)) : !skinny_inst(wn, wk)) return MDH_ERR_UNSUPPORTED;
    const int S = p->prt[MDH_L_WG][3];
    const int fused = p->out_region == MDH_MR_HBM;
    if (narrow && (S != 1 || fused)) return MDH_ERR_UNSUPPORTED;
    if (fused && (S <= 1 || skinny_strips(s) > kArrivalCounters)) return MDH_ERR_UNSUPPORTED;
    GemmExPlan pl = narrow ? skinny_narrow_plan(s, wk, lds) : skinny_plan(s, wn, wk, S, fused);
    mdh_tile_params chk;
    params_from_plan(s, pl, &chk);
    if (!same_table(chk, *p)) return MDH_ERR_UNSUPPORTED;
    *out = pl;
    return MDH_OK;
  }
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
