// Host-side de-composition planner: turns a configuration of the paper's tuning
// parameters (Table "Tuning parameters of our low-level expressions") into a launch
// descriptor of one of the library's kernel instantiations and back, and checks the
// algorithmic constraint of parameter 0 (prod_l #PRT(l,d) = N_d) and the model
// constraints (lanes per workgroup, LDS budget; Appendix "Constraints of Programming
// Models").  Integer arithmetic only; no GPU call in this file.
#include <string.h>

#include "mdh_internal.h"

namespace mdh {

namespace {
constexpr int kMaxLanesPerWG = 1024;        // model constraint 0 of the CUDA/OpenCL tables
constexpr int64_t kLdsBytesPerWG = 160 * 1024;  // gfx950 LDS per workgroup
}  // namespace

namespace detail {

void clear_params(mdh_tile_params* p, int D) {
  memset(p, 0, sizeof(*p));
  p->D = D;
  for (int l = 0; l < MDH_NUM_LAYERS; ++l)
    for (int d = 0; d < MDH_MAX_D; ++d) p->prt[l][d] = 1;
  for (int d = 0; d < MDH_MAX_D; ++d) p->blk[d] = 1;
}

// Fused loop order D1=S1=R1: workgroup parts outermost (one workgroup = one iteration of
// them), then the sequential HBM-layer parts, then wavefront and lane parts (parallel
// inside the workgroup), then the LDS- and VGPR-layer sequential parts; within a layer,
// dimensions in the given order.
void set_order(mdh_tile_params* p, const int* dim_order) {
  static const int layer_order[MDH_NUM_LAYERS] = {MDH_L_WG,   MDH_L_HBM, MDH_L_WAVE,
                                                  MDH_L_LANE, MDH_L_LDS, MDH_L_VGPR};
  int n = 0;
  for (int li = 0; li < MDH_NUM_LAYERS; ++li)
    for (int di = 0; di < p->D; ++di)
      p->order[n++] = (uint8_t)(layer_order[li] * MDH_MAX_D + dim_order[di]);
}

int64_t extent(const mdh_tile_params* p, int d) {
  int64_t e = p->blk[d];
  for (int l = 0; l < MDH_NUM_LAYERS; ++l) e *= p->prt[l][d];
  return e;
}

// Algorithmic constraint of parameter 0 (with the predicated-tail extension).
mdh_status check_products(const mdh_tile_params* p, const int64_t* sizes, bool* ragged) {
  *ragged = false;
  for (int d = 0; d < p->D; ++d) {
    if (p->blk[d] < 1) return MDH_ERR_TILE_NOT_DIVIDING;
    for (int l = 0; l < MDH_NUM_LAYERS; ++l)
      if (p->prt[l][d] < 1) return MDH_ERR_TILE_NOT_DIVIDING;
    const int64_t e = extent(p, d);
    if (e == sizes[d]) continue;
    if (!p->ragged || e < sizes[d]) return MDH_ERR_TILE_NOT_DIVIDING;
    *ragged = true;
  }
  return MDH_OK;
}

mdh_status check_lanes(const mdh_tile_params* p) {
  int64_t lanes = 1;
  for (int d = 0; d < p->D; ++d) lanes *= (int64_t)p->prt[MDH_L_WAVE][d] * p->prt[MDH_L_LANE][d];
  return lanes > kMaxLanesPerWG ? MDH_ERR_TILE_RESOURCES : MDH_OK;
}

// A configuration is supported iff regenerating the table from the derived launch
// descriptor reproduces it (apart from the ragged flag).
bool same_table(const mdh_tile_params& a, const mdh_tile_params& b) {
  mdh_tile_params x = a, y = b;
  x.ragged = y.ragged = 0;
  memset(x.reserved, 0, sizeof(x.reserved));
  memset(y.reserved, 0, sizeof(y.reserved));
  return memcmp(&x, &y, sizeof(x)) == 0;
}

}  // namespace detail
using namespace detail;

// =============================================================================== stencil

static bool stencil_inst(int RJ, int TY, int LK) {
  static const int menu[][3] = {{4, 2, 128}, {2, 2, 128}, {8, 2, 128}, {4, 4, 128}, {2, 4, 128},
                                {4, 1, 128}, {8, 1, 128}, {4, 4, 64},  {2, 4, 64},  {4, 2, 64},
                                {4, 8, 32},  {4, 16, 16}};
  for (auto& m : menu)
    if (m[0] == RJ && m[1] == TY && m[2] == LK) return true;
  return false;
}

int64_t stencil_lds_bytes(int RJ, int TY, int LK) {
  return 2ll * (TY * RJ + 2) * (LK * 4 + 8) * 4;
}

void params_from_plan(const int64_t* sizes, const StencilPlan& pl, mdh_tile_params* p) {
  clear_params(p, 3);
  const int TJ = pl.TY * pl.RJ, KT = pl.LK * 4;
  p->prt[MDH_L_WG][0] = (int32_t)cdiv(sizes[0], pl.SI);
  p->prt[MDH_L_WG][1] = (int32_t)cdiv(sizes[1], TJ);
  p->prt[MDH_L_WG][2] = (int32_t)cdiv(sizes[2], KT);
  p->prt[MDH_L_HBM][0] = pl.SI;
  if (pl.LK >= 64) {
    p->prt[MDH_L_WAVE][1] = pl.TY;
    p->prt[MDH_L_WAVE][2] = pl.LK / 64;
    p->prt[MDH_L_LANE][2] = 64;
  } else {  // narrow grids: a wavefront is 64/LK lane-rows of LK lanes
    p->prt[MDH_L_WAVE][1] = pl.TY * pl.LK / 64;
    p->prt[MDH_L_LANE][1] = 64 / pl.LK;
    p->prt[MDH_L_LANE][2] = pl.LK;
  }
  p->prt[MDH_L_VGPR][1] = pl.RJ;
  p->prt[MDH_L_VGPR][2] = 4;
  static const int dims[3] = {0, 1, 2};
  set_order(p, dims);
  p->strided = 0;
  p->lane_fast_dim = 2;            // k is contiguous in both buffers
  p->in_region[0] = MDH_MR_LDS;    // current plane staged in LDS
  p->out_region = MDH_MR_VGPR;     // results leave from registers
  p->ragged = (uint8_t)pl.ragged;
}

static StencilPlan stencil_default(const int64_t* s) {
  StencilPlan pl;
  pl.RJ = 4;
  pl.TY = 4;
  pl.LK = s[2] <= 256 ? 64 : 128;
  // narrow grids: fewer lanes along k, more lane-rows along j, so that no lane idles beyond nz
  // (512 x 512 x 64: 0.189 ms with 64 lanes along k against 0.069 ms for the best of those tiles)
  if (s[2] <= 128) pl.LK = 32, pl.TY = 8;
  if (s[2] <= 64) pl.LK = 16, pl.TY = 16;
  pl.SI = 64;
  // Tiles of 512 columns only where they fit nz (within 10 %); otherwise 256 columns, two rows per
  // lane and at most 32 planes per workgroup -- more and smaller workgroups, whose partly filled last
  // tile costs little.  Measured: 384^3 0.234 -> 0.111 ms; 256 x 256 x 320 0.069 -> 0.043 ms; 640^3
  // 0.563 -> 0.486 ms; 1024 x 256 x 256 0.107 -> 0.095 ms; 256^3 0.0299 -> 0.0285 ms.
  if (s[2] > 128 && (s[2] <= 256 || cdiv(s[2], 512) * 512 * 10 > s[2] * 11)) {
    pl.RJ = 2;
    pl.TY = 4;
    pl.LK = 64;
    pl.SI = 32;
  }
  const int TJ = pl.TY * pl.RJ, KT = pl.LK * 4;
  // keep at least one workgroup per compute unit when the grid is small (the four-wavefront
  // workgroups of the variant above: four per compute unit, down to 16 planes each)
  if (pl.RJ == 2)
    while (pl.SI > 16 && cdiv(s[0], pl.SI) * cdiv(s[1], TJ) * cdiv(s[2], KT) < 1024) pl.SI /= 2;
  while (pl.SI > 4 && cdiv(s[0], pl.SI) * cdiv(s[1], TJ) * cdiv(s[2], KT) < 256) pl.SI /= 2;
  if (s[0] > 0 && pl.SI > s[0]) pl.SI = (int)s[0];
  pl.ragged = (s[0] % pl.SI) || (s[1] % TJ) || (s[2] % KT);
  return pl;
}

int stencil_candidates(const int64_t* s, StencilPlan* out, int cap) {
  int n = 0;
  auto push = [&](int RJ, int TY, int LK, int SI) {
    if (n >= cap) return;
    if (s[0] > 0 && SI > s[0]) SI = (int)s[0];
    StencilPlan pl{RJ, TY, LK, SI, 0};
    pl.ragged = (s[0] % SI) || (s[1] % (TY * RJ)) || (s[2] % (LK * 4));
    for (int i = 0; i < n; ++i)
      if (out[i].RJ == RJ && out[i].TY == TY && out[i].LK == LK && out[i].SI == SI) return;
    out[n++] = pl;
  };
  StencilPlan d = stencil_default(s);
  push(d.RJ, d.TY, d.LK, d.SI);
  static const int menu[][3] = {{4, 2, 128}, {2, 2, 128}, {8, 2, 128}, {4, 4, 128}, {2, 4, 128},
                                {4, 1, 128}, {8, 1, 128}, {4, 4, 64},  {2, 4, 64},  {4, 2, 64},
                                {4, 8, 32},  {4, 16, 16}};
  static const int sis[] = {16, 32, 64, 128};
  for (auto& m : menu)
    for (int si : sis) push(m[0], m[1], m[2], si);
  return n;
}

mdh_status plan_stencil(const int64_t* s, const mdh_tile_params* p, StencilPlan* out) {
  if (!p) {
    *out = stencil_default(s);
    return MDH_OK;
  }
  if (p->D != 3) return MDH_ERR_UNSUPPORTED;
  bool ragged;
  mdh_status st = check_products(p, s, &ragged);
  if (st != MDH_OK) return st;
  if ((st = check_lanes(p)) != MDH_OK) return st;
  StencilPlan pl;
  pl.RJ = p->prt[MDH_L_VGPR][1];
  pl.TY = p->prt[MDH_L_WAVE][1] * p->prt[MDH_L_LANE][1];
  pl.LK = p->prt[MDH_L_WAVE][2] * p->prt[MDH_L_LANE][2];
  pl.SI = p->prt[MDH_L_HBM][0];
  pl.ragged = ragged;
  if (stencil_lds_bytes(pl.RJ, pl.TY, pl.LK) > kLdsBytesPerWG) return MDH_ERR_TILE_RESOURCES;
  mdh_tile_params chk;
  params_from_plan(s, pl, &chk);
  if (!same_table(chk, *p) || !stencil_inst(pl.RJ, pl.TY, pl.LK)) return MDH_ERR_UNSUPPORTED;
  *out = pl;
  return MDH_OK;
}

// =============================================================================== matmul

struct GemmInst {
  int BM, BN, BK, WM, WN;
};
static const GemmInst kGemmMenu[] = {
    {128, 128, 16, 64, 64}, {256, 128, 16, 128, 64}, {128, 64, 16, 64, 32},
    {64, 64, 16, 32, 32},   {128, 128, 32, 64, 64},  {256, 128, 32, 128, 64},
    {256, 64, 16, 64, 64},  {256, 64, 32, 64, 64},   {128, 64, 32, 64, 32},
    {128, 64, 64, 64, 32},  {256, 64, 64, 64, 64},   {64, 64, 32, 32, 32},
};

// wavefront-layer split of k: (BM, BN, WK) = workgroup tile and wavefronts along k; the 16 x 16 tile is
// one 16 x 16 x 4 block, the others are made of 32 x 32 x 2 blocks
static const int kGemmKsplitMenu[][3] = {{32, 32, 8}, {32, 32, 4}, {32, 32, 16}, {64, 32, 8}, {64, 64, 4},
                                         {64, 64, 8}, {16, 16, 4}, {16, 16, 2}, {16, 16, 8}};

static bool gemm_inst(const GemmPlan& pl) {
  if (pl.WK > 1) {
    for (auto& m : kGemmKsplitMenu)
      if (pl.BM == m[0] && pl.BN == m[1] && pl.WK == m[2]) return true;
    return false;
  }
  for (auto& m : kGemmMenu)
    if (m.BM == pl.BM && m.BN == pl.BN && m.BK == pl.BK && m.WM == pl.WM && m.WN == pl.WN)
      return true;
  return false;
}

int64_t gemm_lds_bytes(int BM, int BN, int BK) {
  // two stages of an A tile [BM][BK+4] and a B tile [BK][BN+4]
  return 2ll * ((int64_t)BM * (BK + 4) + (int64_t)BK * (BN + 4)) * 4;
}

void params_from_plan(const int64_t* s, const GemmPlan& pl, mdh_tile_params* p) {
  clear_params(p, 3);
  p->blk[0] = 32;
  p->blk[1] = 32;
  p->blk[2] = 2;  // one v_mfma_f32_32x32x2_f32
  if (pl.WK > 1) {
    // k on the wavefront layer: every wavefront owns the whole tile and walks groups of 8 k (4 MFMA
    // steps of 2; with the 16 x 16 x 4 block: groups of 16 k, 4 steps of 4) read straight into
    // registers; the wavefront results are combined in LDS
    const int b = pl.BM == 16 ? 16 : 32, bk = pl.BM == 16 ? 4 : 2;
    p->blk[0] = p->blk[1] = b;
    p->blk[2] = bk;
    p->prt[MDH_L_WG][0] = (int32_t)cdiv(s[0], pl.BM);
    p->prt[MDH_L_WG][1] = (int32_t)cdiv(s[1], pl.BN);
    p->prt[MDH_L_WG][2] = pl.S;
    p->prt[MDH_L_WAVE][2] = pl.WK;
    p->prt[MDH_L_HBM][2] = (int32_t)cdiv(cdiv(s[2], (int64_t)pl.S * pl.WK), 4 * bk);
    p->prt[MDH_L_VGPR][0] = pl.BM / b;
    p->prt[MDH_L_VGPR][1] = pl.BN / b;
    p->prt[MDH_L_VGPR][2] = 4;
    static const int kdims[3] = {0, 1, 2};
    set_order(p, kdims);
    p->strided = 0;
    p->lane_fast_dim = 1;
    p->in_region[0] = MDH_MR_VGPR;
    p->in_region[1] = MDH_MR_VGPR;
    p->out_region = MDH_MR_LDS;
    p->ragged = (uint8_t)pl.ragged;
    return;
  }
  p->prt[MDH_L_WG][0] = (int32_t)cdiv(s[0], pl.BM);
  p->prt[MDH_L_WG][1] = (int32_t)cdiv(s[1], pl.BN);
  p->prt[MDH_L_WG][2] = pl.S;
  p->prt[MDH_L_HBM][2] = (int32_t)cdiv(cdiv(s[2], pl.S), pl.BK);
  p->prt[MDH_L_WAVE][0] = pl.BM / pl.WM;
  p->prt[MDH_L_WAVE][1] = pl.BN / pl.WN;
  p->prt[MDH_L_LDS][2] = pl.BK / 2;
  p->prt[MDH_L_VGPR][0] = pl.WM / 32;
  p->prt[MDH_L_VGPR][1] = pl.WN / 32;
  static const int dims[3] = {0, 1, 2};
  set_order(p, dims);
  if (pl.jmajor) {  // workgroup layer: j before i
    p->order[0] = (uint8_t)(MDH_L_WG * MDH_MAX_D + 1);
    p->order[1] = (uint8_t)(MDH_L_WG * MDH_MAX_D + 0);
  }
  p->strided = 0;
  p->lane_fast_dim = 1;
  p->in_region[0] = MDH_MR_LDS;
  p->in_region[1] = MDH_MR_LDS;
  p->out_region = MDH_MR_VGPR;
  p->ragged = (uint8_t)pl.ragged;
}

static int gemm_ragged(const int64_t* s, const GemmPlan& pl) {
  if (pl.WK > 1) return (s[0] % pl.BM) || (s[1] % pl.BN) || (s[2] % ((int64_t)pl.S * pl.WK * (pl.BM == 16 ? 16 : 8)));
  return (s[0] % pl.BM) || (s[1] % pl.BN) || (s[2] % ((int64_t)pl.S * pl.BK));
}

static GemmPlan gemm_default(const int64_t* s) {
  const int64_t M = s[0], N = s[1], K = s[2];
  // Outputs of few tiles: k over the wavefronts of a workgroup, one launch, tiles small enough to give
  // every compute unit a workgroup.  Kernel durations (rocprofv3 kernel trace, us; the LDS-tiled kernel
  // with 64 x 64 tiles beside it, second pass included where it splits k):
  //   128^3: 2.9 (16 x 16 tiles, 2 wavefronts) / 5.1      256^3: 3.3 (16 x 16, 4) / 8.4
  //   200 x 300 x 500: 5.1 (16 x 16, 4) / 8.6             256 x 256 x 4096: 13.7 (16 x 16, 4) / 15.3
  //   384^3: 5.5 (32 x 32, 4) / 7.5                       512^3: 6.5 (32 x 32, 4) / 9.9
  //   768^3 and 1024^3: the LDS-tiled kernel stays ahead (18.9 against 20.0; 26.3 against 28.1)
  if (K >= 32 && K <= 8192 && M > 0 && N > 0) {
    const int64_t t16 = cdiv(M, 16) * cdiv(N, 16), t32 = cdiv(M, 32) * cdiv(N, 32);
    if (t16 <= 320 || t32 <= 320) {
      const int b = t16 <= 320 ? 16 : 32;
      GemmPlan pl{b, b, b == 16 ? 16 : 8, b, b, 1, 0};
      pl.WK = (b == 16 && K <= 128) ? 2 : 4;
      pl.ragged = gemm_ragged(s, pl);
      return pl;
    }
  }
  // Tile: the largest of 128x128, 128x64, 64x64 that still gives two workgroups per compute unit
  // (measured best at 4096^3, 2048^3 and 1024^3 respectively); narrow problems keep 128x64 / 64x64.
  GemmPlan pl{128, 128, 32, 64, 64, 1, 0};
  const bool narrow = N <= 64 || M <= 64;
  if (narrow) {
    // one tile spans the short dimension.  Measured (65536 x 64 x 4096 / 16384 x 64 x 4096 /
    // 64 x 65536 x 1024): 128x64 tiles only where they still give two workgroups per compute unit
    // (0.312 against 0.327 ms), 64x64 tiles otherwise (0.085 against 0.088 ms; 0.087 against 0.19 ms
    // when M = 64 would leave half of a 128-row tile empty)
    pl = GemmPlan{64, 64, 32, 32, 32, 1, 0};
    if (M > 64 && cdiv(M, 128) * cdiv(N, 64) >= 512) pl = GemmPlan{128, 64, 32, 64, 32, 1, 0};
  } else if (cdiv(M, 128) * cdiv(N, 128) < 512) {
    pl = GemmPlan{128, 64, 32, 64, 32, 1, 0};
    if (cdiv(M, 128) * cdiv(N, 64) < 512) pl = GemmPlan{64, 64, 32, 32, 32, 1, 0};
  } else {
    // wave quantisation: 512 tiles of 128 x 128 run at once; when the last round would be mostly
    // empty the 64 x 64 tile (about 0.8 of the rate, but four times the tiles) is faster.  Measured:
    // 3000^3 (576 tiles) 0.66 -> 0.52 ms; 4100 x 4096 x 4096 (1056 tiles) 1.32 -> 1.18 ms.
    const double rounds = (double)(cdiv(M, 128) * cdiv(N, 128)) / 512.0;
    const double whole = (double)cdiv(cdiv(M, 128) * cdiv(N, 128), 512);
    if (whole > 1.3 * rounds) pl = GemmPlan{64, 64, 32, 32, 32, 1, 0};
  }
  // Split the reduction dimension over workgroups only while there is less than one workgroup per
  // compute unit (two for the narrow shapes, whose tiles are small) AND every part keeps at least 8
  // k-tiles: below that the second pass and the shortened pipelines cost more than the parallelism
  // gains (256^3 is fastest unsplit, 8.7 us against 14.6 us with 16 parts; 256 x 256 x 4096 is
  // fastest with 16 parts; 8192 x 64 x 4096 with 4 parts: 0.046 against 0.089 ms unsplit).
  const int64_t tiles = cdiv(M, pl.BM) * cdiv(N, pl.BN);
  const int64_t want = narrow ? 512 : 256;
  int S = 1;
  while (tiles * S < want && S < 64 && K / (S * 2) >= 8 * pl.BK) S *= 2;
  // beyond 64 parts only while a part keeps 2048 elements of k (64 x 64 x 2^20: 0.22 ms with 256
  // parts against 0.55 ms with 64; 32 x 32 x 65536 is fastest with 64)
  while (tiles * S < want && S >= 64 && S < 256 && K / (S * 2) >= 2048) S *= 2;
  pl.S = S;
  pl.ragged = gemm_ragged(s, pl);
  return pl;
}

int matmul_candidates(const int64_t* s, GemmPlan* out, int cap) {
  int n = 0;
  auto push = [&](GemmPlan pl) {
    if (n >= cap) return;
    if (pl.S > 1 && s[2] / pl.S < pl.BK) return;
    if (pl.WK == 1 && gemm_lds_bytes(pl.BM, pl.BN, pl.BK) > kLdsBytesPerWG) return;
    pl.ragged = gemm_ragged(s, pl);
    for (int i = 0; i < n; ++i)
      if (out[i].BM == pl.BM && out[i].BN == pl.BN && out[i].BK == pl.BK && out[i].WM == pl.WM &&
          out[i].S == pl.S && out[i].WK == pl.WK && out[i].jmajor == pl.jmajor)
        return;
    out[n++] = pl;
  };
  push(gemm_default(s));
  {  // the default's tile with the other loop order of the workgroup layer (column bands)
    GemmPlan d = gemm_default(s);
    if (d.WK == 1 && cdiv(s[0], d.BM) > 1 && cdiv(s[1], d.BN) > 1) {
      d.jmajor = !d.jmajor;
      push(d);
    }
  }
  // k over the wavefronts of a workgroup, for outputs of few tiles (every wavefront keeps 8 k or more)
  if (cdiv(s[0], 32) * cdiv(s[1], 32) <= 1024)
    for (auto& m : kGemmKsplitMenu)
      for (int S : {1, 2, 4}) {
        if (s[2] / ((int64_t)S * m[2]) < 16) continue;
        if (S > 1 && cdiv(s[0], m[0]) * cdiv(s[1], m[1]) * (S / 2) >= 256) continue;
        if (m[0] == 16 && cdiv(s[0], 16) * cdiv(s[1], 16) > 1024) continue;
        GemmPlan pl{m[0], m[1], m[0] == 16 ? 16 : 8, m[0], m[1], S, 0};
        pl.WK = m[2];
        push(pl);
      }
  static const int splits[] = {1, 2, 4, 8, 16};
  for (auto& m : kGemmMenu)
    for (int S : splits) {
      const int64_t tiles = cdiv(s[0], m.BM) * cdiv(s[1], m.BN);
      if (S > 1 && tiles * (S / 2) >= 2048) continue;  // splitting a full grid only adds traffic
      push(GemmPlan{m.BM, m.BN, m.BK, m.WM, m.WN, S, 0});
    }
  return n;
}

mdh_status plan_matmul(const int64_t* s, const mdh_tile_params* p, GemmPlan* out) {
  if (!p) {
    *out = gemm_default(s);
    return MDH_OK;
  }
  if (p->D != 3) return MDH_ERR_UNSUPPORTED;
  bool ragged;
  mdh_status st = check_products(p, s, &ragged);
  if (st != MDH_OK) return st;
  if ((st = check_lanes(p)) != MDH_OK) return st;
  if (p->prt[MDH_L_WAVE][2] > 1) {
    // wavefront-layer parts of k: the register-streaming kernel
    GemmPlan pl;
    const bool b16 = p->blk[0] == 16;
    if (!((p->blk[0] == 32 && p->blk[1] == 32 && p->blk[2] == 2) || (b16 && p->blk[1] == 16 && p->blk[2] == 4)))
      return MDH_ERR_UNSUPPORTED;
    pl.BM = pl.WM = p->prt[MDH_L_VGPR][0] * p->blk[0];
    pl.BN = pl.WN = p->prt[MDH_L_VGPR][1] * p->blk[1];
    pl.BK = b16 ? 16 : 8;
    pl.S = p->prt[MDH_L_WG][2];
    pl.WK = p->prt[MDH_L_WAVE][2];
    pl.ragged = ragged;
    // model constraints: lanes per workgroup, and the LDS that holds the WK partial tiles
    if ((int64_t)pl.WK * 64 > kMaxLanesPerWG) return MDH_ERR_TILE_RESOURCES;
    if ((int64_t)pl.WK * pl.BM * pl.BN * 4 > kLdsBytesPerWG) return MDH_ERR_TILE_RESOURCES;
    mdh_tile_params chk;
    params_from_plan(s, pl, &chk);
    if (!same_table(chk, *p) || !gemm_inst(pl)) return MDH_ERR_UNSUPPORTED;
    *out = pl;
    return MDH_OK;
  }
  GemmPlan pl;
  pl.WM = p->prt[MDH_L_VGPR][0] * 32;
  pl.WN = p->prt[MDH_L_VGPR][1] * 32;
  pl.BM = p->prt[MDH_L_WAVE][0] * pl.WM;
  pl.BN = p->prt[MDH_L_WAVE][1] * pl.WN;
  pl.BK = p->prt[MDH_L_LDS][2] * 2;
  pl.S = p->prt[MDH_L_WG][2];
  pl.ragged = ragged;
  // parameter D1 on the workgroup layer: (WG,j) before (WG,i) selects the column-band tile order; any
  // other permutation has no instantiation (the regenerated table below differs)
  pl.jmajor = (p->order[0] == MDH_L_WG * MDH_MAX_D + 1 && p->order[1] == MDH_L_WG * MDH_MAX_D + 0) ? 1 : 0;
  if (p->blk[0] != 32 || p->blk[1] != 32 || p->blk[2] != 2) return MDH_ERR_UNSUPPORTED;
  if (gemm_lds_bytes(pl.BM, pl.BN, pl.BK) > kLdsBytesPerWG) return MDH_ERR_TILE_RESOURCES;
  if ((int64_t)p->prt[MDH_L_WAVE][0] * p->prt[MDH_L_WAVE][1] * 64 > kMaxLanesPerWG)
    return MDH_ERR_TILE_RESOURCES;
  mdh_tile_params chk;
  params_from_plan(s, pl, &chk);
  if (!same_table(chk, *p) || !gemm_inst(pl)) return MDH_ERR_UNSUPPORTED;
  *out = pl;
  return MDH_OK;
}

// ---- MatMul with few rows: the small-M kernel of the batched instance, one batch entry

bool small_m_matmul(const int64_t* s, const mdh_tile_params* p) {
  if (!p) return s[0] > 0 && s[0] <= 16 && s[1] > 0;
  // both strip widths of that kernel (64 or 16 columns per wavefront); the kernel that splits k over
  // wavefronts has 16 x 16 x 4 blocks too, but combines in LDS
  return p->D == 3 && p->blk[0] == 16 && (p->prt[MDH_L_VGPR][1] == 4 || p->out_region != MDH_MR_LDS);
}

static void move_dims(const mdh_tile_params& src, mdh_tile_params* dst, int D, int shift) {
  // dimension d of dst is dimension d + shift of src (shift = 1 drops the batch, -1 inserts it)
  clear_params(dst, D);
  for (int d = 0; d < D; ++d) {
    const int e = d + shift;
    if (e < 0 || e >= src.D) continue;  // the inserted batch dimension: one part everywhere, blk 1
    dst->blk[d] = src.blk[e];
    for (int l = 0; l < MDH_NUM_LAYERS; ++l) dst->prt[l][d] = src.prt[l][e];
  }
  int dims[MDH_MAX_D];
  for (int d = 0; d < D; ++d) dims[d] = d;
  set_order(dst, dims);
  dst->strided = src.strided;
  dst->lane_fast_dim = (uint8_t)(src.lane_fast_dim - shift);
  dst->ragged = src.ragged;
  memcpy(dst->in_region, src.in_region, sizeof(src.in_region));
  dst->out_region = src.out_region;
  memcpy(dst->in_transposed, src.in_transposed, sizeof(src.in_transposed));
  dst->out_transposed = src.out_transposed;
}

void lift_batch(const mdh_tile_params& p3, mdh_tile_params* p4) { move_dims(p3, p4, 4, -1); }
void drop_batch(const mdh_tile_params& p4, mdh_tile_params* p3) { move_dims(p4, p3, 3, 1); }

// the batched instance's view of a small-M MatMul call: sizes and (if given) the lifted table
static mdh_status plan_small_m(const int64_t* s, const mdh_tile_params* p, GemmExPlan* out) {
  const int64_t s4[7] = {1, s[0], s[1], s[2], 0, 0, 0};
  if (!p) return plan_matmul_ex(s4, nullptr, out);
  mdh_tile_params p4;
  lift_batch(*p, &p4);
  // the order entries of the caller's table must be the ones this library generates
  mdh_tile_params back;
  drop_batch(p4, &back);
  if (!same_table(back, *p)) return MDH_ERR_UNSUPPORTED;
  return plan_matmul_ex(s4, &p4, out);
}

mdh_status plan_matmul_small_m(const int64_t* s, const mdh_tile_params* p, GemmExPlan* out) {
  return plan_small_m(s, p, out);
}

// =============================================================================== MCC

int64_t mcc_flat_lds_bytes(int QB, int TP, int BN, int64_t C, int64_t R, int64_t S, int64_t sh, int64_t sw);

struct MccInst {
  int TP, TQ, BN, CK, WM, WN;
};
static const MccInst kMccMenu[] = {  // channel-chunked kernel
    {4, 32, 128, 16, 64, 64},
    {8, 32, 128, 16, 128, 64},
    {2, 32, 64, 16, 32, 32},
    {4, 32, 64, 16, 64, 32},
    {8, 16, 128, 16, 64, 64},  // blocks of 2 x 16 pixels (images narrower than 32 output columns)
    {8, 16, 64, 16, 64, 32},
    {8, 8, 128, 16, 32, 64},   // blocks of 4 x 8 pixels
    {8, 8, 64, 16, 32, 32},
    {4, 32, 128, 32, 64, 64},  // channel chunks of 32: twice the MFMAs between two barriers
    {4, 32, 64, 32, 64, 32},
    {8, 16, 128, 32, 64, 64},
    {8, 16, 64, 32, 64, 32},
    {8, 8, 128, 32, 32, 64},
    {8, 8, 64, 32, 32, 32},
};
// few-channel kernel (s and c fused): TP rows x TQ = QB columns of pixels, BN channels, WM, WN
static const MccInst kMccFlatMenu[] = {
    {8, 16, 64, 0, 32, 64},  {4, 32, 64, 0, 32, 64},   {8, 16, 32, 0, 32, 32},
    {4, 32, 32, 0, 32, 32},  {8, 16, 128, 0, 64, 64},  {4, 32, 128, 0, 64, 64},
    {8, 16, 64, 0, 32, 32},  {4, 32, 64, 0, 32, 32},   {16, 16, 32, 0, 32, 32},  {8, 32, 32, 0, 32, 32},  // eight wavefronts
};

static bool mcc_inst(const MccPlan& pl) {
  const MccInst* menu = pl.flat ? kMccFlatMenu : kMccMenu;
  const int n = pl.flat ? (int)(sizeof(kMccFlatMenu) / sizeof(MccInst)) : (int)(sizeof(kMccMenu) / sizeof(MccInst));
  for (int i = 0; i < n; ++i) {
    const MccInst& m = menu[i];
    if (m.TP == pl.TP && m.TQ == pl.TQ && m.BN == pl.BN && m.CK == pl.CK && m.WM == pl.WM && m.WN == pl.WN)
      return true;
  }
  return false;
}

// sizes: N, P, Q, K, C, R, S, stride_h, stride_w
int64_t mcc_lds_bytes(const MccPlan& pl, const int64_t* s) {
  if (pl.flat) return mcc_flat_lds_bytes(pl.TQ, pl.TP, pl.BN, s[4], s[5], s[6], s[7], s[8]);
  const int64_t ph = (pl.TP - 1) * s[7] + s[5], pw = (pl.TQ - 1) * s[8] + s[6];
  return (ph * pw * (pl.CK + 4) + 2ll * pl.BN * (pl.CK + 4)) * 4;
}

void params_from_plan(const int64_t* s, const MccPlan& pl, mdh_tile_params* p) {
  // dims: 0 n, 1 p, 2 q, 3 k, 4 c, 5 r, 6 s
  clear_params(p, 7);
  p->prt[MDH_L_WG][0] = (int32_t)s[0];
  p->prt[MDH_L_WG][1] = (int32_t)cdiv(s[1], pl.TP);
  p->prt[MDH_L_WG][2] = (int32_t)cdiv(cdiv(s[2], pl.TQ), pl.flat ? pl.QT : 1);
  p->prt[MDH_L_WG][3] = (int32_t)cdiv(s[3], pl.BN);
  if (pl.flat) p->prt[MDH_L_HBM][2] = pl.QT;  // column tiles walked with the filter slice resident
  p->prt[MDH_L_LDS][5] = (int32_t)s[5];
  p->prt[MDH_L_LDS][6] = (int32_t)s[6];
  p->prt[MDH_L_WAVE][3] = pl.BN / pl.WN;
  p->prt[MDH_L_VGPR][3] = pl.WN / 32;
  p->blk[3] = 32;  // 32 output channels
  if (pl.flat) {
    // few channels: the block is (32/QB rows of p) x (QB consecutive q); s and c are walked as one
    // sequential LDS-layer dimension of S*C single steps (two of them feed one MFMA)
    const int rb = 32 / pl.TQ, mi = pl.WM / 32;
    p->blk[1] = rb;
    p->blk[2] = pl.TQ;
    p->prt[MDH_L_LDS][4] = (int32_t)s[4];
    p->prt[MDH_L_WAVE][1] = pl.TP / (rb * mi);
    p->prt[MDH_L_VGPR][1] = mi;
  } else {
    // the block: 32 pixels = (32/TQ rows of p) x (TQ consecutive q), 2 input channels per MFMA
    const int rb = 32 / pl.TQ, mi = pl.WM / 32;
    p->blk[1] = rb;
    p->blk[2] = pl.TQ;
    p->blk[4] = 2;
    p->prt[MDH_L_WG][4] = pl.S;  // parts of the reduction dimension c over workgroups
    p->prt[MDH_L_HBM][4] = (int32_t)cdiv(cdiv(s[4], pl.S), pl.CK);
    p->prt[MDH_L_LDS][4] = pl.CK / 2;
    // wavefront grid: TP/(mi*rb) along p, BN/WN along k; mi blocks along p per wavefront
    p->prt[MDH_L_WAVE][1] = pl.TP / (mi * rb);
    p->prt[MDH_L_VGPR][1] = mi;
  }
  static const int dims[7] = {0, 1, 2, 3, 4, 5, 6};
  set_order(p, dims);
  // few-channel kernel: 0 = a workgroup owns a run of column tiles, 1 = the tiles of (n, p, q) are dealt
  // out one at a time to the workgroups resident on the chip
  p->strided = (pl.flat && pl.dealt) ? 1 : 0;
  p->lane_fast_dim = 3;
  p->in_region[0] = MDH_MR_LDS;
  p->in_region[1] = MDH_MR_LDS;
  p->out_region = MDH_MR_VGPR;
  p->ragged = (uint8_t)pl.ragged;
}

static int mcc_ragged(const int64_t* s, const MccPlan& pl) {
  if (pl.flat) return (s[1] % pl.TP) || (s[2] % ((int64_t)pl.TQ * pl.QT)) || (s[3] % pl.BN);
  return (s[1] % pl.TP) || (s[2] % pl.TQ) || (s[3] % pl.BN) || (s[4] % ((int64_t)pl.S * pl.CK));
}

// Column tiles per workgroup of the few-channel kernel: at most `want`, fewer while the grid would
// drop below one workgroup per compute unit; normalised so that no workgroup is without a tile.
static int flat_qt(const int64_t* s, const MccPlan& pl, int want, int min_wgs = 256) {
  const int64_t tiles = cdiv(s[2] > 0 ? s[2] : 1, pl.TQ);
  const int64_t other = (s[0] > 0 ? s[0] : 1) * cdiv(s[1] > 0 ? s[1] : 1, pl.TP) * cdiv(s[3] > 0 ? s[3] : 1, pl.BN);
  int64_t qt = want < tiles ? want : tiles;
  while (qt > 1 && other * cdiv(tiles, qt) < min_wgs) qt = cdiv(qt, 2);
  return (int)cdiv(tiles, cdiv(tiles, qt));
}

static MccPlan mcc_flat_plan(const int64_t* s) {
  // Measured on the first-layer shapes of ResNet-50, VGG-16 and MobileNet: 32 channels per
  // workgroup up to K = 64 (more workgroups, each stages a smaller filter slice; a lane stores 16
  // bytes of a pixel, so narrow channel slices still write whole 128-byte lines), a workgroup keeps
  // its filter slice and walks up to 8 column tiles (ResNet-50: 56 us against 64 us with one tile;
  // VGG-16: 66 us against 80 us with 64 channels), blocks of 8 x 16 pixels where 16 divides Q and
  // 32 does not (Q = 112), of 4 x 32 pixels otherwise.
  // Where the grid is large enough, eight wavefronts per workgroup -- two along k from 64 channels
  // on (they share one input patch), otherwise all along p -- blocks of 8 x 16 pixels, and up to 16
  // column tiles per workgroup while 192 workgroups remain.  Candidates measured in alternation
  // (medians): VGG-16 first layer, N = 16: 67.7 us against 71.2 us for the rule below; MobileNet:
  // 18.9 against 19.2 us; ResNet-50, N = 4: 20.0 against 21.7 us; N = 16 and 32: equal to the rule
  // below at 32 channels per workgroup (54.1 us, 89 us), one patch staging instead of two; with
  // N = 1 the four-wavefront workgroups below stay faster (10.0 against 11.4 us).
  {
    MccPlan w = s[3] > 32 ? MccPlan{8, 16, 64, 0, 32, 32, 0, 1} : MccPlan{16, 16, 32, 0, 32, 32, 0, 1};
    const int64_t wgs = (s[0] > 0 ? s[0] : 1) * cdiv(s[1] > 0 ? s[1] : 1, w.TP) * cdiv(s[2] > 0 ? s[2] : 1, w.TQ) *
                        cdiv(s[3] > 0 ? s[3] : 1, w.BN);
    if (wgs >= 256 && mcc_lds_bytes(w, s) <= kLdsBytesPerWG) {
      // Long walks per tile (ResNet-50's 7 x 7 filter: 21 steps of 8; the 3 x 3 filters have 6): tiles of
      // 16 x 16 pixels x 32 channels dealt out to resident workgroups instead of owned -- every compute
      // unit stays busy to the end and two workgroups per unit cover each other's tile hand-over.
      // ResNet-50 first layer, N = 16: 46.9 against 55.3 us; N = 32: 81 against 96 us; N = 4: 17.4 against
      // 19.1 us.  VGG-16 (70 against 81 us) and MobileNet (16.5 against 16.9 us) stay with owned tiles.
      MccPlan d{16, 16, 32, 0, 32, 32, 0, 1};
      d.dealt = 1;
      if (s[5] * cdiv(s[6] * s[4], 8) >= 16 && cdiv(s[3] > 0 ? s[3] : 1, d.BN) <= 8 && mcc_lds_bytes(d, s) <= kLdsBytesPerWG) {
        d.ragged = mcc_ragged(s, d);
        return d;
      }
      w.QT = flat_qt(s, w, 16, 192);
      w.ragged = mcc_ragged(s, w);
      return w;
    }
  }
  const int qb = (s[2] % 32 != 0 && s[2] % 16 == 0) ? 16 : 32;
  const int tp = qb == 16 ? 8 : 4;
  MccPlan pl{tp, qb, 32, 0, 32, 32, 0, 1};
  if (s[3] > 64) pl = MccPlan{tp, qb, 64, 0, 32, 64, 0, 1};
  pl.QT = flat_qt(s, pl, 8);
  pl.ragged = mcc_ragged(s, pl);
  return pl;
}

// The few-channel kernel reads its input in 16-byte pieces and needs an input of at least four elements;
// the smallest input these output sizes can have is N x ((P-1) sh + R) x ((Q-1) sw + S) x C.
static bool flat_input_ok(const int64_t* s) {
  return (s[0] > 0 ? s[0] : 1) * ((s[1] > 0 ? s[1] - 1 : 0) * s[7] + s[5]) * ((s[2] > 0 ? s[2] - 1 : 0) * s[8] + s[6]) * s[4] >= 4;
}

static MccPlan mcc_default(const int64_t* s) {
  if (s[4] <= 8 && flat_input_ok(s)) {  // fewer channels than half a channel chunk: fuse s and c
    MccPlan f = mcc_flat_plan(s);
    if (mcc_lds_bytes(f, s) <= kLdsBytesPerWG) return f;
  }
  // Pixel block: 32 consecutive q of one row, 2 x 16 or 4 x 8 pixels -- the shape whose tiles (4 x 32,
  // 8 x 16, 8 x 8 pixels) pad the image least; on a tie the widest.  Squarer tiles also stage less
  // halo.  Measured against blocks of 32 columns throughout: 32 x 112 x 112 x 64 -> 32, 3 x 3: 0.144
  // against 0.191 ms; 16 x 56 x 56, 1 x 1, 256 -> 64 / 64 -> 256: 28 / 32 us against 41 / 55 us;
  // 16 x 14 x 14 x 256 -> 256, 3 x 3: 122 against 137 us.
  const int64_t P = s[1] > 0 ? s[1] : 1, Q = s[2] > 0 ? s[2] : 1;
  // (on a tie the widest that still gives two workgroups per compute unit at 64 channels per
  // workgroup and with c split as far as it goes, else the narrowest)
  int tq = 32, tp = 4;
  int64_t area = -1;
  bool enough = false;
  for (int t : {32, 16, 8}) {
    const int rows = t == 32 ? 4 : 8;
    const int64_t a = cdiv(P, rows) * rows * cdiv(Q, t) * t;
    int smax = 1;  // parts the reduction dimension c can be split into (at least one chunk each)
    while (smax < 8 && s[4] / (2 * smax) >= 16) smax *= 2;
    const bool many = (s[0] > 0 ? s[0] : 1) * cdiv(P, rows) * cdiv(Q, t) * cdiv(s[3] > 0 ? s[3] : 1, 64) * smax >= 512;
    if (area < 0 || a < area || (a == area && !enough)) area = a, tq = t, tp = rows, enough = many;
  }
  const int wm = tq == 8 ? 32 : 64;  // two blocks along p per wavefront, one for the 4 x 8 block
  MccPlan pl{tp, tq, 128, 16, wm, 64, 0, 0};
  if (s[3] <= 64) pl = MccPlan{tp, tq, 64, 16, wm, 32, 0, 0};
  // small images: narrower channel slices when there are fewer than two workgroups per compute unit
  // (16 x 28 x 28 x 128 -> 128, 3 x 3: 76 us against 124 us; 7 x 7 x 512: 283 against 462 us; fewer
  // rows per workgroup on top of that measured slower)
  auto wgs = [&](const MccPlan& m) {
    return (s[0] > 0 ? s[0] : 1) * cdiv(P, m.TP) * cdiv(Q, m.TQ) * cdiv(s[3] > 0 ? s[3] : 1, m.BN);
  };
  if (wgs(pl) < 512 && pl.BN == 128) pl = MccPlan{tp, tq, 64, 16, wm, 32, 0, 0};
  // still few workgroups: parts of the reduction dimension c over workgroups (partial outputs in the
  // workspace + second pass) up to ~450 workgroups, every part keeping at least one channel chunk.
  // 16 x 7 x 7 x 512 -> 512, 3 x 3: 85 us with 4 or 8 parts, 137 us with 2, 267 us unsplit (MIOpen
  // 118 us); 16 x 14 x 14 x 256 -> 256: 68 us with 4 parts, 80 with 2, 143 unsplit; 16 x 28 x 28 x 128
  // -> 128: 69 us with 2 parts, 73 with 4, 75 unsplit; 1 x 28 x 28 x 128: 15 us with 8 parts, 41 with 2.
  while (wgs(pl) * pl.S < 448 && pl.S < 8 && s[4] / (2 * pl.S) >= pl.CK) pl.S *= 2;
  // many channels per part: chunks of 32 channels, twice the MFMAs between two barriers (16 x 14 x 14
  // x 256 -> 256: 55.5 against 58.8 us; 16 x 7 x 7 x 2048 -> 512, 1 x 1: 37.5 against 44.3 us; with 32
  // channels in all, or 7 x 7 taps on 64, chunks of 16 are as fast or faster)
  if (s[4] / pl.S >= 128 || (s[4] / pl.S >= 64 && s[5] * s[6] <= 9)) {
    MccPlan w = pl;
    w.CK = 32;
    if (mcc_lds_bytes(w, s) <= kLdsBytesPerWG) pl = w;
  }
  // parts are whole channel chunks: no part may end up without channels (e.g. 200 channels in 8 parts)
  while (pl.S > 1 && (int64_t)(pl.S - 1) * cdiv(cdiv(s[4], pl.S), pl.CK) * pl.CK >= s[4]) pl.S /= 2;
  pl.ragged = mcc_ragged(s, pl);
  return pl;
}

int mcc_candidates(const int64_t* s, MccPlan* out, int cap) {
  int n = 0;
  auto push = [&](MccPlan pl) {
    if (n >= cap) return;
    if (mcc_lds_bytes(pl, s) > kLdsBytesPerWG) return;
    pl.ragged = mcc_ragged(s, pl);
    for (int i = 0; i < n; ++i)
      if (out[i].flat == pl.flat && out[i].TP == pl.TP && out[i].TQ == pl.TQ && out[i].BN == pl.BN && out[i].CK == pl.CK &&
          out[i].WM == pl.WM && out[i].WN == pl.WN && out[i].QT == pl.QT && out[i].S == pl.S && out[i].dealt == pl.dealt)
        return;
    out[n++] = pl;
  };
  push(mcc_default(s));
  for (auto& m : kMccMenu) push(MccPlan{m.TP, m.TQ, m.BN, m.CK, m.WM, m.WN, 0, 0});
  // the reduction dimension c over workgroups, where the concatenation dimensions leave the chip empty
  for (int S : {2, 4, 8})
    for (auto& m : kMccMenu) {
      MccPlan pl{m.TP, m.TQ, m.BN, m.CK, m.WM, m.WN, 0, 0};
      pl.S = S;
      const int64_t wg = (s[0] > 0 ? s[0] : 1) * cdiv(s[1] > 0 ? s[1] : 1, m.TP) * cdiv(s[2] > 0 ? s[2] : 1, m.TQ) *
                         cdiv(s[3] > 0 ? s[3] : 1, m.BN);
      if (wg * (S / 2) >= 1024 || (int64_t)(S - 1) * cdiv(cdiv(s[4], S), m.CK) * m.CK >= s[4]) continue;
      push(pl);
    }
  if (s[4] <= 16 && flat_input_ok(s))
    for (int want : {1, 2, 4, 8, 16})
      for (auto& m : kMccFlatMenu) {
        MccPlan pl{m.TP, m.TQ, m.BN, m.CK, m.WM, m.WN, 0, 1};
        const int64_t tiles = cdiv(s[2] > 0 ? s[2] : 1, pl.TQ);
        const int64_t qt = want < tiles ? want : tiles;
        pl.QT = (int)cdiv(tiles, cdiv(tiles, qt));
        push(pl);
        if (want == 1 && cdiv(s[3] > 0 ? s[3] : 1, pl.BN) <= 8) {  // the same tile, dealt out
          pl.dealt = 1;
          push(pl);
        }
      }
  return n;
}

mdh_status plan_mcc(const int64_t* s, const mdh_tile_params* p, MccPlan* out) {
  if (!p) {
    *out = mcc_default(s);
    if (mcc_lds_bytes(*out, s) > kLdsBytesPerWG) return MDH_ERR_TILE_RESOURCES;
    return MDH_OK;
  }
  if (p->D != 7) return MDH_ERR_UNSUPPORTED;
  bool ragged;
  mdh_status st = check_products(p, s, &ragged);
  if (st != MDH_OK) return st;
  if ((st = check_lanes(p)) != MDH_OK) return st;
  MccPlan pl;
  pl.flat = p->blk[4] == 1 ? 1 : 0;
  pl.WN = p->prt[MDH_L_VGPR][3] * 32;
  pl.BN = p->prt[MDH_L_WAVE][3] * pl.WN;
  if (pl.flat) {
    pl.TQ = p->blk[2];
    if ((pl.TQ != 16 && pl.TQ != 32) || !flat_input_ok(s)) return MDH_ERR_UNSUPPORTED;
    pl.WM = p->prt[MDH_L_VGPR][1] * 32;
    pl.TP = p->prt[MDH_L_WAVE][1] * p->prt[MDH_L_VGPR][1] * (32 / pl.TQ);
    pl.CK = 0;
    pl.QT = p->prt[MDH_L_HBM][2];
    pl.dealt = p->strided ? 1 : 0;
    // dealt tiles: one column tile per part, at most 8 filter slices (one ticket counter each)
    if (pl.dealt && (pl.QT != 1 || p->prt[MDH_L_WG][3] > 8)) return MDH_ERR_UNSUPPORTED;
    // a workgroup part of q that owns no tile is not a partition of the columns
    if ((int64_t)(p->prt[MDH_L_WG][2] - 1) * pl.QT * pl.TQ >= (s[2] > 0 ? s[2] : 1)) return MDH_ERR_TILE_NOT_DIVIDING;
  } else {
    pl.TQ = p->blk[2];
    if (pl.TQ != 8 && pl.TQ != 16 && pl.TQ != 32) return MDH_ERR_UNSUPPORTED;
    pl.WM = p->prt[MDH_L_VGPR][1] * 32;
    pl.TP = p->prt[MDH_L_WAVE][1] * p->prt[MDH_L_VGPR][1] * (32 / pl.TQ);
    pl.CK = p->prt[MDH_L_LDS][4] * 2;
    pl.S = p->prt[MDH_L_WG][4];
    // a workgroup part of c that owns no channel would leave its partial output unset
    if (pl.S > 1 && pl.CK > 0 && (int64_t)(pl.S - 1) * cdiv(cdiv(s[4], pl.S), pl.CK) * pl.CK >= s[4])
      return MDH_ERR_TILE_NOT_DIVIDING;
  }
  pl.ragged = ragged;
  if (mcc_lds_bytes(pl, s) > kLdsBytesPerWG) return MDH_ERR_TILE_RESOURCES;
  mdh_tile_params chk;
  params_from_plan(s, pl, &chk);
  if (!same_table(chk, *p) || !mcc_inst(pl)) return MDH_ERR_UNSUPPORTED;
  *out = pl;
  return MDH_OK;
}

// =============================================================================== custom reduce

static bool prl_inst(const PrlPlan& pl) {
  static const int menu[][3] = {{2, 4, 1}, {4, 4, 1}, {1, 4, 1}, {2, 2, 2}, {4, 2, 2},
                                {2, 1, 4}, {4, 1, 4}, {2, 8, 1}, {4, 8, 1}};
  for (auto& m : menu)
    if (m[0] == pl.RA && m[1] == pl.WB && m[2] == pl.WA) return true;
  return false;
}

void params_from_plan(const int64_t* s, const PrlPlan& pl, mdh_tile_params* p) {
  clear_params(p, 2);
  p->prt[MDH_L_WG][0] = (int32_t)cdiv(s[0], (int64_t)pl.WA * 64 * pl.RA);
  p->prt[MDH_L_WG][1] = pl.S;
  p->prt[MDH_L_WAVE][0] = pl.WA;
  p->prt[MDH_L_WAVE][1] = pl.WB;
  p->prt[MDH_L_LANE][0] = 64;
  p->prt[MDH_L_VGPR][0] = pl.RA;
  p->prt[MDH_L_HBM][1] = (int32_t)cdiv(s[1], (int64_t)pl.S * pl.WB);
  static const int dims[2] = {0, 1};
  set_order(p, dims);
  p->strided = 0;
  p->lane_fast_dim = 0;
  p->in_region[0] = MDH_MR_VGPR;  // a lane's records of A stay in registers
  p->in_region[1] = MDH_MR_HBM;   // records of B are wavefront-uniform: scalar loads, no staging
  p->out_region = MDH_MR_VGPR;
  p->ragged = (uint8_t)pl.ragged;
}

static int prl_ragged(const int64_t* s, const PrlPlan& pl) {
  return (s[0] % ((int64_t)pl.WA * 64 * pl.RA)) || (s[1] % ((int64_t)pl.S * pl.WB));
}

static PrlPlan prl_default(const int64_t* s) {
  // two records of A per lane, four wavefronts along b (2^16 x 2^18, 8 fields: 7.04 ms with 32 parts of
  // b over workgroups, 7.22 with 16; eight wavefronts along b: 7.42 / 7.51; four records per lane: 7.16)
  PrlPlan pl{2, 4, 1, 1, 0};
  const int64_t wgs_a = cdiv(s[0], (int64_t)pl.WA * 64 * pl.RA);
  int S = 1;
  // split B over workgroups until there are ~64 wavefronts per SIMD of the chip to draw from
  // (2^16 x 2^18: 10.35 ms with 4 parts, 10.0 with 8, 9.8 with 16, 9.75 with 32) while a wavefront
  // keeps 256 records of B; with few records of A first of all a workgroup per compute unit, down to
  // 32 records of B per wavefront (2^10 x 2^14: 30 us with 32 parts, 41 with 16, 69 with 8;
  // 2^8 x 2^18: 104 us with 128 parts, 129 with 256)
  while (wgs_a * S < 256 && S < 256 && s[1] / (2ll * S * pl.WB) >= 32) S *= 2;
  while (wgs_a * S * pl.WB * pl.WA < 65536 && S < 256 && s[1] / (2ll * S * pl.WB) >= 256) S *= 2;
  pl.S = S;
  pl.ragged = prl_ragged(s, pl);
  return pl;
}

int prl_candidates(const int64_t* s, PrlPlan* out, int cap) {
  int n = 0;
  auto push = [&](PrlPlan pl) {
    if (n >= cap) return;
    if (s[1] / ((int64_t)pl.S * pl.WB) < 1) return;
    pl.ragged = prl_ragged(s, pl);
    for (int i = 0; i < n; ++i)
      if (out[i].RA == pl.RA && out[i].WB == pl.WB && out[i].WA == pl.WA && out[i].S == pl.S) return;
    out[n++] = pl;
  };
  PrlPlan d = prl_default(s);
  push(d);
  static const int menu[][3] = {{2, 4, 1}, {4, 4, 1}, {1, 4, 1}, {2, 2, 2}, {4, 2, 2},
                                {2, 1, 4}, {4, 1, 4}, {2, 8, 1}, {4, 8, 1}};
  for (auto& m : menu)
    for (int S = d.S / 2 > 0 ? d.S / 2 : 1; S <= d.S * 2; S *= 2) push(PrlPlan{m[0], m[1], m[2], S, 0});
  return n;
}

mdh_status plan_prl(const int64_t* s, const mdh_tile_params* p, PrlPlan* out) {
  if (!p) {
    *out = prl_default(s);
    return MDH_OK;
  }
  if (p->D != 2) return MDH_ERR_UNSUPPORTED;
  bool ragged;
  mdh_status st = check_products(p, s, &ragged);
  if (st != MDH_OK) return st;
  if ((st = check_lanes(p)) != MDH_OK) return st;
  PrlPlan pl;
  pl.RA = p->prt[MDH_L_VGPR][0];
  pl.WA = p->prt[MDH_L_WAVE][0];
  pl.WB = p->prt[MDH_L_WAVE][1];
  pl.S = p->prt[MDH_L_WG][1];
  pl.ragged = ragged;
  mdh_tile_params chk;
  params_from_plan(s, pl, &chk);
  if (!same_table(chk, *p) || !prl_inst(pl)) return MDH_ERR_UNSUPPORTED;
  *out = pl;
  return MDH_OK;
}

}  // namespace mdh

// =============================================================================== C ABI (host-only part)

using namespace mdh;

extern "C" {

const char* mdh_strerror(mdh_status s) {
  switch (s) {
    case MDH_OK: return "ok";
    case MDH_ERR_NULL: return "a required pointer is NULL";
    case MDH_ERR_SIZE: return "invalid size (negative, empty reduction dimension, or beyond 2^31-1 elements)";
    case MDH_ERR_TILE_NOT_DIVIDING: return "tile parameters violate prod_l #PRT(l,d) * blk[d] == N_d";
    case MDH_ERR_TILE_RESOURCES: return "tile parameters exceed lanes-per-workgroup or LDS budget";
    case MDH_ERR_WORKSPACE: return "workspace missing or too small for the split reduction";
    case MDH_ERR_UNSUPPORTED: return "no kernel instantiation for this configuration";
    case MDH_ERR_LAUNCH: return "HIP launch failed";
    case MDH_ERR_STATIC_LIMIT: return "the call needs more scratch memory than the library's static buffer holds";
  }
  return "unknown status";
}

const char* mdh_version(void) { return "0.1"; }

mdh_status mdh_part_offset(int64_t N, int32_t L, const int32_t* P, const int32_t* p,
                           int64_t* offset, int64_t* part_size) {
  if (!P || !p || !offset || !part_size) return MDH_ERR_NULL;
  if (N < 0 || L < 0) return MDH_ERR_SIZE;
  int64_t prod = 1, os = 0;
  for (int l = 0; l < L; ++l) {
    if (P[l] < 1) return MDH_ERR_TILE_NOT_DIVIDING;
    if (p[l] < 0 || p[l] >= P[l]) return MDH_ERR_SIZE;
    prod *= P[l];
    if (N % prod) return MDH_ERR_TILE_NOT_DIVIDING;
    os += (int64_t)p[l] * (N / prod);
  }
  *offset = os;
  *part_size = N / prod;
  return MDH_OK;
}

static mdh_status check_sizes(mdh_instance inst, const int64_t* s) {
  if (!s) return MDH_ERR_NULL;
  const int D = (inst == MDH_MCC || inst == MDH_MCC_CAPSULE) ? 9 : (inst == MDH_CUSTOM_REDUCE || inst == MDH_MATVEC || inst == MDH_SCAN) ? 2
                                  : inst == MDH_DOT ? 1 : inst == MDH_BMATMUL ? 7 : 3;
  for (int d = 0; d < D; ++d)
    if (s[d] < 0 || s[d] > 0x7fffffff) return MDH_ERR_SIZE;
  switch (inst) {
    case MDH_DOT:
      if (s[0] < 1) return MDH_ERR_SIZE;
      break;
    case MDH_BMATMUL:
      if (s[3] < 1 || s[0] > 65535 || s[4] > 1 || s[5] > 1 || s[6] > 1) return MDH_ERR_SIZE;
      break;
    case MDH_MATVEC:
      if (s[1] < 1) return MDH_ERR_SIZE;
      break;
    case MDH_MATMUL:
      if (s[2] < 1) return MDH_ERR_SIZE;
      break;
    case MDH_STENCIL:
    case MDH_SCAN:
      break;
    case MDH_MCC:
    case MDH_MCC_CAPSULE:
      if (s[4] < 1 || s[5] < 1 || s[6] < 1 || s[7] < 1 || s[8] < 1) return MDH_ERR_SIZE;
      break;
    case MDH_CUSTOM_REDUCE:
      if (s[1] < 1) return MDH_ERR_SIZE;
      break;
    default:
      return MDH_ERR_UNSUPPORTED;
  }
  return MDH_OK;
}

mdh_status mdh_default_params(mdh_instance inst, const int64_t* sizes, mdh_tile_params* out) {
  if (!out) return MDH_ERR_NULL;
  mdh_status st = check_sizes(inst, sizes);
  if (st != MDH_OK) return st;
  switch (inst) {
    case MDH_MATMUL: {
      if (small_m_matmul(sizes, nullptr)) {
        GemmExPlan ex;
        if ((st = plan_small_m(sizes, nullptr, &ex)) != MDH_OK) return st;
        const int64_t s4[7] = {1, sizes[0], sizes[1], sizes[2], 0, 0, 0};
        mdh_tile_params p4;
        params_from_plan(s4, ex, &p4);
        drop_batch(p4, out);
        return MDH_OK;
      }
      GemmPlan pl;
      if ((st = plan_matmul(sizes, nullptr, &pl)) == MDH_OK) params_from_plan(sizes, pl, out);
      return st;
    }
    case MDH_STENCIL: {
      StencilPlan pl;
      if ((st = plan_stencil(sizes, nullptr, &pl)) == MDH_OK) params_from_plan(sizes, pl, out);
      return st;
    }
    case MDH_MCC: {
      MccPlan pl;
      if ((st = plan_mcc(sizes, nullptr, &pl)) == MDH_OK) params_from_plan(sizes, pl, out);
      return st;
    }
    case MDH_CUSTOM_REDUCE: {
      PrlPlan pl;
      if ((st = plan_prl(sizes, nullptr, &pl)) == MDH_OK) params_from_plan(sizes, pl, out);
      return st;
    }
    case MDH_DOT: {
      DotPlan pl;
      if ((st = plan_dot(sizes, nullptr, &pl)) == MDH_OK) params_from_plan(sizes, pl, out);
      return st;
    }
    case MDH_BMATMUL: {
      GemmExPlan pl;
      if ((st = plan_matmul_ex(sizes, nullptr, &pl)) == MDH_OK) params_from_plan(sizes, pl, out);
      return st;
    }
    case MDH_MATVEC: {
      MatVecPlan pl;
      if ((st = plan_matvec(sizes, nullptr, &pl)) == MDH_OK) params_from_plan(sizes, pl, out);
      return st;
    }
    case MDH_SCAN: {
      ScanPlan pl;
      if ((st = plan_scan(sizes, nullptr, &pl)) == MDH_OK) params_from_plan(sizes, pl, out);
      return st;
    }
    case MDH_MCC_CAPSULE: {
      CapsulePlan pl;
      if ((st = plan_capsule(sizes, nullptr, &pl)) == MDH_OK) params_from_plan(sizes, pl, out);
      return st;
    }
  }
  return MDH_ERR_UNSUPPORTED;
}

mdh_status mdh_validate_params(mdh_instance inst, const int64_t* sizes, const mdh_tile_params* p) {
  if (!p) return MDH_ERR_NULL;
  mdh_status st = check_sizes(inst, sizes);
  if (st != MDH_OK) return st;
  switch (inst) {
    case MDH_MATMUL: {
      if (small_m_matmul(sizes, p)) {
        GemmExPlan ex;
        return plan_small_m(sizes, p, &ex);
      }
      GemmPlan pl;
      return plan_matmul(sizes, p, &pl);
    }
    case MDH_STENCIL: {
      StencilPlan pl;
      return plan_stencil(sizes, p, &pl);
    }
    case MDH_MCC: {
      MccPlan pl;
      return plan_mcc(sizes, p, &pl);
    }
    case MDH_CUSTOM_REDUCE: {
      PrlPlan pl;
      return plan_prl(sizes, p, &pl);
    }
    case MDH_DOT: {
      DotPlan pl;
      return plan_dot(sizes, p, &pl);
    }
    case MDH_BMATMUL: {
      GemmExPlan pl;
      return plan_matmul_ex(sizes, p, &pl);
    }
    case MDH_MATVEC: {
      MatVecPlan pl;
      return plan_matvec(sizes, p, &pl);
    }
    case MDH_SCAN: {
      ScanPlan pl;
      return plan_scan(sizes, p, &pl);
    }
    case MDH_MCC_CAPSULE: {
      CapsulePlan pl;
      return plan_capsule(sizes, p, &pl);
    }
  }
  return MDH_ERR_UNSUPPORTED;
}

size_t mdh_workspace_size(mdh_instance inst, const int64_t* sizes, const mdh_tile_params* params) {
  if (check_sizes(inst, sizes) != MDH_OK) return 0;
  switch (inst) {
    case MDH_MATMUL: {
      if (small_m_matmul(sizes, params)) {
        GemmExPlan ex;
        if (plan_small_m(sizes, params, &ex) != MDH_OK || ex.g.S <= 1) return 0;
        return (size_t)ex.g.S * (size_t)sizes[0] * (size_t)sizes[1] * sizeof(float);
      }
      GemmPlan pl;
      if (plan_matmul(sizes, params, &pl) != MDH_OK || pl.S <= 1) return 0;
      return (size_t)pl.S * (size_t)sizes[0] * (size_t)sizes[1] * sizeof(float);
    }
    case MDH_MCC: {
      MccPlan pl;
      if (plan_mcc(sizes, params, &pl) != MDH_OK || pl.flat || pl.S <= 1) return 0;
      return (size_t)pl.S * (size_t)(sizes[0] * sizes[1] * sizes[2] * sizes[3]) * sizeof(float);
    }
    case MDH_CUSTOM_REDUCE: {
      PrlPlan pl;
      if (plan_prl(sizes, params, &pl) != MDH_OK || pl.S <= 1) return 0;
      return (size_t)pl.S * (size_t)sizes[0] * 2 * sizeof(int32_t);
    }
    case MDH_DOT: {
      DotPlan pl;
      if (plan_dot(sizes, params, &pl) != MDH_OK || pl.S <= 1) return 0;
      return (size_t)pl.S * sizeof(float);
    }
    case MDH_BMATMUL: {
      GemmExPlan pl;
      if (plan_matmul_ex(sizes, params, &pl) != MDH_OK || pl.g.S <= 1) return 0;
      return (size_t)pl.g.S * (size_t)sizes[0] * (size_t)sizes[1] * (size_t)sizes[2] * sizeof(float);
    }
    case MDH_MATVEC: {
      MatVecPlan pl;
      if (plan_matvec(sizes, params, &pl) != MDH_OK || pl.S <= 1) return 0;
      return (size_t)pl.S * (size_t)sizes[0] * sizeof(float);
    }
    case MDH_SCAN: {
      ScanPlan pl;
      if (plan_scan(sizes, params, &pl) != MDH_OK) return 0;
      return scan_workspace_bytes(pl, sizes[0]);
    }
    default:
      return 0;
  }
}

int32_t mdh_num_candidates(mdh_instance inst, const int64_t* sizes) {
  if (check_sizes(inst, sizes) != MDH_OK) return 0;
  constexpr int CAP = 128;
  switch (inst) {
    case MDH_MATMUL: {
      GemmPlan c[CAP];
      return matmul_candidates(sizes, c, CAP);
    }
    case MDH_STENCIL: {
      StencilPlan c[CAP];
      return stencil_candidates(sizes, c, CAP);
    }
    case MDH_MCC: {
      MccPlan c[CAP];
      return mcc_candidates(sizes, c, CAP);
    }
    case MDH_CUSTOM_REDUCE: {
      PrlPlan c[CAP];
      return prl_candidates(sizes, c, CAP);
    }
    case MDH_DOT: {
      DotPlan c[CAP];
      return dot_candidates(sizes, c, CAP);
    }
    case MDH_BMATMUL: {
      GemmExPlan c[CAP];
      return matmul_ex_candidates(sizes, c, CAP);
    }
    case MDH_MATVEC: {
      MatVecPlan c[CAP];
      return matvec_candidates(sizes, c, CAP);
    }
    case MDH_SCAN: {
      ScanPlan c[CAP];
      return scan_candidates(sizes, c, CAP);
    }
    case MDH_MCC_CAPSULE: {
      CapsulePlan c[CAP];
      return capsule_candidates(sizes, c, CAP);
    }
  }
  return 0;
}

mdh_status mdh_candidate(mdh_instance inst, const int64_t* sizes, int32_t idx, mdh_tile_params* out) {
  if (!out) return MDH_ERR_NULL;
  mdh_status st = check_sizes(inst, sizes);
  if (st != MDH_OK) return st;
  constexpr int CAP = 128;
  switch (inst) {
    case MDH_MATMUL: {
      GemmPlan c[CAP];
      int n = matmul_candidates(sizes, c, CAP);
      if (idx < 0 || idx >= n) return MDH_ERR_SIZE;
      // candidate 0 is the default: for few rows the small-M kernel, which the tiled menu does not hold
      if (idx == 0 && small_m_matmul(sizes, nullptr)) return mdh_default_params(inst, sizes, out);
      params_from_plan(sizes, c[idx], out);
      return MDH_OK;
    }
    case MDH_STENCIL: {
      StencilPlan c[CAP];
      int n = stencil_candidates(sizes, c, CAP);
      if (idx < 0 || idx >= n) return MDH_ERR_SIZE;
      params_from_plan(sizes, c[idx], out);
      return MDH_OK;
    }
    case MDH_MCC: {
      MccPlan c[CAP];
      int n = mcc_candidates(sizes, c, CAP);
      if (idx < 0 || idx >= n) return MDH_ERR_SIZE;
      params_from_plan(sizes, c[idx], out);
      return MDH_OK;
    }
    case MDH_CUSTOM_REDUCE: {
      PrlPlan c[CAP];
      int n = prl_candidates(sizes, c, CAP);
      if (idx < 0 || idx >= n) return MDH_ERR_SIZE;
      params_from_plan(sizes, c[idx], out);
      return MDH_OK;
    }
    case MDH_DOT: {
      DotPlan c[CAP];
      int n = dot_candidates(sizes, c, CAP);
      if (idx < 0 || idx >= n) return MDH_ERR_SIZE;
      params_from_plan(sizes, c[idx], out);
      return MDH_OK;
    }
    case MDH_BMATMUL: {
      GemmExPlan c[CAP];
      int n = matmul_ex_candidates(sizes, c, CAP);
      if (idx < 0 || idx >= n) return MDH_ERR_SIZE;
      params_from_plan(sizes, c[idx], out);
      return MDH_OK;
    }
    case MDH_MATVEC: {
      MatVecPlan c[CAP];
      int n = matvec_candidates(sizes, c, CAP);
      if (idx < 0 || idx >= n) return MDH_ERR_SIZE;
      params_from_plan(sizes, c[idx], out);
      return MDH_OK;
    }
    case MDH_SCAN: {
      ScanPlan c[CAP];
      int n = scan_candidates(sizes, c, CAP);
      if (idx < 0 || idx >= n) return MDH_ERR_SIZE;
      params_from_plan(sizes, c[idx], out);
      return MDH_OK;
    }
    case MDH_MCC_CAPSULE: {
      CapsulePlan c[CAP];
      int n = capsule_candidates(sizes, c, CAP);
      if (idx < 0 || idx >= n) return MDH_ERR_SIZE;
      params_from_plan(sizes, c[idx], out);
      return MDH_OK;
    }
  }
  return MDH_ERR_UNSUPPORTED;
}

}  // extern "C"
