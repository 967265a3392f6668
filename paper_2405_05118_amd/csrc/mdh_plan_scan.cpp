// Planner for the row-wise scan: md_hom(id, (++, prefix-sum(+))) over (i, j)
// (paper: Section "Examples", Subfigure 8; Appendix, Example "Prefix-Sum").
// Table: a workgroup owns one row i and one chunk of j; the chunk is TPC tiles of WAVES wavefronts
// x 64 lanes x 4 consecutive elements, walked one after the other with a carry (HBM-layer parts) or
// all held in registers (register-layer parts: single pass over long rows, short rows); blocked assignment
// (a part of j is a contiguous range, so that a part's result only needs ONE value of the parts
// before it: their last prefix).
#include <string.h>

#include "mdh_internal.h"

namespace mdh {
using namespace detail;

static const int kScanWaves[] = {4, 8, 16};
// single-pass variant (the chunk stays in registers): tiles per chunk are a template parameter
static const int kOnePassWaves[] = {8, 16};
static const int kOnePassTpc[] = {1, 2, 4, 8};  // 5 registers per tile and lane

void params_from_plan(const int64_t* s, const ScanPlan& pl, mdh_tile_params* p) {
  clear_params(p, 2);
  p->prt[MDH_L_WG][0] = (int32_t)(s[0] > 0 ? s[0] : 1);  // an empty call still has a valid table
  if (pl.WAVES == 1) {  // short rows: 4 rows per workgroup, one wavefront each
    p->prt[MDH_L_WG][0] = (int32_t)cdiv(s[0] > 0 ? s[0] : 1, 4);
    p->prt[MDH_L_WAVE][0] = 4;
  }
  p->prt[MDH_L_WG][1] = pl.C;
  p->prt[MDH_L_WAVE][1] = pl.WAVES;
  p->prt[MDH_L_LANE][1] = 64;
  if (pl.onepass) {  // the TPC tiles of a chunk are register-layer parts: a lane holds 4 * TPC elements
    p->prt[MDH_L_HBM][1] = 1;
    p->prt[MDH_L_VGPR][1] = 4 * pl.TPC;
  } else {  // sequential tiles with a carry, 4 elements of a lane in registers at a time
    p->prt[MDH_L_HBM][1] = pl.TPC;
    p->prt[MDH_L_VGPR][1] = 4;
  }
  static const int dims[2] = {0, 1};
  set_order(p, dims);
  p->strided = 0;
  p->lane_fast_dim = 1;
  // where a chunk waits while the workgroups exchange their totals: in registers (one pass over
  // the input), or not at all (it is read from HBM a second time)
  p->in_region[0] = (pl.C > 1 && !pl.onepass) ? MDH_MR_HBM : MDH_MR_VGPR;
  p->out_region = MDH_MR_VGPR;
  p->ragged = (uint8_t)pl.ragged;
}

static int scan_ragged(const int64_t* s, const ScanPlan& pl) {
  return s[0] == 0 || s[1] != (int64_t)pl.C * pl.TPC * pl.WAVES * 256 || (pl.WAVES == 1 && s[0] % 4);
}

static ScanPlan scan_plan(const int64_t* s, int waves, int64_t chunks) {
  ScanPlan pl{waves, 1, 1, 0, 0};
  const int64_t tile = (int64_t)waves * 256;
  const int64_t tiles = cdiv(s[1] > 0 ? s[1] : 1, tile);
  if (chunks < 1) chunks = 1;
  if (chunks > tiles) chunks = tiles;
  pl.TPC = (int)cdiv(tiles, chunks);
  pl.C = (int)cdiv(tiles, pl.TPC);  // no empty chunk
  pl.ragged = scan_ragged(s, pl);
  return pl;
}

static ScanPlan scan_onepass_plan(const int64_t* s, int waves, int tpc) {
  ScanPlan pl{waves, tpc, 1, 0, 1};
  const int64_t tiles = cdiv(s[1] > 0 ? s[1] : 1, (int64_t)waves * 256);
  pl.C = (int)cdiv(tiles, tpc);
  if (pl.C <= 1) {  // the whole row in one workgroup's registers: as few tiles as cover it
    pl.C = 1;
    while (pl.TPC > 1 && pl.TPC / 2 >= tiles) pl.TPC /= 2;
    if (pl.TPC == 1) pl.onepass = 0;  // one tile: the same as the sequential kernel
  }
  pl.ragged = scan_ragged(s, pl);
  return pl;
}

static ScanPlan scan_wave_plan(const int64_t* s) {
  ScanPlan pl{1, (int)cdiv(s[1] > 0 ? s[1] : 1, 256), 1, 0, 0};
  pl.ragged = scan_ragged(s, pl);
  return pl;
}

static ScanPlan scan_default(const int64_t* s) {
  // many short rows: a wavefront per row (no LDS, no barriers); measured best up to 768 elements
  if (s[1] <= 768 && s[0] >= 4096) return scan_wave_plan(s);
  // enough rows: one workgroup per row walks the whole row (one pass over the data); few rows:
  // chunks of j over workgroups until ~2048 workgroups, chunk totals scanned by a second kernel
  const int64_t rows = s[0] > 0 ? s[0] : 1;
  int64_t chunks = 1;
  while (rows * chunks < 2048 && cdiv(s[1], 2048 * chunks * 2) >= 4) chunks *= 2;
  if (chunks == 1) {
    // a row of up to 8 tiles stays in registers (two barriers per row); longer rows are walked tile
    // by tile with a carry; 8 wavefronts per workgroup measured fastest (4 and 16 within 7 %)
    // (65536 x 4096: 0.330 ms resident against 0.349 ms; 8192 x 32768: 0.364 against 0.403 ms; rows
    // beyond 4096 elements with 16 wavefronts, which keeps the tiles per lane few)
    const ScanPlan res = s[1] <= 4096 ? scan_onepass_plan(s, 8, 8) : scan_onepass_plan(s, 16, 8);
    if (res.C == 1 && res.onepass) return res;
    // rows of one or two tiles of 1024: four wavefronts (65536 x 1000: 84 us against 128 us with
    // eight wavefronts and half of them idle; 65536 x 1536: 126 against 146 us)
    return scan_plan(s, s[1] <= 1536 ? 4 : 8, 1);
  }
  // few long rows: chunks of j over workgroups, a chunk resident in registers (one pass over the
  // input); as many tiles per chunk as still give a workgroup per compute unit
  int tpc = 8;
  while (tpc > 2 && rows * cdiv(s[1], (int64_t)4096 * tpc) < 256) tpc /= 2;
  return scan_onepass_plan(s, 16, tpc);  // 16 wavefronts measured fastest (8: +8 %)
}

int scan_candidates(const int64_t* s, ScanPlan* out, int cap) {
  int n = 0;
  auto push = [&](const ScanPlan& pl) {
    if (n >= cap) return;
    for (int i = 0; i < n; ++i)
      if (out[i].WAVES == pl.WAVES && out[i].C == pl.C && out[i].TPC == pl.TPC && out[i].onepass == pl.onepass) return;
    out[n++] = pl;
  };
  const ScanPlan d0 = scan_default(s);
  push(d0);
  if (s[1] <= 65536) push(scan_wave_plan(s));
  // chunk counts are swept around those of the workgroup-per-chunk default
  int64_t chunks0 = 1;
  while ((s[0] > 0 ? s[0] : 1) * chunks0 < 2048 && cdiv(s[1], 2048 * chunks0 * 2) >= 4) chunks0 *= 2;
  const ScanPlan d = scan_plan(s, 8, chunks0);
  push(d);
  for (int w : kScanWaves)
    for (int64_t c = d.C / 4 > 0 ? d.C / 4 : 1; c <= (int64_t)d.C * 8; c *= 2) push(scan_plan(s, w, c));
  for (int w : kOnePassWaves)
    for (int t : kOnePassTpc) {
      const ScanPlan pl = scan_onepass_plan(s, w, t);
      if (pl.onepass && (d.C > 1 || pl.C == 1)) push(pl);
    }
  return n;
}

mdh_status plan_scan(const int64_t* s, const mdh_tile_params* p, ScanPlan* out) {
  if (!p) {
    *out = scan_default(s);
    return MDH_OK;
  }
  if (p->D != 2) return MDH_ERR_UNSUPPORTED;
  bool ragged;
  mdh_status st = check_products(p, s, &ragged);
  if (st != MDH_OK) return st;
  if ((st = check_lanes(p)) != MDH_OK) return st;
  ScanPlan pl{p->prt[MDH_L_WAVE][1], p->prt[MDH_L_HBM][1], p->prt[MDH_L_WG][1], ragged, 0};
  const int vg = p->prt[MDH_L_VGPR][1];
  pl.onepass = (pl.C > 1 && p->in_region[0] == MDH_MR_VGPR) || (pl.C == 1 && vg > 4);
  if (pl.onepass) {
    if (vg % 4 || pl.TPC != 1) return MDH_ERR_UNSUPPORTED;  // register-layer tiles, no sequential ones
    pl.TPC = vg / 4;
  }
  bool inst = pl.WAVES == 1 && pl.C == 1;
  if (pl.onepass) {
    bool w_ok = false, t_ok = false;
    for (int w : kOnePassWaves) w_ok = w_ok || (w == pl.WAVES);
    for (int t : kOnePassTpc) t_ok = t_ok || (t == pl.TPC);
    inst = w_ok && t_ok && (pl.C > 1 || pl.TPC > 1);
  } else {
    for (int w : kScanWaves) inst = inst || (w == pl.WAVES);
  }
  // a chunk that owns no index would leave its total unset
  if ((int64_t)(pl.C - 1) * pl.TPC * pl.WAVES * 256 >= (s[1] > 0 ? s[1] : 1)) return MDH_ERR_TILE_NOT_DIVIDING;
  mdh_tile_params chk;
  params_from_plan(s, pl, &chk);
  if (!same_table(chk, *p) || !inst) return MDH_ERR_UNSUPPORTED;
  *out = pl;
  return MDH_OK;
}

// Three-kernel variant: R*C chunk totals (fp64).  Single-pass variant: a ticket counter and a
// time-out flag (2 words), R*C chunk totals and R*ceil(C/64) group sums, 8 bytes each.
size_t scan_workspace_bytes(const ScanPlan& pl, int64_t R) {
  if (pl.C <= 1) return 0;
  if (!pl.onepass) return (size_t)pl.C * (size_t)R * sizeof(double);
  return (2 + (size_t)R * (size_t)pl.C + (size_t)R * (size_t)cdiv(pl.C, 64)) * 8;
}

}  // namespace mdh
