// Generic md_hom with a runtime-compiled scalar function and combine operator
// (paper: Definition "Higher-Order Function md_hom"; Definitions "Input View" / "Output View";
// Section "Low-Level Representation": de-composition, scalar phase, re-composition).
//
// The kernel source is generated for ONE description and ONE tuning configuration: sizes, part
// counts and the lane layout are compile-time constants of the generated code, the user's f, op,
// index functions and types are pasted in, and hipRTC compiles it for gfx950.
//
// Per dimension d: index = ((q*WG_d + g)*L_d + l)*V_d + v  (strided)  or  ((g*Q_d + q)*L_d + l)*V_d + v
// (blocked), g = workgroup part, l = lane part, q = sequential part on the device-memory layer, v =
// part on the register layer (concatenation dimensions only).  A lane walks its sequential parts of
// the concatenation dimensions (outer loops) and, for each, its sequential parts of the reduced
// dimensions (inner loops); innermost, unrolled, are the V = prod V_d register parts: V results are
// combined in registers at once, and an input element whose index function does not depend on a
// register-blocked dimension is loaded once for all of its parts (register tiling).  The lanes that share a point combine
// in an LDS tree, workgroups that share it write to the workspace and a second kernel folds the
// parts in ascending order.  No neutral element: a part starts with its first value, and a flag
// says whether a lane has one.
#include <hip/hiprtc.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <string>
#include <vector>

#include "mdh_internal.h"

namespace mdh {
using namespace detail;

namespace {

constexpr int kMaxLanes = 1024;
constexpr int64_t kLdsBytes = 64 * 1024;

struct CustomPlan {
  int D;
  int64_t N[MDH_MAX_D];
  int red[MDH_MAX_D];
  int64_t WG[MDH_MAX_D], L[MDH_MAX_D], Q[MDH_MAX_D];
  int64_t V[MDH_MAX_D];  // register-layer parts (concatenation dimensions; 1 elsewhere)
  int scan;  // the prefix-sum dimension (at most one), -1: none
  int strided;
  int fast;  // dimension with the fastest lane index
  int ragged;
  // derived
  int VT;          // register parts per lane (product of V)
  int NT;          // lanes per workgroup
  int RL, CL;      // lanes over reduced / concatenation dimensions
  int64_t SG, CG;  // workgroup parts over reduced / concatenation dimensions
  int64_t CCN;     // points of the concatenation dimensions
};

bool desc_ok(const mdh_custom_desc* d) {
  if (d->D < 1 || d->D > MDH_MAX_D) return false;
  if (d->n_in < 1 || d->n_in > MDH_CUSTOM_MAX_IN) return false;
  if (d->n_acc < 1 || d->n_acc > MDH_CUSTOM_MAX_ACC) return false;
  if (d->out_elem_bytes < 1 || d->out_elem_bytes > 256) return false;
  if (d->fast_dim >= d->D) return false;
  int scans = 0;
  for (int i = 0; i < d->D; ++i) {
    if (d->reduce[i] > 2) return false;
    scans += d->reduce[i] == 2;
  }
  if (scans > 1) return false;
  int64_t total = 1;
  for (int i = 0; i < d->D; ++i) {
    if (d->sizes[i] < 1 || d->sizes[i] > 0x7fffffff) return false;
    if (total > (int64_t)1 << 50) return false;
    total *= d->sizes[i];
  }
  for (int a = 0; a < d->n_acc; ++a)
    if (d->acc_buf[a] < 0 || d->acc_buf[a] >= d->n_in) return false;
  return true;
}

mdh_status desc_ptrs(const mdh_custom_desc* d) {
  if (!d->out_type || !d->f) return MDH_ERR_NULL;
  for (int b = 0; b < d->n_in; ++b)
    if (!d->in_type[b]) return MDH_ERR_NULL;
  for (int a = 0; a < d->n_acc; ++a)
    if (!d->acc_index[a]) return MDH_ERR_NULL;
  for (int i = 0; i < d->D; ++i)
    if (d->reduce[i] && !d->op) return MDH_ERR_NULL;
  return MDH_OK;
}

void derive(CustomPlan* p) {
  p->NT = 1, p->RL = 1, p->CL = 1, p->SG = 1, p->CG = 1, p->CCN = 1, p->VT = 1;
  for (int d = 0; d < p->D; ++d) {
    p->NT *= (int)p->L[d];
    p->VT *= (int)p->V[d];
    if (p->red[d]) {
      p->RL *= (int)p->L[d];
      p->SG *= p->WG[d];
    } else {
      p->CL *= (int)p->L[d];
      p->CG *= p->WG[d];
      p->CCN *= p->N[d];
    }
  }
}

void params_from_custom(const CustomPlan& pl, mdh_tile_params* p) {
  clear_params(p, pl.D);
  int dims[MDH_MAX_D];
  for (int d = 0; d < pl.D; ++d) {
    p->prt[MDH_L_WG][d] = (int32_t)pl.WG[d];
    p->prt[MDH_L_LANE][d] = (int32_t)pl.L[d];
    p->prt[MDH_L_HBM][d] = (int32_t)pl.Q[d];
    p->prt[MDH_L_VGPR][d] = (int32_t)pl.V[d];
    dims[d] = d;
  }
  set_order(p, dims);
  p->strided = (uint8_t)pl.strided;
  p->lane_fast_dim = (uint8_t)pl.fast;
  p->out_region = MDH_MR_VGPR;  // results are combined in registers, inputs stay in device memory
  p->ragged = (uint8_t)pl.ragged;
}

void fill_from_desc(const mdh_custom_desc* d, CustomPlan* pl) {
  memset(pl, 0, sizeof(*pl));
  pl->D = d->D;
  for (int i = 0; i < d->D; ++i) {
    pl->N[i] = d->sizes[i];
    pl->red[i] = d->reduce[i] == 1 ? 1 : 0;
    pl->WG[i] = pl->L[i] = pl->Q[i] = pl->V[i] = 1;
  }
  pl->scan = -1;
  for (int i = 0; i < d->D; ++i)
    if (d->reduce[i] == 2) pl->scan = i;
  pl->fast = d->fast_dim < 0 ? d->D - 1 : d->fast_dim;
  // the prefix-sum dimension is walked sequentially by a lane: the lanes go to another dimension
  if (pl->fast == pl->scan)
    for (int i = 0; i < d->D; ++i)
      if (i != pl->scan) pl->fast = i;
  pl->strided = 1;
}

// Does the C expression `e` use the identifier `id` (e.g. "i2")?
bool uses_identifier(const char* e, const char* id) {
  const size_t n = strlen(id);
  auto word = [](char c) { return (c >= '0' && c <= '9') || (c >= 'a' && c <= 'z') || (c >= 'A' && c <= 'Z') || c == '_'; };
  for (const char* p = strstr(e, id); p; p = strstr(p + 1, id))
    if ((p == e || !word(p[-1])) && !word(p[n])) return true;
  return false;
}

// A concatenation dimension is worth blocking in registers if some input access does not depend on
// it: that element is then loaded once for all register parts of the dimension.
bool reused_across(const mdh_custom_desc* d, int dim) {
  char id[8];
  snprintf(id, sizeof id, "i%d", dim);
  for (int a = 0; a < d->n_acc; ++a)
    if (!uses_identifier(d->acc_index[a], id)) return true;
  return false;
}

int pow2_floor(int64_t x) {
  int p = 1;
  while ((int64_t)p * 2 <= x) p *= 2;
  return p;
}

// lanes: `nt` lanes, first along the fast dimension, the rest along the largest other dimension
// (concatenation dimensions preferred); workgroup parts: all of the concatenation dimensions, and
// the reduced dimensions `split` ways in total while every part keeps at least 8 sequential steps.
CustomPlan make_plan(const mdh_custom_desc* d, int nt, int64_t split, int vreg = 1, int vec = 1) {
  CustomPlan pl;
  fill_from_desc(d, &pl);
  int left = nt;
  if (pl.scan >= 0) split = 1;  // the parts of the other reduced dimensions meet inside the workgroup
  if (pl.fast != pl.scan) pl.L[pl.fast] = pow2_floor(pl.N[pl.fast] < left ? pl.N[pl.fast] : left);
  left /= (int)pl.L[pl.fast];
  while (left > 1) {
    int best = -1;
    for (int pass = 0; pass < 2 && best < 0; ++pass)
      for (int i = pl.D - 1; i >= 0; --i) {
        if (i == pl.fast || i == pl.scan || (pass == 0 && pl.red[i])) continue;
        if (pl.N[i] / pl.L[i] < 2) continue;
        if (best < 0 || pl.N[i] / pl.L[i] > pl.N[best] / pl.L[best]) best = i;
      }
    if (best < 0) break;
    pl.L[best] *= 2;
    left /= 2;
  }
  // register parts: `vreg` per reusable concatenation dimension, at most 16 results per lane
  if (vreg > 1 && pl.scan < 0) {
    int vt = 1;
    for (int i = pl.D - 1; i >= 0; --i) {
      if (pl.red[i] || !d->acc_index[0] || !reused_across(d, i)) continue;
      if (pl.N[i] < 2 * pl.L[i] * vreg || vt * vreg > 16) continue;
      pl.V[i] = vreg;
      vt *= vreg;
    }
  }
  // `vec` consecutive indices of the fast dimension per lane whether or not anything is reused
  // across them: neighbouring register parts read and write neighbouring addresses
  if (vec > 1 && pl.scan < 0 && !pl.red[pl.fast] && pl.V[pl.fast] == 1 && pl.N[pl.fast] >= 2 * pl.L[pl.fast] * vec)
    pl.V[pl.fast] = vec;
  for (int i = 0; i < pl.D; ++i)
    if (!pl.red[i] && i != pl.scan) pl.WG[i] = cdiv(pl.N[i], pl.L[i] * pl.V[i]);
  // sequential parts of the concatenation dimensions only when the grid would not fit
  for (int i = 0; i < pl.D; ++i) {
    if (pl.red[i]) continue;
    int64_t grid = 1;
    for (int j = 0; j < pl.D; ++j) grid *= pl.WG[j];
    while (grid > (1 << 24) && pl.WG[i] > 1) {
      pl.WG[i] = cdiv(pl.WG[i], 2);
      grid = cdiv(grid, 2);
    }
  }
  for (int i = 0; i < pl.D && split > 1; ++i) {
    if (!pl.red[i]) continue;
    while (split > 1 && cdiv(pl.N[i], pl.L[i] * pl.WG[i] * 2) >= 8) {  // reduced dimensions: V = 1
      pl.WG[i] *= 2;
      split /= 2;
    }
  }
  pl.ragged = 0;
  for (int i = 0; i < pl.D; ++i) {
    pl.Q[i] = cdiv(pl.N[i], pl.WG[i] * pl.L[i] * pl.V[i]);
    // no empty workgroup part: shrink WG to the parts that own at least one index
    pl.WG[i] = cdiv(pl.N[i], pl.Q[i] * pl.L[i] * pl.V[i]);
    if (pl.WG[i] * pl.L[i] * pl.Q[i] * pl.V[i] != pl.N[i]) pl.ragged = 1;
  }
  // with a blocked walk every workgroup part starts at g*Q*L; strided parts start at g*L: both
  // are non-empty now.  Blocked is the safe choice when Q*L*WG overshoots N by more than one part.
  pl.strided = 0;
  derive(&pl);
  return pl;
}

CustomPlan default_plan(const mdh_custom_desc* d) {
  // register parts on the reusable concatenation dimensions, unless the grid gets too small for it;
  // few workgroups: split the reduced dimensions over workgroups up to ~2048 workgroups
  // (results wider than 4 bytes -- user-defined structs -- are not blocked by default: measured
  // slower on the record-linkage example; such configurations are among the candidates)
  // eight parts on one reusable dimension first (Histo, 256 bins x 2^24 elements: 0.32 ms against
  // 0.37 ms with four; MatMul 1024^3: 25 TFLOP/s against 18 with four parts on each of i and j)
  // lanes: a workgroup of 256 (1024 when every dimension is a concatenation dimension), but a single
  // wavefront when the lanes run along a reduced dimension
  // and the concatenation dimensions alone fill the chip (MatVec 8192^2: 6.7 TB/s against 5.0 TB/s --
  // the wavefront's partial results meet in registers, no LDS tree)
  int nt = 256;
  {
    CustomPlan probe;
    fill_from_desc(d, &probe);
    int64_t cc = 1;
    for (int i = 0; i < probe.D; ++i)
      if (!probe.red[i] && i != probe.scan) cc *= probe.N[i];
    if (probe.scan < 0 && probe.red[probe.fast] && cc >= 2048 && probe.N[probe.fast] >= 64) nt = 64;
    bool any_red = false;
    for (int i = 0; i < probe.D; ++i) any_red = any_red || probe.red[i] || i == probe.scan;
    // nothing but concatenation: four consecutive indices of the fast dimension per lane, so that
    // neighbouring parts share 16-byte accesses (Jacobi1D 2^26: 6.0 TB/s against 3.8 TB/s with one
    // index per lane; 64, 256 and 1024 lanes per workgroup within 1 %), while that leaves 1024 workgroups
    if (!any_red) {
      CustomPlan pl = make_plan(d, 256, 1, 1, 4);
      if (pl.CG >= 1024 && d->out_elem_bytes <= 16) return pl;
      if (cc >= (1 << 20)) nt = 1024;
    }
  }
  // an access that depends on every dimension streams its buffer once whatever the blocking
  // (MatVec's matrix): register parts then only cost lanes (MatVec 8192^2: 6.4 TB/s without them,
  // 5.6 TB/s with eight)
  bool streams = false;
  for (int a = 0; a < d->n_acc && d->D > 1; ++a) {
    bool all = true;
    for (int i = 0; i < d->D && all; ++i) {
      char id[8];
      snprintf(id, sizeof id, "i%d", i);
      all = uses_identifier(d->acc_index[a], id);
    }
    streams = streams || all;
  }
  const int v8 = (d->out_elem_bytes <= 4 && !streams) ? 8 : 1, v4 = (d->out_elem_bytes <= 4 && !streams) ? 4 : 1;
  CustomPlan pl;
  for (int vreg : {v8, v4, 1}) {
    pl = make_plan(d, nt, 1, vreg);
    const int64_t grid = pl.SG * pl.CG;
    int64_t steps = 1;  // sequential steps of a lane over the reduced dimensions
    for (int i = 0; i < pl.D; ++i)
      if (pl.red[i]) steps *= pl.Q[i];
    // split up to ~2048 workgroups, and further while a lane would walk more than ~1024 steps
    // (custom reduce 2^16 x 2^18: 10.0 ms with 1024 steps per lane, 13.9 ms with 32768)
    // ... as long as the second pass stays small beside the first: a part keeps at least 32 points of
    // the reduced dimensions, and at least 256 when there are few output points, because the second
    // pass folds the parts of a point sequentially in one lane and few points mean few lanes
    // (custom reduce 2^10 x 2^14: 83 us with 64 parts, 236 us with 512; MatMul 512^3 is fastest
    // with 16 parts of 32)
    int64_t points = 1;
    for (int i = 0; i < pl.D; ++i)
      if (pl.red[i]) points *= pl.N[i];
    const int64_t per_part = pl.CCN < 4096 && pl.CCN >= 256 ? 256 : 32;
    const int64_t cap = points / per_part > 1 ? points / per_part : 1;
    int64_t split = 1;
    while (grid * split < 2048 && grid < 1024 && split * 2 <= cap) split *= 2;
    while (steps / split > 1024 && grid * split < 32768 && split * 2 <= cap) split *= 2;
    if (split > 1) pl = make_plan(d, nt, split, vreg);
    if (pl.SG * pl.CG >= 512) break;
  }
  return pl;
}

int candidates(const mdh_custom_desc* d, CustomPlan* out, int cap) {
  int n = 0;
  auto push = [&](const CustomPlan& c) {
    if (n >= cap) return;
    for (int i = 0; i < n; ++i) {
      bool same = out[i].strided == c.strided;
      for (int k = 0; k < c.D && same; ++k)
        same = out[i].WG[k] == c.WG[k] && out[i].L[k] == c.L[k] && out[i].Q[k] == c.Q[k] && out[i].V[k] == c.V[k];
      if (same) return;
    }
    out[n++] = c;
  };
  push(default_plan(d));
  bool any_red = false;
  for (int i = 0; i < d->D; ++i) any_red |= d->reduce[i] != 0;
  static const int nts[] = {256, 64, 128, 512, 1024};
  static const int64_t splits[] = {1, 4, 16, 64, 256, 1024, 4096};
  for (int nt : nts)
    for (int64_t s : splits) {
      if (s > 1 && !any_red) continue;
      push(make_plan(d, nt, s));
    }
  for (int vec : {4, 2})
    for (int nt : {256, 1024, 64}) push(make_plan(d, nt, any_red ? 16 : 1, 1, vec));
  static const int vregs[] = {2, 4, 8};
  for (int v : vregs)
    for (int nt : {256, 64})
      for (int64_t s : {(int64_t)1, (int64_t)16, (int64_t)256}) {
        if (s > 1 && !any_red) continue;
        push(make_plan(d, nt, s, v));
      }
  return n;
}

mdh_status plan_from_params(const mdh_custom_desc* d, const mdh_tile_params* p, CustomPlan* out) {
  if (!p) {
    *out = default_plan(d);
    return MDH_OK;
  }
  if (p->D != d->D) return MDH_ERR_UNSUPPORTED;
  bool ragged;
  mdh_status st = check_products(p, d->sizes, &ragged);
  if (st != MDH_OK) return st;
  if ((st = check_lanes(p)) != MDH_OK) return st;
  CustomPlan pl;
  fill_from_desc(d, &pl);
  for (int i = 0; i < d->D; ++i) {
    pl.WG[i] = p->prt[MDH_L_WG][i];
    pl.L[i] = p->prt[MDH_L_LANE][i];
    pl.Q[i] = p->prt[MDH_L_HBM][i];
    pl.V[i] = p->prt[MDH_L_VGPR][i];
    // register parts only on concatenation dimensions (a lane's parts of a reduced dimension are
    // the sequential parts)
    if (pl.V[i] > 1 && (pl.red[i] || pl.scan >= 0)) return MDH_ERR_UNSUPPORTED;
    // a workgroup part of any dimension that owns no index would leave its partial result unset
    const int64_t first_of_last =
        (p->strided ? (pl.WG[i] - 1) * pl.L[i] : (pl.WG[i] - 1) * pl.Q[i] * pl.L[i]) * pl.V[i];
    if (first_of_last >= pl.N[i]) return MDH_ERR_TILE_NOT_DIVIDING;
  }
  if (p->lane_fast_dim >= d->D) return MDH_ERR_UNSUPPORTED;
  pl.fast = p->lane_fast_dim;
  pl.strided = p->strided ? 1 : 0;
  pl.ragged = ragged;
  derive(&pl);
  // a prefix-sum dimension is sequential in this kernel, and the other reduced dimensions may then
  // not be split over workgroups
  if (pl.scan >= 0 && (pl.WG[pl.scan] != 1 || pl.L[pl.scan] != 1 || pl.SG != 1)) return MDH_ERR_UNSUPPORTED;
  mdh_tile_params chk;
  params_from_custom(pl, &chk);
  if (!same_table(chk, *p)) return MDH_ERR_UNSUPPORTED;  // e.g. parts on the LDS / register layers
  *out = pl;
  return MDH_OK;
}

mdh_status plan_resources(const mdh_custom_desc* d, const CustomPlan& pl) {
  if (pl.NT > kMaxLanes) return MDH_ERR_TILE_RESOURCES;
  if ((int64_t)pl.VT * d->out_elem_bytes > 1024) return MDH_ERR_TILE_RESOURCES;  // results held in registers
  if (pl.RL > 1 && (int64_t)pl.NT * (d->out_elem_bytes + 1) > kLdsBytes) return MDH_ERR_TILE_RESOURCES;
  if (pl.SG * pl.CG > 0x7fffffff) return MDH_ERR_SIZE;
  return MDH_OK;
}

// ------------------------------------------------------------------------------ code generation

struct Src {
  std::string s;
  void line(const std::string& t) { s += t, s += '\n'; }
  template <class... A>
  void f(const char* fmt, A... a) {
    char buf[1024];
    snprintf(buf, sizeof buf, fmt, a...);
    s += buf;
    s += '\n';
  }
};

std::string index_expr(const CustomPlan& pl, int d) {
  char buf[160];
  if (pl.strided)
    snprintf(buf, sizeof buf, "(((i64)q%d * %lldLL + g%d) * %lldLL + l%d) * %lldLL", d, (long long)pl.WG[d], d,
             (long long)pl.L[d], d, (long long)pl.V[d]);
  else
    snprintf(buf, sizeof buf, "(((i64)g%d * %lldLL + q%d) * %lldLL + l%d) * %lldLL", d, (long long)pl.Q[d], d,
             (long long)pl.L[d], d, (long long)pl.V[d]);
  return buf;
}

std::string generate(const mdh_custom_desc* d, const CustomPlan& pl) {
  Src o;
  const int D = pl.D;
  o.line("// generated by libmdh: one md_hom description, one tuning configuration");
  o.line("typedef long long i64;");
  for (int i = 0; i < D; ++i) o.f("#define N%d %lldLL", i, (long long)pl.N[i]);
  if (d->prelude) o.line(d->prelude);
  o.line(std::string("typedef ") + d->out_type + " mdh_T;");
  o.f("static_assert(sizeof(mdh_T) == %d, \"out_elem_bytes does not match sizeof(out_type)\");", d->out_elem_bytes);
  for (int b = 0; b < d->n_in; ++b)
    o.line(std::string("typedef ") + d->in_type[b] + " mdh_in" + std::to_string(b) + "_t;");

  // scalar function and combine operator
  std::string sig;
  for (int a = 0; a < d->n_acc; ++a) {
    char buf[96];
    snprintf(buf, sizeof buf, "const mdh_in%d_t& a%d, ", d->acc_buf[a], a);
    sig += buf;
  }
  for (int i = 0; i < D; ++i) {
    char buf[48];
    snprintf(buf, sizeof buf, "%si64 i%d", i ? ", " : "", i);
    sig += buf;
  }
  o.line("__device__ __forceinline__ mdh_T mdh_f(" + sig + ") {");
  o.line("  mdh_T r;");
  for (int i = 0; i < D; ++i) o.f("  (void)i%d;", i);
  o.line(d->f);
  o.line("  return r;");
  o.line("}");
  o.line("__device__ __forceinline__ mdh_T mdh_op(const mdh_T& x, const mdh_T& y) {");
  o.line("  mdh_T r;");
  o.line(d->op ? d->op : "  r = x; (void)y;");
  o.line("  return r;");
  o.line("}");

  // emission order of the lane coordinates: the group (reduced / concatenation) of the fast
  // dimension first, the fast dimension first inside it
  std::vector<int> order;
  const int fast_red = pl.red[pl.fast];
  for (int grp = 0; grp < 2; ++grp) {
    const int want = grp == 0 ? fast_red : !fast_red;
    if (pl.red[pl.fast] == want) order.push_back(pl.fast);
    for (int i = D - 1; i >= 0; --i)
      if (i != pl.fast && pl.red[i] == want) order.push_back(i);
  }

  std::string params;
  for (int b = 0; b < d->n_in; ++b) {
    char buf[96];
    snprintf(buf, sizeof buf, "const mdh_in%d_t* __restrict__ in%d, ", b, b);
    params += buf;
  }
  o.line("extern \"C\" __global__ __launch_bounds__(" + std::to_string(pl.NT) + ") void mdh_custom_main(" + params +
         "mdh_T* __restrict__ out, mdh_T* __restrict__ ws) {");
  o.line("  const int tid = (int)threadIdx.x;");
  o.line("  int t_ = tid;");
  for (int i : order) o.f("  const int l%d = t_ %% %lld; t_ /= %lld;", i, (long long)pl.L[i], (long long)pl.L[i]);
  o.line("  unsigned b_ = blockIdx.x;");
  for (int i : order) o.f("  const int g%d = (int)(b_ %% %lldu); b_ /= %lldu;", i, (long long)pl.WG[i], (long long)pl.WG[i]);
  // flat lane index over the reduced dimensions and flat workgroup part over them
  {
    std::string rl = "0", sg = "0";
    int64_t mul = 1, gm = 1;
    for (int i : order)
      if (pl.red[i]) {
        char buf[96];
        snprintf(buf, sizeof buf, " + l%d * %lld", i, (long long)mul);
        rl += buf;
        snprintf(buf, sizeof buf, " + (i64)g%d * %lldLL", i, (long long)gm);
        sg += buf;
        mul *= pl.L[i];
        gm *= pl.WG[i];
      }
    o.line("  const int rl = " + rl + ";");
    o.line("  const i64 sg = " + sg + ";");
  }
  o.line("  (void)rl; (void)sg; (void)ws;");
  if (pl.RL > 1) {
    o.f("  __shared__ mdh_T sh_val[%d];", pl.NT);
    o.f("  __shared__ unsigned char sh_ok[%d];", pl.NT);
  }
  // concatenation dimensions: outer sequential loops; the prefix-sum dimension (which keeps its
  // index set like a concatenation dimension) innermost of them, with a running value across it
  std::string ind = "  ";
  std::vector<int> outer;
  for (int i = 0; i < D; ++i)
    if (!pl.red[i] && i != pl.scan) outer.push_back(i);
  if (pl.scan >= 0) outer.push_back(pl.scan);
  for (int i : outer) {
    if (i == pl.scan) {
      o.f("%smdh_T run;", ind.c_str());
      o.f("%sbool have_run = false;", ind.c_str());
    }
    o.f("%sfor (int q%d = 0; q%d < %lld; ++q%d) {", ind.c_str(), i, i, (long long)pl.Q[i], i);
    ind += "  ";
    o.f("%sconst i64 b%d = %s;", ind.c_str(), i, index_expr(pl, i).c_str());
  }
  // the V register parts of the concatenation dimensions: unrolled loops v<d>, flat index vf.
  // In the scalar phase the indices are clamped to the index space (a ragged edge then computes a
  // duplicate that is never stored), so that validity does not enter the inner loops.
  // lanes whose register parts all lie inside the index space take copies of the scalar phase and
  // of the stores without clamps and bounds checks on the register-blocked dimensions (see below)
  bool clamp_now = true;
  auto covers = [&](int i) { return pl.WG[i] * pl.Q[i] * pl.L[i] * pl.V[i] == pl.N[i]; };
  bool inside_now = false;
  auto open_v = [&](std::string& in, bool clamp) {
    std::string vf = "0", ok = "true";
    for (int i : outer) {
      o.f("%s_Pragma(\"unroll\") for (int v%d = 0; v%d < %lld; ++v%d) {", in.c_str(), i, i, (long long)pl.V[i], i);
      in += "  ";
      // (a dimension whose parts cover its extent exactly needs no clamp: consecutive register parts
      // then read consecutive addresses, which the compiler merges into 8- and 16-byte accesses)
      if (clamp && !covers(i) && (clamp_now || pl.V[i] == 1))
        o.f("%sconst i64 i%d = b%d + v%d < N%d ? b%d + v%d : N%d - 1;", in.c_str(), i, i, i, i, i, i, i);
      else
        o.f("%sconst i64 i%d = b%d + v%d;", in.c_str(), i, i, i);
      vf = "(" + vf + ") * " + std::to_string(pl.V[i]) + " + v" + std::to_string(i);
      if (!covers(i) && (!inside_now || pl.V[i] == 1)) ok += " && i" + std::to_string(i) + " < N" + std::to_string(i);
    }
    o.line(in + "const int vf = " + vf + ";");
    if (!clamp) o.line(in + "const bool cc_ok = " + ok + "; (void)cc_ok;");
    o.line(in + "(void)vf;");
  };
  auto close_v = [&](std::string& in) {
    for (size_t i = 0; i < outer.size(); ++i) {
      in.resize(in.size() - 2);
      o.f("%s}", in.c_str());
    }
  };
  // one evaluation of f for every register part; `first`: the part may still be empty (had == false)
  auto emit_body = [&](std::string in, bool first) {
    open_v(in, true);
    // the accessed elements are copied to registers first: f then works on values, and a
    // conditional between two of them is a register select, not a load through a selected address
    std::string call;
    for (int a = 0; a < d->n_acc; ++a) {
      const std::string b = std::to_string(d->acc_buf[a]), n = std::to_string(a);
      o.line(in + "const mdh_in" + b + "_t e" + n + "_ = in" + b + "[" + d->acc_index[a] + "];");
      call += "e" + n + "_, ";
    }
    for (int i = 0; i < D; ++i) call += (i ? ", i" : "i") + std::to_string(i);
    o.line(in + "const mdh_T v = mdh_f(" + call + ");");
    if (first)
      o.line(in + "if (had) acc[vf] = mdh_op(acc[vf], v); else acc[vf] = v;");
    else
      o.line(in + "acc[vf] = mdh_op(acc[vf], v);");
    close_v(in);
  };
  o.f("%smdh_T acc[%d];", ind.c_str(), pl.VT);
  o.f("%sbool have = false;", ind.c_str());
  std::vector<int> reds;
  for (int i = 0; i < D; ++i)
    if (pl.red[i]) reds.push_back(i);
  auto emit_scalar_phase = [&](std::string ind) {
    if (reds.empty()) {
      o.line(ind + "{");
      o.line(ind + "  const bool had = false;");
      emit_body(ind + "  ", true);
      o.line(ind + "  have = true;");
      o.line(ind + "}");
    } else {
      // outer reduced dimensions: plain loops that skip indices beyond the index space
      std::string ind2 = ind;
      for (size_t k = 0; k + 1 < reds.size(); ++k) {
        const int i = reds[k];
        o.f("%sfor (int q%d = 0; q%d < %lld; ++q%d) {", ind2.c_str(), i, i, (long long)pl.Q[i], i);
        ind2 += "  ";
        o.f("%sconst i64 i%d = %s + 0;", ind2.c_str(), i, index_expr(pl, i).c_str());
        o.f("%sif (i%d >= N%d) continue;", ind2.c_str(), i, i);
      }
      // innermost reduced dimension: the first step may start the part (no neutral element); after it
      // a lane either has a value or has no index at all in this row, so the remaining steps combine
      // unconditionally; rows that lie completely inside the index space run without bounds checks
      const int r = reds.back();
      const long long step = pl.strided ? (long long)(pl.WG[r] * pl.L[r]) : (long long)pl.L[r];
      o.f("%s{", ind2.c_str());
      ind2 += "  ";
      o.f("%sconst int q%d = 0; (void)q%d;", ind2.c_str(), r, r);
      o.f("%sconst i64 r0_ = %s + 0;", ind2.c_str(), index_expr(pl, r).c_str());
      o.f("%sif (r0_ < N%d) {", ind2.c_str(), r);
      o.f("%s  const bool had = have;", ind2.c_str());
      o.f("%s  const i64 i%d = r0_;", ind2.c_str(), r);
      emit_body(ind2 + "  ", true);
      o.f("%s  have = true;", ind2.c_str());
      o.f("%s}", ind2.c_str());
      if (pl.Q[r] > 1) {
        o.f("%sif (r0_ + %lldLL < N%d) {", ind2.c_str(), (long long)(pl.Q[r] - 1) * step, r);
        o.f("%s  _Pragma(\"unroll 4\") for (int s_ = 1; s_ < %lld; ++s_) {", ind2.c_str(), (long long)pl.Q[r]);
        o.f("%s    const i64 i%d = r0_ + s_ * %lldLL;", ind2.c_str(), r, step);
        emit_body(ind2 + "    ", false);
        o.f("%s  }", ind2.c_str());
        o.f("%s} else {", ind2.c_str());
        o.f("%s  for (int s_ = 1; s_ < %lld; ++s_) {", ind2.c_str(), (long long)pl.Q[r]);
        o.f("%s    const i64 i%d = r0_ + s_ * %lldLL;", ind2.c_str(), r, step);
        o.f("%s    if (i%d >= N%d) break;", ind2.c_str(), r, r);
        emit_body(ind2 + "    ", false);
        o.f("%s  }", ind2.c_str());
        o.f("%s}", ind2.c_str());
      }
      ind2.resize(ind2.size() - 2);
      o.f("%s}", ind2.c_str());
      for (size_t k = 0; k + 1 < reds.size(); ++k) {
        ind2.resize(ind2.size() - 2);
        o.f("%s}", ind2.c_str());
      }
    }
  };
  // ragged register-blocked dimensions: the clamp (a select on every index) and the bounds check
  // of every store would keep the compiler from merging the accesses of neighbouring parts, so a
  // lane whose parts all lie inside the index space -- all but those at the edge -- runs a copy
  // without them
  std::string inside;
  for (int i : outer)
    if (i != pl.scan && pl.V[i] > 1 && !covers(i)) {
      char buf[96];
      snprintf(buf, sizeof buf, "%sb%d + %lld <= N%d", inside.empty() ? "" : " && ", i, (long long)pl.V[i], i);
      inside += buf;
    }
  if (inside.empty()) {
    emit_scalar_phase(ind);
  } else {
    o.line(ind + "if (" + inside + ") {");
    clamp_now = false;
    emit_scalar_phase(ind + "  ");
    clamp_now = true;
    o.line(ind + "} else {");
    emit_scalar_phase(ind + "  ");
    o.line(ind + "}");
  }
  // re-composition of every register part: lane -> workgroup in an LDS tree over the lanes of the
  // reduced dimensions, then the output view or the workspace
  auto emit_recompose = [&](std::string in3) {
    open_v(in3, false);
    o.line(in3 + "mdh_T a_ = acc[vf];");
    o.line(in3 + "bool h_ = have;");
    if (pl.RL > 1) {
      const int step = fast_red ? 1 : pl.CL;  // distance in tid between neighbouring reduced-lane indices
      int p2 = 1;
      while (p2 < pl.RL) p2 *= 2;
      o.f("%ssh_val[tid] = a_; sh_ok[tid] = h_ ? 1 : 0;", in3.c_str());
      o.f("%s__syncthreads();", in3.c_str());
      o.f("%sfor (int s_ = %d; s_ > 0; s_ >>= 1) {", in3.c_str(), p2 / 2);
      o.f("%s  if (rl < s_ && rl + s_ < %d) {", in3.c_str(), pl.RL);
      o.f("%s    const int p_ = tid + s_ * %d;", in3.c_str(), step);
      o.f("%s    if (sh_ok[p_]) { if (h_) a_ = mdh_op(a_, sh_val[p_]); else { a_ = sh_val[p_]; h_ = true; } }", in3.c_str());
      o.f("%s    sh_val[tid] = a_; sh_ok[tid] = h_ ? 1 : 0;", in3.c_str());
      o.f("%s  }", in3.c_str());
      o.f("%s  __syncthreads();", in3.c_str());
      o.f("%s}", in3.c_str());
    }
    std::string ccflat = "0";
    for (int i = 0; i < D; ++i)
      if (!pl.red[i]) ccflat = "(" + ccflat + ") * N" + std::to_string(i) + " + i" + std::to_string(i);
    if (pl.scan >= 0) {
      // prefix-sum: the value of this index is the running combination of everything up to it
      o.f("%sif (h_) { if (have_run) run = mdh_op(run, a_); else { run = a_; have_run = true; } }", in3.c_str());
      o.f("%sif (rl == 0 && cc_ok && have_run) {", in3.c_str());
    } else {
      o.f("%sif (rl == 0 && cc_ok && h_) {", in3.c_str());
    }
    for (int i = 0; i < D; ++i)
      if (pl.red[i]) o.f("%s  const i64 i%d = 0; (void)i%d;", in3.c_str(), i, i);
    o.line(in3 + "  const i64 cc_ = " + ccflat + ";");
    const char* val = pl.scan >= 0 ? "run" : "a_";
    if (pl.SG > 1)
      o.f("%s  ws[sg * %lldLL + cc_] = %s;", in3.c_str(), (long long)pl.CCN, val);
    else
      o.line(in3 + "  out[" + (d->out_index ? d->out_index : "cc_") + "] = " + val + "; (void)cc_;");
    o.f("%s}", in3.c_str());
    close_v(in3);
  };
  if (!inside.empty() && pl.RL == 1) {  // no barrier in the re-composition: lanes may take different copies
    o.line(ind + "if (" + inside + ") {");
    inside_now = true;
    emit_recompose(ind + "  ");
    inside_now = false;
    o.line(ind + "} else {");
    emit_recompose(ind + "  ");
    o.line(ind + "}");
  } else {
    emit_recompose(ind);
  }
  for (size_t i = 0; i < outer.size(); ++i) {
    ind.resize(ind.size() - 2);
    o.f("%s}", ind.c_str());
  }
  o.line("}");

  // second pass: fold the workgroup parts of the reduced dimensions in ascending order
  // Few output points and many parts (e.g. Dot): one workgroup per point, the 256 lanes fold strided
  // shares of the parts and meet in an LDS tree (fixed order).  Otherwise one lane per point.
  const bool wide = pl.CCN < 256 && pl.SG > 64;
  o.line("extern \"C\" __global__ __launch_bounds__(256) void mdh_custom_combine(const mdh_T* __restrict__ ws, mdh_T* __restrict__ out) {");
  if (wide) {
    o.line("  __shared__ mdh_T sh_val[256];");
    o.line("  const int tid = (int)threadIdx.x;");
    o.f("  for (i64 cc_ = blockIdx.x; cc_ < %lldLL; cc_ += gridDim.x) {", (long long)pl.CCN);
    o.f("    const i64 parts = %lldLL;", (long long)pl.SG);
    o.line("    mdh_T acc;");
    o.line("    const bool have = tid < parts;");
    o.f("    if (have) { acc = ws[(i64)tid * %lldLL + cc_];", (long long)pl.CCN);
    o.f("      for (i64 s_ = tid + 256; s_ < parts; s_ += 256) acc = mdh_op(acc, ws[s_ * %lldLL + cc_]); }", (long long)pl.CCN);
    o.line("    if (have) sh_val[tid] = acc;");
    o.line("    __syncthreads();");
    o.line("    for (int s_ = 128; s_ > 0; s_ >>= 1) {");
    o.line("      if (tid < s_ && tid + s_ < parts) { acc = mdh_op(acc, sh_val[tid + s_]); sh_val[tid] = acc; }");
    o.line("      __syncthreads();");
    o.line("    }");
    o.line("    if (tid == 0) {");
  } else {
    o.f("  for (i64 cc_ = (i64)blockIdx.x * 256 + threadIdx.x; cc_ < %lldLL; cc_ += (i64)gridDim.x * 256) {", (long long)pl.CCN);
    o.line("    mdh_T acc = ws[cc_];");
    o.f("    for (i64 s_ = 1; s_ < %lldLL; ++s_) acc = mdh_op(acc, ws[s_ * %lldLL + cc_]);", (long long)pl.SG, (long long)pl.CCN);
    o.line("    {");
  }
  o.line("      i64 c_ = cc_;");
  for (int i = D - 1; i >= 0; --i) {
    if (pl.red[i])
      o.f("      const i64 i%d = 0; (void)i%d;", i, i);
    else
      o.f("      const i64 i%d = c_ %% N%d; c_ /= N%d; (void)i%d;", i, i, i, i);
  }
  o.line(std::string("      out[") + (d->out_index ? d->out_index : "cc_") + "] = acc;");
  o.line("    }");
  o.line("  }");
  o.line("}");
  return o.s;
}

}  // namespace
}  // namespace mdh

using namespace mdh;

struct mdh_custom_op {
  CustomPlan plan;
  int n_in;
  int out_bytes;
  std::string source;
  std::vector<char> code;
  std::mutex load_mutex;  // the first run loads the code object; concurrent first runs wait here
  hipModule_t module = nullptr;
  hipFunction_t fmain = nullptr, fcombine = nullptr;
};

extern "C" {

mdh_status mdh_custom_default_params(const mdh_custom_desc* desc, mdh_tile_params* out) {
  if (!desc || !out) return MDH_ERR_NULL;
  if (!desc_ok(desc)) return MDH_ERR_SIZE;
  params_from_custom(default_plan(desc), out);
  return MDH_OK;
}

mdh_status mdh_custom_validate_params(const mdh_custom_desc* desc, const mdh_tile_params* params) {
  if (!desc || !params) return MDH_ERR_NULL;
  if (!desc_ok(desc)) return MDH_ERR_SIZE;
  CustomPlan pl;
  mdh_status st = plan_from_params(desc, params, &pl);
  if (st != MDH_OK) return st;
  return plan_resources(desc, pl);
}

int32_t mdh_custom_num_candidates(const mdh_custom_desc* desc) {
  if (!desc || !desc_ok(desc)) return 0;
  CustomPlan c[64];
  return candidates(desc, c, 64);
}

mdh_status mdh_custom_candidate(const mdh_custom_desc* desc, int32_t idx, mdh_tile_params* out) {
  if (!desc || !out) return MDH_ERR_NULL;
  if (!desc_ok(desc)) return MDH_ERR_SIZE;
  CustomPlan c[64];
  const int n = candidates(desc, c, 64);
  if (idx < 0 || idx >= n) return MDH_ERR_SIZE;
  params_from_custom(c[idx], out);
  return MDH_OK;
}

mdh_status mdh_custom_create(const mdh_custom_desc* desc, const mdh_tile_params* params,
                             mdh_custom_op** out, char* log, size_t log_bytes) {
  if (log && log_bytes) log[0] = 0;
  if (!desc || !out) return MDH_ERR_NULL;
  *out = nullptr;
  if (!desc_ok(desc)) return MDH_ERR_SIZE;
  mdh_status st = desc_ptrs(desc);
  if (st != MDH_OK) return st;
  CustomPlan pl;
  if ((st = plan_from_params(desc, params, &pl)) != MDH_OK) return st;
  if ((st = plan_resources(desc, pl)) != MDH_OK) return st;

  mdh_custom_op* op = new mdh_custom_op;
  op->plan = pl;
  op->n_in = desc->n_in;
  op->out_bytes = desc->out_elem_bytes;
  op->source = generate(desc, pl);

  hiprtcProgram prog;
  if (hiprtcCreateProgram(&prog, op->source.c_str(), "mdh_custom.hip", 0, nullptr, nullptr) != HIPRTC_SUCCESS) {
    delete op;
    return MDH_ERR_LAUNCH;
  }
  // same code generation switches as the rest of the library
  const char* opts[] = {"--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature",
                        "-Xclang", "-packed-fp32-ops"};
  const hiprtcResult rc = hiprtcCompileProgram(prog, (int)(sizeof opts / sizeof opts[0]), opts);
  if (log && log_bytes) {
    size_t n = 0;
    if (hiprtcGetProgramLogSize(prog, &n) == HIPRTC_SUCCESS && n > 1) {
      std::vector<char> full(n + 1, 0);
      hiprtcGetProgramLog(prog, full.data());
      snprintf(log, log_bytes, "%s", full.data());
    }
  }
  if (rc != HIPRTC_SUCCESS) {
    hiprtcDestroyProgram(&prog);
    delete op;
    return MDH_ERR_UNSUPPORTED;
  }
  size_t csz = 0;
  hiprtcGetCodeSize(prog, &csz);
  op->code.resize(csz);
  hiprtcGetCode(prog, op->code.data());
  hiprtcDestroyProgram(&prog);
  *out = op;
  return MDH_OK;
}

const char* mdh_custom_source(const mdh_custom_op* op) { return op ? op->source.c_str() : ""; }

size_t mdh_custom_workspace_size(const mdh_custom_op* op) {
  if (!op || op->plan.SG <= 1) return 0;
  return (size_t)op->plan.SG * (size_t)op->plan.CCN * (size_t)op->out_bytes;
}

mdh_status mdh_custom_run(mdh_custom_op* op, const void* const* inputs, void* output, void* workspace,
                          size_t workspace_bytes, void* stream) {
  if (!op || !inputs || !output) return MDH_ERR_NULL;
  for (int b = 0; b < op->n_in; ++b)
    if (!inputs[b]) return MDH_ERR_NULL;
  const CustomPlan& pl = op->plan;
  if (pl.SG > 1 && (!workspace || workspace_bytes < mdh_custom_workspace_size(op))) return MDH_ERR_WORKSPACE;
  clear_stale_error();
  {
    std::lock_guard<std::mutex> lock(op->load_mutex);
    if (!op->module) {
      // the handle only becomes "loaded" once both kernels have been found
      hipModule_t mod = nullptr;
      hipFunction_t fm = nullptr, fc = nullptr;
      if (hipModuleLoadData(&mod, op->code.data()) != hipSuccess) {
        launch_status();
        return MDH_ERR_LAUNCH;
      }
      if (hipModuleGetFunction(&fm, mod, "mdh_custom_main") != hipSuccess ||
          hipModuleGetFunction(&fc, mod, "mdh_custom_combine") != hipSuccess) {
        launch_status();
        hipModuleUnload(mod);
        return MDH_ERR_LAUNCH;
      }
      op->fmain = fm;
      op->fcombine = fc;
      op->module = mod;
    }
  }
  const void* in[MDH_CUSTOM_MAX_IN];
  void* args[MDH_CUSTOM_MAX_IN + 2];
  int na = 0;
  for (int b = 0; b < op->n_in; ++b) {
    in[b] = inputs[b];
    args[na++] = (void*)&in[b];
  }
  args[na++] = (void*)&output;
  args[na++] = (void*)&workspace;
  const unsigned grid = (unsigned)(pl.SG * pl.CG);
  if (hipModuleLaunchKernel(op->fmain, grid, 1, 1, (unsigned)pl.NT, 1, 1, 0, (hipStream_t)stream, args, nullptr) != hipSuccess) {
    launch_status();
    return MDH_ERR_LAUNCH;
  }
  if (pl.SG > 1) {
    void* cargs[2] = {(void*)&workspace, (void*)&output};
    int64_t blocks = (pl.CCN < 256 && pl.SG > 64) ? pl.CCN : cdiv(pl.CCN, 256);  // as in the generator
    if (blocks > 4096) blocks = 4096;
    if (hipModuleLaunchKernel(op->fcombine, (unsigned)blocks, 1, 1, 256, 1, 1, 0, (hipStream_t)stream, cargs, nullptr) != hipSuccess) {
      launch_status();
      return MDH_ERR_LAUNCH;
    }
  }
  return MDH_OK;
}

mdh_status mdh_custom_tune(const mdh_custom_desc* desc, const void* const* inputs, void* output,
                           void* workspace, size_t workspace_bytes, void* stream, int32_t reps,
                           int32_t max_candidates, mdh_tile_params* best, float* best_ms) {
  if (!desc || !inputs || !output || !best) return MDH_ERR_NULL;
  if (!desc_ok(desc)) return MDH_ERR_SIZE;
  if (reps < 1) reps = 3;
  CustomPlan c[64];
  int n = candidates(desc, c, 64);
  if (max_candidates > 0 && n > max_candidates) n = max_candidates;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return MDH_ERR_LAUNCH;
  if (hipEventCreate(&e1) != hipSuccess) {
    hipEventDestroy(e0);
    return MDH_ERR_LAUNCH;
  }
  float best_t = -1.f;
  mdh_status last = MDH_ERR_UNSUPPORTED;
  for (int i = 0; i < n; ++i) {
    mdh_tile_params p;
    params_from_custom(c[i], &p);
    mdh_custom_op* op = nullptr;
    mdh_status st = mdh_custom_create(desc, &p, &op, nullptr, 0);
    if (st != MDH_OK) {
      last = st;
      continue;
    }
    st = mdh_custom_run(op, inputs, output, workspace, workspace_bytes, stream);  // warm-up, loads the code
    if (st == MDH_OK) {
      hipEventRecord(e0, (hipStream_t)stream);
      for (int r = 0; r < reps && st == MDH_OK; ++r)
        st = mdh_custom_run(op, inputs, output, workspace, workspace_bytes, stream);
      hipEventRecord(e1, (hipStream_t)stream);
      if (hipEventSynchronize(e1) != hipSuccess) st = MDH_ERR_LAUNCH;
    }
    if (st == MDH_OK) {
      float ms = 0.f;
      hipEventElapsedTime(&ms, e0, e1);
      ms /= reps;
      if (best_t < 0.f || ms < best_t) {
        best_t = ms;
        *best = p;
      }
    } else {
      last = st;  // e.g. a candidate that needs more workspace than was given
    }
    mdh_custom_destroy(op);
  }
  hipEventDestroy(e0);
  hipEventDestroy(e1);
  if (best_t < 0.f) return last;
  if (best_ms) *best_ms = best_t;
  return MDH_OK;
}

void mdh_custom_destroy(mdh_custom_op* op) {
  if (!op) return;
  if (op->module) hipModuleUnload(op->module);
  delete op;
}

}  // extern "C"
