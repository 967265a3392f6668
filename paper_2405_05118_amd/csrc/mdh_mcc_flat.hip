// Multi-channel convolution for FEW input channels (e.g. the first layer of an image network,
// C = 3, stride 2; paper: Appendix "Data Characteristics used in Deep Neural Networks").
//
// With few channels the reduction dimensions c and s cannot each fill the two-wide k of an
// MFMA, but in NHWC / KRSC they are adjacent in memory: for a fixed row r,
//     in  [n, p*sh + r, q*sw + s, c]  =  row_in [ (q*sw)*C + (s*C + c) ]
//     filt[k, r, s, c]               =  row_flt[ s*C + c ]
// so s and c are re-composed as ONE sequential dimension sc of extent S*C (any order of the +
// parts is a valid evaluation).  sc is padded to a multiple of 8 with zero filter entries.
//
// De-composition, dims (n,p,q,k,c,r,s):
//   workgroup layer : N x (P/TP) x (Q/(QB*QT)) x (K/BN)
//   HBM layer       : QT tiles of QB columns q walked sequentially by a workgroup: the BN x R x S*C
//                     filter slice stays in LDS; the input patch ((TP-1)*sh + R rows of
//                     (QB-1)*sw*C + S*C floats) of the NEXT tile is requested from memory before the
//                     current one is computed and written to the other of two LDS buffers after it
//   wavefront layer : WAVES_M along p  x  WAVES_N along k
//   block           : (32/QB rows of p) x (QB consecutive q) x 32 output channels x 2 of sc
#include <algorithm>

#include "mdh_internal.h"

namespace mdh {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));  // dword-aligned 16-byte access
typedef float f16 __attribute__((ext_vector_type(16)));

template <int QB, int MI, int NI, int WAVES_M, int WAVES_N>
struct FlatCfg {
  static constexpr int RB = 32 / QB;  // output rows per MFMA block
  static constexpr int TP = WAVES_M * MI * RB, TQ = QB;
  static constexpr int BN = WAVES_N * NI * 32;
  static constexpr int NT = WAVES_M * WAVES_N * 64;
};

// Input patch of a tile, 16 bytes at a time (rows are only dword aligned).  Cells of the patch outside
// the image only meet zero filter entries (the padding of s*c) or outputs that are not stored, so any
// FINITE value will do for them: rows below the image are clamped to its last row, pieces beyond the end
// of a row read on into the next row, and only the end of the whole buffer needs care -- an offset
// beyond the last 16 bytes is clamped to them and the piece is shifted back into place when it is
// written to LDS (one tile per launch at most).  No branches, no masks: a handful of instructions per
// piece.  A lane's pieces (patch row, offset) are the same for every tile; only the origin moves.
// 16-byte pieces per lane: a template parameter PV of the kernels (1, 2, 4 or 8, the smallest that holds the
// patch: registers, and no loads that fetch nothing)
constexpr int kPatchPieces = 8;

struct PatchOrigin {   // of one tile; every member is wavefront-uniform
  const float* img;    // first element of the tile's image
  int row0, x0;        // image row of the patch's first row, offset of its first element inside a row
  int lim;             // largest offset inside the image a 16-byte load may start at
};

template <int NT, int PV>
struct PatchPieces {
  // piece i of a lane: (patch row << 16) | offset inside the patch row, -1: none.  One register per
  // piece; the LDS offset and the offset in the image are recomputed where they are used (registers
  // decide how many workgroups share a compute unit here).
  int pk[PV];
  int ph_n, pwf, wc, h;  // rows and padded width of the patch, floats per image row, image rows (uniform)
  // piece i of a lane is piece tid + i*NT of the patch: one division for i = 0, then steps of
  // (NT / pw4 rows, NT % pw4 pieces) -- both uniform, passed in by the launcher
  __device__ __forceinline__ void init(int tid, int PH, int PWF, int WC, int H, int pstep_rows, int pstep_x4) {
    const int pw4 = PWF >> 2;
    const int npiece = PH * pw4;
    ph_n = PH;
    pwf = PWF;
    wc = WC;
    h = H;
    int ph = tid / pw4, x4 = tid - ph * pw4;
#pragma unroll
    for (int i = 0; i < PV; ++i) {
      pk[i] = (tid + i * NT) < npiece ? (ph << 16) | (x4 << 2) : -1;
      ph += pstep_rows;
      x4 += pstep_x4;
      if (x4 >= pw4) {
        x4 -= pw4;
        ++ph;
      }
    }
  }
  // n, row0, x0: wavefront-uniform.  in_elems >= 4 (checked by the launcher).
  __device__ __forceinline__ PatchOrigin origin(const float* __restrict__ in, int n, int row0, int x0,
                                                int64_t in_elems) const {
    const int64_t first = (int64_t)n * h * wc;
    // negative only for a last image of fewer than 4 elements: the clamped load then starts in the image
    // before it, still inside the buffer
    const int64_t room = in_elems - 4 - first;
    PatchOrigin o;
    o.img = in + first;
    o.row0 = row0;
    o.x0 = x0;
    o.lim = room < 0x7fffffff ? (int)room : 0x7fffffff;
    return o;
  }
  __device__ __forceinline__ int offset_of(const PatchOrigin& o, int i) const {
    const int y = min(o.row0 + (pk[i] >> 16), h - 1);
    return y * wc + o.x0 + (pk[i] & 0xffff);
  }
  __device__ __forceinline__ void load(const PatchOrigin& o, f4 (&v)[PV]) const {
#pragma unroll
    for (int i = 0; i < PV; ++i) {
      // no piece: the image's first 16 bytes (never written to LDS); loads without control flow
      const int off = pk[i] >= 0 ? offset_of(o, i) : 0;
      v[i] = *(const f4u*)(o.img + min(off, o.lim));
    }
  }
  __device__ __forceinline__ void store(float* ps, const PatchOrigin& o, const f4 (&v)[PV]) const {
    // the tile at the end of the whole buffer: a piece whose load was moved back by d elements holds its
    // first 4-d elements at positions d..3 (the others lie beyond the buffer and are never used)
    if (min(o.row0 + ph_n, h) * wc - wc + o.x0 + pwf - 4 > o.lim) {
#pragma unroll
      for (int i = 0; i < PV; ++i)
        if (pk[i] >= 0) {
          const int d = offset_of(o, i) - o.lim;
          const f4 t = v[i];
          f4 w;
          w[0] = d <= 0 ? t[0] : d == 1 ? t[1] : d == 2 ? t[2] : t[3];
          w[1] = d <= 0 ? t[1] : d == 1 ? t[2] : t[3];
          w[2] = d <= 0 ? t[2] : t[3];
          w[3] = t[3];
          *(f4*)(ps + (pk[i] >> 16) * pwf + (pk[i] & 0xffff)) = w;
        }
      return;
    }
#pragma unroll
    for (int i = 0; i < PV; ++i)
      if (pk[i] >= 0) *(f4*)(ps + (pk[i] >> 16) * pwf + (pk[i] & 0xffff)) = v[i];
  }
};

// A filter row's s*c values are walked in groups of 8 (4 MFMAs of 2: the lower lane half supplies elements
// 0..3 of a group, the upper half elements 4..7).  The last group of a row has only v = SC mod 8 values:
// it takes ceil(v/2) MFMAs instead of 4 when the lower half supplies its first ceil(v/2) values and the
// upper half the others.  In LDS the group keeps its two 4-float halves (so both halves still read 16
// aligned bytes): value x of the row sits at
__device__ __forceinline__ int last_group_slot(int x, int SC) {
  const int LB = (SC >> 3) << 3, v = SC - LB, nlast = (v + 1) >> 1;
  if (x < LB) return x;
  const int k = x - LB;
  return k < nlast ? LB + k : LB + 4 + (k - nlast);
}

// Filter slice of a workgroup -> LDS: row k holds R groups of SCP floats (s*c padded with zeros).
// Staging without integer divisions in the loops: a filter row k is R*SC contiguous floats in memory, so
// a lane's elements e = lane, lane+64, ... have the same (r, x) for every k and that split is computed
// once; wavefronts take the rows k in turn.
template <class Cf>
__device__ __forceinline__ void stage_filter(float* fs, const float* __restrict__ filt, int k0, int K, int R,
                                             int SC, int SCP, int PFR, int tid, int lane, int wave) {
  constexpr int NW = Cf::NT / 64;
  const int RSC = R * SC;
  for (int e0 = 0; e0 < RSC; e0 += 256) {
    int off[4];  // LDS offset inside a filter row, -1: beyond the row
    int ge[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int e = e0 + u * 64 + lane;
      const int r = e / SC;
      ge[u] = e;
      off[u] = e < RSC ? r * SCP + last_group_slot(e - r * SC, SC) : -1;
    }
    // all loads of a group of 8 rows are issued before the first LDS write: one round trip to
    // memory per group instead of one per row
    constexpr int KI = Cf::BN / NW;  // rows k per wavefront
    constexpr int KG = KI < 8 ? KI : 8;
#pragma unroll
    for (int kb = 0; kb < KI; kb += KG) {
      float v[KG][4];
#pragma unroll
      for (int ki = 0; ki < KG; ++ki) {
        const int k = wave + (kb + ki) * NW;
        const bool kin = k0 + k < K;
        const float* src = filt + (int64_t)(k0 + k) * RSC;
#pragma unroll
        for (int u = 0; u < 4; ++u) v[ki][u] = (kin && off[u] >= 0) ? src[ge[u]] : 0.f;
      }
#pragma unroll
      for (int ki = 0; ki < KG; ++ki) {
        const int k = wave + (kb + ki) * NW;
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (off[u] >= 0) fs[k * PFR + off[u]] = v[ki][u];
      }
    }
  }
  // zero the unused slots of every filter row's last group: they meet patch values in the MFMAs
  const int padn = SCP - SC;
  const int LB = (SC >> 3) << 3, v = SC - LB, nlast = (v + 1) >> 1;
  for (int i = tid; i < Cf::BN * R * padn; i += Cf::NT) {
    const int row = i / padn, pi = i - row * padn;
    const int k = row / R, r = row - k * R;
    const int x = pi < 4 - nlast ? LB + nlast + pi : LB + 4 + (v - nlast) + (pi - (4 - nlast));
    fs[k * PFR + r * SCP + x] = 0.f;
  }
}

// The walk over (r, s*c) in steps of 8 for one tile, software-pipelined over two operand sets: the LDS
// reads of step t+1 are issued before the MFMAs of step t.  The scheduling barriers keep the compiler
// from sinking the reads below the MFMAs (it would then wait for them at once).  sa/sb are the
// wavefront-uniform offsets of a step in the patch / in the filter row (contiguous over r).
// arow: the lane's first patch element; brow: the lane's first filter element.
template <class Cf, int MI, int NI>
__device__ __forceinline__ void walk_tile(const float* arow, const float* brow, int R, int SC, int SCP, int PWF,
                                          int PFR, int sh, int lh, f16 (&acc)[MI][NI]) {
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;
  // the last group of a row (see last_group_slot): nlast MFMAs, and the upper lane half's patch elements
  // start nlast (not 4) after the lower half's
  const int vlast = SC & 7;
  const int nlast = vlast ? (vlast + 1) >> 1 : 4;
  const int afix = lh * (nlast - 4);
  auto is_last = [&](int sc) { return vlast != 0 && sc == SCP - 8; };  // wavefront-uniform
  auto ld = [&](f4 (&af)[MI], f4 (&bf)[NI], int sa, int sb, bool last) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const float* a = arow + mi * Cf::RB * sh * PWF + sa + (last ? afix : 0);
#pragma unroll
      for (int e = 0; e < 4; ++e) af[mi][e] = a[e];
    }
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) bf[ni] = *(const f4*)(brow + ni * 32 * PFR + sb);
  };
  auto mma = [&](const f4 (&af)[MI], const f4 (&bf)[NI], int n) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (e >= n) break;  // wavefront-uniform
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(bf[ni][e], af[mi][e], acc[mi][ni], 0, 0, 0);
    }
  };
  const int nsteps = R * (SCP >> 3);
  f4 a0[MI], b0[NI], a1[MI], b1[NI];
  int sa = 0, sb = 0, sc0 = 0;
  int n0 = is_last(0) ? nlast : 4, n1 = 4;
  ld(a0, b0, 0, 0, is_last(0));
  int st = 0;
  for (; st + 2 <= nsteps; st += 2) {
    sb += 8;
    sa += 8;
    sc0 += 8;
    if (sc0 == SCP) {  // next filter row r: next patch row
      sc0 = 0;
      sa += PWF - SCP;
    }
    n1 = is_last(sc0) ? nlast : 4;
    ld(a1, b1, sa, sb, is_last(sc0));
    __builtin_amdgcn_sched_barrier(0);
    mma(a0, b0, n0);
    __builtin_amdgcn_sched_barrier(0);
    // operands of step st+2; past the end of the walk the reads repeat step st+1 and are unused
    int na = sa + 8, nc = sc0 + 8;
    if (nc == SCP) {
      nc = 0;
      na += PWF - SCP;
    }
    const bool nxt = st + 2 < nsteps;
    sa = nxt ? na : sa;
    sb = nxt ? sb + 8 : sb;
    sc0 = nxt ? nc : sc0;
    n0 = is_last(sc0) ? nlast : 4;
    ld(a0, b0, sa, sb, is_last(sc0));
    __builtin_amdgcn_sched_barrier(0);
    mma(a1, b1, n1);
    __builtin_amdgcn_sched_barrier(0);
  }
  if (st < nsteps) mma(a0, b0, n0);  // odd number of steps
}

// output view (n,p,q,k,0,0,0) -> out[n,p,q,k]; the buffer has fewer than 2^31 elements (checked by the
// caller), so 32-bit offsets are exact.  The filter is the row operand of the MFMA: the lane's pixel is
// l32 and registers 4g..4g+3 hold channels 8g + 4*lh + (0..3) of the block, one 16-byte store (four
// times fewer store instructions than with one channel per lane).
template <class Cf, int MI, int NI>
__device__ __forceinline__ void store_tile(float* obase, const f16 (&acc)[MI][NI], int prow0, int q, int kw0,
                                           int lh, int P, int Q, int K) {
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int p = prow0 + mi * Cf::RB;
    if (p >= P || q >= Q) continue;
    float* o = obase + (p * Q + q) * K;
    if (kw0 + NI * 32 <= K) {  // wavefront-uniform: every channel of the wavefront's blocks exists
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *(f4u*)(o + kw0 + ni * 32 + 8 * g + 4 * lh) = (f4){acc[mi][ni][4 * g], acc[mi][ni][4 * g + 1],
                                                          acc[mi][ni][4 * g + 2], acc[mi][ni][4 * g + 3]};
      continue;
    }
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int k = kw0 + ni * 32 + 8 * g + 4 * lh;
        if (k + 3 < K) {
          *(f4u*)(o + k) = (f4){acc[mi][ni][4 * g], acc[mi][ni][4 * g + 1], acc[mi][ni][4 * g + 2],
                                acc[mi][ni][4 * g + 3]};
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (k + e < K) o[k + e] = acc[mi][ni][4 * g + e];
        }
      }
  }
}

template <int QB, int MI, int NI, int WAVES_M, int WAVES_N, int PV>
__global__ __launch_bounds__((WAVES_M * WAVES_N * 64)) void mcc_flat_kernel(
    const float* __restrict__ in, const float* __restrict__ filt, float* __restrict__ out, int H,
    int W, int C, int K, int R, int S, int sh, int sw, int P, int Q, int tp_n, int tq_n, int tk_n,
    int SCP, int PWF, int PFR, int QT, int pstep_rows, int pstep_x4, int64_t in_elems) {
  using Cf = FlatCfg<QB, MI, NI, WAVES_M, WAVES_N>;
  extern __shared__ __attribute__((aligned(16))) float lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int l32 = lane & 31, lh = lane >> 5;
  int b = blockIdx.x;
  const int nb = gridDim.x;
  if ((nb & 7) == 0) b = (b & 7) * (nb >> 3) + (b >> 3);  // contiguous run of tiles per XCD
  const int tk = b % tk_n;
  const int tq = (b / tk_n) % tq_n;
  const int tp = (b / (tk_n * tq_n)) % tp_n;
  const int n = b / (tk_n * tq_n * tp_n);
  const int p0 = tp * Cf::TP, k0 = tk * Cf::BN;
  const int SC = S * C, WC = W * C;
  const int PH = (Cf::TP - 1) * sh + R;
  float* fs = lds;                    // filter slice [BN][PFR]: row k holds R groups of SCP floats
  float* ps0 = lds + Cf::BN * PFR;    // input patch [2][PH][PWF]: two buffers

  PatchPieces<Cf::NT, PV> pp;
  pp.init(tid, PH, PWF, WC, H, pstep_rows, pstep_x4);
  auto origin = [&](int q0) { return pp.origin(in, n, p0 * sh, q0 * sw * C, in_elems); };

  // the lane's pixel inside a block: dp rows down, dq columns right
  const int dp = l32 / QB, dq = l32 % QB;
  const int aoff = ((wm * MI * Cf::RB + dp) * sh) * PWF + dq * sw * C + lh * 4;
  const float* brow = fs + (wn * NI * 32 + l32) * PFR + lh * 4;
  float* obase = out + (int64_t)n * P * Q * K;

  const int tile0 = tq * QT;
  f4 pv[PV];
  PatchOrigin po = origin(tile0 * Cf::TQ);
  pp.load(po, pv);  // requested first: in flight while the filter slice is staged

  stage_filter<Cf>(fs, filt, k0, K, R, SC, SCP, PFR, tid, lane, wave);

  pp.store(ps0, po, pv);
  __syncthreads();

  for (int t = 0; t < QT; ++t) {
    const int q0 = (tile0 + t) * Cf::TQ;
    if (q0 >= Q) break;  // workgroup-uniform
    const float* ps = ps0 + (t & 1) * PH * PWF;
    const bool more = t + 1 < QT && q0 + Cf::TQ < Q;
    if (more) {  // in flight while this tile is computed
      po = origin(q0 + Cf::TQ);
      pp.load(po, pv);
    }

    f16 acc[MI][NI];
    walk_tile<Cf, MI, NI>(ps + aoff, brow, R, SC, SCP, PWF, PFR, sh, lh, acc);
    // the next tile's patch goes to the other buffer (its last readers passed the barrier of the
    // previous iteration) BEFORE this tile's results are stored: the wait for the patch loads would
    // otherwise also wait for the stores issued after them (one in-order counter for both)
    if (more) pp.store(ps0 + ((t + 1) & 1) * PH * PWF, po, pv);
    store_tile<Cf, MI, NI>(obase, acc, p0 + wm * MI * Cf::RB + dp, q0 + dq, k0 + wn * NI * 32, lh, P, Q, K);
    __syncthreads();
  }
}

// Ticket counters of the kernel below, one per filter slice.  Zero when the library is loaded; the last
// ticket of a launch wraps its counter back to zero (atomic increment with a bound), so every call and
// every graph replay leaves them as it found them.  Calls that overlap on one GPU would share them.
constexpr int kFlatSlices = 8;
static __device__ unsigned g_flat_tickets[kFlatSlices];

// The same de-composition with the workgroup-layer parts of (n, p, q) DEALT OUT instead of owned: G
// workgroups per filter slice stay resident (two per compute unit), stage the slice once and take tiles
// (image, row band, column tile) until none is left -- the first two by position, the others from a
// ticket counter in arrival order.  With 224 workgroups of 7 tiles on 256 compute units an eighth of the
// chip idles; with one workgroup per tile every tile pays the staging of the slice.  A ticket is drawn one
// tile ahead (the patch of the next tile is requested before the current one is computed), handed to the
// other lanes through LDS at the tile's barrier.  `grabs` = tickets all workgroups of a slice draw in
// total (units - G when that is positive): the bound at which the counter wraps.
template <int QB, int MI, int NI, int WAVES_M, int WAVES_N, int PV>
__global__ __launch_bounds__((WAVES_M * WAVES_N * 64)) void mcc_flat_dealt_kernel(
    const float* __restrict__ in, const float* __restrict__ filt, float* __restrict__ out, int H,
    int W, int C, int K, int R, int S, int sh, int sw, int P, int Q, int tp_n, int tq_n, int tk_n,
    int SCP, int PWF, int PFR, int pstep_rows, int pstep_x4, int64_t in_elems, int units, int G,
    unsigned grabs) {
  using Cf = FlatCfg<QB, MI, NI, WAVES_M, WAVES_N>;
  extern __shared__ __attribute__((aligned(16))) float lds[];
  __shared__ int next_unit[2];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int l32 = lane & 31, lh = lane >> 5;
  const int tk = blockIdx.x % tk_n, w = blockIdx.x / tk_n;
  const int k0 = tk * Cf::BN;
  const int SC = S * C, WC = W * C;
  const int PH = (Cf::TP - 1) * sh + R;
  float* fs = lds;                  // filter slice [BN][PFR]
  float* ps0 = lds + Cf::BN * PFR;  // input patch [2][PH][PWF]
  int cur = w, nxt = w + G;
  if (cur >= units) return;  // workgroup-uniform

  PatchPieces<Cf::NT, PV> pp;
  pp.init(tid, PH, PWF, WC, H, pstep_rows, pstep_x4);
  // unit -> (image, row band, column tile), column tiles fastest
  auto origin = [&](int u) {
    const int tq = u % tq_n, band = u / tq_n;
    const int tp = band % tp_n, n = band / tp_n;
    return pp.origin(in, n, tp * Cf::TP * sh, tq * Cf::TQ * sw * C, in_elems);
  };
  const int dp = l32 / QB, dq = l32 % QB;
  const int aoff = ((wm * MI * Cf::RB + dp) * sh) * PWF + dq * sw * C + lh * 4;
  const float* brow = fs + (wn * NI * 32 + l32) * PFR + lh * 4;

  f4 pv[PV];
  PatchOrigin po = origin(cur);
  pp.load(po, pv);  // requested first: in flight while the filter slice is staged
  stage_filter<Cf>(fs, filt, k0, K, R, SC, SCP, PFR, tid, lane, wave);
  pp.store(ps0, po, pv);
  __syncthreads();

  // (declared outside the loop: re-initialising the register every tile would make the compiler wait for
  // the patch loads just issued -- it keeps writes to a register with a pending atomic in order by waiting)
  unsigned ticket = 0;
  for (int it = 0;; ++it) {
    const bool more = nxt < units;  // workgroup-uniform
    if (more) {  // in flight while this tile is computed
      po = origin(nxt);
      pp.load(po, pv);
    }
    if (more && tid == 0) ticket = __builtin_amdgcn_atomic_inc32(&g_flat_tickets[tk], grabs - 1u, __ATOMIC_RELAXED, "agent");

    const int tq = cur % tq_n, band = cur / tq_n;
    const int tp = band % tp_n, n = band / tp_n;
    f16 acc[MI][NI];
    walk_tile<Cf, MI, NI>(ps0 + (it & 1) * PH * PWF + aoff, brow, R, SC, SCP, PWF, PFR, sh, lh, acc);
    // the next tile's patch goes to the other buffer (its last readers passed the barrier of the
    // previous iteration) BEFORE this tile's results are stored: the wait for the patch loads would
    // otherwise also wait for the stores issued after them (one in-order counter for both).  The tile
    // after the next: ticket t is unit 2G + t.
    if (more) {
      pp.store(ps0 + ((it + 1) & 1) * PH * PWF, po, pv);
      if (tid == 0) next_unit[it & 1] = 2 * G + (int)ticket;
    }
    store_tile<Cf, MI, NI>(out + (int64_t)n * P * Q * K, acc, tp * Cf::TP + wm * MI * Cf::RB + dp,
                           tq * Cf::TQ + dq, k0 + wn * NI * 32, lh, P, Q, K);
    if (!more) break;
    __syncthreads();
    cur = nxt;
    // (rewritten two iterations on, after every lane has passed the next barrier; the same value in
    // every lane: kept in a scalar register)
    nxt = __builtin_amdgcn_readfirstlane(next_unit[it & 1]);
  }
}

// Sizes both launchers derive from the tile and the problem, with the checks they share.
struct FlatGeom {
  int64_t P, Q, SCP, PWF, PFR, PH, lds_bytes;
  int pieces;  // 16-byte pieces of a patch per lane
};

template <class Cf>
mdh_status flat_geom(int64_t N, int64_t H, int64_t W, int64_t C, int64_t R, int64_t S, int64_t sh, int64_t sw,
                     FlatGeom* g) {
  g->P = (H - R) / sh + 1;
  g->Q = (W - S) / sw + 1;
  g->SCP = cdiv(S * C, 8) * 8;
  g->PWF = cdiv((Cf::TQ - 1) * sw * C + g->SCP + 4, 4) * 4;
  g->PFR = R * g->SCP + 4;
  g->PH = (Cf::TP - 1) * sh + R;
  g->lds_bytes = (Cf::BN * g->PFR + 2 * g->PH * g->PWF) * 4;
  if (g->lds_bytes > 160 * 1024) return MDH_ERR_TILE_RESOURCES;
  const int64_t pieces = cdiv(g->PH * (g->PWF / 4), Cf::NT);
  if (pieces > kPatchPieces) return MDH_ERR_TILE_RESOURCES;  // prefetch registers per lane
  g->pieces = (int)pieces;
  // 16-byte loads need 16 bytes of input; the piece table packs (row, offset) into one word
  if (N * H * W * C < 4 || g->PH > 0x7fff || g->PWF > 0xffff) return MDH_ERR_UNSUPPORTED;
  return MDH_OK;
}

template <int QB, int MI, int NI, int WAVES_M, int WAVES_N, int PV>
mdh_status launch_owned_pv(const FlatGeom& g, int QT, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K,
                           int64_t R, int64_t S, int64_t sh, int64_t sw, const float* in, const float* filt,
                           float* out, hipStream_t st) {
  using Cf = FlatCfg<QB, MI, NI, WAVES_M, WAVES_N>;
  auto kern = mcc_flat_kernel<QB, MI, NI, WAVES_M, WAVES_N, PV>;
  static int64_t lds_allowed[kMaxDevices] = {};
  if (allow_dynamic_lds((const void*)kern, g.lds_bytes, lds_allowed) != MDH_OK) return MDH_ERR_LAUNCH;
  const int64_t tp_n = cdiv(g.P, Cf::TP), tq_n = cdiv(cdiv(g.Q, Cf::TQ), QT), tk_n = cdiv(K, Cf::BN);
  const int64_t nblocks = N * tp_n * tq_n * tk_n;
  if (nblocks > 0x7fffffff) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(Cf::NT), (size_t)g.lds_bytes, st, in, filt, out,
                     (int)H, (int)W, (int)C, (int)K, (int)R, (int)S, (int)sh, (int)sw, (int)g.P, (int)g.Q,
                     (int)tp_n, (int)tq_n, (int)tk_n, (int)g.SCP, (int)g.PWF, (int)g.PFR, QT,
                     (int)(Cf::NT / (g.PWF / 4)), (int)(Cf::NT % (g.PWF / 4)), N * H * W * C);
  return launch_status();
}

template <int QB, int MI, int NI, int WAVES_M, int WAVES_N, int PV>
mdh_status launch_dealt_pv(const FlatGeom& g, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R,
                           int64_t S, int64_t sh, int64_t sw, const float* in, const float* filt, float* out,
                           hipStream_t st) {
  using Cf = FlatCfg<QB, MI, NI, WAVES_M, WAVES_N>;
  auto kern = mcc_flat_dealt_kernel<QB, MI, NI, WAVES_M, WAVES_N, PV>;
  static int64_t lds_allowed[kMaxDevices] = {};
  if (allow_dynamic_lds((const void*)kern, g.lds_bytes, lds_allowed) != MDH_OK) return MDH_ERR_LAUNCH;
  const int64_t tp_n = cdiv(g.P, Cf::TP), tq_n = cdiv(g.Q, Cf::TQ), tk_n = cdiv(K, Cf::BN);
  const int64_t units = N * tp_n * tq_n;
  if (tk_n > kFlatSlices || units > 0x3fffffff) return MDH_ERR_UNSUPPORTED;
  // resident workgroups per filter slice: what the LDS of 256 compute units holds at once (at most 4 of
  // a workgroup's size per unit), shared between the slices
  const int64_t per_cu = std::min<int64_t>(160 * 1024 / (g.lds_bytes + 64), std::min<int64_t>(4, 2048 / Cf::NT));
  const int64_t G = std::max<int64_t>(1, std::min<int64_t>(units, 256 * std::max<int64_t>(per_cu, 1) / tk_n));
  const int64_t grabs = units > G ? units - G : 0;
  clear_stale_error();
  hipLaunchKernelGGL(kern, dim3((unsigned)(G * tk_n)), dim3(Cf::NT), (size_t)g.lds_bytes, st, in, filt, out, (int)H,
                     (int)W, (int)C, (int)K, (int)R, (int)S, (int)sh, (int)sw, (int)g.P, (int)g.Q, (int)tp_n,
                     (int)tq_n, (int)tk_n, (int)g.SCP, (int)g.PWF, (int)g.PFR, (int)(Cf::NT / (g.PWF / 4)),
                     (int)(Cf::NT % (g.PWF / 4)), N * H * W * C, (int)units, (int)G, (unsigned)grabs);
  return launch_status();
}

// QT >= 1: a workgroup owns QT consecutive column tiles; QT == 0: tiles dealt out
template <int QB, int MI, int NI, int WAVES_M, int WAVES_N>
mdh_status launch_t(int QT, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                    int64_t sh, int64_t sw, const float* in, const float* filt, float* out,
                    hipStream_t st) {
  using Cf = FlatCfg<QB, MI, NI, WAVES_M, WAVES_N>;
  FlatGeom g;
  const mdh_status r = flat_geom<Cf>(N, H, W, C, R, S, sh, sw, &g);
  if (r != MDH_OK) return r;
#define MDH_PV(pv)                                                                                              \
  if (g.pieces <= pv)                                                                                           \
    return QT ? launch_owned_pv<QB, MI, NI, WAVES_M, WAVES_N, pv>(g, QT, N, H, W, C, K, R, S, sh, sw, in, filt, out, st) \
              : launch_dealt_pv<QB, MI, NI, WAVES_M, WAVES_N, pv>(g, N, H, W, C, K, R, S, sh, sw, in, filt, out, st);
  MDH_PV(1)
  MDH_PV(2)
  MDH_PV(4)
  MDH_PV(8)
#undef MDH_PV
  return MDH_ERR_TILE_RESOURCES;
}

}  // namespace

// LDS bytes of the flat kernel for a tile; used by the planner to decide whether it applies.
int64_t mcc_flat_lds_bytes(int QB, int TP, int BN, int64_t C, int64_t R, int64_t S, int64_t sh, int64_t sw) {
  const int64_t SCP = cdiv(S * C, 8) * 8;
  const int64_t PWF = cdiv((QB - 1) * sw * C + SCP + 4, 4) * 4;
  const int64_t PH = (TP - 1) * sh + R;
  if (PH * (PWF / 4) > 8 * 256) return (int64_t)1 << 40;  // the patch prefetch would not fit in registers
  return ((int64_t)BN * (R * SCP + 4) + 2 * PH * PWF) * 4;
}

mdh_status launch_mcc_flat(const MccPlan& pl, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K,
                           int64_t R, int64_t S, int64_t sh, int64_t sw, const float* in,
                           const float* filt, float* out, hipStream_t st) {
  // pl.TQ is the block width QB, pl.TP the rows per workgroup, pl.BN the channels per workgroup
  if (!pl.dealt && pl.QT < 1) return MDH_ERR_UNSUPPORTED;
#define MDH_FL(qb, mi, ni, wm, wn)                                                              \
  if (pl.TQ == qb && pl.TP == wm * mi * (32 / qb) && pl.BN == wn * ni * 32 && pl.WM == mi * 32 && \
      pl.WN == ni * 32)                                                                         \
    return launch_t<qb, mi, ni, wm, wn>(pl.dealt ? 0 : pl.QT, N, H, W, C, K, R, S, sh, sw, in, filt, out, st);
  MDH_FL(16, 1, 2, 4, 1)  // 8 x 16 pixels x 64 channels
  MDH_FL(32, 1, 2, 4, 1)  // 4 x 32 pixels x 64 channels
  MDH_FL(16, 1, 1, 4, 1)  // 8 x 16 pixels x 32 channels
  MDH_FL(32, 1, 1, 4, 1)  // 4 x 32 pixels x 32 channels
  MDH_FL(16, 2, 2, 2, 2)  // 8 x 16 pixels x 128 channels
  MDH_FL(32, 2, 2, 2, 2)  // 4 x 32 pixels x 128 channels
  MDH_FL(16, 1, 1, 4, 2)  // 8 x 16 pixels x 64 channels, eight wavefronts
  MDH_FL(32, 1, 1, 4, 2)  // 4 x 32 pixels x 64 channels, eight wavefronts
  MDH_FL(16, 1, 1, 8, 1)  // 16 x 16 pixels x 32 channels, eight wavefronts
  MDH_FL(32, 1, 1, 8, 1)  // 8 x 32 pixels x 32 channels, eight wavefronts
#undef MDH_FL
  return MDH_ERR_UNSUPPORTED;
}

}  // namespace mdh
