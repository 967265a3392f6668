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

template <int QB, int MI, int NI, int WAVES_M, int WAVES_N>
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

  // Input patch, 16 bytes at a time (rows are only dword aligned); cells outside the image read as
  // 0 (they only meet zero filter entries or outputs that are not stored).  A lane's pieces
  // (row ph, offset x) are the same for every tile; only the column origin moves.
  constexpr int PV = 8;  // 16-byte pieces per lane the prefetch can hold (checked by the launcher)
  const int pw4 = PWF >> 2;
  const int npiece = PH * pw4;
  int poff[PV];   // LDS offset of piece i, -1: none
  int pgx[PV];    // offset inside the image row, relative to the tile's first column
  int phy[PV];    // image row
  {
    // piece i of a lane is piece tid + i*NT of the patch: one division for i = 0, then steps of
    // (NT / pw4 rows, NT % pw4 pieces) -- both uniform, passed in by the launcher
    int ph = tid / pw4, x4 = tid - ph * pw4;
#pragma unroll
    for (int i = 0; i < PV; ++i) {
      poff[i] = (tid + i * Cf::NT) < npiece ? ph * PWF + (x4 << 2) : -1;
      pgx[i] = x4 << 2;
      phy[i] = p0 * sh + ph;
      ph += pstep_rows;
      x4 += pstep_x4;
      if (x4 >= pw4) {
        x4 -= pw4;
        ++ph;
      }
    }
  }
  auto load_patch = [&](int q0, f4 (&v)[PV]) {
#pragma unroll
    for (int i = 0; i < PV; ++i) {
      v[i] = (f4){0.f, 0.f, 0.f, 0.f};
      if (poff[i] >= 0 && phy[i] < H) {
        const int gx = q0 * sw * C + pgx[i];
        const int64_t off = ((int64_t)n * H + phy[i]) * WC + gx;
        if (gx < WC) {
          if (off + 3 < in_elems) {
            // a piece that straddles the end of an image row is still one 16-byte load (the next
            // row follows in memory); the elements beyond the row read as 0
            const f4 t = *(const f4u*)(in + off);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[i][e] = gx + e < WC ? t[e] : 0.f;
          } else {  // the last few elements of the whole buffer
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (gx + e < WC) v[i][e] = in[off + e];
          }
        }
      }
    }
  };
  auto store_patch = [&](float* ps, const f4 (&v)[PV]) {
#pragma unroll
    for (int i = 0; i < PV; ++i)
      if (poff[i] >= 0) *(f4*)(ps + poff[i]) = v[i];
  };

  // the lane's pixel inside a block: dp rows down, dq columns right
  const int dp = l32 / QB, dq = l32 % QB;
  const int aoff = ((wm * MI * Cf::RB + dp) * sh) * PWF + dq * sw * C + lh * 4;
  const float* brow = fs + (wn * NI * 32 + l32) * PFR + lh * 4;
  float* obase = out + (int64_t)n * P * Q * K;

  const int tile0 = tq * QT;
  f4 pv[PV];
  load_patch(tile0 * Cf::TQ, pv);  // requested first: in flight while the filter slice is staged

  // Staging without integer divisions in the loops: a filter row k is R*SC contiguous floats in
  // memory, so a lane's elements e = lane, lane+64, ... have the same (r, x) for every k and that
  // split is computed once; wavefronts take the rows k (filter) and ph (patch) in turn.
  {
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
        off[u] = e < RSC ? r * SCP + (e - r * SC) : -1;
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
    // zero the padding of every filter row (x in [SC, SCP)): it meets patch values in the MFMAs
    const int padn = SCP - SC;
    for (int i = tid; i < Cf::BN * R * padn; i += Cf::NT) {
      const int row = i / padn, x = SC + (i - row * padn);
      const int k = row / R, r = row - k * R;
      fs[k * PFR + r * SCP + x] = 0.f;
    }
  }

  store_patch(ps0, pv);
  __syncthreads();

  for (int t = 0; t < QT; ++t) {
    const int q0 = (tile0 + t) * Cf::TQ;
    if (q0 >= Q) break;  // workgroup-uniform
    const float* ps = ps0 + (t & 1) * PH * PWF;
    const bool more = t + 1 < QT && q0 + Cf::TQ < Q;
    if (more) load_patch(q0 + Cf::TQ, pv);  // in flight while this tile is computed

    f16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    // The walk over (r, s*c) in steps of 8, software-pipelined over two operand sets: the LDS reads
    // of step t+1 are issued before the MFMAs of step t.  The scheduling barriers keep the compiler
    // from sinking the reads below the MFMAs (it would then wait for them at once).  sa/sb are the
    // wavefront-uniform offsets of a step in the patch / in the filter row (contiguous over r).
    const float* arow = ps + aoff;
    auto ld = [&](f4 (&af)[MI], f4 (&bf)[NI], int sa, int sb) {
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const float* a = arow + mi * Cf::RB * sh * PWF + sa;
#pragma unroll
        for (int e = 0; e < 4; ++e) af[mi][e] = a[e];
      }
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) bf[ni] = *(const f4*)(brow + ni * 32 * PFR + sb);
    };
    auto mma = [&](const f4 (&af)[MI], const f4 (&bf)[NI]) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(bf[ni][e], af[mi][e], acc[mi][ni], 0, 0, 0);
    };
    {
      const int nsteps = R * (SCP >> 3);
      f4 a0[MI], b0[NI], a1[MI], b1[NI];
      int sa = 0, sb = 0, sc0 = 0;
      ld(a0, b0, 0, 0);
      int st = 0;
      for (; st + 2 <= nsteps; st += 2) {
        sb += 8;
        sa += 8;
        sc0 += 8;
        if (sc0 == SCP) {  // next filter row r: next patch row
          sc0 = 0;
          sa += PWF - SCP;
        }
        ld(a1, b1, sa, sb);
        __builtin_amdgcn_sched_barrier(0);
        mma(a0, b0);
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
        ld(a0, b0, sa, sb);
        __builtin_amdgcn_sched_barrier(0);
        mma(a1, b1);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (st < nsteps) mma(a0, b0);  // odd number of steps
    }

    // output view (n,p,q,k,0,0,0) -> out[n,p,q,k]; the buffer has fewer than 2^31 elements (checked
    // by the caller), so 32-bit offsets are exact.  The filter is the row operand of the MFMA: the
    // lane's pixel is l32 and registers 4g..4g+3 hold channels 8g + 4*lh + (0..3) of the block, one
    // 16-byte store (four times fewer store instructions than with one channel per lane).
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int p = p0 + (wm * MI + mi) * Cf::RB + dp, q = q0 + dq;
      if (p >= P || q >= Q) continue;
      float* o = obase + (p * Q + q) * K;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int k = k0 + (wn * NI + ni) * 32 + 8 * g + 4 * lh;
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

    // the next tile's patch goes to the other buffer (its last readers passed the barrier of the
    // previous iteration)
    if (more) store_patch(ps0 + ((t + 1) & 1) * PH * PWF, pv);
    __syncthreads();
  }
}

template <int QB, int MI, int NI, int WAVES_M, int WAVES_N>
mdh_status launch_t(int QT, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                    int64_t sh, int64_t sw, const float* in, const float* filt, float* out,
                    hipStream_t st) {
  using Cf = FlatCfg<QB, MI, NI, WAVES_M, WAVES_N>;
  if (QT < 1) return MDH_ERR_UNSUPPORTED;
  const int64_t P = (H - R) / sh + 1, Q = (W - S) / sw + 1;
  const int64_t SCP = cdiv(S * C, 8) * 8;
  const int64_t PWF = cdiv((Cf::TQ - 1) * sw * C + SCP + 4, 4) * 4;
  const int64_t PFR = R * SCP + 4;
  const int64_t PH = (Cf::TP - 1) * sh + R;
  const int64_t lds_bytes = (Cf::BN * PFR + 2 * PH * PWF) * 4;
  if (lds_bytes > 160 * 1024) return MDH_ERR_TILE_RESOURCES;
  if (PH * (PWF / 4) > 8 * Cf::NT) return MDH_ERR_TILE_RESOURCES;  // prefetch registers per lane
  auto kern = mcc_flat_kernel<QB, MI, NI, WAVES_M, WAVES_N>;
  static int64_t lds_allowed[kMaxDevices] = {};
  if (allow_dynamic_lds((const void*)kern, lds_bytes, lds_allowed) != MDH_OK) return MDH_ERR_LAUNCH;
  const int64_t tp_n = cdiv(P, Cf::TP), tq_n = cdiv(cdiv(Q, Cf::TQ), QT), tk_n = cdiv(K, Cf::BN);
  const int64_t nblocks = N * tp_n * tq_n * tk_n;
  if (nblocks > 0x7fffffff) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(Cf::NT), (size_t)lds_bytes, st, in, filt, out,
                     (int)H, (int)W, (int)C, (int)K, (int)R, (int)S, (int)sh, (int)sw, (int)P, (int)Q,
                     (int)tp_n, (int)tq_n, (int)tk_n, (int)SCP, (int)PWF, (int)PFR, QT,
                     (int)(Cf::NT / (PWF / 4)), (int)(Cf::NT % (PWF / 4)), N * H * W * C);
  return launch_status();
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
#define MDH_FL(qb, mi, ni, wm, wn)                                                              \
  if (pl.TQ == qb && pl.TP == wm * mi * (32 / qb) && pl.BN == wn * ni * 32 && pl.WM == mi * 32 && \
      pl.WN == ni * 32)                                                                         \
    return launch_t<qb, mi, ni, wm, wn>(pl.QT, N, H, W, C, K, R, S, sh, sw, in, filt, out, st);
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
