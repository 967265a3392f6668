// MCC_Capsule: multi-channel convolution on 4 x 4 matrices instead of scalars (paper: Section
// "Examples", Subfigure 2; Appendix "Data Characteristics used in Deep Neural Networks": MCC with
// three more dimensions MI, MJ, MK of size 4).  Ten dimensions (n,p,q,k,mi,mj | c,r,s,mk):
//   out[n,p,q,k,mi,mj] = sum_{c,r,s,mk} in[n, p*sh+r, q*sw+s, c, mi, mk] * filt[k, r, s, c, mk, mj]
//
// As a contraction the rows are (pixel, mi), the columns (k, mj) and the reduction (r, s, c, mk).
// In both buffers mk is contiguous for the A operand only; the filter slice is therefore staged in
// LDS with its 4 x 4 matrices transposed ([mj][mk]), after which BOTH MFMA operands are one 16-byte
// LDS read: a lane's four consecutive values are mk = 0..3 of one (s,c) pair, and the two lane
// halves of v_mfma_f32_32x32x2_f32 take two consecutive (s,c) pairs.  s and c are fused into one
// sequential dimension j = s*C + c (adjacent in memory for a fixed r), padded to an even extent
// with zero filter entries.
//
// De-composition:
//   workgroup layer : N x (P/4) x (Q/(8*QT)) x (K/(8*NI))
//   HBM layer       : QT tiles of 8 columns q, walked sequentially: the filter slice is staged once
//                     per workgroup, the input patch (3*sh+R rows) once per tile; the patch of the
//                     next tile is requested into registers before the walk of the current one
//   wavefront layer : 4 output rows p x RW parts of the fused (r, s, c) walk; the RW partial
//                     blocks of a row are added in LDS (two wavefronts per SIMD hide the LDS
//                     latency of the operand reads; the LDS footprint allows one workgroup per CU)
//   block           : (8 k x 4 mj) x (8 q x 4 mi) x 2 of mk; NI blocks along k per wavefront
#include "mdh_internal.h"

namespace mdh {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
typedef float f16 __attribute__((ext_vector_type(16)));

constexpr int CAP_TP = 4, CAP_TQ = 8;

template <int NI, int RW, int CAP_PV>
__global__ __launch_bounds__(256 * RW) void capsule_kernel(const float* __restrict__ in,
                                                         const float* __restrict__ filt,
                                                         float* __restrict__ out, int H, int W, int C,
                                                         int K, int R, int S, int sh, int sw, int P,
                                                         int Q, int tp_n, int tq_n, int tk_n, int J2,
                                                         int PWF, int PFR, int QT, int pstep_rows,
                                                         int pstep_x) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  constexpr int CAP_NT = 256 * RW;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  // wavefront-uniform values are made scalar explicitly: the walk below then runs on scalar
  // loop counters instead of per-lane masks
  const int wave = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);  // output row of the workgroup
  const int rw = __builtin_amdgcn_readfirstlane(tid >> 8);          // part of the reduction walk
  const int l32 = lane & 31, h = lane >> 5;
  int b = blockIdx.x;
  const int nb = gridDim.x;
  if ((nb & 7) == 0) b = (b & 7) * (nb >> 3) + (b >> 3);  // contiguous run of tiles per XCD
  const int tk = b % tk_n;
  const int tq = (b / tk_n) % tq_n;
  const int tp = (b / (tk_n * tq_n)) % tp_n;
  const int n = b / (tk_n * tq_n * tp_n);
  const int p0 = tp * CAP_TP, k0 = tk * (8 * NI);
  const int SCJ = S * C, JP = 2 * J2;
  const int PH = (CAP_TP - 1) * sh + R;
  const int64_t WC16 = (int64_t)W * C * 16;
  float* fs = lds;                   // [8*NI][PFR]: (r*JP + j)*16 + mj*4 + mk
  float* ps = lds + 8 * NI * PFR;    // [PH][PWF]: as in memory, (pixel column, c, mi, mk)
  float* cs = ps + PH * PWF;         // [RW-1][4][NI][16][64]: partial blocks of the upper parts
  // this wavefront's share [t0, t1) of the R*J2 steps of the walk (a step = two (s,c) pairs)
  const int steps = R * J2;
  const int t0 = (steps * rw) / RW, t1 = (steps * (rw + 1)) / RW;

  // The input patch of a column tile travels HBM -> registers -> LDS in 16-byte pieces; piece
  // u*CAP_NT + tid sits in patch row ph at 16-byte column x, and stepping u advances (ph, x) by a
  // fixed amount (CAP_NT = pstep_rows*pw4 + pstep_x, from the host), so only one division is needed.
  // The pieces of the NEXT tile are requested before the MFMA walk of the current one and are
  // written to LDS after it: the HBM/L2 latency hides behind the walk.  Pieces beyond CAP_PV per
  // lane (very wide patches) are staged directly.  CAP_PV is 8 or 16: the smaller one saves registers
  // (a second workgroup per compute unit for short walks).
  const int pw4 = PWF >> 2;
  const int npieces = PH * pw4;
  const int pv_n = (npieces + CAP_NT - 1) / CAP_NT;  // pieces per lane (workgroup-uniform)
  const int ph_first = tid / pw4, x_first = tid - ph_first * pw4;
  const float* img = in + (int64_t)n * H * WC16;
  f4 pre[CAP_PV];
  auto fetch = [&](int q0) {
    int ph = ph_first, x = x_first;
    const int64_t gq = (int64_t)q0 * sw * C * 16;
#pragma unroll
    for (int u = 0; u < CAP_PV; ++u) {
      if (u >= pv_n) break;
      f4 v = {0.f, 0.f, 0.f, 0.f};
      const int hy = p0 * sh + ph;
      const int64_t gx = gq + (x << 2);
      if (u * CAP_NT + tid < npieces && hy < H && gx < WC16) v = *(const f4u*)(img + hy * WC16 + gx);
      pre[u] = v;
      x += pstep_x;
      ph += pstep_rows;
      if (x >= pw4) {
        x -= pw4;
        ++ph;
      }
    }
  };
  auto stash = [&]() {
    int ph = ph_first, x = x_first;
#pragma unroll
    for (int u = 0; u < CAP_PV; ++u) {
      if (u >= pv_n) break;
      if (u * CAP_NT + tid < npieces) *(f4*)(ps + ph * PWF + (x << 2)) = pre[u];
      x += pstep_x;
      ph += pstep_rows;
      if (x >= pw4) {
        x -= pw4;
        ++ph;
      }
    }
  };
  if (tq * QT * CAP_TQ < Q) fetch(tq * QT * CAP_TQ);

  // filter slice: global order [mk][mj] -> LDS order [mj][mk].  A filter row k is R*S*C*16 contiguous
  // floats, so the split of a lane's 16-byte pieces into (r, j, mk) is the same for every k and is
  // computed once; the wavefronts take the rows k in turn (no integer division per element).
  {
    constexpr int NW = CAP_NT / 64;
    const int wid = tid >> 6;
    const int row4 = R * SCJ * 4;  // 16-byte pieces of a filter row
    for (int e0 = 0; e0 < row4; e0 += 256) {
      int off[4], ge[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int e = e0 + u * 64 + lane;  // piece (r, j, mk): mj = 0..3 of one mk
        const int rj = e >> 2, mk = e & 3;
        const int r = rj / SCJ, j = rj - r * SCJ;
        ge[u] = e << 2;
        off[u] = e < row4 ? ((r * JP + j) << 4) + mk : -1;
      }
      for (int k = wid; k < 8 * NI; k += NW) {
        const bool kin = k0 + k < K;
        const float* src = filt + (int64_t)(k0 + k) * row4 * 4;
        f4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
          v[u] = (kin && off[u] >= 0) ? *(const f4u*)(src + ge[u]) : (f4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (off[u] >= 0) {
            float* d = fs + k * PFR + off[u];
#pragma unroll
            for (int mj = 0; mj < 4; ++mj) d[mj * 4] = v[u][mj];
          }
      }
    }
    // zero the padding pair of every filter row r (j in [S*C, JP)): it meets patch values
    if (JP > SCJ)
      for (int i = tid; i < 8 * NI * R * 16; i += CAP_NT) {
        const int e = i & 15, row = i >> 4;
        const int k = row / R, r = row - k * R;
        fs[k * PFR + ((r * JP + SCJ) << 4) + e] = 0.f;
      }
  }

  // patch operand: (dq, mi) of the block; filter operand: (dk, mj); the lane half h takes the odd
  // (s,c) pair
  const int d4 = l32 >> 2, m4 = l32 & 3;
  const float* arow = ps + (wave * sh) * PWF + d4 * sw * C * 16 + h * 16 + m4 * 4;
  const float* brow = fs + d4 * PFR + h * 16 + m4 * 4;
  const int p = p0 + wave;

  // pieces of a patch beyond CAP_PV per lane go straight from memory to LDS
  auto stage_rest = [&](int q0) {
    for (int idx = CAP_PV * CAP_NT + tid; idx < npieces; idx += CAP_NT) {
      const int ph = idx / pw4, x = (idx - ph * pw4) << 2;
      const int hy = p0 * sh + ph;
      const int64_t gx = (int64_t)q0 * sw * C * 16 + x;
      f4 v = {0.f, 0.f, 0.f, 0.f};
      if (hy < H && gx < WC16) v = *(const f4u*)(img + hy * WC16 + gx);
      *(f4*)(ps + ph * PWF + x) = v;
    }
  };
  // input patch of the first tile (cells outside the image read as 0)
  if (tq * QT * CAP_TQ < Q) {
    stash();
    stage_rest(tq * QT * CAP_TQ);
  }
  __syncthreads();

  for (int qt = 0; qt < QT; ++qt) {
    const int q0 = (tq * QT + qt) * CAP_TQ;
    if (q0 >= Q) break;  // workgroup-uniform
    // the patch of this tile is in LDS; the next one is requested now and written to LDS after the walk,
    // BEFORE this tile's results are stored: loads and stores share one in-order counter, and waiting for
    // the patch after the stores were issued would wait for the stores as well
    const bool more = qt + 1 < QT && q0 + CAP_TQ < Q;  // workgroup-uniform
    if (more) fetch(q0 + CAP_TQ);

    f16 acc[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[ni][r] = 0.f;

    {
      // Software pipeline over two operand sets: the LDS reads of step t+1 are issued before the
      // MFMAs of step t, so their latency hides behind 4*NI MFMAs.  The scheduling barriers keep the
      // compiler from sinking the reads below the MFMAs (it would then wait for them at once).
      // sa/sb: wavefront-uniform offsets of the step in the patch row / the filter row.
      int r = t0 / J2, jj = t0 - r * J2;
      int sa = r * PWF + jj * 32, sb = t0 * 32;  // the filter rows are contiguous over (r, j)
      f4 a0 = *(const f4*)(arow + sa), a1;
      f4 b0[NI], b1[NI];
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) b0[ni] = *(const f4*)(brow + sb + ni * 8 * PFR);
      int t = t0;
      for (; t + 2 <= t1; t += 2) {
        sb += 32;
        sa += 32;
        if (++jj == J2) {  // next filter row r: next patch row
          jj = 0;
          sa += PWF - J2 * 32;
        }
        a1 = *(const f4*)(arow + sa);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) b1[ni] = *(const f4*)(brow + sb + ni * 8 * PFR);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
            acc[ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(b0[ni][e], a0[e], acc[ni], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        // operands of step t+2; past the end of the walk the reads repeat step t+1 and are unused
        int na = sa + 32, nj = jj + 1;
        if (nj == J2) {
          nj = 0;
          na += PWF - J2 * 32;
        }
        const bool more = t + 2 < t1;
        sa = more ? na : sa;
        sb = more ? sb + 32 : sb;
        jj = more ? nj : jj;
        a0 = *(const f4*)(arow + sa);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) b0[ni] = *(const f4*)(brow + sb + ni * 8 * PFR);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
            acc[ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(b1[ni][e], a1[e], acc[ni], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (t < t1) {  // odd number of steps
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
            acc[ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(b0[ni][e], a0[e], acc[ni], 0, 0, 0);
      }
    }

    // wavefront -> workgroup: the parts of the reduction walk meet in LDS, added in a fixed order
    if (RW > 1) {
      if (rw > 0) {
        float* c = cs + (((rw - 1) * 4 + wave) * NI) * 16 * 64 + lane;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
          for (int g = 0; g < 16; ++g) c[(ni * 16 + g) * 64] = acc[ni][g];
      }
      __syncthreads();  // also: every wavefront is done reading the patch
      if (rw == 0) {
#pragma unroll
        for (int w = 1; w < RW; ++w) {
          const float* c = cs + (((w - 1) * 4 + wave) * NI) * 16 * 64 + lane;
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int g = 0; g < 16; ++g) acc[ni][g] += c[(ni * 16 + g) * 64];
        }
      }
    } else if (more) {
      __syncthreads();  // every wavefront is done reading the patch
    }
    if (more) {
      stash();
      stage_rest(q0 + CAP_TQ);
    }

    // output view (n,p,q,k,mi,mj,0,0,0,0) -> out[n,p,q,k,mi,mj].  The filter is the row operand of
    // the MFMA, so registers 4g..4g+3 of a lane hold mj = 0..3 of filter k = 2g + h for the lane's
    // (pixel, mi) column: one 16-byte store, and a store instruction writes 128-byte runs.
    if (rw == 0 && p < P) {
      const int q = q0 + d4;
      float* o = out + ((((int64_t)n * P + p) * Q * K) << 4) + m4 * 4;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int k = k0 + ni * 8 + 2 * g + h;
          if (q < Q && k < K)
            *(f4u*)(o + ((q * K + k) << 4)) =
                (f4){acc[ni][4 * g], acc[ni][4 * g + 1], acc[ni][4 * g + 2], acc[ni][4 * g + 3]};
        }
    }
    if (more) __syncthreads();  // the next patch is in LDS
  }
}

struct CapGeom {
  int64_t J2, PWF, PFR, lds_bytes;
};

CapGeom geom(int NI, int RW, int64_t C, int64_t R, int64_t S, int64_t sh, int64_t sw) {
  CapGeom g;
  g.J2 = cdiv(S * C, 2);
  const int64_t JP = 2 * g.J2;
  g.PWF = ((CAP_TQ - 1) * sw * C + JP) * 16 + 4;
  // filter row pitch = 16 (mod 64) floats: the 8 k-rows of a block start in different banks
  const int64_t base = R * JP * 16;
  g.PFR = base + ((16 - base % 64) + 64) % 64;
  g.lds_bytes = (8 * NI * g.PFR + ((CAP_TP - 1) * sh + R) * g.PWF + (RW - 1) * 4 * NI * 16 * 64) * 4;
  return g;
}

template <int NI, int RW, int PV>
mdh_status launch_pv(int QT, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                    int64_t sh, int64_t sw, const float* in, const float* filt, float* out,
                    hipStream_t st) {
  const int64_t P = (H - R) / sh + 1, Q = (W - S) / sw + 1;
  const CapGeom g = geom(NI, RW, C, R, S, sh, sw);
  if (QT < 1) return MDH_ERR_UNSUPPORTED;
  if (g.lds_bytes > 160 * 1024) return MDH_ERR_TILE_RESOURCES;
  auto kern = capsule_kernel<NI, RW, PV>;
  static int64_t lds_allowed[kMaxDevices] = {};
  if (allow_dynamic_lds((const void*)kern, g.lds_bytes, lds_allowed) != MDH_OK) return MDH_ERR_LAUNCH;
  const int64_t tp_n = cdiv(P, CAP_TP), tq_n = cdiv(cdiv(Q, CAP_TQ), QT), tk_n = cdiv(K, 8 * NI);
  const int64_t nblocks = N * tp_n * tq_n * tk_n;
  if (nblocks > 0x7fffffff) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(256 * RW), (size_t)g.lds_bytes, st, in, filt, out,
                     (int)H, (int)W, (int)C, (int)K, (int)R, (int)S, (int)sh, (int)sw, (int)P, (int)Q,
                     (int)tp_n, (int)tq_n, (int)tk_n, (int)g.J2, (int)g.PWF, (int)g.PFR, QT,
                     (int)((256 * RW) / (g.PWF / 4)), (int)((256 * RW) % (g.PWF / 4)));
  return launch_status();
}

template <int NI, int RW>
mdh_status launch_t(int QT, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                    int64_t sh, int64_t sw, const float* in, const float* filt, float* out,
                    hipStream_t st) {
  // 16-byte pieces of the input patch per lane: up to 8 take the instantiation with fewer registers
  const CapGeom g = geom(NI, RW, C, R, S, sh, sw);
  const int64_t pieces = ((CAP_TP - 1) * sh + R) * (g.PWF / 4);
  if (pieces <= 8 * 256 * RW) return launch_pv<NI, RW, 8>(QT, N, H, W, C, K, R, S, sh, sw, in, filt, out, st);
  return launch_pv<NI, RW, 16>(QT, N, H, W, C, K, R, S, sh, sw, in, filt, out, st);
}

}  // namespace

int64_t capsule_lds_bytes(int NI, int RW, int64_t C, int64_t R, int64_t S, int64_t sh, int64_t sw) {
  return geom(NI, RW, C, R, S, sh, sw).lds_bytes;
}

mdh_status launch_capsule(const CapsulePlan& pl, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K,
                          int64_t R, int64_t S, int64_t sh, int64_t sw, const float* in,
                          const float* filt, float* out, hipStream_t st) {
#define MDH_CAP(ni, rw) \
  if (pl.NI == ni && pl.RW == rw) return launch_t<ni, rw>(pl.QT, N, H, W, C, K, R, S, sh, sw, in, filt, out, st);
  MDH_CAP(1, 1)
  MDH_CAP(2, 1)
  MDH_CAP(4, 1)
  MDH_CAP(1, 2)
  MDH_CAP(2, 2)
#undef MDH_CAP
  return MDH_ERR_UNSUPPORTED;
}

}  // namespace mdh
