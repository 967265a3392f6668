// Multi-channel convolution instance of md_hom(*, (++,++,++,++,+,+,+)) for gfx950:
//   out[n,p,q,k] = sum_{c,r,s} in[n, p*sh + r, q*sw + s, c] * filt[k,r,s,c]      (NHWC, KRSC, NPQK)
// (paper: Section "Examples", Subfigure 2: index functions p+r, q+s read neighbouring cells).
//
// De-composition, dims (n,p,q,k,c,r,s):
//   workgroup layer : N x (P/TP) x (Q/TQ) x (K/BN) x SC -- one TP x TQ patch of output pixels of one
//                     image and BN output channels per workgroup; SC > 1 splits the reduction
//                     dimension c (small images with many channels would otherwise leave compute
//                     units idle): the SC partial outputs go to a device-memory workspace and the
//                     second pass of MatMul adds them in ascending part order
//   HBM layer       : C/(SC*CK) sequential channel chunks; per chunk the (TP-1)*sh+R by (TQ-1)*sw+S
//                     input patch is staged ONCE in LDS and reused by all R*S filter taps
//   LDS layer       : R x S filter taps x CK/2 channel steps, sequential inside the staged patch;
//                     the BN x CK filter slice of a tap is staged in LDS (double buffered)
//   wavefront layer : rows of the patch x (BN/WN)
//   VGPR layer      : (WM/32) x (WN/32) accumulator blocks per wavefront
//   block           : (32/TQ rows of p) x (TQ consecutive q) x 32 output channels x 2 input channels
//                     per v_mfma_f32_32x32x2_f32; TQ = 32, or 16 / 8 for images narrower than 32
//                     output columns (a block then spans 2 / 4 output rows instead of idle lanes)
// The three + dimensions are re-composed inside the MFMA accumulators (register region); the
// order c-chunk, r, s, c is free because + is their common combine operator.
#include "mdh_internal.h"

namespace mdh {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
typedef float f16 __attribute__((ext_vector_type(16)));

template <int TP, int TQ, int BN, int CK, int WM, int WN>
struct MccCfg {
  static_assert(TQ == 32 || TQ == 16 || TQ == 8, "an MFMA block spans 32 pixels: 32/TQ rows of TQ columns");
  static constexpr int RB = 32 / TQ;  // output rows per block
  static constexpr int MI = WM / 32, NI = WN / 32;
  static_assert(TP % (MI * RB) == 0, "rows of the tile = wavefronts x blocks x rows per block");
  static constexpr int WAVES_M = TP / (MI * RB), WAVES_N = BN / WN;
  static constexpr int NT = WAVES_M * WAVES_N * 64;
  static constexpr int PC = CK + 4;  // floats per staged pixel / filter row (c contiguous)
  static constexpr int F_STAGE = BN * PC;
  static constexpr int F_F4 = BN * CK / 4;
  static constexpr int F_LD = (F_F4 + NT - 1) / NT;
};

template <int TP, int TQ, int BN, int CK, int WM, int WN, int MODE>
__device__ __forceinline__ void mcc_tile(const float* __restrict__ in, const float* __restrict__ filt,
                                         float* __restrict__ out, int H, int W, int C, int K, int R,
                                         int S, int sh, int sw, int P, int Q, int n, int p0, int q0,
                                         int k0, int cbeg, int cend, float* lds) {
  using Cf = MccCfg<TP, TQ, BN, CK, WM, WN>;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / Cf::WAVES_N, wn = wave % Cf::WAVES_N;
  const int l32 = lane & 31, lh = lane >> 5;
  const int PH = (TP - 1) * sh + R, PW = (TQ - 1) * sw + S;
  float* fs = lds;                        // two filter stages
  float* ps = lds + 2 * Cf::F_STAGE;      // input patch [PH][PW][PC]
  const int npix = PH * PW;

  f16 acc[Cf::MI][Cf::NI];
#pragma unroll
  for (int mi = 0; mi < Cf::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < Cf::NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  f4 gf[Cf::F_LD];
  // MODE 0: interior tile, whole channel chunks -- no checks at all;  MODE 1: interior tile, the
  // last channel chunk incomplete -- only that chunk is checked (a workgroup-uniform test per
  // chunk);  MODE 2: the tile touches the edge of p, q or k.
  constexpr bool GUARD = MODE == 2;
  auto load_filter = [&](int r, int s, int c0) {
    const bool fast = MODE == 0 || (MODE == 1 && c0 + CK <= cend);
#pragma unroll
    for (int x = 0; x < Cf::F_LD; ++x) {
      const int f = tid + x * Cf::NT;
      const int kk = f / (CK / 4), c4 = f % (CK / 4);
      f4 v = {0.f, 0.f, 0.f, 0.f};
      if (Cf::F_F4 % Cf::NT == 0 || f < Cf::F_F4) {
        const float* p = filt + (((int64_t)(k0 + kk) * R + r) * S + s) * C + c0 + c4 * 4;
        if (fast) {
          v = *(const f4u*)p;
        } else if (k0 + kk < K) {
          // edge tiles and ragged channel counts: one 16-byte load wherever all four channels exist
          if (c0 + c4 * 4 + 3 < cend) {
            v = *(const f4u*)p;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (c0 + c4 * 4 + e < cend) v[e] = p[e];
          }
        }
      }
      gf[x] = v;
    }
  };
  auto store_filter = [&](float* st) {
#pragma unroll
    for (int x = 0; x < Cf::F_LD; ++x) {
      const int f = tid + x * Cf::NT;
      const int kk = f / (CK / 4), c4 = f % (CK / 4);
      if (Cf::F_F4 % Cf::NT == 0 || f < Cf::F_F4) *(f4*)(st + kk * Cf::PC + c4 * 4) = gf[x];
    }
  };
  auto stage_patch = [&](int c0) {
    const bool fast = MODE == 0 || (MODE == 1 && c0 + CK <= cend);
    const int total = npix * (CK / 4);
    for (int f = tid; f < total; f += Cf::NT) {
      const int pix = f / (CK / 4), c4 = f % (CK / 4);
      const int ph = pix / PW, pw = pix - ph * PW;
      const int hy = p0 * sh + ph, wx = q0 * sw + pw;
      f4 v = {0.f, 0.f, 0.f, 0.f};
      const float* p = in + (((int64_t)n * H + hy) * W + wx) * C + c0 + c4 * 4;
      if (fast) {
        v = *(const f4u*)p;
      } else if (hy < H && wx < W) {
        if (c0 + c4 * 4 + 3 < cend) {
          v = *(const f4u*)p;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (c0 + c4 * 4 + e < cend) v[e] = p[e];
        }
      }
      *(f4*)(ps + pix * Cf::PC + c4 * 4) = v;
    }
  };
  // lanes 0-31 of an MFMA supply channels {cc..cc+3}, lanes 32-63 {cc+4..cc+7} of both operands
  struct Frag {
    f4 a[Cf::MI], b[Cf::NI];
  };
  const int a_row = Cf::RB * sh * PW * Cf::PC;  // LDS distance between consecutive blocks of a wavefront
  const int dp = l32 / TQ, dq = l32 % TQ;      // the lane's pixel inside a block
  auto load_frag = [&](Frag& f, const float* as, const float* bs, int cc) {
#pragma unroll
    for (int mi = 0; mi < Cf::MI; ++mi) f.a[mi] = *(const f4*)(as + mi * a_row + cc);
#pragma unroll
    for (int ni = 0; ni < Cf::NI; ++ni) f.b[ni] = *(const f4*)(bs + ni * 32 * Cf::PC + cc);
  };
  auto mma = [&](const Frag& f) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int mi = 0; mi < Cf::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < Cf::NI; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[mi][t], f.b[ni][t], acc[mi][ni], 0, 0, 0);
  };
  auto compute = [&](const float* fst, int r, int s) {
    const float* as = ps + (((wm * Cf::MI * Cf::RB + dp) * sh + r) * PW + dq * sw + s) * Cf::PC + lh * 4;
    const float* bs = fst + (wn * WN + l32) * Cf::PC + lh * 4;
#pragma unroll
    for (int cc = 0; cc < CK; cc += 8) {
      Frag f;
      load_frag(f, as, bs, cc);
      mma(f);
    }
  };

  const int taps = R * S;
  for (int c0 = cbeg; c0 < cend; c0 += CK) {
    __syncthreads();  // every wavefront is done with the previous patch and filter stages
    stage_patch(c0);
    load_filter(0, 0, c0);
    store_filter(fs);
    __syncthreads();
    int r = 0, s = 0;
    for (int tap = 0; tap < taps; ++tap) {
      float* cur = fs + (tap & 1) * Cf::F_STAGE;
      float* nxt = fs + ((tap + 1) & 1) * Cf::F_STAGE;
      int rn = r, sn = s + 1;
      if (sn == S) {
        sn = 0;
        rn = r + 1;
      }
      if (tap + 1 < taps) load_filter(rn, sn, c0);
      compute(cur, r, s);
      if (tap + 1 < taps) store_filter(nxt);
      __syncthreads();
      r = rn;
      s = sn;
    }
  }

  // output view (n,p,q,k,0,0,0) -> out[n,p,q,k]
#pragma unroll
  for (int mi = 0; mi < Cf::MI; ++mi) {
#pragma unroll
    for (int ni = 0; ni < Cf::NI; ++ni) {
      const int k = k0 + wn * WN + ni * 32 + l32;
#pragma unroll
      for (int rg = 0; rg < 16; ++rg) {
        const int pix = 8 * (rg / 4) + 4 * lh + (rg % 4);  // pixel of the block this register holds
        const int p = p0 + (wm * Cf::MI + mi) * Cf::RB + pix / TQ;
        const int q = q0 + pix % TQ;
        if (!GUARD || (p < P && q < Q && k < K))
          out[(((int64_t)n * P + p) * Q + q) * K + k] = acc[mi][ni][rg];
      }
    }
  }
}

// Wave tiles of up to four blocks are held to the registers of three wavefronts per SIMD: LDS (50 KB
// at the default tile) admits three workgroups per compute unit, and without the bound the kernel
// takes 184 registers and runs two (ResNet-50 configuration: 4.95 -> 4.87 ms).
template <int TP, int TQ, int BN, int CK, int WM, int WN>
__global__ __launch_bounds__((MccCfg<TP, TQ, BN, CK, WM, WN>::NT),
                             (MccCfg<TP, TQ, BN, CK, WM, WN>::MI * MccCfg<TP, TQ, BN, CK, WM, WN>::NI <= 4 ? 3 : 1)) void mcc_kernel(
    const float* __restrict__ in, const float* __restrict__ filt, float* __restrict__ out,
    float* __restrict__ ws, int H, int W, int C, int K, int R, int S, int sh, int sw, int P, int Q,
    int tp_n, int tq_n, int tk_n, int n_img, int SC, int cchunk) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  // XCD-aware order: each of the 8 XCDs gets a contiguous run of tiles; inside a run the
  // channel tiles of one pixel patch come first (they share the patch), then q, p, n.
  int b = blockIdx.x;
  const int nb = gridDim.x;
  if ((nb & 7) == 0) b = (b & 7) * (nb >> 3) + (b >> 3);
  const int tk = b % tk_n;
  const int tq = (b / tk_n) % tq_n;
  const int tp = (b / (tk_n * tq_n)) % tp_n;
  const int n = (b / (tk_n * tq_n * tp_n)) % n_img;
  const int sc = b / (tk_n * tq_n * tp_n * n_img);  // part of the reduction dimension c
  const int p0 = tp * TP, q0 = tq * TQ, k0 = tk * BN;
  const int cbeg = sc * cchunk, cend = min(C, cbeg + cchunk);
  float* dst = SC > 1 ? ws + (int64_t)sc * n_img * P * Q * K : out;
  const bool full = (p0 + TP <= P) && (q0 + TQ <= Q) && (k0 + BN <= K);
  if (full && (cend - cbeg) % CK == 0)
    mcc_tile<TP, TQ, BN, CK, WM, WN, 0>(in, filt, dst, H, W, C, K, R, S, sh, sw, P, Q, n, p0, q0, k0, cbeg, cend, lds);
  else if (full)
    mcc_tile<TP, TQ, BN, CK, WM, WN, 1>(in, filt, dst, H, W, C, K, R, S, sh, sw, P, Q, n, p0, q0, k0, cbeg, cend, lds);
  else
    mcc_tile<TP, TQ, BN, CK, WM, WN, 2>(in, filt, dst, H, W, C, K, R, S, sh, sw, P, Q, n, p0, q0, k0, cbeg, cend, lds);
}

template <int TP, int TQ, int BN, int CK, int WM, int WN>
mdh_status launch_t(int SC, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                    int64_t sh, int64_t sw, const float* in, const float* filt, float* out, void* ws,
                    hipStream_t st) {
  using Cf = MccCfg<TP, TQ, BN, CK, WM, WN>;
  const int64_t P = (H - R) / sh + 1, Q = (W - S) / sw + 1;
  const int64_t PH = (TP - 1) * sh + R, PW = (TQ - 1) * sw + S;
  const int64_t lds_bytes = (2ll * Cf::F_STAGE + PH * PW * Cf::PC) * 4;
  if (lds_bytes > 160 * 1024) return MDH_ERR_TILE_RESOURCES;
  auto kern = mcc_kernel<TP, TQ, BN, CK, WM, WN>;
  static int64_t lds_allowed[kMaxDevices] = {};
  if (allow_dynamic_lds((const void*)kern, lds_bytes, lds_allowed) != MDH_OK) return MDH_ERR_LAUNCH;
  const int64_t tp_n = cdiv(P, TP), tq_n = cdiv(Q, TQ), tk_n = cdiv(K, BN);
  if (SC < 1) return MDH_ERR_UNSUPPORTED;
  const int64_t cchunk = cdiv(cdiv(C, SC), CK) * CK;
  if ((SC - 1) * cchunk >= C) return MDH_ERR_TILE_NOT_DIVIDING;  // a part without channels
  const int64_t nblocks = N * tp_n * tq_n * tk_n * SC;
  if (nblocks > 0x7fffffff) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(Cf::NT), (size_t)lds_bytes, st, in, filt, out,
                     (float*)ws, (int)H, (int)W, (int)C, (int)K, (int)R, (int)S, (int)sh, (int)sw, (int)P,
                     (int)Q, (int)tp_n, (int)tq_n, (int)tk_n, (int)N, SC, (int)cchunk);
  mdh_status r = launch_status();
  if (r != MDH_OK || SC <= 1) return r;
  return launch_combine_sum((const float*)ws, out, N * P * Q * K, SC, st);
}

}  // namespace

mdh_status launch_mcc(const MccPlan& pl, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K,
                      int64_t R, int64_t S, int64_t sh, int64_t sw, const float* in,
                      const float* filt, float* out, void* ws, hipStream_t st) {
#define MDH_MCC(tp, tq, bn, ck, wm, wn)                                                          \
  if (pl.TP == tp && pl.TQ == tq && pl.BN == bn && pl.CK == ck && pl.WM == wm && pl.WN == wn)    \
    return launch_t<tp, tq, bn, ck, wm, wn>(pl.S, N, H, W, C, K, R, S, sh, sw, in, filt, out, ws, st);
  MDH_MCC(4, 32, 128, 16, 64, 64)
  MDH_MCC(8, 32, 128, 16, 128, 64)
  MDH_MCC(2, 32, 64, 16, 32, 32)
  MDH_MCC(4, 32, 64, 16, 64, 32)
  MDH_MCC(8, 16, 128, 16, 64, 64)  // blocks of 2 x 16 pixels
  MDH_MCC(8, 16, 64, 16, 64, 32)
  MDH_MCC(8, 8, 128, 16, 32, 64)   // blocks of 4 x 8 pixels
  MDH_MCC(8, 8, 64, 16, 32, 32)
  MDH_MCC(4, 32, 128, 32, 64, 64)  // channel chunks of 32
  MDH_MCC(4, 32, 64, 32, 64, 32)
  MDH_MCC(8, 16, 128, 32, 64, 64)
  MDH_MCC(8, 16, 64, 32, 64, 32)
  MDH_MCC(8, 8, 128, 32, 32, 64)
  MDH_MCC(8, 8, 64, 32, 32, 32)
#undef MDH_MCC
  return MDH_ERR_UNSUPPORTED;
}

}  // namespace mdh
