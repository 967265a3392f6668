// MatMul instance of md_hom(*, (++,++,+)) for gfx950: C[i,j] = sum_k A[i,k]*B[k,j].
//
// De-composition (tuning parameter 0 / D2 of the paper's table), dims (i,j,k):
//   workgroup layer : (M/BM) x (N/BN) x S     -- S > 1 splits the reduction dimension
//   HBM layer       : K/(S*BK) sequential k-tiles, each staged in LDS (double buffered)
//   wavefront layer : (BM/WM) x (BN/WN)
//   LDS layer       : BK/2 sequential k-steps inside the staged tile
//   VGPR layer      : (WM/32) x (WN/32) accumulator blocks per wavefront
//   block           : 32 x 32 x 2, one v_mfma_f32_32x32x2_f32 (true fp32 multiply-add)
// Re-composition of the + dimension: inside the MFMA accumulators (register region) over
// the sequential parts; if S > 1 the S workgroup results are written to a device-memory
// workspace and a second kernel adds them in ascending part order (workgroup results can
// only be combined in device memory; Appendix "Constraints of Programming Models").
#include "mdh_internal.h"

namespace mdh {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
typedef float f16 __attribute__((ext_vector_type(16)));

template <int BM, int BN, int BK, int WM, int WN>
struct GemmCfg {
  static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN;
  static constexpr int NT = WAVES_M * WAVES_N * 64;
  static constexpr int PA = BK + 4;  // floats per LDS row of the A tile [BM][PA] (k contiguous)
  static constexpr int PB = BN + 4;  // floats per LDS row of the B tile [BK][PB] (n contiguous)
  static constexpr int A_STAGE = BM * PA, B_STAGE = BK * PB;
  static constexpr int STAGE = A_STAGE + B_STAGE;
  static constexpr int LDS_BYTES = 2 * STAGE * 4;
  static constexpr int A_F4 = BM * BK / 4, B_F4 = BK * BN / 4;  // float4 per tile
  static constexpr int A_LD = (A_F4 + NT - 1) / NT, B_LD = (B_F4 + NT - 1) / NT;
  static constexpr int MI = WM / 32, NI = WN / 32;
};

template <int BM, int BN, int BK, int WM, int WN, int MODE>
__device__ __forceinline__ void gemm_tile(const float* __restrict__ A, const float* __restrict__ B,
                                          float* __restrict__ Cout, int M, int N, int K, int m0,
                                          int n0, int kbeg, int kend, float* lds) {
  using C = GemmCfg<BM, BN, BK, WM, WN>;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;
  const int l32 = lane & 31, lh = lane >> 5;

  // register staging of one k-tile on its way from global memory to LDS
  struct Staged {
    f4 a[C::A_LD], b[C::B_LD];
  };

  // MODE 0: interior tile, the reduction extent a multiple of BK -- no checks at all;
  // MODE 1: interior tile, ragged reduction extent -- only the last k-tile is checked (a
  //         workgroup-uniform test per k-tile);  MODE 2: the tile touches the edge of M or N.
  constexpr bool GUARD = MODE == 2;
  auto load_global = [&](Staged& g, int k0) {
    const bool fast = MODE == 0 || (MODE == 1 && k0 + BK <= kend);
#pragma unroll
    for (int x = 0; x < C::A_LD; ++x) {
      const int f = tid + x * C::NT;
      const int row = f / (BK / 4), c4 = f % (BK / 4);
      f4 v = {0.f, 0.f, 0.f, 0.f};
      if (C::A_F4 % C::NT == 0 || f < C::A_F4) {
        const float* p = A + (int64_t)(m0 + row) * K + (k0 + c4 * 4);
        if (fast) {
          v = *(const f4u*)p;
        } else if (m0 + row < M) {
          // edge tiles and ragged k: still one 16-byte load wherever all four elements exist
          if (k0 + c4 * 4 + 3 < kend) {
            v = *(const f4u*)p;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (k0 + c4 * 4 + e < kend) v[e] = p[e];
          }
        }
      }
      g.a[x] = v;
    }
#pragma unroll
    for (int x = 0; x < C::B_LD; ++x) {
      const int f = tid + x * C::NT;
      const int row = f / (BN / 4), c4 = f % (BN / 4);
      f4 v = {0.f, 0.f, 0.f, 0.f};
      if (C::B_F4 % C::NT == 0 || f < C::B_F4) {
        const float* p = B + (int64_t)(k0 + row) * N + (n0 + c4 * 4);
        if (fast) {
          v = *(const f4u*)p;
        } else if (k0 + row < kend) {
          if (n0 + c4 * 4 + 3 < N) {
            v = *(const f4u*)p;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (n0 + c4 * 4 + e < N) v[e] = p[e];
          }
        }
      }
      g.b[x] = v;
    }
  };
  auto store_lds = [&](const Staged& g, float* st) {
#pragma unroll
    for (int x = 0; x < C::A_LD; ++x) {
      const int f = tid + x * C::NT;
      const int row = f / (BK / 4), c4 = f % (BK / 4);
      if (C::A_F4 % C::NT == 0 || f < C::A_F4) *(f4*)(st + row * C::PA + c4 * 4) = g.a[x];
    }
#pragma unroll
    for (int x = 0; x < C::B_LD; ++x) {
      const int f = tid + x * C::NT;
      const int row = f / (BN / 4), c4 = f % (BN / 4);
      if (C::B_F4 % C::NT == 0 || f < C::B_F4) *(f4*)(st + C::A_STAGE + row * C::PB + c4 * 4) = g.b[x];
    }
  };

  f16 acc[C::MI][C::NI];
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  // One MFMA consumes k = {kk, kk+4} (lanes 0-31 supply the first, lanes 32-63 the second
  // column of A / row of B), so that a lane's four consecutive k of A come from one 16-byte
  // LDS read; the order in which the k are added is free (+ is the combine operator of k).
  struct Frag {
    f4 a[C::MI];
    float b[C::NI][4];
  };
  auto load_frag = [&](Frag& f, const float* as, const float* bs, int kk) {
#pragma unroll
    for (int mi = 0; mi < C::MI; ++mi) f.a[mi] = *(const f4*)(as + mi * 32 * C::PA + kk);
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni)
#pragma unroll
      for (int t = 0; t < 4; ++t) f.b[ni][t] = bs[(kk + t) * C::PB + ni * 32];
  };
  auto mma = [&](const Frag& f) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < C::NI; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[mi][t], f.b[ni][t], acc[mi][ni], 0, 0, 0);
  };
  auto compute = [&](const float* st) {
    const float* as = st + (wm * WM + l32) * C::PA + lh * 4;
    const float* bs = st + C::A_STAGE + (lh * 4) * C::PB + wn * WN + l32;
    if (C::MI * C::NI >= 4) {
      // wave tiles of four or more blocks: the fragments of k-step kk+8 are read while the MFMAs of
      // step kk run -- one LDS read, then a few MFMAs, and so on (scheduling groups).  Measured:
      // 4096^3 1.03 -> 1.00 ms; smaller wave tiles are faster with the compiler's own order
      // (1024^3 with 32 x 32 wave tiles: 24.7 us against 27 us).
      constexpr int NR = C::MI + 2 * C::NI, NM = 4 * C::MI * C::NI, PER = NM / NR;
      Frag f[2];
      load_frag(f[0], as, bs, 0);
#pragma unroll
      for (int kk = 0; kk < BK; kk += 8) {
        const int cur = (kk >> 3) & 1;
        if (kk + 8 < BK) load_frag(f[cur ^ 1], as, bs, kk + 8);
        mma(f[cur]);
        if (kk + 8 < BK) {
#pragma unroll
          for (int i = 0; i < NR; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);
          }
          __builtin_amdgcn_sched_group_barrier(0x008, NM - NR * PER, 0);
        }
      }
    } else {
#pragma unroll
      for (int kk = 0; kk < BK; kk += 8) {
        Frag f;
        load_frag(f, as, bs, kk);
        mma(f);
      }
    }
  };

  const int nk = (kend - kbeg + BK - 1) / BK;
  float* const st0 = lds;
  float* const st1 = lds + C::STAGE;
  {
    // two k-tiles in flight: tile kt+2 is requested while tile kt is computed and tile kt+1
    // waits in registers -- twice the bytes in flight per workgroup, for operands that stream
    // from HBM (tall-skinny shapes) rather than from L2 (one tile in flight measured slower on every
    // shape: 4096^3 1.08 against 1.05 ms; 65536 x 64 x 4096 0.32 against 0.31 ms)
    Staged g0, g1;  // g0 carries even tiles, g1 odd tiles
    load_global(g0, kbeg);
    if (nk > 1) load_global(g1, kbeg + BK);
    store_lds(g0, st0);
    __syncthreads();
    for (int kt = 0; kt < nk; kt += 2) {
      if (kt + 2 < nk) load_global(g0, kbeg + (kt + 2) * BK);
      compute(st0);
      if (kt + 1 < nk) store_lds(g1, st1);
      __syncthreads();
      if (kt + 1 < nk) {
        if (kt + 3 < nk) load_global(g1, kbeg + (kt + 3) * BK);
        compute(st1);
        if (kt + 2 < nk) store_lds(g0, st0);
        __syncthreads();
      }
    }
  }

  // output view (i,j,0) -> C[i,j]: accumulator register r of lane l holds
  // row 8*(r/4) + 4*(l/32) + r%4, column l%32 of its 32x32 block
#pragma unroll
  for (int mi = 0; mi < C::MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < C::NI; ++ni) {
      const int col = n0 + wn * WN + ni * 32 + l32;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * WM + mi * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
        if (!GUARD || (row < M && col < N)) Cout[(int64_t)row * N + col] = acc[mi][ni][r];
      }
    }
}

template <int BM, int BN, int BK, int WM, int WN>
__global__ __launch_bounds__((GemmCfg<BM, BN, BK, WM, WN>::NT)) void matmul_kernel(
    const float* __restrict__ A, const float* __restrict__ B, float* __restrict__ C,
    float* __restrict__ ws, int M, int N, int K, int tiles_m, int tiles_n, int S, int kchunk, int jmajor) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  // XCD-aware tile order: workgroup ids are dealt round-robin to the 8 XCDs; hand each XCD a
  // contiguous run of tiles, walked in bands of 8 tile-rows so that the tiles resident on one
  // XCD at a time share few panels of A and B in that XCD's L2.  jmajor: the other loop order of the
  // workgroup layer -- bands of 8 tile-columns, j fastest inside a band.
  int b = blockIdx.x;
  const int nb = gridDim.x;
  if ((nb & 7) == 0) b = (b & 7) * (nb >> 3) + (b >> 3);
  const int tiles = tiles_m * tiles_n;
  const int s = b / tiles;
  int t = b % tiles;
  constexpr int GM = 8;
  const int fast_n = jmajor ? tiles_n : tiles_m, slow_n = jmajor ? tiles_m : tiles_n;  // banded / walked dimension
  const int band = t / (GM * slow_n);
  const int band_w = min(GM, fast_n - band * GM);
  const int in_band = t - band * GM * slow_n;
  const int tf = band * GM + in_band % band_w;
  const int tsl = in_band / band_w;
  const int tm = jmajor ? tsl : tf, tn = jmajor ? tf : tsl;

  const int m0 = tm * BM, n0 = tn * BN;
  const int kbeg = s * kchunk;
  const int kend = min(K, kbeg + kchunk);
  float* out = S > 1 ? ws + (int64_t)s * M * N : C;
  const bool full = (m0 + BM <= M) && (n0 + BN <= N) && kend > kbeg;
  if (full && (kend - kbeg) % BK == 0)
    gemm_tile<BM, BN, BK, WM, WN, 0>(A, B, out, M, N, K, m0, n0, kbeg, kend, lds);
  else if (full)
    gemm_tile<BM, BN, BK, WM, WN, 1>(A, B, out, M, N, K, m0, n0, kbeg, kend, lds);
  else
    gemm_tile<BM, BN, BK, WM, WN, 2>(A, B, out, M, N, K, m0, n0, kbeg, kend, lds);
}

// Second pass of the re-composition: C = part_0 + part_1 + ... + part_{S-1}, in that order.
__global__ __launch_bounds__(256) void combine_sum_kernel(const float* __restrict__ ws,
                                                          float* __restrict__ C, int64_t n, int S) {
  const int64_t i4 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i4 + 3 < n) {
    f4 a = *(const f4u*)(ws + i4);
    for (int s = 1; s < S; ++s) a += *(const f4u*)(ws + (int64_t)s * n + i4);
    *(f4u*)(C + i4) = a;
  } else {
    for (int64_t i = i4; i < n; ++i) {
      float a = ws[i];
      for (int s = 1; s < S; ++s) a += ws[(int64_t)s * n + i];
      C[i] = a;
    }
  }
}

template <int BM, int BN, int BK, int WM, int WN>
mdh_status launch_t(const GemmPlan& pl, int64_t M, int64_t N, int64_t K, const float* A,
                    const float* B, float* C, void* ws, hipStream_t st) {
  using Cfg = GemmCfg<BM, BN, BK, WM, WN>;
  auto kern = matmul_kernel<BM, BN, BK, WM, WN>;
  static int64_t lds_allowed[kMaxDevices] = {};
  if (allow_dynamic_lds((const void*)kern, Cfg::LDS_BYTES, lds_allowed) != MDH_OK) return MDH_ERR_LAUNCH;
  const int64_t tm = cdiv(M, BM), tn = cdiv(N, BN);
  const int64_t kchunk = cdiv(cdiv(K, pl.S), BK) * BK;
  const int64_t nblocks = tm * tn * pl.S;
  if (nblocks > 0x7fffffff) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(Cfg::NT), Cfg::LDS_BYTES, st, A, B, C,
                     (float*)ws, (int)M, (int)N, (int)K, (int)tm, (int)tn, pl.S, (int)kchunk, pl.jmajor);
  mdh_status r = launch_status();
  if (r != MDH_OK || pl.S <= 1) return r;
  const int64_t n = M * N;
  clear_stale_error();
  hipLaunchKernelGGL(combine_sum_kernel, dim3((unsigned)cdiv(n, 1024)), dim3(256), 0, st,
                     (const float*)ws, C, n, pl.S);
  return launch_status();
}

}  // namespace

mdh_status launch_combine_sum(const float* ws, float* dst, int64_t n, int S, hipStream_t st) {
  clear_stale_error();
  hipLaunchKernelGGL(combine_sum_kernel, dim3((unsigned)cdiv(n, 1024)), dim3(256), 0, st, ws, dst, n, S);
  return launch_status();
}

mdh_status launch_matmul(const GemmPlan& pl, int64_t M, int64_t N, int64_t K, const float* A,
                         const float* B, float* C, void* ws, hipStream_t st) {
  if (pl.WK > 1) return launch_matmul_ksplit(pl, M, N, K, A, B, C, ws, st);
#define MDH_MM(bm, bn, bk, wm, wn)                                                   \
  if (pl.BM == bm && pl.BN == bn && pl.BK == bk && pl.WM == wm && pl.WN == wn)       \
    return launch_t<bm, bn, bk, wm, wn>(pl, M, N, K, A, B, C, ws, st);
  MDH_MM(128, 128, 16, 64, 64)
  MDH_MM(256, 128, 16, 128, 64)
  MDH_MM(128, 64, 16, 64, 32)
  MDH_MM(64, 64, 16, 32, 32)
  MDH_MM(128, 128, 32, 64, 64)
  MDH_MM(256, 128, 32, 128, 64)
  MDH_MM(256, 64, 16, 64, 64)
  MDH_MM(256, 64, 32, 64, 64)
  MDH_MM(128, 64, 32, 64, 32)
  MDH_MM(128, 64, 64, 64, 32)
  MDH_MM(256, 64, 64, 64, 64)
  MDH_MM(64, 64, 32, 32, 32)
#undef MDH_MM
  return MDH_ERR_UNSUPPORTED;
}

}  // namespace mdh
