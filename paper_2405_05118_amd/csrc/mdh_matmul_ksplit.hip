// MatMul with the reduction dimension k parallelised on the WAVEFRONT layer, for outputs too small to
// fill the chip with output tiles (MatMul 256^3: 16 tiles of 64 x 64, but 64 tiles of 32 x 32 with eight
// wavefronts each).  De-composition, dims (i,j,k):
//   workgroup layer : (M/BM) x (N/BN) x S        -- BM = 32*MI, BN = 32*NI
//   wavefront layer : 1 x 1 x WK                 -- #PRT(WAVE,k) = WK: every wavefront owns the whole
//                                                   output tile and 1/WK of the workgroup's k-range
//   HBM layer       : sequential groups of 8 k per wavefront, read straight into MFMA operand registers
//                     (no LDS staging: wavefronts of a workgroup share no operand element)
//   VGPR layer      : MI x NI accumulator blocks, 4 MFMA steps per group
//   block           : 32 x 32 x 2, one v_mfma_f32_32x32x2_f32
// Re-composition of k: MFMA accumulators over a wavefront's sequential parts; then the WK wavefront
// results are combined in LDS, added in ascending wavefront order (wavefront results combine in
// shared memory: Appendix "Constraints of Programming Models"; the parameters D2/R3 of the tuning table
// choose this assignment and this memory region); if S > 1, workgroup results go through the
// device-memory workspace and the second pass as in the LDS-tiled kernel.
#include "mdh_internal.h"

namespace mdh {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
typedef float f16 __attribute__((ext_vector_type(16)));

constexpr int SLAB = 32;  // k per wavefront and pipeline stage: 4 groups of 8

template <int MI, int NI>
struct Slab {
  f4 a[MI][SLAB / 8];        // A[row][k0 + g*8 + lh*4 + 0..3]
  float b[NI][SLAB / 8][4];  // B[k0 + g*8 + lh*4 + t][col]
};

template <int MI, int NI, int WK, bool GUARD>
__device__ __forceinline__ void ksplit_tile(const float* __restrict__ A, const float* __restrict__ B,
                                            float* __restrict__ Cout, int M, int N, int K, int m0, int n0,
                                            int kbeg, int kend, float* lds) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l32 = lane & 31, lh = lane >> 5;

  // One MFMA consumes k = {kk, kk+4}: lanes 0-31 supply the first, lanes 32-63 the second, so that a
  // lane's four consecutive k of A are one 16-byte load (the order of the + parts is free).
  auto load = [&](Slab<MI, NI>& s, int k0) {
#pragma unroll
    for (int g = 0; g < SLAB / 8; ++g) {
      const int k = k0 + g * 8 + lh * 4;
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const int row = m0 + mi * 32 + l32;
        const float* p = A + (int64_t)row * K + k;
        f4 v = {0.f, 0.f, 0.f, 0.f};
        if (!GUARD) {
          v = *(const f4u*)p;
        } else if (row < M) {
          if (k + 3 < kend) {
            v = *(const f4u*)p;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (k + e < kend) v[e] = p[e];
          }
        }
        s.a[mi][g] = v;
      }
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) {
        const int col = n0 + ni * 32 + l32;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          float v = 0.f;
          if (!GUARD || (col < N && k + t < kend)) v = B[(int64_t)(k + t) * N + col];
          s.b[ni][g][t] = v;
        }
      }
    }
  };

  f16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  auto mma = [&](const Slab<MI, NI>& s) {
#pragma unroll
    for (int g = 0; g < SLAB / 8; ++g)
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(s.a[mi][g][t], s.b[ni][g][t], acc[mi][ni], 0, 0, 0);
  };

  // the wavefront's sequential parts: slab i+1 is in flight while slab i is multiplied
  const int nslab = (kend - kbeg + SLAB - 1) / SLAB;  // wavefront-uniform; 0 for an empty part
  Slab<MI, NI> s0, s1;
  if (nslab > 0) load(s0, kbeg);
  for (int i = 0; i < nslab; i += 2) {
    if (i + 1 < nslab) load(s1, kbeg + (i + 1) * SLAB);
    mma(s0);
    if (i + 1 < nslab) {
      if (i + 2 < nslab) load(s0, kbeg + (i + 2) * SLAB);
      mma(s1);
    }
  }

  // wavefront layer -> workgroup: all WK partial tiles to LDS (register-major, lane-contiguous: no bank
  // conflicts), one barrier, then every lane adds its share of the tile over the wavefronts in
  // ascending order and stores it through the output view (i,j,0) -> C[i,j]
  constexpr int REGS = MI * NI * 16;
  constexpr int PER = REGS / WK;  // accumulator registers a wavefront folds
  static_assert(REGS % WK == 0, "the tile's registers must divide over the wavefronts");
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) lds[(wave * REGS + (mi * NI + ni) * 16 + r) * 64 + lane] = acc[mi][ni][r];
  __syncthreads();
#pragma unroll
  for (int x = 0; x < PER; ++x) {
    const int q = wave * PER + x;  // register index in the tile: block q/16, register q%16
    float sum = lds[q * 64 + lane];
#pragma unroll
    for (int w = 1; w < WK; ++w) sum += lds[(w * REGS + q) * 64 + lane];
    const int blk = q / 16, r = q % 16;
    const int row = m0 + (blk / NI) * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
    const int col = n0 + (blk % NI) * 32 + l32;
    if (!GUARD || (row < M && col < N)) Cout[(int64_t)row * N + col] = sum;
  }
}

template <int MI, int NI, int WK>
__global__ __launch_bounds__(WK * 64) void matmul_ksplit_kernel(const float* __restrict__ A,
                                                                const float* __restrict__ B,
                                                                float* __restrict__ C, float* __restrict__ ws,
                                                                int M, int N, int K, int tiles_m, int tiles_n,
                                                                int S, int kwave) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  const int tiles = tiles_m * tiles_n;
  const int s = blockIdx.x / tiles;
  const int t = blockIdx.x % tiles;
  const int tm = t / tiles_n, tn = t % tiles_n;
  const int m0 = tm * 32 * MI, n0 = tn * 32 * NI;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kbeg = min(K, (s * WK + wave) * kwave);
  const int kend = min(K, kbeg + kwave);
  float* out = S > 1 ? ws + (int64_t)s * M * N : C;
  // every wavefront takes the same path: the barrier of the combine is reached by all of them
  const bool full = (m0 + 32 * MI <= M) && (n0 + 32 * NI <= N) && (K % ((int64_t)S * WK * SLAB) == 0) &&
                    (kwave % SLAB == 0);
  if (full)
    ksplit_tile<MI, NI, WK, false>(A, B, out, M, N, K, m0, n0, kbeg, kend, lds);
  else
    ksplit_tile<MI, NI, WK, true>(A, B, out, M, N, K, m0, n0, kbeg, kend, lds);
}

// The same de-composition with the 16 x 16 x 4 block (v_mfma_f32_16x16x4_f32): workgroup tile 16 x 16,
// four times the workgroups of the 32 x 32 tile -- for outputs so small that even those leave most of
// the chip idle (256 x 256: 256 workgroups instead of 64).  A wavefront walks groups of 16 k: lane
// (i or j = lane % 16, q = lane / 16) loads A[i][16g + 4q .. 4q+3] as 16 bytes and B[16g + 4q + t][j],
// and MFMA step t of group g consumes k = {16g + 4q + t : q = 0..3}.
typedef float f4v __attribute__((ext_vector_type(4)));

template <int WK, bool GUARD>
__device__ __forceinline__ void ksplit16_tile(const float* __restrict__ A, const float* __restrict__ B,
                                              float* __restrict__ Cout, int M, int N, int K, int m0, int n0,
                                              int kbeg, int kend, float* lds) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l16 = lane & 15, q = lane >> 4;
  constexpr int G = 4;  // groups of 16 k per pipeline stage
  struct Stage {
    f4 a[G];
    float b[G][4];
  };
  auto load = [&](Stage& s, int k0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const int k = k0 + g * 16 + q * 4;
      const int row = m0 + l16, col = n0 + l16;
      const float* p = A + (int64_t)row * K + k;
      f4 v = {0.f, 0.f, 0.f, 0.f};
      if (!GUARD) {
        v = *(const f4u*)p;
      } else if (row < M) {
        if (k + 3 < kend) {
          v = *(const f4u*)p;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (k + e < kend) v[e] = p[e];
        }
      }
      s.a[g] = v;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float w = 0.f;
        if (!GUARD || (col < N && k + t < kend)) w = B[(int64_t)(k + t) * N + col];
        s.b[g][t] = w;
      }
    }
  };
  f4v acc = {0.f, 0.f, 0.f, 0.f};
  auto mma = [&](const Stage& s) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int t = 0; t < 4; ++t) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(s.a[g][t], s.b[g][t], acc, 0, 0, 0);
  };
  constexpr int STAGE_K = G * 16;
  const int nst = (kend - kbeg + STAGE_K - 1) / STAGE_K;
  Stage s0, s1;
  if (nst > 0) load(s0, kbeg);
  for (int i = 0; i < nst; i += 2) {
    if (i + 1 < nst) load(s1, kbeg + (i + 1) * STAGE_K);
    mma(s0);
    if (i + 1 < nst) {
      if (i + 2 < nst) load(s0, kbeg + (i + 2) * STAGE_K);
      mma(s1);
    }
  }
  // wavefront layer -> workgroup in LDS, ascending wavefront order; accumulator register r of lane l
  // is row 4*(l/16) + r, column l%16 of the tile
#pragma unroll
  for (int r = 0; r < 4; ++r) lds[(wave * 4 + r) * 64 + lane] = acc[r];
  __syncthreads();
  constexpr int PER = WK >= 4 ? 1 : 4 / WK;
  if (wave * PER < 4) {
#pragma unroll
    for (int x = 0; x < PER; ++x) {
      const int r = wave * PER + x;
      float sum = lds[r * 64 + lane];
#pragma unroll
      for (int w = 1; w < WK; ++w) sum += lds[(w * 4 + r) * 64 + lane];
      const int row = m0 + 4 * q + r, col = n0 + l16;
      if (!GUARD || (row < M && col < N)) Cout[(int64_t)row * N + col] = sum;
    }
  }
}

template <int WK>
__global__ __launch_bounds__(WK * 64) void matmul_ksplit16_kernel(const float* __restrict__ A,
                                                                  const float* __restrict__ B,
                                                                  float* __restrict__ C, float* __restrict__ ws,
                                                                  int M, int N, int K, int tiles_m, int tiles_n,
                                                                  int S, int kwave) {
  __shared__ float lds[WK * 4 * 64];
  const int tiles = tiles_m * tiles_n;
  const int s = blockIdx.x / tiles;
  const int t = blockIdx.x % tiles;
  const int m0 = (t / tiles_n) * 16, n0 = (t % tiles_n) * 16;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kbeg = min(K, (s * WK + wave) * kwave);
  const int kend = min(K, kbeg + kwave);
  float* out = S > 1 ? ws + (int64_t)s * M * N : C;
  const bool full = (m0 + 16 <= M) && (n0 + 16 <= N) && (K % ((int64_t)S * WK * 64) == 0);
  if (full)
    ksplit16_tile<WK, false>(A, B, out, M, N, K, m0, n0, kbeg, kend, lds);
  else
    ksplit16_tile<WK, true>(A, B, out, M, N, K, m0, n0, kbeg, kend, lds);
}

template <int WK>
mdh_status launch16_t(const GemmPlan& pl, int64_t M, int64_t N, int64_t K, const float* A, const float* B,
                      float* C, void* ws, hipStream_t st) {
  const int64_t tm = cdiv(M, 16), tn = cdiv(N, 16);
  const int64_t kwave = cdiv(cdiv(K, (int64_t)pl.S * WK), 16) * 16;  // whole groups of 16
  const int64_t nblocks = tm * tn * pl.S;
  if (nblocks > 0x7fffffff) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL(matmul_ksplit16_kernel<WK>, dim3((unsigned)nblocks), dim3(WK * 64), 0, st, A, B, C,
                     (float*)ws, (int)M, (int)N, (int)K, (int)tm, (int)tn, pl.S, (int)kwave);
  mdh_status r = launch_status();
  if (r != MDH_OK || pl.S <= 1) return r;
  return launch_combine_sum((const float*)ws, C, M * N, pl.S, st);
}

template <int MI, int NI, int WK>
mdh_status launch_t(const GemmPlan& pl, int64_t M, int64_t N, int64_t K, const float* A, const float* B,
                    float* C, void* ws, hipStream_t st) {
  auto kern = matmul_ksplit_kernel<MI, NI, WK>;
  constexpr int LDS_BYTES = WK * MI * NI * 16 * 64 * 4;
  static int64_t lds_allowed[kMaxDevices] = {};
  if (allow_dynamic_lds((const void*)kern, LDS_BYTES, lds_allowed) != MDH_OK) return MDH_ERR_LAUNCH;
  const int64_t tm = cdiv(M, 32 * MI), tn = cdiv(N, 32 * NI);
  // k per wavefront: whole groups of 8
  const int64_t kwave = cdiv(cdiv(K, (int64_t)pl.S * WK), 8) * 8;
  const int64_t nblocks = tm * tn * pl.S;
  if (nblocks > 0x7fffffff) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(WK * 64), LDS_BYTES, st, A, B, C, (float*)ws, (int)M,
                     (int)N, (int)K, (int)tm, (int)tn, pl.S, (int)kwave);
  mdh_status r = launch_status();
  if (r != MDH_OK || pl.S <= 1) return r;
  return launch_combine_sum((const float*)ws, C, M * N, pl.S, st);
}

}  // namespace

mdh_status launch_matmul_ksplit(const GemmPlan& pl, int64_t M, int64_t N, int64_t K, const float* A,
                                const float* B, float* C, void* ws, hipStream_t st) {
  if (pl.BM == 16 && pl.BN == 16) {
    if (pl.WK == 2) return launch16_t<2>(pl, M, N, K, A, B, C, ws, st);
    if (pl.WK == 4) return launch16_t<4>(pl, M, N, K, A, B, C, ws, st);
    if (pl.WK == 8) return launch16_t<8>(pl, M, N, K, A, B, C, ws, st);
    return MDH_ERR_UNSUPPORTED;
  }
  const int MI = pl.BM / 32, NI = pl.BN / 32;
#define MDH_KS(mi, ni, wk) \
  if (MI == mi && NI == ni && pl.WK == wk) return launch_t<mi, ni, wk>(pl, M, N, K, A, B, C, ws, st);
  MDH_KS(1, 1, 4)
  MDH_KS(1, 1, 8)
  MDH_KS(1, 1, 16)
  MDH_KS(2, 1, 8)
  MDH_KS(2, 2, 4)
  MDH_KS(2, 2, 8)
#undef MDH_KS
  return MDH_ERR_UNSUPPORTED;
}

}  // namespace mdh
