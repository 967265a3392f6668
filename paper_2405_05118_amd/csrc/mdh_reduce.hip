// Pure-reduction instances for gfx950: Dot = md_hom(*, (+)) and MatVec = md_hom(*, (++,+))
// (paper: Section "Examples", Subfigure 1; MatVec is also the worked example of Section
// "Low-Level Representation").  Both are bound by HBM traffic (every input element is used
// once), and in both the reduction dimension k is the contiguous one, so it is assigned to the
// lanes for coalescing and its re-composition uses every level of the ladder:
//   VGPR      : a lane adds its own sequential parts (4 independent accumulators)
//   lane      : across the 64 lanes of a wavefront in registers -- DPP quad permutes and row
//               mirrors, ds_swizzle across the 16-lane rows, v_readlane across the two halves
//               (lanes within a wavefront may combine in registers; Appendix "Constraints of
//               Programming Models")
//   wavefront : across the wavefronts of a workgroup in LDS
//   workgroup : if k is split over workgroups, partial results in a device-memory workspace and
//               a second kernel that adds them in ascending part order
// Every level adds in a fixed order, so results are bit-identical run to run.
#include "mdh_internal.h"

namespace mdh {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));

template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}

// Sum over the 64 lanes of the wavefront; every lane returns the same value.
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp<0xB1>(v);   // quad_perm [1,0,3,2]: pairs
  v += dpp<0x4E>(v);   // quad_perm [2,3,0,1]: quads
  v += dpp<0x141>(v);  // row_half_mirror: 8 lanes
  v += dpp<0x140>(v);  // row_mirror: a 16-lane row
  // xor 16 inside each group of 32 lanes: and_mask 0x1f, or_mask 0, xor_mask 0x10
  v += __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));
  const float lo = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
  const float hi = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
  return lo + hi;
}

__device__ __forceinline__ float hsum(f4 a) { return (a[0] + a[1]) + (a[2] + a[3]); }

// ------------------------------------------------------------------------------------- Dot

// How many workgroup parts have stored their partial sum.  Zero when the library is loaded; the S-th
// arrival wraps it back to zero (atomicInc with bound S-1), so every call leaves it as it found it.
static __device__ unsigned g_dot_arrivals;

// The S workgroup-layer parts in a fixed order: 16 independent loads per lane and round (one round covers
// S = 1024), so that the loads overlap instead of each addition waiting for its own load.  Called by one
// whole wavefront; every lane returns the sum.
template <bool COHERENT>
__device__ __forceinline__ float dot_fold_parts(const float* __restrict__ ws, int S, int lane) {
  float a = 0.f;
  for (int base = 0; base < S; base += 1024) {
    float v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int i = base + u * 64 + lane;
      v[u] = i < S ? (COHERENT ? coherent_load(ws + i) : ws[i]) : 0.f;
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) a += v[u];
  }
  return wave_sum(a);
}

// STRIDED (parameter D2 of the tuning table, lane and wavefront layers): true = consecutive lanes own
// consecutive 4-element parts and walk the workgroup's chunk in steps of a whole workgroup (coalesced:
// the paper's "inner parallelism"); false = blocked, every lane owns ONE contiguous part of the chunk
// ("outer parallelism": valid, and slow on this hardware because the lanes of a load are far apart).
// FUSED: S > 1 only -- the last workgroup part to arrive folds the S partial sums (one launch);
// otherwise a second kernel does.
template <int WAVES, bool STRIDED>
__global__ __launch_bounds__(WAVES * 64) void dot_kernel(const float* __restrict__ x,
                                                          const float* __restrict__ y,
                                                          float* __restrict__ part_out,
                                                          float* __restrict__ result, int64_t K,
                                                          int64_t chunk, int S, int fused) {
  constexpr int NT = WAVES * 64;
  __shared__ float part[WAVES];
  __shared__ unsigned last;
  const int tid = threadIdx.x;
  const int64_t kbeg = (int64_t)blockIdx.x * chunk;
  const int64_t kend = kbeg + chunk < K ? kbeg + chunk : K;
  // two independent chains of four accumulators keep eight 16-byte loads in flight per lane
  f4 a0 = {0.f, 0.f, 0.f, 0.f}, a1 = {0.f, 0.f, 0.f, 0.f};
  if (STRIDED) {
    int64_t k = kbeg + (int64_t)tid * 4;
    for (; k + NT * 4 + 3 < kend; k += 2 * NT * 4) {
      // both vectors are streamed once: non-temporal loads
      const f4 x0 = __builtin_nontemporal_load((const f4u*)(x + k));
      const f4 y0 = __builtin_nontemporal_load((const f4u*)(y + k));
      const f4 x1 = __builtin_nontemporal_load((const f4u*)(x + k + NT * 4));
      const f4 y1 = __builtin_nontemporal_load((const f4u*)(y + k + NT * 4));
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        a0[e] = __builtin_fmaf(x0[e], y0[e], a0[e]);
        a1[e] = __builtin_fmaf(x1[e], y1[e], a1[e]);
      }
    }
    for (; k < kend; k += NT * 4) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (k + e < kend) a0[e] = __builtin_fmaf(x[k + e], y[k + e], a0[e]);
    }
  } else {
    // blocked: lane tid owns elements [kbeg + tid*len, kbeg + (tid+1)*len) of the chunk, len a multiple of 4
    const int64_t len = chunk / NT;
    int64_t k = kbeg + (int64_t)tid * len;
    const int64_t lend = k + len < kend ? k + len : kend;
    for (; k + 7 < lend; k += 8) {
      const f4 x0 = *(const f4u*)(x + k), y0 = *(const f4u*)(y + k);
      const f4 x1 = *(const f4u*)(x + k + 4), y1 = *(const f4u*)(y + k + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        a0[e] = __builtin_fmaf(x0[e], y0[e], a0[e]);
        a1[e] = __builtin_fmaf(x1[e], y1[e], a1[e]);
      }
    }
    for (; k < lend; ++k) a0[k & 3] = __builtin_fmaf(x[k], y[k], a0[k & 3]);
  }
  const float w = wave_sum(hsum(a0) + hsum(a1));
  if ((tid & 63) == 0) part[tid >> 6] = w;
  __syncthreads();
  if (tid == 0) {
    float s = part[0];
#pragma unroll
    for (int i = 1; i < WAVES; ++i) s += part[i];
    if (fused) {
      // device-coherent single-word store, complete before the part is counted (see mdh_internal.h)
      coherent_store(part_out + blockIdx.x, s);
      wait_stores_done();
      last = arrive_last(&g_dot_arrivals, (unsigned)S);
    } else {
      part_out[blockIdx.x] = s;  // the result itself if the grid is one workgroup, else part blockIdx.x
    }
  }
  if (!fused) return;
  __syncthreads();
  if (!last || tid >= 64) return;
  const float total = dot_fold_parts<true>(part_out, S, tid);
  if (tid == 0) result[0] = total;
}

// Second pass: one wavefront adds the S workgroup-layer parts in a fixed order.
__global__ __launch_bounds__(64) void dot_combine_kernel(const float* __restrict__ ws,
                                                         float* __restrict__ out, int S) {
  const float a = dot_fold_parts<false>(ws, S, threadIdx.x);
  if (threadIdx.x == 0) out[0] = a;
}

template <int WAVES>
mdh_status launch_dot_t(const DotPlan& pl, int64_t K, const float* x, const float* y, float* out,
                        void* ws, hipStream_t st) {
  // chunk per workgroup: a multiple of one workgroup step so that only the last part is ragged
  const int64_t step = (int64_t)WAVES * 256;
  const int64_t chunk = cdiv(cdiv(K, pl.S), step) * step;
  float* dst = pl.S > 1 ? (float*)ws : out;
  const int fused = pl.S > 1 && pl.fused;
  clear_stale_error();
  if (pl.strided)
    hipLaunchKernelGGL((dot_kernel<WAVES, true>), dim3(pl.S), dim3(WAVES * 64), 0, st, x, y, dst, out, K, chunk, pl.S, fused);
  else
    hipLaunchKernelGGL((dot_kernel<WAVES, false>), dim3(pl.S), dim3(WAVES * 64), 0, st, x, y, dst, out, K, chunk, pl.S, fused);
  mdh_status r = launch_status();
  if (r != MDH_OK || pl.S <= 1 || fused) return r;
  clear_stale_error();
  hipLaunchKernelGGL(dot_combine_kernel, dim3(1), dim3(64), 0, st, (const float*)ws, out, pl.S);
  return launch_status();
}

// ------------------------------------------------------------------------------------- MatVec

// STRIDED: as for Dot -- true = consecutive lanes own consecutive 4-element parts of k (coalesced),
// false = blocked, every lane owns one contiguous part of its wavefront's k-range.
template <int RM, int WM, int WK, bool STRIDED>
__global__ __launch_bounds__(WM* WK * 64) void matvec_kernel(const float* __restrict__ A,
                                                               const float* __restrict__ x,
                                                               float* __restrict__ y,
                                                               float* __restrict__ ws, int M, int K,
                                                               int S, int nwg_i, int kchunk) {
  __shared__ float part[WK > 1 ? (WK - 1) * WM * RM : 1];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave % WM, wk = wave / WM;
  const int gi = blockIdx.x % nwg_i;  // workgroup part of i
  const int gs = blockIdx.x / nwg_i;  // workgroup part of k
  const int i0 = (gi * WM + wm) * RM;
  const int kbeg = gs * kchunk;
  const int kend = min(K, kbeg + kchunk);

  const float* row[RM];
#pragma unroll
  for (int r = 0; r < RM; ++r) row[r] = A + (int64_t)min(i0 + r, M - 1) * K;

  f4 acc[RM];
#pragma unroll
  for (int r = 0; r < RM; ++r) acc[r] = (f4){0.f, 0.f, 0.f, 0.f};

  if (STRIDED) {
    // lanes own consecutive 4-element parts of k; the wavefronts along k interleave 256-element steps
    int k = kbeg + (wk * 64 + lane) * 4;
    for (; k + 3 < kend; k += WK * 256) {
      const f4 xv = *(const f4u*)(x + k);
#pragma unroll
      for (int r = 0; r < RM; ++r) {
        const f4 av = __builtin_nontemporal_load((const f4u*)(row[r] + k));  // streamed once
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[r][e] = __builtin_fmaf(av[e], xv[e], acc[r][e]);
      }
    }
    if (k < kend) {  // ragged end of k: at most three elements, in one lane
#pragma unroll
      for (int e = 0; e < 3; ++e)
        if (k + e < kend) {
          const float xe = x[k + e];
#pragma unroll
          for (int r = 0; r < RM; ++r) acc[r][e] = __builtin_fmaf(row[r][k + e], xe, acc[r][e]);
        }
    }
  } else {
    // blocked: lane (wk, lane) owns ONE contiguous part of the workgroup part of k (a multiple of 4 long)
    const int len = kchunk / (WK * 64);
    int k = kbeg + (wk * 64 + lane) * len;
    const int lend = min(kend, k + len);
    for (; k + 3 < lend; k += 4) {
      const f4 xv = *(const f4u*)(x + k);
#pragma unroll
      for (int r = 0; r < RM; ++r) {
        const f4 av = *(const f4u*)(row[r] + k);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[r][e] = __builtin_fmaf(av[e], xv[e], acc[r][e]);
      }
    }
    for (; k < lend; ++k) {
      const float xe = x[k];
#pragma unroll
      for (int r = 0; r < RM; ++r) acc[r][k & 3] = __builtin_fmaf(row[r][k], xe, acc[r][k & 3]);
    }
  }

  float s[RM];
#pragma unroll
  for (int r = 0; r < RM; ++r) s[r] = wave_sum(hsum(acc[r]));

  if (WK > 1) {
    if (wk > 0 && lane == 0) {
#pragma unroll
      for (int r = 0; r < RM; ++r) part[((wk - 1) * WM + wm) * RM + r] = s[r];
    }
    __syncthreads();
    if (wk > 0) return;
#pragma unroll
    for (int w = 1; w < WK; ++w)
#pragma unroll
      for (int r = 0; r < RM; ++r) s[r] += part[((w - 1) * WM + wm) * RM + r];
  }
  if (lane == 0) {
    float* dst = S > 1 ? ws + (int64_t)gs * M : y;
#pragma unroll
    for (int r = 0; r < RM; ++r)
      if (i0 + r < M) dst[i0 + r] = s[r];
  }
}

// The other lane assignment (paper: Section "Generic Low-Level Expression", parameters D2 and the
// choice of the dimension that follows the fastest lane index): lanes along i, a lane owns a row and
// walks all of k.  A load instruction then touches 64 rows x 16 bytes: nothing coalesces.  Kept as a
// selectable configuration (lane_fast_dim = 0), not as a default.
__global__ __launch_bounds__(256) void matvec_rowlane_kernel(const float* __restrict__ A,
                                                             const float* __restrict__ x,
                                                             float* __restrict__ y, int M, int K) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  const float* row = A + (int64_t)min(i, M - 1) * K;
  f4 acc = (f4){0.f, 0.f, 0.f, 0.f};
  int k = 0;
  for (; k + 3 < K; k += 4) {
    const f4 av = *(const f4u*)(row + k), xv = *(const f4u*)(x + k);
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] = __builtin_fmaf(av[e], xv[e], acc[e]);
  }
  for (; k < K; ++k) acc[k & 3] = __builtin_fmaf(row[k], x[k], acc[k & 3]);
  if (i < M) y[i] = hsum(acc);
}

// Second pass: y[i] = part_0[i] + part_1[i] + ... in that order.
__global__ __launch_bounds__(256) void matvec_combine_kernel(const float* __restrict__ ws,
                                                             float* __restrict__ y, int M, int S) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= M) return;
  float a = ws[i];
  for (int s = 1; s < S; ++s) a += ws[(int64_t)s * M + i];
  y[i] = a;
}

template <int RM, int WM, int WK>
mdh_status launch_matvec_t(const MatVecPlan& pl, int64_t M, int64_t K, const float* A,
                           const float* x, float* y, void* ws, hipStream_t st) {
  const int64_t nwg_i = cdiv(M, (int64_t)WM * RM);
  const int64_t step = (int64_t)WK * 256;
  const int64_t kchunk = cdiv(cdiv(K, pl.S), step) * step;
  const int64_t nblocks = nwg_i * pl.S;
  if (nblocks > 0x7fffffff || kchunk > 0x7fffffff) return MDH_ERR_SIZE;
  clear_stale_error();
  if (pl.strided)
    hipLaunchKernelGGL((matvec_kernel<RM, WM, WK, true>), dim3((unsigned)nblocks), dim3(WM * WK * 64), 0, st,
                       A, x, y, (float*)ws, (int)M, (int)K, pl.S, (int)nwg_i, (int)kchunk);
  else
    hipLaunchKernelGGL((matvec_kernel<RM, WM, WK, false>), dim3((unsigned)nblocks), dim3(WM * WK * 64), 0, st,
                       A, x, y, (float*)ws, (int)M, (int)K, pl.S, (int)nwg_i, (int)kchunk);
  mdh_status r = launch_status();
  if (r != MDH_OK || pl.S <= 1) return r;
  clear_stale_error();
  hipLaunchKernelGGL(matvec_combine_kernel, dim3((unsigned)cdiv(M, 256)), dim3(256), 0, st,
                     (const float*)ws, y, (int)M, pl.S);
  return launch_status();
}

}  // namespace

mdh_status launch_dot(const DotPlan& pl, int64_t K, const float* x, const float* y, float* out,
                      void* ws, hipStream_t st) {
  if (pl.WAVES == 4) return launch_dot_t<4>(pl, K, x, y, out, ws, st);
  if (pl.WAVES == 8) return launch_dot_t<8>(pl, K, x, y, out, ws, st);
  if (pl.WAVES == 16) return launch_dot_t<16>(pl, K, x, y, out, ws, st);
  return MDH_ERR_UNSUPPORTED;
}

mdh_status launch_matvec(const MatVecPlan& pl, int64_t M, int64_t K, const float* A, const float* x,
                         float* y, void* ws, hipStream_t st) {
  if (pl.rowlanes) {
    if (cdiv(M, 256) > 0x7fffffff || K > 0x7fffffff || M > 0x7fffffff) return MDH_ERR_SIZE;
    clear_stale_error();
    hipLaunchKernelGGL(matvec_rowlane_kernel, dim3((unsigned)cdiv(M, 256)), dim3(256), 0, st, A, x, y, (int)M, (int)K);
    return launch_status();
  }
#define MDH_MV(rm, wm, wk) \
  if (pl.RM == rm && pl.WM == wm && pl.WK == wk) return launch_matvec_t<rm, wm, wk>(pl, M, K, A, x, y, ws, st);
  MDH_MV(4, 4, 1)
  MDH_MV(2, 4, 1)
  MDH_MV(8, 4, 1)
  MDH_MV(1, 4, 1)
  MDH_MV(4, 2, 2)
  MDH_MV(2, 2, 2)
  MDH_MV(4, 1, 4)
  MDH_MV(2, 1, 4)
  MDH_MV(1, 1, 4)
  MDH_MV(4, 8, 1)
  MDH_MV(1, 1, 8)
  MDH_MV(2, 1, 8)
#undef MDH_MV
  return MDH_ERR_UNSUPPORTED;
}

}  // namespace mdh
