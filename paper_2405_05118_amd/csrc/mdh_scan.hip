// Row-wise scan(+): md_hom(id, (++, prefix-sum(+))) over (i, j), out[i][j] = in[i][0] + ... + in[i][j]
// (paper: Section "Examples", Subfigure 8; Appendix, Example "Prefix-Sum").
//
// The prefix-sum combine operator keeps the dimension (index set function id) and a part's result
// depends on the parts before it only through ONE value, their last prefix.  That is what the
// re-composition passes along on every layer:
//   VGPR      : a lane scans its 4 consecutive elements
//   lane      : inclusive scan of the lane totals across the wavefront (6 shuffle steps)
//   wavefront : the wavefront totals of a tile meet in LDS; every lane adds the totals before it
//   HBM parts : the tiles of a chunk are walked in ascending order with a carry (kept in fp64, so
//               the carry chain of a long row does not accumulate fp32 rounding)
//   workgroup : if a row is cut into several chunks, three kernels: chunk totals -> exclusive scan
//               of the totals per row -> scan of every chunk starting from its offset.  The input
//               is then read twice (12 bytes per element instead of 8).
// Bound: HBM.  Every level combines in a fixed order: bit-identical run to run.
#include "mdh_internal.h"

namespace mdh {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));

// Inclusive scan over the 64 lanes of a wavefront.
__device__ __forceinline__ float wave_scan(float v, int lane) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const float t = __shfl_up(v, d, 64);
    if (lane >= d) v += t;
  }
  return v;
}

__device__ __forceinline__ f4 load4(const float* p, int64_t j, int64_t n) {
  if (j + 3 < n) return __builtin_nontemporal_load((const f4u*)(p + j));
  f4 v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int e = 0; e < 4; ++e)
    if (j + e < n) v[e] = p[j + e];
  return v;
}

// Totals of the chunks: ws[row * C + chunk] (fp64).
template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void scan_totals_kernel(const float* __restrict__ in,
                                                                 double* __restrict__ ws, int64_t n,
                                                                 int C, int TPC) {
  constexpr int NT = WAVES * 64;
  __shared__ double part[WAVES];
  const int tid = threadIdx.x, lane = tid & 63;
  const int64_t row = blockIdx.x / C;
  const int chunk = blockIdx.x % C;
  const float* src = in + row * n;
  const int64_t j0 = (int64_t)chunk * TPC * NT * 4;
  f4 a0 = {0.f, 0.f, 0.f, 0.f}, a1 = {0.f, 0.f, 0.f, 0.f};
  double acc = 0.0;
  for (int t = 0; t < TPC; t += 2) {
    const int64_t j = j0 + ((int64_t)t * NT + tid) * 4;
    a0 += load4(src, j, n);
    if (t + 1 < TPC) a1 += load4(src, j + (int64_t)NT * 4, n);
    if ((t & 62) == 62) {  // fold into fp64 every 64 tiles
      acc += (double)((a0[0] + a0[1]) + (a0[2] + a0[3])) + (double)((a1[0] + a1[1]) + (a1[2] + a1[3]));
      a0 = a1 = (f4){0.f, 0.f, 0.f, 0.f};
    }
  }
  acc += (double)((a0[0] + a0[1]) + (a0[2] + a0[3])) + (double)((a1[0] + a1[1]) + (a1[2] + a1[3]));
  // lanes -> wavefront (fixed order), wavefronts -> workgroup in LDS
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) acc += __shfl_down(acc, d, 64);
  if (lane == 0) part[tid >> 6] = acc;
  __syncthreads();
  if (tid == 0) {
    double s = part[0];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) s += part[w];
    ws[blockIdx.x] = s;
  }
}

// Exclusive scan of the C chunk totals of every row, in place (one workgroup per row).
__global__ __launch_bounds__(256) void scan_offsets_kernel(double* __restrict__ ws, int C) {
  __shared__ double wtot[2][4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  double* row = ws + (int64_t)blockIdx.x * C;
  double carry = 0.0;
  int buf = 0;
  for (int c0 = 0; c0 < C; c0 += 256, buf ^= 1) {
    const int c = c0 + tid;
    const double own = c < C ? row[c] : 0.0;
    double v = own;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const double t = __shfl_up(v, d, 64);
      if (lane >= d) v += t;
    }
    if (lane == 63) wtot[buf][wave] = v;
    __syncthreads();
    double before = 0.0, all = 0.0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const double t = wtot[buf][w];
      if (w < wave) before += t;
      all += t;
    }
    if (c < C) row[c] = carry + before + (v - own);
    carry += all;
  }
}

// Scan of one chunk of one row, starting from the chunk's offset (offs == nullptr: 0).
template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void scan_apply_kernel(const float* __restrict__ in,
                                                                float* __restrict__ out,
                                                                const double* __restrict__ offs,
                                                                int64_t n, int C, int TPC) {
  constexpr int NT = WAVES * 64;
  __shared__ float wtot[2][WAVES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t row = blockIdx.x / C;
  const int chunk = blockIdx.x % C;
  const float* src = in + row * n;
  float* dst = out + row * n;
  const int64_t j0 = (int64_t)chunk * TPC * NT * 4;
  double carry = offs ? offs[blockIdx.x] : 0.0;
  f4 nxt = load4(src, j0 + (int64_t)tid * 4, n);
  for (int t = 0; t < TPC; ++t) {
    const int64_t j = j0 + ((int64_t)t * NT + tid) * 4;
    if (j - (int64_t)tid * 4 >= n) break;  // whole tile beyond the row (workgroup-uniform)
    f4 v = nxt;
    if (t + 1 < TPC) nxt = load4(src, j + (int64_t)NT * 4, n);  // next tile in flight
    v[1] += v[0];
    v[2] += v[1];
    v[3] += v[2];
    const float incl = wave_scan(v[3], lane);
    if (lane == 63) wtot[t & 1][wave] = incl;
    __syncthreads();
    float before = 0.f, all = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float x = wtot[t & 1][w];
      if (w < wave) before += x;
      all += x;
    }
    const float base = (float)(carry + (double)(before + (incl - v[3])));
    v += base;
    if (j + 3 < n) {
      __builtin_nontemporal_store(v, (f4u*)(dst + j));
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (j + e < n) dst[j + e] = v[e];
    }
    carry += (double)all;
  }
}

// Short rows: one wavefront per row, 4 rows per workgroup, no LDS and no barrier; the row is walked
// in tiles of 256 elements with the carry in a register.
__global__ __launch_bounds__(256) void scan_rows_wave_kernel(const float* __restrict__ in,
                                                             float* __restrict__ out, int64_t R,
                                                             int64_t n, int TPC) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= R) return;  // whole wavefront; the kernel has no barrier
  const float* src = in + row * n;
  float* dst = out + row * n;
  double carry = 0.0;
  f4 nxt = load4(src, (int64_t)lane * 4, n);
  for (int t = 0; t < TPC; ++t) {
    const int64_t j = ((int64_t)t * 64 + lane) * 4;
    f4 v = nxt;
    if (t + 1 < TPC) nxt = load4(src, j + 256, n);
    v[1] += v[0];
    v[2] += v[1];
    v[3] += v[2];
    const float incl = wave_scan(v[3], lane);
    const float all = __shfl(incl, 63, 64);
    v += (float)(carry + (double)(incl - v[3]));
    if (j + 3 < n) {
      __builtin_nontemporal_store(v, (f4u*)(dst + j));
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (j + e < n) dst[j + e] = v[e];
    }
    carry += (double)all;
  }
}

template <int WAVES>
mdh_status launch_t(const ScanPlan& pl, int64_t R, int64_t n, const float* in, float* out, void* ws,
                    hipStream_t st) {
  const int64_t blocks = R * pl.C;
  if (blocks > 0x7fffffff) return MDH_ERR_SIZE;
  double* w = (double*)ws;
  if (pl.C > 1) {
    clear_stale_error();
    hipLaunchKernelGGL((scan_totals_kernel<WAVES>), dim3((unsigned)blocks), dim3(WAVES * 64), 0, st, in, w, n, pl.C, pl.TPC);
    mdh_status r = launch_status();
    if (r != MDH_OK) return r;
    clear_stale_error();
    hipLaunchKernelGGL(scan_offsets_kernel, dim3((unsigned)R), dim3(256), 0, st, w, pl.C);
    if ((r = launch_status()) != MDH_OK) return r;
  }
  clear_stale_error();
  hipLaunchKernelGGL((scan_apply_kernel<WAVES>), dim3((unsigned)blocks), dim3(WAVES * 64), 0, st, in, out,
                     pl.C > 1 ? (const double*)w : (const double*)nullptr, n, pl.C, pl.TPC);
  return launch_status();
}

}  // namespace

mdh_status launch_scan(const ScanPlan& pl, int64_t R, int64_t n, const float* in, float* out, void* ws,
                       hipStream_t st) {
  if (pl.WAVES == 1) {
    if (pl.C != 1) return MDH_ERR_UNSUPPORTED;
    const int64_t blocks = cdiv(R, 4);
    if (blocks > 0x7fffffff) return MDH_ERR_SIZE;
    clear_stale_error();
    hipLaunchKernelGGL(scan_rows_wave_kernel, dim3((unsigned)blocks), dim3(256), 0, st, in, out, R, n, pl.TPC);
    return launch_status();
  }
  switch (pl.WAVES) {
    case 4: return launch_t<4>(pl, R, n, in, out, ws, st);
    case 8: return launch_t<8>(pl, R, n, in, out, ws, st);
    case 16: return launch_t<16>(pl, R, n, in, out, ws, st);
  }
  return MDH_ERR_UNSUPPORTED;
}

}  // namespace mdh
