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
//   workgroup : if a row is cut into several chunks, either a single pass (a chunk waits in
//               registers while the workgroups exchange chunk totals through memory: 8 bytes per
//               element) or three kernels: chunk totals -> exclusive scan of the totals per row ->
//               scan of every chunk starting from its offset (the input is read twice: 12 bytes
//               per element).
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

template <bool KEEP = false>
__device__ __forceinline__ f4 load4(const float* p, int64_t j, int64_t n) {
  if (j + 3 < n) return KEEP ? *(const f4u*)(p + j) : __builtin_nontemporal_load((const f4u*)(p + j));
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
    a0 += load4<true>(src, j, n);
    if (t + 1 < TPC) a1 += load4<true>(src, j + (int64_t)NT * 4, n);
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
  // chunks are taken in descending order: the totals pass read them in ascending order, so the
  // chunks it read last may still be in cache
  const unsigned bid = gridDim.x - 1 - blockIdx.x;
  const int64_t row = bid / C;
  const int chunk = bid % C;
  const float* src = in + row * n;
  float* dst = out + row * n;
  const int64_t j0 = (int64_t)chunk * TPC * NT * 4;
  double carry = offs ? offs[bid] : 0.0;
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

// ---------------------------------------------------------------------------- single pass
// The chunks of a row over workgroups with ONE pass over the input: a workgroup loads its chunk
// into registers, scans it locally, publishes the chunk total, adds up the totals of the chunks
// before it in the row (published by other workgroups) and writes the chunk.  Totals travel through
// 8-byte words of the workspace that start as kNotYet (a NaN bit pattern no sum produces) and are
// written and polled with device-scope atomics.  Sums of 64 consecutive totals ("group sums") are
// published too, by the workgroup of the group's last chunk, so that a workgroup reads at most
// 63 totals and C/64 group sums.  Every sum is taken in a fixed order: bit-identical run to run.
//
// Progress: chunk numbers are handed out by a ticket counter to running workgroups, so every chunk a
// workgroup waits for has been drawn by a workgroup that is running it or has finished it; a
// total depends on the chunk alone and a group sum on totals alone, so there is no chain of waits.
// Each wait is also bounded (spin_limit polls); on a time-out the kernel stops waiting, sets word
// 1 of the workspace and finishes with wrong values in that chunk.
constexpr unsigned long long kNotYet = 0xFFFFFFFFFFFFFFFFull;

__global__ __launch_bounds__(256) void scan_onepass_init_kernel(unsigned long long* ws, int64_t words) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < words) ws[i] = i < 2 ? 0ull : kNotYet;
}

__device__ __forceinline__ double wait_for(unsigned long long* slot, int spin_limit, unsigned long long* err) {
  unsigned long long x = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  int spins = 0;
  while (x == kNotYet) {
    if (++spins > spin_limit) {
      __hip_atomic_store(err, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      return 0.0;
    }
    __builtin_amdgcn_s_sleep(4);
    x = __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  return __longlong_as_double((long long)x);
}

// sum over the lanes of a wavefront in a fixed order; the result is valid in lane 0
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) v += __shfl_down(v, d, 64);
  return v;
}

// FULL: the whole chunk lies inside the row (no bounds checks on loads and stores).  SOLO: the
// chunk is the whole row, nothing is exchanged with other workgroups.
template <int WAVES, int TPC, bool FULL, bool SOLO = false>
__device__ __forceinline__ void onepass_body(const float* __restrict__ src, float* __restrict__ dst,
                                             unsigned long long* __restrict__ my_totals,
                                             unsigned long long* __restrict__ my_gsums,
                                             unsigned long long* __restrict__ err, int64_t j0, int64_t n,
                                             int chunk, int spin_limit, double* wex, double* dpart) {
  constexpr int NT = WAVES * 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t jt = j0 + (int64_t)tid * 4;  // the lane's first element of tile 0

  f4 v[TPC];
#pragma unroll
  for (int t = 0; t < TPC; ++t)
    v[t] = FULL ? __builtin_nontemporal_load((const f4u*)(src + jt) + t * NT) : load4(src, jt + (int64_t)t * NT * 4, n);

  // wavefront level, no barrier: v[t] holds the lane's own prefixes, pre[t] what the lanes before
  // it in the wavefront add; the wavefront totals go to LDS in (tile, wavefront) order
  constexpr int NE = TPC * WAVES;  // <= 128
  float pre[TPC];
#pragma unroll
  for (int t = 0; t < TPC; ++t) {
    v[t][1] += v[t][0];
    v[t][2] += v[t][1];
    v[t][3] += v[t][2];
    const float incl = wave_scan(v[t][3], lane);
    if (lane == 63) wex[t * WAVES + wave] = (double)incl;
    pre[t] = incl - v[t][3];
  }
  __syncthreads();

  // workgroup level: wavefront 0 turns the NE totals into exclusive prefixes (fp64, two entries per
  // lane) and publishes the chunk total, then collects the totals of the chunks before it in its
  // group of 64; meanwhile the other wavefronts collect the sums of the groups before
  const int g = chunk >> 6, m = chunk & 63;
  double part = 0.0;
  if (wave == 0) {
    const int e0 = 2 * lane;
    const double a0 = e0 < NE ? wex[e0] : 0.0, a1 = e0 + 1 < NE ? wex[e0 + 1] : 0.0;
    double incl = a0 + a1;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const double x = __shfl_up(incl, d, 64);
      if (lane >= d) incl += x;
    }
    const double excl = incl - (a0 + a1);
    if (e0 < NE) wex[e0] = excl;
    if (e0 + 1 < NE) wex[e0 + 1] = excl + a0;
    if (!SOLO) {
      const double total = __shfl(incl, 63, 64);
      if (lane == 0) {
        wex[NE] = total;
        __hip_atomic_store(my_totals + chunk, (unsigned long long)__double_as_longlong(total), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
      }
      if (lane < m) part = wait_for(my_totals + (g << 6) + lane, spin_limit, err);
    }
  } else if (!SOLO) {
    for (int k = tid - 64; k < g; k += NT - 64) part += wait_for(my_gsums + k, spin_limit, err);
  }
  double off = 0.0;
  if (SOLO) {
    __syncthreads();
  } else {
    part = wave_sum(part);
    if (lane == 0) dpart[wave] = part;
    __syncthreads();
    const double in_group = dpart[0];
    if (tid == 0 && m == 63)  // the group is complete with this chunk
      __hip_atomic_store(my_gsums + g, (unsigned long long)__double_as_longlong(in_group + wex[NE]), __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
    off = in_group;
#pragma unroll
    for (int w = 1; w < WAVES; ++w) off += dpart[w];
  }

#pragma unroll
  for (int t = 0; t < TPC; ++t) {
    const float base = (float)(off + wex[t * WAVES + wave] + (double)pre[t]);
    const f4 r = v[t] + base;
    if (FULL) {
      __builtin_nontemporal_store(r, (f4u*)(dst + jt) + t * NT);
    } else {
      const int64_t j = jt + (int64_t)t * NT * 4;
      if (j + 3 < n) {
        __builtin_nontemporal_store(r, (f4u*)(dst + j));
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (j + e < n) dst[j + e] = r[e];
      }
    }
  }
}

// four wavefronts per SIMD (two workgroups of 8 wavefronts, or one of 16) bound the registers
template <int WAVES, int TPC>
__global__ __launch_bounds__(WAVES * 64, 4) void scan_onepass_kernel(const float* __restrict__ in,
                                                                     float* __restrict__ out,
                                                                     unsigned long long* __restrict__ ws,
                                                                     int64_t n, int C, int G, int64_t RC,
                                                                     int spin_limit) {
  constexpr int NT = WAVES * 64;
  __shared__ double wex[TPC * WAVES + 1];  // wavefront totals, then their exclusive prefixes; chunk total
  __shared__ double dpart[WAVES];
  __shared__ unsigned ticket;
  static_assert(TPC * WAVES <= 128, "two entries per lane of wavefront 0");
  // persistent workgroups: one launch of as many workgroups as the chip holds at once, each drawing
  // chunk numbers until none is left -- the loads of a workgroup's next chunk go out while the
  // stores of its last one drain, instead of a new workgroup starting from an empty compute unit
  for (;;) {
    __syncthreads();  // every lane is done with the previous chunk's LDS values and its number
    if (threadIdx.x == 0) ticket = atomicAdd((unsigned*)ws, 1u);
    __syncthreads();
    const unsigned bid = ticket;
    if ((int64_t)bid >= RC) break;  // workgroup-uniform
    const int64_t row = bid / C;
    const int chunk = bid % C;
    const int64_t j0 = (int64_t)chunk * TPC * NT * 4;
    unsigned long long* my_totals = ws + 2 + row * C;
    unsigned long long* my_gsums = ws + 2 + RC + row * G;
    if (j0 + (int64_t)TPC * NT * 4 <= n)
      onepass_body<WAVES, TPC, true>(in + row * n, out + row * n, my_totals, my_gsums, ws + 1, j0, n, chunk,
                                     spin_limit, wex, dpart);
    else
      onepass_body<WAVES, TPC, false>(in + row * n, out + row * n, my_totals, my_gsums, ws + 1, j0, n, chunk,
                                      spin_limit, wex, dpart);
  }
}

// A whole row per workgroup, resident in registers (rows of up to 8 tiles): the wavefront scans
// need no barrier, one wavefront turns the wavefront totals into exclusive prefixes, two barriers
// per row instead of one per tile.
template <int WAVES, int TPC>
__global__ __launch_bounds__(WAVES * 64, 4) void scan_row_resident_kernel(const float* __restrict__ in,
                                                                          float* __restrict__ out, int64_t n) {
  constexpr int NT = WAVES * 64;
  __shared__ double wex[TPC * WAVES + 1];
  static_assert(TPC * WAVES <= 128, "two entries per lane of wavefront 0");
  const int64_t row = blockIdx.x;
  if ((int64_t)TPC * NT * 4 <= n)
    onepass_body<WAVES, TPC, true, true>(in + row * n, out + row * n, nullptr, nullptr, nullptr, 0, n, 0, 0, wex, nullptr);
  else
    onepass_body<WAVES, TPC, false, true>(in + row * n, out + row * n, nullptr, nullptr, nullptr, 0, n, 0, 0, wex, nullptr);
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

template <int WAVES, int TPC>
mdh_status launch_onepass_t(const ScanPlan& pl, int64_t R, int64_t n, const float* in, float* out, void* ws,
                            hipStream_t st) {
  const int64_t blocks = R * pl.C;
  if (blocks > 0x7fffffff) return MDH_ERR_SIZE;
  const int64_t G = cdiv(pl.C, 64);
  const int64_t words = 2 + blocks + R * G;
  clear_stale_error();
  hipLaunchKernelGGL(scan_onepass_init_kernel, dim3((unsigned)cdiv(words, 256)), dim3(256), 0, st,
                     (unsigned long long*)ws, words);
  mdh_status r = launch_status();
  if (r != MDH_OK) return r;
  clear_stale_error();
  // a poll sleeps ~64 cycles plus a trip to memory: 2^22 polls are seconds, far beyond any real wait
  // as many workgroups as run at once (16 wavefronts per compute unit by the kernel's register bound)
  static int cus[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MDH_ERR_LAUNCH;
  if (cus[dev] == 0) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) return MDH_ERR_LAUNCH;
    cus[dev] = v;
  }
  int64_t grid = (int64_t)cus[dev] * (16 / WAVES);
  if (grid > blocks) grid = blocks;
  hipLaunchKernelGGL((scan_onepass_kernel<WAVES, TPC>), dim3((unsigned)grid), dim3(WAVES * 64), 0, st, in, out,
                     (unsigned long long*)ws, n, pl.C, (int)G, blocks, 1 << 22);
  return launch_status();
}

template <int WAVES, int TPC>
mdh_status launch_resident_t(int64_t R, int64_t n, const float* in, float* out, hipStream_t st) {
  if (R > 0x7fffffff) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL((scan_row_resident_kernel<WAVES, TPC>), dim3((unsigned)R), dim3(WAVES * 64), 0, st, in, out, n);
  return launch_status();
}

mdh_status launch_onepass(const ScanPlan& pl, int64_t R, int64_t n, const float* in, float* out, void* ws,
                          hipStream_t st) {
#define MDH_OP(w, t)                                                                       \
  if (pl.WAVES == w && pl.TPC == t)                                                        \
    return pl.C == 1 ? launch_resident_t<w, t>(R, n, in, out, st) : launch_onepass_t<w, t>(pl, R, n, in, out, ws, st);
  MDH_OP(8, 1)
  MDH_OP(8, 2)
  MDH_OP(8, 4)
  MDH_OP(8, 8)
  MDH_OP(16, 1)
  MDH_OP(16, 2)
  MDH_OP(16, 4)
  MDH_OP(16, 8)
#undef MDH_OP
  return MDH_ERR_UNSUPPORTED;
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
  if (pl.onepass) return launch_onepass(pl, R, n, in, out, ws, st);  // chunks, or a whole row, resident in registers
  switch (pl.WAVES) {
    case 4: return launch_t<4>(pl, R, n, in, out, ws, st);
    case 8: return launch_t<8>(pl, R, n, in, out, ws, st);
    case 16: return launch_t<16>(pl, R, n, in, out, ws, st);
  }
  return MDH_ERR_UNSUPPORTED;
}

}  // namespace mdh
