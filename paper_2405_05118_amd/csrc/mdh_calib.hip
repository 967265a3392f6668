// Calibration kernels: what this chip attains on the three resources the instances are bound by,
// measured with nothing else in the way.  They compute nothing of the method; bench.py prints
// their rates next to the published peaks so that a roofline fraction can be read against both.
//   mdh_calib_copy : streaming device copy (read + write, non-temporal 16-byte accesses)
//   mdh_calib_read : streaming read with a per-lane sum (the access pattern of Dot / MatVec)
//   mdh_calib_mfma : a register-resident loop of independent v_mfma_f32_32x32x2_f32
//   mdh_calib_valu : a register-resident loop of independent 32-bit integer VALU instructions
#include <limits.h>

#include "mdh_internal.h"

namespace mdh {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16 __attribute__((ext_vector_type(16)));

constexpr int CALIB_NT = 256;
// The streaming read: one workgroup of 8 wavefronts per compute unit measured fastest (7.2 TB/s
// against 6.6 TB/s with 2048 workgroups of 4 wavefronts).
constexpr int STREAM_NT = 512, STREAM_BLOCKS = 256;
static_assert(STREAM_NT * STREAM_BLOCKS == MDH_CALIB_STREAM_LANES, "the documented size of `out`");

// The copy: a workgroup of four wavefronts takes ONE contiguous piece of 16 KB (four 16-byte accesses
// per lane, all requested before the first store) and ends; the pieces are handed out in address order
// by the dispatcher.  Measured on two 512 MiB buffers: 6.4-6.5 TB/s, against 5.8-6.0 TB/s for workgroups
// that walk a chunk each or stride over the buffer (8 accesses in flight per lane, with or without the
// next batch requested before the current one is stored), 5.9-6.0 with eight wavefronts per piece and
// 5.6 with 64 KB pieces.
constexpr int COPY_NT = 256, COPY_U = 4, COPY_PIECE = COPY_NT * COPY_U;  // 16-byte elements per workgroup
__global__ __launch_bounds__(COPY_NT) void calib_copy_kernel(const f4* __restrict__ src, f4* __restrict__ dst,
                                                             int64_t n4) {
  const int64_t i = (int64_t)blockIdx.x * COPY_PIECE + threadIdx.x;
  if ((int64_t)(blockIdx.x + 1) * COPY_PIECE <= n4) {  // workgroup-uniform
    f4 v[COPY_U];
#pragma unroll
    for (int u = 0; u < COPY_U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * COPY_NT);
#pragma unroll
    for (int u = 0; u < COPY_U; ++u) __builtin_nontemporal_store(v[u], dst + i + u * COPY_NT);
  } else {
    for (int u = 0; u < COPY_U; ++u)
      if (i + u * COPY_NT < n4) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i + u * COPY_NT), dst + i + u * COPY_NT);
  }
}

template <int U>
__global__ __launch_bounds__(STREAM_NT) void calib_read_kernel(const f4* __restrict__ src, int64_t n4,
                                                               int64_t chunk, float* __restrict__ out) {
  const int64_t beg = (int64_t)blockIdx.x * chunk;
  const int64_t end = beg + chunk < n4 ? beg + chunk : n4;
  f4 s0 = {0, 0, 0, 0}, s1 = {0, 0, 0, 0};
  int64_t i = beg + threadIdx.x;
  for (; i + (U - 1) * STREAM_NT < end; i += U * STREAM_NT) {
    f4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * STREAM_NT);
#pragma unroll
    for (int u = 0; u < U; u += 2) {
      s0 += v[u];
      s1 += v[u + 1];
    }
  }
  for (; i < end; i += STREAM_NT) s0 += __builtin_nontemporal_load(src + i);
  s0 += s1;
  out[(int64_t)blockIdx.x * STREAM_NT + threadIdx.x] = s0.x + s0.y + s0.z + s0.w;
}

// Four independent accumulator blocks per wavefront: the MFMA pipe never waits on a result.
__global__ __launch_bounds__(CALIB_NT) void calib_mfma_kernel(float* __restrict__ out, int iters) {
  const float a = (float)(threadIdx.x & 7) * 0.125f, b = (float)(threadIdx.x & 3) * 0.25f;
  f16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[j][r];
  out[(int64_t)blockIdx.x * CALIB_NT + threadIdx.x] = s;
}

// Eight independent chains per lane; each step max(v ^ c, k) is two two-operand instructions
// (v_xor_b32, v_max_i32) that the compiler cannot fuse, so the count below is instructions x lanes:
// plain 32-bit integer VALU issue rate.
__global__ __launch_bounds__(CALIB_NT) void calib_valu_kernel(int32_t* __restrict__ out, int iters) {
  int32_t v[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = (int32_t)threadIdx.x * (j + 3);
  const int32_t c = (int32_t)blockIdx.x | 1;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = max(v[j] ^ c, j + u - 40);
  }
  int32_t s = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) s ^= v[j];
  out[(int64_t)blockIdx.x * CALIB_NT + threadIdx.x] = s;
}

// ---- VALU issue rate by instruction kind, with the shader clock measured beside it ----
//
// The custom reduce is bound by integer VALU issue.  Its inner loop is made of a few instruction
// kinds; each loop below is register resident, has eight independent chains per lane and issues ONE
// kind (or the custom reduce's own mix), so that rate(kind) / (SIMDs x shader clock) is the issue cost of
// that kind in cycles per wavefront instruction.  The shader clock itself is read in the kernel: the
// wavefront of lane 0 of workgroup 0 samples the shader-clock counter and the constant-rate real-time
// counter before and after its loop.
struct Ticks {
  long long shader, real;
};
__device__ __forceinline__ Ticks ticks_now() {
  Ticks t;
  t.shader = (long long)__builtin_readcyclecounter();       // counts shader-clock cycles
  t.real = (long long)__builtin_amdgcn_s_memrealtime();     // counts at a constant rate
  return t;
}
__device__ __forceinline__ void ticks_store(long long* clk, const Ticks& t0) {
  if (clk && blockIdx.x == 0 && threadIdx.x == 0) {
    const Ticks t1 = ticks_now();
    clk[0] = t1.shader - t0.shader;
    clk[1] = t1.real - t0.real;
  }
}

// kind 1: compare against a wavefront-uniform (scalar-register) operand, then select: 2 instructions a step
__global__ __launch_bounds__(CALIB_NT) void calib_cmpsel_kernel(int32_t* __restrict__ out, int iters,
                                                                int seed, long long* __restrict__ clk) {
  int32_t v[8], w[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = (int32_t)threadIdx.x * (j + 3), w[j] = (int32_t)threadIdx.x + j;
  const Ticks t0 = ticks_now();
  int s = seed;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      s = s * 5 + 1;  // scalar unit
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = (v[j] == s + j) ? w[j] : v[j];
    }
  }
  ticks_store(clk, t0);
  int32_t r = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) r ^= v[j];
  out[(int64_t)blockIdx.x * CALIB_NT + threadIdx.x] = r;
}

// kind 2: three-operand add (two vector registers and a scalar register): 1 instruction a step
__global__ __launch_bounds__(CALIB_NT) void calib_add3_kernel(int32_t* __restrict__ out, int iters,
                                                              int seed, long long* __restrict__ clk) {
  uint32_t v[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = threadIdx.x * (j + 3);
  const Ticks t0 = ticks_now();
  uint32_t s = (uint32_t)seed;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      s = s * 5u + 1u;
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = v[j] + v[(j + 3) & 7] + s;
    }
  }
  ticks_store(clk, t0);
  uint32_t r = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) r ^= v[j];
  out[(int64_t)blockIdx.x * CALIB_NT + threadIdx.x] = (int32_t)r;
}

// kind 3: the custom reduce's own inner loop (8 fields, 2 records of A per lane) with the records of
// B made up on the scalar unit instead of loaded: per pair 8 compares against a scalar operand, 8
// selects, 4.5 adds, and compare + max + select + half a move for max_idx = 24 instructions.
__global__ __launch_bounds__(CALIB_NT) void calib_prlmix_kernel(int32_t* __restrict__ out, int iters,
                                                                int seed, const int32_t* __restrict__ wts,
                                                                long long* __restrict__ clk) {
  constexpr int NF = 8, RA = 2;
  unsigned dw[NF];
  unsigned base = 0;
#pragma unroll
  for (int f = 0; f < NF; ++f) {
    dw[f] = (unsigned)wts[f] - (unsigned)wts[NF + f];
    base += (unsigned)wts[NF + f];
  }
  int ar[RA][NF];
#pragma unroll
  for (int ra = 0; ra < RA; ++ra)
#pragma unroll
    for (int f = 0; f < NF; ++f) ar[ra][f] = wts[2 * NF + (threadIdx.x * RA + ra) * NF + f];
  int bs[RA], bi[RA];
#pragma unroll
  for (int ra = 0; ra < RA; ++ra) bs[ra] = INT_MIN, bi[ra] = INT_MAX;
  const Ticks t0 = ticks_now();
  int s = seed;
  for (int b = 0; b < iters; ++b) {
    int br[NF];  // wavefront-uniform "record of B": scalar registers
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      s = s * 5 + 1;
      br[f] = (s >> 9) & 15;
    }
#pragma unroll
    for (int ra = 0; ra < RA; ++ra) {
      unsigned sc = base;
#pragma unroll
      for (int f = 0; f < NF; ++f) sc += (ar[ra][f] == br[f]) ? dw[f] : 0u;
      const int v = (int)sc;
      const bool take = v > bs[ra];
      bs[ra] = take ? v : bs[ra];
      bi[ra] = take ? b : bi[ra];
    }
  }
  ticks_store(clk, t0);
  int32_t r = 0;
#pragma unroll
  for (int ra = 0; ra < RA; ++ra) r ^= bs[ra] ^ bi[ra];
  out[(int64_t)blockIdx.x * CALIB_NT + threadIdx.x] = r;
}

// kinds 4 and 5: instructions of the kind the vector ALU issues at twice the rate (32 lanes a cycle:
// moves, 32-bit add / subtract, bitwise logic, fp32 add / multiply / fused multiply-add, all on
// vector-register operands).  Written as single instructions so that the compiler cannot fold a chain
// of them; nothing here needs a wait state (no scalar operand, no condition code).
template <bool FMA>
__global__ __launch_bounds__(CALIB_NT) void calib_fastkind_kernel(int32_t* __restrict__ out, int iters,
                                                                  int seed, long long* __restrict__ clk) {
  int32_t v[8], w[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    v[j] = FMA ? __float_as_int(0.5f + (float)(threadIdx.x & 7) * 0.0625f) : (int32_t)threadIdx.x * (j + 3);
    w[j] = FMA ? __float_as_int(0.25f + (float)j * 0.03125f) : (int32_t)threadIdx.x + j + seed;
  }
  const Ticks t0 = ticks_now();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (FMA)
          asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(v[j]) : "v"(w[j]));  // x <- x*w + w, stays in (0, 1)
        else
          asm volatile("v_add_u32 %0, %0, %1" : "+v"(v[j]) : "v"(w[j]));
      }
  }
  ticks_store(clk, t0);
  int32_t r = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) r ^= v[j];
  out[(int64_t)blockIdx.x * CALIB_NT + threadIdx.x] = r;
}

// kind 6: the custom reduce's loop for 8 fields as it is built from the fast kinds (two records of A per
// lane, blocks of four records of B): per pair 8 x (subtract, multiply with clamp, fused multiply-add) and
// a quarter of (two three-operand maxima, compare, select) -- with the records of B made up on the
// scalar unit, not loaded.  Per block of 8 pairs: 192 + 8 instructions, and three moves (block index, copies).
__global__ __launch_bounds__(CALIB_NT) void calib_prlfast_kernel(int32_t* __restrict__ out, int iters,
                                                                 int seed, const int32_t* __restrict__ wts,
                                                                 long long* __restrict__ clk) {
  constexpr int NF = 8, RA = 2;
  constexpr unsigned kCode = 0x4B000000u;
  float ndw[NF];
  float agree = 0.f;
#pragma unroll
  for (int f = 0; f < NF; ++f) {
    ndw[f] = (float)(wts[NF + f] - wts[f]);
    agree += (float)wts[f];
  }
  float fa[RA][NF];
#pragma unroll
  for (int ra = 0; ra < RA; ++ra)
#pragma unroll
    for (int f = 0; f < NF; ++f) fa[ra][f] = __uint_as_float(kCode + (unsigned)wts[2 * NF + (threadIdx.x * RA + ra) * NF + f]);
  float best[RA];
  int blk[RA];
#pragma unroll
  for (int ra = 0; ra < RA; ++ra) best[ra] = -3.0e38f, blk[ra] = 0;
  const float vbase = agree + __uint_as_float(threadIdx.x & 0);
  const Ticks t0 = ticks_now();
  unsigned s = (unsigned)seed;
  for (int bb = 0; bb < iters; ++bb) {
    float fb[4][NF];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int f = 0; f < NF; ++f) {
        s = s * 5u + 1u;  // scalar unit
        fb[u][f] = __uint_as_float(kCode + ((s >> 9) & 15u));
      }
    float acc[4][RA];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      float t[4][RA];
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int ra = 0; ra < RA; ++ra) t[u][ra] = fa[ra][f] - fb[u][f];
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int ra = 0; ra < RA; ++ra) asm("v_mul_f32_e64 %0, %1, %1 clamp" : "=v"(t[u][ra]) : "v"(t[u][ra]));
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int ra = 0; ra < RA; ++ra) acc[u][ra] = __builtin_fmaf(t[u][ra], ndw[f], f == 0 ? vbase : acc[u][ra]);
    }
#pragma unroll
    for (int ra = 0; ra < RA; ++ra) {
      const float m = __builtin_fmaxf(__builtin_fmaxf(acc[0][ra], acc[1][ra]), acc[2][ra]);
      const float nb = __builtin_fmaxf(__builtin_fmaxf(best[ra], m), acc[3][ra]);
      blk[ra] = nb > best[ra] ? bb : blk[ra];
      best[ra] = nb;
    }
  }
  ticks_store(clk, t0);
  int32_t r = 0;
#pragma unroll
  for (int ra = 0; ra < RA; ++ra) r ^= (int32_t)best[ra] ^ blk[ra];
  out[(int64_t)blockIdx.x * CALIB_NT + threadIdx.x] = r;
}

// kind 0 with the clock readings: the loop of calib_valu_kernel
__global__ __launch_bounds__(CALIB_NT) void calib_xormax_kernel(int32_t* __restrict__ out, int iters,
                                                                int seed, long long* __restrict__ clk) {
  int32_t v[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] = (int32_t)threadIdx.x * (j + 3);
  const int32_t c = (int32_t)blockIdx.x | seed | 1;
  const Ticks t0 = ticks_now();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = max(v[j] ^ c, j + u - 40);
  }
  ticks_store(clk, t0);
  int32_t r = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) r ^= v[j];
  out[(int64_t)blockIdx.x * CALIB_NT + threadIdx.x] = r;
}

}  // namespace
}  // namespace mdh

using namespace mdh;

extern "C" {

mdh_status mdh_calib_copy(const void* src, void* dst, int64_t bytes, void* stream) {
  if (!src || !dst) return MDH_ERR_NULL;
  if (bytes <= 0 || bytes % 16) return MDH_ERR_SIZE;
  clear_stale_error();
  const int64_t n4 = bytes / 16;
  const int64_t pieces = cdiv(n4, (int64_t)COPY_PIECE);
  if (pieces > 0x7fffffff) return MDH_ERR_SIZE;
  hipLaunchKernelGGL(calib_copy_kernel, dim3((unsigned)pieces), dim3(COPY_NT), 0, (hipStream_t)stream,
                     (const f4*)src, (f4*)dst, n4);
  return launch_status();
}

mdh_status mdh_calib_read(const void* src, int64_t bytes, float* out, void* stream) {
  if (!src || !out) return MDH_ERR_NULL;
  if (bytes <= 0 || bytes % 16) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL(calib_read_kernel<4>, dim3(STREAM_BLOCKS), dim3(STREAM_NT), 0, (hipStream_t)stream,
                     (const f4*)src, bytes / 16, cdiv(bytes / 16, (int64_t)STREAM_BLOCKS), out);
  return launch_status();
}

mdh_status mdh_calib_mfma(float* out, int32_t iters, int64_t* flop, void* stream) {
  if (!out) return MDH_ERR_NULL;
  if (iters <= 0) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL(calib_mfma_kernel, dim3(MDH_CALIB_BLOCKS), dim3(CALIB_NT), 0, (hipStream_t)stream, out, iters);
  // per wavefront and iteration: 16 MFMAs of 32 x 32 x 2 multiply-adds
  if (flop) *flop = (int64_t)MDH_CALIB_BLOCKS * (CALIB_NT / 64) * iters * 16 * (2LL * 32 * 32 * 2);
  return launch_status();
}

mdh_status mdh_calib_valu(int32_t* out, int32_t iters, int64_t* lane_ops, void* stream) {
  if (!out) return MDH_ERR_NULL;
  if (iters <= 0) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL(calib_valu_kernel, dim3(MDH_CALIB_BLOCKS), dim3(CALIB_NT), 0, (hipStream_t)stream, out, iters);
  // per lane and iteration: 32 xors + 32 maxima
  if (lane_ops) *lane_ops = (int64_t)MDH_CALIB_BLOCKS * CALIB_NT * iters * 64;
  return launch_status();
}

mdh_status mdh_calib_valu_kind(int32_t kind, int32_t* out, const int32_t* weights, int32_t iters,
                               int64_t* lane_ops, int64_t* clocks, void* stream) {
  if (!out || (kind == MDH_CALIB_KIND_PRL_MIX && !weights)) return MDH_ERR_NULL;
  if (iters <= 0) return MDH_ERR_SIZE;
  clear_stale_error();
  const dim3 g(MDH_CALIB_BLOCKS), b(CALIB_NT);
  hipStream_t st = (hipStream_t)stream;
  long long* clk = (long long*)clocks;
  int64_t per_lane = 0;  // VALU instructions a lane issues inside the loop
  switch (kind) {
    case MDH_CALIB_KIND_XOR_MAX:
      hipLaunchKernelGGL(calib_xormax_kernel, g, b, 0, st, out, iters, 0, clk);
      per_lane = (int64_t)iters * 64;  // 32 xors + 32 maxima
      break;
    case MDH_CALIB_KIND_CMP_SELECT:
      hipLaunchKernelGGL(calib_cmpsel_kernel, g, b, 0, st, out, iters, 12345, clk);
      per_lane = (int64_t)iters * 64;  // 32 compares + 32 selects
      break;
    case MDH_CALIB_KIND_ADD3:
      hipLaunchKernelGGL(calib_add3_kernel, g, b, 0, st, out, iters, 12345, clk);
      per_lane = (int64_t)iters * 64;  // 64 three-operand adds
      break;
    case MDH_CALIB_KIND_PRL_MIX:
      hipLaunchKernelGGL(calib_prlmix_kernel, g, b, 0, st, out, iters, 12345, weights, clk);
      per_lane = (int64_t)iters * 48;  // two pairs of 24 instructions
      break;
    case MDH_CALIB_KIND_PRL_FAST_MIX:
      if (!weights) return MDH_ERR_NULL;
      hipLaunchKernelGGL(calib_prlfast_kernel, g, b, 0, st, out, iters, 12345, weights, clk);
      per_lane = (int64_t)iters * 203;  // 8 pairs: 192 + 8 + three moves, as emitted
      break;
    case MDH_CALIB_KIND_FMA_F32:
      hipLaunchKernelGGL(calib_fastkind_kernel<true>, g, b, 0, st, out, iters, 0, clk);
      per_lane = (int64_t)iters * 64;  // 64 fused multiply-adds on vector registers
      break;
    case MDH_CALIB_KIND_ADD_VGPR:
      hipLaunchKernelGGL(calib_fastkind_kernel<false>, g, b, 0, st, out, iters, 12345, clk);
      per_lane = (int64_t)iters * 64;  // 64 two-operand adds on vector registers
      break;
    default:
      return MDH_ERR_UNSUPPORTED;
  }
  if (lane_ops) *lane_ops = (int64_t)MDH_CALIB_BLOCKS * CALIB_NT * per_lane;
  return launch_status();
}

int64_t mdh_calib_realtime_hz(void) {
  int dev = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess) return 0;
  return (int64_t)khz * 1000;
}

}  // extern "C"
