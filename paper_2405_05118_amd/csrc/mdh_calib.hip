// Calibration kernels: what this chip attains on the three resources the instances are bound by,
// measured with nothing else in the way.  They compute nothing of the method; bench.py prints
// their rates next to the published peaks so that a roofline fraction can be read against both.
//   mdh_calib_copy : streaming device copy (read + write, non-temporal 16-byte accesses)
//   mdh_calib_read : streaming read with a per-lane sum (the access pattern of Dot / MatVec)
//   mdh_calib_mfma : a register-resident loop of independent v_mfma_f32_32x32x2_f32
//   mdh_calib_valu : a register-resident loop of independent 32-bit integer VALU instructions
#include "mdh_internal.h"

namespace mdh {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16 __attribute__((ext_vector_type(16)));

constexpr int CALIB_NT = 256;
// The streaming kernels: one workgroup of 8 wavefronts per compute unit measured fastest (read 7.2
// TB/s against 6.6 TB/s with 2048 workgroups of 4 wavefronts; copy 6.0 against 5.5 TB/s).
constexpr int STREAM_NT = 512, STREAM_BLOCKS = 256;
static_assert(STREAM_NT * STREAM_BLOCKS == MDH_CALIB_STREAM_LANES, "the documented size of `out`");

// Every workgroup walks one contiguous chunk (the assignment the Dot and Jacobi kernels use), U
// 16-byte accesses in flight per lane.
template <int U>
__global__ __launch_bounds__(STREAM_NT) void calib_copy_kernel(const f4* __restrict__ src,
                                                               f4* __restrict__ dst, int64_t n4,
                                                               int64_t chunk) {
  const int64_t beg = (int64_t)blockIdx.x * chunk;
  const int64_t end = beg + chunk < n4 ? beg + chunk : n4;
  int64_t i = beg + threadIdx.x;
  for (; i + (U - 1) * STREAM_NT < end; i += U * STREAM_NT) {
    f4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * STREAM_NT);
#pragma unroll
    for (int u = 0; u < U; ++u) __builtin_nontemporal_store(v[u], dst + i + u * STREAM_NT);
  }
  for (; i < end; i += STREAM_NT) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
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

}  // namespace
}  // namespace mdh

using namespace mdh;

extern "C" {

mdh_status mdh_calib_copy(const void* src, void* dst, int64_t bytes, void* stream) {
  if (!src || !dst) return MDH_ERR_NULL;
  if (bytes <= 0 || bytes % 16) return MDH_ERR_SIZE;
  clear_stale_error();
  const int64_t n4 = bytes / 16;
  hipLaunchKernelGGL(calib_copy_kernel<8>, dim3(STREAM_BLOCKS), dim3(STREAM_NT), 0, (hipStream_t)stream,
                     (const f4*)src, (f4*)dst, n4, cdiv(n4, (int64_t)STREAM_BLOCKS));
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

}  // extern "C"
