// Internal declarations shared by the host planner and the kernel launchers of libmdh.
// Nothing here is part of the C ABI (see include/mdh.h for that).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "mdh.h"

namespace mdh {

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- launch descriptors the planner derives from a tile-parameter configuration ----

// Jacobi-3D: a workgroup owns TJ = TY*RJ rows (j) x KT = LK*4 columns (k) and marches
// over SI consecutive planes (i).  Lanes run along k (4 outputs each), TY lane-rows
// along j, RJ rows per lane in registers.
struct StencilPlan {
  int RJ, TY, LK;  // kernel instantiation
  int SI;          // planes per workgroup (sequential HBM-layer parts of dimension i)
  int ragged;
};

// MatMul / MCC contraction core: workgroup tile BM x BN, K-step BK through LDS,
// WM x WN per wavefront out of 32x32x2 FP32 MFMA blocks, split factor S over k.
struct GemmPlan {
  int BM, BN, BK, WM, WN;
  int S;  // workgroup-layer parts of the reduction dimension
  int ragged;
  // wavefront-layer parts of the reduction dimension.  1: the LDS-tiled kernel (wavefronts tile the
  // output).  > 1: the kernel whose WK wavefronts all own the whole BM x BN tile and split k, operands
  // straight from device memory to registers, results combined in LDS (then WM = BM, WN = BN, BK = 8).
  int WK = 1;
  // LDS-tiled kernel, loop order of the workgroup layer (parameter D1): 0 = tiles walked in bands of 8 tile
  // rows, i fastest inside a band (order (WG,i),(WG,j),(WG,k)); 1 = bands of 8 tile columns, j fastest
  // (order (WG,j),(WG,i),(WG,k)).  Decides which panels of A and B the tiles resident together share.
  int jmajor = 0;
};

// MCC: workgroup tile TP x TQ output pixels x BN output channels, CK channels per LDS stage.
struct MccPlan {
  int TP, TQ, BN, CK, WM, WN;
  int ragged;
  int flat;    // 1: few-channel kernel that walks s and c as one fused dimension (TQ = block width)
  int QT = 1;  // few-channel kernel: column tiles a workgroup walks with its filter slice resident
  int S = 1;   // channel-chunked kernel: workgroup-layer parts of the reduction dimension c
  // few-channel kernel: 1 = the workgroup-layer parts of (n, p, q) are dealt out to resident workgroups in
  // arrival order (QT = 1), 0 = a workgroup owns QT consecutive column tiles
  int dealt = 0;
};

// Custom reduce: RA records of A per lane, WB wavefronts of a workgroup split B,
// S workgroup-layer parts of B.
struct PrlPlan {
  int RA, WB, WA;  // WA wavefronts along a
  int S;
  int ragged;
};

// helpers of the planner shared by its translation units (defined in mdh_plan.cpp)
namespace detail {
void clear_params(mdh_tile_params* p, int D);
void set_order(mdh_tile_params* p, const int* dim_order);
mdh_status check_products(const mdh_tile_params* p, const int64_t* sizes, bool* ragged);
mdh_status check_lanes(const mdh_tile_params* p);
bool same_table(const mdh_tile_params& a, const mdh_tile_params& b);
}  // namespace detail

// Dot: WAVES wavefronts per workgroup, S workgroup-layer parts of k; a lane owns 4
// consecutive k per step, steps are strided over the lanes of the workgroup.
struct DotPlan {
  int WAVES;
  int S;
  int ragged;
  int strided = 1;  // lanes interleave 4-element parts (1) or own one contiguous part each (0)
  int fused = 1;    // S > 1: the last workgroup part to arrive folds the partial sums (one launch)
};

// MatVec: a wavefront owns RM rows; WM wavefronts along i, WK wavefronts along k per
// workgroup; lanes along k (4 consecutive k each); S workgroup-layer parts of k.
struct MatVecPlan {
  int RM, WM, WK;
  int S;
  int ragged;
  int strided = 1;  // lanes interleave 4-element parts of k (1) or own one contiguous part each (0)
  // 1: the lanes run along i (a lane owns a row and walks all of k; lane_fast_dim = 0) -- the assignment
  // whose loads of A do not coalesce; RM = 1, WM = 4, WK = 1, S = 1
  int rowlanes = 0;
};

// Row-wise scan: a workgroup owns one chunk of one row = TPC sequential tiles of WAVES*256
// elements; C chunks per row (C > 1: chunk totals are scanned by a second kernel).
struct ScanPlan {
  int WAVES;
  int TPC;
  int C;
  int ragged;
  int onepass;  // C > 1 only: a chunk stays in registers while the workgroups exchange chunk totals
};
// bytes of workspace a scan plan needs for R rows (0: none)
size_t scan_workspace_bytes(const ScanPlan& pl, int64_t R);
mdh_status plan_scan(const int64_t* sizes, const mdh_tile_params* p, ScanPlan* out);
void params_from_plan(const int64_t* sizes, const ScanPlan& pl, mdh_tile_params* out);
int scan_candidates(const int64_t* sizes, ScanPlan* out, int cap);
mdh_status launch_scan(const ScanPlan& pl, int64_t R, int64_t n, const float* in, float* out, void* ws,
                       hipStream_t st);

// MCC_Capsule: NI blocks of 8 output channels per wavefront; a workgroup owns 4 output rows and walks
// QT tiles of 8 columns
struct CapsulePlan {
  int NI;
  int QT;
  int RW;  // wavefront-layer parts of the fused (r, s, c) reduction walk
  int ragged;
};
mdh_status plan_capsule(const int64_t* sizes, const mdh_tile_params* p, CapsulePlan* out);
void params_from_plan(const int64_t* sizes, const CapsulePlan& pl, mdh_tile_params* out);
int capsule_candidates(const int64_t* sizes, CapsulePlan* out, int cap);
int64_t capsule_lds_bytes(int NI, int RW, int64_t C, int64_t R, int64_t S, int64_t sh, int64_t sw);
mdh_status launch_capsule(const CapsulePlan& pl, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K,
                          int64_t R, int64_t S, int64_t sh, int64_t sw, const float* in,
                          const float* filt, float* out, hipStream_t st);

// bMatMul / MatMul^T: the MatMul descriptor plus the transposition of the three views
struct GemmExPlan {
  GemmPlan g;
  int ta, tb, tc;
  // skinny = 1: the small-M kernel (16 x 16 x 4 block, operands straight to registers); then
  // g.BM = 16, g.BN = 64 * wavefronts along j, g.BK = 16 and WK = wavefronts along k
  int skinny = 0, WK = 1;
  // small-M kernel with S > 1: 1 = the last workgroup part of an output strip to arrive adds the S
  // partial results itself (one launch), 0 = a second kernel does
  int fused = 0;
  // small-M kernel with narrow strips and B transposed: 1 = both operands staged through LDS
  // (row-contiguous loads), 0 = read straight into the MFMA layout
  int lds = 0;
};
// Device-coherent accesses for results that pass between workgroups of ONE launch (the parts of a split
// reduction folded by the last part to arrive).  The L2 caches of the chip's eight XCDs are not kept
// coherent for ordinary loads and stores inside a kernel; a device-scope fence would write back and
// invalidate a whole L2 (measured: ~10 us per kernel).  Device-scope atomic loads and stores of single
// words go to the coherent level directly, so: partial results are stored with coherent_store, the
// storing wavefront waits for its stores (wait_stores_done) before it counts itself in with a
// device-scope atomic, and the folding workgroup reads with coherent_load.
#if defined(__HIPCC__)
__device__ __forceinline__ void coherent_store(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float coherent_load(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// all memory operations this wavefront has issued are complete (vmcnt, expcnt, lgkmcnt = 0)
__device__ __forceinline__ void wait_stores_done() { __builtin_amdgcn_s_waitcnt(0); }
// counts the caller in; true for the S-th arrival, which also wraps the counter back to zero
__device__ __forceinline__ bool arrive_last(unsigned* counter, unsigned S) {
  return __builtin_amdgcn_atomic_inc32(counter, S - 1, __ATOMIC_RELAXED, "agent") == S - 1;
}
#endif

// Counters of arriving workgroup parts live in static device arrays of this many words per kernel
// family; a split reduction with more output parts than that takes the second-kernel path.
constexpr int kArrivalCounters = 4096;
mdh_status plan_matmul_ex(const int64_t* sizes, const mdh_tile_params* p, GemmExPlan* out);
void params_from_plan(const int64_t* sizes, const GemmExPlan& pl, mdh_tile_params* out);
int matmul_ex_candidates(const int64_t* sizes, GemmExPlan* out, int cap);
mdh_status launch_matmul_ex(const GemmExPlan& pl, int64_t batch, int64_t M, int64_t N, int64_t K,
                            const float* A, const float* B, float* C, void* ws, hipStream_t st);
mdh_status launch_matmul_skinny(const GemmExPlan& pl, int64_t batch, int64_t M, int64_t N, int64_t K,
                                const float* A, const float* B, float* C, void* ws, hipStream_t st);
mdh_status launch_matmul_ksplit(const GemmPlan& pl, int64_t M, int64_t N, int64_t K, const float* A,
                                const float* B, float* C, void* ws, hipStream_t st);
// dst[i] = part_0[i] + ... + part_{S-1}[i], i < n (defined in mdh_matmul.hip)
mdh_status launch_combine_sum(const float* ws, float* dst, int64_t n, int S, hipStream_t st);

// MatMul with at most 16 rows is evaluated by the small-M kernel of the batched entry point (batch 1,
// plain views).  small_m_matmul: does (sizes, p) of the MatMul instance select that kernel -- the
// default for 0 < M <= 16, or a table with its signature (16 x 16 x 4 block, four register parts of j).
// lift_batch / drop_batch convert between the 3-dimensional MatMul table and the 4-dimensional table of
// the batched instance with one batch entry.
bool small_m_matmul(const int64_t* sizes3, const mdh_tile_params* p);
void lift_batch(const mdh_tile_params& p3, mdh_tile_params* p4);
void drop_batch(const mdh_tile_params& p4, mdh_tile_params* p3);
mdh_status plan_matmul_small_m(const int64_t* sizes3, const mdh_tile_params* p, GemmExPlan* out);

mdh_status plan_dot(const int64_t* sizes, const mdh_tile_params* p, DotPlan* out);
mdh_status plan_matvec(const int64_t* sizes, const mdh_tile_params* p, MatVecPlan* out);
void params_from_plan(const int64_t* sizes, const DotPlan& pl, mdh_tile_params* out);
void params_from_plan(const int64_t* sizes, const MatVecPlan& pl, mdh_tile_params* out);
int dot_candidates(const int64_t* sizes, DotPlan* out, int cap);
int matvec_candidates(const int64_t* sizes, MatVecPlan* out, int cap);
mdh_status launch_dot(const DotPlan& pl, int64_t K, const float* x, const float* y, float* out,
                      void* ws, hipStream_t st);
mdh_status launch_matvec(const MatVecPlan& pl, int64_t M, int64_t K, const float* A, const float* x,
                         float* y, void* ws, hipStream_t st);

mdh_status plan_stencil(const int64_t* sizes, const mdh_tile_params* p, StencilPlan* out);
mdh_status plan_matmul(const int64_t* sizes, const mdh_tile_params* p, GemmPlan* out);
mdh_status plan_mcc(const int64_t* sizes, const mdh_tile_params* p, MccPlan* out);
mdh_status plan_prl(const int64_t* sizes, const mdh_tile_params* p, PrlPlan* out);

// Fill a full parameter table (prt/blk/order/regions) from a launch descriptor.
void params_from_plan(const int64_t* sizes, const StencilPlan& pl, mdh_tile_params* out);
void params_from_plan(const int64_t* sizes, const GemmPlan& pl, mdh_tile_params* out);
void params_from_plan(const int64_t* sizes, const MccPlan& pl, mdh_tile_params* out);
void params_from_plan(const int64_t* sizes, const PrlPlan& pl, mdh_tile_params* out);

// Candidate menus (defaults are candidate 0).
int stencil_candidates(const int64_t* sizes, StencilPlan* out, int cap);
int matmul_candidates(const int64_t* sizes, GemmPlan* out, int cap);
int mcc_candidates(const int64_t* sizes, MccPlan* out, int cap);
int prl_candidates(const int64_t* sizes, PrlPlan* out, int cap);

// ---- launchers (defined in the .hip files) ----
mdh_status launch_stencil(const StencilPlan& pl, int64_t nx, int64_t ny, int64_t nz, const float* in,
                          float* out, float c0, float c1, hipStream_t st);
mdh_status launch_matmul(const GemmPlan& pl, int64_t M, int64_t N, int64_t K, const float* A,
                         const float* B, float* C, void* ws, hipStream_t st);
mdh_status launch_mcc(const MccPlan& pl, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K,
                      int64_t R, int64_t S, int64_t sh, int64_t sw, const float* in,
                      const float* filt, float* out, void* ws, hipStream_t st);
mdh_status launch_mcc_flat(const MccPlan& pl, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K,
                           int64_t R, int64_t S, int64_t sh, int64_t sw, const float* in,
                           const float* filt, float* out, hipStream_t st);
mdh_status launch_prl(const PrlPlan& pl, int64_t nA, int64_t nB, int nF, const int32_t* A,
                      const int32_t* B, const int32_t* wp, const int32_t* wm, int32_t* score,
                      int32_t* index, void* ws, hipStream_t st);

// The runtime's "last error" is sticky per thread and other users of the runtime in the same
// process leave harmless codes there (an event query that is not ready yet, for instance):
// clear it before a launch so that the status read after the launch is that launch's own.
inline void clear_stale_error() { (void)hipGetLastError(); }
extern thread_local hipError_t g_last_launch_error;
inline mdh_status launch_status() {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return MDH_OK;
  g_last_launch_error = e;
  return MDH_ERR_LAUNCH;
}


// A kernel may use more than 64 KB of dynamic LDS only after that has been allowed, per kernel and per
// device.  `done[dev]` remembers the largest size allowed so far on each device (one array per kernel
// instantiation, kept by the caller); two threads racing here both set the same attribute.
constexpr int kMaxDevices = 64;
inline mdh_status allow_dynamic_lds(const void* kern, int64_t bytes, int64_t (&done)[kMaxDevices]) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MDH_ERR_LAUNCH;
  if (bytes <= done[dev]) return MDH_OK;
  const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) {
    g_last_launch_error = e;
    return MDH_ERR_LAUNCH;
  }
  done[dev] = bytes;
  return MDH_OK;
}

}  // namespace mdh
