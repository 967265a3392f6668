// Device entry points of the C ABI declared in include/mdh.h: argument checks, planning,
// launches.  No allocation, no synchronisation (except mdh_tune, which times candidates).
#include <string.h>

#include <functional>

#include "mdh_internal.h"

using namespace mdh;

namespace {

constexpr int64_t kMaxElems = 0x7fffffff;  // kernels index buffers with 32-bit tile-local offsets

bool too_big(int64_t n) { return n < 0 || n > kMaxElems; }

}  // namespace

namespace mdh {
thread_local hipError_t g_last_launch_error = hipSuccess;
}

extern "C" {

const char* mdh_last_launch_error(void) { return hipGetErrorString(mdh::g_last_launch_error); }

mdh_status mdh_matmul(int64_t M, int64_t N, int64_t K, const float* A, const float* B, float* C,
                      const mdh_tile_params* params, void* workspace, size_t workspace_bytes,
                      void* stream) {
  if (M < 0 || N < 0 || K < 1) return MDH_ERR_SIZE;
  if (too_big(M) || too_big(N) || too_big(K) || too_big(M * K) || too_big(K * N) || too_big(M * N))
    return MDH_ERR_SIZE;
  const int64_t sizes[3] = {M, N, K};
  if (small_m_matmul(sizes, params)) {
    // at most 16 rows: the small-M kernel of the batched instance (one batch entry, plain views)
    GemmExPlan ex;
    mdh_status st = plan_matmul_small_m(sizes, params, &ex);
    if (st != MDH_OK) return st;
    if (M == 0 || N == 0) return MDH_OK;
    if (!A || !B || !C) return MDH_ERR_NULL;
    if (ex.g.S > 1) {
      const size_t need = (size_t)ex.g.S * (size_t)M * (size_t)N * sizeof(float);
      if (!workspace || workspace_bytes < need) return MDH_ERR_WORKSPACE;
    }
    return launch_matmul_ex(ex, 1, M, N, K, A, B, C, workspace, (hipStream_t)stream);
  }
  GemmPlan pl;
  mdh_status st = plan_matmul(sizes, params, &pl);
  if (st != MDH_OK) return st;
  if (M == 0 || N == 0) return MDH_OK;
  if (!A || !B || !C) return MDH_ERR_NULL;
  if (pl.S > 1) {
    if (too_big((int64_t)pl.S * M * N)) return MDH_ERR_SIZE;
    const size_t need = (size_t)pl.S * (size_t)M * (size_t)N * sizeof(float);
    if (!workspace || workspace_bytes < need) return MDH_ERR_WORKSPACE;
  }
  return launch_matmul(pl, M, N, K, A, B, C, workspace, (hipStream_t)stream);
}

mdh_status mdh_stencil(int64_t nx, int64_t ny, int64_t nz, const float* in, float* out, float c0,
                       float c1, const mdh_tile_params* params, void* stream) {
  if (nx < 0 || ny < 0 || nz < 0) return MDH_ERR_SIZE;
  if (too_big(nx) || too_big(ny) || too_big(nz)) return MDH_ERR_SIZE;
  if (too_big((nx + 2) * (ny + 2)) || too_big((nx + 2) * (ny + 2) * (nz + 2))) return MDH_ERR_SIZE;
  const int64_t sizes[3] = {nx, ny, nz};
  StencilPlan pl;
  mdh_status st = plan_stencil(sizes, params, &pl);
  if (st != MDH_OK) return st;
  if (nx == 0 || ny == 0 || nz == 0) return MDH_OK;
  if (!in || !out) return MDH_ERR_NULL;
  return launch_stencil(pl, nx, ny, nz, in, out, c0, c1, (hipStream_t)stream);
}

mdh_status mdh_mcc(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                   int64_t stride_h, int64_t stride_w, const float* in, const float* filt,
                   float* out, const mdh_tile_params* params, void* workspace,
                   size_t workspace_bytes, void* stream) {
  if (N < 0 || K < 0 || C < 1 || R < 1 || S < 1 || stride_h < 1 || stride_w < 1) return MDH_ERR_SIZE;
  if (H < R || W < S) return MDH_ERR_SIZE;
  if (too_big(N) || too_big(H) || too_big(W) || too_big(C) || too_big(K) || too_big(R) || too_big(S))
    return MDH_ERR_SIZE;
  const int64_t P = (H - R) / stride_h + 1, Q = (W - S) / stride_w + 1;
  if (too_big(H * W) || too_big(N * H * W) || too_big(N * H * W * C)) return MDH_ERR_SIZE;
  if (too_big(R * S * C) || too_big(K * R * S * C)) return MDH_ERR_SIZE;
  if (too_big(N * P * Q) || too_big(N * P * Q * K)) return MDH_ERR_SIZE;
  const int64_t sizes[9] = {N, P, Q, K, C, R, S, stride_h, stride_w};
  MccPlan pl;
  mdh_status st = plan_mcc(sizes, params, &pl);
  if (st != MDH_OK) return st;
  if (N == 0 || K == 0) return MDH_OK;
  if (!in || !filt || !out) return MDH_ERR_NULL;
  if (pl.flat)
    return launch_mcc_flat(pl, N, H, W, C, K, R, S, stride_h, stride_w, in, filt, out, (hipStream_t)stream);
  if (pl.S > 1) {
    if (too_big((int64_t)pl.S * N * P * Q * K)) return MDH_ERR_SIZE;
    const size_t need = (size_t)pl.S * (size_t)(N * P * Q * K) * sizeof(float);
    if (!workspace || workspace_bytes < need) return MDH_ERR_WORKSPACE;
  }
  return launch_mcc(pl, N, H, W, C, K, R, S, stride_h, stride_w, in, filt, out, workspace, (hipStream_t)stream);
}

mdh_status mdh_mcc_capsule(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                           int64_t stride_h, int64_t stride_w, const float* in, const float* filt,
                           float* out, const mdh_tile_params* params, void* stream) {
  if (N < 0 || K < 0 || C < 1 || R < 1 || S < 1 || stride_h < 1 || stride_w < 1) return MDH_ERR_SIZE;
  if (H < R || W < S) return MDH_ERR_SIZE;
  if (too_big(N) || too_big(H) || too_big(W) || too_big(C) || too_big(K) || too_big(R) || too_big(S))
    return MDH_ERR_SIZE;
  const int64_t P = (H - R) / stride_h + 1, Q = (W - S) / stride_w + 1;
  if (too_big(H * W) || too_big(N * H * W) || too_big(N * H * W * C) || too_big(N * H * W * C * 16)) return MDH_ERR_SIZE;
  if (too_big(R * S * C) || too_big(K * R * S * C) || too_big(K * R * S * C * 16)) return MDH_ERR_SIZE;
  if (too_big(N * P * Q) || too_big(N * P * Q * K) || too_big(N * P * Q * K * 16)) return MDH_ERR_SIZE;
  const int64_t sizes[9] = {N, P, Q, K, C, R, S, stride_h, stride_w};
  CapsulePlan pl;
  mdh_status st = plan_capsule(sizes, params, &pl);
  if (st != MDH_OK) return st;
  if (N == 0 || K == 0) return MDH_OK;
  if (!in || !filt || !out) return MDH_ERR_NULL;
  return launch_capsule(pl, N, H, W, C, K, R, S, stride_h, stride_w, in, filt, out, (hipStream_t)stream);
}

mdh_status mdh_custom_reduce(int64_t nA, int64_t nB, int32_t nF, const int32_t* A,
                             const int32_t* B, const int32_t* w_agree, const int32_t* w_disagree,
                             int32_t* out_score, int32_t* out_index,
                             const mdh_tile_params* params, void* workspace,
                             size_t workspace_bytes, void* stream) {
  if (nA < 0 || nB < 1 || nF < 1 || nF > 16) return MDH_ERR_SIZE;
  if (too_big(nA) || too_big(nB) || too_big(nA * nF) || too_big(nB * nF)) return MDH_ERR_SIZE;
  const int64_t sizes[2] = {nA, nB};
  PrlPlan pl;
  mdh_status st = plan_prl(sizes, params, &pl);
  if (st != MDH_OK) return st;
  if (nA == 0) return MDH_OK;
  if (!A || !B || !w_agree || !w_disagree || !out_score || !out_index) return MDH_ERR_NULL;
  if (pl.S > 1) {
    if (too_big((int64_t)pl.S * nA * 2)) return MDH_ERR_SIZE;
    const size_t need = (size_t)pl.S * (size_t)nA * 2 * sizeof(int32_t);
    if (!workspace || workspace_bytes < need) return MDH_ERR_WORKSPACE;
  }
  return launch_prl(pl, nA, nB, nF, A, B, w_agree, w_disagree, out_score, out_index, workspace,
                    (hipStream_t)stream);
}

mdh_status mdh_matmul_ex(int64_t batch, int64_t M, int64_t N, int64_t K, const float* A,
                         int32_t trans_a, const float* B, int32_t trans_b, float* C,
                         int32_t trans_c, const mdh_tile_params* params, void* workspace,
                         size_t workspace_bytes, void* stream) {
  if (batch < 0 || M < 0 || N < 0 || K < 1 || batch > 65535) return MDH_ERR_SIZE;
  if (too_big(M) || too_big(N) || too_big(K) || too_big(M * K) || too_big(K * N) || too_big(M * N))
    return MDH_ERR_SIZE;
  if (too_big(batch * M * K) || too_big(batch * K * N) || too_big(batch * M * N)) return MDH_ERR_SIZE;
  const int64_t sizes[7] = {batch, M, N, K, trans_a ? 1 : 0, trans_b ? 1 : 0, trans_c ? 1 : 0};
  GemmExPlan pl;
  mdh_status st = plan_matmul_ex(sizes, params, &pl);
  if (st != MDH_OK) return st;
  if (batch == 0 || M == 0 || N == 0) return MDH_OK;
  if (!A || !B || !C) return MDH_ERR_NULL;
  if (pl.g.S > 1) {
    if (too_big((int64_t)pl.g.S * batch * M * N)) return MDH_ERR_SIZE;
    const size_t need = (size_t)pl.g.S * (size_t)batch * (size_t)M * (size_t)N * sizeof(float);
    if (!workspace || workspace_bytes < need) return MDH_ERR_WORKSPACE;
  }
  return launch_matmul_ex(pl, batch, M, N, K, A, B, C, workspace, (hipStream_t)stream);
}

mdh_status mdh_scan(int64_t R, int64_t n, const float* in, float* out, const mdh_tile_params* params,
                    void* workspace, size_t workspace_bytes, void* stream) {
  if (R < 0 || n < 0 || too_big(R) || too_big(n) || too_big(R * n)) return MDH_ERR_SIZE;
  const int64_t sizes[2] = {R, n};
  ScanPlan pl;
  mdh_status st = plan_scan(sizes, params, &pl);
  if (st != MDH_OK) return st;
  if (R == 0 || n == 0) return MDH_OK;
  if (!in || !out) return MDH_ERR_NULL;
  if (pl.C > 1 && (!workspace || workspace_bytes < scan_workspace_bytes(pl, R) || ((uintptr_t)workspace & 7)))
    return MDH_ERR_WORKSPACE;
  return launch_scan(pl, R, n, in, out, workspace, (hipStream_t)stream);
}

mdh_status mdh_scan_timed_out(int64_t R, int64_t n, const mdh_tile_params* params, const void* workspace,
                              void* stream, int32_t* timed_out) {
  if (!timed_out) return MDH_ERR_NULL;
  *timed_out = 0;
  if (R < 0 || n < 0 || too_big(R) || too_big(n) || too_big(R * n)) return MDH_ERR_SIZE;
  const int64_t sizes[2] = {R, n};
  ScanPlan pl;
  mdh_status st = plan_scan(sizes, params, &pl);
  if (st != MDH_OK) return st;
  if (R == 0 || n == 0 || pl.C <= 1 || !pl.onepass) return MDH_OK;  // no waits in this configuration
  if (!workspace) return MDH_ERR_WORKSPACE;
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return MDH_ERR_LAUNCH;
  unsigned long long word = 0;
  if (hipMemcpy(&word, (const char*)workspace + 8, 8, hipMemcpyDeviceToHost) != hipSuccess) return MDH_ERR_LAUNCH;
  *timed_out = word != 0 ? 1 : 0;
  return MDH_OK;
}

mdh_status mdh_dot(int64_t K, const float* x, const float* y, float* out,
                   const mdh_tile_params* params, void* workspace, size_t workspace_bytes,
                   void* stream) {
  if (K < 1 || too_big(K)) return MDH_ERR_SIZE;
  const int64_t sizes[1] = {K};
  DotPlan pl;
  mdh_status st = plan_dot(sizes, params, &pl);
  if (st != MDH_OK) return st;
  if (!x || !y || !out) return MDH_ERR_NULL;
  if (pl.S > 1 && (!workspace || workspace_bytes < (size_t)pl.S * sizeof(float))) return MDH_ERR_WORKSPACE;
  return launch_dot(pl, K, x, y, out, workspace, (hipStream_t)stream);
}

mdh_status mdh_matvec(int64_t M, int64_t K, const float* A, const float* x, float* y,
                      const mdh_tile_params* params, void* workspace, size_t workspace_bytes,
                      void* stream) {
  if (M < 0 || K < 1 || too_big(M) || too_big(K) || too_big(M * K)) return MDH_ERR_SIZE;
  const int64_t sizes[2] = {M, K};
  MatVecPlan pl;
  mdh_status st = plan_matvec(sizes, params, &pl);
  if (st != MDH_OK) return st;
  if (M == 0) return MDH_OK;
  if (!A || !x || !y) return MDH_ERR_NULL;
  if (pl.S > 1) {
    if (too_big((int64_t)pl.S * M)) return MDH_ERR_SIZE;
    if (!workspace || workspace_bytes < (size_t)pl.S * (size_t)M * sizeof(float)) return MDH_ERR_WORKSPACE;
  }
  return launch_matvec(pl, M, K, A, x, y, workspace, (hipStream_t)stream);
}

// ------------------------------------------------------------------------------ tile search

mdh_status mdh_tune(mdh_instance inst, const int64_t* sizes, void* const* buffers,
                    const float* scalars, void* workspace, size_t workspace_bytes, void* stream,
                    int32_t reps, mdh_tile_params* best, float* best_ms) {
  if (!sizes || !buffers || !best) return MDH_ERR_NULL;
  if (reps < 1) reps = 3;
  hipStream_t st = (hipStream_t)stream;
  const int n = mdh_num_candidates(inst, sizes);
  if (n <= 0) return MDH_ERR_UNSUPPORTED;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return MDH_ERR_LAUNCH;
  if (hipEventCreate(&e1) != hipSuccess) {
    hipEventDestroy(e0);
    return MDH_ERR_LAUNCH;
  }
  float best_t = -1.f;
  mdh_status last = MDH_ERR_UNSUPPORTED;
  for (int c = 0; c < n; ++c) {
    mdh_tile_params p;
    if (mdh_candidate(inst, sizes, c, &p) != MDH_OK) continue;
    std::function<mdh_status()> run = [&]() -> mdh_status {
      switch (inst) {
        case MDH_MATMUL:
          return mdh_matmul(sizes[0], sizes[1], sizes[2], (const float*)buffers[0],
                            (const float*)buffers[1], (float*)buffers[2], &p, workspace,
                            workspace_bytes, stream);
        case MDH_STENCIL:
          return mdh_stencil(sizes[0], sizes[1], sizes[2], (const float*)buffers[0],
                             (float*)buffers[1], scalars ? scalars[0] : 0.5f,
                             scalars ? scalars[1] : 1.f / 12.f, &p, stream);
        case MDH_MCC: {
          const int64_t H = (sizes[1] - 1) * sizes[7] + sizes[5], W = (sizes[2] - 1) * sizes[8] + sizes[6];
          return mdh_mcc(sizes[0], H, W, sizes[4], sizes[3], sizes[5], sizes[6], sizes[7], sizes[8],
                         (const float*)buffers[0], (const float*)buffers[1], (float*)buffers[2], &p,
                         workspace, workspace_bytes, stream);
        }
        case MDH_CUSTOM_REDUCE:
          return mdh_custom_reduce(sizes[0], sizes[1], (int32_t)sizes[2], (const int32_t*)buffers[0],
                                   (const int32_t*)buffers[1], (const int32_t*)buffers[2],
                                   (const int32_t*)buffers[3], (int32_t*)buffers[4],
                                   (int32_t*)buffers[5], &p, workspace, workspace_bytes, stream);
        case MDH_BMATMUL:
          return mdh_matmul_ex(sizes[0], sizes[1], sizes[2], sizes[3], (const float*)buffers[0], (int32_t)sizes[4],
                               (const float*)buffers[1], (int32_t)sizes[5], (float*)buffers[2], (int32_t)sizes[6],
                               &p, workspace, workspace_bytes, stream);
        case MDH_SCAN:
          return mdh_scan(sizes[0], sizes[1], (const float*)buffers[0], (float*)buffers[1], &p, workspace,
                          workspace_bytes, stream);
        case MDH_MCC_CAPSULE: {
          const int64_t H = (sizes[1] - 1) * sizes[7] + sizes[5], W = (sizes[2] - 1) * sizes[8] + sizes[6];
          return mdh_mcc_capsule(sizes[0], H, W, sizes[4], sizes[3], sizes[5], sizes[6], sizes[7], sizes[8],
                                 (const float*)buffers[0], (const float*)buffers[1], (float*)buffers[2], &p, stream);
        }
        default:
          break;
      }
      return MDH_ERR_UNSUPPORTED;
    };
    if (inst == MDH_DOT || inst == MDH_MATVEC) {
      run = [&]() -> mdh_status {
        if (inst == MDH_DOT)
          return mdh_dot(sizes[0], (const float*)buffers[0], (const float*)buffers[1], (float*)buffers[2],
                         &p, workspace, workspace_bytes, stream);
        return mdh_matvec(sizes[0], sizes[1], (const float*)buffers[0], (const float*)buffers[1],
                          (float*)buffers[2], &p, workspace, workspace_bytes, stream);
      };
    }
    mdh_status r = run();  // warm-up; candidates that need more workspace are skipped
    if (r != MDH_OK) {
      last = r;
      continue;
    }
    hipEventRecord(e0, st);
    for (int i = 0; i < reps; ++i) run();
    hipEventRecord(e1, st);
    if (hipEventSynchronize(e1) != hipSuccess) {
      hipEventDestroy(e0);
      hipEventDestroy(e1);
      return MDH_ERR_LAUNCH;
    }
    float ms = 0.f;
    hipEventElapsedTime(&ms, e0, e1);
    ms /= reps;
    if (best_t < 0.f || ms < best_t) {
      best_t = ms;
      *best = p;
    }
  }
  hipEventDestroy(e0);
  hipEventDestroy(e1);
  if (best_t < 0.f) return last;
  if (best_ms) *best_ms = best_t;
  return MDH_OK;
}

}  // extern "C"
