// Custom-combine instance md_hom(wght, (++, max_idx)) over (a,b) for gfx950
// (record-linkage style; paper: Section "Examples", Subfigure 5).
//
//   wght(a,b) = ( sum_f (A[a,f]==B[b,f] ? w_agree[f] : w_disagree[f]) , b )       index-carrying f
//   (s1,b1) max_idx (s2,b2) = larger score wins; equal scores: smaller index wins  user-defined op
//
// The work is nA*nB scalar-function evaluations on a few MiB of data: it is bound by
// integer vector-ALU issue, not by memory.  De-composition, dims (a,b):
//   workgroup layer : nA/(WA*64*RA) x S        -- S > 1 splits the reduction dimension b
//   wavefront layer : WA x WB                  -- WB wavefronts of a workgroup split b again
//   lane layer      : 64 x 1                   -- the ++ dimension a runs over the lanes
//   VGPR layer      : RA records of A per lane, held in registers for the whole kernel
//   HBM layer       : nB/(S*WB) records of B, sequential; a record of B is the same for all
//                     lanes of a wavefront, so it is fetched with scalar loads into SGPRs
// Re-composition of b with max_idx: in registers over a lane's sequential parts; across the
// WB wavefronts in LDS; across the S workgroups through a device-memory workspace and a
// second kernel (workgroup results combine in device memory only).
#include <limits.h>

#include <mutex>

#include "mdh_internal.h"

// Scratch memory of mdh_custom_reduce_static, the entry point for callers that cannot allocate: the
// partial (score, index) results of a reduction split over workgroups, 2 * S * nA int32.  One copy per
// GPU, held until the process ends.  In host code the name is a stand-in, not a device address: the
// address is looked up once per device (scratch_of_current_device) and only that pointer is used.
#define MDH_STATIC_SCRATCH_INTS (1u << 22)  // 16 MiB
static __device__ __align__(256) int32_t scratch[MDH_STATIC_SCRATCH_INTS];

namespace mdh {
namespace {

struct Best {
  int s, i;
};

__device__ __forceinline__ void max_idx(Best& x, int s, int i) {
  const bool take = (s > x.s) || (s == x.s && i < x.i);
  x.s = take ? s : x.s;
  x.i = take ? i : x.i;
}

// NF: number of fields the unrolled loops cover; if EXACT, nF == NF and a record of B is NF
// consecutive ints; otherwise nF < NF, the weights of the padding fields are 0 and their
// loads are clamped to the last real field (whatever they compare, they add 0).
template <int NF, bool EXACT, int RA, int WB, int WA>
__global__ __launch_bounds__(WA* WB * 64) void prl_kernel(
    const int* __restrict__ A, const int* __restrict__ B, const int* __restrict__ wp,
    const int* __restrict__ wm, int* __restrict__ out_s, int* __restrict__ out_i,
    int* __restrict__ ws, int nA, int nB, int nF, int S, int bchunk) {
  __shared__ int red_s[WB > 1 ? (WB - 1) * WA * RA * 64 : 1];
  __shared__ int red_i[WB > 1 ? (WB - 1) * WA * RA * 64 : 1];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wa = wave % WA, wb = wave / WA;
  const int nWGa = (nA + WA * 64 * RA - 1) / (WA * 64 * RA);
  const int ga = blockIdx.x % nWGa;  // workgroup part of a
  const int gs = blockIdx.x / nWGa;  // workgroup part of b
  const int abase = (ga * WA + wa) * 64 * RA;

  // weights: score = sum_f w_disagree[f] + sum_f [agree_f] * (w_agree[f] - w_disagree[f]),
  // evaluated in wrap-around unsigned arithmetic (exact whenever the true sums fit int32)
  unsigned dw[NF];
  unsigned base = 0;
#pragma unroll
  for (int f = 0; f < NF; ++f) {
    const bool real = EXACT || f < nF;
    const unsigned p = real ? (unsigned)wp[f] : 0u, m = real ? (unsigned)wm[f] : 0u;
    dw[f] = p - m;
    base += m;
  }

  // the lane's records of A (record a = abase + ra*64 + lane)
  int ar[RA][NF];
#pragma unroll
  for (int ra = 0; ra < RA; ++ra) {
    const int a = min(abase + ra * 64 + lane, nA - 1);
#pragma unroll
    for (int f = 0; f < NF; ++f) ar[ra][f] = A[(int64_t)a * nF + (EXACT ? f : min(f, nF - 1))];
  }

  const int part = gs * WB + wb;
  const int b0 = min((int64_t)part * bchunk, (int64_t)nB);
  const int b1 = min((int64_t)b0 + bchunk, (int64_t)nB);
  // The running best starts below every score; a part that holds records starts at its first index, so
  // that a true score of INT_MIN (which the strict test below never takes) still reports that index;
  // an empty part keeps INT_MAX and loses against every real pair under max_idx.
  Best best[RA];
#pragma unroll
  for (int ra = 0; ra < RA; ++ra) best[ra] = Best{INT_MIN, b0 < b1 ? b0 : INT_MAX};

  for (int b = b0; b < b1; ++b) {
    int br[NF];  // wavefront-uniform: scalar loads
    const int* rb = B + (int64_t)b * nF;
#pragma unroll
    for (int f = 0; f < NF; ++f) br[f] = rb[EXACT ? f : min(f, nF - 1)];
#pragma unroll
    for (int ra = 0; ra < RA; ++ra) {
      unsigned sc = base;
#pragma unroll
      for (int f = 0; f < NF; ++f) sc += (ar[ra][f] == br[f]) ? dw[f] : 0u;
      // b ascends, so a strict improvement keeps the smallest index among equal scores
      const int s = (int)sc;
      const bool take = s > best[ra].s;
      best[ra].s = take ? s : best[ra].s;
      best[ra].i = take ? b : best[ra].i;
    }
  }

  // wavefront layer -> workgroup: combine the WB partial results in LDS
  if (WB > 1) {
    if (wb > 0) {
#pragma unroll
      for (int ra = 0; ra < RA; ++ra) {
        const int o = (((wb - 1) * WA + wa) * RA + ra) * 64 + lane;
        red_s[o] = best[ra].s;
        red_i[o] = best[ra].i;
      }
    }
    __syncthreads();
    if (wb > 0) return;
#pragma unroll
    for (int w = 1; w < WB; ++w)
#pragma unroll
      for (int ra = 0; ra < RA; ++ra) {
        const int o = (((w - 1) * WA + wa) * RA + ra) * 64 + lane;
        max_idx(best[ra], red_s[o], red_i[o]);
      }
  }

  // output view (a,0) -> out_score[a], out_index[a]; or the workspace of part gs
#pragma unroll
  for (int ra = 0; ra < RA; ++ra) {
    const int a = abase + ra * 64 + lane;
    if (a < nA) {
      if (S > 1) {
        ws[(int64_t)gs * nA + a] = best[ra].s;
        ws[(int64_t)(S + gs) * nA + a] = best[ra].i;
      } else {
        out_s[a] = best[ra].s;
        out_i[a] = best[ra].i;
      }
    }
  }
}

// ---- the same instance for nF = 8 in the instruction kinds the vector ALU issues at twice the rate ----
//
// On this chip a wavefront instruction of the kinds {fp32 add / subtract / multiply / fused multiply-add,
// 32-bit integer add / subtract, bitwise logic, move} takes ~2.3 cycles of a SIMD (also with one scalar
// operand), every other kind (compare, select, min / max, three-operand integer forms) ~4.1; a result can
// feed an instruction issued four or more instructions later at no cost (all measured: the calibration
// kernels of this library).  The loop above spends 24 instructions of the slow kinds per pair.  Here
// wght is evaluated with three fast ones per field:
//     d = a_f - b_f            exact in fp32: both sides are stored as the float 2^23 + value
//     t = clamp(d * d)         1 if the fields differ (|d| >= 1), 0 if they agree
//     acc = fma(t, w_disagree_f - w_agree_f, acc)      acc starts at sum_f w_agree_f
// over eight independent (record of A, record of B) chains per lane, and max_idx is applied to blocks of
// four consecutive records of B: two three-operand maxima, one compare and one select per block instead
// of compare + maximum + select per record; which record of the winning block scored the maximum is
// found once at the end by scoring that block again.  Everything stays exact under these conditions,
// which the kernel checks itself: field values in [0, 2^23) (the records of A up front, those of B as
// they stream by -- a part that saw a value outside is evaluated again by the integer loop), and
// sum_f max(|w_agree_f|, |w_disagree_f|) < 2^24 (all partial sums are then integers fp32 holds exactly).
// The result is the unique (score, index) of the definition, bit for bit, on either path.
template <int RA, int WB, int WA>
__global__ __launch_bounds__(WA* WB * 64) void prl_fast_kernel(
    const int* __restrict__ A, const int* __restrict__ B, const int* __restrict__ wp,
    const int* __restrict__ wm, int* __restrict__ out_s, int* __restrict__ out_i,
    int* __restrict__ ws, int nA, int nB, int S, int bchunk) {
  constexpr int NF = 8;
  constexpr int BI = 8 / RA;  // records of B interleaved per step: RA * BI = 8 independent chains
  static_assert(RA == 2 || RA == 4, "eight chains per lane");
  __shared__ int red_s[WB > 1 ? (WB - 1) * WA * RA * 64 : 1];
  __shared__ int red_i[WB > 1 ? (WB - 1) * WA * RA * 64 : 1];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wa = wave % WA, wb = wave / WA;
  const int nWGa = (nA + WA * 64 * RA - 1) / (WA * 64 * RA);
  const int ga = blockIdx.x % nWGa, gs = blockIdx.x / nWGa;
  const int abase = (ga * WA + wa) * 64 * RA;
  const int part = gs * WB + wb;
  const int b0 = min((int64_t)part * bchunk, (int64_t)nB);
  const int b1 = min((int64_t)b0 + bchunk, (int64_t)nB);

  // weights (wavefront-uniform): integer form for the fallback loop, float form for the fast one
  unsigned dw[NF];
  unsigned base = 0;
  float ndw[NF];
  float agree_sum = 0.f;
  int64_t wabs = 0;
#pragma unroll
  for (int f = 0; f < NF; ++f) {
    const int p = wp[f], m = wm[f];
    dw[f] = (unsigned)p - (unsigned)m;
    base += (unsigned)m;
    ndw[f] = (float)((int64_t)m - (int64_t)p);
    agree_sum += (float)p;
    wabs += max(abs((int64_t)p), abs((int64_t)m));
  }
  bool fast = wabs < (1 << 24);

  // the lane's records of A, float-coded (the integer loop, should it be needed, reads them again)
  constexpr unsigned kCode = 0x4B000000u;  // bits of 2^23: kCode + v is the float 2^23 + v for 0 <= v < 2^23
  float fa[RA][NF];
  unsigned a_or = 0;
#pragma unroll
  for (int ra = 0; ra < RA; ++ra) {
    const int a = min(abase + ra * 64 + lane, nA - 1);
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      const unsigned v = (unsigned)A[(int64_t)a * NF + f];
      a_or |= v;
      fa[ra][f] = __uint_as_float(kCode + v);
    }
  }
  fast = fast && __builtin_amdgcn_ballot_w64((a_or >> 23) != 0) == 0;  // wavefront-uniform

  Best best[RA];
#pragma unroll
  for (int ra = 0; ra < RA; ++ra) best[ra] = Best{INT_MIN, b0 < b1 ? b0 : INT_MAX};

  unsigned b_or = 0;  // OR of every field value of B this wavefront has met (scalar)
  if (fast && b0 < b1) {
    float fbest[RA];
    int blk[RA];
#pragma unroll
    for (int ra = 0; ra < RA; ++ra) fbest[ra] = -3.0e38f, blk[ra] = b0;
    const float vbase = agree_sum + __uint_as_float(__float_as_uint(0.f) | (lane & 0));  // a vector register

    for (int bb = b0; bb < b1; bb += 4) {
      float sc[4][RA];
#pragma unroll
      for (int h = 0; h < 4; h += BI) {
        float fb[BI][NF];  // wavefront-uniform: scalar loads, coded on the scalar unit
#pragma unroll
        for (int u = 0; u < BI; ++u) {
          const int* rb = B + (int64_t)min(bb + h + u, b1 - 1) * NF;  // the tail repeats the last record
#pragma unroll
          for (int f = 0; f < NF; ++f) {
            const unsigned v = (unsigned)rb[f];
            b_or |= v;
            fb[u][f] = __uint_as_float(kCode + v);
          }
        }
        float acc[BI][RA];
#pragma unroll
        for (int f = 0; f < NF; ++f) {
          float t[BI][RA];
#pragma unroll
          for (int u = 0; u < BI; ++u)
#pragma unroll
            for (int ra = 0; ra < RA; ++ra) t[u][ra] = fa[ra][f] - fb[u][f];
#pragma unroll
          for (int u = 0; u < BI; ++u)
#pragma unroll
            for (int ra = 0; ra < RA; ++ra) asm("v_mul_f32_e64 %0, %1, %1 clamp" : "=v"(t[u][ra]) : "v"(t[u][ra]));
#pragma unroll
          for (int u = 0; u < BI; ++u)
#pragma unroll
            for (int ra = 0; ra < RA; ++ra)
              acc[u][ra] = __builtin_fmaf(t[u][ra], ndw[f], f == 0 ? vbase : acc[u][ra]);
        }
#pragma unroll
        for (int u = 0; u < BI; ++u)
#pragma unroll
          for (int ra = 0; ra < RA; ++ra) sc[h + u][ra] = acc[u][ra];
      }
      // max_idx over the block: a strictly larger maximum takes the block (b ascends: first block wins ties)
#pragma unroll
      for (int ra = 0; ra < RA; ++ra) {
        const float m = __builtin_fmaxf(__builtin_fmaxf(sc[0][ra], sc[1][ra]), sc[2][ra]);
        const float nb = __builtin_fmaxf(__builtin_fmaxf(fbest[ra], m), sc[3][ra]);
        blk[ra] = nb > fbest[ra] ? bb : blk[ra];
        fbest[ra] = nb;
      }
    }
    fast = (b_or >> 23) == 0;  // every value of B met on the way was in range: the scores are exact
    if (fast) {
      // which record of the winning block: score its (up to) four records again, the first that
      // reaches the maximum is the answer
#pragma unroll
      for (int ra = 0; ra < RA; ++ra) {
        int idx = blk[ra];
        bool found = false;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int b = min(blk[ra] + u, b1 - 1);
          const int* rb = B + (int64_t)b * NF;
          float acc = vbase;
#pragma unroll
          for (int f = 0; f < NF; ++f) {
            float t = fa[ra][f] - __uint_as_float(kCode + (unsigned)rb[f]);
            asm("v_mul_f32_e64 %0, %1, %1 clamp" : "=v"(t) : "v"(t));
            acc = __builtin_fmaf(t, ndw[f], acc);
          }
          const bool hit = !found && acc == fbest[ra];
          idx = hit ? b : idx;
          found = found || hit;
        }
        best[ra] = Best{(int)fbest[ra], idx};
      }
    }
  }
  if (!fast && b0 < b1) {
    // the integer loop of prl_kernel: any int32 field values and weights
    int ar[RA][NF];
#pragma unroll
    for (int ra = 0; ra < RA; ++ra) {
      const int a = min(abase + ra * 64 + lane, nA - 1);
#pragma unroll
      for (int f = 0; f < NF; ++f) ar[ra][f] = A[(int64_t)a * NF + f];
    }
    for (int b = b0; b < b1; ++b) {
      int br[NF];
      const int* rb = B + (int64_t)b * NF;
#pragma unroll
      for (int f = 0; f < NF; ++f) br[f] = rb[f];
#pragma unroll
      for (int ra = 0; ra < RA; ++ra) {
        unsigned sc = base;
#pragma unroll
        for (int f = 0; f < NF; ++f) sc += (ar[ra][f] == br[f]) ? dw[f] : 0u;
        const int s = (int)sc;
        const bool take = s > best[ra].s;
        best[ra].s = take ? s : best[ra].s;
        best[ra].i = take ? b : best[ra].i;
      }
    }
  }

  if (WB > 1) {
    if (wb > 0) {
#pragma unroll
      for (int ra = 0; ra < RA; ++ra) {
        const int o = (((wb - 1) * WA + wa) * RA + ra) * 64 + lane;
        red_s[o] = best[ra].s;
        red_i[o] = best[ra].i;
      }
    }
    __syncthreads();
    if (wb > 0) return;
#pragma unroll
    for (int w = 1; w < WB; ++w)
#pragma unroll
      for (int ra = 0; ra < RA; ++ra) {
        const int o = (((w - 1) * WA + wa) * RA + ra) * 64 + lane;
        max_idx(best[ra], red_s[o], red_i[o]);
      }
  }
#pragma unroll
  for (int ra = 0; ra < RA; ++ra) {
    const int a = abase + ra * 64 + lane;
    if (a < nA) {
      if (S > 1) {
        ws[(int64_t)gs * nA + a] = best[ra].s;
        ws[(int64_t)(S + gs) * nA + a] = best[ra].i;
      } else {
        out_s[a] = best[ra].s;
        out_i[a] = best[ra].i;
      }
    }
  }
}

// Second pass: fold the S workgroup-layer partial results with max_idx.
__global__ __launch_bounds__(256) void combine_maxidx_kernel(const int* __restrict__ ws,
                                                             int* __restrict__ out_s,
                                                             int* __restrict__ out_i, int nA, int S) {
  const int a = blockIdx.x * 256 + threadIdx.x;
  if (a >= nA) return;
  Best x{ws[a], ws[(int64_t)S * nA + a]};
  for (int s = 1; s < S; ++s) max_idx(x, ws[(int64_t)s * nA + a], ws[(int64_t)(S + s) * nA + a]);
  out_s[a] = x.s;
  out_i[a] = x.i;
}

template <int NF, bool EXACT, int RA, int WB, int WA>
mdh_status launch_t(const PrlPlan& pl, int64_t nA, int64_t nB, int nF, const int32_t* A,
                    const int32_t* B, const int32_t* wp, const int32_t* wm, int32_t* score,
                    int32_t* index, void* ws, hipStream_t st) {
  const int64_t nWGa = cdiv(nA, (int64_t)WA * 64 * RA);
  const int64_t nblocks = nWGa * pl.S;
  if (nblocks > 0x7fffffff) return MDH_ERR_SIZE;
  const int64_t bchunk = cdiv(nB, (int64_t)pl.S * WB);
  clear_stale_error();
  hipLaunchKernelGGL((prl_kernel<NF, EXACT, RA, WB, WA>), dim3((unsigned)nblocks), dim3(WA * WB * 64),
                     0, st, A, B, wp, wm, score, index, (int*)ws, (int)nA, (int)nB, nF, pl.S,
                     (int)bchunk);
  mdh_status r = launch_status();
  if (r != MDH_OK || pl.S <= 1) return r;
  clear_stale_error();
  hipLaunchKernelGGL(combine_maxidx_kernel, dim3((unsigned)cdiv(nA, 256)), dim3(256), 0, st,
                     (const int*)ws, score, index, (int)nA, pl.S);
  return launch_status();
}

template <int RA, int WB, int WA>
mdh_status launch_fast(const PrlPlan& pl, int64_t nA, int64_t nB, const int32_t* A, const int32_t* B,
                       const int32_t* wp, const int32_t* wm, int32_t* score, int32_t* index, void* ws,
                       hipStream_t st) {
  const int64_t nWGa = cdiv(nA, (int64_t)WA * 64 * RA);
  const int64_t nblocks = nWGa * pl.S;
  if (nblocks > 0x7fffffff) return MDH_ERR_SIZE;
  const int64_t bchunk = cdiv(nB, (int64_t)pl.S * WB);
  clear_stale_error();
  hipLaunchKernelGGL((prl_fast_kernel<RA, WB, WA>), dim3((unsigned)nblocks), dim3(WA * WB * 64), 0, st, A, B,
                     wp, wm, score, index, (int*)ws, (int)nA, (int)nB, pl.S, (int)bchunk);
  mdh_status r = launch_status();
  if (r != MDH_OK || pl.S <= 1) return r;
  clear_stale_error();
  hipLaunchKernelGGL(combine_maxidx_kernel, dim3((unsigned)cdiv(nA, 256)), dim3(256), 0, st,
                     (const int*)ws, score, index, (int)nA, pl.S);
  return launch_status();
}

template <int RA, int WB, int WA>
mdh_status launch_nf(const PrlPlan& pl, int64_t nA, int64_t nB, int nF, const int32_t* A,
                     const int32_t* B, const int32_t* wp, const int32_t* wm, int32_t* score,
                     int32_t* index, void* ws, hipStream_t st) {
  // eight fields, two or four records of A per lane: the loop built from the fast instruction kinds
  if constexpr (RA == 2 || RA == 4)
    if (nF == 8) return launch_fast<RA, WB, WA>(pl, nA, nB, A, B, wp, wm, score, index, ws, st);
  if (nF == 8) return launch_t<8, true, RA, WB, WA>(pl, nA, nB, nF, A, B, wp, wm, score, index, ws, st);
  if (nF <= 4) return launch_t<4, false, RA, WB, WA>(pl, nA, nB, nF, A, B, wp, wm, score, index, ws, st);
  if (nF < 8) return launch_t<8, false, RA, WB, WA>(pl, nA, nB, nF, A, B, wp, wm, score, index, ws, st);
  return launch_t<16, false, RA, WB, WA>(pl, nA, nB, nF, A, B, wp, wm, score, index, ws, st);
}

std::mutex g_scratch_mutex;
int32_t* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, looked up on the first call per device.
mdh_status scratch_of_current_device(int32_t** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MDH_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      g_last_launch_error = e;
      return MDH_ERR_LAUNCH;
    }
    g_scratch_ptr[dev] = (int32_t*)p;
  }
  *out = g_scratch_ptr[dev];
  return MDH_OK;
}

}  // namespace

mdh_status launch_prl(const PrlPlan& pl, int64_t nA, int64_t nB, int nF, const int32_t* A,
                      const int32_t* B, const int32_t* wp, const int32_t* wm, int32_t* score,
                      int32_t* index, void* ws, hipStream_t st) {
#define MDH_PRL(ra, wb, wa) \
  if (pl.RA == ra && pl.WB == wb && pl.WA == wa) return launch_nf<ra, wb, wa>(pl, nA, nB, nF, A, B, wp, wm, score, index, ws, st);
  MDH_PRL(2, 4, 1)
  MDH_PRL(4, 4, 1)
  MDH_PRL(1, 4, 1)
  MDH_PRL(2, 2, 2)
  MDH_PRL(4, 2, 2)
  MDH_PRL(2, 1, 4)
  MDH_PRL(4, 1, 4)
  MDH_PRL(2, 8, 1)
  MDH_PRL(4, 8, 1)
#undef MDH_PRL
  return MDH_ERR_UNSUPPORTED;
}

}  // namespace mdh

extern "C" mdh_status mdh_custom_reduce_static(int64_t nA, int64_t nB, int32_t nF, const int32_t* A,
                                               const int32_t* B, const int32_t* w_agree,
                                               const int32_t* w_disagree, int32_t* out_score,
                                               int32_t* out_index, const mdh_tile_params* params,
                                               void* stream) {
  using namespace mdh;
  constexpr int64_t kMaxElems = 0x7fffffff;
  if (nA < 0 || nB < 1 || nF < 1 || nF > 16) return MDH_ERR_SIZE;
  if (nA > kMaxElems || nB > kMaxElems || nA * nF > kMaxElems || nB * nF > kMaxElems) return MDH_ERR_SIZE;
  const int64_t sizes[2] = {nA, nB};
  PrlPlan pl;
  mdh_status st = plan_prl(sizes, params, &pl);
  if (st != MDH_OK) return st;
  if (nA == 0) return MDH_OK;
  if (!A || !B || !w_agree || !w_disagree || !out_score || !out_index) return MDH_ERR_NULL;
  // the split reduction's partial results must fit the static array; nothing is allocated instead
  if (pl.S > 1 && (int64_t)pl.S * nA * 2 > (int64_t)MDH_STATIC_SCRATCH_INTS) return MDH_ERR_STATIC_LIMIT;
  int32_t* ws = nullptr;
  if (pl.S > 1 && (st = scratch_of_current_device(&ws)) != MDH_OK) return st;
  // every (part, record) slot the second pass reads is written by the first kernel of this call:
  // nothing left by an earlier call is read, so nothing has to be cleared
  return launch_prl(pl, nA, nB, nF, A, B, w_agree, w_disagree, out_score, out_index, ws, (hipStream_t)stream);
}

extern "C" size_t mdh_static_scratch_bytes(void) { return (size_t)MDH_STATIC_SCRATCH_INTS * sizeof(int32_t); }
