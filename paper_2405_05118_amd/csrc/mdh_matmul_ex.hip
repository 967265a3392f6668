// Batched MatMul with transposed views for gfx950:
//   bMatMul  = md_hom(*, (++,++,++,+)) over (b,i,j,k)  -- one more concatenation dimension
//   MatMul^T = the same md_hom as MatMul; only the index functions of the views change:
//              (i,j,k)->A[k,i] instead of A[i,k], (i,j,k)->B[j,k] instead of B[k,j],
//              (i,j,0)->C[j,i] instead of C[i,j]
// (paper: Section "Examples", Subfigure 1, routines 4 and 5; output view example "transposed
// matrix multiplication").  The (de/re)-composition is the one of mdh_matmul.hip; what the
// transposed views change is which dimension of an operand tile is contiguous in memory, i.e.
// the layout of the staged tile (parameters D4/R4 of the tuning table):
//   k contiguous    (A plain, B transposed): tile kept as [free][k]; a lane's four k of one MFMA
//                                            step group come from one 16-byte LDS read
//   free contiguous (A transposed, B plain): tile kept as [k][free]; four 4-byte LDS reads
//   C transposed: the four consecutive rows an accumulator register group holds become four
//                 consecutive addresses -> 16-byte stores
#include "mdh_internal.h"

namespace mdh {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
typedef float f16 __attribute__((ext_vector_type(16)));

// One operand tile of EXT free-dimension elements x BK reduction elements.
//   KC (k contiguous in memory):    element (f, k) at  base[f * ld + k];  LDS [EXT][BK + 4]
//   !KC (free dimension contiguous): element (f, k) at  base[k * ld + f];  LDS [BK][EXT + 4]
template <int EXT, int BK, bool KC, int NT>
struct Operand {
  static constexpr int ROWS = KC ? EXT : BK;   // rows of the tile as it lies in memory
  static constexpr int COLS = KC ? BK : EXT;   // contiguous extent
  static constexpr int P = COLS + 4;           // LDS pitch
  static constexpr int SIZE = ROWS * P;
  static constexpr int F4 = ROWS * COLS / 4;
  static constexpr int LD = (F4 + NT - 1) / NT;

  f4 r[LD];

  // f0: first free index of the tile, flim: extent of the free dimension; k0/klim likewise
  // MODE 0: interior tile, the reduction extent a multiple of BK -- no checks at all;
  // MODE 1: interior tile, ragged reduction extent -- only the last k-tile is checked (a
  //         workgroup-uniform test per k-tile);  MODE 2: the tile touches an edge of C.
  template <int MODE>
  __device__ __forceinline__ void load(const float* __restrict__ base, int64_t ld, int f0, int flim,
                                       int k0, int klim) {
    const int tid = threadIdx.x;
    const bool fast = MODE == 0 || (MODE == 1 && k0 + BK <= klim);
#pragma unroll
    for (int x = 0; x < LD; ++x) {
      const int f = tid + x * NT;
      const int row = f / (COLS / 4), c4 = f % (COLS / 4);
      f4 v = {0.f, 0.f, 0.f, 0.f};
      if (F4 % NT == 0 || f < F4) {
        const int grow = (KC ? f0 : k0) + row, gcol = (KC ? k0 : f0) + c4 * 4;
        const int rlim = KC ? flim : klim, clim = KC ? klim : flim;
        const float* p = base + (int64_t)grow * ld + gcol;
        if (fast) {
          v = *(const f4u*)p;
        } else if (grow < rlim) {
          // edge tiles and ragged k: still one 16-byte load wherever all four elements exist
          if (gcol + 3 < clim) {
            v = *(const f4u*)p;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (gcol + e < clim) v[e] = p[e];
          }
        }
      }
      r[x] = v;
    }
  }
  __device__ __forceinline__ void store(float* st) const {
    const int tid = threadIdx.x;
#pragma unroll
    for (int x = 0; x < LD; ++x) {
      const int f = tid + x * NT;
      const int row = f / (COLS / 4), c4 = f % (COLS / 4);
      if (F4 % NT == 0 || f < F4) *(f4*)(st + row * P + c4 * 4) = r[x];
    }
  }
  // A lane's view of the staged tile: lane (l32, lh) of the wavefront whose blocks start at free
  // offset woff contributes, to the MFMAs of k-step group kk and block blk, the four values
  // k = kk + 4*lh + t, t = 0..3, of free index woff + 32*blk + l32.  The lane-dependent part of the
  // address is folded into one pointer so that the reads of a step differ by constants only (the
  // 4-byte reads then pair up into two-address LDS instructions).
  static __device__ __forceinline__ const float* lane_base(const float* st, int woff, int l32, int lh) {
    return KC ? st + (woff + l32) * P + 4 * lh : st + (4 * lh) * P + woff + l32;
  }
  static __device__ __forceinline__ f4 frag(const float* lb, int blk, int kk) {
    if (KC) return *(const f4*)(lb + blk * 32 * P + kk);
    f4 v;
#pragma unroll
    for (int t = 0; t < 4; ++t) v[t] = lb[(kk + t) * P + blk * 32];
    return v;
  }
};

template <int BM, int BN, int BK, int WM, int WN, bool TA, bool TB, bool TC, int MODE>
__device__ __forceinline__ void gemm_ex_tile(const float* __restrict__ A, const float* __restrict__ B,
                                             float* __restrict__ Cout, int M, int N, int K, int m0,
                                             int n0, int kbeg, int kend, float* lds) {
  constexpr bool GUARD = MODE == 2;
  constexpr int WAVES_N = BN / WN, NT = (BM / WM) * WAVES_N * 64;
  constexpr int MI = WM / 32, NI = WN / 32;
  using OpA = Operand<BM, BK, !TA, NT>;
  using OpB = Operand<BN, BK, TB, NT>;
  constexpr int STAGE = OpA::SIZE + OpB::SIZE;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int l32 = lane & 31, lh = lane >> 5;
  const int64_t lda = TA ? M : K, ldb = TB ? K : N;

  f16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  struct Frag {
    f4 a[MI], b[NI];
  };
  auto load_frag = [&](Frag& f, const float* as, const float* bs, int kk) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) f.a[mi] = OpA::frag(as, mi, kk);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) f.b[ni] = OpB::frag(bs, ni, kk);
  };
  auto mma = [&](const Frag& f) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.a[mi][t], f.b[ni][t], acc[mi][ni], 0, 0, 0);
  };
  auto compute = [&](const float* st) {
    const float* as = OpA::lane_base(st, wm * WM, l32, lh);
    const float* bs = OpB::lane_base(st + OpA::SIZE, wn * WN, l32, lh);
    if (MI * NI >= 4) {
      // as in the MatMul kernel: the fragments of k-step kk+8 are read while the MFMAs of step kk
      // run, one LDS read instruction per few MFMAs.  A k-contiguous operand block is one 16-byte
      // read, the other layout four 4-byte reads that pair up into two instructions.
      constexpr int NR = (TA ? 2 : 1) * MI + (TB ? 1 : 2) * NI, NM = 4 * MI * NI, PER = NM / NR;
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

  // two k-tiles in flight (tile kt+2 is requested while tile kt is computed and tile kt+1 waits in
  // registers), the pipeline of the MatMul kernel
  struct Staged {
    OpA a;
    OpB b;
  };
  auto load_global = [&](Staged& g, int k0) {
    g.a.template load<MODE>(A, lda, m0, M, k0, kend);
    g.b.template load<MODE>(B, ldb, n0, N, k0, kend);
  };
  auto store_lds = [&](const Staged& g, float* st) {
    g.a.store(st);
    g.b.store(st + OpA::SIZE);
  };
  const int nk = (kend - kbeg + BK - 1) / BK;
  float* const st0 = lds;
  float* const st1 = lds + STAGE;
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

  // output view: (i,j,0) -> C[i,j], or C[j,i] for the transposed view
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int col = n0 + wn * WN + ni * 32 + l32;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int row = m0 + wm * WM + mi * 32 + 8 * g + 4 * lh;  // rows row..row+3 in registers 4g..4g+3
        if (TC) {
          float* p = Cout + (int64_t)col * M + row;
          if (!GUARD) {
            *(f4u*)p = (f4){acc[mi][ni][4 * g], acc[mi][ni][4 * g + 1], acc[mi][ni][4 * g + 2], acc[mi][ni][4 * g + 3]};
          } else if (col < N) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (row + e < M) p[e] = acc[mi][ni][4 * g + e];
          }
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (!GUARD || (row + e < M && col < N)) Cout[(int64_t)(row + e) * N + col] = acc[mi][ni][4 * g + e];
        }
      }
    }
}

template <int BM, int BN, int BK, int WM, int WN, bool TA, bool TB, bool TC>
__global__ __launch_bounds__(((BM / WM) * (BN / WN) * 64)) void matmul_ex_kernel(
    const float* __restrict__ A, const float* __restrict__ B, float* __restrict__ C,
    float* __restrict__ ws, int M, int N, int K, int tiles_m, int tiles_n, int S, int kchunk,
    int nbatch) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  // one more ++ dimension on the workgroup layer: the grid is batch x S x tiles, flattened.
  // XCD-aware order: workgroup ids are dealt round-robin to the 8 XCDs; each XCD gets a contiguous
  // run (whole batches when there are at least 8), walked in bands of 8 tile-rows so that the tiles
  // resident on one XCD at a time share few panels of A and B in that XCD's L2.
  int b = blockIdx.x;
  const int nb = gridDim.x;
  if ((nb & 7) == 0) b = (b & 7) * (nb >> 3) + (b >> 3);
  const int tiles = tiles_m * tiles_n;
  const int batch = b / (tiles * S);
  b -= batch * tiles * S;
  const int s = b / tiles;
  const int t = b % tiles;
  constexpr int GM = 8;
  const int band = t / (GM * tiles_n);
  const int band_rows = min(GM, tiles_m - band * GM);
  const int in_band = t - band * GM * tiles_n;
  const int tm = band * GM + in_band % band_rows;
  const int tn = in_band / band_rows;
  const int m0 = tm * BM, n0 = tn * BN;
  const int kbeg = s * kchunk;
  const int kend = min(K, kbeg + kchunk);
  const int64_t mn = (int64_t)M * N;
  const float* Ab = A + (int64_t)batch * M * K;
  const float* Bb = B + (int64_t)batch * K * N;
  float* out = S > 1 ? ws + ((int64_t)s * nbatch + batch) * mn : C + (int64_t)batch * mn;
  const bool full = (m0 + BM <= M) && (n0 + BN <= N) && kend > kbeg;
  if (full && (kend - kbeg) % BK == 0)
    gemm_ex_tile<BM, BN, BK, WM, WN, TA, TB, TC, 0>(Ab, Bb, out, M, N, K, m0, n0, kbeg, kend, lds);
  else if (full)
    gemm_ex_tile<BM, BN, BK, WM, WN, TA, TB, TC, 1>(Ab, Bb, out, M, N, K, m0, n0, kbeg, kend, lds);
  else
    gemm_ex_tile<BM, BN, BK, WM, WN, TA, TB, TC, 2>(Ab, Bb, out, M, N, K, m0, n0, kbeg, kend, lds);
}

template <int BM, int BN, int BK, int WM, int WN, bool TA, bool TB, bool TC>
mdh_status launch_t(const GemmExPlan& pl, int64_t batch, int64_t M, int64_t N, int64_t K,
                    const float* A, const float* B, float* C, void* ws, hipStream_t st) {
  constexpr int NT = (BM / WM) * (BN / WN) * 64;
  using OpA = Operand<BM, BK, !TA, NT>;
  using OpB = Operand<BN, BK, TB, NT>;
  constexpr int LDS_BYTES = 2 * (OpA::SIZE + OpB::SIZE) * 4;
  auto kern = matmul_ex_kernel<BM, BN, BK, WM, WN, TA, TB, TC>;
  static int64_t lds_allowed[kMaxDevices] = {};
  if (allow_dynamic_lds((const void*)kern, LDS_BYTES, lds_allowed) != MDH_OK) return MDH_ERR_LAUNCH;
  const int S = pl.g.S;
  const int64_t tm = cdiv(M, BM), tn = cdiv(N, BN);
  const int64_t kchunk = cdiv(cdiv(K, S), BK) * BK;
  const int64_t nblocks = tm * tn * S * batch;
  if (nblocks > 0x7fffffff) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(NT), LDS_BYTES, st, A, B, C,
                     (float*)ws, (int)M, (int)N, (int)K, (int)tm, (int)tn, S, (int)kchunk, (int)batch);
  mdh_status r = launch_status();
  if (r != MDH_OK || S <= 1) return r;
  return launch_combine_sum((const float*)ws, C, batch * M * N, S, st);
}

template <int BM, int BN, int BK, int WM, int WN>
mdh_status launch_trans(const GemmExPlan& pl, int64_t batch, int64_t M, int64_t N, int64_t K,
                        const float* A, const float* B, float* C, void* ws, hipStream_t st) {
  const int code = (pl.ta ? 4 : 0) | (pl.tb ? 2 : 0) | (pl.tc ? 1 : 0);
  switch (code) {
#define MDH_T(c, ta, tb, tc) \
  case c: return launch_t<BM, BN, BK, WM, WN, ta, tb, tc>(pl, batch, M, N, K, A, B, C, ws, st);
    MDH_T(0, false, false, false)
    MDH_T(1, false, false, true)
    MDH_T(2, false, true, false)
    MDH_T(3, false, true, true)
    MDH_T(4, true, false, false)
    MDH_T(5, true, false, true)
    MDH_T(6, true, true, false)
    MDH_T(7, true, true, true)
#undef MDH_T
  }
  return MDH_ERR_UNSUPPORTED;
}

}  // namespace

mdh_status launch_matmul_ex(const GemmExPlan& pl, int64_t batch, int64_t M, int64_t N, int64_t K,
                            const float* A, const float* B, float* C, void* ws, hipStream_t st) {
  if (pl.skinny) return launch_matmul_skinny(pl, batch, M, N, K, A, B, C, ws, st);
#define MDH_MX(bm, bn, bk, wm, wn)                                                                   \
  if (pl.g.BM == bm && pl.g.BN == bn && pl.g.BK == bk && pl.g.WM == wm && pl.g.WN == wn)             \
    return launch_trans<bm, bn, bk, wm, wn>(pl, batch, M, N, K, A, B, C, ws, st);
  MDH_MX(128, 128, 32, 64, 64)
  MDH_MX(128, 64, 32, 64, 32)
  MDH_MX(64, 64, 32, 32, 32)
  MDH_MX(128, 128, 16, 64, 64)
  MDH_MX(128, 64, 16, 64, 32)
  MDH_MX(64, 64, 16, 32, 32)
  MDH_MX(32, 128, 16, 32, 32)
  MDH_MX(32, 64, 16, 32, 32)
#undef MDH_MX
  return MDH_ERR_UNSUPPORTED;
}

}  // namespace mdh
