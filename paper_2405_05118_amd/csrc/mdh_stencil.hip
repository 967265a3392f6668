// Jacobi-3D instance of md_hom(J_3D, (++,++,++)) for gfx950.
//
// All three dimensions are concatenation dimensions, so the whole computation is a
// de-composition of the output index space (paper: Section "Examples", Subfigure 4)
// and the kernel is bound by HBM traffic: every input cell should cross HBM once.
//
// De-composition (tuning parameter 0 and D2 in the paper's table):
//   workgroup layer : (nx/SI) x (ny/TJ) x (nz/KT) parts, TJ = TY*RJ, KT = 4*LK
//   HBM layer       : SI consecutive planes of dimension i, streamed sequentially
//   wavefront layer : TY lane-rows along j  x  LK/64 wavefronts along k
//   lane layer      : 64 lanes along k (k is the contiguous dimension -> coalescing); for narrow
//                     grids LK = 32 or 16 lanes along k and 2 or 4 lane-rows of j per wavefront
//   VGPR layer      : RJ rows (j) x 4 columns (k) per lane
// Input staging (parameter D3): the plane being processed lives in LDS so that the j- and
// k-neighbours owned by other lanes are read from LDS instead of HBM/L2; the i-neighbours
// are the lane's own values of the previous/next plane and stay in registers.
#include "mdh_internal.h"

namespace mdh {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));

// Streaming accesses: the centre rows of the input and the whole output are touched once per
// kernel, so both are non-temporal (measured 5.5 -> 6.0 TB/s; halo rows stay cacheable).
__device__ __forceinline__ f4 ld_stream(const float* p) { return __builtin_nontemporal_load((const f4u*)p); }
__device__ __forceinline__ void st_stream(float* p, f4 v) { __builtin_nontemporal_store(v, (f4u*)p); }

template <int RJ, int TY, int LK>
struct StencilCfg {
  static constexpr int TJ = TY * RJ;
  static constexpr int KT = LK * 4;
  static constexpr int NT = TY * LK;
  static constexpr int PITCH = KT + 8;  // floats per LDS row: 3 pad | halo | KT | halo | 3 pad
  static constexpr int ROWS = TJ + 2;
  static constexpr int PLANE = ROWS * PITCH;
};

// Values a lane holds for one input plane: its RJ x 4 centre block.
template <int RJ>
struct Block {
  f4 v[RJ];
};

template <int RJ, int TY, int LK, bool GUARD>
__device__ __forceinline__ void stencil_tile(const float* __restrict__ in, float* __restrict__ out,
                                             int nx, int ny, int nz, int i_begin, int i_end,
                                             int jt0, int kt0, float c0, float c1, float* lds) {
  using C = StencilCfg<RJ, TY, LK>;
  const int tk = threadIdx.x % LK;
  const int ty = threadIdx.x / LK;
  const int j0 = jt0 + ty * RJ;  // first output row of this lane
  const int k0 = kt0 + tk * 4;   // first output column of this lane
  const int64_t sy = nz + 2;
  const int64_t sx = (int64_t)(ny + 2) * sy;

  // LDS position of input cell (row r of the tile, column c of the tile), r in [0,TJ+2), c in [0,KT+2)
  auto lpos = [](int r, int c) { return r * C::PITCH + c + 3; };

  // ---- global loads of one input plane (input coordinate ip) into registers ----
  auto load_centres = [&](int ip, Block<RJ>& b) {
    const float* base = in + (int64_t)ip * sx + (int64_t)(j0 + 1) * sy + (k0 + 1);
#pragma unroll
    for (int jj = 0; jj < RJ; ++jj) {
      if (!GUARD) {
        b.v[jj] = ld_stream(base + jj * sy);
      } else {
        // guard on the INPUT coordinates (row j0+jj+1 <= ny+1, column k0+e+1 <= nz+1): the
        // cells just outside a ragged tile's valid outputs are still neighbours of valid cells
        f4 t = {0.f, 0.f, 0.f, 0.f};
        if (j0 + jj <= ny) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (k0 + e <= nz) t[e] = base[jj * sy + e];
        }
        b.v[jj] = t;
      }
    }
  };
  // j-halo rows (tile rows 0 and TJ+1) and k-halo columns (tile columns 0 and KT+1)
  constexpr int NH = (2 + TY - 1) / TY;  // halo rows per lane-row
  auto load_halos = [&](int ip, f4 (&hj)[NH], float& hk) {
    const float* pl = in + (int64_t)ip * sx;
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      const int side = ty + h * TY;  // 0: row above the tile, 1: row below
      f4 t = {0.f, 0.f, 0.f, 0.f};
      if (side < 2) {
        const int jr = jt0 + (side ? C::TJ + 1 : 0);  // input row
        const float* p = pl + (int64_t)jr * sy + (k0 + 1);
        if (!GUARD) {
          t = *(const f4u*)p;  // halo rows are shared with the neighbouring workgroup: keep them cached
        } else if (jr < ny + 2) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (k0 + e <= nz) t[e] = p[e];
        }
      }
      hj[h] = t;
    }
    hk = 0.f;
    if (threadIdx.x < 2 * C::TJ) {
      const int side = threadIdx.x / C::TJ, r = threadIdx.x % C::TJ;
      const int jr = jt0 + r + 1;                       // input row
      const int kc = kt0 + (side ? C::KT + 1 : 0);      // input column
      if (!GUARD || (jr < ny + 2 && kc < nz + 2)) hk = pl[(int64_t)jr * sy + kc];
    }
  };
  auto stage = [&](float* buf, const Block<RJ>& b, const f4 (&hj)[NH], float hk) {
#pragma unroll
    for (int jj = 0; jj < RJ; ++jj) *(f4*)(buf + lpos(ty * RJ + jj + 1, tk * 4 + 1)) = b.v[jj];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      const int side = ty + h * TY;
      if (side < 2) *(f4*)(buf + lpos(side ? C::TJ + 1 : 0, tk * 4 + 1)) = hj[h];
    }
    if (threadIdx.x < 2 * C::TJ) {
      const int side = threadIdx.x / C::TJ, r = threadIdx.x % C::TJ;
      buf[lpos(r + 1, side ? C::KT + 1 : 0)] = hk;
    }
  };
  // in-plane neighbour sum of the lane's block: (j-1) + (j+1) + (k-1) + (k+1)
  auto inplane = [&](const float* buf, const Block<RJ>& b, Block<RJ>& s) {
    const f4 up = *(const f4*)(buf + lpos(ty * RJ, tk * 4 + 1));
    const f4 dn = *(const f4*)(buf + lpos(ty * RJ + RJ + 1, tk * 4 + 1));
#pragma unroll
    for (int jj = 0; jj < RJ; ++jj) {
      const f4 jm = jj == 0 ? up : b.v[jj - 1];
      const f4 jp = jj == RJ - 1 ? dn : b.v[jj + 1];
      const float kl = buf[lpos(ty * RJ + jj + 1, tk * 4)];
      const float kr = buf[lpos(ty * RJ + jj + 1, tk * 4 + 5)];
      const f4 c = b.v[jj];
      f4 km = {kl, c[0], c[1], c[2]};
      f4 kp = {c[1], c[2], c[3], kr};
      s.v[jj] = (jm + jp) + (km + kp);
    }
  };

  Block<RJ> cm, cc, acc, nxt;  // centres of plane q-1, of plane q; partial sums; plane q+1
  f4 hj[NH];
  float hk;

  // plane i_begin: only an i-neighbour, no in-plane work
  load_centres(i_begin, cm);
  // plane i_begin+1: first centre plane
  load_centres(i_begin + 1, cc);
  load_halos(i_begin + 1, hj, hk);
  // iteration q handles input plane q as the centre plane of output plane q-1
  for (int q = i_begin + 1; q <= i_end; ++q) {
    float* buf = lds + ((q & 1) ? C::PLANE : 0);
    stage(buf, cc, hj, hk);
    // prefetch plane q+1 (always needed as an i-neighbour; halos only if it is a centre plane)
    load_centres(q + 1, nxt);
    if (q + 1 <= i_end) load_halos(q + 1, hj, hk);
    __syncthreads();
    inplane(buf, cc, acc);
    // out[q-1] = c0*x[q] + c1*(inplane(q) + x[q-1] + x[q+1])
    float* orow = out + ((int64_t)(q - 1) * ny + j0) * nz + k0;
#pragma unroll
    for (int jj = 0; jj < RJ; ++jj) {
      const f4 nb = (acc.v[jj] + cm.v[jj]) + nxt.v[jj];
      f4 r;
#pragma unroll
      for (int e = 0; e < 4; ++e) r[e] = __builtin_fmaf(c0, cc.v[jj][e], c1 * nb[e]);
      if (!GUARD) {
        st_stream(orow + (int64_t)jj * nz, r);
      } else if (j0 + jj < ny) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (k0 + e < nz) orow[(int64_t)jj * nz + e] = r[e];
      }
    }
#pragma unroll
    for (int jj = 0; jj < RJ; ++jj) {
      cm.v[jj] = cc.v[jj];
      cc.v[jj] = nxt.v[jj];
    }
  }
}

template <int RJ, int TY, int LK>
__global__ __launch_bounds__(TY* LK) void stencil_kernel(const float* __restrict__ in,
                                                          float* __restrict__ out, int nx, int ny,
                                                          int nz, int SI, int njt, int nkt,
                                                          float c0, float c1) {
  using C = StencilCfg<RJ, TY, LK>;
  __shared__ __attribute__((aligned(16))) float lds[2 * C::PLANE];

  // XCD-aware order: consecutive workgroup ids go to different XCDs (8 of them, each with
  // its own L2); give every XCD one contiguous chunk of tiles so that tiles sharing halo
  // rows/planes hit the same L2.
  int b = blockIdx.x;
  const int nb = gridDim.x;
  if ((nb & 7) == 0) b = (b & 7) * (nb >> 3) + (b >> 3);
  const int kt = b % nkt;
  const int jt = (b / nkt) % njt;
  const int is = b / (nkt * njt);

  const int i_begin = is * SI;
  const int i_end = min(i_begin + SI, nx);
  const int jt0 = jt * C::TJ, kt0 = kt * C::KT;
  const bool full = (jt0 + C::TJ <= ny) && (kt0 + C::KT <= nz);
  if (full)
    stencil_tile<RJ, TY, LK, false>(in, out, nx, ny, nz, i_begin, i_end, jt0, kt0, c0, c1, lds);
  else
    stencil_tile<RJ, TY, LK, true>(in, out, nx, ny, nz, i_begin, i_end, jt0, kt0, c0, c1, lds);
}

template <int RJ, int TY, int LK>
mdh_status launch_t(const StencilPlan& pl, int64_t nx, int64_t ny, int64_t nz, const float* in,
                    float* out, float c0, float c1, hipStream_t st) {
  using C = StencilCfg<RJ, TY, LK>;
  const int64_t njt = cdiv(ny, C::TJ), nkt = cdiv(nz, C::KT), nis = cdiv(nx, pl.SI);
  const int64_t nblocks = njt * nkt * nis;
  if (nblocks <= 0 || nblocks > 0x7fffffff) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL((stencil_kernel<RJ, TY, LK>), dim3((unsigned)nblocks), dim3(C::NT), 0, st, in,
                     out, (int)nx, (int)ny, (int)nz, pl.SI, (int)njt, (int)nkt, c0, c1);
  return launch_status();
}

}  // namespace

mdh_status launch_stencil(const StencilPlan& pl, int64_t nx, int64_t ny, int64_t nz,
                          const float* in, float* out, float c0, float c1, hipStream_t st) {
#define MDH_ST(rj, ty, lk) \
  if (pl.RJ == rj && pl.TY == ty && pl.LK == lk) return launch_t<rj, ty, lk>(pl, nx, ny, nz, in, out, c0, c1, st);
  MDH_ST(4, 2, 128)
  MDH_ST(2, 2, 128)
  MDH_ST(8, 2, 128)
  MDH_ST(4, 4, 128)
  MDH_ST(2, 4, 128)
  MDH_ST(4, 1, 128)
  MDH_ST(8, 1, 128)
  MDH_ST(4, 4, 64)
  MDH_ST(2, 4, 64)
  MDH_ST(4, 2, 64)
  MDH_ST(4, 8, 32)   // narrow grids (nz <= 128): a wavefront spans 2 lane-rows of 32 lanes
  MDH_ST(4, 16, 16)  // nz <= 64: 4 lane-rows of 16 lanes
#undef MDH_ST
  return MDH_ERR_UNSUPPORTED;
}

}  // namespace mdh
