// MCC_Capsule: multi-channel convolution on 4 x 4 matrices instead of scalars (paper: Section
// "Examples", Subfigure 2; Appendix "Data Characteristics used in Deep Neural Networks": MCC with
// three more dimensions MI, MJ, MK of size 4).  Ten dimensions (n,p,q,k,mi,mj | c,r,s,mk):
//   out[n,p,q,k,mi,mj] = sum_{c,r,s,mk} in[n, p*sh+r, q*sw+s, c, mi, mk] * filt[k, r, s, c, mk, mj]
//
// As a contraction the rows are (pixel, mi), the columns (k, mj) and the reduction (r, s, c, mk).
// In both buffers mk is contiguous for the A operand only; the filter slice is therefore staged in
// LDS with its 4 x 4 matrices transposed ([mj][mk]), after which BOTH MFMA operands are one 16-byte
// LDS read: a lane's four consecutive values are mk = 0..3 of one (s,c) pair, and the two lane
// halves of v_mfma_f32_32x32x2_f32 take two consecutive (s,c) pairs.  s and c are fused into one
// sequential dimension j = s*C + c (adjacent in memory for a fixed r), padded to an even extent
// with zero filter entries.
//
// De-composition:
//   workgroup layer : N x (P/4) x (Q/8) x (K/(8*NI))
//   LDS             : the input patch (3*sh+R rows) and the whole filter slice, staged once
//   wavefront layer : 4 output rows p (one per wavefront)
//   block           : (8 q x 4 mi) x (8 k x 4 mj) x 2 of mk; NI blocks along k per wavefront
#include "mdh_internal.h"

namespace mdh {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
typedef float f16 __attribute__((ext_vector_type(16)));

constexpr int CAP_TP = 4, CAP_TQ = 8, CAP_NT = 256;

template <int NI>
__global__ __launch_bounds__(CAP_NT) void capsule_kernel(const float* __restrict__ in,
                                                         const float* __restrict__ filt,
                                                         float* __restrict__ out, int H, int W, int C,
                                                         int K, int R, int S, int sh, int sw, int P,
                                                         int Q, int tp_n, int tq_n, int tk_n, int J2,
                                                         int PWF, int PFR) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, h = lane >> 5;
  int b = blockIdx.x;
  const int nb = gridDim.x;
  if ((nb & 7) == 0) b = (b & 7) * (nb >> 3) + (b >> 3);  // contiguous run of tiles per XCD
  const int tk = b % tk_n;
  const int tq = (b / tk_n) % tq_n;
  const int tp = (b / (tk_n * tq_n)) % tp_n;
  const int n = b / (tk_n * tq_n * tp_n);
  const int p0 = tp * CAP_TP, q0 = tq * CAP_TQ, k0 = tk * (8 * NI);
  const int SCJ = S * C, JP = 2 * J2;
  const int PH = (CAP_TP - 1) * sh + R;
  const int64_t WC16 = (int64_t)W * C * 16;
  float* fs = lds;                   // [8*NI][PFR]: (r*JP + j)*16 + mj*4 + mk
  float* ps = lds + 8 * NI * PFR;    // [PH][PWF]: as in memory, (pixel column, c, mi, mk)

  // filter slice: global order [mk][mj] -> LDS order [mj][mk]; zeros beyond S*C and beyond K
  for (int idx = tid; idx < 8 * NI * R * JP * 16; idx += CAP_NT) {
    const int e = idx & 15, t = idx >> 4;
    const int j = t % JP, t2 = t / JP;
    const int r = t2 % R, k = t2 / R;
    float v = 0.f;
    if (k0 + k < K && j < SCJ) v = filt[((((int64_t)(k0 + k) * R + r) * SCJ + j) << 4) + e];
    fs[k * PFR + ((r * JP + j) << 4) + ((e & 3) << 2) + (e >> 2)] = v;
  }
  // input patch, 16 bytes at a time; cells outside the image read as 0
  const int pw4 = PWF >> 2;
  for (int idx = tid; idx < PH * pw4; idx += CAP_NT) {
    const int ph = idx / pw4, x = (idx - ph * pw4) << 2;
    const int hy = p0 * sh + ph;
    const int64_t gx = (int64_t)q0 * sw * C * 16 + x;
    f4 v = {0.f, 0.f, 0.f, 0.f};
    if (hy < H && gx < WC16) v = *(const f4u*)(in + ((int64_t)n * H + hy) * WC16 + gx);
    *(f4*)(ps + ph * PWF + x) = v;
  }
  __syncthreads();

  f16 acc[NI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[ni][r] = 0.f;

  // A: row (dq, mi) of the block; B: column (dk, mj); the lane half h takes the odd (s,c) pair
  const int d4 = l32 >> 2, m4 = l32 & 3;
  const float* arow = ps + (wave * sh) * PWF + d4 * sw * C * 16 + h * 16 + m4 * 4;
  const float* brow = fs + d4 * PFR + h * 16 + m4 * 4;
  for (int r = 0; r < R; ++r) {
    const float* a = arow + r * PWF;
    const float* bb = brow + r * JP * 16;
#pragma unroll 2
    for (int jj = 0; jj < J2; ++jj) {
      const f4 af = *(const f4*)(a + jj * 32);
      f4 bf[NI];
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) bf[ni] = *(const f4*)(bb + ni * 8 * PFR + jj * 32);
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
          acc[ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[t], bf[ni][t], acc[ni], 0, 0, 0);
    }
  }

  // output view (n,p,q,k,mi,mj,0,0,0,0) -> out[n,p,q,k,mi,mj]
  const int p = p0 + wave;
  if (p >= P) return;
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    const int k = k0 + ni * 8 + d4;
    if (k >= K) continue;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int q = q0 + 2 * g + h;  // registers 4g..4g+3 hold mi = 0..3 of this pixel
      if (q >= Q) continue;
      float* o = out + (((((int64_t)n * P + p) * Q + q) * K + k) << 4) + m4;
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) o[mi * 4] = acc[ni][4 * g + mi];
    }
  }
}

struct CapGeom {
  int64_t J2, PWF, PFR, lds_bytes;
};

CapGeom geom(int NI, int64_t C, int64_t R, int64_t S, int64_t sh, int64_t sw) {
  CapGeom g;
  g.J2 = cdiv(S * C, 2);
  const int64_t JP = 2 * g.J2;
  g.PWF = ((CAP_TQ - 1) * sw * C + JP) * 16 + 4;
  // filter row pitch = 16 (mod 64) floats: the 8 k-rows of a block start in different banks
  const int64_t base = R * JP * 16;
  g.PFR = base + ((16 - base % 64) + 64) % 64;
  g.lds_bytes = (8 * NI * g.PFR + ((CAP_TP - 1) * sh + R) * g.PWF) * 4;
  return g;
}

template <int NI>
mdh_status launch_t(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                    int64_t sh, int64_t sw, const float* in, const float* filt, float* out,
                    hipStream_t st) {
  const int64_t P = (H - R) / sh + 1, Q = (W - S) / sw + 1;
  const CapGeom g = geom(NI, C, R, S, sh, sw);
  if (g.lds_bytes > 160 * 1024) return MDH_ERR_TILE_RESOURCES;
  auto kern = capsule_kernel<NI>;
  static int64_t attr_bytes = 0;
  if (g.lds_bytes > attr_bytes) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)g.lds_bytes) != hipSuccess)
      return MDH_ERR_LAUNCH;
    attr_bytes = g.lds_bytes;
  }
  const int64_t tp_n = cdiv(P, CAP_TP), tq_n = cdiv(Q, CAP_TQ), tk_n = cdiv(K, 8 * NI);
  const int64_t nblocks = N * tp_n * tq_n * tk_n;
  if (nblocks > 0x7fffffff) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(CAP_NT), (size_t)g.lds_bytes, st, in, filt, out,
                     (int)H, (int)W, (int)C, (int)K, (int)R, (int)S, (int)sh, (int)sw, (int)P, (int)Q,
                     (int)tp_n, (int)tq_n, (int)tk_n, (int)g.J2, (int)g.PWF, (int)g.PFR);
  return launch_status();
}

}  // namespace

int64_t capsule_lds_bytes(int NI, int64_t C, int64_t R, int64_t S, int64_t sh, int64_t sw) {
  return geom(NI, C, R, S, sh, sw).lds_bytes;
}

mdh_status launch_capsule(const CapsulePlan& pl, int64_t N, int64_t H, int64_t W, int64_t C, int64_t K,
                          int64_t R, int64_t S, int64_t sh, int64_t sw, const float* in,
                          const float* filt, float* out, hipStream_t st) {
  switch (pl.NI) {
    case 1: return launch_t<1>(N, H, W, C, K, R, S, sh, sw, in, filt, out, st);
    case 2: return launch_t<2>(N, H, W, C, K, R, S, sh, sw, in, filt, out, st);
    case 4: return launch_t<4>(N, H, W, C, K, R, S, sh, sw, in, filt, out, st);
  }
  return MDH_ERR_UNSUPPORTED;
}

}  // namespace mdh
