// MatMul with very few rows (M <= 16 per block row): the small-M shapes of the paper's
// deep-learning study, e.g. 16 x 1000 x 2048 and 16 x 4096 x 25088 (paper: Appendix "Data
// Characteristics used in Deep Neural Networks"; Section "Experimental Results" on why these shapes
// need the reduction dimension parallelised).
//
// With M = 16 every element of B is used 16 times: 8 FLOP per byte, far below the ridge of the
// chip, so B streaming once from HBM is the bound and nothing is gained by staging it in LDS.
// De-composition, dims (b, i, j, k), MFMA block = 16 x 16 x 4 (v_mfma_f32_16x16x4_f32):
//   workgroup layer : batch x ceil(M/16) x ceil(N/(64*WAVES_N)) x S parts of k
//   wavefront layer : WAVES_N strips of 64 columns x WAVES_K interleaved 16-row parts of k
//   register layer  : both operands go from HBM straight to registers (memory region parameter =
//                     register memory for A and B); per step of 16 k a lane loads 4 rows x 4
//                     consecutive columns of B (16-byte loads, 256 contiguous bytes per 16 lanes)
//                     and 4 consecutive k of its row of A
// A lane's 4 columns feed 4 different MFMAs (one per column residue mod 4), so the block's 16
// output columns are the strided set {4*l + c}; the output view un-permutes for free because a
// lane then holds 4 consecutive columns of 4 rows.  The k parts are permuted the same way the
// large-tile kernel does it (lane group g owns k in {4g..4g+3} of a step): + combines them.
// Re-composition: registers (MFMA accumulators) -> LDS across the WAVES_K wavefronts of a
// workgroup -> workspace + second kernel across the S workgroup parts.
//
// Transposed view of B (B stored [N][K], the layout of a weight matrix applied as x * W^T): k is
// contiguous for both operands.  A block's 16 columns are then 16 consecutive columns, a lane
// loads 4 consecutive k of its column (16 bytes) for four steps of 16 k at once, so that a row of B
// is read in runs of 256 bytes, and the output view writes 64-byte runs.
//
// Strips of one block column (16 columns, all of k inside the workgroup, no workspace) exist in two forms:
// operands loaded straight into the MFMA layout (either view of B), and, for the transposed view, operands
// read as whole 512-byte runs of k and passed through a wavefront-private LDS area (memory region parameter =
// LDS for A and B), which lifts large transposed B from 3.8 to 5.6 TB/s.
#include "mdh_internal.h"

namespace mdh {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));  // dword-aligned 16-byte access

constexpr int SK_PF = 2;  // 16-row steps requested together by a wavefront

// One counter per output strip (batch entry, tile, wavefront along j): how many of the S workgroup
// parts of k have stored their partial strip.  Zero when the library is loaded; the S-th arrival wraps
// it back to zero (atomicInc with bound S-1), so every call leaves it as it found it.
static __device__ unsigned g_strip_arrivals[kArrivalCounters];

template <int WAVES_N, int WAVES_K, bool TB>
__global__ __launch_bounds__((WAVES_N * WAVES_K * 64)) void matmul_skinny_kernel(
    const float* __restrict__ A, const float* __restrict__ B, float* __restrict__ C,
    float* __restrict__ ws, int M, int N, int K, int tiles_m, int tiles_n, int S, int kchunk,
    int nbatch, int fused) {
  __shared__ f4 part[WAVES_K > 1 ? (WAVES_K - 1) * WAVES_N * 4 * 64 : 1];
  __shared__ unsigned last_flag;  // "this workgroup stored the last part of its strip", for all its wavefronts
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wn = wave % WAVES_N, wk = wave / WAVES_N;
  const int g = lane >> 4, l16 = lane & 15;
  const int batch = blockIdx.y;
  const int tiles = tiles_m * tiles_n;
  const int s = blockIdx.x / tiles, t = blockIdx.x % tiles;
  const int m0 = (t % tiles_m) * 16;
  const int n0 = ((t / tiles_m) * WAVES_N + wn) * 64;  // first column of this wavefront's strip
  const int kbeg = s * kchunk;
  const int kend = min(K, kbeg + kchunk);
  const int64_t mn = (int64_t)M * N;
  const float* Ab = A + (int64_t)batch * M * K;
  const float* Bb = B + (int64_t)batch * K * N;
  float* out = S > 1 ? ws + ((int64_t)s * nbatch + batch) * mn : C + (int64_t)batch * mn;

  const int arow = m0 + l16;            // the row of A this lane supplies
  const bool arow_ok = arow < M;
  const float* ap = Ab + (int64_t)(arow_ok ? arow : 0) * K + 4 * g;
  const int col = n0 + 4 * l16;         // the lane's 4 consecutive columns
  const float* bp = Bb + (int64_t)(4 * g) * N + col;
  const bool cols_full = n0 + 64 <= N;  // wavefront-uniform

  f4 acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) acc[c] = (f4){0.f, 0.f, 0.f, 0.f};

  if (TB) {
    // B[b, j, k]: block c of the strip = columns n0 + 16c + l16; lane group g owns k = 4g..4g+3 of
    // every 16
    const float* bt = Bb + (int64_t)(n0 + l16) * K + 4 * g;
    auto mma_t = [&](const f4& a, const f4 (&b)[4]) {
#pragma unroll
      for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int c = 0; c < 4; ++c)
          acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[tt], b[c][tt], acc[c], 0, 0, 0);
    };
    int k = kbeg + wk * 64;
    if (cols_full) {
      for (; k + 64 <= kend; k += 64 * WAVES_K) {
        f4 a[4], b[4][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          a[j] = arow_ok ? *(const f4u*)(ap + k + 16 * j) : (f4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int c = 0; c < 4; ++c)
            b[j][c] = __builtin_nontemporal_load((const f4u*)(bt + (int64_t)(16 * c) * K + k + 16 * j));
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) mma_t(a[j], b[j]);
      }
    }
    // the wavefront's remaining chunks (ragged columns, the ragged end of k): every element predicated
    for (; k < kend; k += 64 * WAVES_K)
      for (int kk = k; kk < kend && kk < k + 64; kk += 16) {
        f4 a, b[4];
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const bool kin = kk + 4 * g + tt < kend;
          a[tt] = (arow_ok && kin) ? ap[kk + tt] : 0.f;
#pragma unroll
          for (int c = 0; c < 4; ++c)
            b[c][tt] = (kin && n0 + 16 * c + l16 < N) ? bt[(int64_t)(16 * c) * K + kk + tt] : 0.f;
        }
        mma_t(a, b);
      }
  } else {

  auto mma = [&](const f4& a, const f4 (&b)[4]) {
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
      for (int c = 0; c < 4; ++c)
        acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[tt], b[tt][c], acc[c], 0, 0, 0);
  };

  int k = kbeg + wk * 16;
  constexpr int KSTEP = 16 * WAVES_K;
  if (cols_full) {
    // interior: SK_PF steps of 16 rows requested before the first is consumed
    for (; k + (SK_PF - 1) * KSTEP + 16 <= kend; k += SK_PF * KSTEP) {
      f4 a[SK_PF], b[SK_PF][4];
#pragma unroll
      for (int u = 0; u < SK_PF; ++u) {
        const int ku = k + u * KSTEP;
        a[u] = arow_ok ? *(const f4u*)(ap + ku) : (f4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int tt = 0; tt < 4; ++tt)
          b[u][tt] = __builtin_nontemporal_load((const f4u*)(bp + (int64_t)(ku + tt) * N));
      }
#pragma unroll
      for (int u = 0; u < SK_PF; ++u) mma(a[u], b[u]);
    }
    // whole single steps (a part of k of one step per wavefront, or an odd number of them)
    for (; k + 16 <= kend; k += KSTEP) {
      f4 a1, b1[4];
      a1 = arow_ok ? *(const f4u*)(ap + k) : (f4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) b1[tt] = __builtin_nontemporal_load((const f4u*)(bp + (int64_t)(k + tt) * N));
      mma(a1, b1);
    }
  }
  // remaining steps, ragged columns and the ragged end of k: every element predicated
  for (; k < kend; k += KSTEP) {
    f4 a, b[4];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
      const int kk = k + 4 * g + tt;
      a[tt] = (arow_ok && kk < kend) ? ap[k + tt] : 0.f;
#pragma unroll
      for (int c = 0; c < 4; ++c)
        b[tt][c] = (kk < kend && col + c < N) ? bp[(int64_t)(k + tt) * N + c] : 0.f;
    }
    mma(a, b);
  }
  }  // plain view of B

  // wavefront -> workgroup: the wavefronts that split k add their blocks in LDS, in a fixed order
  // With one strip per workgroup the combination over workgroups (below) is done by all wavefronts of the
  // last workgroup to arrive; they stay for it.
  constexpr bool WG_FOLD = WAVES_N == 1 && WAVES_K >= 4;
  const bool stay = WG_FOLD && S > 1 && fused;  // workgroup-uniform
  if (WAVES_K > 1) {
    if (wk > 0) {
#pragma unroll
      for (int c = 0; c < 4; ++c) part[(((wk - 1) * WAVES_N + wn) * 4 + c) * 64 + lane] = acc[c];
    }
    __syncthreads();
    if (wk > 0 && !stay) return;
    if (wk == 0) {
#pragma unroll
      for (int w = 1; w < WAVES_K; ++w)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] += part[(((w - 1) * WAVES_N + wn) * 4 + c) * 64 + lane];
    }
  }

  // output view: register r of block c is C[m0 + 4g + r][col + c]; with the transposed view of B,
  // C[m0 + 4g + r][n0 + 16c + l16]
  auto store_strip = [&](float* dst) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = m0 + 4 * g + r;
      if (row >= M) continue;
      float* p = dst + (int64_t)row * N + col;
      if (TB) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (n0 + 16 * c + l16 < N) dst[(int64_t)row * N + n0 + 16 * c + l16] = acc[c][r];
      } else if (cols_full) {
        *(f4u*)p = (f4){acc[0][r], acc[1][r], acc[2][r], acc[3][r]};
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if (col + c < N) p[c] = acc[c][r];
      }
    }
  };
  if (S <= 1 || !fused) {
    store_strip(out);
    return;
  }

  // workgroup layer -> grid in the same launch: the wavefront that stores the S-th partial strip adds
  // all S of them, in ascending part order (the order of the second kernel: same bits), into C.
  // (device-coherent single-word stores and loads instead of fences: see mdh_internal.h)
  unsigned last = 0;
  if (wk == 0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = m0 + 4 * g + r;
      if (row >= M) continue;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int cc = TB ? n0 + 16 * c + l16 : col + c;
        if (cc < N) coherent_store(out + (int64_t)row * N + cc, acc[c][r]);
      }
    }
    wait_stores_done();  // the partial strip has reached the coherent level before it is counted
    if (lane == 0) last = arrive_last(&g_strip_arrivals[((unsigned)batch * tiles + t) * WAVES_N + wn], (unsigned)S);
    last = __builtin_amdgcn_readfirstlane(last);
  }
  const int64_t part_stride = (int64_t)nbatch * mn;
  const float* w0 = ws + (int64_t)batch * mn;
  if (WG_FOLD) {
    // All wavefronts of the last workgroup fold: wavefront w takes ROWS rows of the strip, a lane one
    // column of them (consecutive lanes, consecutive addresses), and requests 16 parts of its elements
    // together (each load is a round trip to the coherent level): a strip of S = 16 parts is one round
    // instead of four.
    if (wk == 0 && lane == 0) last_flag = last;
    __syncthreads();
    if (!last_flag) return;  // workgroup-uniform
    constexpr int ROWS = 16 / WAVES_K;  // 4 or 2
    constexpr int PR = 16;
    const int rbase = m0 + wk * ROWS;
    const int cc = n0 + lane;
    float sum[ROWS];
#pragma unroll
    for (int e = 0; e < ROWS; ++e) sum[e] = 0.f;
    for (int sp0 = 0; sp0 < S; sp0 += PR) {
      float v[PR][ROWS];
#pragma unroll
      for (int u = 0; u < PR; ++u) {
        const float* src = w0 + (int64_t)min(sp0 + u, S - 1) * part_stride;
#pragma unroll
        for (int e = 0; e < ROWS; ++e) {
          const int row = min(rbase + e, M - 1);
          v[u][e] = cc < N ? coherent_load(src + (int64_t)row * N + cc) : 0.f;
        }
      }
#pragma unroll
      for (int u = 0; u < PR; ++u) {
        if (sp0 + u >= S) break;
#pragma unroll
        for (int e = 0; e < ROWS; ++e) sum[e] = (sp0 + u == 0) ? v[u][e] : sum[e] + v[u][e];
      }
    }
    float* dst = C + (int64_t)batch * mn;
#pragma unroll
    for (int e = 0; e < ROWS; ++e)
      if (rbase + e < M && cc < N) dst[(int64_t)(rbase + e) * N + cc] = sum[e];
    return;
  }
  if (!last) return;
#pragma unroll
  for (int c = 0; c < 4; ++c) acc[c] = (f4){0.f, 0.f, 0.f, 0.f};
  // four parts are requested together (each load is a round trip to the coherent level), then added in
  // ascending part order; part 0 overrides (first write, no neutral element)
  for (int sp0 = 0; sp0 < S; sp0 += 4) {
    f4 v[4][4];  // [part][row r] -> the lane's 4 columns
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float* src = w0 + (int64_t)min(sp0 + u, S - 1) * part_stride;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = min(m0 + 4 * g + r, M - 1);
        v[u][r] = (f4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int cc = TB ? n0 + 16 * c + l16 : col + c;
          if (cc < N) v[u][r][c] = coherent_load(src + (int64_t)row * N + cc);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (sp0 + u >= S) break;
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c][r] = (sp0 + u == 0) ? v[u][r][c] : acc[c][r] + v[u][r][c];
    }
  }
  store_strip(C + (int64_t)batch * mn);
}

// Narrow strips: a workgroup owns 16 columns (ONE block column) and all of k, split over its WAVES_K
// wavefronts in interleaved parts of 128; nothing is combined between workgroups.  For a B of a few
// MB (16 x 1000 x 2048: 8 MB) a 64-column strip leaves the choice between 16 workgroups (16 compute
// units pulling 512 KB each) and a split of k over workgroups whose combination costs three more
// round trips to the coherent level; 16-column strips give N/16 workgroups, each requesting its
// whole 64 B x K slice of B in one round (a lane loads single words: 4 rows x 64 contiguous bytes per
// instruction; with the transposed view 16 bytes of its column's row).  Consecutive strips share cache
// lines where a row of B is not a multiple of 64 bytes, so consecutive strips go to the same XCD.
// Re-composition: MFMA accumulator -> LDS across the WAVES_K wavefronts, added in ascending order.
template <int WAVES_K, bool TB>
__global__ __launch_bounds__((WAVES_K * 64)) void matmul_skinny16_kernel(
    const float* __restrict__ A, const float* __restrict__ B, float* __restrict__ C, int M, int N, int K,
    int strips, int strips_per_xcd) {
  __shared__ f4 part[(WAVES_K - 1) * 64];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int g = lane >> 4, l16 = lane & 15;
  const int batch = blockIdx.y;
  const int strip = (blockIdx.x & 7) * strips_per_xcd + (blockIdx.x >> 3);
  if (strip >= strips) return;  // workgroup-uniform
  const int n0 = strip * 16;
  const int64_t mn = (int64_t)M * N;
  const float* Ab = A + (int64_t)batch * M * K;
  const float* Bb = B + (int64_t)batch * K * N;
  const bool arow_ok = l16 < M;
  const float* ap = Ab + (int64_t)(arow_ok ? l16 : 0) * K + 4 * g;  // the lane's row of A, its 4 k of every 16
  const int col = n0 + l16;
  const bool col_ok = col < N;
  // lane group g owns k = 4g..4g+3 of every 16: B[k + 4g + tt][col], or with the transposed view 16
  // contiguous bytes of row col
  const float* bp = TB ? Bb + (int64_t)(col_ok ? col : 0) * K + 4 * g : Bb + (int64_t)(4 * g) * N + (col_ok ? col : 0);

  f4 acc = (f4){0.f, 0.f, 0.f, 0.f};
  constexpr int CH = 128;  // k per wavefront and round: 8 steps of 16, all requested before the first MFMA
  for (int k = wave * CH; k < K; k += CH * WAVES_K) {
    f4 a[8], b[8];
    if (k + CH <= K) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        a[j] = *(const f4u*)(ap + k + 16 * j);
        if (TB) {
          b[j] = __builtin_nontemporal_load((const f4u*)(bp + k + 16 * j));
        } else {
#pragma unroll
          for (int tt = 0; tt < 4; ++tt) b[j][tt] = __builtin_nontemporal_load(bp + (int64_t)(k + 16 * j + tt) * N);
        }
      }
    } else {  // the ragged end of k: every element predicated
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const int kk = k + 16 * j + tt;  // + 4g is in ap / bp
          const bool kin = kk + 4 * g < K;
          a[j][tt] = kin ? ap[kk] : 0.f;
          b[j][tt] = kin ? (TB ? bp[kk] : bp[(int64_t)kk * N]) : 0.f;
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        // rows of A beyond M and columns beyond N hold values of row 0 / column 0: they only reach
        // outputs that are not stored
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j][tt], b[j][tt], acc, 0, 0, 0);
      }
  }

  if (WAVES_K > 1) {
    if (wave > 0) part[(wave - 1) * 64 + lane] = acc;
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int w = 1; w < WAVES_K; ++w) acc += part[(w - 1) * 64 + lane];
  }
  // register r of the block is C[4g + r][col]
  if (col_ok) {
    float* out = C + (int64_t)batch * mn + col;
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (4 * g + r < M) out[(int64_t)(4 * g + r) * N] = acc[r];
  }
}

// Narrow strips with B transposed, operands staged through LDS (memory-region parameter = LDS).  Read
// straight into the MFMA layout, an operand load touches 16 rows x 64 bytes (16 cache lines for 1 KB): the
// address path of the compute unit, not HBM, bounds the kernel (3.8 TB/s).  Here a wavefront reads whole
// 512-byte runs of a row -- a load instruction covers two rows, 8 cache lines for 1 KB -- writes them to its
// own part of LDS as they lie in memory ([16 rows][128 k], pitch 132 floats), and reads the MFMA operands
// from there (a lane's four consecutive k of its row: one 16-byte read, free of bank conflicts at this
// pitch).  Both operands take this way: A is as long as the workgroup's slice of B.  The LDS parts are
// private to a wavefront: no barrier in the walk.  The loads of a wavefront's next round are requested
// before the current one is computed.
template <int WAVES_K>
__global__ __launch_bounds__((WAVES_K * 64)) void matmul_skinny16_lds_kernel(
    const float* __restrict__ A, const float* __restrict__ B, float* __restrict__ C, int M, int N, int K,
    int strips, int strips_per_xcd) {
  constexpr int CH = 128, PITCH = CH + 4;
  extern __shared__ __attribute__((aligned(16))) float lds[];  // [wavefront][A | B][16 * PITCH], then the partial blocks
  f4* part = (f4*)(lds + WAVES_K * 2 * 16 * PITCH);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int g = lane >> 4, l16 = lane & 15;
  const int batch = blockIdx.y;
  const int strip = (blockIdx.x & 7) * strips_per_xcd + (blockIdx.x >> 3);
  if (strip >= strips) return;  // workgroup-uniform
  const int n0 = strip * 16;
  const int64_t mn = (int64_t)M * N;
  const float* Ab = A + (int64_t)batch * M * K;
  const float* Bb = B + (int64_t)batch * K * N;
  // loads: lane -> (row parity, 16-byte segment of a 512-byte run); instruction i covers rows 2i, 2i+1.
  // Rows of A beyond M and columns beyond N are clamped: they only reach outputs that are not stored.
  const int seg = lane & 31, rpar = lane >> 5;
  float* sa = lds + wave * 2 * 16 * PITCH;
  float* sb = sa + 16 * PITCH;
  // row bases of this lane's pieces (the same in every round)
  const float* pa[8];
  const float* pb[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = 2 * i + rpar;
    pa[i] = Ab + (int64_t)min(row, M - 1) * K + seg * 4;
    pb[i] = Bb + (int64_t)min(n0 + row, N - 1) * K + seg * 4;
  }
  auto compute = [&](f4& acc) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const f4 a = *(const f4*)(sa + l16 * PITCH + 16 * j + 4 * g);
      const f4 b = *(const f4*)(sb + l16 * PITCH + 16 * j + 4 * g);
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[tt], b[tt], acc, 0, 0, 0);
    }
  };
  f4 acc = (f4){0.f, 0.f, 0.f, 0.f};
  // whole rounds of 128 k, taken by the wavefronts in turn: loads without conditions (the request after a
  // wavefront's last round repeats that round and is not used)
  const int nwhole = K / CH;
  if (wave < nwhole) {  // wavefront-uniform
    f4 va[8], vb[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      va[i] = *(const f4u*)(pa[i] + wave * CH);
      vb[i] = __builtin_nontemporal_load((const f4u*)(pb[i] + wave * CH));
    }
    for (int r = wave; r < nwhole; r += WAVES_K) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        *(f4*)(sa + (2 * i + rpar) * PITCH + seg * 4) = va[i];
        *(f4*)(sb + (2 * i + rpar) * PITCH + seg * 4) = vb[i];
      }
      const int kn = min(r + WAVES_K, nwhole - 1) * CH;  // in flight while this round is computed
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        va[i] = *(const f4u*)(pa[i] + kn);
        vb[i] = __builtin_nontemporal_load((const f4u*)(pb[i] + kn));
      }
      __builtin_amdgcn_sched_barrier(0);  // the requests stay ahead of the MFMAs they overlap with
      compute(acc);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // the ragged end of k: the next wavefront in turn takes it, every element predicated, straight to LDS
  if (K % CH != 0 && wave == nwhole % WAVES_K) {
    const int k = nwhole * CH;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      f4 ta, tb;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool kin = k + seg * 4 + e < K;
        ta[e] = kin ? pa[i][k + e] : 0.f;
        tb[e] = kin ? pb[i][k + e] : 0.f;
      }
      *(f4*)(sa + (2 * i + rpar) * PITCH + seg * 4) = ta;
      *(f4*)(sb + (2 * i + rpar) * PITCH + seg * 4) = tb;
    }
    compute(acc);
  }
  if (WAVES_K > 1) {
    if (wave > 0) part[(wave - 1) * 64 + lane] = acc;
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int w = 1; w < WAVES_K; ++w) acc += part[(w - 1) * 64 + lane];
  }
  const int col = n0 + l16;
  if (col < N) {
    float* out = C + (int64_t)batch * mn + col;
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (4 * g + r < M) out[(int64_t)(4 * g + r) * N] = acc[r];
  }
}

template <int WAVES_N, int WAVES_K, bool TB>
mdh_status launch_t(const GemmExPlan& pl, int64_t batch, int64_t M, int64_t N, int64_t K,
                    const float* A, const float* B, float* C, void* ws, hipStream_t st) {
  const int S = pl.g.S;
  const int64_t tm = cdiv(M, 16), tn = cdiv(N, 64 * WAVES_N);
  const int64_t kstep = TB ? 64 : 16;  // k a wavefront takes per step
  const int64_t kchunk = cdiv(cdiv(K, S), kstep) * kstep;
  const int64_t nblocks = tm * tn * S;
  if (nblocks > 0x7fffffff || batch > 65535) return MDH_ERR_SIZE;
  clear_stale_error();
  const int fused = (S > 1 && pl.fused && batch * tm * tn * WAVES_N <= kArrivalCounters) ? 1 : 0;
  hipLaunchKernelGGL((matmul_skinny_kernel<WAVES_N, WAVES_K, TB>), dim3((unsigned)nblocks, (unsigned)batch),
                     dim3(WAVES_N * WAVES_K * 64), 0, st, A, B, C, (float*)ws, (int)M, (int)N, (int)K,
                     (int)tm, (int)tn, S, (int)kchunk, (int)batch, fused);
  mdh_status r = launch_status();
  if (r != MDH_OK || S <= 1 || fused) return r;
  return launch_combine_sum((const float*)ws, C, batch * M * N, S, st);
}

template <int WAVES_K, bool TB>
mdh_status launch_narrow(int64_t batch, int64_t M, int64_t N, int64_t K, const float* A, const float* B,
                         float* C, hipStream_t st) {
  if (M > 16 || batch > 65535) return MDH_ERR_SIZE;
  const int64_t strips = cdiv(N, 16), per_xcd = cdiv(strips, 8);
  if (per_xcd * 8 > 0x7fffffff) return MDH_ERR_SIZE;
  clear_stale_error();
  hipLaunchKernelGGL((matmul_skinny16_kernel<WAVES_K, TB>), dim3((unsigned)(per_xcd * 8), (unsigned)batch),
                     dim3(WAVES_K * 64), 0, st, A, B, C, (int)M, (int)N, (int)K, (int)strips, (int)per_xcd);
  return launch_status();
}

template <int WAVES_K>
mdh_status launch_narrow_lds(int64_t batch, int64_t M, int64_t N, int64_t K, const float* A, const float* B,
                             float* C, hipStream_t st) {
  if (M > 16 || batch > 65535) return MDH_ERR_SIZE;
  const int64_t strips = cdiv(N, 16), per_xcd = cdiv(strips, 8);
  if (per_xcd * 8 > 0x7fffffff) return MDH_ERR_SIZE;
  auto kern = matmul_skinny16_lds_kernel<WAVES_K>;
  const int64_t lds_bytes = ((int64_t)WAVES_K * 2 * 16 * 132 + (WAVES_K - 1) * 64 * 4) * 4;
  static int64_t lds_allowed[kMaxDevices] = {};
  if (allow_dynamic_lds((const void*)kern, lds_bytes, lds_allowed) != MDH_OK) return MDH_ERR_LAUNCH;
  clear_stale_error();
  hipLaunchKernelGGL(kern, dim3((unsigned)(per_xcd * 8), (unsigned)batch), dim3(WAVES_K * 64), (size_t)lds_bytes, st, A,
                     B, C, (int)M, (int)N, (int)K, (int)strips, (int)per_xcd);
  return launch_status();
}

}  // namespace

mdh_status launch_matmul_skinny(const GemmExPlan& pl, int64_t batch, int64_t M, int64_t N, int64_t K,
                                const float* A, const float* B, float* C, void* ws, hipStream_t st) {
  if (pl.ta || pl.tc) return MDH_ERR_UNSUPPORTED;
  if (pl.g.BN == 16) {  // narrow strips: one block column per workgroup, k inside the workgroup only
    if (pl.g.S != 1) return MDH_ERR_UNSUPPORTED;
    if (pl.lds) {
      if (!pl.tb) return MDH_ERR_UNSUPPORTED;
      if (pl.WK == 8) return launch_narrow_lds<8>(batch, M, N, K, A, B, C, st);
      if (pl.WK == 4) return launch_narrow_lds<4>(batch, M, N, K, A, B, C, st);
      return MDH_ERR_UNSUPPORTED;
    }
    if (pl.WK == 16) return pl.tb ? launch_narrow<16, true>(batch, M, N, K, A, B, C, st) : launch_narrow<16, false>(batch, M, N, K, A, B, C, st);
    if (pl.WK == 8) return pl.tb ? launch_narrow<8, true>(batch, M, N, K, A, B, C, st) : launch_narrow<8, false>(batch, M, N, K, A, B, C, st);
    return MDH_ERR_UNSUPPORTED;
  }
#define MDH_SK(wn, wk)                                                                                   \
  if (pl.g.BN == 64 * wn && pl.WK == wk)                                                                 \
    return pl.tb ? launch_t<wn, wk, true>(pl, batch, M, N, K, A, B, C, ws, st)                           \
                 : launch_t<wn, wk, false>(pl, batch, M, N, K, A, B, C, ws, st);
  MDH_SK(1, 4)
  MDH_SK(1, 8)
  MDH_SK(2, 2)
  MDH_SK(4, 1)
  MDH_SK(1, 1)
#undef MDH_SK
  return MDH_ERR_UNSUPPORTED;
}

}  // namespace mdh
