/*
 * mdh_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Plain, slow, from-the-definition CPU evaluation of the four md_hom instances
 * the GPU library computes.  Only tests, the smoke check and the bench's
 * cpu_baseline leg may call this; it shares no code with the HIP path.
 *
 * Every function is the paper's definition
 *
 *     md_hom(f,(op_1..op_D))(a) = op_1_{i_1 in I_1} ... op_D_{i_D in I_D} f(a[i_1..i_D])
 *
 * (Definition "Higher-Order Function md_hom") composed with the instance's
 * input and output views (Definitions "Input View"/"Output View"), written as
 * nested loops: the ++ dimensions are the outer loops (they index the output
 * buffer through the output view), the reduction dimensions the inner loops,
 * iterated in ascending index order.  Floating-point instances accumulate in
 * fp64 over the fp32 inputs.  OpenMP only distributes the outermost ++ loop.
 *
 * Parity status: every function below is pinned by tests/test_oracle_*.py
 * (closed forms, brute force against the generic evaluator in mdhom.py, the
 * homomorphic split property, special cases that reduce to each other).
 * Unpinned by anything the paper prints: the record-linkage weight function
 * and the Jacobi-3D coefficients of the paper's evaluation (both only in a
 * figure that is not part of the text); the explicit definitions in the
 * function comments stand in for them.
 */
#include <stdint.h>
#include <stdlib.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- Dot: md_hom(*, (+)) over (k); views (k)->x[k], (k)->y[k]; (0)->out (a scalar)
 * (Section "Examples", Subfigure 1, first routine).  outabs (nullable) receives sum_k |x*y|. */
void oracle_dot(int64_t K, const float* x, const float* y, double* out, double* outabs) {
  double acc = 0.0, aabs = 0.0;
  for (int64_t k = 0; k < K; ++k) {
    double t = (double)x[k] * (double)y[k];
    acc += t;
    aabs += fabs(t);
  }
  *out = acc;
  if (outabs) *outabs = aabs;
}

/* ---- MatVec: md_hom(*, (++,+)) over (i,k); views (i,k)->A[i,k], (i,k)->x[k]; (i,0)->y[i]
 * (the paper's introductory example and the worked low-level example). */
void oracle_matvec(int64_t M, int64_t K, const float* A, const float* x, double* y, double* yabs) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < M; ++i) {
    double acc = 0.0, aabs = 0.0;
    for (int64_t k = 0; k < K; ++k) {
      double t = (double)A[i * K + k] * (double)x[k];
      acc += t;
      aabs += fabs(t);
    }
    y[i] = acc;
    if (yabs) yabs[i] = aabs;
  }
}

/* ---- MatMul: md_hom(*, (++,++,+)), views (i,j,k)->A[i,k], B[k,j]; (i,j,0)->C[i,j] ----
 * (Section "Examples", Subfigure 1).  Cabs (nullable) receives sum_k |A[i,k]*B[k,j]|,
 * the denominator of the componentwise error measure the tests use. */
void oracle_matmul(int64_t M, int64_t N, int64_t K, const float* A, const float* B, double* C,
                   double* Cabs) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < M; ++i) {
    for (int64_t j = 0; j < N; ++j) {
      double acc = 0.0, aabs = 0.0;
      for (int64_t k = 0; k < K; ++k) {
        double t = (double)A[i * K + k] * (double)B[k * N + j];
        acc += t;
        aabs += fabs(t);
      }
      C[i * N + j] = acc;
      if (Cabs) Cabs[i * N + j] = aabs;
    }
  }
}

/* Same definition evaluated at nS chosen output positions (is[s], js[s]). */
void oracle_matmul_at(int64_t M, int64_t N, int64_t K, const float* A, const float* B,
                      int64_t nS, const int64_t* is, const int64_t* js, double* out,
                      double* outabs) {
  (void)M;
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < nS; ++s) {
    int64_t i = is[s], j = js[s];
    double acc = 0.0, aabs = 0.0;
    for (int64_t k = 0; k < K; ++k) {
      double t = (double)A[i * K + k] * (double)B[k * N + j];
      acc += t;
      aabs += fabs(t);
    }
    out[s] = acc;
    if (outabs) outabs[s] = aabs;
  }
}

/* ---- Jacobi-3D: md_hom(J_3D, (++,++,++)); the input view reads the one input
 * buffer seven times with offset index functions (3-D form of Example "Input
 * View -- Jacobi1D"); output view (i,j,k)->(i,j,k) on the compact nx*ny*nz grid.
 *   J_3D(x_c, x_im, x_ip, x_jm, x_jp, x_km, x_kp) = c0*x_c + c1*(x_im+x_ip+x_jm+x_jp+x_km+x_kp)
 * c0, c1 are the fp32 constants the GPU receives, promoted to fp64. */
void oracle_jacobi3d(int64_t nx, int64_t ny, int64_t nz, const float* in, double* out, float c0,
                     float c1) {
  const int64_t sy = nz + 2, sx = (ny + 2) * (nz + 2);
  const double d0 = (double)c0, d1 = (double)c1;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < nx; ++i)
    for (int64_t j = 0; j < ny; ++j)
      for (int64_t k = 0; k < nz; ++k) {
        const float* c = in + (i + 1) * sx + (j + 1) * sy + (k + 1);
        double nb = (double)c[-sx] + (double)c[sx] + (double)c[-sy] + (double)c[sy] +
                    (double)c[-1] + (double)c[1];
        out[(i * ny + j) * nz + k] = d0 * (double)c[0] + d1 * nb;
      }
}

/* ---- MCC: md_hom(*, (++,++,++,++,+,+,+)) over (n,p,q,k,c,r,s); input view
 * (n,p,q,k,c,r,s)->in[n,p*sh+r,q*sw+s,c], filt[k,r,s,c]; output view ->out[n,p,q,k]
 * (Section "Examples", Subfigure 2; NHWC/KRSC/NPQK as in the appendix's data
 * characteristics).  No filter flip, no implicit padding. */
static inline void mcc_point(int64_t H, int64_t W, int64_t C, int64_t R, int64_t S, int64_t sh,
                             int64_t sw, const float* in, const float* filt, int64_t n, int64_t p,
                             int64_t q, int64_t k, double* acc_out, double* abs_out) {
  double acc = 0.0, aabs = 0.0;
  for (int64_t c = 0; c < C; ++c)
    for (int64_t r = 0; r < R; ++r)
      for (int64_t s = 0; s < S; ++s) {
        double t = (double)in[((n * H + (p * sh + r)) * W + (q * sw + s)) * C + c] *
                   (double)filt[((k * R + r) * S + s) * C + c];
        acc += t;
        aabs += fabs(t);
      }
  *acc_out = acc;
  *abs_out = aabs;
}

void oracle_mcc(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                int64_t sh, int64_t sw, const float* in, const float* filt, double* out,
                double* outabs) {
  const int64_t P = (H - R) / sh + 1, Q = (W - S) / sw + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t p = 0; p < P; ++p)
      for (int64_t q = 0; q < Q; ++q)
        for (int64_t k = 0; k < K; ++k) {
          double acc, aabs;
          mcc_point(H, W, C, R, S, sh, sw, in, filt, n, p, q, k, &acc, &aabs);
          int64_t o = ((n * P + p) * Q + q) * K + k;
          out[o] = acc;
          if (outabs) outabs[o] = aabs;
        }
}

/* Same definition at nS chosen output positions; idx holds (n,p,q,k) quadruples. */
void oracle_mcc_at(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                   int64_t sh, int64_t sw, const float* in, const float* filt, int64_t nS,
                   const int64_t* idx, double* out, double* outabs) {
  (void)N;
  (void)K;
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < nS; ++t) {
    double acc, aabs;
    mcc_point(H, W, C, R, S, sh, sw, in, filt, idx[4 * t], idx[4 * t + 1], idx[4 * t + 2],
              idx[4 * t + 3], &acc, &aabs);
    out[t] = acc;
    if (outabs) outabs[t] = aabs;
  }
}

/* ---- Custom reduce: md_hom(wght, (++, max_idx)) over (a,b); the scalar function
 * receives the MDA index b (Appendix "Design Decisions: md_hom"):
 *   wght(a,b) = ( sum_f (A[a,f]==B[b,f] ? w_agree[f] : w_disagree[f]), b )
 *   (s1,b1) max_idx (s2,b2) = s1>s2 ? (s1,b1) : s2>s1 ? (s2,b2) : (s1, min(b1,b2))
 * The reduction starts from the b=0 element (no neutral element is assumed). */
static inline void maxidx(int32_t* s1, int32_t* b1, int32_t s2, int32_t b2) {
  if (s2 > *s1) {
    *s1 = s2;
    *b1 = b2;
  } else if (s2 == *s1 && b2 < *b1) {
    *b1 = b2;
  }
}

static inline int32_t wght(int32_t nF, const int32_t* ra, const int32_t* rb, const int32_t* wp,
                           const int32_t* wm) {
  int32_t s = 0;
  for (int32_t f = 0; f < nF; ++f) s += (ra[f] == rb[f]) ? wp[f] : wm[f];
  return s;
}

void oracle_custom_reduce(int64_t nA, int64_t nB, int32_t nF, const int32_t* A, const int32_t* B,
                          const int32_t* wp, const int32_t* wm, int32_t* score, int32_t* index) {
#pragma omp parallel for schedule(static)
  for (int64_t a = 0; a < nA; ++a) {
    int32_t bs = wght(nF, A + a * nF, B, wp, wm), bi = 0;
    for (int64_t b = 1; b < nB; ++b)
      maxidx(&bs, &bi, wght(nF, A + a * nF, B + b * nF, wp, wm), (int32_t)b);
    score[a] = bs;
    index[a] = bi;
  }
}

/* Same definition for nS chosen records as[s] of A. */
void oracle_custom_reduce_rows(int64_t nA, int64_t nB, int32_t nF, const int32_t* A,
                               const int32_t* B, const int32_t* wp, const int32_t* wm, int64_t nS,
                               const int64_t* as, int32_t* score, int32_t* index) {
  (void)nA;
#pragma omp parallel for schedule(static)
  for (int64_t s = 0; s < nS; ++s) {
    const int32_t* ra = A + as[s] * nF;
    int32_t bs = wght(nF, ra, B, wp, wm), bi = 0;
    for (int64_t b = 1; b < nB; ++b)
      maxidx(&bs, &bi, wght(nF, ra, B + b * nF, wp, wm), (int32_t)b);
    score[s] = bs;
    index[s] = bi;
  }
}

/* The combine operator alone, exported so that tests can apply the homomorphic
 * property (split B, reduce both halves, combine) with the oracle's own operator. */
void oracle_maxidx_combine(int64_t n, int32_t* s1, int32_t* b1, const int32_t* s2,
                           const int32_t* b2) {
  for (int64_t i = 0; i < n; ++i) maxidx(&s1[i], &b1[i], s2[i], b2[i]);
}

/* Threads the OpenMP loops above run on (reported next to oracle timings). */
int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---- scan(+), row-wise: md_hom(id, (++, prefix-sum(+))) over (i,j); out[i,j] = x[i,0] + ... + x[i,j]
 * (Section "Examples", Subfigure 8; Appendix, Example "Prefix-Sum": folding the singletons of j in
 * ascending order with that operator gives the inclusive scan).  outabs (nullable) receives the same
 * scan of |x|, the denominator of the scaled error the tests use. */
void oracle_scan_rows(int64_t R, int64_t n, const float* x, double* out, double* outabs) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < R; ++i) {
    double acc = 0.0, aabs = 0.0;
    for (int64_t j = 0; j < n; ++j) {
      acc += (double)x[i * n + j];
      aabs += fabs((double)x[i * n + j]);
      out[i * n + j] = acc;
      if (outabs) outabs[i * n + j] = aabs;
    }
  }
}

/* ---- Histo: md_hom(f_Histo, (++, +)) over (b, e), f_Histo(e, b) = 1 if the element equals the
 * bin value, else 0 (Section "Examples", Subfigures 4-6; Appendix on GenHisto: work E*B, every
 * element is compared with every bin).  Input views (b,e)->elems[e], (b,e)->bins[b]; output view
 * (b,0)->out[b].  Written as the definition: the ++ dimension outside, the + dimension inside. */
void oracle_histo(int64_t nB, int64_t nE, const int32_t* elems, const int32_t* bins, int64_t* out) {
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < nB; ++b) {
    int64_t acc = 0;
    for (int64_t e = 0; e < nE; ++e) acc += elems[e] == bins[b] ? 1 : 0;
    out[b] = acc;
  }
}

/* ---- MCC_Capsule: the 10-dimensional generalisation of MCC that operates on MI x MK and MK x MJ
 * matrices instead of scalars (Section "Examples", Subfigure 2; Appendix "Data Characteristics
 * used in Deep Neural Networks": three more dimensions MI, MJ, MK).  Reading of the missing figure:
 * md_hom(*, (++ n,p,q,k,mi,mj ; + c,r,s,mk)) with views
 *   (..)->in[n, p*sh+r, q*sw+s, c, mi, mk],  (..)->filt[k, r, s, c, mk, mj],  out[n,p,q,k,mi,mj]:
 * every scalar product of MCC becomes a matrix product.  One output position per call; idx =
 * (n,p,q,k,mi,mj). */
static void capsule_point(int64_t H, int64_t W, int64_t C, int64_t R, int64_t S, int64_t sh, int64_t sw,
                          int64_t MI, int64_t MJ, int64_t MK, const float* in, const float* filt,
                          int64_t n, int64_t p, int64_t q, int64_t k, int64_t mi, int64_t mj,
                          double* acc_out, double* abs_out) {
  double acc = 0.0, aabs = 0.0;
  for (int64_t c = 0; c < C; ++c)
    for (int64_t r = 0; r < R; ++r)
      for (int64_t s = 0; s < S; ++s)
        for (int64_t mk = 0; mk < MK; ++mk) {
          double a = (double)in[((((n * H + (p * sh + r)) * W + (q * sw + s)) * C + c) * MI + mi) * MK + mk];
          double b = (double)filt[((((k * R + r) * S + s) * C + c) * MK + mk) * MJ + mj];
          acc += a * b;
          aabs += fabs(a * b);
        }
  *acc_out = acc;
  *abs_out = aabs;
}

void oracle_mcc_capsule(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                        int64_t sh, int64_t sw, int64_t MI, int64_t MJ, int64_t MK, const float* in,
                        const float* filt, double* out, double* outabs) {
  const int64_t P = (H - R) / sh + 1, Q = (W - S) / sw + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t n = 0; n < N; ++n)
    for (int64_t p = 0; p < P; ++p)
      for (int64_t q = 0; q < Q; ++q)
        for (int64_t k = 0; k < K; ++k)
          for (int64_t mi = 0; mi < MI; ++mi)
            for (int64_t mj = 0; mj < MJ; ++mj) {
              double acc, aabs;
              capsule_point(H, W, C, R, S, sh, sw, MI, MJ, MK, in, filt, n, p, q, k, mi, mj, &acc, &aabs);
              int64_t o = ((((n * P + p) * Q + q) * K + k) * MI + mi) * MJ + mj;
              out[o] = acc;
              if (outabs) outabs[o] = aabs;
            }
}

void oracle_mcc_capsule_at(int64_t H, int64_t W, int64_t C, int64_t R, int64_t S, int64_t sh, int64_t sw,
                           int64_t MI, int64_t MJ, int64_t MK, const float* in, const float* filt,
                           int64_t nS, const int64_t* idx, double* out, double* outabs) {
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < nS; ++t) {
    double acc, aabs;
    capsule_point(H, W, C, R, S, sh, sw, MI, MJ, MK, in, filt, idx[6 * t], idx[6 * t + 1], idx[6 * t + 2],
                  idx[6 * t + 3], idx[6 * t + 4], idx[6 * t + 5], &acc, &aabs);
    out[t] = acc;
    outabs[t] = aabs;
  }
}
