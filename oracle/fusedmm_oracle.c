/*
 * CPU ORACLE for the fused SDDMM-SpMM operation (FusedMM).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  Only tests/, __graft_entry__.smoke() and
 * the cpu_baseline leg of bench.py may build, load or call it.  It shares no
 * code, header, constant or table with the GPU library and the GPU library
 * never falls back to it.
 *
 * What it computes (paper: Eq. 1; Section II "SDDMM" Eq. 2 and "SpMM" Eq. 3;
 * Section III-A steps 1-5; Algorithm 1 procedure UpdateU; Table III):
 *
 *   Phase 1, general SDDMM (Eq. 2): for every stored entry e = (u, v) of the
 *   m x n CSR matrix A, in CSR order,
 *        t    = VOP(x_u, y_v)          a length-d vector           (step 1)
 *        s    = ROP(t)                 a scalar                    (step 2)
 *        H[e] = SOP(s)  or  a_uv       the scalar edge message     (step 3)
 *   and H is MATERIALISED: one double per stored entry.
 *
 *   Phase 2, general SpMM (Eq. 3): for every row u, entries in CSR order,
 *        w    = MOP(H[e], y_v or t)    a length-d vector           (step 4)
 *        z_u  = AOP(z_u, w) = z_u + w                              (step 5)
 *   with z_u starting at zero (Algorithm 1, first line of UpdateU), so a row
 *   without entries yields zeros.
 *
 * The GPU kernel never writes H; this oracle always does.  That is the point:
 * the paper states that fusing changes memory traffic, not the result.
 *
 * All arithmetic is done in ORACLE_REAL (double unless the file is compiled
 * with -DORACLE_REAL=float, which exists only so that bench.py can time an
 * fp32 unfused CPU baseline).  Inputs X, Y, values are fp32, as in the paper's
 * experiments (Section V-A), and are widened element by element.
 *
 * Readings of the paper taken here:
 *   - t-distribution pattern (author notes on recognised patterns): the VOP
 *     output t = x_u - y_v is kept and reused by MOP ("MUL_T"); ROP is the dot
 *     product of t with itself; SOP is 1/(1+s).
 *   - force-directed (FR) pattern (Table III row 1: ADD, NORM, SCAL, MUL,
 *     ASUM): t = x_u - y_v (the "addition" of a negated operand), NORM is the
 *     Euclidean norm, SCAL multiplies by alpha, MOP scales t.
 *   - GCN pattern (Table III row 3): VOP = SEL2ND, ROP and SOP are no-ops and
 *     the message is the stored edge value a_uv.
 *   - the edge value a_uv is ignored by every SOP except EDGE_VALUE.
 *
 * Parity status: every function here is pinned by tests/test_oracle_pins.py
 * (dense brute force written independently in numpy, closed forms, the
 * SpMM special case, invariants).  The FR *reading* itself cannot be pinned
 * against the paper because its defining formula is only in a figure.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORACLE_REAL
#define ORACLE_REAL double
#endif
typedef ORACLE_REAL real;

#ifndef ORACLE_SUFFIX
#define ORACLE_SUFFIX f64
#endif
#define CAT_(a, b) a##_##b
#define CAT(a, b) CAT_(a, b)
#define FN(name) CAT(name, ORACLE_SUFFIX)

/* The oracle's own op codes (the Python wrapper maps names to these). */
enum { O_VOP_MUL = 0, O_VOP_SEL2ND = 1, O_VOP_SUB = 2 };
enum { O_ROP_NOOP = 0, O_ROP_RSUM = 1, O_ROP_SUMSQ = 2, O_ROP_NORM = 3 };
enum { O_SOP_EDGE_VALUE = 0, O_SOP_SIGMOID = 1, O_SOP_ONE_MINUS_SIGMOID = 2, O_SOP_INV1P = 3, O_SOP_SCAL = 4 };
enum { O_MOP_MUL_Y = 0, O_MOP_MUL_T = 1 };

/* Step 1 (Section III-A, VOP), one element. */
static inline real vop_elem(int vop, real x, real y) {
  switch (vop) {
    case O_VOP_MUL: return x * y;
    case O_VOP_SEL2ND: return y;
    default: return x - y; /* O_VOP_SUB */
  }
}

/* Steps 1+2 for one edge: s = ROP(VOP(x_u, y_v)). */
static real vop_rop(int vop, int rop, int64_t d, const float* x, const float* y) {
  real s = 0;
  if (rop == O_ROP_NOOP) return 0;
  for (int64_t k = 0; k < d; ++k) {
    real t = vop_elem(vop, (real)x[k], (real)y[k]);
    s += (rop == O_ROP_RSUM) ? t : t * t;
  }
  if (rop == O_ROP_NORM) s = (real)sqrt((double)s);
  return s;
}

/* Step 3 (SOP) on a scalar. */
static real sop_scalar(int sop, real s, real a_uv, real alpha) {
  switch (sop) {
    case O_SOP_EDGE_VALUE: return a_uv;
    case O_SOP_SIGMOID: return (real)(1.0 / (1.0 + exp(-(double)s)));
    /* 1 - sigmoid(s) = sigmoid(-s) identically; written this way because the literal difference
     * cancels (it is 0 in double from s = 37 on, where the true value is still 1e-16 and falling) */
    case O_SOP_ONE_MINUS_SIGMOID: return (real)(1.0 / (1.0 + exp((double)s)));
    case O_SOP_INV1P: return (real)1 / ((real)1 + s);
    default: return alpha * s; /* O_SOP_SCAL */
  }
}

/* Phase 1: general SDDMM (Eq. 2).  H has nnz entries.  X may be NULL only if
 * vop == SEL2ND; values may be NULL unless sop == EDGE_VALUE. */
int FN(fmm_oracle_sddmm)(int64_t m, int64_t d, const int64_t* rowptr, const int32_t* colidx,
                         const float* values, const float* X, int64_t ldx,
                         const float* Y, int64_t ldy, int vop, int rop, int sop, double alpha,
                         real* H) {
  if (sop == O_SOP_EDGE_VALUE && !values && rowptr[m] > 0) return -1;
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t u = 0; u < m; ++u) {
    const float* xu = X ? X + u * ldx : 0;
    for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
      const float* yv = Y + (int64_t)colidx[e] * ldy;
      real s = (rop == O_ROP_NOOP) ? 0 : vop_rop(vop, rop, d, xu ? xu : yv, yv);
      H[e] = sop_scalar(sop, s, values ? (real)values[e] : 0, (real)alpha);
    }
  }
  return 0;
}

/* Phase 2: general SpMM (Eq. 3) with the scalar messages of phase 1.
 * Z and S are m x d, dense, leading dimension d.  S receives the sum of the
 * absolute values of the accumulated terms (the comparison denominator). */
int FN(fmm_oracle_spmm)(int64_t m, int64_t d, const int64_t* rowptr, const int32_t* colidx,
                        const float* X, int64_t ldx, const float* Y, int64_t ldy,
                        int vop, int mop, const real* H, real* Z, real* S) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t u = 0; u < m; ++u) {
    real* z = Z + u * d;
    real* sabs = S ? S + u * d : 0;
    for (int64_t k = 0; k < d; ++k) z[k] = 0;
    if (sabs) for (int64_t k = 0; k < d; ++k) sabs[k] = 0;
    const float* xu = X ? X + u * ldx : 0;
    for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
      const float* yv = Y + (int64_t)colidx[e] * ldy;
      const real h = H[e];
      for (int64_t k = 0; k < d; ++k) {
        real operand = (mop == O_MOP_MUL_Y) ? (real)yv[k]
                                            : vop_elem(vop, xu ? (real)xu[k] : 0, (real)yv[k]);
        real w = h * operand;
        z[k] += w;
        if (sabs) sabs[k] += (real)fabs((double)w);
      }
    }
  }
  return 0;
}

/* The literal picture of the unfused pipeline with VECTOR messages: phase 1
 * writes the full nnz x d message tensor W[e,:] = MOP(SOP(ROP(VOP))), ...),
 * phase 2 only adds rows of W.  O(nnz*d) memory: tiny graphs only. */
int FN(fmm_oracle_message_tensor)(int64_t m, int64_t d, const int64_t* rowptr, const int32_t* colidx,
                                  const float* values, const float* X, int64_t ldx,
                                  const float* Y, int64_t ldy, int vop, int rop, int sop, int mop,
                                  double alpha, real* W) {
  if (sop == O_SOP_EDGE_VALUE && !values && rowptr[m] > 0) return -1;
  for (int64_t u = 0; u < m; ++u) {
    const float* xu = X ? X + u * ldx : 0;
    for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
      const float* yv = Y + (int64_t)colidx[e] * ldy;
      real s = (rop == O_ROP_NOOP) ? 0 : vop_rop(vop, rop, d, xu ? xu : yv, yv);
      real h = sop_scalar(sop, s, values ? (real)values[e] : 0, (real)alpha);
      for (int64_t k = 0; k < d; ++k) {
        real operand = (mop == O_MOP_MUL_Y) ? (real)yv[k]
                                            : vop_elem(vop, xu ? (real)xu[k] : 0, (real)yv[k]);
        W[e * d + k] = h * operand;
      }
    }
  }
  return 0;
}

int FN(fmm_oracle_aggregate_tensor)(int64_t m, int64_t d, const int64_t* rowptr, const real* W, real* Z) {
  for (int64_t u = 0; u < m; ++u) {
    for (int64_t k = 0; k < d; ++k) Z[u * d + k] = 0;
    for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e)
      for (int64_t k = 0; k < d; ++k) Z[u * d + k] += W[e * d + k];
  }
  return 0;
}

/* Algorithm 1, procedure UpdateU, taken step by step for every row: the five
 * steps run per stored entry, each writing its output before the next reads
 * it (the paper's "general" kernel).  Used to check that the two-phase
 * pipeline above and the per-row fused order give the same numbers. */
int FN(fmm_oracle_update_u_all)(int64_t m, int64_t d, const int64_t* rowptr, const int32_t* colidx,
                                const float* values, const float* X, int64_t ldx,
                                const float* Y, int64_t ldy, int vop, int rop, int sop, int mop,
                                double alpha, real* Z) {
  if (sop == O_SOP_EDGE_VALUE && !values && rowptr[m] > 0) return -1;
  real* t = (real*)malloc((size_t)(d > 0 ? d : 1) * sizeof(real));
  real* w = (real*)malloc((size_t)(d > 0 ? d : 1) * sizeof(real));
  if (!t || !w) { free(t); free(w); return -2; }
  for (int64_t u = 0; u < m; ++u) {
    real* zu = Z + u * d;
    for (int64_t k = 0; k < d; ++k) zu[k] = 0;                 /* z_u <- 0 */
    const float* xu = X ? X + u * ldx : 0;
    for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
      const float* yv = Y + (int64_t)colidx[e] * ldy;          /* y_v <- Y[v,:] */
      for (int64_t k = 0; k < d; ++k)                          /* VOP */
        t[k] = vop_elem(vop, xu ? (real)xu[k] : 0, (real)yv[k]);
      real s = 0;                                              /* ROP */
      if (rop != O_ROP_NOOP) {
        for (int64_t k = 0; k < d; ++k) s += (rop == O_ROP_RSUM) ? t[k] : t[k] * t[k];
        if (rop == O_ROP_NORM) s = (real)sqrt((double)s);
      }
      real h = sop_scalar(sop, s, values ? (real)values[e] : 0, (real)alpha); /* SOP */
      for (int64_t k = 0; k < d; ++k)                          /* MOP */
        w[k] = h * ((mop == O_MOP_MUL_Y) ? (real)yv[k] : t[k]);
      for (int64_t k = 0; k < d; ++k) zu[k] += w[k];           /* AOP */
    }
  }
  free(t); free(w);
  return 0;
}

/* ------------------------------------------------------------------------------------------
 * The general five-step path (Section III-A, Table II): every standard operation the paper
 * lists for the five steps, including the ones outside the three application patterns:
 *   VOP  ADD (x + y)                                   Table II "ADD"
 *   ROP  RMUL (product of the elements)                Table II "RMUL"
 *   SOP  NOOP (h = s, or h = t when there was no ROP)  Section III-A: a step may be skipped
 *   SOP  on a VECTOR: when ROP is a no-op, SOP is applied to every element of t and the edge
 *        message h is a length-d vector (Algorithm 1, SOP step: without a reduction SOP takes the
 *        VOP output; Fig. 3: messages can be vectors); MOP is then element-wise h (.) operand
 *   MOP  SEL2ND (w = y_v, the second operand)          Table II "SEL2ND ... VOP, MOP"
 *   AOP  AMAX / AMIN                                   Table II "AMAX" (AMIN: its mirror image)
 *   AOP  AMEAN                                         Section III-B, GCN paragraph: mean pooling
 * Reading for AMAX/AMIN: Algorithm 1 sets z_u to 0 before the loop and AOP combines z_u with
 * every message, so the result is max(0, max_v w) (resp. min(0, min_v w)); a row without
 * entries yields 0.
 * Reading for AMEAN: the messages of a row are summed as with ASUM and the sum is divided by
 * the number of stored entries of the row; a row without entries yields 0.
 * H holds one real per stored entry when h is a scalar and d reals per stored entry when it
 * is a vector: the unfused pipeline's sparse tensor.
 * S (comparison denominator) is the sum of |w| for ASUM, the largest |w| for AMAX/AMIN and
 * the mean of |w| for AMEAN.
 * ------------------------------------------------------------------------------------------ */
enum { O_VOP_ADD = 3 };
enum { O_ROP_RMUL = 4 };
enum { O_SOP_NOOP = 5 };
enum { O_MOP_SEL2ND = 2 };
enum { O_AOP_SUM = 0, O_AOP_MAX = 1, O_AOP_MIN = 2, O_AOP_MEAN = 3 };

static inline real g_vop(int vop, real x, real y) {
  switch (vop) {
    case O_VOP_MUL: return x * y;
    case O_VOP_SEL2ND: return y;
    case O_VOP_SUB: return x - y;
    default: return x + y; /* O_VOP_ADD */
  }
}

static inline real g_sop(int sop, real s, real a_uv, real alpha) {
  switch (sop) {
    case O_SOP_EDGE_VALUE: return a_uv;
    case O_SOP_SIGMOID: return (real)(1.0 / (1.0 + exp(-(double)s)));
    /* 1 - sigmoid(s) = sigmoid(-s) identically; written this way because the literal difference
     * cancels (it is 0 in double from s = 37 on, where the true value is still 1e-16 and falling) */
    case O_SOP_ONE_MINUS_SIGMOID: return (real)(1.0 / (1.0 + exp((double)s)));
    case O_SOP_INV1P: return (real)1 / ((real)1 + s);
    case O_SOP_SCAL: return alpha * s;
    default: return s; /* O_SOP_NOOP */
  }
}

/* 1 when the message h is a vector (no reduction and SOP acts on t), 0 when it is a scalar */
int FN(fmm_oracle_h_is_vector)(int rop, int sop) { return rop == O_ROP_NOOP && sop != O_SOP_EDGE_VALUE; }

/* Phase 1 of the general path: H[e] (scalar h) or H[e*d .. e*d+d) (vector h). */
int FN(fmm_oracle_sddmm_general)(int64_t m, int64_t d, const int64_t* rowptr, const int32_t* colidx,
                                 const float* values, const float* X, int64_t ldx, const float* Y, int64_t ldy,
                                 int vop, int rop, int sop, double alpha, real* H) {
  if (sop == O_SOP_EDGE_VALUE && !values && rowptr[m] > 0) return -1;
  if (vop != O_VOP_SEL2ND && !X && rowptr[m] > 0) return -3;
  const int vec = FN(fmm_oracle_h_is_vector)(rop, sop);
  for (int64_t u = 0; u < m; ++u) {
    for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
      const float* yv = Y + (int64_t)colidx[e] * ldy;
      if (vec) {
        for (int64_t k = 0; k < d; ++k) {
          real t = g_vop(vop, X ? (real)X[u * ldx + k] : 0, (real)yv[k]);
          H[e * d + k] = g_sop(sop, t, 0, (real)alpha);
        }
      } else {
        real s = 0;
        if (rop == O_ROP_RMUL) s = 1;
        for (int64_t k = 0; k < d && rop != O_ROP_NOOP; ++k) {
          real t = g_vop(vop, X ? (real)X[u * ldx + k] : 0, (real)yv[k]);
          if (rop == O_ROP_RSUM) s += t;
          else if (rop == O_ROP_RMUL) s *= t;
          else s += t * t;
        }
        if (rop == O_ROP_NORM) s = (real)sqrt((double)s);
        H[e] = g_sop(sop, s, values ? (real)values[e] : 0, (real)alpha);
      }
    }
  }
  return 0;
}

/* Phase 2 of the general path: MOP then AOP over the materialised H. */
int FN(fmm_oracle_spmm_general)(int64_t m, int64_t d, const int64_t* rowptr, const int32_t* colidx,
                                const float* X, int64_t ldx, const float* Y, int64_t ldy,
                                int vop, int mop, int aop, int h_is_vector, const real* H, real* Z, real* S) {
  for (int64_t u = 0; u < m; ++u) {
    for (int64_t k = 0; k < d; ++k) { Z[u * d + k] = 0; if (S) S[u * d + k] = 0; }
    for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
      const float* yv = Y + (int64_t)colidx[e] * ldy;
      for (int64_t k = 0; k < d; ++k) {
        const real h = h_is_vector ? H[e * d + k] : H[e];
        real w;
        if (mop == O_MOP_SEL2ND) w = (real)yv[k];
        else if (mop == O_MOP_MUL_Y) w = h * (real)yv[k];
        else w = h * g_vop(vop, X ? (real)X[u * ldx + k] : 0, (real)yv[k]);
        real* z = &Z[u * d + k];
        const real aw = (real)fabs((double)w);
        if (aop == O_AOP_SUM || aop == O_AOP_MEAN) { *z += w; if (S) S[u * d + k] += aw; }
        else {
          if (aop == O_AOP_MAX) { if (w > *z) *z = w; } else { if (w < *z) *z = w; }
          if (S && aw > S[u * d + k]) S[u * d + k] = aw;
        }
      }
    }
    const int64_t deg = rowptr[u + 1] - rowptr[u];
    if (aop == O_AOP_MEAN && deg > 0) {
      for (int64_t k = 0; k < d; ++k) { Z[u * d + k] /= (real)deg; if (S) S[u * d + k] /= (real)deg; }
    }
  }
  return 0;
}
