/*
 * CPU oracle for the Collage MCF-AdamW optimizer step (arXiv 2405.03637).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * step-by-step restatement of what the paper's method computes, used only by
 * the tests, the smoke check and the benchmark's cpu_baseline leg to judge the
 * GPU library.  It shares no code with the GPU library and the GPU library
 * never calls it.
 *
 * Conventions
 *   bf16      : uint16_t holding the upper 16 bits of an IEEE binary32.
 *   F(a o b)  : the paper's bf16 operation (Sec. 3.1): the operands are widened
 *               exactly to fp32, ONE fp32 operation is done, and the result is
 *               rounded once to bf16 with round-to-nearest-even.
 *   R(f)      : fp32 -> bf16, round-to-nearest-even, NaN -> 0x7FC0.
 *   B(x)      : fp64 -> bf16 in ONE rounding (not through float).
 *   format    : the paper states its algorithms for any low-precision component format and names
 *               fp16 beside bf16 (Sec. 1, App. A Table 7).  Functions ending in _fmt take a format
 *               id (ORC_BF16 = 0, ORC_FP16 = 1: IEEE binary16 in a uint16_t) and do the same
 *               steps with W, R and B of that format; the step takes ORC_FMT_FP16 OR-ed onto its
 *               variant.  The names without _fmt are the bf16 ones.  The two FP8 formats of Table 7
 *               (ids 2 and 3) are the paper's "direct extension to 8-bit" (Sec. 7) read as the
 *               same chain with W, R, B of those formats; E5M2 is IEEE-style, E4M3 has no
 *               infinities (see the format structs in mcf_oracle.cpp for the overflow reading).
 *
 * Parity status: every function below is pinned by tests/test_oracle_*.py to
 * values the paper prints, to exact rational arithmetic, to closed forms or to
 * a textbook fp64 AdamW.  The bit-level choice of where roundings fall inside
 * Algorithm 2 (one rounding per elementary operation, bf16 scalars, epsilon
 * outside the square root) is a reading of the paper, which prints no worked
 * AdamW step; that reading is the definition and is listed with the repository's
 * design notes.  For fp16 the chain code is the same template; its decode and its two roundings
 * are pinned by tests/test_oracle_fp16.py to exact rational arithmetic and to numpy's binary16.
 */
#ifndef MCF_ORACLE_H
#define MCF_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- rounding primitives (Sec. 3.1, Def. 3.1, App. A Table 7) ---- */
uint16_t orc_R(float f);          /* fp32 -> bf16 RNE */
uint16_t orc_B(double x);         /* fp64 -> bf16 RNE, single rounding */
float    orc_widen(uint16_t h);   /* bf16 -> fp32, exact */
void     orc_R_array(const float *f, uint16_t *out, uint64_t n);   /* R over an array */
#define ORC_BF16 0
#define ORC_FP16 1
#define ORC_FP8_E5M2 2       /* 8-bit patterns travel in the low byte of the uint16_t arrays */
#define ORC_FP8_E4M3 3
uint16_t orc_R_fmt(int fmt, float f);
uint16_t orc_B_fmt(int fmt, double x);
float    orc_widen_fmt(int fmt, uint16_t h);
void     orc_R_array_fmt(int fmt, const float *f, uint16_t *out, uint64_t n);
void     orc_widen_array_fmt(int fmt, const uint16_t *h, float *out, uint64_t n);
/* Host threads the array functions (R over arrays, binop, prim) split their elements over; 1 at
 * start.  Elements are independent, so the results do not depend on it. */
void     orc_set_array_threads(int n);
/* 1 if fp32 subnormals are neither flushed on input nor on output here. */
int      orc_fp_env_ok(void);

/* ---- one bf16 operation over arrays: out[i] = F(a[i] op b[i]) ----
 * op: 0 add, 1 sub, 2 mul, 3 div, 4 sqrt (b ignored, may be NULL). */
void orc_binop(int op, const uint16_t *a, const uint16_t *b, uint16_t *out, uint64_t n);
void orc_binop_fmt(int fmt, int op, const uint16_t *a, const uint16_t *b, uint16_t *out, uint64_t n);

/* ---- error-free transformations ---- */
/* Thm 4.1: x = F(a+b), y = F(b - F(x-a)). */
void orc_fast2sum(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *y, uint64_t n);
/* Alg. 3 (TwoSum), six operations, no ordering assumption. */
void orc_two_sum(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *y, uint64_t n);
/* Alg. 1 (Grow): (x,y) <- Grow((x,y), a), in place. */
void orc_grow(uint16_t *x, uint16_t *y, const uint16_t *a, uint64_t n);
/* Alg. 1 with TwoSum in place of Fast2Sum (App. C: the same expansion without the ordering), in place. */
void orc_grow_two_sum(uint16_t *x, uint16_t *y, const uint16_t *a, uint64_t n);
/* Alg. 6 (TwoProdFMA): x = F(a*b), e = F(fma(a,b,-x)). */
void orc_two_prod_fma(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *e, uint64_t n);
/* Alg. 7 (Scaling): (x,e) = v * (a1,a2). */
void orc_scaling(const uint16_t *v, const uint16_t *a1, const uint16_t *a2, uint16_t *x, uint16_t *e, uint64_t n);
/* Alg. 8 (Mul): (x,e) = (a1,a2)*(b1,b2), all arrays of length n. */
void orc_mul_expansion(const uint16_t *a1, const uint16_t *a2, const uint16_t *b1, const uint16_t *b2,
                       uint16_t *x, uint16_t *e, uint64_t n);

/* Any of the seven above in either format.  which: 0 Fast2Sum(p0,p1), 1 TwoSum(p0,p1),
 * 2 Grow((p0,p1),p2), 3 Grow on TwoSum, 4 TwoProdFMA(p0,p1), 5 Scaling(v=p0,(p1,p2)),
 * 6 Mul((p0,p1),(p2,p3)); the two results go to o0 and o1 (which may alias inputs). */
void orc_prim_fmt(int fmt, int which, const uint16_t *p0, const uint16_t *p1, const uint16_t *p2, const uint16_t *p3,
                  uint16_t *o0, uint16_t *o1, uint64_t n);

/* ---- AdamW scalars (Alg. 2 line 1, Table 2, App. D "Scalar and Bias Correction") ---- */
typedef struct { double lr, beta1, beta2, eps, weight_decay; } orc_hyper;
#define ORC_GROW_TWOSUM 0x100
#define ORC_EPS_INSIDE_SQRT 0x200   /* line 12 as printed: m_hat / sqrt(v_hat + eps) instead of m_hat / (sqrt(v_hat) + eps) */
#define ORC_FMT_FP16 0x1000    /* OR-ed onto the step's variant: every array and scalar is fp16 */
#define ORC_FMT_FP8_E5M2 0x2000   /* ... FP8 E5M2 (format id << 12) */
#define ORC_FMT_FP8_E4M3 0x3000   /* ... FP8 E4M3 */
typedef struct {
  uint16_t b1;   /* B(beta1)            */
  uint16_t c1;   /* B(1-beta1)          */
  uint16_t b2;   /* B(beta2)   (first component of the beta2 expansion) */
  uint16_t b2l;  /* B(beta2 - b2)  (second component; used by plus only) */
  uint16_t c2;   /* B(1-beta2)          */
  uint16_t bc1;  /* B(1-beta1^t)        */
  uint16_t bc2;  /* B(1-beta2^t)        */
  uint16_t e;    /* B(eps)              */
  uint16_t lam;  /* B(weight_decay)     */
  uint16_t na;   /* B(-lr)              */
} orc_scalars;
void orc_scalars_derive(const orc_hyper *h, uint64_t t, orc_scalars *out);
void orc_scalars_derive_fmt(int fmt, const orc_hyper *h, uint64_t t, orc_scalars *out);

/* ---- the step (Alg. 2 lines 8-13) ----
 * variant 0 = Collage-light (option B), 1 = Collage-plus (option C; dv required),
 *         2 = plain bf16 (option A: line 13 is theta <- F(theta + delta), Eq. 1; dtheta unused, may be NULL),
 *         3 = Kahan-compensated bf16 (App. B; dtheta holds the Kahan variable c),
 *         4 = MCF-SGD with momentum (Sec. 1): m <- beta1*m + g, delta <- -lr*(m + wd*theta), Grow;
 *             beta1 is the momentum coefficient, beta2 and eps are ignored, v is unused (may be NULL).
 * ORC_GROW_TWOSUM may be OR-ed onto variants 0 and 1: every Grow then uses TwoSum (Alg. 3)
 * instead of Fast2Sum, which drops the |x| >= |a| precondition of Alg. 1.
 * ORC_FMT_FP16 may be OR-ed onto any variant: the same steps on fp16 arrays with fp16 scalars.
 * ORC_EPS_INSIDE_SQRT may be OR-ed onto variants 0-3: the denominator of line 12 is F(sqrt(F(v_hat + eps)))
 * as Alg. 2 prints it, instead of F(F(sqrt(v_hat)) + eps).
 * All state is updated in place.  delta_out, if not NULL, receives the bf16
 * update Delta-theta of line 12 for every element.  nthreads >= 1 splits the
 * elements evenly over that many host threads (elements are independent). */
void orc_adamw_step(uint16_t *theta, uint16_t *dtheta, uint16_t *m, uint16_t *v, uint16_t *dv,
                    const uint16_t *grad, uint64_t n, int variant, const orc_hyper *h, uint64_t t,
                    uint16_t *delta_out, int nthreads);

/* ---- option D: bf16 theta/grad, fp32 m, v and master weights (Sec. 2.1, Table 1) ---- */
void orc_fp32mw_step(uint16_t *theta, float *master, float *m, float *v, const uint16_t *grad,
                     uint64_t n, const orc_hyper *h, uint64_t t, int nthreads);

/* ---- effective descent quality (Def. 3.3, Eq. 2-3), fp64 ----
 * delta      : intended update Delta-theta (bf16)
 * th0,dth0   : parameter expansion before the step (dth0 may be NULL = 0)
 * th1,dth1   : parameter expansion after the step  (dth1 may be NULL = 0)
 * Adds this slice's contributions to s1 (sum delta*effective) and s2 (sum
 * delta^2); orc_edq_finish turns the totals into EDQ = s1/sqrt(s2) (0 if s2=0).
 * lost, if not NULL, is increased by the number of elements with a non-zero update
 * whose value did not change (lost arithmetic, Def. 3.2; the "imprecision
 * percentage" of the BERT case study is this count over n). */
void   orc_edq_accumulate(const uint16_t *delta, const uint16_t *th0, const uint16_t *dth0,
                          const uint16_t *th1, const uint16_t *dth1, uint64_t n,
                          double *s1, double *s2, uint64_t *lost /* may be NULL */);
void   orc_edq_accumulate_fmt(int fmt, const uint16_t *delta, const uint16_t *th0, const uint16_t *dth0,
                              const uint16_t *th1, const uint16_t *dth1, uint64_t n,
                              double *s1, double *s2, uint64_t *lost /* may be NULL */);
double orc_edq_finish(double s1, double s2);

#ifdef __cplusplus
}
#endif
#endif
