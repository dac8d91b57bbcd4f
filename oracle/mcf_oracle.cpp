/*
 * CPU oracle for the Collage MCF-AdamW optimizer step.  TEST INFRASTRUCTURE:
 * see mcf_oracle.h.  Build with -O2 -ffp-contract=off and no fast-math, so
 * that every fp32 operation written below is one IEEE binary32 operation.
 */
#include "mcf_oracle.h"

#include <cmath>
#include <cstring>
#include <thread>
#include <vector>
#include <xmmintrin.h>

namespace {

inline uint32_t f32_bits(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float bits_f32(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }

/* bf16 -> fp32: the 16 bits become the upper half of the binary32 pattern. */
inline float W(uint16_t h) { return bits_f32((uint32_t)h << 16); }

/* R: fp32 -> bf16, round to nearest, ties to even (Sec. 3.1; the correctness
 * of every algorithm below assumes round-to-nearest, Sec. 4.1 footnote).
 * bf16 keeps fp32's exponent field, so rounding the low 16 bits away on the
 * bit pattern is right for normals, subnormals and the carry into infinity. */
inline uint16_t R(float f) {
  uint32_t u = f32_bits(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;   /* every NaN -> one quiet NaN */
  uint32_t keep_is_odd = (u >> 16) & 1u;
  u += 0x7fffu + keep_is_odd;
  return (uint16_t)(u >> 16);
}

/* B: fp64 -> bf16 in one rounding.  bf16 has 8 significand bits (7 stored),
 * minimum normal exponent -126, so the spacing at |x| in [2^e, 2^(e+1)) is
 * 2^(max(e,-126)-7) (Def. 3.1 with P = 7 stored bits, Table 7).  Scale |x| by
 * that spacing, round the quotient to an integer (ties to even) and assemble. */
inline uint16_t Bround(double x) {
  if (std::isnan(x)) return 0x7fc0;
  uint16_t sign = std::signbit(x) ? 0x8000 : 0;
  double a = std::fabs(x);
  if (a == 0.0) return sign;
  if (std::isinf(a)) return sign | 0x7f80;
  int e;
  (void)std::frexp(a, &e);          /* a = fr * 2^e, fr in [0.5,1)  =>  2^(e-1) <= a < 2^e */
  e -= 1;
  int emax = e < -126 ? -126 : e;
  int qe = emax - 7;                 /* spacing = 2^qe */
  double s = std::ldexp(a, -qe);     /* exact power-of-two scaling; s < 256 */
  double fl = std::floor(s);
  double rem = s - fl;               /* exact */
  uint32_t k = (uint32_t)fl;
  if (rem > 0.5 || (rem == 0.5 && (k & 1u))) k += 1;
  uint32_t bits;
  if (e >= -126) {
    /* k in [128,256]; k == 256 carries into the next exponent by plain addition */
    bits = ((uint32_t)(e + 127) << 7) + (k - 128u);
    if (bits >= 0x7f80u) bits = 0x7f80u;      /* overflow -> infinity */
  } else {
    bits = k;                                  /* subnormal; k == 128 is the least normal */
  }
  return sign | (uint16_t)bits;
}

/* One bf16 operation F(a o b): widen, one fp32 op, one rounding. */
inline uint16_t Fadd(uint16_t a, uint16_t b) { float r = W(a) + W(b); return R(r); }
inline uint16_t Fsub(uint16_t a, uint16_t b) { float r = W(a) - W(b); return R(r); }
inline uint16_t Fmul(uint16_t a, uint16_t b) { float r = W(a) * W(b); return R(r); }
inline uint16_t Fdiv(uint16_t a, uint16_t b) { float r = W(a) / W(b); return R(r); }
inline uint16_t Fsqrt(uint16_t a)            { float r = std::sqrt(W(a)); return R(r); }
/* F(a*b - x) with the product not rounded before the subtraction (Alg. 6). */
inline uint16_t Ffms(uint16_t a, uint16_t b, uint16_t x) { float r = std::fmaf(W(a), W(b), -W(x)); return R(r); }

struct Pair { uint16_t hi, lo; };

/* Thm 4.1 */
inline Pair fast2sum(uint16_t a, uint16_t b) {
  uint16_t x = Fadd(a, b);
  uint16_t y = Fsub(b, Fsub(x, a));
  return {x, y};
}

/* Alg. 3 */
inline Pair two_sum(uint16_t a, uint16_t b) {
  uint16_t x = Fadd(a, b);
  uint16_t b_virtual = Fsub(x, a);
  uint16_t a_virtual = Fsub(x, b_virtual);
  uint16_t b_roundoff = Fsub(b, b_virtual);
  uint16_t a_roundoff = Fsub(a, a_virtual);
  uint16_t y = Fadd(a_roundoff, b_roundoff);
  return {x, y};
}

/* Alg. 1: add the float a to the expansion (x, y). */
inline Pair grow(Pair xy, uint16_t a) {
  Pair uv = fast2sum(xy.hi, a);
  return fast2sum(uv.hi, Fadd(xy.lo, uv.lo));
}

/* Alg. 1 with TwoSum (Alg. 3) in place of Fast2Sum: the same expansion where |x| >= |a| holds
 * (App. C), and still exact where it does not. */
inline Pair grow_two_sum(Pair xy, uint16_t a) {
  Pair uv = two_sum(xy.hi, a);
  return two_sum(uv.hi, Fadd(xy.lo, uv.lo));
}

/* Alg. 6 */
inline Pair two_prod_fma(uint16_t a, uint16_t b) {
  uint16_t x = Fmul(a, b);
  uint16_t e = Ffms(a, b, x);
  return {x, e};
}

/* Alg. 7: float v times the expansion (a1, a2). */
inline Pair scaling(uint16_t v, Pair a) {
  Pair xe = two_prod_fma(a.hi, v);
  uint16_t e = Fadd(Fmul(a.lo, v), xe.lo);
  return fast2sum(xe.hi, e);
}

/* Alg. 8: product of two length-2 expansions. */
inline Pair mul_expansion(Pair a, Pair b) {
  Pair xe = two_prod_fma(a.hi, b.hi);
  uint16_t cross = Fadd(Fmul(a.hi, b.lo), Fmul(a.lo, b.hi));
  uint16_t e = Fadd(xe.lo, cross);
  return fast2sum(xe.hi, e);
}

/* Scalars: computed in fp64, cast once (App. D "Scalar and Bias Correction";
 * Table 2 for the beta2 expansion; Sec. 4.2 treats beta2 as a bf16 value). */
void derive_scalars(const orc_hyper &h, uint64_t t, orc_scalars &s) {
  double td = (double)t;
  s.b1 = Bround(h.beta1);
  s.c1 = Bround(1.0 - h.beta1);
  s.b2 = Bround(h.beta2);
  s.b2l = Bround(h.beta2 - (double)W(s.b2));
  s.c2 = Bround(1.0 - h.beta2);
  s.bc1 = Bround(1.0 - std::pow(h.beta1, td));
  s.bc2 = Bround(1.0 - std::pow(h.beta2, td));
  s.e = Bround(h.eps);
  s.lam = Bround(h.weight_decay);
  s.na = Bround(-h.lr);
}

/* Alg. 2 lines 8-13 for one element. */
inline void adamw_element(uint16_t &theta, uint16_t &dtheta, uint16_t &m, uint16_t &v, uint16_t *dv,
                          uint16_t g, int variant_and_flags, const orc_scalars &s, uint16_t *delta_out) {
  const int variant = variant_and_flags & 0xff;
  const bool sorted_free = (variant_and_flags & ORC_GROW_TWOSUM) != 0;   /* Grow built on TwoSum */
  if (variant == 4) {
    /* MCF-SGD with momentum (Sec. 1 calls the extension to SGD straightforward and prints no
     * algorithm; this is SGD with the same two changes as Alg. 2: the decay term inside the summed
     * update, App. D, and Grow for the parameter).  s.b1 holds the momentum coefficient mu:
     *   m <- mu*m + g ;  delta <- -alpha*(m + lambda*theta) ;  (theta,dtheta) <- Grow(., delta) */
    uint16_t m_new = Fadd(Fmul(s.b1, m), g);
    uint16_t delta = Fmul(s.na, Fadd(m_new, Fmul(s.lam, theta)));
    Pair th = grow(Pair{theta, dtheta}, delta);
    theta = th.hi;
    dtheta = th.lo;
    m = m_new;
    if (delta_out) *delta_out = delta;
    return;
  }
  /* line 8: m <- beta1*m + (1-beta1)*g */
  uint16_t m_new = Fadd(Fmul(s.b1, m), Fmul(s.c1, g));

  /* line 9: the increment (1-beta2)*g^2 */
  uint16_t inc = Fmul(s.c2, Fmul(g, g));
  uint16_t v_new;
  if (variant != 1) {
    /* light (and the plain-bf16 and Kahan baselines): v <- beta2*v + (1-beta2)*g^2 */
    v_new = Fadd(Fmul(s.b2, v), inc);
  } else {
    /* plus: (v,dv) <- Grow(Mul((b2,b2l),(v,dv)), (1-beta2)*g^2) */
    Pair scaled = mul_expansion(Pair{s.b2, s.b2l}, Pair{v, *dv});
    Pair vv = sorted_free ? grow_two_sum(scaled, inc) : grow(scaled, inc);
    v_new = vv.hi;
    *dv = vv.lo;
  }

  /* lines 10-11: bias correction (first components only) */
  uint16_t m_hat = Fdiv(m_new, s.bc1);
  uint16_t v_hat = Fdiv(v_new, s.bc2);

  /* line 12: delta <- -alpha * ( m_hat/(sqrt(v_hat)+eps) + lambda*theta )
   * (weight decay inside the summed update, App. D "Weight Decay") */
  uint16_t denom = Fadd(Fsqrt(v_hat), s.e);
  uint16_t ratio = Fdiv(m_hat, denom);
  uint16_t decay = Fmul(s.lam, theta);
  uint16_t delta = Fmul(s.na, Fadd(ratio, decay));

  if (variant == 2) {
    /* option A, Eq. 1: theta <- F(theta + delta); nothing else is kept */
    theta = Fadd(theta, delta);
  } else if (variant == 3) {
    /* Kahan summation (App. B): the auxiliary variable c (stored in dtheta) is first added to
     * the update, the sum is added to the parameter, and what that addition lost becomes the new c:
     * c <- F(u - F(theta_new - theta_old)) */
    uint16_t u = Fadd(delta, dtheta);
    uint16_t theta_new = Fadd(theta, u);
    dtheta = Fsub(u, Fsub(theta_new, theta));
    theta = theta_new;
  } else {
    /* line 13: (theta,dtheta) <- Grow((theta,dtheta), delta) */
    Pair th = sorted_free ? grow_two_sum(Pair{theta, dtheta}, delta) : grow(Pair{theta, dtheta}, delta);
    theta = th.hi;
    dtheta = th.lo;
  }
  m = m_new;
  v = v_new;
  if (delta_out) *delta_out = delta;
}

/* Option D for one element: the same formulas in plain fp32, one IEEE
 * operation per arithmetic symbol, master weight kept in fp32 and the bf16
 * parameter refreshed from it by one rounding. */
struct F32Scalars { float b1, c1, b2, c2, bc1, bc2, e, lam, na; };

inline void fp32mw_element(uint16_t &theta, float &master, float &m, float &v, uint16_t g16,
                           const F32Scalars &s) {
  float g = W(g16);
  float t1 = s.b1 * m;
  float t2 = s.c1 * g;
  float m_new = t1 + t2;
  float g2 = g * g;
  float t3 = s.b2 * v;
  float t4 = s.c2 * g2;
  float v_new = t3 + t4;
  float m_hat = m_new / s.bc1;
  float v_hat = v_new / s.bc2;
  float root = std::sqrt(v_hat);
  float denom = root + s.e;
  float ratio = m_hat / denom;
  float decay = s.lam * master;
  float sum = ratio + decay;
  float delta = s.na * sum;
  float w = master + delta;
  master = w;
  m = m_new;
  v = v_new;
  theta = R(w);
}

/* Give a worker thread IEEE defaults (round to nearest, subnormals kept),
 * whatever the embedding process did to its own control register. */
inline void ieee_defaults() { _mm_setcsr(0x1f80); }

template <class Fn>
void parallel_ranges(uint64_t n, int nthreads, Fn fn) {
  if (nthreads < 1) nthreads = 1;
  if ((uint64_t)nthreads > n) nthreads = n ? (int)n : 1;
  if (nthreads == 1) {
    unsigned saved = _mm_getcsr();
    ieee_defaults();
    fn((uint64_t)0, n);
    _mm_setcsr(saved);
    return;
  }
  std::vector<std::thread> pool;
  uint64_t per = n / (uint64_t)nthreads, extra = n % (uint64_t)nthreads, lo = 0;
  for (int k = 0; k < nthreads; ++k) {
    uint64_t len = per + ((uint64_t)k < extra ? 1 : 0);
    uint64_t hi = lo + len;
    pool.emplace_back([=]() { ieee_defaults(); fn(lo, hi); });
    lo = hi;
  }
  for (auto &th : pool) th.join();
}

}  // namespace

extern "C" {

uint16_t orc_R(float f) { return R(f); }
uint16_t orc_B(double x) { return Bround(x); }
float orc_widen(uint16_t h) { return W(h); }
void orc_R_array(const float *f, uint16_t *out, uint64_t n) { for (uint64_t i = 0; i < n; ++i) out[i] = R(f[i]); }

int orc_fp_env_ok(void) {
  volatile float tiny = bits_f32(0x00000001u);     /* least subnormal */
  volatile float two = 2.0f;
  volatile float r = tiny * two;
  return f32_bits(r) == 0x00000002u;
}

void orc_binop(int op, const uint16_t *a, const uint16_t *b, uint16_t *out, uint64_t n) {
  parallel_ranges(n, 1, [=](uint64_t lo, uint64_t hi) {
    for (uint64_t i = lo; i < hi; ++i) {
      switch (op) {
        case 0: out[i] = Fadd(a[i], b[i]); break;
        case 1: out[i] = Fsub(a[i], b[i]); break;
        case 2: out[i] = Fmul(a[i], b[i]); break;
        case 3: out[i] = Fdiv(a[i], b[i]); break;
        default: out[i] = Fsqrt(a[i]); break;
      }
    }
  });
}

void orc_fast2sum(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *y, uint64_t n) {
  parallel_ranges(n, 1, [=](uint64_t lo, uint64_t hi) {
    for (uint64_t i = lo; i < hi; ++i) { Pair p = fast2sum(a[i], b[i]); x[i] = p.hi; y[i] = p.lo; }
  });
}

void orc_two_sum(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *y, uint64_t n) {
  parallel_ranges(n, 1, [=](uint64_t lo, uint64_t hi) {
    for (uint64_t i = lo; i < hi; ++i) { Pair p = two_sum(a[i], b[i]); x[i] = p.hi; y[i] = p.lo; }
  });
}

void orc_grow(uint16_t *x, uint16_t *y, const uint16_t *a, uint64_t n) {
  parallel_ranges(n, 1, [=](uint64_t lo, uint64_t hi) {
    for (uint64_t i = lo; i < hi; ++i) { Pair p = grow(Pair{x[i], y[i]}, a[i]); x[i] = p.hi; y[i] = p.lo; }
  });
}

void orc_grow_two_sum(uint16_t *x, uint16_t *y, const uint16_t *a, uint64_t n) {
  parallel_ranges(n, 1, [=](uint64_t lo, uint64_t hi) {
    for (uint64_t i = lo; i < hi; ++i) { Pair p = grow_two_sum(Pair{x[i], y[i]}, a[i]); x[i] = p.hi; y[i] = p.lo; }
  });
}

void orc_two_prod_fma(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *e, uint64_t n) {
  parallel_ranges(n, 1, [=](uint64_t lo, uint64_t hi) {
    for (uint64_t i = lo; i < hi; ++i) { Pair p = two_prod_fma(a[i], b[i]); x[i] = p.hi; e[i] = p.lo; }
  });
}

void orc_scaling(const uint16_t *v, const uint16_t *a1, const uint16_t *a2, uint16_t *x, uint16_t *e, uint64_t n) {
  parallel_ranges(n, 1, [=](uint64_t lo, uint64_t hi) {
    for (uint64_t i = lo; i < hi; ++i) { Pair p = scaling(v[i], Pair{a1[i], a2[i]}); x[i] = p.hi; e[i] = p.lo; }
  });
}

void orc_mul_expansion(const uint16_t *a1, const uint16_t *a2, const uint16_t *b1, const uint16_t *b2,
                       uint16_t *x, uint16_t *e, uint64_t n) {
  parallel_ranges(n, 1, [=](uint64_t lo, uint64_t hi) {
    for (uint64_t i = lo; i < hi; ++i) {
      Pair p = mul_expansion(Pair{a1[i], a2[i]}, Pair{b1[i], b2[i]});
      x[i] = p.hi; e[i] = p.lo;
    }
  });
}

void orc_scalars_derive(const orc_hyper *h, uint64_t t, orc_scalars *out) { derive_scalars(*h, t, *out); }

void orc_adamw_step(uint16_t *theta, uint16_t *dtheta, uint16_t *m, uint16_t *v, uint16_t *dv,
                    const uint16_t *grad, uint64_t n, int variant, const orc_hyper *h, uint64_t t,
                    uint16_t *delta_out, int nthreads) {
  orc_scalars s;
  derive_scalars(*h, t, s);
  parallel_ranges(n, nthreads, [=](uint64_t lo, uint64_t hi) {
    uint16_t unused = 0;
    const int base = variant & 0xff;
    uint16_t no_v = 0;
    for (uint64_t i = lo; i < hi; ++i)
      adamw_element(theta[i], base == 2 ? unused : dtheta[i], m[i], base == 4 ? no_v : v[i], base == 1 ? &dv[i] : nullptr,
                    grad[i], variant, s, delta_out ? &delta_out[i] : nullptr);
  });
}

void orc_fp32mw_step(uint16_t *theta, float *master, float *m, float *v, const uint16_t *grad,
                     uint64_t n, const orc_hyper *h, uint64_t t, int nthreads) {
  double td = (double)t;
  F32Scalars s;
  s.b1 = (float)h->beta1;
  s.c1 = (float)(1.0 - h->beta1);
  s.b2 = (float)h->beta2;
  s.c2 = (float)(1.0 - h->beta2);
  s.bc1 = (float)(1.0 - std::pow(h->beta1, td));
  s.bc2 = (float)(1.0 - std::pow(h->beta2, td));
  s.e = (float)h->eps;
  s.lam = (float)h->weight_decay;
  s.na = (float)(-h->lr);
  parallel_ranges(n, nthreads, [=](uint64_t lo, uint64_t hi) {
    for (uint64_t i = lo; i < hi; ++i) fp32mw_element(theta[i], master[i], m[i], v[i], grad[i], s);
  });
}

void orc_edq_accumulate(const uint16_t *delta, const uint16_t *th0, const uint16_t *dth0,
                        const uint16_t *th1, const uint16_t *dth1, uint64_t n, double *s1, double *s2,
                        uint64_t *lost) {
  double a1 = 0.0, a2 = 0.0;
  uint64_t nl = 0;
  for (uint64_t i = 0; i < n; ++i) {
    double d = (double)W(delta[i]);
    double before = (double)W(th0[i]) + (dth0 ? (double)W(dth0[i]) : 0.0);
    double after = (double)W(th1[i]) + (dth1 ? (double)W(dth1[i]) : 0.0);
    double effective = after - before;           /* Eq. 2, extended to the expansion's value */
    a1 += d * effective;
    a2 += d * d;
    if (d != 0.0 && effective == 0.0) nl += 1;  /* lost arithmetic (Def. 3.2): a non-zero update that changed nothing */
  }
  *s1 += a1;
  *s2 += a2;
  if (lost) *lost += nl;
}

double orc_edq_finish(double s1, double s2) {
  if (s2 == 0.0) return 0.0;
  return s1 / std::sqrt(s2);                     /* Eq. 3: <delta/||delta||, effective> */
}

}  // extern "C"
