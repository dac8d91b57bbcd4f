/*
 * CPU oracle for the Collage MCF-AdamW optimizer step.  TEST INFRASTRUCTURE:
 * see mcf_oracle.h.  Build with -O2 -ffp-contract=off and no fast-math, so
 * that every fp32 operation written below is one IEEE binary32 operation.
 */
#include "mcf_oracle.h"

#include <cmath>
#include <cstring>
#include <limits>
#include <thread>
#include <vector>
#include <xmmintrin.h>

namespace {

inline uint32_t f32_bits(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float bits_f32(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }

/* fp64 -> a 16-bit binary format with MBITS stored significand bits and minimum normal exponent
 * EMIN (exponent bias 1-EMIN), in ONE rounding, round to nearest, ties to even.  The spacing at |x| in
 * [2^e, 2^(e+1)) is 2^(max(e,EMIN)-MBITS) (Def. 3.1 with P = MBITS stored bits, Table 7).  Scale |x| by
 * that spacing, round the quotient to an integer (ties to even) and assemble the fields. */
template <int MBITS, int EMIN>
inline uint16_t round_f64_to_16bit(double x) {
  const uint32_t expo_all_ones = (uint32_t)(2 * (1 - EMIN) + 1);     /* 255 for bf16, 31 for fp16 */
  const uint16_t inf_bits = (uint16_t)(expo_all_ones << MBITS);
  if (std::isnan(x)) return (uint16_t)(inf_bits | (1u << (MBITS - 1)));   /* one quiet NaN: 0x7FC0 / 0x7E00 */
  uint16_t sign = std::signbit(x) ? 0x8000 : 0;
  double a = std::fabs(x);
  if (a == 0.0) return sign;
  if (std::isinf(a)) return sign | inf_bits;
  int e;
  (void)std::frexp(a, &e);          /* a = fr * 2^e, fr in [0.5,1)  =>  2^(e-1) <= a < 2^e */
  e -= 1;
  int emax = e < EMIN ? EMIN : e;
  int qe = emax - MBITS;             /* spacing = 2^qe */
  double s = std::ldexp(a, -qe);     /* exact power-of-two scaling; s < 2^(MBITS+1) */
  double fl = std::floor(s);
  double rem = s - fl;               /* exact */
  uint32_t k = (uint32_t)fl;
  if (rem > 0.5 || (rem == 0.5 && (k & 1u))) k += 1;
  const uint32_t hidden = 1u << MBITS;
  uint32_t bits;
  if (e >= EMIN) {
    /* k in [hidden, 2*hidden]; k == 2*hidden carries into the next exponent by plain addition */
    bits = ((uint32_t)(e - EMIN + 1) << MBITS) + (k - hidden);
    if (bits >= inf_bits) bits = inf_bits;      /* overflow -> infinity */
  } else {
    bits = k;                                   /* subnormal; k == hidden is the least normal */
  }
  return sign | (uint16_t)bits;
}

/* bf16: the upper half of an IEEE binary32 (8 exponent bits, 7 stored significand bits). */
struct Bf16 {
  /* bf16 -> fp32: the 16 bits become the upper half of the binary32 pattern. */
  static float W(uint16_t h) { return bits_f32((uint32_t)h << 16); }
  /* R: fp32 -> bf16, round to nearest, ties to even (Sec. 3.1; the correctness of every algorithm
   * below assumes round-to-nearest, Sec. 4.1 footnote).  bf16 keeps fp32's exponent field, so rounding
   * the low 16 bits away on the bit pattern is right for normals, subnormals and the carry into infinity. */
  static uint16_t R(float f) {
    uint32_t u = f32_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;   /* every NaN -> one quiet NaN */
    uint32_t keep_is_odd = (u >> 16) & 1u;
    u += 0x7fffu + keep_is_odd;
    return (uint16_t)(u >> 16);
  }
  static uint16_t B(double x) { return round_f64_to_16bit<7, -126>(x); }
};

/* fp16: IEEE binary16 (5 exponent bits, 10 stored significand bits, App. A Table 7). */
struct Fp16 {
  static float W(uint16_t h) {
    const int e = (h >> 10) & 0x1f, m = h & 0x3ff;
    float mag;
    if (e == 0) mag = std::ldexp((float)m, -24);                       /* subnormal: m * 2^-24 */
    else if (e == 31) mag = m ? std::numeric_limits<float>::quiet_NaN() : std::numeric_limits<float>::infinity();
    else mag = std::ldexp((float)(1024 + m), e - 25);                  /* (1 + m/1024) * 2^(e-15) */
    return (h & 0x8000) ? -mag : mag;
  }
  /* fp32 -> fp16 in one rounding: widen to fp64 (exact), then the generic single rounding. */
  static uint16_t R(float f) { return round_f64_to_16bit<10, -14>((double)f); }
  static uint16_t B(double x) { return round_f64_to_16bit<10, -14>(x); }
};

/* FP8 E5M2 (App. A Table 7: 5 exponent bits, 2 stored significand bits): an IEEE-style format, the
 * upper byte of a binary16 pattern, with infinities and NaN.  Patterns travel in the low byte of a
 * uint16_t.  Overflow rounds to infinity; every NaN is stored as 0x7E. */
struct Fp8E5M2 {
  static float W(uint16_t h) { return Fp16::W((uint16_t)((h & 0xff) << 8)); }
  static uint16_t fold(uint16_t r) { return (uint16_t)((r & 0x7f) | ((r & 0x8000) >> 8)); }   /* sign from bit 15 to bit 7 */
  static uint16_t R(float f) { return fold(round_f64_to_16bit<2, -14>((double)f)); }
  static uint16_t B(double x) { return fold(round_f64_to_16bit<2, -14>(x)); }
};

/* FP8 E4M3 (Table 7: 4 exponent bits, 3 stored significand bits) in the form the 8-bit formats are
 * deployed in (and the paper's FP8 reference uses): bias 7, NO infinities, the all-ones exponent holds
 * ordinary numbers up to 448 = 0x7E, and only the pattern with all exponent and significand bits set
 * (0x7F, 0xFF) is NaN.  The paper gives no overflow rule; the reading here is the format's non-saturating
 * conversion: whatever rounds beyond 448 (infinities included) becomes NaN.  Every NaN is stored as 0x7F. */
struct Fp8E4M3 {
  static float W(uint16_t h) {
    const int e = (h >> 3) & 0xf, m = h & 7;
    float mag;
    if (e == 15 && m == 7) mag = std::numeric_limits<float>::quiet_NaN();
    else if (e == 0) mag = std::ldexp((float)m, -9);                  /* subnormal: m * 2^-9 */
    else mag = std::ldexp((float)(8 + m), e - 10);                    /* (1 + m/8) * 2^(e-7) */
    return (h & 0x80) ? -mag : mag;
  }
  static uint16_t B(double x) {
    if (std::isnan(x)) return 0x7f;
    const uint16_t sign = std::signbit(x) ? 0x80 : 0;
    const double a = std::fabs(x);
    if (a == 0.0) return sign;
    if (std::isinf(a)) return 0x7f;
    int e;
    (void)std::frexp(a, &e);
    e -= 1;                                    /* 2^e <= a < 2^(e+1) */
    const int emax = e < -6 ? -6 : e;
    const int qe = emax - 3;                   /* spacing 2^qe */
    const double sc = std::ldexp(a, -qe);      /* exact */
    const double fl = std::floor(sc);
    const double rem = sc - fl;
    uint32_t k = (uint32_t)(fl > 64.0 ? 64.0 : fl);      /* anything this large is far out of range anyway */
    if (fl <= 64.0 && (rem > 0.5 || (rem == 0.5 && (k & 1u)))) k += 1;
    if (e > 8) return 0x7f;                    /* 512 and above */
    uint32_t bits = e >= -6 ? ((uint32_t)(e + 7) << 3) + (k - 8) : k;      /* a carry moves into the exponent */
    if (bits >= 0x7f) return 0x7f;             /* beyond 448: no infinity to round to */
    return (uint16_t)(sign | bits);
  }
  static uint16_t R(float f) { return B((double)f); }
};

struct Pair { uint16_t hi, lo; };

/* Everything the method computes, for one 16-bit component format Fm. */
template <class Fm>
struct Chain {
  /* One operation F(a o b): widen, one fp32 op, one rounding (Sec. 3.1). */
  static uint16_t add(uint16_t a, uint16_t b) { float r = Fm::W(a) + Fm::W(b); return Fm::R(r); }
  static uint16_t sub(uint16_t a, uint16_t b) { float r = Fm::W(a) - Fm::W(b); return Fm::R(r); }
  static uint16_t mul(uint16_t a, uint16_t b) { float r = Fm::W(a) * Fm::W(b); return Fm::R(r); }
  static uint16_t div(uint16_t a, uint16_t b) { float r = Fm::W(a) / Fm::W(b); return Fm::R(r); }
  static uint16_t sqrt(uint16_t a) { float r = std::sqrt(Fm::W(a)); return Fm::R(r); }
  /* F(a*b - x) with the product not rounded before the subtraction (Alg. 6). */
  static uint16_t fms(uint16_t a, uint16_t b, uint16_t x) { float r = std::fmaf(Fm::W(a), Fm::W(b), -Fm::W(x)); return Fm::R(r); }

  /* Thm 4.1 */
  static Pair fast2sum(uint16_t a, uint16_t b) {
    uint16_t x = add(a, b);
    uint16_t y = sub(b, sub(x, a));
    return {x, y};
  }

  /* Alg. 3 */
  static Pair two_sum(uint16_t a, uint16_t b) {
    uint16_t x = add(a, b);
    uint16_t b_virtual = sub(x, a);
    uint16_t a_virtual = sub(x, b_virtual);
    uint16_t b_roundoff = sub(b, b_virtual);
    uint16_t a_roundoff = sub(a, a_virtual);
    uint16_t y = add(a_roundoff, b_roundoff);
    return {x, y};
  }

  /* Alg. 1: add the float a to the expansion (x, y). */
  static Pair grow(Pair xy, uint16_t a) {
    Pair uv = fast2sum(xy.hi, a);
    return fast2sum(uv.hi, add(xy.lo, uv.lo));
  }

  /* Alg. 1 with TwoSum (Alg. 3) in place of Fast2Sum: the same expansion where |x| >= |a| holds
   * (App. C), and still exact where it does not. */
  static Pair grow_two_sum(Pair xy, uint16_t a) {
    Pair uv = two_sum(xy.hi, a);
    return two_sum(uv.hi, add(xy.lo, uv.lo));
  }

  /* Alg. 6 */
  static Pair two_prod_fma(uint16_t a, uint16_t b) {
    uint16_t x = mul(a, b);
    uint16_t e = fms(a, b, x);
    return {x, e};
  }

  /* Alg. 7: float v times the expansion (a1, a2). */
  static Pair scaling(uint16_t v, Pair a) {
    Pair xe = two_prod_fma(a.hi, v);
    uint16_t e = add(mul(a.lo, v), xe.lo);
    return fast2sum(xe.hi, e);
  }

  /* Alg. 8: product of two length-2 expansions. */
  static Pair mul_expansion(Pair a, Pair b) {
    Pair xe = two_prod_fma(a.hi, b.hi);
    uint16_t cross = add(mul(a.hi, b.lo), mul(a.lo, b.hi));
    uint16_t e = add(xe.lo, cross);
    return fast2sum(xe.hi, e);
  }

  /* Scalars: computed in fp64, cast once (App. D "Scalar and Bias Correction";
   * Table 2 for the beta2 expansion; Sec. 4.2 treats beta2 as a low-precision value). */
  static void derive_scalars(const orc_hyper &h, uint64_t t, orc_scalars &s) {
    double td = (double)t;
    s.b1 = Fm::B(h.beta1);
    s.c1 = Fm::B(1.0 - h.beta1);
    s.b2 = Fm::B(h.beta2);
    s.b2l = Fm::B(h.beta2 - (double)Fm::W(s.b2));
    s.c2 = Fm::B(1.0 - h.beta2);
    s.bc1 = Fm::B(1.0 - std::pow(h.beta1, td));
    s.bc2 = Fm::B(1.0 - std::pow(h.beta2, td));
    s.e = Fm::B(h.eps);
    s.lam = Fm::B(h.weight_decay);
    s.na = Fm::B(-h.lr);
  }

  /* Alg. 2 lines 8-13 for one element. */
  static void adamw_element(uint16_t &theta, uint16_t &dtheta, uint16_t &m, uint16_t &v, uint16_t *dv,
                            uint16_t g, int variant_and_flags, const orc_scalars &s, uint16_t *delta_out) {
    const int variant = variant_and_flags & 0xff;
    const bool sorted_free = (variant_and_flags & ORC_GROW_TWOSUM) != 0;   /* Grow built on TwoSum */
    if (variant == 4) {
      /* MCF-SGD with momentum (Sec. 1 calls the extension to SGD straightforward and prints no
       * algorithm; this is SGD with the same two changes as Alg. 2: the decay term inside the summed
       * update, App. D, and Grow for the parameter).  s.b1 holds the momentum coefficient mu:
       *   m <- mu*m + g ;  delta <- -alpha*(m + lambda*theta) ;  (theta,dtheta) <- Grow(., delta) */
      uint16_t m_new = add(mul(s.b1, m), g);
      uint16_t delta = mul(s.na, add(m_new, mul(s.lam, theta)));
      Pair th = grow(Pair{theta, dtheta}, delta);
      theta = th.hi;
      dtheta = th.lo;
      m = m_new;
      if (delta_out) *delta_out = delta;
      return;
    }
    /* line 8: m <- beta1*m + (1-beta1)*g */
    uint16_t m_new = add(mul(s.b1, m), mul(s.c1, g));

    /* line 9: the increment (1-beta2)*g^2 */
    uint16_t inc = mul(s.c2, mul(g, g));
    uint16_t v_new;
    if (variant != 1) {
      /* light (and the plain and Kahan baselines): v <- beta2*v + (1-beta2)*g^2 */
      v_new = add(mul(s.b2, v), inc);
    } else {
      /* plus: (v,dv) <- Grow(Mul((b2,b2l),(v,dv)), (1-beta2)*g^2) */
      Pair scaled = mul_expansion(Pair{s.b2, s.b2l}, Pair{v, *dv});
      Pair vv = sorted_free ? grow_two_sum(scaled, inc) : grow(scaled, inc);
      v_new = vv.hi;
      *dv = vv.lo;
    }

    /* lines 10-11: bias correction (first components only) */
    uint16_t m_hat = div(m_new, s.bc1);
    uint16_t v_hat = div(v_new, s.bc2);

    /* line 12: delta <- -alpha * ( m_hat/(sqrt(v_hat)+eps) + lambda*theta )
     * (weight decay inside the summed update, App. D "Weight Decay") */
    /* Alg. 2 prints the epsilon under the root sign; the default reading puts it outside, as in the
     * AdamW the paper says it modifies.  ORC_EPS_INSIDE_SQRT selects the printed form. */
    const bool eps_inside = (variant_and_flags & ORC_EPS_INSIDE_SQRT) != 0;
    uint16_t denom = eps_inside ? sqrt(add(v_hat, s.e)) : add(sqrt(v_hat), s.e);
    uint16_t ratio = div(m_hat, denom);
    uint16_t decay = mul(s.lam, theta);
    uint16_t delta = mul(s.na, add(ratio, decay));

    if (variant == 2) {
      /* option A, Eq. 1: theta <- F(theta + delta); nothing else is kept */
      theta = add(theta, delta);
    } else if (variant == 3) {
      /* Kahan summation (App. B): the auxiliary variable c (stored in dtheta) is first added to
       * the update, the sum is added to the parameter, and what that addition lost becomes the new c:
       * c <- F(u - F(theta_new - theta_old)) */
      uint16_t u = add(delta, dtheta);
      uint16_t theta_new = add(theta, u);
      dtheta = sub(u, sub(theta_new, theta));
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

  /* Def. 3.3 totals over one slice, fp64. */
  static void edq_accumulate(const uint16_t *delta, const uint16_t *th0, const uint16_t *dth0, const uint16_t *th1,
                             const uint16_t *dth1, uint64_t n, double *s1, double *s2, uint64_t *lost) {
    double a1 = 0.0, a2 = 0.0;
    uint64_t nl = 0;
    for (uint64_t i = 0; i < n; ++i) {
      double d = (double)Fm::W(delta[i]);
      double before = (double)Fm::W(th0[i]) + (dth0 ? (double)Fm::W(dth0[i]) : 0.0);
      double after = (double)Fm::W(th1[i]) + (dth1 ? (double)Fm::W(dth1[i]) : 0.0);
      double effective = after - before;           /* Eq. 2, extended to the expansion's value */
      a1 += d * effective;
      a2 += d * d;
      if (d != 0.0 && effective == 0.0) nl += 1;  /* lost arithmetic (Def. 3.2): a non-zero update that changed nothing */
    }
    *s1 += a1;
    *s2 += a2;
    if (lost) *lost += nl;
  }
};

inline uint16_t R(float f) { return Bf16::R(f); }      /* the fp32-master baseline rounds its master weight to bf16 */
inline float W(uint16_t h) { return Bf16::W(h); }

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

/* Host threads the array functions below split their elements over (results do not depend on it). */
int g_array_threads = 1;

}  // namespace

/* Run `body` with Chain<Bf16> or Chain<Fp16> bound to the name C. */
#define ORC_WITH_FORMAT(fmt, ...)                                                               \
  do {                                                                                          \
    if ((fmt) == ORC_FP16) { using C = Chain<Fp16>; using Fm = Fp16; __VA_ARGS__; }             \
    else if ((fmt) == ORC_FP8_E5M2) { using C = Chain<Fp8E5M2>; using Fm = Fp8E5M2; __VA_ARGS__; } \
    else if ((fmt) == ORC_FP8_E4M3) { using C = Chain<Fp8E4M3>; using Fm = Fp8E4M3; __VA_ARGS__; } \
    else { using C = Chain<Bf16>; using Fm = Bf16; __VA_ARGS__; }                               \
  } while (0)

extern "C" {

void orc_set_array_threads(int n) { g_array_threads = n < 1 ? 1 : n; }

uint16_t orc_R_fmt(int fmt, float f) { ORC_WITH_FORMAT(fmt, { (void)sizeof(C); return Fm::R(f); }); return 0; }
uint16_t orc_B_fmt(int fmt, double x) { ORC_WITH_FORMAT(fmt, { (void)sizeof(C); return Fm::B(x); }); return 0; }
float orc_widen_fmt(int fmt, uint16_t h) { ORC_WITH_FORMAT(fmt, { (void)sizeof(C); return Fm::W(h); }); return 0; }
void orc_R_array_fmt(int fmt, const float *f, uint16_t *out, uint64_t n) {
  ORC_WITH_FORMAT(fmt, {
    (void)sizeof(C);
    parallel_ranges(n, g_array_threads, [=](uint64_t lo, uint64_t hi) { for (uint64_t i = lo; i < hi; ++i) out[i] = Fm::R(f[i]); });
  });
}
void orc_widen_array_fmt(int fmt, const uint16_t *h, float *out, uint64_t n) {
  ORC_WITH_FORMAT(fmt, { (void)sizeof(C); for (uint64_t i = 0; i < n; ++i) out[i] = Fm::W(h[i]); });
}
uint16_t orc_R(float f) { return orc_R_fmt(0, f); }
uint16_t orc_B(double x) { return orc_B_fmt(0, x); }
float orc_widen(uint16_t h) { return orc_widen_fmt(0, h); }
void orc_R_array(const float *f, uint16_t *out, uint64_t n) { orc_R_array_fmt(0, f, out, n); }

int orc_fp_env_ok(void) {
  volatile float tiny = bits_f32(0x00000001u);     /* least subnormal */
  volatile float two = 2.0f;
  volatile float r = tiny * two;
  return f32_bits(r) == 0x00000002u;
}

void orc_binop_fmt(int fmt, int op, const uint16_t *a, const uint16_t *b, uint16_t *out, uint64_t n) {
  ORC_WITH_FORMAT(fmt, {
    (void)sizeof(Fm);
    parallel_ranges(n, g_array_threads, [=](uint64_t lo, uint64_t hi) {
      for (uint64_t i = lo; i < hi; ++i) {
        switch (op) {
          case 0: out[i] = C::add(a[i], b[i]); break;
          case 1: out[i] = C::sub(a[i], b[i]); break;
          case 2: out[i] = C::mul(a[i], b[i]); break;
          case 3: out[i] = C::div(a[i], b[i]); break;
          default: out[i] = C::sqrt(a[i]); break;
        }
      }
    });
  });
}
void orc_binop(int op, const uint16_t *a, const uint16_t *b, uint16_t *out, uint64_t n) { orc_binop_fmt(0, op, a, b, out, n); }

/* which: 0 Fast2Sum(p0,p1)  1 TwoSum(p0,p1)  2 Grow((p0,p1),p2)  3 Grow on TwoSum  4 TwoProdFMA(p0,p1)
 *        5 Scaling(v=p0,(p1,p2))  6 Mul((p0,p1),(p2,p3));  results to (o0, o1). */
void orc_prim_fmt(int fmt, int which, const uint16_t *p0, const uint16_t *p1, const uint16_t *p2, const uint16_t *p3,
                  uint16_t *o0, uint16_t *o1, uint64_t n) {
  ORC_WITH_FORMAT(fmt, {
    (void)sizeof(Fm);
    parallel_ranges(n, g_array_threads, [=](uint64_t lo, uint64_t hi) {
      for (uint64_t i = lo; i < hi; ++i) {
        Pair r;
        switch (which) {
          case 0: r = C::fast2sum(p0[i], p1[i]); break;
          case 1: r = C::two_sum(p0[i], p1[i]); break;
          case 2: r = C::grow(Pair{p0[i], p1[i]}, p2[i]); break;
          case 3: r = C::grow_two_sum(Pair{p0[i], p1[i]}, p2[i]); break;
          case 4: r = C::two_prod_fma(p0[i], p1[i]); break;
          case 5: r = C::scaling(p0[i], Pair{p1[i], p2[i]}); break;
          default: r = C::mul_expansion(Pair{p0[i], p1[i]}, Pair{p2[i], p3[i]}); break;
        }
        o0[i] = r.hi;
        o1[i] = r.lo;
      }
    });
  });
}
void orc_fast2sum(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *y, uint64_t n) { orc_prim_fmt(0, 0, a, b, nullptr, nullptr, x, y, n); }
void orc_two_sum(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *y, uint64_t n) { orc_prim_fmt(0, 1, a, b, nullptr, nullptr, x, y, n); }
void orc_grow(uint16_t *x, uint16_t *y, const uint16_t *a, uint64_t n) { orc_prim_fmt(0, 2, x, y, a, nullptr, x, y, n); }
void orc_grow_two_sum(uint16_t *x, uint16_t *y, const uint16_t *a, uint64_t n) { orc_prim_fmt(0, 3, x, y, a, nullptr, x, y, n); }
void orc_two_prod_fma(const uint16_t *a, const uint16_t *b, uint16_t *x, uint16_t *e, uint64_t n) { orc_prim_fmt(0, 4, a, b, nullptr, nullptr, x, e, n); }
void orc_scaling(const uint16_t *v, const uint16_t *a1, const uint16_t *a2, uint16_t *x, uint16_t *e, uint64_t n) { orc_prim_fmt(0, 5, v, a1, a2, nullptr, x, e, n); }
void orc_mul_expansion(const uint16_t *a1, const uint16_t *a2, const uint16_t *b1, const uint16_t *b2,
                       uint16_t *x, uint16_t *e, uint64_t n) { orc_prim_fmt(0, 6, a1, a2, b1, b2, x, e, n); }

void orc_scalars_derive_fmt(int fmt, const orc_hyper *h, uint64_t t, orc_scalars *out) {
  ORC_WITH_FORMAT(fmt, { (void)sizeof(Fm); C::derive_scalars(*h, t, *out); });
}
void orc_scalars_derive(const orc_hyper *h, uint64_t t, orc_scalars *out) { orc_scalars_derive_fmt(0, h, t, out); }

void orc_adamw_step(uint16_t *theta, uint16_t *dtheta, uint16_t *m, uint16_t *v, uint16_t *dv,
                    const uint16_t *grad, uint64_t n, int variant, const orc_hyper *h, uint64_t t,
                    uint16_t *delta_out, int nthreads) {
  const int fmt = (variant >> 12) & 3;          /* ORC_FMT_* flags carry the format id in bits 12-13 */
  ORC_WITH_FORMAT(fmt, {
    (void)sizeof(Fm);
    orc_scalars s;
    C::derive_scalars(*h, t, s);
    parallel_ranges(n, nthreads, [=](uint64_t lo, uint64_t hi) {
      uint16_t unused = 0;
      const int base = variant & 0xff;
      uint16_t no_v = 0;
      for (uint64_t i = lo; i < hi; ++i)
        C::adamw_element(theta[i], base == 2 ? unused : dtheta[i], m[i], base == 4 ? no_v : v[i], base == 1 ? &dv[i] : nullptr,
                         grad[i], variant, s, delta_out ? &delta_out[i] : nullptr);
    });
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

void orc_edq_accumulate_fmt(int fmt, const uint16_t *delta, const uint16_t *th0, const uint16_t *dth0,
                            const uint16_t *th1, const uint16_t *dth1, uint64_t n, double *s1, double *s2,
                            uint64_t *lost) {
  ORC_WITH_FORMAT(fmt, { (void)sizeof(Fm); C::edq_accumulate(delta, th0, dth0, th1, dth1, n, s1, s2, lost); });
}
void orc_edq_accumulate(const uint16_t *delta, const uint16_t *th0, const uint16_t *dth0,
                        const uint16_t *th1, const uint16_t *dth1, uint64_t n, double *s1, double *s2,
                        uint64_t *lost) {
  orc_edq_accumulate_fmt(0, delta, th0, dth0, th1, dth1, n, s1, s2, lost);
}

double orc_edq_finish(double s1, double s2) {
  if (s2 == 0.0) return 0.0;
  return s1 / std::sqrt(s2);                     /* Eq. 3: <delta/||delta||, effective> */
}

}  // extern "C"
