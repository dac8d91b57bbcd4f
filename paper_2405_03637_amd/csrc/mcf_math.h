// Device-side arithmetic of the Collage step for gfx950: the bf16 operation F(a o b)
// (Sec. 3.1), the error-free transformations (Thm 4.1, Alg. 1, 3, 6, 8) and the AdamW
// chains (Alg. 2), written over PAIRS of neighbouring elements because the hardware
// converts two fp32 values to packed bf16 in one instruction.
//
// Two arithmetic modes produce identical bits wherever both apply:
//   Exact : IEEE fp32 divide and square root, rounding done on the bit pattern with every
//           NaN stored as 0x7FC0.  Correct for all inputs.
//   Fast  : v_cvt_pk_bf16_f32 for the rounding, v_rcp_f32 / v_sqrt_f32 (1 ulp) for divide
//           and square root.  Because every operand is a bf16 value (8 significant bits),
//           a/b and sqrt(a) can never fall on a bf16 rounding midpoint and stay at least
//           2^-17 (divide) or 2^-19 (root) away from one in relative terms, so a result
//           with relative error 2^-22 rounds to the same bf16 as the correctly rounded
//           one.  That argument needs the fp32 result to be a normal number; a pair that
//           meets a subnormal intermediate, or produces any NaN, raises `redo` and the
//           caller recomputes that slot in Exact mode.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mcfd {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

struct P2 { float lo, hi; };   // elements 2k and 2k+1, widened to fp32

__device__ __forceinline__ uint32_t fbits(float f) { return __builtin_bit_cast(uint32_t, f); }
__device__ __forceinline__ float bitsf(uint32_t u) { return __builtin_bit_cast(float, u); }

// A dword holds two bf16, element 2k in the low half.
__device__ __forceinline__ P2 widen2(uint32_t w) { return {bitsf(w << 16), bitsf(w & 0xffff0000u)}; }
// Pack two fp32 values that already are bf16 values (low halves zero): one v_perm_b32 taking
// the upper halves of both.
__device__ __forceinline__ uint32_t pack2(P2 x) { return __builtin_amdgcn_perm(fbits(x.hi), fbits(x.lo), 0x07060302u); }

// fp32 -> bf16 round-to-nearest-even on the bit pattern, result left widened; NaN -> 0x7FC0.
__device__ __forceinline__ float round_bits(float f) {
  uint32_t u = fbits(f);
  uint32_t r = (u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u;
  return bitsf((u & 0x7fffffffu) > 0x7f800000u ? 0x7fc00000u : r);
}

__device__ __forceinline__ bool is_subnormal(float x) { return __builtin_amdgcn_classf(x, 0x90); }
__device__ __forceinline__ bool is_nan(float x) { return x != x; }

struct Exact {
  static constexpr bool kFast = false;
  static __device__ __forceinline__ P2 rnd(P2 x) { return {round_bits(x.lo), round_bits(x.hi)}; }
  static __device__ __forceinline__ float div1(float a, float b, float, bool &) { return a / b; }
  static __device__ __forceinline__ float divg1(float a, float b, bool &) { return a / b; }
  static __device__ __forceinline__ float sqrt1(float a, bool &) { return __builtin_sqrtf(a); }
};

struct Fast {
  static constexpr bool kFast = true;
  // v_cvt_pk_bf16_f32 with 0 as its first source leaves bf16(x) in the upper half of the result and
  // bf16(0) = 0 in the lower half: that IS the rounded value widened back to fp32, in one instruction.
  static __device__ __forceinline__ float rnd1(float x) {
    const f32x2_t v = {0.0f, x};
    const bf16x2_t r = __builtin_convertvector(v, bf16x2_t);      // v_cvt_pk_bf16_f32 dst, 0, x
    return __builtin_bit_cast(float, r);
  }
  static __device__ __forceinline__ P2 rnd(P2 x) { return {rnd1(x.lo), rnd1(x.hi)}; }
  // a / b where b is a positive normal scalar with known fp32 reciprocal rb (|rel err| <= 2^-24)
  static __device__ __forceinline__ float div1(float a, float, float rb, bool &redo) {
    float p = a * rb;
    redo |= is_subnormal(p);
    return p;
  }
  // a / b, b any value whose magnitude is 0, infinite or within [2^-126, 2^126]
  static __device__ __forceinline__ float divg1(float a, float b, bool &redo) {
    float p = a * __builtin_amdgcn_rcpf(b);
    redo |= is_subnormal(p);
    return p;
  }
  // sqrt(a), a zero, normal, infinite or NaN
  static __device__ __forceinline__ float sqrt1(float a, bool &) { return __builtin_amdgcn_sqrtf(a); }
};

// The bf16 operations on pairs.  Every function is one F(.): one fp32 operation per
// element, then one rounding.
template <class M> struct Ops {
  static __device__ __forceinline__ P2 add(P2 a, P2 b) { return M::rnd({a.lo + b.lo, a.hi + b.hi}); }
  static __device__ __forceinline__ P2 sub(P2 a, P2 b) { return M::rnd({a.lo - b.lo, a.hi - b.hi}); }
  static __device__ __forceinline__ P2 mul(P2 a, P2 b) { return M::rnd({a.lo * b.lo, a.hi * b.hi}); }
  static __device__ __forceinline__ P2 adds(P2 a, float s) { return M::rnd({a.lo + s, a.hi + s}); }
  static __device__ __forceinline__ P2 muls(float s, P2 a) { return M::rnd({s * a.lo, s * a.hi}); }
  // F(s*a - x), product unrounded (the FMA of Alg. 6)
  static __device__ __forceinline__ P2 fmss(float s, P2 a, P2 x) {
    return M::rnd({__builtin_fmaf(s, a.lo, -x.lo), __builtin_fmaf(s, a.hi, -x.hi)});
  }
  static __device__ __forceinline__ P2 fms(P2 a, P2 b, P2 x) {
    return M::rnd({__builtin_fmaf(a.lo, b.lo, -x.lo), __builtin_fmaf(a.hi, b.hi, -x.hi)});
  }
  static __device__ __forceinline__ P2 divs(P2 a, float b, float rb, bool &redo) {
    return M::rnd({M::div1(a.lo, b, rb, redo), M::div1(a.hi, b, rb, redo)});
  }
  static __device__ __forceinline__ P2 divg(P2 a, P2 b, bool &redo) {
    return M::rnd({M::divg1(a.lo, b.lo, redo), M::divg1(a.hi, b.hi, redo)});
  }
  static __device__ __forceinline__ P2 sqrt(P2 a, bool &redo) {
    return M::rnd({M::sqrt1(a.lo, redo), M::sqrt1(a.hi, redo)});
  }

  // Thm 4.1: (x, y) = Fast2Sum(a, b)
  static __device__ __forceinline__ void fast2sum(P2 a, P2 b, P2 &x, P2 &y) {
    x = add(a, b);
    y = sub(b, sub(x, a));
  }
  // Alg. 3
  static __device__ __forceinline__ void two_sum(P2 a, P2 b, P2 &x, P2 &y) {
    x = add(a, b);
    P2 bv = sub(x, a);
    P2 av = sub(x, bv);
    P2 br = sub(b, bv);
    P2 ar = sub(a, av);
    y = add(ar, br);
  }
  // Alg. 1: (x, y) <- Grow((x, y), a)
  static __device__ __forceinline__ void grow(P2 x, P2 y, P2 a, P2 &xo, P2 &yo) {
    P2 u, w;
    fast2sum(x, a, u, w);
    fast2sum(u, add(y, w), xo, yo);
  }
  // Alg. 1 on TwoSum (Alg. 3): no |x| >= |a| precondition
  static __device__ __forceinline__ void grow2(P2 x, P2 y, P2 a, P2 &xo, P2 &yo) {
    P2 u, w;
    two_sum(x, a, u, w);
    two_sum(u, add(y, w), xo, yo);
  }
};

// bf16 scalars of one step, widened to fp32 (exact), plus fp32 reciprocals of the two
// bias corrections for the Fast mode.
struct StepScalars {
  float b1, c1, b2, b2l, c2, bc1, bc2, rbc1, rbc2, e, lam, na;
};

struct ElemIO {          // one pair of elements of every stream
  P2 th, dth, m, v, dv, g;
};

// Variants of the step.  Light and plus are Collage (Sec. 4.2); the other two are the paper's
// comparison strategies built on the same chain: plain bf16 (option A: line 13 is Eq. 1,
// theta <- F(theta + delta)) and Kahan-compensated bf16 (App. B; dtheta holds the Kahan variable).
// V_SGD is MCF-SGD with momentum (Sec. 1): m <- mu*m + g, delta <- -alpha*(m + lambda*theta), Grow.
enum : int { V_LIGHT = 0, V_PLUS = 1, V_BF16 = 2, V_KAHAN = 3, V_SGD = 4 };

// Alg. 2 lines 8-13 on one pair.  GROW2 builds every Grow on TwoSum.  On return io holds the new theta, dtheta, m, v (and dv);
// delta receives line 12's update.  redo is raised (Fast mode) when this pair must be
// recomputed in Exact mode.
template <class M, int VARIANT, bool GROW2 = false>
__device__ __forceinline__ void adamw_pair(ElemIO &io, const StepScalars &s, P2 &delta, bool &redo) {
  using O = Ops<M>;
  if (VARIANT == V_SGD) {
    const P2 m1 = O::add(O::muls(s.b1, io.m), io.g);            // s.b1 = momentum coefficient
    delta = O::muls(s.na, O::add(m1, O::muls(s.lam, io.th)));
    P2 th1, dth1;
    O::grow(io.th, io.dth, delta, th1, dth1);
    if (M::kFast) redo |= is_nan(th1.lo) | is_nan(dth1.lo) | is_nan(th1.hi) | is_nan(dth1.hi);
    io.th = th1;
    io.dth = dth1;
    io.m = m1;
    return;
  }
  // line 8
  P2 m1 = O::add(O::muls(s.b1, io.m), O::muls(s.c1, io.g));
  // line 9
  P2 inc = O::muls(s.c2, O::mul(io.g, io.g));
  P2 v1, dv1 = {0.f, 0.f};
  if (VARIANT != V_PLUS) {
    v1 = O::add(O::muls(s.b2, io.v), inc);
  } else {
    // Mul((b2, b2l), (v, dv)), Alg. 8 with TwoProdFMA (Alg. 6)
    P2 x = O::muls(s.b2, io.v);
    P2 ex = O::fmss(s.b2, io.v, x);
    P2 cross = O::add(O::muls(s.b2, io.dv), O::muls(s.b2l, io.v));
    P2 e2 = O::add(ex, cross);
    P2 X, E;
    O::fast2sum(x, e2, X, E);
    if (GROW2) O::grow2(X, E, inc, v1, dv1); else O::grow(X, E, inc, v1, dv1);
  }
  // lines 10-11
  P2 mh = O::divs(m1, s.bc1, s.rbc1, redo);
  P2 vh = O::divs(v1, s.bc2, s.rbc2, redo);
  // line 12 (epsilon outside the root; weight decay inside the summed update)
  P2 dn = O::adds(O::sqrt(vh, redo), s.e);
  P2 q = O::divg(mh, dn, redo);
  P2 w = O::muls(s.lam, io.th);
  delta = O::muls(s.na, O::add(q, w));
  // line 13
  P2 th1, dth1 = {0.f, 0.f};
  if (VARIANT == V_BF16) {
    th1 = O::add(io.th, delta);                       // Eq. 1
  } else if (VARIANT == V_KAHAN) {
    const P2 u = O::add(delta, io.dth);               // compensate the update with the Kahan variable
    O::fast2sum(io.th, u, th1, dth1);                 // c <- F(u - F(theta' - theta))
  } else if (GROW2) {
    O::grow2(io.th, io.dth, delta, th1, dth1);
  } else {
    O::grow(io.th, io.dth, delta, th1, dth1);
  }
  if (M::kFast) {
    // Any NaN produced or consumed above reaches theta' or dtheta' (or dv'): m' and v' feed
    // the quotient, the quotient feeds delta, delta feeds theta'.
    redo |= is_nan(th1.lo) | is_nan(dth1.lo) | is_nan(th1.hi) | is_nan(dth1.hi);
    if (VARIANT == V_PLUS) redo |= is_nan(dv1.lo) | is_nan(dv1.hi);
  }
  io.th = th1;
  io.dth = dth1;
  io.m = m1;
  io.v = v1;
  io.dv = dv1;
}

}  // namespace mcfd
