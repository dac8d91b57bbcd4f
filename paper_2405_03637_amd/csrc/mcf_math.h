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
//           a normal a/b or sqrt(a) can never fall on a bf16 rounding midpoint and stays at
//           least 2^-17 (divide) or 2^-19 (root) away from one in relative terms, so a result
//           with relative error 2^-22 rounds to the same bf16 as the correctly rounded one.
//           Quotients below 2^-126 sit on fp32's fixed grid of 2^-149: one that is not a tie of
//           the bf16 rounding (spacing 2^-133 there) is at least 2^-142 from the nearest, far more
//           than the error of a*r; one that is a tie has a divisor whose significand divides
//           the dividend's, so it is either below 2^-127.5, where the error of a*r is under half
//           a grid step and the fp32 rounding of the product lands on the tie itself, or has a
//           power of two as divisor, whose reciprocal is exact.  (Checked on the CPU for all bf16
//           pairs with such quotients with r anywhere within one unit of 1/b, and for every bf16
//           dividend against every bias correction in [2^-60, 1]; on the hardware for all 2^32
//           pairs.)  v_sqrt_f32 takes a subnormal operand for
//           zero, and the hardware conversion keeps a NaN's payload where 0x7FC0 is to be stored: the first
//           pass over a slot raises `redo` on either (a second moment that decayed to nothing under zero
//           gradients; any NaN), and the caller computes that slot again in the second-pass flavour of this
//           mode, whose root scales tiny operands by 2^64 and whose pack stores the one NaN pattern.  What is
//           left for Exact mode: launches whose scalars the host finds outside the ranges above, and the
//           fallback of the single-operation primitives.
// The same chains run over three more component formats (App. A Table 7), each with a first-pass mode
// and a mode that stores the format's one NaN: fp16 in packed half arithmetic (Hf), and FP8 E5M2 and
// E4M3 through the hardware conversions (F8).  Every mode offers the same static interface (T, S,
// unpack, pack, add ... sqrt), and Ops<M> builds the expansion algorithms on it.
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

// ---- bf16 -------------------------------------------------------------------------------
// Rounders: how one fp32 result becomes a bf16 value (left widened in an fp32 register).
struct ExactR {
  static constexpr bool kFast = false;      // never asks for a redo
  static constexpr bool kCanon = false;     // its rounding already stores every NaN as 0x7FC0
  static __device__ __forceinline__ P2 rnd(P2 x) { return {round_bits(x.lo), round_bits(x.hi)}; }
  static __device__ __forceinline__ float div1(float a, float b, float, bool &) { return a / b; }
  static __device__ __forceinline__ float divg1(float a, float b, bool &) { return a / b; }
  static __device__ __forceinline__ float sqrt1(float a, bool &) { return __builtin_sqrtf(a); }
};

// SCALED selects how the root treats a subnormal operand, which v_sqrt_f32 takes for zero: false raises
// `redo` (first pass: such operands are rare and the test is one instruction), true scales it by the
// exact factor 2^64 first and the root by 2^-32 afterwards (the pass that redoes those slots).
// CANON: the pair is packed with every NaN replaced by 0x7FC0 (the hardware conversion keeps payloads and signs).
// The first pass (SCALED, CANON both false) is the only one that asks for a redo; the second pass
// (both true) is right for every input the first pass gives up on: the restricted divide is wrong for
// no value the chain can meet (its divisors are normal, zero or infinite by the host's checks on the
// scalars; x/0, 0/0, x/inf and inf/inf come out as IEEE has them through v_rcp_f32's inf and 0), the scaled root
// takes subnormal operands, and a NaN is a NaN in either arithmetic -- only its stored pattern differs.
template <bool SCALED, bool CANON = false> struct FastRT {
  static constexpr bool kFast = !(SCALED && CANON);
  static constexpr bool kCanon = CANON;
  // v_cvt_pk_bf16_f32 with 0 as its first source leaves bf16(x) in the upper half of the result and
  // bf16(0) = 0 in the lower half: that IS the rounded value widened back to fp32, in one instruction.
  static __device__ __forceinline__ float rnd1(float x) {
    const f32x2_t v = {0.0f, x};
    const bf16x2_t r = __builtin_convertvector(v, bf16x2_t);      // v_cvt_pk_bf16_f32 dst, 0, x
    return __builtin_bit_cast(float, r);
  }
  static __device__ __forceinline__ P2 rnd(P2 x) { return {rnd1(x.lo), rnd1(x.hi)}; }
  // a / b where b is a positive normal scalar with known fp32 reciprocal rb (|rel err| <= 2^-24)
  static __device__ __forceinline__ float div1(float a, float, float rb, bool &) { return a * rb; }
  // a / b, b any value whose magnitude is 0, infinite or within [2^-126, 2^126]
  static __device__ __forceinline__ float divg1(float a, float b, bool &) { return a * __builtin_amdgcn_rcpf(b); }
  static __device__ __forceinline__ float sqrt1(float a, bool &redo) {
    if constexpr (SCALED) {
      const bool tiny = a < 0x1p-96f;          // every subnormal operand, and whatever else is cheap to include
      const float r = __builtin_amdgcn_sqrtf(a * (tiny ? 0x1p64f : 1.0f));
      return r * (tiny ? 0x1p-32f : 1.0f);
    } else {
      redo |= is_subnormal(a);
      return __builtin_amdgcn_sqrtf(a);
    }
  }
};

// The bf16 operations on pairs, held widened.  Every function is one F(.): one fp32 operation
// per element, then one rounding.
template <class R> struct Bf {
  using T = P2;        // a pair of elements
  using S = float;     // a wave-uniform scalar
  static constexpr bool kFast = R::kFast;      // may raise redo
  static constexpr bool kHalf = false;
  static constexpr bool kGuarded = R::kFast;   // the reciprocal route needs its divisor checked for range (single operations)
  static constexpr bool kNanOnWords = false;
  static constexpr int kBytes = 2;             // bytes per stored element
  using Rcp = float;   // reciprocal of a scalar
  static __device__ __forceinline__ T unpack(uint32_t w) { return widen2(w); }
  static __device__ __forceinline__ uint32_t pack(T x) {
    const uint32_t w = pack2(x);
    if constexpr (!R::kCanon) return w;
    // a half is NaN iff its magnitude bits exceed 0x7F80; +0x007F carries exactly those into bit 15
    const uint32_t nan = (((w & 0x7fff7fffu) + 0x007f007fu) & 0x80008000u) >> 15;      // bit 0 / bit 16
    const uint32_t halves = nan * 0xffffu;
    return (w & ~halves) | (0x7fc07fc0u & halves);
  }
  static __device__ __forceinline__ T zero() { return {0.f, 0.f}; }
  static __device__ __forceinline__ float lo(T x) { return x.lo; }
  static __device__ __forceinline__ float hi(T x) { return x.hi; }
  static __device__ __forceinline__ uint16_t bits_lo(T x) { return (uint16_t)(fbits(x.lo) >> 16); }
  static __device__ __forceinline__ uint16_t bits_hi(T x) { return (uint16_t)(fbits(x.hi) >> 16); }
  static __device__ __forceinline__ bool any_nan(T x) { return is_nan(x.lo) | is_nan(x.hi); }
  static __device__ __forceinline__ T round_f32(float a, float b) { return R::rnd({a, b}); }

  static __device__ __forceinline__ T add(T a, T b) { return R::rnd({a.lo + b.lo, a.hi + b.hi}); }
  static __device__ __forceinline__ T sub(T a, T b) { return R::rnd({a.lo - b.lo, a.hi - b.hi}); }
  static __device__ __forceinline__ T mul(T a, T b) { return R::rnd({a.lo * b.lo, a.hi * b.hi}); }
  static __device__ __forceinline__ T adds(T a, S s) { return R::rnd({a.lo + s, a.hi + s}); }
  static __device__ __forceinline__ T muls(S s, T a) { return R::rnd({s * a.lo, s * a.hi}); }
  // F(s*a - x), product unrounded (the FMA of Alg. 6)
  static __device__ __forceinline__ T fmss(S s, T a, T x) {
    return R::rnd({__builtin_fmaf(s, a.lo, -x.lo), __builtin_fmaf(s, a.hi, -x.hi)});
  }
  static __device__ __forceinline__ T fms(T a, T b, T x) {
    return R::rnd({__builtin_fmaf(a.lo, b.lo, -x.lo), __builtin_fmaf(a.hi, b.hi, -x.hi)});
  }
  static __device__ __forceinline__ T divs(T a, S b, S rb, bool &redo) {
    return R::rnd({R::div1(a.lo, b, rb, redo), R::div1(a.hi, b, rb, redo)});
  }
  static __device__ __forceinline__ T divg(T a, T b, bool &redo) {
    return R::rnd({R::divg1(a.lo, b.lo, redo), R::divg1(a.hi, b.hi, redo)});
  }
  static __device__ __forceinline__ T sqrt(T a, bool &redo) {
    return R::rnd({R::sqrt1(a.lo, redo), R::sqrt1(a.hi, redo)});
  }
};
using Exact = Bf<ExactR>;
using Fast = Bf<FastRT<false>>;          // first pass
using FastSecond = Bf<FastRT<true, true>>;     // second pass: slots whose root met a subnormal operand, slots that hold a NaN, slots at a tensor's ends

// ---- fp16 -------------------------------------------------------------------------------
// The same operation F(a o b) for IEEE binary16 components (App. A Table 7).  The pair stays packed
// in one register.  For +, -, * the hardware's packed fp16 instructions round the exact result
// once to fp16, which equals rounding it first to fp32 and then to fp16 (fp32's 24 bits are at least
// 2*11+2, so the first rounding can never create or destroy a tie of the second).  The fused
// multiply-subtract is only ever used as F(a*b - F(a*b)) (Alg. 6): that difference is exactly
// representable in fp32, so again both routes round the same exact number.  Division and square
// root have no correctly rounded fp16 instruction: they are done per element, widened.  The square
// root is the definition itself (correctly rounded fp32 root, then narrow).  The quotient is
// q' = q + (a - b*q)*r with r = v_rcp_f32(b), q = a*r: the residual a - b*q is exact in one FMA
// (a and b have 11 significant bits, q agrees with a/b to 2^-22), so q' is the fp32 rounding of a
// number within 2^-44 of a/b: it equals a/b whenever that is an fp32 number (so exact fp16 results
// and exact ties survive) and is otherwise within 2^-24(1+2^-20) of it, while a quotient of two
// 11-bit numbers that is not itself a rounding boundary stays more than 2^-23 (relative) away from
// every fp16 rounding boundary, subnormal results and the overflow threshold included.  Zero or
// infinite operands make the residual NaN, and a zero dividend loses its sign in the correction; in
// both cases q is already the IEEE result and is kept.
// NaN: the hardware propagates payloads, the stored format has one NaN (0x7E00).  NaN-ness itself
// propagates the same way in both, so only stored values need fixing: the first pass over a slot
// (kFast) just detects a NaN in its results; the slot is then redone in the mode that replaces every
// NaN it stores by the one NaN.
typedef _Float16 h2_t __attribute__((ext_vector_type(2)));

// Keeps the optimizer from folding widen / fp32 op / narrow into an fp16 operation of its own choice.
__device__ __forceinline__ float opaque(float f) { asm("" : "+v"(f)); return f; }

template <bool HOT> struct Hf {
  using T = h2_t;
  using S = h2_t;      // a scalar is the same value in both halves
  static constexpr bool kFast = HOT;
  static constexpr bool kHalf = true;
  static constexpr bool kGuarded = false;
  static constexpr bool kNanOnWords = false;
  static constexpr int kBytes = 2;
  using Rcp = float;   // unused: fp16 divides by the scalar itself
  static __device__ __forceinline__ T unpack(uint32_t w) { return __builtin_bit_cast(h2_t, w); }
  static __device__ __forceinline__ uint32_t raw(T x) { return __builtin_bit_cast(uint32_t, x); }
  // What is stored: the raw pair on the vector path (which has checked that it holds no NaN), the pair
  // with every NaN replaced by the format's one NaN otherwise.
  static __device__ __forceinline__ uint32_t pack(T x) {
    if (HOT) return raw(x);
    return (uint32_t)canon(raw(x) & 0xffffu) | ((uint32_t)canon(raw(x) >> 16) << 16);
  }
  static __device__ __forceinline__ T zero() { return h2_t{(_Float16)0, (_Float16)0}; }
  static __device__ __forceinline__ float lo(T x) { return (float)x.x; }
  static __device__ __forceinline__ float hi(T x) { return (float)x.y; }
  static __device__ __forceinline__ uint16_t canon(uint32_t h) { return (h & 0x7fffu) > 0x7c00u ? (uint16_t)0x7e00 : (uint16_t)h; }
  static __device__ __forceinline__ uint16_t bits_lo(T x) { return canon(raw(x) & 0xffffu); }
  static __device__ __forceinline__ uint16_t bits_hi(T x) { return canon(raw(x) >> 16); }
  // a half is NaN iff its magnitude bits exceed 0x7C00; +0x03FF carries exactly those into bit 15
  static __device__ __forceinline__ bool any_nan(T x) { return (((raw(x) & 0x7fff7fffu) + 0x03ff03ffu) & 0x80008000u) != 0; }
  static __device__ __forceinline__ T round_f32(float a, float b) { return h2_t{(_Float16)a, (_Float16)b}; }

  static __device__ __forceinline__ T add(T a, T b) { return a + b; }
  static __device__ __forceinline__ T sub(T a, T b) { return a - b; }
  static __device__ __forceinline__ T mul(T a, T b) { return a * b; }
  static __device__ __forceinline__ T adds(T a, S s) { return a + s; }
  static __device__ __forceinline__ T muls(S s, T a) { return s * a; }
  static __device__ __forceinline__ T fmss(S s, T a, T x) { return __builtin_elementwise_fma(s, a, -x); }
  static __device__ __forceinline__ T fms(T a, T b, T x) { return __builtin_elementwise_fma(a, b, -x); }
  static __device__ __forceinline__ _Float16 div1(_Float16 ah, _Float16 bh) {
    const float a = (float)ah, b = (float)bh;
    const float r = __builtin_amdgcn_rcpf(b);
    const float q = a * r;
    const float res = __builtin_fmaf(-b, q, a);
    const float q1 = __builtin_fmaf(res, r, q);
    return (_Float16)(__builtin_fabsf(q1) > 0.0f ? q1 : q);     // NaN or zero: keep q (a zero quotient keeps a's sign there)
  }
  static __device__ __forceinline__ T divs(T a, S b, float, bool &) { return h2_t{div1(a.x, b.x), div1(a.y, b.y)}; }
  static __device__ __forceinline__ T divg(T a, T b, bool &) { return h2_t{div1(a.x, b.x), div1(a.y, b.y)}; }
  static __device__ __forceinline__ T sqrt(T a, bool &) {
    return h2_t{(_Float16)__builtin_sqrtf(opaque((float)a.x)), (_Float16)__builtin_sqrtf(opaque((float)a.y))};
  }
};
using HalfHot = Hf<true>;
using HalfCold = Hf<false>;

// ---- FP8 --------------------------------------------------------------------------------
// The two 8-bit formats of App. A Table 7 (the 8-bit extension named in Sec. 7): E5M2, IEEE-style
// with infinities, and E4M3 without infinities (largest 448, only S.1111.111 is NaN, whatever rounds
// beyond 448 becomes NaN).  gfx950 converts to and from both in hardware, round to nearest even,
// non-saturating, which is exactly that reading: from fp32 (v_cvt_pk_{bf8,fp8}_f32, checked against the
// definition over all 2^32 inputs by the test suite) and from fp16 (v_cvt_scalef32_pk_{bf8,fp8}_f16 with
// scale 1, equal to the definition on all 2^16 fp16 inputs).
//
// Every FP8 number is an fp16 number, so a pair is held as packed fp16 and +, -, * and the FMA of Alg. 6
// are the packed fp16 instructions followed by the conversion to the 8-bit format and back: three
// instructions per pair.  That is F(a o b): the fp16 instruction rounds the exact result to 11 bits, and
// rounding that again to 3 or 4 bits gives what rounding the exact result (or its fp32 rounding) once
// would, since 11 >= 2*4+2; where fp16 itself runs out, the results agree too -- sums and differences
// of FP8 numbers and products of E4M3 numbers are fp16 numbers exactly; an E5M2 product below fp16's
// grid (2^-24) is below 2^-19 and rounds to zero either way; whatever overflows fp16 (65520 and up) is
// beyond both formats' ranges.  For the FMA, a*b - F(a*b) is an fp16 number whenever a*b >= 2^-17, and
// rounds to zero either way below.
//
// A pair also carries the two 8-bit patterns it was decoded from (every rounding produces them on the
// way): packing a result is then one byte permute, and the fp32 operations below widen from the
// patterns, one instruction per pair.
//
// Quotient: fl32(a * r), r = v_rcp_f32(b), rounded to fp16 and then to the format.  A quotient of two
// 3- or 4-bit significands that is an exact tie of the 8-bit rounding is an fp16 number, and a*r lies
// within 2^-22 of it, so the fp16 rounding lands on it and the tie is seen as a tie; every other
// quotient is further than 2^-9 (relative; 2^-22 absolute among E5M2's subnormal results) from the
// nearest rounding boundary and cannot cross it.  a * inf, a * 0 and their NaN cases are IEEE's a / 0
// and a / inf.  Checked on the CPU against the definition for all 256 x 256 operands with r anywhere
// within two units in the last place of 1/b, and on the GPU for all of them.
// Quotient by a scalar b: one packed fp16 multiplication by RN16(1/b), then the conversion: right for
// every a and b (checked the same way) except E5M2's b = +-2^-16, whose reciprocal is not an fp16 number; the
// host sends such a step straight to the second arithmetic pass, whose mode divides by b as above.
// Root: v_sqrt_f32, then one conversion from fp32 (a root of a 3- or 4-bit number is either exact or
// further than 2^-12 from any boundary; checked on every input).
// NaN: as for fp16, the first pass detects, the redo stores the format's one NaN (0x7E, 0x7F).
typedef short s16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

template <bool E4M3> struct F8Cvt {
  // two fp32 -> two 8-bit patterns in the low half of the result (the other half comes from `old`)
  static __device__ __forceinline__ uint32_t enc_f32(float a, float b, uint32_t old) {
    if constexpr (E4M3) return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)old, false);
    else return (uint32_t)__builtin_amdgcn_cvt_pk_bf8_f32(a, b, (int)old, false);
  }
  // packed fp16 pair -> two 8-bit patterns in the low half of the result
  static __device__ __forceinline__ uint32_t enc(h2_t x, uint32_t old) {
    const s16x2_t o = __builtin_bit_cast(s16x2_t, old);
    if constexpr (E4M3) return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_fp8_f16(o, x, 1.0f, false));
    else return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf8_f16(o, x, 1.0f, false));
  }
  // the two 8-bit patterns in the low or high half of w -> packed fp16 pair (exact)
  template <bool HIGH> static __device__ __forceinline__ h2_t dec(uint32_t w) {
    if constexpr (E4M3) return __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, HIGH);
    else return __builtin_amdgcn_cvt_scalef32_pk_f16_bf8(w, 1.0f, HIGH);
  }
  // the two 8-bit patterns in the low half of w -> two fp32 (exact)
  static __device__ __forceinline__ f32x2_t dec_f32(uint32_t w) {
    if constexpr (E4M3) return __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
    else return __builtin_amdgcn_cvt_pk_f32_bf8((int)w, false);
  }
  static __device__ __forceinline__ uint32_t canon(uint32_t b) {      // one 8-bit pattern
    if constexpr (E4M3) return (b & 0x7fu) == 0x7fu ? 0x7fu : b;
    else return (b & 0x7fu) > 0x7cu ? 0x7eu : b;
  }
  // Adding this to the magnitude bits of a pattern carries into bit 7 exactly for the NaN patterns.
  static constexpr uint32_t kNanCarry = E4M3 ? 0x01u : 0x03u;
};

struct F8Pair {
  h2_t h;         // the two values
  uint32_t e;     // their 8-bit patterns in bits 0-15; bits 16-31 are not meaningful
};

template <bool E4M3, bool HOT> struct F8 {
  using C = F8Cvt<E4M3>;
  using T = F8Pair;
  using S = h2_t;      // a scalar is the same fp16 value in both halves
  using Rcp = h2_t;    // reciprocal of a scalar, likewise
  static constexpr bool kFast = HOT;       // may raise redo (NaN among the results)
  static constexpr bool kHalf = false;
  static constexpr bool kGuarded = false;
  static constexpr bool kNanOnWords = true;      // the step looks for NaN in the packed result words instead of per pair
  static constexpr int kBytes = 1;
  static __device__ __forceinline__ uint32_t raw(h2_t x) { return __builtin_bit_cast(uint32_t, x); }
  // pair PAIR (0 or 1) of the four elements in a dword
  template <int PAIR> static __device__ __forceinline__ T unpack(uint32_t w) { return T{C::template dec<PAIR == 1>(w), PAIR == 1 ? w >> 16 : w}; }
  static __device__ __forceinline__ T unpack(uint32_t w) { return unpack<0>(w); }
  static __device__ __forceinline__ uint32_t pack(T a, T b) {          // four elements -> one dword
    const uint32_t w = __builtin_amdgcn_perm(b.e, a.e, 0x05040100u);   // a's two low bytes, then b's
    if (HOT) return w;
    return C::canon(w & 0xffu) | (C::canon((w >> 8) & 0xffu) << 8) | (C::canon((w >> 16) & 0xffu) << 16) | (C::canon(w >> 24) << 24);
  }
  static __device__ __forceinline__ T zero() { return T{h2_t{(_Float16)0, (_Float16)0}, 0u}; }
  static __device__ __forceinline__ float lo(T x) { return (float)x.h.x; }
  static __device__ __forceinline__ float hi(T x) { return (float)x.h.y; }
  static __device__ __forceinline__ uint16_t bits_lo(T x) { return (uint16_t)C::canon(x.e & 0xffu); }
  static __device__ __forceinline__ uint16_t bits_hi(T x) { return (uint16_t)C::canon((x.e >> 8) & 0xffu); }
  static __device__ __forceinline__ bool any_nan(T x) { return (((x.e & 0x7f7fu) + C::kNanCarry * 0x0101u) & 0x8080u) != 0; }
  static __device__ __forceinline__ bool word_has_nan(uint32_t w) { return (((w & 0x7f7f7f7fu) + C::kNanCarry * 0x01010101u) & 0x80808080u) != 0; }
  // The conversion writes one half of its destination and keeps the other half from `old`.  Only the
  // written half is read back, so `old` is given a value that dies here (the unrounded x) and the
  // destination can take over its register; a constant would cost a move per rounding.
  static __device__ __forceinline__ T rnd(h2_t x, uint32_t old) { const uint32_t e = C::enc(x, old); return T{C::template dec<false>(e), e}; }
  static __device__ __forceinline__ T rnd(h2_t x) { return rnd(x, raw(x)); }
  static __device__ __forceinline__ T rnd_f32(float a, float b) { const uint32_t e = C::enc_f32(a, b, fbits(a)); return T{C::template dec<false>(e), e}; }
  static __device__ __forceinline__ T round_f32(float a, float b) { return rnd_f32(a, b); }

  static __device__ __forceinline__ T add(T a, T b) { return rnd(a.h + b.h); }
  static __device__ __forceinline__ T sub(T a, T b) { return rnd(a.h - b.h); }
  static __device__ __forceinline__ T mul(T a, T b) { return rnd(a.h * b.h); }
  static __device__ __forceinline__ T adds(T a, S s) { return rnd(a.h + s); }
  static __device__ __forceinline__ T muls(S s, T a) { return rnd(s * a.h); }
  static __device__ __forceinline__ T fmss(S s, T a, T x) { return rnd(__builtin_elementwise_fma(s, a.h, -x.h)); }
  static __device__ __forceinline__ T fms(T a, T b, T x) { return rnd(__builtin_elementwise_fma(a.h, b.h, -x.h)); }
  static __device__ __forceinline__ T quotient(f32x2_t a, float blo, float bhi) {
    const float qlo = a.x * __builtin_amdgcn_rcpf(blo), qhi = a.y * __builtin_amdgcn_rcpf(bhi);
    return rnd(h2_t{(_Float16)qlo, (_Float16)qhi}, fbits(qlo));
  }
  static __device__ __forceinline__ T divs(T a, S b, Rcp rb, bool &) {
    if (HOT) return rnd(a.h * rb);
    return quotient(C::dec_f32(a.e), (float)b.x, (float)b.y);
  }
  static __device__ __forceinline__ T divg(T a, T b, bool &) {
    const f32x2_t fb = C::dec_f32(b.e);
    return quotient(C::dec_f32(a.e), fb.x, fb.y);
  }
  static __device__ __forceinline__ T sqrt(T a, bool &) {
    const f32x2_t fa = C::dec_f32(a.e);
    return rnd_f32(__builtin_amdgcn_sqrtf(fa.x), __builtin_amdgcn_sqrtf(fa.y));
  }
};

// The expansion algorithms over any of the modes above.
template <class M> struct Ops : M {
  using T = typename M::T;
  using M::add;
  using M::sub;
  // Thm 4.1: (x, y) = Fast2Sum(a, b)
  static __device__ __forceinline__ void fast2sum(T a, T b, T &x, T &y) {
    x = add(a, b);
    y = sub(b, sub(x, a));
  }
  // Alg. 3
  static __device__ __forceinline__ void two_sum(T a, T b, T &x, T &y) {
    x = add(a, b);
    T bv = sub(x, a);
    T av = sub(x, bv);
    T br = sub(b, bv);
    T ar = sub(a, av);
    y = add(ar, br);
  }
  // Alg. 1: (x, y) <- Grow((x, y), a)
  static __device__ __forceinline__ void grow(T x, T y, T a, T &xo, T &yo) {
    T u, w;
    fast2sum(x, a, u, w);
    fast2sum(u, add(y, w), xo, yo);
  }
  // Alg. 1 on TwoSum (Alg. 3): no |x| >= |a| precondition
  static __device__ __forceinline__ void grow2(T x, T y, T a, T &xo, T &yo) {
    T u, w;
    two_sum(x, a, u, w);
    two_sum(u, add(y, w), xo, yo);
  }
};

// Scalars of one step in the mode's scalar type (bf16 values widened to fp32, or fp16 values in both
// halves of a packed register), plus reciprocals of the two bias corrections for the modes that
// multiply by them.
template <class S, class Rcp> struct StepScalarsT {
  S b1, c1, b2, b2l, c2, bc1, bc2, e, lam, na;
  Rcp rbc1, rbc2;                // 1/bc1, 1/bc2 rounded to Rcp: the bf16 Fast mode and the FP8 first pass multiply by them
  uint32_t eps_inside_sqrt;      // 1: line 12's denominator is F(sqrt(F(v_hat + eps))), as Alg. 2 prints it
  uint32_t elementwise;          // 1: every slot of this launch goes straight to the second arithmetic mode
  uint32_t head_sleep, tail_sleep;   // launch pacing: s_sleep units a wave idles before its first load / after its last store
  uint32_t write_through;        // 1: the set is far larger than the caches, and the kernel marks its stores to be written through
};
using StepScalars = StepScalarsT<float, float>;      // bf16
using StepScalarsH = StepScalarsT<h2_t, float>;      // fp16
using StepScalarsF8 = StepScalarsT<h2_t, h2_t>;      // FP8

template <class T> struct ElemIOT {          // one pair of elements of every stream
  T th, dth, m, v, dv, g;
};

// Variants of the step.  Light and plus are Collage (Sec. 4.2); the other two are the paper's
// comparison strategies built on the same chain: plain bf16 (option A: line 13 is Eq. 1,
// theta <- F(theta + delta)) and Kahan-compensated bf16 (App. B; dtheta holds the Kahan variable).
// V_SGD is MCF-SGD with momentum (Sec. 1): m <- mu*m + g, delta <- -alpha*(m + lambda*theta), Grow.
enum : int { V_LIGHT = 0, V_PLUS = 1, V_BF16 = 2, V_KAHAN = 3, V_SGD = 4 };

// Alg. 2 lines 8-13 on one pair.  GROW2 builds every Grow on TwoSum, EPS_INSIDE puts epsilon under the root.  On return io holds the new theta, dtheta, m, v (and dv);
// delta receives line 12's update.  redo is raised (modes with kFast) when this pair must be
// recomputed in the second-pass mode.
template <class M, int VARIANT, bool GROW2 = false, bool EPS_INSIDE = false>
__device__ __forceinline__ void adamw_pair(ElemIOT<typename M::T> &io, const StepScalarsT<typename M::S, typename M::Rcp> &s,
                                           typename M::T &delta, bool &redo) {
  using O = Ops<M>;
  using T = typename M::T;
  if (VARIANT == V_SGD) {
    const T m1 = O::add(O::muls(s.b1, io.m), io.g);            // s.b1 = momentum coefficient
    delta = O::muls(s.na, O::add(m1, O::muls(s.lam, io.th)));
    T th1, dth1;
    O::grow(io.th, io.dth, delta, th1, dth1);
    if (M::kFast && !M::kNanOnWords) redo |= M::any_nan(th1) | M::any_nan(dth1);
    io.th = th1;
    io.dth = dth1;
    io.m = m1;
    return;
  }
  // line 8
  T m1 = O::add(O::muls(s.b1, io.m), O::muls(s.c1, io.g));
  // line 9
  T inc = O::muls(s.c2, O::mul(io.g, io.g));
  T v1, dv1 = M::zero();
  if (VARIANT != V_PLUS) {
    v1 = O::add(O::muls(s.b2, io.v), inc);
  } else {
    // Mul((b2, b2l), (v, dv)), Alg. 8 with TwoProdFMA (Alg. 6)
    T x = O::muls(s.b2, io.v);
    T ex = O::fmss(s.b2, io.v, x);
    T cross = O::add(O::muls(s.b2, io.dv), O::muls(s.b2l, io.v));
    T e2 = O::add(ex, cross);
    T X, E;
    O::fast2sum(x, e2, X, E);
    if (GROW2) O::grow2(X, E, inc, v1, dv1); else O::grow(X, E, inc, v1, dv1);
  }
  // lines 10-11
  T mh = O::divs(m1, s.bc1, s.rbc1, redo);
  T vh = O::divs(v1, s.bc2, s.rbc2, redo);
  // line 12 (epsilon outside the root unless the caller asked for the printed form; weight decay
  // inside the summed update)
  T dn;
  if (EPS_INSIDE) {
    dn = O::sqrt(O::adds(vh, s.e), redo);
  } else {
    dn = O::adds(O::sqrt(vh, redo), s.e);
  }
  T q = O::divg(mh, dn, redo);
  T w = O::muls(s.lam, io.th);
  delta = O::muls(s.na, O::add(q, w));
  // line 13
  T th1, dth1 = M::zero();
  if (VARIANT == V_BF16) {
    th1 = O::add(io.th, delta);                       // Eq. 1
  } else if (VARIANT == V_KAHAN) {
    const T u = O::add(delta, io.dth);                // compensate the update with the Kahan variable
    O::fast2sum(io.th, u, th1, dth1);                 // c <- F(u - F(theta' - theta))
  } else if (GROW2) {
    O::grow2(io.th, io.dth, delta, th1, dth1);
  } else {
    O::grow(io.th, io.dth, delta, th1, dth1);
  }
  if (M::kFast && !M::kNanOnWords) {
    // Any NaN produced or consumed above reaches theta' or dtheta' (or dv'): m' and v' feed
    // the quotient, the quotient feeds delta, delta feeds theta'.  (Modes with kNanOnWords leave this
    // check to the caller, on the packed words of the same three results.)
    redo |= M::any_nan(th1) | M::any_nan(dth1);
    if (VARIANT == V_PLUS) redo |= M::any_nan(dv1);
  }
  io.th = th1;
  io.dth = dth1;
  io.m = m1;
  io.v = v1;
  io.dv = dv1;
}

}  // namespace mcfd
