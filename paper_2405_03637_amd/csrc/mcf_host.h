// Host-side preparation for the Collage step: argument checks and the bf16 (or fp16) scalars of
// Alg. 2 (computed in fp64 and cast once, App. D "Scalar and Bias Correction").
#pragma once
#include <stdint.h>

#include <cmath>
#include <cstring>

#include "../../include/mcf.h"
#include "mcf_math.h"

namespace mcfh {

// fp64 -> bf16 with a single round-to-nearest-even, working on the double's fields:
// the 53-bit significand is shifted right so that 8 bits (fewer in the subnormal range)
// remain, and the discarded bits decide the rounding.
inline uint16_t f64_to_bf16(double x) {
  uint64_t u;
  std::memcpy(&u, &x, 8);
  const uint16_t sign = (uint16_t)((u >> 48) & 0x8000u);
  const int ef = (int)((u >> 52) & 0x7ff);
  const uint64_t frac = u & ((1ull << 52) - 1);
  if (ef == 0x7ff) return frac ? (uint16_t)0x7fc0 : (uint16_t)(sign | 0x7f80);
  if (ef == 0) return sign;                        // below 2^-1022: rounds to zero
  const int e = ef - 1023;                         // value = sig * 2^(e-52)
  const uint64_t sig = frac | (1ull << 52);
  int shift = 45;                                  // normal: keep 8 of the 53 bits
  if (e < -126) shift += -126 - e;                 // subnormal: coarser fixed spacing 2^-133
  if (shift > 54) return sign;                     // less than a quarter of the least subnormal
  const uint64_t q = sig >> shift;
  const uint64_t rem = sig & ((1ull << shift) - 1);
  const uint64_t half = 1ull << (shift - 1);
  const uint64_t up = (rem > half || (rem == half && (q & 1))) ? 1 : 0;
  uint32_t bits;
  if (e >= -126) {
    bits = (uint32_t)((e + 127) << 7) + (uint32_t)(q + up - 128);   // a carry moves into the exponent
    if (bits >= 0x7f80u) bits = 0x7f80u;
  } else {
    bits = (uint32_t)(q + up);
  }
  return (uint16_t)(sign | bits);
}

inline float bf16_to_f32(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

// fp64 -> fp16 (IEEE binary16) with a single round-to-nearest-even, the same way: 11 of the 53
// bits remain (fewer in the subnormal range, fixed spacing 2^-24); every NaN becomes 0x7E00.
inline uint16_t f64_to_f16(double x) {
  uint64_t u;
  std::memcpy(&u, &x, 8);
  const uint16_t sign = (uint16_t)((u >> 48) & 0x8000u);
  const int ef = (int)((u >> 52) & 0x7ff);
  const uint64_t frac = u & ((1ull << 52) - 1);
  if (ef == 0x7ff) return frac ? (uint16_t)0x7e00 : (uint16_t)(sign | 0x7c00);
  if (ef == 0) return sign;
  const int e = ef - 1023;
  const uint64_t sig = frac | (1ull << 52);
  int shift = 42;                                  // normal: keep 11 of the 53 bits
  if (e < -14) shift += -14 - e;
  if (shift > 54) return sign;                     // less than a quarter of the least subnormal
  const uint64_t q = sig >> shift;
  const uint64_t rem = sig & ((1ull << shift) - 1);
  const uint64_t half = 1ull << (shift - 1);
  const uint64_t up = (rem > half || (rem == half && (q & 1))) ? 1 : 0;
  uint32_t bits;
  if (e >= -14) {
    bits = (uint32_t)((e + 15) << 10) + (uint32_t)(q + up - 1024);   // a carry moves into the exponent
    if (bits >= 0x7c00u) bits = 0x7c00u;
  } else {
    bits = (uint32_t)(q + up);
  }
  return (uint16_t)(sign | bits);
}

// Exact value of a finite fp16 pattern as a double.
inline double f16_to_f64(uint16_t h) {
  const int e = (h >> 10) & 0x1f, m = h & 0x3ff;
  const double mag = e == 0 ? std::ldexp((double)m, -24) : std::ldexp((double)(1024 + m), e - 25);
  return (h & 0x8000) ? -mag : mag;
}

// fp64 -> FP8 with a single round-to-nearest-even on the double's fields.  E5M2 (bias 15) is
// IEEE-style: overflow gives infinity, NaN is 0x7E.  E4M3 (bias 7) has no infinities: its largest
// number is 448 = 0x7E and whatever rounds beyond it, infinities included, becomes NaN = 0x7F.
template <int MBITS, int EMIN>
inline bool f64_to_small(double x, uint32_t &magnitude_bits, uint16_t &sign) {      // false: x is NaN
  uint64_t u;
  std::memcpy(&u, &x, 8);
  sign = (uint16_t)((u >> 56) & 0x80u);
  const int ef = (int)((u >> 52) & 0x7ff);
  const uint64_t frac = u & ((1ull << 52) - 1);
  if (ef == 0x7ff) { magnitude_bits = 0xffffffffu; return frac == 0; }     // infinity: "beyond everything"
  if (ef == 0) { magnitude_bits = 0; return true; }
  const int e = ef - 1023;
  if (e > 40) { magnitude_bits = 0xffffffffu; return true; }
  const uint64_t sig = frac | (1ull << 52);
  int shift = 52 - MBITS;
  if (e < EMIN) shift += EMIN - e;
  if (shift > 54) { magnitude_bits = 0; return true; }
  const uint64_t q = sig >> shift;
  const uint64_t rem = sig & ((1ull << shift) - 1);
  const uint64_t half = 1ull << (shift - 1);
  const uint64_t up = (rem > half || (rem == half && (q & 1))) ? 1 : 0;
  if (e >= EMIN) magnitude_bits = (uint32_t)((e - EMIN + 1) << MBITS) + (uint32_t)(q + up - (1u << MBITS));
  else magnitude_bits = (uint32_t)(q + up);
  return true;
}

inline uint16_t f64_to_e5m2(double x) {
  uint32_t mag; uint16_t sign;
  if (!f64_to_small<2, -14>(x, mag, sign)) return 0x7e;
  if (mag >= 0x7c) mag = 0x7c;
  return (uint16_t)(sign | mag);
}

inline uint16_t f64_to_e4m3(double x) {
  uint32_t mag; uint16_t sign;
  if (!f64_to_small<3, -6>(x, mag, sign)) return 0x7f;
  if (mag >= 0x7f) return 0x7f;
  return (uint16_t)(sign | mag);
}

inline double e5m2_to_f64(uint16_t h) { return f16_to_f64((uint16_t)((h & 0xff) << 8)); }     // finite patterns only
inline double e4m3_to_f64(uint16_t h) {
  const int e = (h >> 3) & 0xf, m = h & 7;
  const double mag = e == 0 ? std::ldexp((double)m, -9) : std::ldexp((double)(8 + m), e - 10);
  return (h & 0x80) ? -mag : mag;
}

inline int check_hyper(const mcf_hyper *h, uint64_t step) {
  if (!h) return MCF_ERR_NULL;
  if (step < 1) return MCF_ERR_STEP;
  const double v[5] = {h->lr, h->beta1, h->beta2, h->eps, h->weight_decay};
  for (double x : v)
    if (!std::isfinite(x)) return MCF_ERR_HYPER;
  if (h->lr < 0 || h->eps < 0 || h->weight_decay < 0) return MCF_ERR_HYPER;
  if (h->beta1 < 0 || h->beta1 >= 1 || h->beta2 < 0 || h->beta2 >= 1) return MCF_ERR_HYPER;
  return MCF_OK;
}

// The ten scalars of one step as 16-bit patterns of the component format, in the order of
// mcf_step_scalars(): beta1, 1-beta1, beta2 (first component), beta2's second component, 1-beta2,
// 1-beta1^t, 1-beta2^t, eps, lambda, -alpha.  Each is computed in fp64 and cast once.
enum { K_B1, K_C1, K_B2, K_B2L, K_C2, K_BC1, K_BC2, K_EPS, K_LAM, K_NA, K_COUNT };
struct ScalarBits { uint16_t v[K_COUNT]; };

template <uint16_t (*TO16)(double), double (*TO64)(uint16_t)>
inline ScalarBits derive_bits(const mcf_hyper &h, uint64_t step) {
  const double t = (double)step;
  ScalarBits s;
  s.v[K_B1] = TO16(h.beta1);
  s.v[K_C1] = TO16(1.0 - h.beta1);
  s.v[K_B2] = TO16(h.beta2);
  s.v[K_B2L] = TO16(h.beta2 - TO64(s.v[K_B2]));
  s.v[K_C2] = TO16(1.0 - h.beta2);
  s.v[K_BC1] = TO16(1.0 - std::pow(h.beta1, t));
  s.v[K_BC2] = TO16(1.0 - std::pow(h.beta2, t));
  s.v[K_EPS] = TO16(h.eps);
  s.v[K_LAM] = TO16(h.weight_decay);
  s.v[K_NA] = TO16(-h.lr);
  return s;
}

inline double bf16_to_f64(uint16_t h) { return (double)bf16_to_f32(h); }
inline ScalarBits scalar_bits_bf16(const mcf_hyper &h, uint64_t step) { return derive_bits<f64_to_bf16, bf16_to_f64>(h, step); }
inline ScalarBits scalar_bits_fp16(const mcf_hyper &h, uint64_t step) { return derive_bits<f64_to_f16, f16_to_f64>(h, step); }
inline ScalarBits scalar_bits_e5m2(const mcf_hyper &h, uint64_t step) { return derive_bits<f64_to_e5m2, e5m2_to_f64>(h, step); }
inline ScalarBits scalar_bits_e4m3(const mcf_hyper &h, uint64_t step) { return derive_bits<f64_to_e4m3, e4m3_to_f64>(h, step); }

// Returns the scalars and whether the Fast arithmetic mode may be used with them: the two
// bias corrections must be numbers in [2^-60, 1] (their fp32 reciprocals are then normal and correctly
// rounded) and epsilon zero or a normal number of sane size (so that sqrt(v)+eps is zero, or
// normal with a normal reciprocal).
inline bool derive_scalars(const mcf_hyper &h, uint64_t step, mcfd::StepScalars &s) {
  const ScalarBits b = scalar_bits_bf16(h, step);
  s.b1 = bf16_to_f32(b.v[K_B1]);
  s.c1 = bf16_to_f32(b.v[K_C1]);
  s.b2 = bf16_to_f32(b.v[K_B2]);
  s.b2l = bf16_to_f32(b.v[K_B2L]);
  s.c2 = bf16_to_f32(b.v[K_C2]);
  s.bc1 = bf16_to_f32(b.v[K_BC1]);
  s.bc2 = bf16_to_f32(b.v[K_BC2]);
  s.rbc1 = (float)(1.0 / (double)s.bc1);
  s.rbc2 = (float)(1.0 / (double)s.bc2);
  s.e = bf16_to_f32(b.v[K_EPS]);
  s.lam = bf16_to_f32(b.v[K_LAM]);
  s.na = bf16_to_f32(b.v[K_NA]);
  s.eps_inside_sqrt = s.elementwise = s.head_sleep = s.tail_sleep = s.write_through = 0;
  auto sane_bc = [](float x) { return x >= 0x1p-60f && x <= 1.0f; };
  const bool eps_ok = (s.e == 0.0f) || (s.e >= 0x1p-100f && s.e <= 0x1p60f);
  return sane_bc(s.bc1) && sane_bc(s.bc2) && eps_ok;
}

// The same scalars as fp16 patterns, each copied into both halves of a packed register.  The fp16
// arithmetic has no restricted mode, so there is nothing to report.
inline void derive_scalars_fp16(const mcf_hyper &h, uint64_t step, mcfd::StepScalarsH &s) {
  const ScalarBits b = scalar_bits_fp16(h, step);
  auto splat = [](uint16_t x) { return __builtin_bit_cast(mcfd::h2_t, (uint32_t)x * 0x00010001u); };
  s.b1 = splat(b.v[K_B1]);
  s.c1 = splat(b.v[K_C1]);
  s.b2 = splat(b.v[K_B2]);
  s.b2l = splat(b.v[K_B2L]);
  s.c2 = splat(b.v[K_C2]);
  s.bc1 = splat(b.v[K_BC1]);
  s.bc2 = splat(b.v[K_BC2]);
  s.rbc1 = s.rbc2 = 0.0f;    // unused by the fp16 arithmetic
  s.e = splat(b.v[K_EPS]);
  s.lam = splat(b.v[K_LAM]);
  s.na = splat(b.v[K_NA]);
  s.eps_inside_sqrt = s.elementwise = s.head_sleep = s.tail_sleep = s.write_through = 0;
}

// FP8 scalars as fp16 values (every FP8 number is one; infinities and NaN carry over: a scalar that
// left the format's range poisons the step exactly as it does in the definition), each copied into both
// halves of a packed register, with the fp16 roundings of the reciprocals of the two bias corrections.
// Returns false when one of those reciprocals is not an fp16 number (E5M2's +-2^-16): the first pass
// multiplies by them, so such a step must take the second arithmetic pass (the caller sets `elementwise`).
inline bool derive_scalars_fp8(const mcf_hyper &h, uint64_t step, bool e4m3, mcfd::StepScalarsF8 &s) {
  const ScalarBits b = e4m3 ? scalar_bits_e4m3(h, step) : scalar_bits_e5m2(h, step);
  auto half_bits = [e4m3](uint16_t x) -> uint16_t {
    if (!e4m3) return (uint16_t)((x & 0xff) << 8);                        // E5M2 is the upper byte of an fp16
    if ((x & 0x7f) == 0x7f) return 0x7e00;                                // NaN
    return f64_to_f16(e4m3_to_f64(x));                                    // exact
  };
  auto splat16 = [](uint16_t hb) { return __builtin_bit_cast(mcfd::h2_t, (uint32_t)hb * 0x00010001u); };
  auto splat = [&](uint16_t x) { return splat16(half_bits(x)); };
  bool ok = true;
  auto reciprocal = [&](uint16_t x) {
    const uint16_t hb = half_bits(x);
    const uint16_t sign = hb & 0x8000, mag = hb & 0x7fff;
    if (mag > 0x7c00) return splat16(0x7e00);                             // NaN
    if (mag == 0x7c00) return splat16(sign);                              // 1/inf = 0
    if (mag == 0) return splat16(sign | 0x7c00);                          // a * inf is the IEEE result of a / 0
    const double r = 1.0 / f16_to_f64(hb);
    if (std::fabs(r) > 65504.0) ok = false;
    return splat16(f64_to_f16(r));
  };
  s.b1 = splat(b.v[K_B1]);
  s.c1 = splat(b.v[K_C1]);
  s.b2 = splat(b.v[K_B2]);
  s.b2l = splat(b.v[K_B2L]);
  s.c2 = splat(b.v[K_C2]);
  s.bc1 = splat(b.v[K_BC1]);
  s.bc2 = splat(b.v[K_BC2]);
  s.rbc1 = reciprocal(b.v[K_BC1]);
  s.rbc2 = reciprocal(b.v[K_BC2]);
  s.e = splat(b.v[K_EPS]);
  s.lam = splat(b.v[K_LAM]);
  s.na = splat(b.v[K_NA]);
  s.eps_inside_sqrt = s.elementwise = s.head_sleep = s.tail_sleep = s.write_through = 0;
  return ok;
}

}  // namespace mcfh
