"""Mutation check of the oracle's pins.  CPU only; not collected by pytest (run it by hand:
`python tests/oracle_mutants.py`, about half an hour on 8 cores; `ONLY=name,name` picks mutants, extra
arguments go to pytest).

One plausible mistake at a time is planted in a COPY of oracle/mcf_oracle.cpp -- a swapped operand, a
dropped term, a flag that is accepted and ignored, an association read differently, a double rounding, a
wrong special value -- the copy is compiled, and the `not gpu` test suite is run against it.  A mistake the
suite does not notice is reported as SURVIVED: either the two versions compute the same thing on every
input that matters (listed at the bottom, with the reason), or a pin is missing.  Nothing here touches the GPU, the
HIP library or the real oracle; the copies live in a temporary directory and are deleted.
"""
import concurrent.futures as cf
import os
import shutil
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = open(os.path.join(ROOT, "oracle", "mcf_oracle.cpp")).read()

# (name, text in the oracle's source -- must occur exactly once --, replacement)
MUTANTS = [
 ("f2s_wrong_inner", "uint16_t y = sub(b, sub(x, a));\n    return {x, y};\n  }\n\n  /* Alg. 3 */", "uint16_t y = sub(b, sub(x, b));\n    return {x, y};\n  }\n\n  /* Alg. 3 */"),
 ("f2s_roles_swapped", "uint16_t y = sub(b, sub(x, a));\n    return {x, y};\n  }\n\n  /* Alg. 3 */", "uint16_t y = sub(a, sub(x, b));\n    return {x, y};\n  }\n\n  /* Alg. 3 */"),
 ("twosum_avirtual", "uint16_t a_virtual = sub(x, b_virtual);", "uint16_t a_virtual = sub(x, b);"),
 ("twosum_y_sub", "uint16_t y = add(a_roundoff, b_roundoff);", "uint16_t y = sub(a_roundoff, b_roundoff);"),
 ("twosum_broundoff", "uint16_t b_roundoff = sub(b, b_virtual);", "uint16_t b_roundoff = sub(b_virtual, b);"),
 ("grow_second_uses_hi", "return fast2sum(uv.hi, add(xy.lo, uv.lo));", "return fast2sum(uv.hi, add(xy.lo, uv.hi));"),
 ("grow_first_swapped", "Pair uv = fast2sum(xy.hi, a);", "Pair uv = fast2sum(a, xy.hi);"),
 ("grow_drops_y", "return fast2sum(uv.hi, add(xy.lo, uv.lo));", "return fast2sum(uv.hi, uv.lo);"),
 ("grow_second_swapped", "return fast2sum(uv.hi, add(xy.lo, uv.lo));", "return fast2sum(add(xy.lo, uv.lo), uv.hi);"),
 ("grow2_second_is_f2s", "return two_sum(uv.hi, add(xy.lo, uv.lo));", "return fast2sum(uv.hi, add(xy.lo, uv.lo));"),
 ("grow2_first_is_f2s", "Pair uv = two_sum(xy.hi, a);", "Pair uv = fast2sum(xy.hi, a);"),
 ("twoprod_no_fma", "uint16_t e = fms(a, b, x);", "uint16_t e = sub(mul(a, b), x);"),
 ("fms_sign", "std::fmaf(Fm::W(a), Fm::W(b), -Fm::W(x))", "std::fmaf(Fm::W(a), Fm::W(b), Fm::W(x))"),
 ("scaling_adds_hi", "uint16_t e = add(mul(a.lo, v), xe.lo);", "uint16_t e = add(mul(a.lo, v), xe.hi);"),
 ("scaling_drops_lo", "uint16_t e = add(mul(a.lo, v), xe.lo);", "uint16_t e = xe.lo;"),
 ("scaling_uses_lo_first", "Pair xe = two_prod_fma(a.hi, v);", "Pair xe = two_prod_fma(a.lo, v);"),
 ("mulx_cross_wrong", "add(mul(a.hi, b.lo), mul(a.lo, b.hi))", "add(mul(a.hi, b.lo), mul(a.lo, b.lo))"),
 ("mulx_no_cross", "uint16_t e = add(xe.lo, cross);", "uint16_t e = xe.lo; (void)cross;"),
 ("mulx_half_cross", "add(mul(a.hi, b.lo), mul(a.lo, b.hi))", "mul(a.hi, b.lo)"),
 ("c1_from_rounded", "s.c1 = Fm::B(1.0 - h.beta1);", "s.c1 = Fm::B(1.0 - (double)Fm::W(s.b1));"),
 ("c2_from_rounded", "s.c2 = Fm::B(1.0 - h.beta2);", "s.c2 = Fm::B(1.0 - (double)Fm::W(s.b2));"),
 ("bc1_from_rounded", "s.bc1 = Fm::B(1.0 - std::pow(h.beta1, td));", "s.bc1 = Fm::B(1.0 - std::pow((double)Fm::W(s.b1), td));"),
 ("bc2_from_rounded", "s.bc2 = Fm::B(1.0 - std::pow(h.beta2, td));", "s.bc2 = Fm::B(1.0 - std::pow((double)Fm::W(s.b2), td));"),
 ("bc_swapped", "s.bc1 = Fm::B(1.0 - std::pow(h.beta1, td));", "s.bc1 = Fm::B(1.0 - std::pow(h.beta2, td));"),
 ("b2l_zero", "s.b2l = Fm::B(h.beta2 - (double)Fm::W(s.b2));", "s.b2l = 0;"),
 ("b2l_sign", "s.b2l = Fm::B(h.beta2 - (double)Fm::W(s.b2));", "s.b2l = Fm::B((double)Fm::W(s.b2) - h.beta2);"),
 ("na_positive", "s.na = Fm::B(-h.lr);", "s.na = Fm::B(h.lr);"),
 ("scalars_via_float", "s.e = Fm::B(h.eps);", "s.e = Fm::R((float)h.eps);"),
 ("inc_assoc", "uint16_t inc = mul(s.c2, mul(g, g));", "uint16_t inc = mul(mul(s.c2, g), g);"),
 ("m_uses_b1_twice", "uint16_t m_new = add(mul(s.b1, m), mul(s.c1, g));", "uint16_t m_new = add(mul(s.b1, m), mul(s.b1, g));"),
 ("v_uses_c1", "uint16_t inc = mul(s.c2, mul(g, g));", "uint16_t inc = mul(s.c1, mul(g, g));"),
 ("mhat_bc2", "uint16_t m_hat = div(m_new, s.bc1);", "uint16_t m_hat = div(m_new, s.bc2);"),
 ("vhat_old_v", "uint16_t v_hat = div(v_new, s.bc2);", "uint16_t v_hat = div(v, s.bc2);"),
 ("mhat_old_m", "uint16_t m_hat = div(m_new, s.bc1);", "uint16_t m_hat = div(m, s.bc1);"),
 ("eps_default_inside", "eps_inside ? sqrt(add(v_hat, s.e)) : add(sqrt(v_hat), s.e)", "eps_inside ? add(sqrt(v_hat), s.e) : sqrt(add(v_hat, s.e))"),
 ("ratio_skips_mhat", "uint16_t ratio = div(m_hat, denom);", "uint16_t ratio = div(m_new, denom);"),
 ("decay_full_value", "uint16_t decay = mul(s.lam, theta);", "uint16_t decay = mul(s.lam, add(theta, dtheta));"),
 ("delta_distributed", "uint16_t delta = mul(s.na, add(ratio, decay));\n\n    if (variant == 2)", "uint16_t delta = add(mul(s.na, ratio), mul(s.na, decay));\n\n    if (variant == 2)"),
 ("delta_no_decay", "uint16_t delta = mul(s.na, add(ratio, decay));\n\n    if (variant == 2)", "uint16_t delta = mul(s.na, ratio); (void)decay;\n\n    if (variant == 2)"),
 ("decay_decoupled", "uint16_t delta = mul(s.na, add(ratio, decay));\n\n    if (variant == 2)", "uint16_t delta = mul(s.na, ratio); theta = add(theta, mul(s.na, decay));\n\n    if (variant == 2)"),
 ("kahan_sign", "dtheta = sub(u, sub(theta_new, theta));", "dtheta = sub(sub(theta_new, theta), u);"),
 ("kahan_u_sub", "uint16_t u = add(delta, dtheta);", "uint16_t u = sub(delta, dtheta);"),
 ("kahan_c_from_delta", "dtheta = sub(u, sub(theta_new, theta));", "dtheta = sub(delta, sub(theta_new, theta));"),
 ("plus_ignores_dv", "Pair{v, *dv});", "Pair{v, 0});"),
 ("plus_ignores_b2l", "mul_expansion(Pair{s.b2, s.b2l}, Pair{v, *dv});", "mul_expansion(Pair{s.b2, 0}, Pair{v, *dv});"),
 ("plus_grow_drops_lo", "sorted_free ? grow_two_sum(scaled, inc) : grow(scaled, inc);", "sorted_free ? grow_two_sum(scaled, inc) : grow(Pair{scaled.hi, 0}, inc);"),
 ("plus_twosum_ignored", "sorted_free ? grow_two_sum(scaled, inc) : grow(scaled, inc);", "grow(scaled, inc);"),
 ("theta_twosum_ignored", "sorted_free ? grow_two_sum(Pair{theta, dtheta}, delta) : grow(Pair{theta, dtheta}, delta);", "grow(Pair{theta, dtheta}, delta);"),
 ("plus_scaling_instead", "Pair scaled = mul_expansion(Pair{s.b2, s.b2l}, Pair{v, *dv});", "Pair scaled = scaling(s.b2, Pair{v, *dv});"),
 ("sgd_dampened", "uint16_t m_new = add(mul(s.b1, m), g);", "uint16_t m_new = add(mul(s.b1, m), mul(s.c1, g));"),
 ("sgd_no_decay", "uint16_t delta = mul(s.na, add(m_new, mul(s.lam, theta)));", "uint16_t delta = mul(s.na, m_new);"),
 ("sgd_old_m", "uint16_t delta = mul(s.na, add(m_new, mul(s.lam, theta)));", "uint16_t delta = mul(s.na, add(m, mul(s.lam, theta)));"),
 ("edq_s1_eff2", "a1 += d * effective;", "a1 += effective * effective;"),
 ("edq_s2_eff", "a2 += d * d;", "a2 += d * effective;"),
 ("edq_lost_any_zero", "if (d != 0.0 && effective == 0.0) nl += 1;", "if (effective == 0.0) nl += 1;"),
 ("edq_ignores_dth0", "(dth0 ? (double)Fm::W(dth0[i]) : 0.0)", "0.0"),
 ("edq_ignores_dth1", "(dth1 ? (double)Fm::W(dth1[i]) : 0.0)", "0.0"),
 ("edq_sign", "double effective = after - before;", "double effective = before - after;"),
 ("rne_ties_away", "if (rem > 0.5 || (rem == 0.5 && (k & 1u))) k += 1;\n  const uint32_t hidden", "if (rem >= 0.5) k += 1;\n  const uint32_t hidden"),
 ("rne_truncates", "if (rem > 0.5 || (rem == 0.5 && (k & 1u))) k += 1;\n  const uint32_t hidden", "if (rem > 0.5) k += 1;\n  const uint32_t hidden"),
 ("bf16_R_ties_away", "u += 0x7fffu + keep_is_odd;", "u += 0x8000u;"),
 ("bf16_R_truncate", "u += 0x7fffu + keep_is_odd;", "u += 0;"),
 ("bf16_nan_sign", "return 0x7fc0;   /* every NaN", "return (uint16_t)(0x7fc0 | ((u >> 16) & 0x8000));   /* every NaN"),
 ("generic_subnormal_emin", "int emax = e < EMIN ? EMIN : e;", "int emax = e < EMIN - 1 ? EMIN - 1 : e;"),
 ("generic_overflow_max", "if (bits >= inf_bits) bits = inf_bits;      /* overflow -> infinity */", "if (bits >= inf_bits) bits = inf_bits - 1;"),
 ("e4m3_saturates", "if (bits >= 0x7f) return 0x7f;             /* beyond 448", "if (bits >= 0x7f) return (uint16_t)(sign | 0x7e);             /* beyond 448"),
 ("e4m3_ties_away", "if (fl <= 64.0 && (rem > 0.5 || (rem == 0.5 && (k & 1u)))) k += 1;", "if (fl <= 64.0 && rem >= 0.5) k += 1;"),
 ("e4m3_subnormal_scale", "mag = std::ldexp((float)m, -9);", "mag = std::ldexp((float)m, -10);"),
 ("e4m3_nan_is_inf_row", "if (e == 15 && m == 7) mag", "if (e == 15) mag"),
 ("e5m2_nan_code", "return (uint16_t)((r & 0x7f) | ((r & 0x8000) >> 8));", "return (uint16_t)((r & 0x7f) | ((r & 0x8000) >> 8) | ((r & 0x7f) > 0x7c ? 1 : 0));"),
 ("fp16_subnormal_scale", "mag = std::ldexp((float)m, -24);", "mag = std::ldexp((float)m, -25);"),
 ("fp16_R_via_bf16ish", "static uint16_t R(float f) { return round_f64_to_16bit<10, -14>((double)f); }", "static uint16_t R(float f) { return round_f64_to_16bit<10, -14>((double)bits_f32(f32_bits(f) & 0xffffe000u)); }"),
 ("op_div_is_mul_rcp", "float r = Fm::W(a) / Fm::W(b); return Fm::R(r);", "float r = Fm::W(a) * (1.0f / Fm::W(b)); return Fm::R(r);"),
 ("op_sqrt_double", "float r = std::sqrt(Fm::W(a)); return Fm::R(r);", "float r = (float)std::sqrt((double)Fm::W(a) * 1.0000001); return Fm::R(r);"),
 ("op_add_in_double", "float r = Fm::W(a) + Fm::W(b); return Fm::R(r);", "double r = (double)Fm::W(a) + (double)Fm::W(b); return Fm::B(r);"),
 ("mw_decay_theta16", "float decay = s.lam * master;", "float decay = s.lam * W(theta);"),
 ("mw_eps_inside", "float root = std::sqrt(v_hat);\n  float denom = root + s.e;", "float root = std::sqrt(v_hat + s.e);\n  float denom = root;"),
 ("mw_no_bc1", "float m_hat = m_new / s.bc1;", "float m_hat = m_new;"),
 ("mw_no_bc2", "float v_hat = v_new / s.bc2;", "float v_hat = v_new;"),
 ("mw_vhat_old", "float v_hat = v_new / s.bc2;", "float v_hat = v / s.bc2;"),
 ("mw_theta_trunc", "theta = R(w);", "theta = (uint16_t)(f32_bits(w) >> 16);"),
 ("mw_theta_from_old", "theta = R(w);", "theta = R(master - delta + delta);"),
 ("mw_g2_c2", "float t4 = s.c2 * g2;", "float t4 = s.c1 * g2;"),
 ("mw_delta_sign", "float w = master + delta;", "float w = master - delta;"),
 ("mw_c1_rounded", "s.c1 = (float)(1.0 - h->beta1);", "s.c1 = 1.0f - (float)h->beta1;"),
 ("mw_c2_rounded", "s.c2 = (float)(1.0 - h->beta2);", "s.c2 = 1.0f - (float)h->beta2;"),
 ("mw_bc_float_pow", "s.bc2 = (float)(1.0 - std::pow(h->beta2, td));", "s.bc2 = 1.0f - std::pow((float)h->beta2, (float)td);"),
 ("mw_distributed", "float sum = ratio + decay;\n  float delta = s.na * sum;", "float sum = ratio + decay; (void)sum;\n  float delta = s.na * ratio + s.na * decay;"),
 ("edq_finish_no_sqrt", "return s1 / std::sqrt(s2);", "return s1 / s2;"),
 ("edq_finish_zero", "if (s2 == 0.0) return 0.0;", "if (s2 == 0.0) return 1.0;"),
 ("step_bf16_touches_dtheta", "base == 2 ? unused : dtheta[i]", "dtheta[i]"),
 ("step_fmt_ignored", "const int fmt = (variant >> 12) & 3;          /* ORC_FMT", "const int fmt = 0 * (variant >> 12);          /* ORC_FMT"),
 ("step_threads_overlap", "uint64_t hi = lo + len;\n    pool.emplace_back", "uint64_t hi = lo + len + (k + 1 < nthreads ? 1 : 0);\n    pool.emplace_back"),
 ("step_threads_gap", "uint64_t len = per + ((uint64_t)k < extra ? 1 : 0);", "uint64_t len = per;"),
 ("e5m2_W_low_byte", "return Fp16::W((uint16_t)((h & 0xff) << 8));", "return Fp16::W((uint16_t)((h & 0xff) << 8 | 0x80));"),
 ("e5m2_R_double_round", "static uint16_t R(float f) { return fold(round_f64_to_16bit<2, -14>((double)f)); }", "static uint16_t R(float f) { return fold(round_f64_to_16bit<2, -14>((double)Fp16::W(Fp16::R(f)))); }"),
 ("e4m3_R_double_round", "static uint16_t R(float f) { return B((double)f); }\n};\n\nstruct Pair", "static uint16_t R(float f) { return B((double)Fp16::W(Fp16::R(f))); }\n};\n\nstruct Pair"),
 ("e4m3_max_is_480", "if (bits >= 0x7f) return 0x7f;             /* beyond 448", "if (bits > 0x7f) return 0x7f;             /* beyond 448"),
 ("e4m3_emin", "const int emax = e < -6 ? -6 : e;", "const int emax = e < -7 ? -7 : e;"),
 ("fp16_W_exp", "else mag = std::ldexp((float)(1024 + m), e - 25);", "else mag = std::ldexp((float)(1024 + m), e - 24);"),
 ("fp16_inf_nan", "else if (e == 31) mag = m ? std::numeric_limits<float>::quiet_NaN() : std::numeric_limits<float>::infinity();", "else if (e == 31) mag = std::numeric_limits<float>::infinity();"),
 ("generic_nan_payload", "return (uint16_t)(inf_bits | (1u << (MBITS - 1)));", "return (uint16_t)(inf_bits | 1u);"),
 ("generic_neg_zero", "if (a == 0.0) return sign;\n  if (std::isinf(a)) return sign | inf_bits;", "if (a == 0.0) return 0;\n  if (std::isinf(a)) return sign | inf_bits;"),
 ("bf16_W_shift", "return bits_f32((uint32_t)h << 16); }", "return bits_f32(((uint32_t)h << 16) | 0x8000u); }"),
 ("prim_scaling_roles", "case 5: r = C::scaling(p0[i], Pair{p1[i], p2[i]}); break;", "case 5: r = C::scaling(p1[i], Pair{p0[i], p2[i]}); break;"),
 ("prim_grow_roles", "case 2: r = C::grow(Pair{p0[i], p1[i]}, p2[i]); break;", "case 2: r = C::grow(Pair{p0[i], p2[i]}, p1[i]); break;"),
 ("kahan_theta_plain", "uint16_t theta_new = add(theta, u);", "uint16_t theta_new = add(theta, delta);"),
 ("bf16_keeps_dtheta_grow", "theta = add(theta, delta);\n    } else if (variant == 3)", "theta = add(theta, add(delta, dtheta));\n    } else if (variant == 3)"),
 ("light_vhat_adds_dv", "uint16_t v_hat = div(v_new, s.bc2);", "uint16_t v_hat = div(dv ? add(v_new, *dv) : v_new, s.bc2);"),
 ("sqrt_of_vnew", "add(sqrt(v_hat), s.e)", "add(sqrt(v_new), s.e)"),
]

# Mistakes that no result can show, and why (they are reported as SURVIVED and that is expected):
EQUIVALENT = {
    "op_add_in_double": "fp64 sum then one rounding equals the fp32 sum then rounding: 24 >= 2p+2 for every format here",
    "step_bf16_touches_dtheta": "the plain-bf16 branch never writes its second argument",
    "bf16_keeps_dtheta_grow": "the plain-bf16 branch is handed a zero in place of dtheta by the array wrapper",
    "light_vhat_adds_dv": "F(v + dv) = v for the expansions Grow leaves behind (|dv| <= ulp(v)/2)",
    "mw_theta_from_old": "(w - delta) + delta is w or its fp32 neighbour, and the bf16 rounding that follows hides the neighbour",
}


def run(mutant, extra):
    name, old, new = mutant
    if SRC.count(old) != 1:
        return name, "BAD-PATTERN(%d)" % SRC.count(old), ""
    d = tempfile.mkdtemp(prefix="oracle_mutant_" + name + "_")
    try:
        os.makedirs(os.path.join(d, "oracle"))
        for f in ("oracle.py", "mcf_oracle.h", "__init__.py"):
            p = os.path.join(ROOT, "oracle", f)
            if os.path.exists(p):
                shutil.copy(p, os.path.join(d, "oracle", f))
        with open(os.path.join(d, "oracle", "mcf_oracle.cpp"), "w") as f:
            f.write(SRC.replace(old, new))
        for f in ("tests", "paper_2405_03637_amd", "include", "bench.py", "__graft_entry__.py", "BASELINE.json"):
            os.symlink(os.path.join(ROOT, f), os.path.join(d, f))
        r = subprocess.run(["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-pthread",
                            "-o", os.path.join(d, "oracle", "libmcf_oracle.so"), os.path.join(d, "oracle", "mcf_oracle.cpp")],
                           capture_output=True, text=True)
        if r.returncode:
            return name, "COMPILE-ERROR", r.stderr[-300:]
        env = dict(os.environ, PYTHONDONTWRITEBYTECODE="1")
        r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(d, "tests"), "-x", "-q", "-m", "not gpu",
                            "-p", "no:cacheprovider", *extra], cwd=d, capture_output=True, text=True, env=env)
        tail = [l for l in r.stdout.splitlines() if l.startswith("FAILED") or " passed" in l or " failed" in l]
        return name, ("killed" if r.returncode else "SURVIVED"), " | ".join(tail)[-200:]
    finally:
        shutil.rmtree(d, ignore_errors=True)


def main():
    only = os.environ.get("ONLY")
    todo = [m for m in MUTANTS if not only or m[0] in only.split(",")]
    survivors = []
    with cf.ThreadPoolExecutor(int(os.environ.get("WORKERS", "4"))) as ex:
        for name, res, info in ex.map(lambda m: run(m, sys.argv[1:]), todo):
            note = "  (equivalent: %s)" % EQUIVALENT[name] if res == "SURVIVED" and name in EQUIVALENT else ""
            print(f"{res:10s} {name:28s} {info}{note}", flush=True)
            if res != "killed" and name not in EQUIVALENT:
                survivors.append(name)
    print(f"{len(todo)} mutants, {len(survivors)} not caught and not known to be equivalent: {survivors}")
    return 1 if survivors else 0


if __name__ == "__main__":
    sys.exit(main())
