"""Mutation check of the oracle's pins (CPU only, not collected by pytest):

    python tests/mutate_oracle.py [substring of a mutation's name ...]

For each planted mistake (a wrong index, sign, operand, term, tie-break or exactness bound, one at a time) the oracle's
source is copied to a scratch directory with that mistake, rebuilt, and tests/test_oracle_pins.py is run against it;
every mistake must make some pin fail ("KILLED").  A mistake that survives names a hole in the pins."""
import os, shutil, subprocess, sys, tempfile
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
MUTS = [
 ("fwd wrong column", "widen(X, dt, (size_t)(t * q + 4 * g + c))", "widen(X, dt, (size_t)(t * q + 4 * g + (3 - c)))"),
 ("fwd swapped pair", "widen(vals, dt, (size_t)(o * (q / 2) + 2 * g + s))", "widen(vals, dt, (size_t)(o * (q / 2) + 2 * g + (1 - s)))"),
 ("dx index from s", "widen(dY, dt, (size_t)(t * r + 4 * g + c))", "widen(dY, dt, (size_t)(t * r + 4 * g + s))"),
 ("dx beta dropped", "dX[n * q + i] = (dX0 ? beta * dX0[n * q + i] : 0.0) + acc;", "dX[n * q + i] = acc;"),
 ("dw transposed operand", "widen(dY, dt, (size_t)(t * r + o)) * widen(X, dt, (size_t)(t * q + i))", "widen(dY, dt, (size_t)(o * p + t)) * widen(X, dt, (size_t)(t * q + i))"),
 ("dw beta dropped", "dW[n * q + i] = (dW0 ? beta * dW0[n * q + i] : 0.0) + acc;", "dW[n * q + i] = acc;"),
 ("dense gemm transposed W", "widen(W, dt, (size_t)(o * q + i))", "widen(W, dt, (size_t)(i * r + o))"),
 ("decay on kept", "if (!mask_bit(mask, bq, o, i)) g +=", "if (mask_bit(mask, bq, o, i)) g +="),
 ("decay sign", "g += (double)lambda * widen(W, wdt", "g -= (double)lambda * widen(W, wdt"),
 ("silu' sign", "dG[t * f + c] = d * u * s * (1.0 + g * (1.0 - s));", "dG[t * f + c] = d * u * s * (1.0 - g * (1.0 - s));"),
 ("silu' term", "dG[t * f + c] = d * u * s * (1.0 + g * (1.0 - s));", "dG[t * f + c] = d * u * s * (1.0 + g * (1.0 + s));"),
 ("dU wrong operand", "dU[t * f + c] = d * g * s;", "dU[t * f + c] = d * u * s;"),
 ("swiglu gate second", "H[t * f + c] = g * sigmoid(g) * u;", "H[t * f + c] = u * sigmoid(u) * g;"),
 ("gelu scale", "else H[k] = 0.5 * z * (1.0 + erf(z / sqrt(2.0)));", "else H[k] = 0.5 * z * (1.0 + erf(z / 2.0));"),
 ("gelu' sign", "+ z * inv_sqrt_2pi * exp(-0.5 * z * z);", "- z * inv_sqrt_2pi * exp(-0.5 * z * z);"),
 ("relu'(0)", "dz = z > 0.0 ? 1.0 : 0.0;", "dz = z >= 0.0 ? 1.0 : 0.0;"),
 ("gate_slope gelu exp", "x * 0.39894228040143267794 * exp(-0.5 * x * x);", "x * 0.39894228040143267794 * exp(-x * x);"),
 ("gate_value silu", "return gate == ORC_GATE_SILU ? x * sigmoid(x) :", "return gate == ORC_GATE_SILU ? sigmoid(x) :"),
 ("glu halves swapped in bwd", "dZ[t * 2 * r + c] = d * z2 * gate_slope(gate, z1);\n            dZ[t * 2 * r + r + c] = d * gate_value(gate, z1);", "dZ[t * 2 * r + r + c] = d * z2 * gate_slope(gate, z1);\n            dZ[t * 2 * r + c] = d * gate_value(gate, z1);"),
 ("glu fwd up from gate half", "z2 = widen(Z, dt, at(layout, ldz, t, r + c));\n            H[t * r + c]", "z2 = widen(Z, dt, at(layout, ldz, t, c));\n            H[t * r + c]"),
 ("col-major index", "return (size_t)(layout == ORC_COL_MAJOR ? c * ld + t : t * ld + c);", "return (size_t)(layout == ORC_COL_MAJOR ? t * ld + c : t * ld + c);"),
 ("bias grad drops last token", "for (int64_t t = 0; t < p; ++t) s += widen(dZ, dt, at(layout, ld, t, c));", "for (int64_t t = 0; t + 1 < p; ++t) s += widen(dZ, dt, at(layout, ld, t, c));"),
 ("meta nibble order", "return (int)((nib >> (2 * s)) & 3u);", "return (int)((nib >> (2 * (1 - s))) & 3u);"),
 ("meta word order", "(meta[row * words_per_row + g / 4] >> (4 * (g % 4))) & 0xFu", "(meta[row * words_per_row + g / 4] >> (4 * (3 - g % 4))) & 0xFu"),
 ("argmax last max wins", "if (s > best_s) { best_s = s; best = k; }", "if (s >= best_s) { best_s = s; best = k; }"),
 ("argmax wide last wins", "if (k == 0 || wide_cmp(&s, &best_w) > 0)", "if (k == 0 || wide_cmp(&s, &best_w) >= 0)"),
 ("mask no abs", "a[4 * i + j] = fabs(widen(W, dt, (size_t)((4 * bi + i) * ldw + 4 * bj + j)));", "a[4 * i + j] = widen(W, dt, (size_t)((4 * bi + i) * ldw + 4 * bj + j));"),
 ("mask transposed block", "a[4 * i + j] = fabs(", "a[4 * j + i] = fabs("),
 ("exactness window too wide", "return (top + 3) - low <= 53;", "return (top + 3) - low <= 58;"),
 ("sigmoid neg branch", "return e / (1.0 + e);", "return 1.0 / (1.0 + e);"),
 ("pattern row check dropped", "if (m[i][0] + m[i][1] + m[i][2] + m[i][3] != 2) ok = 0;", "if (m[i][0] + m[i][1] + m[i][2] + m[i][3] > 4) ok = 0;"),
 ("pattern bit order", "if (m[t / 4][t % 4]) enc |= (uint16_t)(1u << t);", "if (m[t % 4][t / 4]) enc |= (uint16_t)(1u << (15 - t));"),
 ("pattern string order", "m[t / 4][t % 4] = (int)((s >> (15 - t)) & 1u);", "m[t / 4][t % 4] = (int)((s >> t) & 1u);"),
 ("mvue cap test", "const int capped = 2.0f * mx > S;", "const int capped = mx > S;"),
 ("mvue uncapped value", "mag[i] = capped ? R : 0.5f * S;", "mag[i] = capped ? R : S;"),
 ("mvue capped value", "mag[i] = capped ? R : 0.5f * S;", "mag[i] = capped ? S : 0.5f * S;"),
 ("mvue probability scale", "const float D = capped ? R : S, scale = capped ? 1.0f : 2.0f;", "const float D = capped ? R : S, scale = 1.0f;"),
 ("mvue top not forced", "if (capped && m[i] == mx) { pi[i] = 1.0f; mag[i] = m[i]; }", "if (capped && m[i] == mx) { mag[i] = m[i]; }"),
 ("mvue second point", "v = u + 1.0f;", "v = u + 0.5f;"),
 ("mvue sign lost", "*v0 = m[a0] == 0.0f ? 0.0f : copysignf(mag[a0], a[a0]);", "*v0 = m[a0] == 0.0f ? 0.0f : mag[a0];"),
 ("mvue hash ignores feature", "const uint32_t key = mix32(mix32(seed) + feature * 0x9E3779B9U);", "const uint32_t key = mix32(mix32(seed));"),
 ("mvue hash ignores group", "return mix32(key + group * 0x85EBCA6BU) >> 9;", "return mix32(key) >> 9;"),
 ("mvue seed meets group unmixed", "const uint32_t key = mix32(mix32(seed) + feature * 0x9E3779B9U);\n    return mix32(key + group * 0x85EBCA6BU) >> 9;", "return mix32(mix32(group ^ seed) + feature * 0x9E3779B9U) >> 9;"),
 ("mvue token stride", "a[i] = (float)widen(dY, dt, (size_t)((4 * g + i) * ld + f));", "a[i] = (float)widen(dY, dt, (size_t)((4 * g + i) * r + f));"),
 ("flips count blocks", "for (int t = 0; t < 16; ++t) c += (x >> t) & 1u;", "c = x != 0;"),
 ("gap second best", "else if (k == 1 || wide_cmp(&s, &second) > 0) second = s;", "else if (k == 1) second = s;"),
 ("gap demotes first", "if (wide_cmp(&s, &first) > 0) { second = first; first = s; }", "if (wide_cmp(&s, &first) > 0) { first = s; }"),
 ("compress kept order", "unsigned nib = (unsigned)kept[0] | ((unsigned)kept[1] << 2);\n            meta[o", "unsigned nib = (unsigned)kept[1] | ((unsigned)kept[0] << 2);\n            meta[o"),
 ("compress value column", "(const char *)W + (size_t)(o * ldw + 4 * g + kept[s]) * es, es);", "(const char *)W + (size_t)(o * ldw + 4 * g + s) * es, es);"),
 ("compressT row/col", "if (mask_bit(mask, bq, 4 * g + c, i)) kept[n < 4 ? n++ : 3] = c;", "if (mask_bit(mask, bq, i, 4 * g + c)) kept[n < 4 ? n++ : 3] = c;"),
 ("compressT value", "(const char *)W + (size_t)((4 * g + kept[s]) * ldw + i) * es, es);", "(const char *)W + (size_t)((4 * g + s) * ldw + i) * es, es);"),
 ("mask bit index", "return (b >> (4 * (row % 4) + (col % 4))) & 1;", "return (b >> (4 * (col % 4) + (row % 4))) & 1;"),
 ("pack chunk values", "(const char *)vals + (size_t)(o * (K / 2) + 32 * c + j) * es, es);", "(const char *)vals + (size_t)(o * (K / 2) + 32 * c + (j ^ 1)) * es, es);"),
 ("pack chunk meta", "meta_p[(c * R + o) * 4 + j] = meta[o * (K / 16) + 4 * c + j];", "meta_p[(c * R + o) * 4 + j] = meta[o * (K / 16) + 4 * c + (3 - j)];"),
 ("half subnormal scale", "if (e == 0) v = ldexp((double)f, -24);", "if (e == 0) v = ldexp((double)f, -25);"),
 ("half exponent bias", "else v = ldexp((double)(1024 + f), e - 25);", "else v = ldexp((double)(1024 + f), e - 24);"),
 ("half sign lost", "return sign ? -v : v;\n}\n\nstatic double widen", "return v;\n}\n\nstatic double widen"),
 ("bf16 widen shift", "uint32_t u = ((uint32_t)((const uint16_t *)base)[idx]) << 16;", "uint32_t u = ((uint32_t)((const uint16_t *)base)[idx]) << 15;"),
 ("round_bf16 truncates", "uint32_t lsb = (u >> 16) & 1u;\n        u += 0x7FFFu + lsb;", "uint32_t lsb = 0;\n        u += 0 * lsb;"),
 ("round_bf16 ties away", "uint32_t lsb = (u >> 16) & 1u;\n        u += 0x7FFFu + lsb;", "uint32_t lsb = 1u;\n        u += 0x7FFFu + lsb;"),
 ("mvue bf16 rounding ties away", "u += 0x7FFFu + ((u >> 16) & 1u);\n    return (uint16_t)(u >> 16);", "u += 0x8000u;\n    return (uint16_t)(u >> 16);"),
 ("wide add limb carry", "acc->limb[li + 1] += v >> 32;", "acc->limb[li + 1] += v >> 33;"),
 ("wide add offset", "int shift = low + 149;", "int shift = low + 150;"),
 ("wide normalise carry", "carry = t >> 32;", "carry = 0;"),
 ("wide cmp from low limb", "for (int i = WIDE_LIMBS - 1; i >= 0; --i) {\n        if (a->limb[i] > b->limb[i]) return 1;", "for (int i = 0; i < WIDE_LIMBS; ++i) {\n        if (a->limb[i] > b->limb[i]) return 1;"),
 ("round_f16 subnormal boundary", "if (e - 1 < -14) return", "if (e - 1 < -15) return"),
]
def main():
    src = open(os.path.join(ROOT, "oracle/s24_oracle.c")).read()
    work = os.path.join(tempfile.gettempdir(), "s24_oracle_mutant")
    results = []
    only = sys.argv[1:]
    for name, old, new in MUTS:
        if only and not any(o in name for o in only): continue
        if src.count(old) < 1:
            results.append((name, "NOT FOUND")); print(name, "NOT FOUND", flush=True); continue
        if os.path.exists(work): shutil.rmtree(work)
        os.makedirs(work)
        for d in ("oracle", "tests", "include"):
            shutil.copytree(os.path.join(ROOT, d), os.path.join(work, d), ignore=shutil.ignore_patterns("__pycache__", "*.so"))
        for f in ("s24_inputs.py",):
            shutil.copy(os.path.join(ROOT, f), work)
        os.makedirs(os.path.join(work, "paper_2404_01847_amd"))
        open(os.path.join(work, "oracle/s24_oracle.c"), "w").write(src.replace(old, new, 1))
        r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"],
                           cwd=work, capture_output=True, text=True, timeout=900)
        tail = [l for l in r.stdout.splitlines() if l.strip()][-1] if r.stdout.strip() else r.stderr[-200:]
        failed = [l for l in r.stdout.splitlines() if l.startswith("FAILED")]
        status = "KILLED" if r.returncode != 0 else "SURVIVED"
        results.append((name, status))
        print(f"{status:9s} {name:32s} {failed[0][:110] if failed else tail[:110]}", flush=True)
    survivors = [n for n, s in results if s != "KILLED"]
    print("survivors:", survivors)
    return 1 if survivors else 0


if __name__ == "__main__":
    sys.exit(main())
