"""Mutation check of the oracle's pins (test infrastructure: `python oracle/mutation_check.py`, or
tests/test_mutation_checks.py; the full set takes a quarter of an hour). Plants one plausible mistake at a time -- a wrong bias, tie rule, clamp, sign, index,
transposed operand, dropped term -- into a scratch copy of oracle/mxfp8_oracle.c and runs
tests/test_oracle_pins.py and tests/test_oracle_modes.py against it. Every mutant must be caught; a survivor means a pin is missing.
Arguments, if any, select the mutants whose description contains one of them."""
import os
import shutil
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
M=[
 ("decode: exponent bias 8", "v = ldexp(1.0 + (double)m / 8.0, e - 7);", "v = ldexp(1.0 + (double)m / 8.0, e - 8);"),
 ("decode: subnormal unit 2^-10", "v = ldexp((double)m, -9);", "v = ldexp((double)m, -10);"),
 ("decode: every exponent-15 code is NaN", "if (e == 0xF && m == 0x7)", "if (e == 0xF)"),
 ("decode: 2 mantissa bits", "(double)m / 8.0", "(double)m / 4.0"),
 ("encode: ties to odd", "(d == best_d && (c & 1) == 0)", "(d == best_d && (c & 1) == 1)"),
 ("encode: ties away from zero", "if (d < best_d || (d == best_d && (c & 1) == 0)) {", "if (d <= best_d) {"),
 ("encode: ties toward zero", "if (d < best_d || (d == best_d && (c & 1) == 0)) {", "if (d < best_d) {"),
 ("encode: overflow gives NaN instead of saturating", "return (uint8_t)(sign | 0x7E);", "return (uint8_t)(sign | 0x7F);"),
 ("encode: sign dropped", "return (uint8_t)(sign | best);", "return (uint8_t)(best);"),
 ("encode: 448 unreachable", "for (c = 1; c <= 0x7E; ++c) {", "for (c = 1; c < 0x7E; ++c) {"),
 ("encode: NaN sign kept", "if (isnan(t))\n        return 0x7F;", "if (isnan(t))\n        return sign | 0x7F;"),
 ("scale: strict inequality (448*2^k rounds up)", "if (amax <= ldexp(448.0, n))", "if (amax < ldexp(448.0, n))"),
 ("scale: destination maximum 256", "ldexp(448.0, n)", "ldexp(256.0, n)"),
 ("scale: destination maximum 480", "ldexp(448.0, n)", "ldexp(480.0, n)"),
 ("scale: round down (OCP rule)", "if (amax <= ldexp(448.0, n))", "if (amax < ldexp(896.0, n))"),
 ("scale: lower clamp -126", "for (n = -127; n < 127; ++n)", "for (n = -126; n < 127; ++n)"),
 ("scale: upper clamp 126", "for (n = -127; n < 127; ++n)", "for (n = -127; n < 126; ++n)"),
 ("scale: bias 128", "return n + 127;\n}", "return n + 128;\n}"),
 ("scale: NaN not flagged", "    if (isnan(amax))\n        return 0xFF;\n    for", "    for"),
 ("block: amax of signed values", "double a = fabs(v[i]);\n        if (isnan(a))", "double a = v[i];\n        if (isnan(a))"),
 ("block: NaN block bytes 0xFF", "q[i * qs] = 0x7F;", "q[i * qs] = 0xFF;"),
 ("block: NaN block scale 254", "*s = 0xFF;", "*s = 254;"),
 ("block: multiplies by X instead of dividing", "ldexp(v[i], -n)", "ldexp(v[i], n)"),
 ("block: amax over 31 elements", "for (i = 0; i < MX_K; ++i) {\n        double a", "for (i = 1; i < MX_K; ++i) {\n        double a"),
 ("rowwise: leading dimension ignored", "WIDEN(src[r * ld + b * MX_K + i])", "WIDEN(src[r * cols + b * MX_K + i])"),
 ("colwise: leading dimension ignored", "WIDEN(src[(b * MX_K + i) * ld + c])", "WIDEN(src[(b * MX_K + i) * cols + c])"),
 ("colwise: scales not transposed", "sT + c * nb + b", "sT + b * cols + c"),
 ("colwise: blocks along the row", "WIDEN(src[(b * MX_K + i) * ld + c])", "WIDEN(src[c * ld + b * MX_K + i])"),
 ("bf16 widening shift", "(uint32_t)h << 16", "(uint32_t)h << 15"),
 ("decode_one: bias 128", "ldexp(mxo_e4m3_decode(q), (int)s - 127)", "ldexp(mxo_e4m3_decode(q), (int)s - 128)"),
 ("decode_one: NaN scale ignored", "    if (s == 0xFF)\n        return NAN;\n    return ldexp", "    return ldexp"),
 ("dequantize f32: neighbouring block's scale", "dst[r * ld + c] = (float)decode_one(q[r * cols + c], s[r * nb + c / MX_K]);", "dst[r * ld + c] = (float)decode_one(q[r * cols + c], s[r * nb + (c / MX_K + 1) % nb]);"),
 ("dequantize f64: neighbouring block's scale", "dst[r * cols + c] = decode_one(q[r * cols + c], s[r * nb + c / MX_K]);", "dst[r * cols + c] = decode_one(q[r * cols + c], s[r * nb + (c / MX_K + 1) % nb]);"),
 ("bf16 rounding: ties away", "if (rem > 0.5 || (rem == 0.5 && (mant & 1)))\n        mant += 1;\n    if (mant == 256)", "if (rem >= 0.5)\n        mant += 1;\n    if (mant == 256)"),
 ("bf16 rounding: truncation", "if (rem > 0.5 || (rem == 0.5 && (mant & 1)))\n        mant += 1;\n    if (mant == 256)", "if (mant == 256)"),
 ("bf16 rounding: subnormal ties away", "if (rem > 0.5 || (rem == 0.5 && (mant & 1)))\n            mant += 1;\n        return", "if (rem >= 0.5)\n            mant += 1;\n        return"),
 ("bf16 rounding: overflow to max finite", "if (be >= 255)\n        return (uint16_t)(sign | 0x7F80);", "if (be >= 255)\n        return (uint16_t)(sign | 0x7F7F);"),
 ("gemm: B read transposed", "double p = a[idx * K + k] * b[n * K + k];", "double p = a[idx * K + k] * b[(n * K + k) % K * N + (n * K + k) / K % N];"),
 ("gemm: abs-sum without abs", "aacc += fabs(p);", "aacc += p;"),
 ("gemm: last k dropped", "for (k = 0; k < K; ++k) {\n                double p", "for (k = 0; k < K - 1; ++k) {\n                double p"),
 ("gemm: row selection ignored", "mxo_dequantize_f64(a_q + row_idx[idx] * K, a_s + row_idx[idx] * nb, 1, K, a + idx * K);", "mxo_dequantize_f64(a_q + idx * K, a_s + idx * nb, 1, K, a + idx * K);"),
 ("gemm: A scales of the wrong row", "mxo_dequantize_f64(a_q + row_idx[idx] * K, a_s + row_idx[idx] * nb, 1, K, a + idx * K);", "mxo_dequantize_f64(a_q + row_idx[idx] * K, a_s + idx * nb, 1, K, a + idx * K);"),
 ("gemm: product sign", "acc += p;", "acc -= p;"),
 # ablation arms (pinned by tests/test_oracle_modes.py)
 ("e5m2 decode: exponent bias 16", "ldexp(1.0 + (double)m / 4.0, e - 15)", "ldexp(1.0 + (double)m / 4.0, e - 16)"),
 ("e5m2 decode: subnormal unit 2^-17", "v = ldexp((double)m, -16);", "v = ldexp((double)m, -17);"),
 ("e5m2 decode: no infinities", "return m ? NAN : (sign ? -INFINITY : INFINITY);", "return NAN;"),
 ("e5m2 encode: overflow gives Inf instead of saturating", "return (uint8_t)(sign | 0x7B);", "return (uint8_t)(sign | 0x7C);"),
 ("e5m2 encode: ties to odd", "if (d < best_d || (d == best_d && (c & 1) == 0)) {\n            best_d = d;\n            best = c;\n        }\n    }\n    return (uint8_t)(sign | best);\n}\n\nstatic double fmt_max",
  "if (d < best_d || (d == best_d && (c & 1) == 1)) {\n            best_d = d;\n            best = c;\n        }\n    }\n    return (uint8_t)(sign | best);\n}\n\nstatic double fmt_max"),
 ("ocp rule: strict inequality (powers of two round down a binade)", "if (ldexp(1.0, n + fmt_emax(fmt)) <= amax)", "if (ldexp(1.0, n + fmt_emax(fmt)) < amax)"),
 ("ocp rule: E4M3 emax 7", "return fmt ? 15 : 8;", "return fmt ? 15 : 7;"),
 ("mode quantize: scale bias off by one", "ldexp((double)v[i], -(sb - 127))", "ldexp((double)v[i], -(sb - 128))"),
 ("mode quantize: E5M2 destination maximum 448", "return fmt ? 57344.0 : 448.0;", "return fmt ? 448.0 : 448.0;"),
]
src=open(os.path.join(ROOT,'oracle','mxfp8_oracle.c')).read()
results=[]
only=sys.argv[1:]
for name,old,new in M:
    if only and not any(o in name for o in only): continue
    assert src.count(old)>=1, (name, src.count(old))
    mutated=src.replace(old,new,1)
    tmp=tempfile.mkdtemp(prefix='mut_')
    try:
        os.makedirs(os.path.join(tmp,'oracle'))
        shutil.copy(os.path.join(ROOT,'oracle','__init__.py'), os.path.join(tmp,'oracle'))
        open(os.path.join(tmp,'oracle','mxfp8_oracle.c'),'w').write(mutated)
        shutil.copytree(os.path.join(ROOT,'tests','golden'), os.path.join(tmp,'tests','golden'))
        for f in ('conftest.py','test_oracle_pins.py','test_oracle_modes.py'):
            shutil.copy(os.path.join(ROOT,'tests',f), os.path.join(tmp,'tests'))
        os.makedirs(os.path.join(tmp,'paper_2506_08027_amd'))
        shutil.copy(os.path.join(ROOT,'paper_2506_08027_amd','synth_inputs.py'), os.path.join(tmp,'paper_2506_08027_amd'))
        open(os.path.join(tmp,'paper_2506_08027_amd','__init__.py'),'w').write('')
        r=subprocess.run([sys.executable,'-m','pytest','-q','-x','-p','no:cacheprovider','tests/test_oracle_pins.py','tests/test_oracle_modes.py'],cwd=tmp,capture_output=True,text=True,timeout=900)
        killed = r.returncode!=0
        first=[l for l in r.stdout.splitlines() if l.startswith('FAILED') or 'Error' in l][:1]
        results.append((name,killed,first[0][:110] if first else ''))
        print(('KILLED  ' if killed else 'SURVIVED'), name, '|', first[0][:110] if first else '', flush=True)
    finally:
        shutil.rmtree(tmp,ignore_errors=True)
print(sum(k for _,k,_ in results),'of',len(results),'killed')
sys.exit(0 if all(k for _, k, _ in results) else 1)
