"""Sensitivity check of the CPU execution model (test infrastructure; `python tests/host_model/mutation_check.py`,
or tests/test_mutation_checks.py with --runslow). Plants one mistake at a time into a scratch
copy of the GEMM kernel source -- a removed barrier, a wait count that is one too loose, a missing wait,
a swizzle mismatch, a prefetch into the wrong buffer or of the wrong K step, a missing ragged-tile clamp,
a wrong output row -- builds the host model from it and runs a few products against the oracle in all
four scheduling modes (lazy / eager DMA completion, either wavefront running ahead). Every mutant must
be caught, by a wrong or NaN result or by the model's range check. A second group plants mistakes into the
converters (scale-rule constants, the staging swizzle of the transposed copy, a removed barrier, the infinity patch,
the narrow formats' scale rules) and compares the quantized bytes with the oracle's. Arguments, if any, select the
mutants whose description contains one of them."""
import os
import shutil
import subprocess
import sys
import tempfile

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
import oracle  # noqa: E402

MID = ("                MXFP8_WAIT_VMCNT(Cfg::NA + Cfg::NB);  // all but this step's requests: A(kt+1) is in LDS\n"
       "                __syncthreads();")
END = ("        MXFP8_WAIT_VMCNT(Cfg::NA);  // everything older than this step's A requests: B(kt+1) is in LDS\n"
       "        __syncthreads();")
PRO = ("        MXFP8_WAIT_VMCNT(0);\n        __syncthreads();\n#pragma unroll\n        for (int i = 0; i < TM; ++i) {\n"
       "            fa[i] = read_frag(lds + Cfg::A_OFF")
MUTANTS = [  # (description, old text, new text): first occurrence, i.e. in the one-tile-per-workgroup kernel
    ("barrier before the last MFMA column removed", MID, MID.replace("\n                __syncthreads();", "")),
    ("barrier at the end of the K step removed", END, END.replace("\n        __syncthreads();", "")),
    ("mid-step wait one request too loose", "MXFP8_WAIT_VMCNT(Cfg::NA + Cfg::NB);  // all but",
     "MXFP8_WAIT_VMCNT(Cfg::NA + Cfg::NB + 1);  // all but"),
    ("end-of-step wait one request too loose", "MXFP8_WAIT_VMCNT(Cfg::NA);  // everything older",
     "MXFP8_WAIT_VMCNT(Cfg::NA + 1);  // everything older"),
    ("prologue does not wait for its loads", PRO, PRO.replace("        MXFP8_WAIT_VMCNT(0);\n", "")),
    ("fragment read uses another swizzle than the load", "const int a_off0 = a_row * BK + ((g ^ ((a_row >> 1) & 7)) << 4)",
     "const int a_off0 = a_row * BK + ((g ^ ((a_row >> 2) & 7)) << 4)"),
    ("A prefetch goes to the buffer still in use", "issue_a(a_slot, kt2, cur);", "issue_a(a_slot, kt2, nxt);"),
    ("B prefetch fetches the wrong K step", "const int kt1 = min(kt + 1, KT - 1), kt2", "const int kt1 = min(kt + 2, KT - 1), kt2"),
    ("ragged tile reads past the last row", "a_goff[i] = (uint32_t)min(row, M - 1 - m0) * (uint32_t)K + chunk * 16;",
     "a_goff[i] = (uint32_t)row * (uint32_t)K + chunk * 16;"),
    ("row-major scale dwords land in the wrong 64-row group",
     "                dma_load<4>(as_tile + (kt * SDW + dw) * 4, as_goff[i],\n                            lds_base + Cfg::SA_OFF + buf * Cfg::SA_BYTES + dw * Cfg::BM * 4 + a_grp(i) * 256);",
     "                dma_load<4>(as_tile + (kt * SDW + dw) * 4, as_goff[i],\n                            lds_base + Cfg::SA_OFF + buf * Cfg::SA_BYTES + dw * Cfg::BM * 4 + ((a_grp(i) + 1) % (Cfg::BM / 64)) * 256);"),
    ("epilogue stores to the rows of another wavefront", "const int m = m0 + wm * Cfg::WM + i * 16 + r16;",
     "const int m = m0 + wn * Cfg::WM + i * 16 + r16;"),
]
# the same kinds of mistake in the persistent kernel (last occurrence of the text; run with several tiles per workgroup)
PERSISTENT_MUTANTS = [
    ("persistent: barrier before the last MFMA column removed",
     "                MXFP8_WAIT_VMCNT(Cfg::NA + Cfg::NB);\n                MXFP8_BARRIER();",
     "                MXFP8_WAIT_VMCNT(Cfg::NA + Cfg::NB);"),
    ("persistent: end-of-step wait one request too loose", "        MXFP8_WAIT_VMCNT_AND_LDS(Cfg::NA);\n        MXFP8_BARRIER();",
     "        MXFP8_WAIT_VMCNT_AND_LDS(Cfg::NA + 1);\n        MXFP8_BARRIER();"),
    ("persistent: barrier at the end of the K step removed",
     "        MXFP8_WAIT_VMCNT_AND_LDS(Cfg::NA);\n        MXFP8_BARRIER();", "        MXFP8_WAIT_VMCNT_AND_LDS(Cfg::NA);"),
    ("persistent: next tile's B fetched one K step late", "                b_src = next_tile.b;\n", "                b_src = next_tile.b + BK;\n"),
    ("persistent: next tile's first A step fetched from the current tile",
     "                a_src = next_tile.a + (int64_t)(kt + 2 - KT) * BK;", "                a_src = cur_tile.a + (int64_t)(kt + 2 - KT) * BK;"),
    ("persistent: accumulators not cleared between tiles", "                acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};\n        cur_tile = next_tile;",
     "                ;\n        cur_tile = next_tile;"),
    ("persistent: buffer parity not carried across tiles", "            step(par, b_src, bs_src, a_src, as_src, a_lim);\n            par ^= 1;",
     "            step(kt & 1, b_src, bs_src, a_src, as_src, a_lim);\n            par ^= 1;"),
]
MODES = [{}, {"WAVESIM_ORDER": "down"}, {"WAVESIM_DMA": "eager"}, {"WAVESIM_DMA": "eager", "WAVESIM_ORDER": "down"}]


def build(work, text, name="gemm.hip"):
    csrc = os.path.join(work, "csrc")
    shutil.copytree(os.path.join(ROOT, "paper_2506_08027_amd", "csrc"), csrc)
    open(os.path.join(csrc, name), "w").write(text)
    inc = os.path.join(ROOT, "include", "mxfp8.h")
    for name, path in (("api.hip", csrc), ("driver.cpp", work)):
        src = os.path.join(csrc if name == "api.hip" else HERE, name)
        text = open(src).read().replace('"../../include/mxfp8.h"', f'"{inc}"').replace('"wavesim.h"', f'"{HERE}/wavesim.h"')
        open(os.path.join(path, name), "w").write(text)
    binary = os.path.join(work, "hostmodel")
    cmd = ["/opt/rocm/llvm/bin/clang++", "-std=c++17", "-x", "c++", "-I", os.path.join(HERE, "shim"), "-O2",
           "-Wno-unknown-pragmas", "-Wno-psabi", "-o", binary, os.path.join(work, "driver.cpp")]
    cmd += [os.path.join(csrc, f) for f in sorted(os.listdir(csrc)) if f.endswith(".hip")]
    subprocess.run(cmd, check=True, capture_output=True)
    return binary


def caught(binary, work, persistent=0):
    for M, N, K in ([(256, 384, 384), (2048, 4096, 384)] if persistent else [(256, 256, 512), (200, 136, 384), (2048, 4096, 512)]):
        rng = np.random.default_rng(M + N)
        a = rng.standard_normal((M, K)).astype(np.float32)
        b = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
        ops = oracle.quantize_rowwise(a) + oracle.quantize_rowwise(b)
        names = []
        for n, v in zip(("aq", "as", "bq", "bs"), ops):
            names.append(os.path.join(work, n + ".bin"))
            v.tofile(names[-1])
        out = os.path.join(work, "c.bin")
        case = os.path.join(work, "case.txt")
        # persistent: 6 small tiles on 2 workgroups, 128 large tiles on 64: K = 3 steps (odd: parity flips per tile)
        wg = f" wg={2 if M == 256 else 64}" if persistent else ""
        open(case, "w").write(f"gemm 0 {M} {N} {K} f32 {N} {' '.join(names)} {out}{wg}\n")
        for mode in MODES:
            env = dict(os.environ, WAVESIM_BLOCKS="2", **mode)
            r = subprocess.run([binary, case], capture_output=True, text=True, env=env)
            if r.returncode != 0:
                return f"model stopped: {r.stderr.strip().splitlines()[-1][:100]}"
            c = np.fromfile(out, np.uint32).reshape(M, N)
            written = c != 0xA5A5A5A5
            rows = np.unique(np.nonzero(written)[0])
            ref, absum = oracle.gemm_rows(*ops, rows)
            val = c.view(np.float32)[rows]
            w = written[rows]
            if np.isnan(val[w]).any() or (np.abs(val - ref)[w] > (2.0 ** -23 * absum + 1e-300)[w]).any():
                return f"wrong result at {M}x{N}x{K} in mode {mode or 'default'}"
    return None


# mistakes in the converters: (description, source file, old text, new text), first occurrence
QUANT_MUTANTS = [
    ("quantizer: FP32 scale rule carries at 1.875 instead of 1.75", "mxfp8_device.h",
     "(abs_bits + 0x1FFFFFu) >> 23) - 8", "(abs_bits + 0x0FFFFFu) >> 23) - 8"),
    ("quantizer: BF16 scale rule carries at 1.875 instead of 1.75", "mxfp8_device.h",
     "(abs_bits16 + 0x1Fu) >> 7) - 8", "(abs_bits16 + 0x0Fu) >> 7) - 8"),
    ("quantizer: staging swizzle of the transposed copy differs from the write-out's", "quantize.hip",
     "const int slot16 = (lrow0 >> 4) ^ (cc & 7);", "const int slot16 = (lrow0 >> 4) ^ ((cc + 1) & 7);"),
    ("quantizer: barrier between staging and write-out removed", "quantize.hip",
     "        __syncthreads();\n\n        // ---- write-out of the staged pieces", "\n        // ---- write-out of the staged pieces"),
    ("quantizer: infinities keep the converter's NaN code in the row copy", "quantize.hip",
     "f0 |= inf_byte<BF16, MODE>(elem_at<BF16>(x[i], j), (q0 >> (8 * j)) & 0xFFu) << (8 * j);",
     "f0 |= ((q0 >> (8 * j)) & 0xFFu) << (8 * j);"),
    ("quantizer: MXFP4 scale rule carries at 1.75 instead of 1.5", "mxfp4.hip",
     "(abs_bits + 0x3FFFFFu) >> 23) - 2", "(abs_bits + 0x1FFFFFu) >> 23) - 2"),
    ("quantizer: MXFP6 scale exponent one too large", "mxfp6.hip",
     "(0x7FFFFFu - F::TOP_FRAC)) >> 23) - F::EMAX;", "(0x7FFFFFu - F::TOP_FRAC)) >> 23) - F::EMAX + 1;"),
]


def caught_quant(binary, work):
    """Quantizes the tiny configuration (every special block) as FP32 and as BF16 along both axes, and hard cases of
    the narrow formats, and compares every output byte with the oracle."""
    from oracle import mxfp4, mxfp6
    from paper_2506_08027_amd import synth_inputs as si
    x = si.tiny_with_specials(256, seed=0)
    cases = []
    for bf16 in (False, True):
        src = si.to_bf16_bits(x) if bf16 else x
        cases.append((f"quantize {'bf16' if bf16 else 'f32'} 256 256 256 3", src,
                      (oracle.quantize_rowwise(src), oracle.quantize_colwise(src))))
    h4 = si.fp4_hard_cases(160, 96, seed=12)
    cases.append(("quantfp4 f32 160 96 96 3", h4, (mxfp4.quantize_rowwise(h4), mxfp4.quantize_colwise(h4))))
    h6 = si.fp6_hard_cases(160, 96, seed=12, top=7.5)
    cases.append(("quantfp6 f32 160 96 96 3 0", h6, (mxfp6.quantize_rowwise(h6, "e2m3"), mxfp6.quantize_colwise(h6, "e2m3"))))
    for head, src, ((q, s), (qT, sT)) in cases:
        path = os.path.join(work, "src.bin")
        np.ascontiguousarray(src).tofile(path)
        prefix = os.path.join(work, "o")
        case = os.path.join(work, "case.txt")
        open(case, "w").write(f"{head} {path} {prefix}\n")
        r = subprocess.run([binary, case], capture_output=True, text=True)
        if r.returncode != 0:
            return f"model stopped: {r.stderr.strip().splitlines()[-1][:100]}"
        for suffix, want in ((".q_row", q), (".s_row", s), (".q_colT", qT), (".s_colT", sT)):
            if not np.array_equal(np.fromfile(prefix + suffix, np.uint8), want.ravel()):
                return f"wrong bytes in {suffix[1:]} of '{head}'"
    return None


def main():
    source = open(os.path.join(ROOT, "paper_2506_08027_amd", "csrc", "gemm.hip")).read()
    survivors = 0
    todo = [("(unmutated source: must pass)", "", "", 0), ("(unmutated source, persistent kernel: must pass)", "", "", 1)]
    todo += [m + (0,) for m in MUTANTS] + [m + (1,) for m in PERSISTENT_MUTANTS]
    only = sys.argv[1:]
    for desc, old, new, persistent in todo:   # every pattern must still be in the source: a stale one would test nothing
        assert old == "" or old in source, desc
    for desc, old, new, persistent in todo:
        if only and not any(o in desc for o in only):
            continue
        assert old == "" or old in source, desc
        work = tempfile.mkdtemp(prefix="kmut_")
        try:
            if old == "":
                text = source
            elif persistent:
                at = source.rindex(old)
                text = source[:at] + new + source[at + len(old):]
            else:
                text = source.replace(old, new, 1)
            how = caught(build(work, text), work, persistent)
        finally:
            shutil.rmtree(work, ignore_errors=True)
        ok = (how is None) if old == "" else (how is not None)
        survivors += not ok
        print(("ok      " if ok else "PROBLEM ") + desc + (f" -> {how}" if how else ""), flush=True)
    csrc = os.path.join(ROOT, "paper_2506_08027_amd", "csrc")
    quant = [("(unmutated converters: must pass)", "gemm.hip", "", "")] + QUANT_MUTANTS
    for desc, name, old, new in quant:
        assert old == "" or old in open(os.path.join(csrc, name)).read(), desc
    for desc, name, old, new in quant:
        if only and not any(o in desc for o in only):
            continue
        text = open(os.path.join(csrc, name)).read()
        work = tempfile.mkdtemp(prefix="kmut_")
        try:
            how = caught_quant(build(work, text.replace(old, new, 1) if old else text, name), work)
        finally:
            shutil.rmtree(work, ignore_errors=True)
        ok = (how is None) if old == "" else (how is not None)
        survivors += not ok
        print(("ok      " if ok else "PROBLEM ") + desc + (f" -> {how}" if how else ""), flush=True)
    sys.exit(1 if survivors else 0)


if __name__ == "__main__":
    main()
