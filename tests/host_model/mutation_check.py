"""Sensitivity check of the CPU execution model (test infrastructure; `python tests/host_model/mutation_check.py`,
or tests/test_mutation_checks.py with --runslow). Plants one mistake at a time into a scratch
copy of the GEMM kernel source -- a removed barrier, a wait count that is one too loose, a missing wait,
a swizzle mismatch, a prefetch into the wrong buffer or of the wrong K step, a missing ragged-tile clamp,
a wrong output row -- builds the host model from it and runs a few products against the oracle in all
four scheduling modes (lazy / eager DMA completion, either wavefront running ahead). Every mutant must
be caught, by a wrong or NaN result or by the model's range check. Arguments, if any, select the mutants
whose description contains one of them."""
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


def build(work, gemm_text):
    csrc = os.path.join(work, "csrc")
    shutil.copytree(os.path.join(ROOT, "paper_2506_08027_amd", "csrc"), csrc)
    open(os.path.join(csrc, "gemm.hip"), "w").write(gemm_text)
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
    sys.exit(1 if survivors else 0)


if __name__ == "__main__":
    main()
