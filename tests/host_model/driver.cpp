// Runs the library's C ABI on the CPU execution model (tests/host_model/wavesim.h): reads a list
// of calls from a text file, feeds them binary inputs, writes the outputs back as files.
// Every buffer is an exact-size heap block (AddressSanitizer guards its ends), outputs start out
// filled with 0xA5, and inputs are checked to be unchanged after the call.
//
//   quantize   <f32|bf16> <rows> <cols> <ld> <axis 1|2|3> <src.bin> <out-prefix> [tiled]
//   gemm       <pass 0|1|2> <M> <N> <K> <f32|bf16> <ldc> <a_q> <a_s> <b_q> <b_s> <c.bin> [tiled]
//   dequantize <rows> <cols> <f32|bf16> <ld> <q.bin> <s.bin> <out.bin> [tiled]
//   gemmbf16   <M> <N> <K> <f32|bf16> <ldc> <a.bin> <b.bin> <c.bin>      (BF16 operands, no scales)
//   gemmgrp    <M> <N> <K> <f32|bf16> <ldc> <groups> <a_q> <a_s> <b_q> <b_s> <ends.bin (int32)> <c.bin> [tiled]
//              (b_q = groups x N x K bytes, b_s = groups scale operands; rows outside every group keep 0xA5)
//   gemmgrpk   <M> <N> <K> <f32|bf16> <ldc> <groups> <a_q> <a_s> <b_q> <b_s> <ends.bin (int32)> <c.bin> [tiled]
//              (weight-gradient form: the ends split K; c = groups x M x ldc elements)
//   requant    <rows> <cols> <q_row.bin> <s_row.bin> <out-prefix> [tiled]   (column copy from the row copy: .q_colT .s_colT)
//   copy       <bytes> <workgroups> <mode 0|1|2> <src.bin> <dst.bin>      (the plain-copy rate probe)
//   gemmq      <pass 0|1|2> <M> <N> <K> <ldc> <axis 1|2|3> <a_q> <a_s> <b_q> <b_s> <out-prefix> [tiled]
//              (BF16 product <prefix>.c plus the MXFP8 copies of it: .q_row .s_row .q_colT .s_colT)
// "tiled" selects MXFP8_SCALES_TILED for every scale buffer of the call (sizes from mxfp8_scale_bytes);
// "wg=<n>" is the max_workgroups argument of gemm / gemmq (default 0 = one per compute unit).
// Each call prints "status <code> blocks <ids of the simulated workgroups...>".
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <fstream>
#include <sstream>
#include <string>
#include <vector>

#include "../../include/mxfp8.h"
#include "wavesim.h"

// buffers live until the process ends and fiber stacks are reused across launches: no leak report wanted
extern "C" const char *__asan_default_options() { return "detect_leaks=0:detect_stack_use_after_return=0"; }

namespace {

struct Buf {
    uint8_t *p = nullptr;
    size_t n = 0;
    std::vector<uint8_t> copy;
};

Buf load(const std::string &path, size_t expect)
{
    Buf b;
    FILE *f = fopen(path.c_str(), "rb");
    if (!f) {
        fprintf(stderr, "cannot open %s\n", path.c_str());
        exit(2);
    }
    fseek(f, 0, SEEK_END);
    b.n = (size_t)ftell(f);
    fseek(f, 0, SEEK_SET);
    if (b.n != expect) {
        fprintf(stderr, "%s holds %zu bytes, the call needs %zu\n", path.c_str(), b.n, expect);
        exit(2);
    }
    b.p = b.n ? (uint8_t *)aligned_alloc(16, (b.n + 15) / 16 * 16) : nullptr;
    // aligned_alloc rounds the size up; re-allocate exactly when that would hide an overrun
    if (b.n % 16) {
        free(b.p);
        void *q = nullptr;
        if (posix_memalign(&q, 16, b.n) != 0)
            exit(2);
        b.p = (uint8_t *)q;
    }
    if (b.n && fread(b.p, 1, b.n, f) != b.n)
        exit(2);
    fclose(f);
    b.copy.assign(b.p, b.p + b.n);
    wavesim::register_buffer(b.p, b.n, path.c_str());
    return b;
}

Buf output(size_t n)
{
    Buf b;
    b.n = n;
    if (n) {
        void *q = nullptr;
        if (posix_memalign(&q, 16, n) != 0)
            exit(2);
        b.p = (uint8_t *)q;
        memset(b.p, 0xA5, n);
        wavesim::register_buffer(b.p, n, "output");
    }
    return b;
}

void save(const std::string &path, const Buf &b)
{
    FILE *f = fopen(path.c_str(), "wb");
    if (!f || (b.n && fwrite(b.p, 1, b.n, f) != b.n)) {
        fprintf(stderr, "cannot write %s\n", path.c_str());
        exit(2);
    }
    fclose(f);
}

void unchanged(const Buf &b, const char *what)
{
    if (b.n && memcmp(b.p, b.copy.data(), b.n) != 0) {
        fprintf(stderr, "the call modified its input %s\n", what);
        exit(4);
    }
}

mxfp8_dtype dtype_of(const std::string &s)
{
    if (s == "f32")
        return MXFP8_F32;
    if (s == "bf16")
        return MXFP8_BF16;
    fprintf(stderr, "unknown dtype %s\n", s.c_str());
    exit(2);
}

int g_max_workgroups = 0;  // "wg=<n>" of the current line

mxfp8_scale_layout layout_of(std::istringstream &ls)
{
    std::string tok;
    mxfp8_scale_layout lay = MXFP8_SCALES_ROWMAJOR;
    g_max_workgroups = 0;
    while (ls >> tok) {
        if (tok == "tiled") {
            lay = MXFP8_SCALES_TILED;
        } else if (tok.rfind("wg=", 0) == 0) {
            g_max_workgroups = atoi(tok.c_str() + 3);
        } else {
            fprintf(stderr, "unknown trailing token %s\n", tok.c_str());
            exit(2);
        }
    }
    return lay;
}

void report(int status)
{
    printf("status %d blocks", status);
    if (status == 0)
        for (unsigned b : wavesim::g.simulated)
            printf(" %u", b);
    printf("\n");
    fflush(stdout);
}

}  // namespace

int main(int argc, char **argv)
{
    if (argc != 2) {
        fprintf(stderr, "usage: %s <case file>\n", argv[0]);
        return 2;
    }
    std::ifstream in(argv[1]);
    std::string line;
    while (std::getline(in, line)) {
        std::istringstream ls(line);
        std::string op;
        if (!(ls >> op) || op[0] == '#')
            continue;
        wavesim::clear_buffers();
        wavesim::g.simulated.clear();
        if (op == "quantize") {
            std::string dt, src, prefix;
            long rows, cols, ld;
            int axis;
            ls >> dt >> rows >> cols >> ld >> axis >> src >> prefix;
            const mxfp8_scale_layout lay = layout_of(ls);
            const size_t es = dt == "bf16" ? 2 : 4;
            // the source spans (rows-1)*ld + cols elements: no padding after the last row
            Buf s = load(src, rows > 0 ? ((size_t)(rows - 1) * ld + cols) * es : 0);
            const bool r = axis & 1, c = axis & 2;
            Buf qr = output(r ? (size_t)rows * cols : 0), sr = output(r ? (size_t)mxfp8_scale_bytes(rows, cols, lay) : 0);
            Buf qc = output(c ? (size_t)rows * cols : 0), sc = output(c ? (size_t)mxfp8_scale_bytes(cols, rows, lay) : 0);
            const int st = mxfp8_quantize_ex(s.p, dtype_of(dt), rows, cols, ld, (mxfp8_axis)axis, qr.p, sr.p, qc.p, sc.p,
                                             lay, nullptr);
            unchanged(s, "src");
            report(st);
            if (r) {
                save(prefix + ".q_row", qr);
                save(prefix + ".s_row", sr);
            }
            if (c) {
                save(prefix + ".q_colT", qc);
                save(prefix + ".s_colT", sc);
            }
        } else if (op == "gemm") {
            int pass;
            long M, N, K, ldc;
            std::string dt, aq, as, bq, bs, cout;
            ls >> pass >> M >> N >> K >> dt >> ldc >> aq >> as >> bq >> bs >> cout;
            const mxfp8_scale_layout lay = layout_of(ls);
            const size_t es = dt == "bf16" ? 2 : 4;
            Buf a = load(aq, (size_t)M * K), sa = load(as, (size_t)mxfp8_scale_bytes(M, K, lay));
            Buf b = load(bq, (size_t)N * K), sb = load(bs, (size_t)mxfp8_scale_bytes(N, K, lay));
            Buf c = output(M > 0 ? ((size_t)(M - 1) * ldc + N) * es : 0);
            const int st = mxfp8_gemm_ex((mxfp8_pass)pass, a.p, sa.p, b.p, sb.p, M, N, K, c.p, dtype_of(dt), ldc, lay, g_max_workgroups, nullptr);
            unchanged(a, "a_q");
            unchanged(sa, "a_s");
            unchanged(b, "b_q");
            unchanged(sb, "b_s");
            report(st);
            save(cout, c);
        } else if (op == "gemmgrp") {
            long M, N, K, ldc, groups;
            std::string dt, aq, as, bq, bs, ends, cout;
            ls >> M >> N >> K >> dt >> ldc >> groups >> aq >> as >> bq >> bs >> ends >> cout;
            const mxfp8_scale_layout lay = layout_of(ls);
            const size_t es = dt == "bf16" ? 2 : 4;
            Buf a = load(aq, (size_t)M * K), sa = load(as, (size_t)mxfp8_scale_bytes(M, K, lay));
            Buf b = load(bq, (size_t)groups * N * K), sb = load(bs, (size_t)groups * mxfp8_scale_bytes(N, K, lay));
            Buf e = load(ends, (size_t)groups * 4);
            Buf c = output(M > 0 ? ((size_t)(M - 1) * ldc + N) * es : 0);
            const int st = mxfp8_gemm_grouped_ex(MXFP8_FPROP, a.p, sa.p, b.p, sb.p, (const int32_t *)e.p, (int32_t)groups, M, N, K,
                                                 c.p, dtype_of(dt), ldc, lay, g_max_workgroups, nullptr);
            unchanged(a, "a_q");
            unchanged(sa, "a_s");
            unchanged(b, "b_q");
            unchanged(sb, "b_s");
            unchanged(e, "group_ends");
            report(st);
            save(cout, c);
        } else if (op == "gemmgrpk") {
            long M, N, K, ldc, groups;
            std::string dt, aq, as, bq, bs, ends, cout;
            ls >> M >> N >> K >> dt >> ldc >> groups >> aq >> as >> bq >> bs >> ends >> cout;
            const mxfp8_scale_layout lay = layout_of(ls);
            const size_t es = dt == "bf16" ? 2 : 4;
            Buf a = load(aq, (size_t)M * K), sa = load(as, (size_t)mxfp8_scale_bytes(M, K, lay));
            Buf b = load(bq, (size_t)N * K), sb = load(bs, (size_t)mxfp8_scale_bytes(N, K, lay));
            Buf e = load(ends, (size_t)groups * 4);
            Buf c = output(M > 0 && groups > 0 ? (((size_t)groups * M - 1) * ldc + N) * es : 0);
            const int st = mxfp8_gemm_grouped_ex(MXFP8_WGRAD, a.p, sa.p, b.p, sb.p, (const int32_t *)e.p, (int32_t)groups, M, N, K,
                                                 c.p, dtype_of(dt), ldc, lay, 0, nullptr);
            unchanged(a, "a_q");
            unchanged(sa, "a_s");
            unchanged(b, "b_q");
            unchanged(sb, "b_s");
            unchanged(e, "group_ends");
            report(st);
            save(cout, c);
        } else if (op == "requant") {
            long rows, cols;
            std::string q, sc, prefix;
            ls >> rows >> cols >> q >> sc >> prefix;
            const mxfp8_scale_layout lay = layout_of(ls);
            Buf qb = load(q, (size_t)rows * cols), sb = load(sc, (size_t)mxfp8_scale_bytes(rows, cols, lay));
            Buf qc = output((size_t)rows * cols), scT = output((size_t)mxfp8_scale_bytes(cols, rows, lay));
            const int st = mxfp8_requantize_colwise_ex(qb.p, sb.p, rows, cols, qc.p, scT.p, lay, nullptr);
            unchanged(qb, "q_row");
            unchanged(sb, "s_row");
            report(st);
            save(prefix + ".q_colT", qc);
            save(prefix + ".s_colT", scT);
        } else if (op == "copy") {
            long bytes, wgs, mode;
            std::string src, dst;
            ls >> bytes >> wgs >> mode >> src >> dst;
            Buf a = load(src, (size_t)bytes);
            Buf d = output((size_t)bytes);
            const int st = mxfp8_copy_rate_probe(a.p, d.p, bytes, (int32_t)wgs, (int32_t)mode, nullptr);
            unchanged(a, "src");
            report(st);
            save(dst, d);
        } else if (op == "gemmbf16") {
            long M, N, K, ldc;
            std::string dt, af, bf, cout;
            ls >> M >> N >> K >> dt >> ldc >> af >> bf >> cout;
            layout_of(ls);  // only wg=<n> means something here
            const size_t es = dt == "bf16" ? 2 : 4;
            Buf a = load(af, (size_t)M * K * 2), b = load(bf, (size_t)N * K * 2);
            Buf c = output(M > 0 ? ((size_t)(M - 1) * ldc + N) * es : 0);
            const int st = mxfp8_gemm_bf16(a.p, b.p, M, N, K, c.p, dtype_of(dt), ldc, g_max_workgroups, nullptr);
            unchanged(a, "a");
            unchanged(b, "b");
            report(st);
            save(cout, c);
        } else if (op == "gemmq") {
            int pass, axis;
            long M, N, K, ldc;
            std::string aq, as, bq, bs, prefix;
            ls >> pass >> M >> N >> K >> ldc >> axis >> aq >> as >> bq >> bs >> prefix;
            const mxfp8_scale_layout lay = layout_of(ls);
            Buf a = load(aq, (size_t)M * K), sa = load(as, (size_t)mxfp8_scale_bytes(M, K, lay));
            Buf b = load(bq, (size_t)N * K), sb = load(bs, (size_t)mxfp8_scale_bytes(N, K, lay));
            Buf c = output(M > 0 ? ((size_t)(M - 1) * ldc + N) * 2 : 0);
            const bool r = axis & 1, t = axis & 2;
            Buf qr = output(r ? (size_t)M * N : 0), sr = output(r ? (size_t)mxfp8_scale_bytes(M, N, lay) : 0);
            Buf qc = output(t ? (size_t)M * N : 0), sc = output(t ? (size_t)mxfp8_scale_bytes(N, M, lay) : 0);
            const int st = mxfp8_gemm_quantize_ex((mxfp8_pass)pass, a.p, sa.p, b.p, sb.p, M, N, K, c.p, ldc, (mxfp8_axis)axis,
                                                  qr.p, sr.p, qc.p, sc.p, lay, g_max_workgroups, nullptr);
            unchanged(a, "a_q");
            unchanged(sa, "a_s");
            unchanged(b, "b_q");
            unchanged(sb, "b_s");
            report(st);
            save(prefix + ".c", c);
            if (r) {
                save(prefix + ".q_row", qr);
                save(prefix + ".s_row", sr);
            }
            if (t) {
                save(prefix + ".q_colT", qc);
                save(prefix + ".s_colT", sc);
            }
        } else if (op == "dequantize") {
            long rows, cols, ld;
            std::string dt, q, s, out;
            ls >> rows >> cols >> dt >> ld >> q >> s >> out;
            const mxfp8_scale_layout lay = layout_of(ls);
            const size_t es = dt == "bf16" ? 2 : 4;
            Buf qb = load(q, (size_t)rows * cols), sb = load(s, (size_t)mxfp8_scale_bytes(rows, cols, lay));
            Buf o = output(rows > 0 ? ((size_t)(rows - 1) * ld + cols) * es : 0);
            const int st = mxfp8_dequantize_ex(qb.p, sb.p, rows, cols, o.p, dtype_of(dt), ld, lay, nullptr);
            unchanged(qb, "q");
            unchanged(sb, "s");
            report(st);
            save(out, o);
        } else if (op == "gemmmode") {
            int pass, ea, eb;
            long M, N, K, ldc;
            std::string dt, aq, as, bq, bs, cout;
            ls >> pass >> M >> N >> K >> ea >> eb >> dt >> ldc >> aq >> as >> bq >> bs >> cout;
            const mxfp8_scale_layout lay = layout_of(ls);
            const size_t es = dt == "bf16" ? 2 : 4;
            Buf a = load(aq, (size_t)M * K), sa = load(as, (size_t)mxfp8_scale_bytes(M, K, lay));
            Buf b = load(bq, (size_t)N * K), sb = load(bs, (size_t)mxfp8_scale_bytes(N, K, lay));
            Buf c = output(M > 0 ? ((size_t)(M - 1) * ldc + N) * es : 0);
            const int st = mxfp8_gemm_mode_ex((mxfp8_pass)pass, a.p, sa.p, (mxfp8_element)ea, b.p, sb.p, (mxfp8_element)eb, M, N, K, c.p,
                                              dtype_of(dt), ldc, lay, g_max_workgroups, nullptr);
            unchanged(a, "a_q");
            unchanged(sa, "a_s");
            unchanged(b, "b_q");
            unchanged(sb, "b_s");
            report(st);
            save(cout, c);
        } else if (op == "gemmfp4") {
            int pass;
            long M, N, K, ldc;
            std::string dt, aq, as, bq, bs, cout;
            ls >> pass >> M >> N >> K >> dt >> ldc >> aq >> as >> bq >> bs >> cout;
            const mxfp8_scale_layout lay = layout_of(ls);
            const size_t es = dt == "bf16" ? 2 : 4;
            Buf a = load(aq, (size_t)M * K / 2), sa = load(as, (size_t)mxfp8_scale_bytes(M, K, lay));
            Buf b = load(bq, (size_t)N * K / 2), sb = load(bs, (size_t)mxfp8_scale_bytes(N, K, lay));
            Buf c = output(M > 0 ? ((size_t)(M - 1) * ldc + N) * es : 0);
            const int st = mxfp8_fp4_gemm_ex((mxfp8_pass)pass, a.p, sa.p, b.p, sb.p, M, N, K, c.p, dtype_of(dt), ldc, lay,
                                             g_max_workgroups, nullptr);
            unchanged(a, "a_q");
            unchanged(sa, "a_s");
            unchanged(b, "b_q");
            unchanged(sb, "b_s");
            report(st);
            save(cout, c);
        } else if (op == "quantfp6") {
            std::string dt, src, prefix;
            long rows, cols, ld;
            int axis, element;
            ls >> dt >> rows >> cols >> ld >> axis >> element >> src >> prefix;
            const mxfp8_scale_layout lay = layout_of(ls);
            const size_t es = dt == "bf16" ? 2 : 4;
            Buf s = load(src, rows > 0 ? ((size_t)(rows - 1) * ld + cols) * es : 0);
            const bool r = axis & 1, c = axis & 2;
            Buf qr = output(r ? (size_t)rows * cols / 4 * 3 : 0), sr = output(r ? (size_t)mxfp8_scale_bytes(rows, cols, lay) : 0);
            Buf qc = output(c ? (size_t)rows * cols / 4 * 3 : 0), sc = output(c ? (size_t)mxfp8_scale_bytes(cols, rows, lay) : 0);
            const int st = mxfp8_fp6_quantize_ex(s.p, dtype_of(dt), rows, cols, ld, (mxfp8_axis)axis, (mxfp8_fp6_element)element,
                                                 qr.p, sr.p, qc.p, sc.p, lay, nullptr);
            unchanged(s, "src");
            report(st);
            if (r) {
                save(prefix + ".q_row", qr);
                save(prefix + ".s_row", sr);
            }
            if (c) {
                save(prefix + ".q_colT", qc);
                save(prefix + ".s_colT", sc);
            }
        } else if (op == "dequantfp6") {
            long rows, cols, ld;
            int element;
            std::string dt, q, s, out;
            ls >> rows >> cols >> element >> dt >> ld >> q >> s >> out;
            const mxfp8_scale_layout lay = layout_of(ls);
            const size_t es = dt == "bf16" ? 2 : 4;
            Buf qb = load(q, (size_t)rows * cols / 4 * 3), sb = load(s, (size_t)mxfp8_scale_bytes(rows, cols, lay));
            Buf o = output(rows > 0 ? ((size_t)(rows - 1) * ld + cols) * es : 0);
            const int st = mxfp8_fp6_dequantize_ex(qb.p, sb.p, rows, cols, (mxfp8_fp6_element)element, o.p, dtype_of(dt), ld, lay, nullptr);
            unchanged(qb, "q");
            unchanged(sb, "s");
            report(st);
            save(out, o);
        } else if (op == "expandfp6") {
            long rows, cols;
            int element;
            std::string q, out;
            ls >> rows >> cols >> element >> q >> out;
            Buf qb = load(q, (size_t)rows * cols / 4 * 3);
            Buf o = output((size_t)rows * cols);
            const int st = mxfp8_fp6_expand_ex(qb.p, rows, cols, (mxfp8_fp6_element)element, o.p, nullptr);
            unchanged(qb, "q");
            report(st);
            save(out, o);
        } else if (op == "quantfp4") {
            std::string dt, src, prefix;
            long rows, cols, ld;
            int axis;
            ls >> dt >> rows >> cols >> ld >> axis >> src >> prefix;
            const mxfp8_scale_layout lay = layout_of(ls);
            const size_t es = dt == "bf16" ? 2 : 4;
            Buf s = load(src, rows > 0 ? ((size_t)(rows - 1) * ld + cols) * es : 0);
            const bool r = axis & 1, c = axis & 2;
            Buf qr = output(r ? (size_t)rows * cols / 2 : 0), sr = output(r ? (size_t)mxfp8_scale_bytes(rows, cols, lay) : 0);
            Buf qc = output(c ? (size_t)rows * cols / 2 : 0), sc = output(c ? (size_t)mxfp8_scale_bytes(cols, rows, lay) : 0);
            const int st = mxfp8_fp4_quantize_ex(s.p, dtype_of(dt), rows, cols, ld, (mxfp8_axis)axis, qr.p, sr.p, qc.p, sc.p,
                                                 lay, nullptr);
            unchanged(s, "src");
            report(st);
            if (r) {
                save(prefix + ".q_row", qr);
                save(prefix + ".s_row", sr);
            }
            if (c) {
                save(prefix + ".q_colT", qc);
                save(prefix + ".s_colT", sc);
            }
        } else if (op == "dequantfp4") {
            long rows, cols, ld;
            std::string dt, q, s, out;
            ls >> rows >> cols >> dt >> ld >> q >> s >> out;
            const mxfp8_scale_layout lay = layout_of(ls);
            const size_t es = dt == "bf16" ? 2 : 4;
            Buf qb = load(q, (size_t)rows * cols / 2), sb = load(s, (size_t)mxfp8_scale_bytes(rows, cols, lay));
            Buf o = output(rows > 0 ? ((size_t)(rows - 1) * ld + cols) * es : 0);
            const int st = mxfp8_fp4_dequantize_ex(qb.p, sb.p, rows, cols, o.p, dtype_of(dt), ld, lay, nullptr);
            unchanged(qb, "q");
            unchanged(sb, "s");
            report(st);
            save(out, o);
        } else {
            fprintf(stderr, "unknown operation %s\n", op.c_str());
            return 2;
        }
    }
    return 0;
}
