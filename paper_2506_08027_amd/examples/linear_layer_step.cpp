// One MXFP8 linear-layer step through the C ABI alone (no Python, no PyTorch): quantize X, W and dY along both axes,
// run the forward, activation-gradient and weight-gradient products (Section 3.2, Figure 2: which copy feeds which
// product), decode X again, and check samples of every result on the host against the block-scaled sums of Section 2
// computed from the very bytes the library produced.
//
//   hipcc --offload-arch=gfx950 linear_layer_step.cpp -I ../../include -L .. -lmxfp8 -Wl,-rpath,'$ORIGIN/..' -o linear_layer_step
//   ./linear_layer_step [tokens hidden out]        (multiples of 128; default 1024 512 768)
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "mxfp8.h"

#define HIP_OK(call)                                                                      \
    do {                                                                                  \
        const hipError_t e_ = (call);                                                     \
        if (e_ != hipSuccess) {                                                           \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));             \
            return 2;                                                                     \
        }                                                                                 \
    } while (0)
#define MX_OK(call)                                                                       \
    do {                                                                                  \
        const mxfp8_status s_ = (call);                                                   \
        if (s_ != MXFP8_OK) {                                                             \
            fprintf(stderr, "%s failed: %s\n", #call, mxfp8_status_string(s_));           \
            return 3;                                                                     \
        }                                                                                 \
    } while (0)

// E4M3 (Table 1): sign, 4 exponent bits (bias 7), 3 mantissa bits; exponent field 0 is subnormal; 0x7F is NaN
static double e4m3(uint8_t c)
{
    const int e = (c >> 3) & 15, m = c & 7;
    if (e == 15 && m == 7)
        return NAN;
    const double mag = e == 0 ? std::ldexp(m / 8.0, -6) : std::ldexp(1.0 + m / 8.0, e - 7);
    return (c & 0x80) ? -mag : mag;
}

// position of scale byte (row r, block b) in the tiled layout of an operand with nb blocks per row
static size_t tiled(int64_t r, int64_t b, int64_t nb)
{
    return (size_t)((((r >> 6) * ((nb + 3) / 4) + (b >> 2)) * 64 + (r & 63)) * 4 + (b & 3));
}

struct Operand {  // one quantized copy on the device, and, after fetch(), on the host
    uint8_t *q = nullptr, *s = nullptr;
    int64_t rows = 0, cols = 0;
    std::vector<uint8_t> hq, hs;
    hipError_t alloc(int64_t r, int64_t c)
    {
        rows = r;
        cols = c;
        hipError_t e = hipMalloc(&q, (size_t)(r * c));
        return e != hipSuccess ? e : hipMalloc(&s, (size_t)mxfp8_scale_bytes(r, c, MXFP8_SCALES_TILED));
    }
    hipError_t fetch()
    {
        hq.resize((size_t)(rows * cols));
        hs.resize((size_t)mxfp8_scale_bytes(rows, cols, MXFP8_SCALES_TILED));
        hipError_t e = hipMemcpy(hq.data(), q, hq.size(), hipMemcpyDeviceToHost);
        return e != hipSuccess ? e : hipMemcpy(hs.data(), s, hs.size(), hipMemcpyDeviceToHost);
    }
    double at(int64_t r, int64_t k) const  // decoded element: Q * 2^(scale - 127)
    {
        return e4m3(hq[(size_t)(r * cols + k)]) * std::ldexp(1.0, (int)hs[tiled(r, k / 32, cols / 32)] - 127);
    }
};

static double dot(const Operand &a, int64_t m, const Operand &b, int64_t n)
{
    double sum = 0;
    for (int64_t k = 0; k < a.cols; ++k)
        sum += a.at(m, k) * b.at(n, k);
    return sum;
}

static uint16_t to_bf16(float x)  // round to nearest even
{
    uint32_t u;
    memcpy(&u, &x, 4);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
static float from_bf16(uint16_t h)
{
    const uint32_t u = (uint32_t)h << 16;
    float x;
    memcpy(&x, &u, 4);
    return x;
}

int main(int argc, char **argv)
{
    const int64_t T = argc > 3 ? atoll(argv[1]) : 1024, H = argc > 3 ? atoll(argv[2]) : 512, O = argc > 3 ? atoll(argv[3]) : 768;
    if (T <= 0 || H <= 0 || O <= 0 || T % 128 || H % 128 || O % 128) {
        fprintf(stderr, "sizes must be positive multiples of 128\n");
        return 1;
    }
    // ---- deterministic inputs: X, W in BF16, dY in FP32
    uint32_t seed = 12345u;
    auto rnd = [&]() { seed = seed * 1664525u + 1013904223u; return ((seed >> 8) & 0xFFFF) / 32768.0f - 1.0f; };
    std::vector<uint16_t> hx((size_t)(T * H)), hw((size_t)(O * H));
    std::vector<float> hdy((size_t)(T * O));
    for (auto &v : hx) v = to_bf16(2.0f * rnd());
    for (auto &v : hw) v = to_bf16(0.05f * rnd());
    for (auto &v : hdy) v = 1e-3f * rnd();
    void *x = nullptr, *w = nullptr, *dy = nullptr, *y = nullptr, *dx = nullptr, *dw = nullptr, *xback = nullptr;
    HIP_OK(hipMalloc(&x, hx.size() * 2));
    HIP_OK(hipMalloc(&w, hw.size() * 2));
    HIP_OK(hipMalloc(&dy, hdy.size() * 4));
    HIP_OK(hipMalloc(&y, (size_t)(T * O) * 2));      // BF16
    HIP_OK(hipMalloc(&dx, (size_t)(T * H) * 2));     // BF16
    HIP_OK(hipMalloc(&dw, (size_t)(O * H) * 4));     // FP32
    HIP_OK(hipMalloc(&xback, (size_t)(T * H) * 2));  // BF16
    HIP_OK(hipMemcpy(x, hx.data(), hx.size() * 2, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(w, hw.data(), hw.size() * 2, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dy, hdy.data(), hdy.size() * 4, hipMemcpyHostToDevice));

    // ---- both copies of every tensor (Section 3.2): row copy [rows x cols], column copy stored transposed [cols x rows]
    Operand x_row, x_colT, w_row, w_colT, dy_row, dy_colT;
    HIP_OK(x_row.alloc(T, H));
    HIP_OK(x_colT.alloc(H, T));
    HIP_OK(w_row.alloc(O, H));
    HIP_OK(w_colT.alloc(H, O));
    HIP_OK(dy_row.alloc(T, O));
    HIP_OK(dy_colT.alloc(O, T));
    const mxfp8_scale_layout lay = MXFP8_SCALES_TILED;
    hipStream_t stream = nullptr;
    MX_OK(mxfp8_quantize_ex(x, MXFP8_BF16, T, H, H, MXFP8_BOTH, x_row.q, x_row.s, x_colT.q, x_colT.s, lay, stream));
    MX_OK(mxfp8_quantize_ex(w, MXFP8_BF16, O, H, H, MXFP8_BOTH, w_row.q, w_row.s, w_colT.q, w_colT.s, lay, stream));
    MX_OK(mxfp8_quantize_ex(dy, MXFP8_F32, T, O, O, MXFP8_BOTH, dy_row.q, dy_row.s, dy_colT.q, dy_colT.s, lay, stream));
    // ---- the three products, each C = A . B^T over K-contiguous operands
    //   forward:              Y  [T x O] = X  . W^T      A = row copy of X,       B = row copy of W        (K = H)
    //   activation gradient:  dX [T x H] = dY . W        A = row copy of dY,      B = column copy of W     (K = O)
    //   weight gradient:      dW [O x H] = dY^T . X      A = column copy of dY,   B = column copy of X     (K = T)
    MX_OK(mxfp8_gemm_ex(MXFP8_FPROP, x_row.q, x_row.s, w_row.q, w_row.s, T, O, H, y, MXFP8_BF16, O, lay, 0, stream));
    MX_OK(mxfp8_gemm_ex(MXFP8_DGRAD, dy_row.q, dy_row.s, w_colT.q, w_colT.s, T, H, O, dx, MXFP8_BF16, H, lay, 0, stream));
    MX_OK(mxfp8_gemm_ex(MXFP8_WGRAD, dy_colT.q, dy_colT.s, x_colT.q, x_colT.s, O, H, T, dw, MXFP8_F32, H, lay, 0, stream));
    MX_OK(mxfp8_dequantize_ex(x_row.q, x_row.s, T, H, xback, MXFP8_BF16, H, lay, stream));
    HIP_OK(hipStreamSynchronize(stream));

    // ---- host check of samples: the products against the decoded bytes, the decode against the source
    for (Operand *op : {&x_row, &x_colT, &w_row, &w_colT, &dy_row, &dy_colT})
        HIP_OK(op->fetch());
    std::vector<uint16_t> hy((size_t)(T * O)), hdx((size_t)(T * H)), hxb((size_t)(T * H));
    std::vector<float> hdw((size_t)(O * H));
    HIP_OK(hipMemcpy(hy.data(), y, hy.size() * 2, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hdx.data(), dx, hdx.size() * 2, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hdw.data(), dw, hdw.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hxb.data(), xback, hxb.size() * 2, hipMemcpyDeviceToHost));
    int bad = 0;
    auto check = [&](const char *what, double got, double want, double tol) {
        if (!(std::fabs(got - want) <= tol)) {
            if (bad++ < 10)
                fprintf(stderr, "%s: got %.9g, expected %.9g (tolerance %.3g)\n", what, got, want, tol);
        }
    };
    for (int i = 0; i < 64; ++i) {
        const int64_t t = (i * 131) % T, o = (i * 197) % O, h = (i * 89) % H;
        const double yv = dot(x_row, t, w_row, o), dxv = dot(dy_row, t, w_colT, h), dwv = dot(dy_colT, o, x_colT, h);
        // BF16 outputs carry one rounding to 8 significant bits; the absolute terms cover the matrix instruction's own
        // error, which scales with the sum of the magnitudes of the products rather than with the result
        check("Y", from_bf16(hy[(size_t)(t * O + o)]), yv, std::fabs(yv) / 128 + 5e-3);
        check("dX", from_bf16(hdx[(size_t)(t * H + h)]), dxv, std::fabs(dxv) / 128 + 1e-5);
        check("dW", hdw[(size_t)(o * H + h)], dwv, std::fabs(dwv) / 1024 + 2e-4);
        // decode of the row copy: within one E4M3 step (2^-3 relative) of the source, and exactly the decoded byte
        const double src = from_bf16(hx[(size_t)(t * H + h)]), back = from_bf16(hxb[(size_t)(t * H + h)]);
        check("decode", back, x_row.at(t, h), 0.0);
        check("round trip", back, src, std::fabs(src) / 8 + 0.05);
    }
    if (bad) {
        fprintf(stderr, "%d sampled values disagree\n", bad);
        return 4;
    }
    printf("linear layer step ok: T=%lld H=%lld O=%lld, 64 samples of Y, dX, dW and the decoded X agree with the host sums\n",
           (long long)T, (long long)H, (long long)O);
    return 0;
}
