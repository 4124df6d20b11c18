/*
 * MXFP8 (E4M3 elements, UE8M0 block scales, K = 32) reference arithmetic on the CPU.
 *
 * THIS FILE IS TEST INFRASTRUCTURE. It is the plain, slow definition that the GPU library is
 * checked against. Only the tests, the smoke check and the benchmark's cpu_baseline leg may call
 * it; the product (the HIP library and its Python binding) never does, and the two share no code.
 *
 * Everything is the paper's definition written out in double precision, which holds every FP32
 * value, every 448 * 2^n for n in [-127, 127] and every V * 2^-n exactly:
 *   - format constants: Section 2 and Table 1 (K = 32, UE8M0 in 2^-127..2^127 or NaN, E4M3 with
 *     max normal 1.75 * 2^8, min subnormal 2^-9, one NaN pattern per sign, no Inf);
 *   - scale: Section 3.3 Algorithm 1 and Appendix A.1 (ratio amax/destmax rounded UP to a power of
 *     two, lower clamp 2^-127), evaluated as "smallest n with amax <= 448 * 2^n" so that no log2
 *     is ever rounded (Appendix A.1 warns about exactly that);
 *   - elements: Section 3.3 and Appendix A.2 (V_i / X, round to nearest ties to even, saturating);
 *   - decode: Section 2 (value = Q_i * X);
 *   - dot products: Section 2 and Appendix A.3 (per-block products, scale applied per block),
 *     here simply the double-precision product of the decoded operands.
 *
 * Readings where the paper is silent ("parity unpinned": pinned by this project's choice only):
 *   - a block containing a NaN gets scale byte 0xFF and all 32 element bytes 0x7F;
 *   - a block containing +-Inf and no NaN takes Algorithm 1 literally: log2(Inf) clamps to 127,
 *     scale byte 254, Inf elements saturate to +-448, finite elements are divided by 2^127;
 *   - the sign bit of every input is kept (so -0.0 and negative underflows give 0x80).
 * Everything else (scale rule, RNE, saturation, decode, GEMM value) is pinned by the CPU tests.
 *
 * Layouts (row-major everywhere): a source tensor is [rows x cols] with leading dimension ld.
 *   rowwise : q [rows x cols],  s [rows x cols/32]   blocks = 32 consecutive columns of a row
 *   colwise : qT[cols x rows],  sT[cols x rows/32]   blocks = 32 consecutive rows of a column,
 *             stored transposed so that the block is again contiguous.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define MX_K 32

int mxo_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- E4M3 (Section 2, Table 1): 1 sign, 4 exponent (bias 7), 3 mantissa bits. ------------- */

/* Value of one code. Exponent field 0 is subnormal (k * 2^-9); S.1111.111 is NaN; every other
 * code with exponent field 15 is an ordinary number, which is what extends the range to 448. */
double mxo_e4m3_decode(uint8_t code)
{
    int sign = code >> 7;
    int e = (code >> 3) & 0xF;
    int m = code & 0x7;
    double v;
    if (e == 0xF && m == 0x7)
        return NAN;
    if (e == 0)
        v = ldexp((double)m, -9);
    else
        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

/* Quantize_to_fp8 (Section 3.3, Appendix A.2): nearest representable value, ties to the code with
 * an even mantissa LSB, magnitudes beyond the maximum clamp to the maximum. Found by scanning all
 * 127 non-negative finite codes. The two candidate distances that can tie are exact in double
 * (Sterbenz: t and its neighbours are within a factor of two), so the comparison is exact. */
uint8_t mxo_e4m3_encode(double t)
{
    uint8_t sign = signbit(t) ? 0x80 : 0x00;
    double a = fabs(t);
    int best = 0;
    double best_d;
    int c;
    if (isnan(t))
        return 0x7F;
    if (a > 448.0)
        return (uint8_t)(sign | 0x7E);
    best_d = fabs(a - mxo_e4m3_decode(0));
    for (c = 1; c <= 0x7E; ++c) {
        double d = fabs(a - mxo_e4m3_decode((uint8_t)c));
        if (d < best_d || (d == best_d && (c & 1) == 0)) {
            best_d = d;
            best = c;
        }
    }
    return (uint8_t)(sign | best);
}

/* ---- UE8M0 scale (Algorithm 1, Appendix A.1). ---------------------------------------------- */

/* Returns the stored byte n + 127, where 2^n is the smallest power of two in [2^-127, 2^127] with
 * amax / 2^n <= 448, i.e. ceil(log2(amax / 448)) clamped, without evaluating a logarithm.
 * NaN -> 0xFF. +Inf -> no n qualifies, the clamp leaves 127 -> byte 254. */
int mxo_scale_byte(double amax)
{
    int n;
    if (isnan(amax))
        return 0xFF;
    for (n = -127; n < 127; ++n)
        if (amax <= ldexp(448.0, n))
            break;
    return n + 127;
}

static double bf16_to_double(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* One block: v[0..31] (already exact in double) -> 32 element bytes (stride qs) and one scale. */
static void quantize_block(const double *v, uint8_t *q, int64_t qs, uint8_t *s)
{
    double amax = 0.0;
    int has_nan = 0;
    int i, sb, n;
    for (i = 0; i < MX_K; ++i) {
        double a = fabs(v[i]);
        if (isnan(a))
            has_nan = 1;
        else if (a > amax)
            amax = a;
    }
    if (has_nan) {
        *s = 0xFF;
        for (i = 0; i < MX_K; ++i)
            q[i * qs] = 0x7F;
        return;
    }
    sb = mxo_scale_byte(amax);
    n = sb - 127;
    *s = (uint8_t)sb;
    for (i = 0; i < MX_K; ++i)
        q[i * qs] = mxo_e4m3_encode(ldexp(v[i], -n)); /* V_i / X, exact */
}

#define DEFINE_QUANTIZE(NAME, T, WIDEN)                                                          \
    void mxo_quantize_rowwise_##NAME(const T *src, int64_t rows, int64_t cols, int64_t ld,       \
                                     uint8_t *q, uint8_t *s)                                     \
    {                                                                                            \
        int64_t nb = cols / MX_K;                                                                \
        int64_t r;                                                                               \
        _Pragma("omp parallel for schedule(static)") for (r = 0; r < rows; ++r)                  \
        {                                                                                        \
            int64_t b;                                                                           \
            for (b = 0; b < nb; ++b) {                                                           \
                double v[MX_K];                                                                  \
                int i;                                                                           \
                for (i = 0; i < MX_K; ++i)                                                       \
                    v[i] = WIDEN(src[r * ld + b * MX_K + i]);                                    \
                quantize_block(v, q + r * cols + b * MX_K, 1, s + r * nb + b);                   \
            }                                                                                    \
        }                                                                                        \
    }                                                                                            \
    void mxo_quantize_colwise_##NAME(const T *src, int64_t rows, int64_t cols, int64_t ld,       \
                                     uint8_t *qT, uint8_t *sT)                                   \
    {                                                                                            \
        int64_t nb = rows / MX_K;                                                                \
        int64_t c;                                                                               \
        _Pragma("omp parallel for schedule(static)") for (c = 0; c < cols; ++c)                  \
        {                                                                                        \
            int64_t b;                                                                           \
            for (b = 0; b < nb; ++b) {                                                           \
                double v[MX_K];                                                                  \
                int i;                                                                           \
                for (i = 0; i < MX_K; ++i)                                                       \
                    v[i] = WIDEN(src[(b * MX_K + i) * ld + c]);                                  \
                quantize_block(v, qT + c * rows + b * MX_K, 1, sT + c * nb + b);                 \
            }                                                                                    \
        }                                                                                        \
    }

#define WIDEN_F32(x) ((double)(x))
#define WIDEN_BF16(x) bf16_to_double(x)
DEFINE_QUANTIZE(f32, float, WIDEN_F32)
DEFINE_QUANTIZE(bf16, uint16_t, WIDEN_BF16)

/* ---- Decode (Section 2): value = Q_i * X, X = 2^(byte - 127), byte 0xFF = NaN. ------------- */

static double decode_one(uint8_t q, uint8_t s)
{
    if (s == 0xFF)
        return NAN;
    return ldexp(mxo_e4m3_decode(q), (int)s - 127);
}

void mxo_dequantize_f64(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, double *dst)
{
    int64_t nb = cols / MX_K;
    int64_t r;
#pragma omp parallel for schedule(static)
    for (r = 0; r < rows; ++r) {
        int64_t c;
        for (c = 0; c < cols; ++c)
            dst[r * cols + c] = decode_one(q[r * cols + c], s[r * nb + c / MX_K]);
    }
}

/* Decoded value rounded once (to nearest even) to FP32. */
void mxo_dequantize_f32(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, float *dst,
                        int64_t ld)
{
    int64_t nb = cols / MX_K;
    int64_t r;
#pragma omp parallel for schedule(static)
    for (r = 0; r < rows; ++r) {
        int64_t c;
        for (c = 0; c < cols; ++c)
            dst[r * ld + c] = (float)decode_one(q[r * cols + c], s[r * nb + c / MX_K]);
    }
}

/* Round a double once to BF16 (8 exponent, 7 mantissa bits), nearest even, overflow to Inf.
 * Done on the scaled integer significand so that no intermediate FP32 rounding happens. */
static uint16_t double_to_bf16(double x)
{
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double a = fabs(x);
    int e;
    double frac, scaled, fl, rem;
    uint32_t mant;
    int be;
    if (isnan(x))
        return (uint16_t)(sign | 0x7FC0);
    if (a == 0.0)
        return sign;
    if (isinf(a))
        return (uint16_t)(sign | 0x7F80);
    frac = frexp(a, &e); /* a = frac * 2^e, frac in [0.5, 1) */
    e -= 1;              /* a = (2 frac) * 2^e, 2 frac in [1, 2) */
    if (e < -126) {
        /* subnormal BF16: multiples of 2^-133 */
        scaled = ldexp(a, 133);
        fl = floor(scaled);
        rem = scaled - fl;
        mant = (uint32_t)fl;
        if (rem > 0.5 || (rem == 0.5 && (mant & 1)))
            mant += 1;
        return (uint16_t)(sign | mant); /* mant == 128 is the smallest normal, encoded right */
    }
    scaled = ldexp(frac, 8); /* in [128, 256): 1.7 significand */
    fl = floor(scaled);
    rem = scaled - fl;
    mant = (uint32_t)fl;
    if (rem > 0.5 || (rem == 0.5 && (mant & 1)))
        mant += 1;
    if (mant == 256) {
        mant = 128;
        e += 1;
    }
    be = e + 127;
    if (be >= 255)
        return (uint16_t)(sign | 0x7F80);
    return (uint16_t)(sign | (uint32_t)(be << 7) | (mant & 0x7F));
}

uint16_t mxo_round_to_bf16(double x) { return double_to_bf16(x); }

void mxo_dequantize_bf16(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols,
                         uint16_t *dst, int64_t ld)
{
    int64_t nb = cols / MX_K;
    int64_t r;
#pragma omp parallel for schedule(static)
    for (r = 0; r < rows; ++r) {
        int64_t c;
        for (c = 0; c < cols; ++c)
            dst[r * ld + c] = double_to_bf16(decode_one(q[r * cols + c], s[r * nb + c / MX_K]));
    }
}

/* ---- Ablation arms (Section 3.1 / Table 1: E5M2 elements; Section 3.3: the OCP v1 scale rule). ----
 * Separate code paths on purpose: the functions above are the recipe and stay untouched. */

/* E5M2 (Table 1): 1 sign, 5 exponent (bias 15), 2 mantissa bits, IEEE-style specials: exponent field
 * 31 is Inf (mantissa 0) or NaN; max normal 1.75 * 2^15, min subnormal 2^-16. */
double mxo_e5m2_decode(uint8_t code)
{
    int sign = code >> 7;
    int e = (code >> 2) & 0x1F;
    int m = code & 0x3;
    double v;
    if (e == 0x1F)
        return m ? NAN : (sign ? -INFINITY : INFINITY);
    if (e == 0)
        v = ldexp((double)m, -16);
    else
        v = ldexp(1.0 + (double)m / 4.0, e - 15);
    return sign ? -v : v;
}

/* Nearest finite E5M2 value, ties to the even code, saturating at +-57344 (code 0x7B); NaN -> 0x7F. */
uint8_t mxo_e5m2_encode(double t)
{
    uint8_t sign = signbit(t) ? 0x80 : 0x00;
    double a = fabs(t);
    int best = 0;
    double best_d;
    int c;
    if (isnan(t))
        return 0x7F;
    if (a > 57344.0)
        return (uint8_t)(sign | 0x7B);
    best_d = a;
    for (c = 1; c <= 0x7B; ++c) {
        double d = fabs(a - mxo_e5m2_decode((uint8_t)c));
        if (d < best_d || (d == best_d && (c & 1) == 0)) {
            best_d = d;
            best = c;
        }
    }
    return (uint8_t)(sign | best);
}

static double fmt_max(int fmt) { return fmt ? 57344.0 : 448.0; }
static int fmt_emax(int fmt) { return fmt ? 15 : 8; }

/* Scale byte for element format fmt (0 = E4M3, 1 = E5M2) under rule 0 (Algorithm 1: smallest n with
 * amax <= max * 2^n) or rule 1 (OCP v1: n = floor(log2(amax)) - emax of the element format, i.e. the
 * ratio rounded DOWN to a power of two), clamped to [-127, 127]; found by loops, no logarithm. */
int mxo_scale_byte_mode(double amax, int fmt, int rule)
{
    int n;
    if (isnan(amax))
        return 0xFF;
    if (rule == 0) {
        for (n = -127; n < 127; ++n)
            if (amax <= ldexp(fmt_max(fmt), n))
                break;
    } else {
        /* largest n with 2^(n + emax) <= amax */
        for (n = 127; n > -127; --n)
            if (ldexp(1.0, n + fmt_emax(fmt)) <= amax)
                break;
    }
    return n + 127;
}

static uint8_t encode_fmt(double t, int fmt) { return fmt ? mxo_e5m2_encode(t) : mxo_e4m3_encode(t); }
static double decode_fmt(uint8_t q, int fmt) { return fmt ? mxo_e5m2_decode(q) : mxo_e4m3_decode(q); }

/* Row-wise quantization of an FP32 tensor under (fmt, rule); NaN blocks as in the recipe. */
void mxo_quantize_rowwise_mode_f32(const float *src, int64_t rows, int64_t cols, int64_t ld, uint8_t *q,
                                   uint8_t *s, int fmt, int rule)
{
    int64_t nb = cols / MX_K;
    int64_t r;
#pragma omp parallel for schedule(static)
    for (r = 0; r < rows; ++r) {
        int64_t b;
        for (b = 0; b < nb; ++b) {
            const float *v = src + r * ld + b * MX_K;
            uint8_t *qq = q + r * cols + b * MX_K;
            double amax = 0.0;
            int has_nan = 0, i, sb;
            for (i = 0; i < MX_K; ++i) {
                double a = fabs((double)v[i]);
                if (isnan(a))
                    has_nan = 1;
                else if (a > amax)
                    amax = a;
            }
            if (has_nan) {
                s[r * nb + b] = 0xFF;
                for (i = 0; i < MX_K; ++i)
                    qq[i] = 0x7F;
                continue;
            }
            sb = mxo_scale_byte_mode(amax, fmt, rule);
            s[r * nb + b] = (uint8_t)sb;
            for (i = 0; i < MX_K; ++i)
                qq[i] = encode_fmt(ldexp((double)v[i], -(sb - 127)), fmt);
        }
    }
}

/* Decode under fmt to double. */
void mxo_dequantize_mode_f64(const uint8_t *q, const uint8_t *s, int64_t rows, int64_t cols, double *dst, int fmt)
{
    int64_t nb = cols / MX_K;
    int64_t r;
#pragma omp parallel for schedule(static)
    for (r = 0; r < rows; ++r) {
        int64_t c;
        for (c = 0; c < cols; ++c) {
            uint8_t sb = s[r * nb + c / MX_K];
            dst[r * cols + c] = sb == 0xFF ? NAN : ldexp(decode_fmt(q[r * cols + c], fmt), (int)sb - 127);
        }
    }
}

/* ---- Block-scaled matrix product (Section 2, Appendix A.3). -------------------------------- */

/* C[m, n] = sum_k a[m, k] * b[n, k] over decoded operands (both K-contiguous), summed in plain k
 * order in double; absC[m, n] = sum_k |a * b| (the scale of the permitted per-element error).
 * Every block's partial sum is exact in double, so this is the block-scaled dot product of the
 * paper up to ~K/32 roundings at 2^-53. Only the output rows listed in row_idx are computed:
 * C and absC are [n_rows x N]. Returns 0, or -1 if memory for the decoded operands is missing. */
int mxo_gemm_rows_f64(const uint8_t *a_q, const uint8_t *a_s, const uint8_t *b_q,
                      const uint8_t *b_s, int64_t M, int64_t N, int64_t K, const int64_t *row_idx,
                      int64_t n_rows, double *C, double *absC)
{
    int64_t nb = K / MX_K;
    double *a = (double *)malloc((size_t)n_rows * K * sizeof(double));
    double *b = (double *)malloc((size_t)N * K * sizeof(double));
    int64_t idx;
    (void)M;
    if (!a || !b) {
        free(a);
        free(b);
        return -1;
    }
    for (idx = 0; idx < n_rows; ++idx)
        mxo_dequantize_f64(a_q + row_idx[idx] * K, a_s + row_idx[idx] * nb, 1, K, a + idx * K);
    mxo_dequantize_f64(b_q, b_s, N, K, b);
    for (idx = 0; idx < n_rows; ++idx) {
        int64_t n;
#pragma omp parallel for schedule(static)
        for (n = 0; n < N; ++n) {
            double acc = 0.0, aacc = 0.0;
            int64_t k;
            for (k = 0; k < K; ++k) {
                double p = a[idx * K + k] * b[n * K + k];
                acc += p;
                aacc += fabs(p);
            }
            C[idx * N + n] = acc;
            absC[idx * N + n] = aacc;
        }
    }
    free(a);
    free(b);
    return 0;
}

/* ---- Simulated MX path (Section 3.1). ------------------------------------------------------- */

/* The paper's own training runs emulate MX arithmetic: every BF16 GEMM input is converted to MXFP8
 * and straight back to BF16, and an ordinary BF16 GEMM with FP32 accumulation follows. The round
 * trip is mxo_quantize_{row,col}wise_bf16 followed by mxo_dequantize_bf16 (composed by the caller);
 * this is the product that follows it: C[m, n] = sum_k a[m, k] * b[n, k] over BF16 operands given as
 * bit patterns (both K-contiguous), summed in plain k order in double, absC = sum_k |a * b|.
 * Every product of two BF16 values is exact in double. Only the rows listed in row_idx are computed:
 * C and absC are [n_rows x N]. */
void mxo_matmul_nt_bf16_rows(const uint16_t *a, const uint16_t *b, int64_t M, int64_t N, int64_t K,
                             const int64_t *row_idx, int64_t n_rows, double *C, double *absC)
{
    int64_t idx;
    (void)M;
    for (idx = 0; idx < n_rows; ++idx) {
        const uint16_t *arow = a + row_idx[idx] * K;
        int64_t n;
#pragma omp parallel for schedule(static)
        for (n = 0; n < N; ++n) {
            double acc = 0.0, aacc = 0.0;
            int64_t k;
            for (k = 0; k < K; ++k) {
                double p = bf16_to_double(arow[k]) * bf16_to_double(b[n * K + k]);
                acc += p;
                aacc += fabs(p);
            }
            C[idx * N + n] = acc;
            absC[idx * N + n] = aacc;
        }
    }
}

