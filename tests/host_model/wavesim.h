// Host-side execution model for the HIP kernels of this library (test infrastructure only).
//
// The kernel sources are compiled unchanged as host C++ against tests/host_model/shim/hip/
// hip_runtime.h; a launch runs each workgroup as one cooperative fiber per work-item on the CPU:
//   * cross-lane instructions (MFMA, DPP, shuffles, readfirstlane) and barriers are rendezvous
//     points of the 64 fibers of a wavefront / of the whole workgroup;
//   * a direct-to-LDS load is queued per wavefront and completes at the s_waitcnt vmcnt(n) that
//     retires it (or, in eager mode, when it is issued); until then its LDS destination holds a
//     poison byte that decodes to NaN both as element and as scale, so a missing wait or a buffer
//     that is overwritten while still being read shows up in the result;
//   * wavefronts run in a fixed priority order (ascending or descending) as far as they can, so
//     one wavefront is always maximally ahead of the others between barriers;
//   * global addresses of direct-to-LDS loads are checked against the registered buffers and LDS
//     addresses against the launch's allocation; ordinary loads and stores are left to
//     AddressSanitizer (buffers are exact-size heap blocks).
// The arithmetic of the emulated instructions is written from their documented behaviour as far
// as the kernels rely on it; it shares no code with the CPU oracle.
#pragma once
#include <ucontext.h>

#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <functional>
#include <vector>

#if defined(__has_feature)
#if __has_feature(address_sanitizer)
#define WAVESIM_ASAN 1
extern "C" void __sanitizer_start_switch_fiber(void **fake_stack_save, const void *bottom, size_t size);
extern "C" void __sanitizer_finish_switch_fiber(void *fake_stack_save, const void **bottom_old, size_t *size_old);
#endif
#endif

struct dim3 {
    unsigned x, y, z;
    constexpr dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};

namespace wavesim {

typedef short v2s __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v8bf16 __attribute__((ext_vector_type(8)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

[[noreturn]] inline void fail(const char *fmt, ...) __attribute__((format(printf, 1, 2)));

constexpr int kWave = 64;
constexpr size_t kStackBytes = 512 * 1024;
constexpr uint8_t kPoison = 0xFF;  // E4M3 NaN and UE8M0 NaN

enum State { RUNNABLE, AT_WAVE_SYNC, AT_BLOCK_SYNC, DONE };

struct Piece {  // one lane's share of a direct-to-LDS load
    const uint8_t *src;
    uint32_t lds_off, bytes;
};
struct Dma {
    std::vector<Piece> pieces;
};

struct Wave {
    int live = 0, arrived = 0;
    // rendezvous slots: each lane publishes up to 96 bytes
    alignas(16) uint8_t slot[kWave][96];
    bool present[kWave];
    std::deque<Dma> pending;  // oldest first
    Dma building;
    uint32_t building_m0 = 0;
    uint64_t issued = 0;
};

struct Fiber {
    ucontext_t ctx;
    uint8_t *stack = nullptr;
    State state = DONE;
    int wave = 0, lane = 0;
    dim3 tid;
    void *asan_fake = nullptr;
};

struct Buffer {
    const uint8_t *p;
    size_t n;
    const char *name;
};

struct Machine {
    // configuration (environment: WAVESIM_DMA = lazy | eager, WAVESIM_ORDER = up | down, WAVESIM_BLOCKS = all | n,
    // WAVESIM_DROP_PARTIAL_WAITS = 1)
    bool lazy_dma = true;
    bool descending = false;
    bool drop_partial_waits = false;  // self-test of the model: s_waitcnt vmcnt(n > 0) does nothing
    long max_blocks = -1;  // simulate at most this many workgroups per launch, spread over the grid (-1: all)
    // launch state
    dim3 grid, block, bid;
    uint8_t *lds = nullptr;
    size_t lds_bytes = 0;
    std::vector<Fiber> fibers;
    std::vector<Wave> waves;
    int block_live = 0, block_arrived = 0;
    Fiber *cur = nullptr;
    ucontext_t sched;
    const std::function<void()> *body = nullptr;
    std::vector<Buffer> buffers;
    std::vector<unsigned> simulated;  // block ids of the last launch that were run
    uint64_t launches = 0;
#ifdef WAVESIM_ASAN
    const void *main_bottom = nullptr;
    size_t main_size = 0;
    void *sched_fake = nullptr;
#endif
};
inline Machine g;

inline void fail(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    fprintf(stderr, "wavesim: ");
    vfprintf(stderr, fmt, ap);
    va_end(ap);
    if (g.cur)
        fprintf(stderr, "  [workgroup %u, wavefront %d, lane %d]", g.bid.x, g.cur->wave, g.cur->lane);
    fprintf(stderr, "\n");
    fflush(stderr);
    _Exit(3);
}

inline void register_buffer(const void *p, size_t n, const char *name) { g.buffers.push_back({(const uint8_t *)p, n, name}); }
inline void clear_buffers() { g.buffers.clear(); }

// ---- fibers ------------------------------------------------------------------------------------
inline void to_scheduler()
{
    Fiber *f = g.cur;
#ifdef WAVESIM_ASAN
    __sanitizer_start_switch_fiber(f->state == DONE ? nullptr : &f->asan_fake, g.main_bottom, g.main_size);
#endif
    swapcontext(&f->ctx, &g.sched);
#ifdef WAVESIM_ASAN
    __sanitizer_finish_switch_fiber(f->asan_fake, nullptr, nullptr);
#endif
}

inline void fiber_entry()
{
#ifdef WAVESIM_ASAN
    __sanitizer_finish_switch_fiber(nullptr, &g.main_bottom, &g.main_size);
#endif
    (*g.body)();
    Fiber *f = g.cur;
    f->state = DONE;
    Wave &w = g.waves[f->wave];
    --w.live;
    w.present[f->lane] = false;
    --g.block_live;
    // lanes that left can no longer be waited for
    if (w.live > 0 && w.arrived == w.live) {
        w.arrived = 0;
        for (Fiber &o : g.fibers)
            if (o.wave == f->wave && o.state == AT_WAVE_SYNC)
                o.state = RUNNABLE;
    }
    if (g.block_live > 0 && g.block_arrived == g.block_live) {
        g.block_arrived = 0;
        for (Fiber &o : g.fibers)
            if (o.state == AT_BLOCK_SYNC)
                o.state = RUNNABLE;
    }
    to_scheduler();
    fail("a finished fiber was resumed");
}

inline Fiber &me() { return *g.cur; }
inline Wave &my_wave() { return g.waves[g.cur->wave]; }

// all live lanes of the wavefront meet here; the last one to arrive runs `on_complete` before anyone
// goes on
template <class F> inline void wave_sync(F on_complete)
{
    Wave &w = my_wave();
    if (++w.arrived == w.live) {
        w.arrived = 0;
        on_complete();
        for (Fiber &o : g.fibers)
            if (o.wave == g.cur->wave && o.state == AT_WAVE_SYNC)
                o.state = RUNNABLE;
        return;
    }
    g.cur->state = AT_WAVE_SYNC;
    to_scheduler();
}
inline void wave_sync() { wave_sync([] {}); }

inline void block_sync()  // __syncthreads()
{
    if (++g.block_arrived == g.block_live) {
        g.block_arrived = 0;
        for (Fiber &o : g.fibers)
            if (o.state == AT_BLOCK_SYNC)
                o.state = RUNNABLE;
        return;
    }
    g.cur->state = AT_BLOCK_SYNC;
    to_scheduler();
}

// publish a value, rendezvous, then read any live lane's value with peek(); unpublish() is the
// rendezvous after which the slots may be overwritten again. present[l] says whether lane l is live.
template <class T> inline Wave &publish(const T &v)
{
    static_assert(sizeof(T) <= 96, "rendezvous slot");
    Wave &w = my_wave();
    memcpy(w.slot[g.cur->lane], &v, sizeof(T));
    wave_sync();
    return w;
}
template <class T> inline T peek(Wave &w, int lane)
{
    T v;
    memcpy(&v, w.slot[lane], sizeof(T));
    return v;
}
inline void unpublish() { wave_sync(); }

// ---- cross-lane instructions -------------------------------------------------------------------
template <class T> inline T readfirstlane(T v)
{
    Wave &w = publish(v);
    int first = 0;
    while (first < kWave && !w.present[first])
        ++first;
    T r = peek<T>(w, first);
    unpublish();
    return r;
}

inline int shfl_xor(int v, int mask)
{
    Wave &w = publish(v);
    const int src = g.cur->lane ^ mask;
    if (src >= kWave || !w.present[src])
        fail("__shfl_xor reads lane %d, which is not active", src);
    int r = peek<int>(w, src);
    unpublish();
    return r;
}

inline int update_dpp(int old, int src, int ctrl, int row_mask, int bank_mask, bool bound_ctrl)
{
    (void)old;
    (void)bound_ctrl;
    if (row_mask != 0xF || bank_mask != 0xF)
        fail("DPP row/bank masks other than 0xF are not modelled");
    const int lane = g.cur->lane;
    int from;
    if (ctrl >= 0 && ctrl <= 0xFF)
        from = (lane & ~3) | ((ctrl >> (2 * (lane & 3))) & 3);  // quad_perm
    else if (ctrl == 0x140)
        from = (lane & ~15) | (15 - (lane & 15));  // row_mirror
    else if (ctrl == 0x141)
        from = (lane & ~7) | (7 - (lane & 7));  // row_half_mirror
    else
        fail("DPP control 0x%x is not modelled", ctrl);
    Wave &w = publish(src);
    if (!w.present[from])
        fail("DPP reads lane %d, which is not active", from);
    int r = peek<int>(w, from);
    unpublish();
    return r;
}

inline uint32_t perm(uint32_t s0, uint32_t s1, uint32_t sel)  // v_perm_b32
{
    const uint64_t src = ((uint64_t)s0 << 32) | s1;
    uint32_t r = 0;
    for (int i = 0; i < 4; ++i) {
        const uint32_t c = (sel >> (8 * i)) & 0xFF;
        uint32_t b;
        if (c <= 7)
            b = (uint32_t)(src >> (8 * c)) & 0xFF;
        else if (c == 12)
            b = 0;
        else if (c >= 13)
            b = 0xFF;
        else
            fail("v_perm_b32 selector %u is not modelled", c);
        r |= b << (8 * i);
    }
    return r;
}

// ---- FP8 (OCP E4M3: 1-4-3, bias 7, subnormals, no infinities, S.1111.111 = NaN) -----------------
inline double e4m3_value_slow(uint8_t code)
{
    const int e = (code >> 3) & 15, m = code & 7;
    if (e == 15 && m == 7)
        return NAN;
    const double mag = e == 0 ? std::ldexp((double)m, -9) : std::ldexp(8.0 + m, e - 10);
    return (code & 0x80) ? -mag : mag;
}
inline double e4m3_value(uint8_t code)
{
    static double table[256];
    static bool ready = false;
    if (!ready) {
        for (int c = 0; c < 256; ++c)
            table[c] = e4m3_value_slow((uint8_t)c);
        ready = true;
    }
    return table[code];
}

// what the scaled conversion instructions do with one value: x / 2^(field - 127) (field 0 counts as
// 2^-127), round to nearest even onto the E4M3 grid, NaN above the rounding range of 448
inline uint8_t cvt_scaled_e4m3(float x, float scale)
{
    uint32_t sbits;
    memcpy(&sbits, &scale, 4);
    const int field = (sbits >> 23) & 0xFF;
    const uint8_t sign = std::signbit(x) ? 0x80 : 0;
    if (std::isnan(x) || field == 0xFF)
        return sign | 0x7F;
    const double v = std::ldexp(std::fabs((double)x), -(field == 0 ? -127 : field - 127));
    if (v > 464.0)
        return sign | 0x7F;
    if (v == 0.0)
        return sign;
    int e;
    std::frexp(v, &e);  // v = f * 2^e, f in [0.5, 1)
    int ue = e - 1;     // v in [2^ue, 2^(ue+1))
    if (ue < -6)
        ue = -6;        // subnormal grid: multiples of 2^-9
    const double q = std::nearbyint(std::ldexp(v, 3 - ue));  // in units of 2^(ue-3); default rounding mode = RNE
    int mant = (int)q, ex = ue;
    if (mant >= 16) {
        mant >>= 1;
        ++ex;
    }
    if (mant < 8)
        return sign | (uint8_t)mant;  // subnormal (or zero after rounding)
    return sign | (uint8_t)(((ex + 7) << 3) | (mant - 8));
}

inline v2s cvt_scalef32_pk_fp8_f32(v2s old, float a, float b, float scale, bool hi)
{
    const uint16_t w = (uint16_t)(cvt_scaled_e4m3(a, scale) | (cvt_scaled_e4m3(b, scale) << 8));
    old[hi ? 1 : 0] = (short)w;
    return old;
}
inline v2s cvt_scalef32_pk_fp8_bf16(v2s old, v2bf p, float scale, bool hi)
{
    return cvt_scalef32_pk_fp8_f32(old, (float)p[0], (float)p[1], scale, hi);
}
// v_cvt_scalef32_pk_fp4_f32: two FP32 values divided by the scale (same reading of the scale operand as the FP8
// forms) and rounded to E2M1, nearest with ties to the even code, saturating at 6, sign kept; the first value goes
// to the low nibble of byte `sel` of the destination, the second to the high nibble. What the instruction makes of
// a NaN is not modelled (the kernels never convert a block that holds one): it stops the model.
inline uint8_t cvt_scaled_e2m1(float x, float scale)
{
    uint32_t sbits;
    memcpy(&sbits, &scale, 4);
    const int field = (sbits >> 23) & 0xFF;
    if (std::isnan(x) || field == 0xFF)
        fail("E2M1 conversion of a NaN (or with a NaN scale) is not modelled");
    const uint8_t sign = std::signbit(x) ? 8 : 0;
    const double t = std::ldexp(std::fabs((double)x), -(field == 0 ? -127 : field - 127));
    static const double mid[7] = {0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0};  // midpoints; a tie goes to the even code
    uint8_t code = 0;
    for (int i = 0; i < 7; ++i)
        code += (i % 2 == 0) ? (t > mid[i]) : (t >= mid[i]);
    return sign | code;
}
inline uint32_t cvt_scalef32_pk_fp4_f32(uint32_t old, float a, float b, float scale, int sel)
{
    const uint32_t byte = (uint32_t)(cvt_scaled_e2m1(a, scale) | (cvt_scaled_e2m1(b, scale) << 4));
    return (old & ~(0xFFu << (8 * sel))) | (byte << (8 * sel));
}
// v_cvt_scalef32_2xpk16_{fp6,bf6}_f32: 2 x 16 FP32 values divided by the scale (same reading of the scale operand
// as the FP8 forms), rounded to E2M3 (fp6) or E3M2 (bf6), nearest with ties to even, saturating, sign kept; the
// 32 six-bit codes are packed little-endian, element 2i from the first source and 2i+1 from the second. What the
// instruction makes of a NaN is not modelled (the kernels never convert a block that holds one).
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned int v6u __attribute__((ext_vector_type(6)));
inline uint32_t cvt_scaled_fp6(float x, float scale, int ebits, int mbits)
{
    uint32_t sbits;
    memcpy(&sbits, &scale, 4);
    const int field = (sbits >> 23) & 0xFF;
    if (std::isnan(x) || field == 0xFF)
        fail("6-bit conversion of a NaN (or with a NaN scale) is not modelled");
    const int bias = (1 << (ebits - 1)) - 1, emin = 1 - bias, emax = (1 << ebits) - 1 - bias;
    const double top = std::ldexp((double)((1 << (mbits + 1)) - 1), emax - mbits);
    double t = std::ldexp(std::fabs((double)x), -(field == 0 ? -127 : field - 127));
    if (t > top)
        t = top;
    int e = emin;
    if (t > 0) {
        int ex;
        std::frexp(t, &ex);
        e = std::min(std::max(ex - 1, emin), emax);
    }
    const int q = (int)std::nearbyint(std::ldexp(t, mbits - e));  // default rounding mode: nearest even
    return (uint32_t)(((e - emin) << mbits) + q) | (std::signbit(x) ? 32u : 0u);
}
inline v6u cvt_scalef32_2xpk16_6bit(v16f a, v16f b, float scale, int ebits, int mbits)
{
    uint64_t bits[3] = {0, 0, 0};
    for (int i = 0; i < 32; ++i) {
        const uint64_t c = cvt_scaled_fp6(i % 2 ? b[i / 2] : a[i / 2], scale, ebits, mbits);
        const int pos = 6 * i;
        bits[pos / 64] |= c << (pos % 64);
        if (pos % 64 > 58)
            bits[pos / 64 + 1] |= c >> (64 - pos % 64);
    }
    v6u r;
    for (int j = 0; j < 6; ++j)
        r[j] = (uint32_t)(bits[j / 2] >> (32 * (j % 2)));
    return r;
}
// ---- FP8 (OCP E5M2: 1-5-2, bias 15, subnormals, exponent field 31 = Inf / NaN) ------------------------
inline double e5m2_value(uint8_t code)
{
    const int e = (code >> 2) & 31, m = code & 3;
    double mag;
    if (e == 31)
        mag = m ? NAN : INFINITY;
    else
        mag = e == 0 ? std::ldexp((double)m, -16) : std::ldexp(4.0 + m, e - 17);
    return (code & 0x80) ? -mag : mag;
}
// the E5M2 form of the scaled conversion: same scaling and rounding; what rounds beyond 57344 becomes Inf
// (the kernels replace every code above the largest finite one, so only "above 0x7B" matters here)
inline uint8_t cvt_scaled_e5m2(float x, float scale)
{
    uint32_t sbits;
    memcpy(&sbits, &scale, 4);
    const int field = (sbits >> 23) & 0xFF;
    const uint8_t sign = std::signbit(x) ? 0x80 : 0;
    if (std::isnan(x) || field == 0xFF)
        return sign | 0x7F;
    const double v = std::ldexp(std::fabs((double)x), -(field == 0 ? -127 : field - 127));
    if (v == 0.0)
        return sign;
    if (std::isinf(v))
        return sign | 0x7C;
    int e;
    std::frexp(v, &e);
    int ue = e - 1;
    if (ue < -14)
        ue = -14;        // subnormal grid: multiples of 2^-16
    const double q = std::nearbyint(std::ldexp(v, 2 - ue));  // in units of 2^(ue-2); RNE
    int mant = (int)q, ex = ue;
    if (mant >= 8) {
        mant >>= 1;
        ++ex;
    }
    if (mant < 4)
        return sign | (uint8_t)mant;
    if (ex > 15)
        return sign | 0x7C;
    return sign | (uint8_t)(((ex + 15) << 2) | (mant - 4));
}
inline v2s cvt_scalef32_pk_bf8_f32(v2s old, float a, float b, float scale, bool hi)
{
    const uint16_t w = (uint16_t)(cvt_scaled_e5m2(a, scale) | (cvt_scaled_e5m2(b, scale) << 8));
    old[hi ? 1 : 0] = (short)w;
    return old;
}
inline v2s cvt_scalef32_pk_bf8_bf16(v2s old, v2bf p, float scale, bool hi)
{
    return cvt_scalef32_pk_bf8_f32(old, (float)p[0], (float)p[1], scale, hi);
}
inline v2f cvt_pk_f32_bf8(int q, bool hi)
{
    const uint32_t u = (uint32_t)q >> (hi ? 16 : 0);
    return v2f{(float)e5m2_value(u & 0xFF), (float)e5m2_value((u >> 8) & 0xFF)};
}

inline v2f cvt_pk_f32_fp8(int q, bool hi)
{
    const uint32_t u = (uint32_t)q >> (hi ? 16 : 0);
    return v2f{(float)e4m3_value(u & 0xFF), (float)e4m3_value((u >> 8) & 0xFF)};
}

// E2M1 (4-bit MX element): sign, 2 exponent bits (bias 1), 1 mantissa bit; no NaN, no Inf
inline double e2m1_value(unsigned code)
{
    const unsigned e = (code >> 1) & 3u, m = code & 1u;
    const double mag = e == 0 ? 0.5 * m : std::ldexp(1.0 + 0.5 * m, (int)e - 1);
    return (code & 8u) ? -mag : mag;
}

// With both operands E2M1 (cbsz = blgp = 4) only dwords 0..3 are used: lane 16g+r holds K 32g..32g+31 of row r,
// eight elements per dword, and its scale byte scales exactly those (K block g).
// v_mfma_scale_f32_16x16x128_f8f6f4 with both operands E4M3: lane 16g+r holds row r of its operand,
// dwords 0..3 = K 16g..16g+15, dwords 4..7 = K 64+16g..64+16g+15; scale byte op_sel of lane (r, g)
// scales row r in K block g; result register v of lane (r, g) is D[4g+v][r] with
// D[x][y] = sum_k first[x][k] * second[y][k] (scaled). Sums are taken in double and rounded once,
// which is at least as accurate as the instruction.
inline v4f mfma_scale_16x16x128(v8i first, v8i second, v4f c, int cbsz, int blgp, int opsel_first, int scale_first,
                                int opsel_second, int scale_second)
{
    if (!((cbsz == 4 && blgp == 4) || (cbsz <= 1 && blgp <= 1)))
        fail("only FP8 x FP8 (E4M3 / E5M2 per operand) and E2M1 x E2M1 operands are modelled");
    const bool fp4 = cbsz == 4;
    const bool first_e5m2 = cbsz == 1, second_e5m2 = blgp == 1;  // format field of the first / second operand
    struct Pub {
        v8i first, second;
        uint8_t s_first, s_second;
    } pub{first, second, (uint8_t)((uint32_t)scale_first >> (8 * opsel_first)),
          (uint8_t)((uint32_t)scale_second >> (8 * opsel_second))};
    Wave &w = publish(pub);
    const int lane = g.cur->lane, r = lane & 15, gq = lane >> 4;
    for (int l = 0; l < kWave; ++l)
        if (!w.present[l])
            fail("MFMA issued with lane %d inactive", l);
    // row y = r of the second operand, all 128 k
    double yv[128], ys[4];
    for (int kg = 0; kg < 4; ++kg) {
        const Pub p = peek<Pub>(w, 16 * kg + r);
        uint8_t bytes[32];
        memcpy(bytes, &p.second, 32);
        for (int t = 0; t < 16; ++t) {
            if (fp4) {
                yv[32 * kg + 2 * t] = e2m1_value(bytes[t] & 0xF);
                yv[32 * kg + 2 * t + 1] = e2m1_value(bytes[t] >> 4);
            } else {
                yv[16 * kg + t] = second_e5m2 ? e5m2_value(bytes[t]) : e4m3_value(bytes[t]);
                yv[64 + 16 * kg + t] = second_e5m2 ? e5m2_value(bytes[16 + t]) : e4m3_value(bytes[16 + t]);
            }
        }
        ys[kg] = p.s_second == 0xFF ? NAN : std::ldexp(1.0, (int)p.s_second - 127);
    }
    v4f out;
    for (int v = 0; v < 4; ++v) {
        const int x = 4 * gq + v;
        double sum = 0.0;
        double xv[128], xs[4];
        for (int kg = 0; kg < 4; ++kg) {
            const Pub p = peek<Pub>(w, 16 * kg + x);
            uint8_t bytes[32];
            memcpy(bytes, &p.first, 32);
            for (int t = 0; t < 16; ++t) {
                if (fp4) {
                    xv[32 * kg + 2 * t] = e2m1_value(bytes[t] & 0xF);
                    xv[32 * kg + 2 * t + 1] = e2m1_value(bytes[t] >> 4);
                } else {
                    xv[16 * kg + t] = first_e5m2 ? e5m2_value(bytes[t]) : e4m3_value(bytes[t]);
                    xv[64 + 16 * kg + t] = first_e5m2 ? e5m2_value(bytes[16 + t]) : e4m3_value(bytes[16 + t]);
                }
            }
            xs[kg] = p.s_first == 0xFF ? NAN : std::ldexp(1.0, (int)p.s_first - 127);
        }
        for (int kb = 0; kb < 4; ++kb) {
            double part = 0.0;
            for (int k = 32 * kb; k < 32 * kb + 32; ++k)
                part += xv[k] * yv[k];
            sum += part * xs[kb] * ys[kb];
        }
        out[v] = (float)((double)c[v] + sum);
    }
    unpublish();
    return out;
}

// v_mfma_f32_16x16x32_bf16: lane 16g+r holds row r of its operand, k = 8g..8g+7; result register v of
// lane (r, g) is D[4g+v][r] with D[x][y] = sum_k first[x][k] * second[y][k]. Every product is exact in
// double; the sum is taken in double and rounded once, which is at least as accurate as the instruction.
inline v4f mfma_16x16x32_bf16(v8bf16 first, v8bf16 second, v4f c, int cbsz, int abid, int blgp)
{
    if (cbsz != 0 || abid != 0 || blgp != 0)
        fail("broadcast / permute modifiers of the BF16 matrix instruction are not modelled");
    struct Pub {
        v8bf16 first, second;
    } pub{first, second};
    Wave &w = publish(pub);
    const int lane = g.cur->lane, r = lane & 15, gq = lane >> 4;
    for (int l = 0; l < kWave; ++l)
        if (!w.present[l])
            fail("MFMA issued with lane %d inactive", l);
    double yv[32];
    for (int kg = 0; kg < 4; ++kg) {
        const Pub p = peek<Pub>(w, 16 * kg + r);
        for (int t = 0; t < 8; ++t)
            yv[8 * kg + t] = (double)(float)p.second[t];
    }
    v4f out;
    for (int v = 0; v < 4; ++v) {
        const int x = 4 * gq + v;
        double sum = 0.0;
        for (int kg = 0; kg < 4; ++kg) {
            const Pub p = peek<Pub>(w, 16 * kg + x);
            for (int t = 0; t < 8; ++t)
                sum += (double)(float)p.first[t] * yv[8 * kg + t];
        }
        out[v] = (float)((double)c[v] + sum);
    }
    unpublish();
    return out;
}

// ---- direct-to-LDS loads and their counter -------------------------------------------------------
inline void check_global(const uint8_t *p, uint32_t bytes)
{
    if (g.buffers.empty())  // a host that registers nothing (not the test driver) gets no range check
        return;
    for (const Buffer &b : g.buffers)
        if (p >= b.p && p + bytes <= b.p + b.n)
            return;
    fail("direct-to-LDS load of %u bytes at %p lies outside every registered buffer", bytes, (const void *)p);
}

inline void retire(Wave &w)
{
    const Dma &d = w.pending.front();
    for (const Piece &p : d.pieces)
        memcpy(g.lds + p.lds_off, p.src, p.bytes);
    w.pending.pop_front();
}

// lane's share of `global_load_lds_dword{,x4}`: BYTES from base + voff to LDS lds_addr + lane * BYTES
inline void dma_issue(const uint8_t *base, uint32_t voff, uint32_t lds_addr, uint32_t bytes)
{
    struct Pub {
        const uint8_t *base;
        uint32_t voff, lds_addr;
    } pub{base, voff, lds_addr};
    Wave &w = publish(pub);
    int first = 0;
    while (!w.present[first])
        ++first;
    const Pub lead = peek<Pub>(w, first);
    if (lead.base != base || lead.lds_addr != lds_addr)
        fail("direct-to-LDS load with a base pointer or LDS address (M0) that is not wavefront-uniform");
    const uint32_t lds_off = lds_addr - (uint32_t)(uintptr_t)g.lds + (uint32_t)g.cur->lane * bytes;
    if ((size_t)lds_off + bytes > g.lds_bytes)
        fail("direct-to-LDS load writes LDS offset %u (+%u), allocation is %zu bytes", lds_off, bytes, g.lds_bytes);
    if ((lds_addr & 3) != 0)
        fail("direct-to-LDS load with an LDS address that is not dword aligned");
    const uint8_t *src = base + voff;
    check_global(src, bytes);
    if ((uintptr_t)src % (bytes < 16 ? bytes : 16) != 0)
        fail("direct-to-LDS load from a misaligned global address %p", (const void *)src);
    w.building.pieces.push_back({src, lds_off, bytes});
    memset(g.lds + lds_off, kPoison, bytes);
    wave_sync([&w] {
        w.pending.push_back(std::move(w.building));
        w.building = Dma{};
        ++w.issued;
        if (!g.lazy_dma)
            while (!w.pending.empty())
                retire(w);
    });
}

// s_waitcnt with the gfx9 immediate layout: vmcnt in bits 3:0 and 15:14 (other counters are not modelled:
// LDS reads and stores are synchronous here)
inline void s_waitcnt(int imm)
{
    const unsigned vmcnt = ((unsigned)imm & 15u) | ((((unsigned)imm >> 14) & 3u) << 4);
    Wave &w = my_wave();
    if (g.drop_partial_waits && vmcnt != 0)
        return;
    while (w.pending.size() > vmcnt)
        retire(w);
}

// ---- launch ------------------------------------------------------------------------------------
inline void configure_from_env()
{
    if (const char *e = getenv("WAVESIM_DMA"))
        g.lazy_dma = strcmp(e, "eager") != 0;
    if (const char *e = getenv("WAVESIM_ORDER"))
        g.descending = strcmp(e, "down") == 0;
    if (const char *e = getenv("WAVESIM_DROP_PARTIAL_WAITS"))
        g.drop_partial_waits = strcmp(e, "1") == 0;
    if (const char *e = getenv("WAVESIM_BLOCKS"))
        g.max_blocks = strcmp(e, "all") == 0 ? -1 : atol(e);
}

inline void run_block(size_t shmem)
{
    const int nthreads = (int)g.block.x;
    if (nthreads % kWave != 0 || g.block.y != 1 || g.block.z != 1)
        fail("workgroup shape %ux%ux%u is not modelled", g.block.x, g.block.y, g.block.z);
    const int nwaves = nthreads / kWave;
    if ((int)g.fibers.size() < nthreads)
        g.fibers.resize(nthreads);
    g.waves.assign(nwaves, Wave{});
    // exact-size LDS block, 1 KB aligned like the hardware allocation, poisoned
    g.lds_bytes = shmem;
    g.lds = nullptr;
    if (shmem) {
        if (shmem > 160 * 1024)
            fail("%zu bytes of LDS requested, a compute unit has 160 KB", shmem);
        void *p = nullptr;
        if (posix_memalign(&p, 1024, shmem) != 0)
            fail("out of memory");
        g.lds = (uint8_t *)p;
        memset(g.lds, kPoison, shmem);
    }
    for (int t = 0; t < nthreads; ++t) {
        Fiber &f = g.fibers[t];
        if (!f.stack)
            f.stack = (uint8_t *)malloc(kStackBytes);
        f.state = RUNNABLE;
        f.wave = t / kWave;
        f.lane = t % kWave;
        f.tid = dim3((unsigned)t);
        f.asan_fake = nullptr;
        getcontext(&f.ctx);
        f.ctx.uc_stack.ss_sp = f.stack;
        f.ctx.uc_stack.ss_size = kStackBytes;
        f.ctx.uc_link = nullptr;
        makecontext(&f.ctx, (void (*)())fiber_entry, 0);
        g.waves[f.wave].live++;
        for (int l = 0; l < kWave; ++l)
            g.waves[f.wave].present[l] = true;
    }
    g.block_live = nthreads;
    g.block_arrived = 0;
    // scheduler: the runnable fiber of the most preferred wavefront, lowest lane first
    for (;;) {
        Fiber *next = nullptr;
        for (int i = 0; i < nthreads && !next; ++i) {
            const int t = g.descending ? (nwaves - 1 - i / kWave) * kWave + i % kWave : i;
            if (g.fibers[t].state == RUNNABLE)
                next = &g.fibers[t];
        }
        if (!next)
            break;
        g.cur = next;
#ifdef WAVESIM_ASAN
        __sanitizer_start_switch_fiber(&g.sched_fake, next->stack, kStackBytes);
#endif
        swapcontext(&g.sched, &next->ctx);
#ifdef WAVESIM_ASAN
        __sanitizer_finish_switch_fiber(g.sched_fake, nullptr, nullptr);
#endif
    }
    g.cur = nullptr;
    for (int t = 0; t < nthreads; ++t)
        if (g.fibers[t].state != DONE)
            fail("deadlock in workgroup %u: work-item %d waits at a %s that the others never reach", g.bid.x, t,
                 g.fibers[t].state == AT_WAVE_SYNC ? "cross-lane instruction" : "barrier");
    for (int wv = 0; wv < nwaves; ++wv)
        if (!g.waves[wv].pending.empty())
            fail("workgroup %u ends with %zu direct-to-LDS loads of wavefront %d still in flight", g.bid.x,
                 g.waves[wv].pending.size(), wv);
    free(g.lds);
    g.lds = nullptr;
}

inline void launch(dim3 grid, dim3 block, size_t shmem, const std::function<void()> &body)
{
    configure_from_env();
    if (grid.y != 1 || grid.z != 1)
        fail("grid shape %ux%ux%u is not modelled", grid.x, grid.y, grid.z);
    g.grid = grid;
    g.block = block;
    g.body = &body;
    g.simulated.clear();
    ++g.launches;
    // all workgroups, or max_blocks of them spread evenly over the grid (first and last included)
    const unsigned n = grid.x;
    const unsigned take = g.max_blocks < 0 || (unsigned long)g.max_blocks >= n ? n : (unsigned)g.max_blocks;
    for (unsigned i = 0; i < take; ++i) {
        const unsigned b = take == n ? i : take == 1 ? 0 : (unsigned)((uint64_t)i * (n - 1) / (take - 1));
        if (!g.simulated.empty() && g.simulated.back() == b)
            continue;
        g.bid = dim3(b);
        g.simulated.push_back(b);
        run_block(shmem);
    }
    g.body = nullptr;
}

}  // namespace wavesim
