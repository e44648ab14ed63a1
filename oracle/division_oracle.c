/*
 * DIVISION activation codec -- CPU ORACLE.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct
 * scalar implementation of what the codec computes, used only by the tests,
 * by the smoke check and by the benchmark's CPU-baseline leg.  The product
 * (the HIP library) shares no code, header, table or constant generator with
 * it, and never calls it.
 *
 * What is computed (paper: "DIVISION: Memory Efficient Training via Dual
 * Activation Precision", Sec. 4.1 compression, Sec. 4.2 decompression,
 * Eq. (quantization), the reconstruction equation, Algorithm 1 steps
 * "AveragePooling / UpSampling / Quant / Cache" and "Dequant / UpSampling+add";
 * Appendix D for the pooled shapes):
 *
 *   for every (sample, channel) plane of an NCHW tensor (or NCDHW: the 3-D maps of Appendix D,
 *   blocks of B x B x B; the 1-D maps are the H = 1 case)
 *     H^L   = average pooling of the plane, window = stride = B      (Sec. 4.1)
 *     H^H   = H - UpSampling(H^L)          (nearest, block replicate) (Sec. 4.1)
 *     delta = min H^H, h_max = max H^H, Delta = (h_max-delta)/(2^Q-1) (Eq. quantization)
 *     V     = stochastic_round( Delta^-1 (H^H - delta) )              (Eq. quantization)
 *     cache (H^L, V packed Q bits per element, Delta, delta)          (Sec. 4.1, last paragraph)
 *   and back
 *     H^H~  = Delta * V + delta                                       (Sec. 4.2)
 *     H~    = UpSampling(H^L) + H^H~                                  (reconstruction equation)
 *
 * Readings taken where the paper is silent or at odds with itself (each is
 * listed with its reason in the design document of this repository):
 *   - pooled size is ceil(H/B) x ceil(W/B); edge windows average only their
 *     valid elements.  Identical to the paper whenever B divides the map size
 *     and whenever the map is smaller than B (one window covering the map).
 *   - one (delta, Delta) pair per (sample, channel) plane, stored as fp32; in the ORACLE_F32_C16
 *     mode (the paper's cached format) as bfloat16, delta rounded down and Delta rounded up so
 *     that the decoder's values bracket every residual (see plane_scale_c16).
 *   - stochastic rounding rounds UP with probability frac(x) (the unbiased
 *     rule the paper's second footnote on Eq. (quantization) requires).
 *   - a plane whose residual range is below 2^-90 is degenerate: Delta = 0,
 *     all codes 0.
 *   - where a plane's smallest residual is zero and both +0 and -0 occur, delta is -0 (and the
 *     maximum of such a pair is +0): the order of IEEE 754-2019 minimum / maximum.
 *   - the scale factor is inv = fl((2^Q-1)/range), bumped by one ulp when
 *     fl(range*inv) would fall short of 2^Q-1, so that the plane's maximum
 *     always receives the top code.
 *   - the random numbers are 16 bits per element from a counter-based hash of
 *     (seed, plane, element-pair index); the paper names no generator.
 *   - the residual is taken against the LFC as stored (after rounding to the
 *     storage type), so that decompression sees exactly what compression used.
 *
 * Arithmetic: every "fp32 op" below is one IEEE-754 binary32 operation,
 * round-to-nearest-even, never fused.  Compile with -ffp-contract=off and
 * without -ffast-math.  Block means are accumulated in binary64.
 *
 * Parity pins: tests/test_oracle_3d_pins.py pins the 3-D maps (library 3-D pooling and
 * up-sampling, an exact-rational brute force over coordinates, reduction to the 2-D
 * codec, axis permutations).  tests/test_oracle_pins.py checks this file against worked
 * examples, closed forms, library pooling/upsampling, a brute-force
 * exact-rational re-derivation and statistical properties.  The random
 * generator has no counterpart in the paper: its pins are this build's own
 * known-answer vectors (an independent big-integer evaluation) and
 * statistical tests.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <math.h>
#include <stdlib.h>

/* element type of x and of the reconstruction / how the tuple is cached:
 *   ORACLE_F32       x fp32;  H^L fp32, (delta, Delta) fp32
 *   ORACLE_BF16      x bf16;  H^L bf16, (delta, Delta) fp32
 *   ORACLE_F32_C16   x fp32;  H^L, delta and Delta cached as bfloat16, the format of the paper
 *                    (Sec. 4.1: "cached in the format of bfloat16"; N^2 Q/8 + 4 bytes per channel) */
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F32_C16 = 2 };

/* ---------- storage types ------------------------------------------------ */

static float bf16_to_float(uint16_t v)
{
    uint32_t u = (uint32_t)v << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest-even fp32 -> bfloat16 (NaN kept quiet) */
static uint16_t float_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

static float load_elem(const void *x, int dt, size_t idx)
{
    if (dt == ORACLE_BF16)
        return bf16_to_float(((const uint16_t *)x)[idx]);
    return ((const float *)x)[idx];
}

static size_t lfc_size(int dt) { return dt == ORACLE_F32 ? 4u : 2u; }             /* of the cached H^L */
static size_t meta_size(int dt) { return dt == ORACLE_F32_C16 ? 4u : 8u; }        /* of (delta, Delta) per plane */

/* largest bfloat16 <= f and smallest bfloat16 >= f (finite f) */
static float bf16_floor(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t t = u & 0xffff0000u;                       /* toward zero */
    if ((u & 0x80000000u) && (u & 0xffffu)) t += 0x10000u;   /* negative: one step away from zero */
    float r;
    memcpy(&r, &t, 4);
    return r;
}
static float bf16_ceil(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t t = u & 0xffff0000u;
    if (!(u & 0x80000000u) && (u & 0xffffu)) t += 0x10000u;  /* positive: one step away from zero */
    float r;
    memcpy(&r, &t, 4);
    return r;
}
static uint16_t bf16_bits_exact(float f)                /* f is a bfloat16 value already */
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}

static size_t align16(size_t v) { return (v + 15u) & ~(size_t)15u; }

/* ---------- random source (paper silent; defined by this build) ---------- */

/* 32-bit xorshift-multiply integer finaliser (shifts 16/15/16). */
static uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

/* the two per-plane keys derived from the 64-bit seed and the plane index */
void oracle_plane_keys(uint64_t seed, uint32_t plane, uint32_t *k1, uint32_t *k2)
{
    uint32_t a = mix32((uint32_t)(seed & 0xffffffffu) ^ 0x243F6A88u);
    uint32_t c = mix32((uint32_t)(seed >> 32) ^ 0x85A308D3u);
    *k1 = mix32(plane ^ a);
    *k2 = mix32(*k1 + c);
}

/* one 32-bit random word per PAIR of elements: j = (index in plane) >> 1 */
uint32_t oracle_hash32(uint64_t seed, uint32_t plane, uint32_t j)
{
    uint32_t k1, k2;
    oracle_plane_keys(seed, plane, &k1, &k2);
    uint32_t x = k1 + j * 0x9E3779B9u;
    x ^= x >> 16;
    x *= 0x7feb352du;
    x = x ^ (x >> 15) ^ k2;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

/* n consecutive words of one plane's stream (test aid for statistical checks) */
void oracle_hash32_fill(uint64_t seed, uint32_t plane, uint32_t j0, size_t n, uint32_t *out)
{
    for (size_t k = 0; k < n; ++k)
        out[k] = oracle_hash32(seed, plane, j0 + (uint32_t)k);
}

/* the 16 random bits of element i of a plane */
uint32_t oracle_rand16(uint64_t seed, uint32_t plane, uint32_t i)
{
    uint32_t w = oracle_hash32(seed, plane, i >> 1);
    return (i & 1u) ? (w >> 16) : (w & 0xffffu);
}

/* ---------- packed layout ------------------------------------------------ */

typedef struct {
    size_t P, HW, LD, LH, LW, WPP;      /* HW = elements per plane (D*H*W); LD x LH x LW pooled */
    size_t codes_off, codes_bytes, meta_off, meta_bytes, lfc_off, lfc_bytes, total;
} layout_t;

/* A plane is D x H x W (Appendix D, 3-D maps); D = 1 is the 2-D map of Sec. 4.1, D = H = 1 the 1-D one. */
static int make_layout(int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int B, int b, int dt, layout_t *L)
{
    if (N <= 0 || C <= 0 || D <= 0 || H <= 0 || W <= 0 || B < 1 || (b != 1 && b != 2 && b != 4 && b != 8))
        return 1;
    if (dt != ORACLE_F32 && dt != ORACLE_BF16 && dt != ORACLE_F32_C16)
        return 1;
    L->P = (size_t)N * (size_t)C;
    L->HW = (size_t)D * (size_t)H * (size_t)W;
    L->LD = ((size_t)D + (size_t)B - 1) / (size_t)B;
    L->LH = ((size_t)H + (size_t)B - 1) / (size_t)B;
    L->LW = ((size_t)W + (size_t)B - 1) / (size_t)B;
    size_t cpw = 32u / (unsigned)b;
    L->WPP = (L->HW + cpw - 1) / cpw;
    L->codes_off = 0;
    L->codes_bytes = 4u * L->P * L->WPP;
    L->meta_off = align16(L->codes_bytes);
    L->meta_bytes = meta_size(dt) * L->P;
    L->lfc_off = align16(L->meta_off + L->meta_bytes);
    L->lfc_bytes = lfc_size(dt) * L->P * L->LD * L->LH * L->LW;
    L->total = align16(L->lfc_off + L->lfc_bytes);
    return 0;
}

size_t oracle_packed_bytes_3d(int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int B, int b, int dt)
{
    layout_t L;
    if (make_layout(N, C, D, H, W, B, b, dt, &L))
        return 0;
    return L.total;
}

size_t oracle_packed_bytes(int64_t N, int64_t C, int64_t H, int64_t W, int B, int b, int dt)
{
    return oracle_packed_bytes_3d(N, C, 1, H, W, B, b, dt);
}

int oracle_packed_layout_3d(int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int B, int b, int dt,
                            size_t *codes_off, size_t *codes_bytes, size_t *meta_off,
                            size_t *meta_bytes, size_t *lfc_off, size_t *lfc_bytes)
{
    layout_t L;
    if (make_layout(N, C, D, H, W, B, b, dt, &L))
        return 1;
    *codes_off = L.codes_off; *codes_bytes = L.codes_bytes;
    *meta_off = L.meta_off;   *meta_bytes = L.meta_bytes;
    *lfc_off = L.lfc_off;     *lfc_bytes = L.lfc_bytes;
    return 0;
}

int oracle_packed_layout(int64_t N, int64_t C, int64_t H, int64_t W, int B, int b, int dt,
                         size_t *codes_off, size_t *codes_bytes, size_t *meta_off,
                         size_t *meta_bytes, size_t *lfc_off, size_t *lfc_bytes)
{
    return oracle_packed_layout_3d(N, C, 1, H, W, B, b, dt, codes_off, codes_bytes, meta_off, meta_bytes,
                                   lfc_off, lfc_bytes);
}

/* ---------- one plane, step by step -------------------------------------- */

/* Sec. 4.1 and Appendix D Eq. (average_poolnd): H^L = AveragePooling(H), window = stride = B in
 * every dimension of the map (B x B x B for a 3-D map, B x B for D = 1), clipped at the
 * border.  The mean is the exact sum (binary64 accumulation, depth-major then
 * row-major) divided by the element count, rounded once to fp32, then rounded to
 * the storage type.  lfc_f receives the stored value widened back to fp32. */
static void plane_lfc(const void *x, int dt, size_t base, size_t D, size_t H, size_t W, size_t B,
                      size_t LD, size_t LH, size_t LW, float *lfc_f)
{
    for (size_t bd = 0; bd < LD; ++bd)
    for (size_t bi = 0; bi < LH; ++bi) {
        for (size_t bj = 0; bj < LW; ++bj) {
            size_t d1 = (bd + 1) * B < D ? (bd + 1) * B : D;
            size_t r1 = (bi + 1) * B < H ? (bi + 1) * B : H;
            size_t c1 = (bj + 1) * B < W ? (bj + 1) * B : W;
            double S = 0.0;
            size_t cnt = 0;
            for (size_t d = bd * B; d < d1; ++d)
                for (size_t r = bi * B; r < r1; ++r)
                    for (size_t c = bj * B; c < c1; ++c) {
                        S += (double)load_elem(x, dt, base + (d * H + r) * W + c);
                        ++cnt;
                    }
            float m = (float)(S / (double)cnt);
            if (dt != ORACLE_F32)
                m = bf16_to_float(float_to_bf16(m));
            lfc_f[(bd * LH + bi) * LW + bj] = m;
        }
    }
}

/* Eq. (quantization): min and max of a plane's residuals.  The paper does not say which zero is the
 * minimum of a plane that holds both +0 and -0; the reading taken is the total order of IEEE 754-2019
 * minimum / maximum (-0 below +0), so that the result does not depend on the order of the elements. */
static int orders_below(float a, float b)
{
    return a < b || (a == b && signbit(a) && !signbit(b));
}

static void plane_extremes(const float *h, size_t HW, float *lo_out, float *hi_out)
{
    float lo = h[0], hi = h[0];
    for (size_t i = 1; i < HW; ++i) {
        if (orders_below(h[i], lo)) lo = h[i];
        if (orders_below(hi, h[i])) hi = h[i];
    }
    *lo_out = lo;
    *hi_out = hi;
}

/* Eq. (quantization): per-plane scale.  Returns delta, Delta and the scale inv. */
static void plane_scale(const float *h, size_t HW, int b, float *delta, float *Delta, float *inv)
{
    float lo, hi;
    plane_extremes(h, HW, &lo, &hi);
    const float Lf = (float)((1 << b) - 1);
    volatile float range = hi - lo;                 /* fp32 sub */
    *delta = lo;
    if (range >= 0x1p-90f && range <= 3.4028234663852886e38f) {
        volatile float D = range / Lf;              /* fp32 div */
        volatile float s = Lf / range;              /* fp32 div */
        volatile float top = range * s;             /* fp32 mul */
        if (top < Lf)
            s = nextafterf(s, INFINITY);
        *Delta = D;
        *inv = s;
    } else {
        *Delta = 0.0f;
        *inv = 0.0f;
    }
}

/* The same with delta and Delta cached as bfloat16 (ORACLE_F32_C16).  Reading: the quantiser
 * must use the very values the decoder will see, and every residual must stay inside their code
 * range, so delta is the plane minimum rounded DOWN to bfloat16 and Delta is
 * fl(fl(max - delta) / L) rounded UP to bfloat16; the scale is inv = fl(1 / Delta).  The top code
 * need not be reached.  A plane with fl(max - delta) below 2^-90 is degenerate (Delta = 0), and so
 * is one whose Delta, rounded up, is beyond the largest bfloat16: the decoder could not multiply by
 * it (with L = 1 and a range between the largest bfloat16 and the largest binary32). */
static void plane_scale_c16(const float *h, size_t HW, int b, float *delta, float *Delta, float *inv)
{
    float lo, hi;
    plane_extremes(h, HW, &lo, &hi);
    const float Lf = (float)((1 << b) - 1);
    const float d = bf16_floor(lo);
    volatile float range = hi - d;                  /* fp32 sub */
    *delta = d;
    if (range >= 0x1p-90f && range <= 3.4028234663852886e38f) {
        volatile float q = range / Lf;              /* fp32 div */
        const float D = bf16_ceil(q);
        if (D <= 3.3895313892515355e38f) {          /* the largest bfloat16 */
            volatile float s = 1.0f / D;            /* fp32 div */
            *Delta = D;
            *inv = s;
        } else {                                    /* Delta has no finite bfloat16 (1-bit codes only) */
            *Delta = 0.0f;
            *inv = 0.0f;
        }
    } else {
        *Delta = 0.0f;
        *inv = 0.0f;
    }
}

/*
 * Compress.  x: N*C*H*W elements of type dt (host memory, NCHW contiguous).
 * packed: oracle_packed_bytes(...) bytes, fully written (pad bytes zero).
 * Optional debug outputs (may be NULL), each N*C*H*W long:
 *   t_out   the fp32 pre-round value t = fl(fl(h - delta) * inv)
 *   r_out   the 16 random bits used for the element
 *   h_out   the fp32 residual h
 * Planes are independent; `threads` > 1 distributes them over OpenMP threads
 * (no arithmetic is reordered by that).  Returns 0, or 1 on invalid arguments.
 */
int oracle_compress_3d(const void *x, int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int dt,
                       int B, int b, uint64_t seed, void *packed,
                       float *t_out, uint16_t *r_out, float *h_out, int threads)
{
    layout_t L;
    if (!x || !packed || make_layout(N, C, D, H, W, B, b, dt, &L))
        return 1;
    if (L.P > 0x7fffffffu || L.HW > 0x7fffffffu)
        return 1;
    memset(packed, 0, L.total);
    uint8_t *pk = (uint8_t *)packed;
    const uint32_t Lq = (1u << b) - 1u;
    const size_t cpw = 32u / (unsigned)b;
    if (threads < 1) threads = 1;

    #pragma omp parallel for schedule(static) num_threads(threads)
    for (int64_t pp = 0; pp < (int64_t)L.P; ++pp) {
        size_t p = (size_t)pp;
        size_t base = p * L.HW;
        const size_t nb = L.LD * L.LH * L.LW;
        float *lfc_f = (float *)malloc(sizeof(float) * nb);
        float *h = (float *)malloc(sizeof(float) * L.HW);

        plane_lfc(x, dt, base, (size_t)D, (size_t)H, (size_t)W, (size_t)B, L.LD, L.LH, L.LW, lfc_f);

        /* store H^L in the storage type */
        for (size_t k = 0; k < nb; ++k) {
            if (dt != ORACLE_F32)
                ((uint16_t *)(pk + L.lfc_off))[p * nb + k] = float_to_bf16(lfc_f[k]);
            else
                ((float *)(pk + L.lfc_off))[p * nb + k] = lfc_f[k];
        }

        /* Sec. 4.1, Eq. (up_samplend): H^H = H - UpSampling(H^L), nearest = block replicate */
        for (size_t z = 0; z < (size_t)D; ++z)
            for (size_t r = 0; r < (size_t)H; ++r)
                for (size_t c = 0; c < (size_t)W; ++c) {
                    size_t i = (z * (size_t)H + r) * (size_t)W + c;
                    volatile float d = load_elem(x, dt, base + i)
                                       - lfc_f[((z / B) * L.LH + (r / B)) * L.LW + (c / B)];
                    h[i] = d;
                }

        float delta, Delta, inv;
        if (dt == ORACLE_F32_C16) {
            plane_scale_c16(h, L.HW, b, &delta, &Delta, &inv);
            ((uint16_t *)(pk + L.meta_off))[2 * p + 0] = bf16_bits_exact(delta);
            ((uint16_t *)(pk + L.meta_off))[2 * p + 1] = bf16_bits_exact(Delta);
        } else {
            plane_scale(h, L.HW, b, &delta, &Delta, &inv);
            ((float *)(pk + L.meta_off))[2 * p + 0] = delta;
            ((float *)(pk + L.meta_off))[2 * p + 1] = Delta;
        }

        uint32_t *codes = (uint32_t *)(pk + L.codes_off) + p * L.WPP;
        for (size_t i = 0; i < L.HW; ++i) {
            uint32_t r16 = oracle_rand16(seed, (uint32_t)p, (uint32_t)i);
            volatile float d = h[i] - delta;        /* fp32 sub */
            volatile float t = d * inv;             /* fp32 mul */
            /* floor(t + u), u = r16 / 2^16, evaluated exactly in binary64:
             * t has <= 24 significant bits and lies in [0, 256], u has 16
             * fraction bits, so the sum needs < 53 bits. */
            double s = floor((double)t + (double)r16 / 65536.0);
            uint32_t q = s < 0.0 ? 0u : (uint32_t)s;
            if (q > Lq) q = Lq;
            codes[i / cpw] |= q << ((i % cpw) * (unsigned)b);
            if (t_out) t_out[base + i] = t;
            if (r_out) r_out[base + i] = (uint16_t)r16;
            if (h_out) h_out[base + i] = h[i];
        }
        free(h);
        free(lfc_f);
    }
    return 0;
}

int oracle_compress(const void *x, int64_t N, int64_t C, int64_t H, int64_t W, int dt,
                    int B, int b, uint64_t seed, void *packed,
                    float *t_out, uint16_t *r_out, float *h_out, int threads)
{
    return oracle_compress_3d(x, N, C, 1, H, W, dt, B, b, seed, packed, t_out, r_out, h_out, threads);
}

/*
 * Decompress (Sec. 4.2 and the reconstruction equation):
 *   hh = fl(q * Delta); hh = fl(hh + delta); v = fl(lfc + hh); xhat = (T)v.
 */
int oracle_decompress_3d(const void *packed, int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int dt,
                         int B, int b, void *xhat, int threads)
{
    layout_t L;
    if (!xhat || !packed || make_layout(N, C, D, H, W, B, b, dt, &L))
        return 1;
    const uint8_t *pk = (const uint8_t *)packed;
    const uint32_t Lq = (1u << b) - 1u;
    const size_t cpw = 32u / (unsigned)b;
    if (threads < 1) threads = 1;

    #pragma omp parallel for schedule(static) num_threads(threads)
    for (int64_t pp = 0; pp < (int64_t)L.P; ++pp) {
        size_t p = (size_t)pp;
        const uint32_t *codes = (const uint32_t *)(pk + L.codes_off) + p * L.WPP;
        float delta, Delta;
        if (dt == ORACLE_F32_C16) {
            delta = bf16_to_float(((const uint16_t *)(pk + L.meta_off))[2 * p + 0]);
            Delta = bf16_to_float(((const uint16_t *)(pk + L.meta_off))[2 * p + 1]);
        } else {
            delta = ((const float *)(pk + L.meta_off))[2 * p + 0];
            Delta = ((const float *)(pk + L.meta_off))[2 * p + 1];
        }
        for (size_t z = 0; z < (size_t)D; ++z)
        for (size_t r = 0; r < (size_t)H; ++r)
            for (size_t c = 0; c < (size_t)W; ++c) {
                size_t i = (z * (size_t)H + r) * (size_t)W + c;
                uint32_t q = (codes[i / cpw] >> ((i % cpw) * (unsigned)b)) & Lq;
                size_t k = p * L.LD * L.LH * L.LW
                           + ((z / (size_t)B) * L.LH + (r / (size_t)B)) * L.LW + (c / (size_t)B);
                float lfc = (dt != ORACLE_F32)
                                ? bf16_to_float(((const uint16_t *)(pk + L.lfc_off))[k])
                                : ((const float *)(pk + L.lfc_off))[k];
                volatile float hh = (float)q * Delta;   /* Sec. 4.2: Delta * V   */
                hh = hh + delta;                        /*           ... + delta */
                volatile float v = lfc + hh;            /* reconstruction eq.    */
                if (dt == ORACLE_BF16)
                    ((uint16_t *)xhat)[p * L.HW + i] = float_to_bf16(v);
                else
                    ((float *)xhat)[p * L.HW + i] = v;
            }
    }
    return 0;
}

int oracle_decompress(const void *packed, int64_t N, int64_t C, int64_t H, int64_t W, int dt,
                      int B, int b, void *xhat, int threads)
{
    return oracle_decompress_3d(packed, N, C, 1, H, W, dt, B, b, xhat, threads);
}

/* bf16 helpers exported so tests can build bf16 inputs without torch */
uint16_t oracle_float_to_bf16(float f) { return float_to_bf16(f); }
float oracle_bf16_to_float(uint16_t v) { return bf16_to_float(v); }

/* ====================================================================== *
 * 1-bit masks of the Relu and Dropout operators (the paper's appendix on
 * operator compression: Algorithms "Relu operator" and "Dropout operator").
 *
 *   Relu forward:     V = sgn(H) (1 where H > 0, else 0),  out = V (.) H,
 *                     V packed one bit per element and cached.
 *   Dropout forward:  V ~ Bernoulli(1 - p) element-wise,   out = V (.) H.
 *   Backward (both):  grad_in = V (.) grad_out.
 *
 * Readings: the products V (.) H and V (.) grad select: where V = 0 the result
 * is +0 whatever the operand (also for NaN and -x).  Dropout does not rescale
 * by 1/(1-p), as in the paper's listing.  The paper names no generator for V;
 * element i keeps its value iff its 16 random bits r satisfy r >= T with
 * T = floor(p * 65536 + 0.5) clipped to [0, 65536] (p is widened to binary64
 * first), the 16 bits being those of element (i mod 2^32) of "plane" i >> 32
 * of the stream above under the seed XOR 0xD509A5B3C2E1F047.
 * Mask layout: bit i%32 of 32-bit word i/32 (little endian), pad bits zero.
 * ====================================================================== */

size_t oracle_mask_bytes(int64_t n) { return n < 0 ? 0 : (size_t)((n + 31) / 32) * 4u; }

static void store_elem(void *y, int dt, size_t idx, float v)
{
    if (dt == ORACLE_BF16) ((uint16_t *)y)[idx] = float_to_bf16(v);
    else ((float *)y)[idx] = v;
}

/* copies element idx bit for bit (no rounding: the value already has type dt) */
static void copy_elem(void *y, const void *x, int dt, size_t idx)
{
    if (dt == ORACLE_BF16) ((uint16_t *)y)[idx] = ((const uint16_t *)x)[idx];
    else memcpy((char *)y + 4 * idx, (const char *)x + 4 * idx, 4);
}

int oracle_relu_forward(const void *x, int64_t n, int dt, void *y, uint32_t *mask)
{
    if (!x || !y || !mask || n < 0 || (dt != ORACLE_F32 && dt != ORACLE_BF16)) return 1;
    memset(mask, 0, oracle_mask_bytes(n));
    for (int64_t i = 0; i < n; ++i) {
        if (load_elem(x, dt, (size_t)i) > 0.0f) {
            mask[i / 32] |= 1u << (i % 32);
            copy_elem(y, x, dt, (size_t)i);
        } else {
            store_elem(y, dt, (size_t)i, 0.0f);
        }
    }
    return 0;
}

uint32_t oracle_dropout_threshold(float p)
{
    double t = floor((double)p * 65536.0 + 0.5);
    if (!(t > 0.0)) return 0u;          /* also NaN */
    if (t > 65536.0) return 65536u;
    return (uint32_t)t;
}

int oracle_dropout_forward(const void *x, int64_t n, int dt, float p, uint64_t seed, void *y, uint32_t *mask)
{
    if (!x || !y || !mask || n < 0 || (dt != ORACLE_F32 && dt != ORACLE_BF16)) return 1;
    const uint32_t T = oracle_dropout_threshold(p);
    const uint64_t s = seed ^ 0xD509A5B3C2E1F047ull;
    memset(mask, 0, oracle_mask_bytes(n));
    for (int64_t i = 0; i < n; ++i) {
        uint32_t r = oracle_rand16(s, (uint32_t)((uint64_t)i >> 32), (uint32_t)((uint64_t)i & 0xffffffffu));
        if (r >= T) {
            mask[i / 32] |= 1u << (i % 32);
            copy_elem(y, x, dt, (size_t)i);
        } else {
            store_elem(y, dt, (size_t)i, 0.0f);
        }
    }
    return 0;
}

int oracle_mask_backward(const uint32_t *mask, const void *grad_out, int64_t n, int dt, void *grad_in)
{
    if (!mask || !grad_out || !grad_in || n < 0 || (dt != ORACLE_F32 && dt != ORACLE_BF16)) return 1;
    for (int64_t i = 0; i < n; ++i) {
        if ((mask[i / 32] >> (i % 32)) & 1u) copy_elem(grad_in, grad_out, dt, (size_t)i);
        else store_elem(grad_in, dt, (size_t)i, 0.0f);
    }
    return 0;
}

/* ====================================================================== *
 * Max-Pooling layer with kernel size = stride = k (the paper's appendix on
 * operator compression, Algorithm "Max-Pooling layer"):
 *
 *   forward:   H_l = Max-Pooling(H_{l-1}, k); V marks, for every k x k window,
 *              where its maximum sits in H_{l-1}; V is packed one bit per
 *              INPUT element and cached.
 *   backward:  grad' = 1_{k x k} (x) grad_out  (every output gradient repeated
 *              over its window), grad_in = V (.) grad'.
 *
 * Readings: output size floor(H/k) x floor(W/k); rows and columns past the last
 * whole window belong to no window (V = 0, zero gradient).  Exactly one element
 * per window is marked: the first maximum in row-major order inside the window
 * (a later element wins only if it compares greater).  Where V = 0 the gradient
 * is +0.  Mask layout: bit i%32 of word i/32 over the flat NCHW input index.
 * ====================================================================== */

int oracle_maxpool_forward(const void *x, int64_t N, int64_t C, int64_t H, int64_t W, int dt, int k,
                           void *y, uint32_t *mask)
{
    if (!x || !y || !mask || N <= 0 || C <= 0 || H <= 0 || W <= 0 || k < 1 ||
        (dt != ORACLE_F32 && dt != ORACLE_BF16))
        return 1;
    const int64_t OH = H / k, OW = W / k;
    memset(mask, 0, oracle_mask_bytes(N * C * H * W));
    for (int64_t p = 0; p < N * C; ++p)
        for (int64_t oi = 0; oi < OH; ++oi)
            for (int64_t oj = 0; oj < OW; ++oj) {
                int64_t best = (p * H + oi * k) * W + oj * k;
                float bv = load_elem(x, dt, (size_t)best);
                for (int64_t r = 0; r < k; ++r)
                    for (int64_t c = 0; c < k; ++c) {
                        int64_t idx = (p * H + oi * k + r) * W + oj * k + c;
                        float v = load_elem(x, dt, (size_t)idx);
                        if (v > bv) { bv = v; best = idx; }
                    }
                mask[best / 32] |= 1u << (best % 32);
                size_t o = (size_t)((p * OH + oi) * OW + oj);
                if (dt == ORACLE_BF16) ((uint16_t *)y)[o] = ((const uint16_t *)x)[best];
                else memcpy((char *)y + 4 * o, (const char *)x + 4 * best, 4);
            }
    return 0;
}

int oracle_maxpool_backward(const uint32_t *mask, const void *grad_out, int64_t N, int64_t C, int64_t H, int64_t W,
                            int dt, int k, void *grad_in)
{
    if (!mask || !grad_out || !grad_in || N <= 0 || C <= 0 || H <= 0 || W <= 0 || k < 1 ||
        (dt != ORACLE_F32 && dt != ORACLE_BF16))
        return 1;
    const int64_t OH = H / k, OW = W / k;
    for (int64_t p = 0; p < N * C; ++p)
        for (int64_t r = 0; r < H; ++r)
            for (int64_t c = 0; c < W; ++c) {
                int64_t idx = (p * H + r) * W + c;
                int bit = (int)((mask[idx / 32] >> (idx % 32)) & 1u);
                if (bit && r / k < OH && c / k < OW) {
                    size_t o = (size_t)((p * OH + r / k) * OW + c / k);
                    if (dt == ORACLE_BF16) ((uint16_t *)grad_in)[idx] = ((const uint16_t *)grad_out)[o];
                    else memcpy((char *)grad_in + 4 * idx, (const char *)grad_out + 4 * o, 4);
                } else {
                    store_elem(grad_in, dt, (size_t)idx, 0.0f);
                }
            }
    return 0;
}
