// DIVISION activation codec for AMD MI355X (gfx950): HIP kernels and C ABI.
//
// Paper: "DIVISION: Memory Efficient Training via Dual Activation Precision".
//   compress   = Sec. 4.1  (AveragePooling -> residual against UpSampling ->
//                           Quant of Eq. (quantization) -> cache the tuple)
//   decompress = Sec. 4.2  (Dequant, then the reconstruction equation)
//
// Compile with -ffp-contract=off: the codec's fp32 steps are single IEEE
// operations (sub, mul, add), never fused, so that codes are reproducible.
//
// Work decomposition (one GPU, planes are independent):
//   * A workgroup owns a chunk of G consecutive (sample, channel) planes.
//   * compress_tile: the chunk is read from HBM exactly once with 16-byte
//     coalesced loads into LDS; block means, residuals, the plane min/max and
//     the quantisation all work out of LDS; the packed words, (delta, Delta)
//     and the LFC are written once.  No intermediate tensor touches HBM.
//   * decompress_*: pure streaming, one packed read and one 16-byte store per
//     four reconstructed elements.
//   * compress_any / decompress_scalar: slow fall-backs for block sizes and
//     plane sizes the tiled kernels do not cover.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/division.h"

namespace {

constexpr int kThreads = 256;              // 4 wavefronts of 64
constexpr uint32_t kLdsTarget = 40u << 10; // preferred LDS bytes per workgroup (4 groups per CU)
constexpr uint32_t kLdsMax = 156u << 10;   // hard limit per workgroup (160 KB per CU)
constexpr uint32_t kWeyl = 0x9E3779B9u;

// ------------------------------------------------------------------ helpers

struct bf16_t { uint16_t v; };
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// fp32 -> bf16, round to nearest even (NaN kept quiet)
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p, size_t i) { return p[i]; }
    static __device__ __forceinline__ void store(float* p, size_t i, float v) { p[i] = v; }
    static __device__ __forceinline__ float round(float v) { return v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t* p, size_t i) { return bf16_bits_to_float(p[i].v); }
    static __device__ __forceinline__ void store(bf16_t* p, size_t i, float v) { p[i].v = (uint16_t)float_to_bf16_bits(v); }
    static __device__ __forceinline__ float round(float v) { return bf16_bits_to_float(float_to_bf16_bits(v)); }
};

// 32-bit xorshift-multiply finaliser (shifts 16/15/16)
__host__ __device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du;
    x ^= x >> 15; x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// random word of element pair j of a plane with keys (k1, k2); xw = k1 + j*kWeyl
__device__ __forceinline__ uint32_t pair_word(uint32_t xw, uint32_t k2) {
    uint32_t x = xw;
    x ^= x >> 16; x *= 0x7feb352du;
    x = x ^ (x >> 15) ^ k2; x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// n / d for n*d < 2^32 with m = floor(2^32/d)+1 (m == 0 encodes d == 1)
struct FastDiv { uint32_t d, m; };
__device__ __forceinline__ uint32_t fdiv(uint32_t n, FastDiv f) { return f.m ? __umulhi(n, f.m) : n; }
static FastDiv make_fastdiv(uint32_t d) {
    FastDiv f; f.d = d; f.m = d <= 1 ? 0u : (uint32_t)((1ull << 32) / d) + 1u; return f;
}

// per-plane scale of Eq. (quantization): delta = min, Delta = range/L,
// inv = L/range bumped by one ulp when range*inv would fall short of L
__device__ __forceinline__ void plane_scale(float mn, float mx, float Lf, float& Delta, float& inv) {
    float range = mx - mn;
    if (range >= 0x1p-90f && range <= 3.4028234663852886e38f) {
        Delta = range / Lf;
        inv = Lf / range;
        if (range * inv < Lf) inv = __uint_as_float(__float_as_uint(inv) + 1u);
    } else {
        Delta = 0.0f;
        inv = 0.0f;
    }
}

// quantise one element against its pair word: floor(t + r/2^16) with
// t = (h - delta) * inv, done exactly in integers (inv16 = inv * 2^16)
template <int ODD>
__device__ __forceinline__ uint32_t quant(float h, float delta, float inv16, uint32_t w) {
    float d = h - delta;
    float t16 = d * inv16;
    uint32_t T = (uint32_t)t16;                  // truncation; t16 >= 0
    uint32_t r = ODD ? (w >> 16) : (w & 0xffffu);
    return (T + r) >> 16;
}

// byte ranges between / after the three regions of the packed buffer that
// must read as zero (each shorter than 16 bytes)
struct Pads { uint8_t* base; size_t off[3]; uint32_t len[3]; };

__device__ __forceinline__ void zero_pads(const Pads& pd, uint32_t tid) {
    if (tid < 48) {
        const uint32_t k = tid >> 4, j = tid & 15u;
        if (j < pd.len[k]) pd.base[pd.off[k] + j] = 0;
    }
}

struct TileArgs {
    Pads pads;
    const void* x;
    uint32_t* codes;
    float* meta;
    void* lfc;
    uint32_t P, H, W, HW, LH, LW, nb, WPP;
    uint32_t G;          // planes per workgroup
    uint32_t ipr;        // item slots per block row (padded to the items-per-block count)
    uint32_t ipp;        // item slots per plane = LH * ipr
    uint32_t S;          // lanes cooperating on one plane's min/max (power of two <= 64)
    uint32_t xs_floats;  // LDS floats reserved for the chunk (multiple of 4)
    uint32_t items_cap;  // LDS floats reserved per item array
    uint32_t vec_load;   // chunk starts are 16-byte aligned
    uint32_t seed_a, seed_c;
    FastDiv d_ipp, d_ipr, d_wpp;
};

// ------------------------------------------------------------------ compress, LDS tile

// T: element type; BITS: code width; B: block size (4 or 8); VEC: elements per
// LDS vector access in the pooling phase (W % VEC == 0, B % VEC == 0).
template <typename T, int BITS, int B, int VEC>
__global__ void __launch_bounds__(kThreads) compress_tile(TileArgs a) {
    extern __shared__ float4 smem4[];
    float4* params = smem4;                                   // [G] (delta, inv16, k1, k2)
    float* xs = reinterpret_cast<float*>(smem4 + a.G);        // [G*HW] x, later the residual h
    float* item_min = xs + a.xs_floats;                       // [items_cap]
    float* item_max = item_min + a.items_cap;                 // [items_cap]

    constexpr int IPB = B / VEC;          // pooling items per block (power of two)
    constexpr int CPW = 32 / BITS;        // codes per word
    constexpr float Lf = float((1 << BITS) - 1);
    const uint32_t tid = threadIdx.x;
    const uint32_t p0 = blockIdx.x * a.G;
    const uint32_t Gc = min(a.G, a.P - p0);
    const uint32_t n = Gc * a.HW;
    if (blockIdx.x == 0) zero_pads(a.pads, tid);

    // ---- phase 0: chunk -> LDS (fp32), coalesced 16-byte loads
    {
        const T* src = static_cast<const T*>(a.x) + (size_t)p0 * a.HW;
        constexpr uint32_t EPV = 16 / sizeof(T);
        uint32_t nv = a.vec_load ? n / EPV : 0;
        const u32x4* src4 = reinterpret_cast<const u32x4*>(src);
        for (uint32_t v0 = 0; v0 < nv; v0 += 4 * kThreads) {
            u32x4 q[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                uint32_t v = v0 + u * kThreads + tid;
                if (v < nv) q[u] = __builtin_nontemporal_load(src4 + v);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                uint32_t v = v0 + u * kThreads + tid;
                if (v < nv) {
                    if constexpr (sizeof(T) == 4) {
                        reinterpret_cast<u32x4*>(xs)[v] = q[u];
                    } else {
                        float4 lo, hi;
                        lo.x = __uint_as_float(q[u].x << 16); lo.y = __uint_as_float(q[u].x & 0xffff0000u);
                        lo.z = __uint_as_float(q[u].y << 16); lo.w = __uint_as_float(q[u].y & 0xffff0000u);
                        hi.x = __uint_as_float(q[u].z << 16); hi.y = __uint_as_float(q[u].z & 0xffff0000u);
                        hi.z = __uint_as_float(q[u].w << 16); hi.w = __uint_as_float(q[u].w & 0xffff0000u);
                        reinterpret_cast<float4*>(xs)[2 * v] = lo;
                        reinterpret_cast<float4*>(xs)[2 * v + 1] = hi;
                    }
                }
            }
        }
        for (uint32_t e = nv * EPV + tid; e < n; e += kThreads) xs[e] = Elem<T>::load(src, e);
    }
    __syncthreads();

    // ---- phase 1: block means (Sec. 4.1 AveragePooling), residual in place
    // item = (plane g, block row bi, slot s): B rows x VEC columns of one block
    const uint32_t nitems = Gc * a.ipp;
    for (uint32_t it0 = 0; it0 < nitems; it0 += kThreads) {
        const uint32_t it = it0 + tid;
        const uint32_t g = fdiv(it, a.d_ipp);
        const uint32_t rem = it - g * a.ipp;
        const uint32_t bi = fdiv(rem, a.d_ipr);
        const uint32_t s = rem - bi * a.ipr;
        const uint32_t col0 = s * VEC;
        const uint32_t r0 = bi * B;
        const bool valid = it < nitems && col0 < a.W;
        const uint32_t base = g * a.HW + r0 * a.W + col0;

        float v[B][VEC];
        double S = 0.0;
#pragma unroll
        for (int rr = 0; rr < B; ++rr) {
            const bool ok = valid && (r0 + rr < a.H);
#pragma unroll
            for (int c = 0; c < VEC; ++c) v[rr][c] = 0.0f;
            if (ok) {
                const float* src = xs + base + rr * a.W;
                if constexpr (VEC == 4) {
                    float4 q = *reinterpret_cast<const float4*>(src);
                    v[rr][0] = q.x; v[rr][1] = q.y; v[rr][2] = q.z; v[rr][3] = q.w;
                } else if constexpr (VEC == 2) {
                    float2 q = *reinterpret_cast<const float2*>(src);
                    v[rr][0] = q.x; v[rr][1] = q.y;
                } else {
                    v[rr][0] = src[0];
                }
            }
#pragma unroll
            for (int c = 0; c < VEC; ++c) S += (double)v[rr][c];
        }
#pragma unroll
        for (int off = 1; off < IPB; off <<= 1) S += __shfl_xor(S, off);

        const uint32_t bj = s / IPB;
        const uint32_t rows = min((uint32_t)B, a.H - min(a.H, r0));
        const uint32_t cols = min((uint32_t)B, a.W - min(a.W, bj * B));
        const uint32_t cnt = max(rows * cols, 1u);
        // exact sum / count, one rounding to fp32, then to the storage type
        float m;
        if ((cnt & (cnt - 1)) == 0) m = (float)(S * (1.0 / (double)cnt));   // power of two: exact scaling
        else m = (float)(S / (double)cnt);
        const float lfc = Elem<T>::round(m);
        if (valid && (s % IPB) == 0)
            Elem<T>::store(static_cast<T*>(a.lfc), (size_t)(p0 + g) * a.nb + bi * a.LW + bj, lfc);

        // Sec. 4.1: H^H = H - UpSampling(H^L); written back over x
        float hmin = __builtin_inff(), hmax = -__builtin_inff();
#pragma unroll
        for (int rr = 0; rr < B; ++rr) {
            const bool ok = valid && (r0 + rr < a.H);
            if (ok) {
                float h[VEC];
#pragma unroll
                for (int c = 0; c < VEC; ++c) {
                    h[c] = v[rr][c] - lfc;
                    hmin = fminf(hmin, h[c]);
                    hmax = fmaxf(hmax, h[c]);
                }
                float* dst = xs + base + rr * a.W;
                if constexpr (VEC == 4) *reinterpret_cast<float4*>(dst) = make_float4(h[0], h[1], h[2], h[3]);
                else if constexpr (VEC == 2) *reinterpret_cast<float2*>(dst) = make_float2(h[0], h[1]);
                else dst[0] = h[0];
            }
        }
        if (it < nitems) { item_min[it] = hmin; item_max[it] = hmax; }
    }
    __syncthreads();

    // ---- phase 2: per-plane min / max, scale of Eq. (quantization), keys
    {
        const uint32_t S = a.S;
        const uint32_t groups = kThreads / S;
        const uint32_t sub = tid & (S - 1);
        for (uint32_t g0 = 0; g0 < Gc; g0 += groups) {
            const uint32_t g = g0 + tid / S;
            const bool live = g < Gc;
            float mn = __builtin_inff(), mx = -__builtin_inff();
            if (live) {
                const uint32_t b0 = g * a.ipp;
                for (uint32_t k = sub; k < a.ipp; k += S) {
                    mn = fminf(mn, item_min[b0 + k]);
                    mx = fmaxf(mx, item_max[b0 + k]);
                }
            }
            for (uint32_t off = S >> 1; off > 0; off >>= 1) {
                mn = fminf(mn, __shfl_xor(mn, off));
                mx = fmaxf(mx, __shfl_xor(mx, off));
            }
            if (live && sub == 0) {
                float Delta, inv;
                plane_scale(mn, mx, Lf, Delta, inv);
                const uint32_t p = p0 + g;
                reinterpret_cast<float2*>(a.meta)[p] = make_float2(mn, Delta);
                const uint32_t k1 = mix32(p ^ a.seed_a);
                const uint32_t k2 = mix32(k1 + a.seed_c);
                params[g] = make_float4(mn, inv * 65536.0f, __uint_as_float(k1), __uint_as_float(k2));
            }
        }
    }
    __syncthreads();

    // ---- phase 3: Quant of Eq. (quantization) + packing, one word per lane
    {
        const uint32_t nwords = Gc * a.WPP;
        const bool hw4 = (a.HW & 3u) == 0;
        for (uint32_t wi = tid; wi < nwords; wi += kThreads) {
            const uint32_t g = fdiv(wi, a.d_wpp);
            const uint32_t k = wi - g * a.WPP;
            const float4 pr = params[g];
            const float delta = pr.x, inv16 = pr.y;
            const uint32_t k1 = __float_as_uint(pr.z), k2 = __float_as_uint(pr.w);
            const uint32_t e0 = k * CPW;
            const uint32_t left = a.HW - e0;
            const float* hp = xs + g * a.HW + e0;
            float h[CPW];
            if (hw4 && left >= (uint32_t)CPW) {
#pragma unroll
                for (int q = 0; q < CPW / 4; ++q) {
                    float4 f = reinterpret_cast<const float4*>(hp)[q];
                    h[4 * q] = f.x; h[4 * q + 1] = f.y; h[4 * q + 2] = f.z; h[4 * q + 3] = f.w;
                }
            } else {
                // ragged tail: elements past the plane take h = delta -> t = 0 -> code 0
#pragma unroll
                for (int e = 0; e < CPW; ++e) h[e] = (uint32_t)e < left ? hp[e] : delta;
            }
            uint32_t xw = k1 + (k * (CPW / 2)) * kWeyl;
            uint32_t word = 0;
#pragma unroll
            for (int j = 0; j < CPW / 2; ++j) {
                const uint32_t w = pair_word(xw, k2);
                xw += kWeyl;
                word |= quant<0>(h[2 * j], delta, inv16, w) << (2 * j * BITS);
                word |= quant<1>(h[2 * j + 1], delta, inv16, w) << ((2 * j + 1) * BITS);
            }
            a.codes[(size_t)(p0 + g) * a.WPP + k] = word;
        }
    }
}

// ------------------------------------------------------------------ compress, any shape (slow)

struct AnyArgs {
    Pads pads;
    const void* x;
    uint32_t* codes;
    float* meta;
    void* lfc;
    uint32_t P, H, W, HW, LH, LW, nb, WPP, B;
    uint32_t seed_a, seed_c;
};

// One workgroup per plane; x is re-read from global memory in each pass.
template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) compress_any(AnyArgs a) {
    __shared__ float red_min[kThreads], red_max[kThreads];
    __shared__ float4 sh_params;
    constexpr int CPW = 32 / BITS;
    constexpr float Lf = float((1 << BITS) - 1);
    const uint32_t tid = threadIdx.x;
    const uint32_t p = blockIdx.x;
    const T* xp = static_cast<const T*>(a.x) + (size_t)p * a.HW;
    T* lfcp = static_cast<T*>(a.lfc) + (size_t)p * a.nb;
    if (p == 0) zero_pads(a.pads, tid);

    // pass A: block means; block min/max of the residual follow from the
    // block min/max of x because x -> fl(x - m) is monotone
    float mn = __builtin_inff(), mx = -__builtin_inff();
    for (uint32_t blk = tid; blk < a.nb; blk += kThreads) {
        const uint32_t bi = blk / a.LW, bj = blk - bi * a.LW;
        const uint32_t r1 = min(a.H, (bi + 1) * a.B), c1 = min(a.W, (bj + 1) * a.B);
        double S = 0.0;
        float xmin = __builtin_inff(), xmax = -__builtin_inff();
        uint32_t cnt = 0;
        for (uint32_t r = bi * a.B; r < r1; ++r)
            for (uint32_t c = bj * a.B; c < c1; ++c) {
                const float v = Elem<T>::load(xp, (size_t)r * a.W + c);
                S += (double)v; xmin = fminf(xmin, v); xmax = fmaxf(xmax, v); ++cnt;
            }
        const float lfc = Elem<T>::round((float)(S / (double)cnt));
        Elem<T>::store(lfcp, blk, lfc);
        mn = fminf(mn, xmin - lfc);
        mx = fmaxf(mx, xmax - lfc);
    }
    red_min[tid] = mn; red_max[tid] = mx;
    __syncthreads();
    for (uint32_t off = kThreads / 2; off > 0; off >>= 1) {
        if (tid < off) {
            red_min[tid] = fminf(red_min[tid], red_min[tid + off]);
            red_max[tid] = fmaxf(red_max[tid], red_max[tid + off]);
        }
        __syncthreads();
    }
    if (tid == 0) {
        float Delta, inv;
        plane_scale(red_min[0], red_max[0], Lf, Delta, inv);
        reinterpret_cast<float2*>(a.meta)[p] = make_float2(red_min[0], Delta);
        const uint32_t k1 = mix32(p ^ a.seed_a);
        const uint32_t k2 = mix32(k1 + a.seed_c);
        sh_params = make_float4(red_min[0], inv * 65536.0f, __uint_as_float(k1), __uint_as_float(k2));
    }
    __syncthreads();
    const float delta = sh_params.x, inv16 = sh_params.y;
    const uint32_t k1 = __float_as_uint(sh_params.z), k2 = __float_as_uint(sh_params.w);

    // pass B: quantise and pack, one word per thread
    for (uint32_t k = tid; k < a.WPP; k += kThreads) {
        uint32_t word = 0;
        for (int e = 0; e < CPW; ++e) {
            const uint32_t i = k * CPW + e;
            if (i >= a.HW) break;
            const uint32_t r = i / a.W, c = i - r * a.W;
            // written by this workgroup in pass A; visible after the barrier above
            const float lfc = Elem<T>::load(lfcp, (r / a.B) * a.LW + c / a.B);
            const float h = Elem<T>::load(xp, i) - lfc;
            const uint32_t w = pair_word(k1 + (i >> 1) * kWeyl, k2);
            const uint32_t q = (i & 1u) ? quant<1>(h, delta, inv16, w) : quant<0>(h, delta, inv16, w);
            word |= q << (e * BITS);
        }
        a.codes[(size_t)p * a.WPP + k] = word;
    }
}

// ------------------------------------------------------------------ decompress

struct DecArgs {
    const uint32_t* codes;
    const float* meta;
    const void* lfc;
    void* xhat;
    uint32_t P, H, W, HW, LH, LW, nb, WPP, B;
    uint32_t G;          // planes per workgroup
    uint32_t q4;         // HW / 4
    uint32_t w4;         // W / 4
    FastDiv d_q4, d_w4, d_B, d_W, d_HW;
};

// Sec. 4.2: hh = Delta*q + delta ; reconstruction: xhat = lfc + hh (three fp32 ops)
__device__ __forceinline__ float dequant(uint32_t q, float Delta, float delta, float lfc) {
    float hh = (float)q * Delta;
    hh = hh + delta;
    return lfc + hh;
}

template <typename T>
__device__ __forceinline__ void store4(T* dst, size_t i, float a, float b, float c, float d) {
    if constexpr (sizeof(T) == 4) {
        *reinterpret_cast<float4*>(dst + i) = make_float4(a, b, c, d);
    } else {
        uint2 o;
        o.x = float_to_bf16_bits(a) | (float_to_bf16_bits(b) << 16);
        o.y = float_to_bf16_bits(c) | (float_to_bf16_bits(d) << 16);
        *reinterpret_cast<uint2*>(dst + i) = o;
    }
}

// W % 4 == 0 and B % 4 == 0: the four elements of a vector lie in one row and
// share one LFC value.  A workgroup streams G whole planes.
template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) decompress_rowvec(DecArgs a) {
    const uint32_t tid = threadIdx.x;
    const uint32_t p0 = blockIdx.x * a.G;
    const uint32_t Gc = min(a.G, a.P - p0);
    const uint32_t nvec = Gc * a.q4;
    constexpr uint32_t Lq = (1u << BITS) - 1u;
    for (uint32_t vi = tid; vi < nvec; vi += kThreads) {
        const uint32_t g = fdiv(vi, a.d_q4);
        const uint32_t fi = vi - g * a.q4;        // vector index inside the plane
        const uint32_t p = p0 + g;
        const float2 dd = reinterpret_cast<const float2*>(a.meta)[p];
        uint32_t c4;                               // the four codes, BITS apart from bit 0
        if constexpr (BITS == 2) c4 = reinterpret_cast<const uint8_t*>(a.codes)[(size_t)p * a.WPP * 4 + fi];
        else c4 = reinterpret_cast<const uint16_t*>(a.codes)[(size_t)p * a.WPP * 2 + fi];
        const uint32_t r = fdiv(fi, a.d_w4);
        const uint32_t c = (fi - r * a.w4) * 4;
        const T* lfcp = static_cast<const T*>(a.lfc) + (size_t)p * a.nb;
        const float lfc = Elem<T>::load(lfcp, fdiv(r, a.d_B) * a.LW + fdiv(c, a.d_B));
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = dequant((c4 >> (e * BITS)) & Lq, dd.y, dd.x, lfc);
        store4(static_cast<T*>(a.xhat), (size_t)p * a.HW + (size_t)fi * 4, o[0], o[1], o[2], o[3]);
    }
}

// Any W, H, B: a workgroup streams G whole planes as one flat run of elements,
// four consecutive elements per lane step; every element finds its own plane,
// row, column and block.  G*HW is a multiple of 4 whenever G < P remains, so
// vector stores stay aligned; the ragged end of the last chunk is scalar.
template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) decompress_flat(DecArgs a) {
    constexpr uint32_t CPW = 32 / BITS;
    constexpr uint32_t Lq = (1u << BITS) - 1u;
    const uint32_t tid = threadIdx.x;
    const uint32_t p0 = blockIdx.x * a.G;
    const uint32_t Gc = min(a.G, a.P - p0);
    const uint32_t n = Gc * a.HW;
    T* out = static_cast<T*>(a.xhat) + (size_t)p0 * a.HW;
    for (uint32_t e0 = tid * 4; e0 < n; e0 += kThreads * 4) {
        uint32_t g = fdiv(e0, a.d_HW);
        uint32_t i = e0 - g * a.HW;
        uint32_t r = fdiv(i, a.d_W);
        uint32_t c = i - r * a.W;
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o[e] = 0.0f;
            if (e0 + e < n) {
                const uint32_t p = p0 + g;
                const float2 dd = reinterpret_cast<const float2*>(a.meta)[p];
                const uint32_t q = (a.codes[(size_t)p * a.WPP + i / CPW] >> ((i % CPW) * BITS)) & Lq;
                const T* lfcp = static_cast<const T*>(a.lfc) + (size_t)p * a.nb;
                const float lfc = Elem<T>::load(lfcp, fdiv(r, a.d_B) * a.LW + fdiv(c, a.d_B));
                o[e] = dequant(q, dd.y, dd.x, lfc);
                ++i;
                if (++c == a.W) { c = 0; ++r; }
                if (i == a.HW) { i = 0; r = 0; ++g; }
            }
        }
        if (e0 + 4 <= n) {
            store4(out, e0, o[0], o[1], o[2], o[3]);
        } else {
            for (int e = 0; e < 4; ++e)
                if (e0 + e < n) Elem<T>::store(out, e0 + e, o[e]);
        }
    }
}

// planes too large for the 32-bit index tricks above: one element per thread step
template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) decompress_scalar(DecArgs a) {
    constexpr uint32_t CPW = 32 / BITS;
    constexpr uint32_t Lq = (1u << BITS) - 1u;
    const uint32_t p = blockIdx.x;
    const float2 dd = reinterpret_cast<const float2*>(a.meta)[p];
    const T* lfcp = static_cast<const T*>(a.lfc) + (size_t)p * a.nb;
    const uint32_t* cp = a.codes + (size_t)p * a.WPP;
    T* out = static_cast<T*>(a.xhat) + (size_t)p * a.HW;
    for (uint32_t i = threadIdx.x; i < a.HW; i += kThreads) {
        const uint32_t r = i / a.W, c = i - r * a.W;
        const uint32_t q = (cp[i / CPW] >> ((i % CPW) * BITS)) & Lq;
        const float lfc = Elem<T>::load(lfcp, (r / a.B) * a.LW + c / a.B);
        Elem<T>::store(out, i, dequant(q, dd.y, dd.x, lfc));
    }
}

// ------------------------------------------------------------------ host side

struct Layout {
    uint64_t P, HW, LH, LW, nb, WPP;
    size_t codes_off, codes_bytes, meta_off, meta_bytes, lfc_off, lfc_bytes, total;
};

size_t align16(size_t v) { return (v + 15u) & ~(size_t)15u; }

int make_layout(int64_t N, int64_t C, int64_t H, int64_t W, int B, int b, int dt, Layout* L) {
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || B < 1 || (b != 2 && b != 4)) return DIVISION_EINVAL;
    if (dt != DIVISION_F32 && dt != DIVISION_BF16) return DIVISION_EINVAL;
    const uint64_t lim31 = 0x7fffffffull;
    if ((uint64_t)N > lim31 || (uint64_t)C > lim31 || (uint64_t)H > lim31 || (uint64_t)W > lim31) return DIVISION_ERANGE;
    L->P = (uint64_t)N * (uint64_t)C;
    L->HW = (uint64_t)H * (uint64_t)W;
    if (L->P > lim31 || L->HW > lim31 || L->P * L->HW > (1ull << 40)) return DIVISION_ERANGE;
    L->LH = ((uint64_t)H + B - 1) / B;
    L->LW = ((uint64_t)W + B - 1) / B;
    L->nb = L->LH * L->LW;
    const uint64_t cpw = 32 / b;
    L->WPP = (L->HW + cpw - 1) / cpw;
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    L->codes_off = 0;
    L->codes_bytes = (size_t)(4 * L->P * L->WPP);
    L->meta_off = align16(L->codes_bytes);
    L->meta_bytes = (size_t)(8 * L->P);
    L->lfc_off = align16(L->meta_off + L->meta_bytes);
    L->lfc_bytes = (size_t)(es * L->P * L->nb);
    L->total = align16(L->lfc_off + L->lfc_bytes);
    return DIVISION_OK;
}

uint64_t gcd_u64(uint64_t a, uint64_t b) { while (b) { uint64_t t = a % b; a = b; b = t; } return a; }

// fdiv(n, d) is exact while n*d < 2^32
bool fastdiv_ok(uint64_t n_max, uint64_t d) { return n_max * d < (1ull << 32); }

Pads make_pads(char* pk, const Layout& L) {
    Pads pd;
    pd.base = reinterpret_cast<uint8_t*>(pk);
    pd.off[0] = L.codes_off + L.codes_bytes; pd.len[0] = (uint32_t)(L.meta_off - pd.off[0]);
    pd.off[1] = L.meta_off + L.meta_bytes;   pd.len[1] = (uint32_t)(L.lfc_off - pd.off[1]);
    pd.off[2] = L.lfc_off + L.lfc_bytes;     pd.len[2] = (uint32_t)(L.total - pd.off[2]);
    return pd;
}

// dynamic LDS above the default limit needs a one-time opt-in per kernel
hipError_t allow_large_lds(void (*kern)(TileArgs), size_t lds) {
    if (lds <= 48u * 1024u) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax);
}

template <typename T, int BITS, int B>
hipError_t launch_tile_vec(int vec, const TileArgs& a, uint32_t grid, size_t lds, hipStream_t st) {
    void (*kern)(TileArgs) = vec == 4 ? compress_tile<T, BITS, B, 4>
                           : vec == 2 ? compress_tile<T, BITS, B, 2>
                                      : compress_tile<T, BITS, B, 1>;
    hipError_t e = allow_large_lds(kern, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, st, a);
    return hipGetLastError();
}

template <typename T, int BITS>
hipError_t launch_tile(int B, int vec, const TileArgs& a, uint32_t grid, size_t lds, hipStream_t st) {
    return B == 8 ? launch_tile_vec<T, BITS, 8>(vec, a, grid, lds, st)
                  : launch_tile_vec<T, BITS, 4>(vec, a, grid, lds, st);
}

// Fills the tiled-compress launch plan; false when the shape is not covered.
bool plan_tile(const Layout& L, int64_t H, int64_t W, int B, size_t es, const void* x,
               TileArgs* a, uint32_t* grid, size_t* lds, int* vec_out) {
    if (B != 4 && B != 8) return false;
    const int vec = (W % 4 == 0) ? 4 : (W % 2 == 0) ? 2 : 1;
    const uint32_t ipb = (uint32_t)B / (uint32_t)vec;
    const uint64_t slots = ((uint64_t)W + vec - 1) / vec;
    const uint64_t ipr = (slots + ipb - 1) / ipb * ipb;
    const uint64_t ipp = L.LH * ipr;
    const uint64_t per_plane = 4ull * L.HW + 8ull * ipp + 16ull;
    if (per_plane + 64 > kLdsMax) return false;
    uint64_t G = kLdsTarget / per_plane;
    if (G < 1) G = 1;
    // chunk starts stay 16-byte aligned when G * (bytes per plane) is a multiple of 16
    const uint64_t unit = 16 / gcd_u64(16, L.HW * es);
    uint32_t vec_load = ((uintptr_t)x % 16) == 0;
    if (vec_load && unit > 1) {
        const uint64_t Gr = (G + unit - 1) / unit * unit;
        if (Gr * per_plane + 64 <= kLdsMax) G = Gr; else vec_load = 0;
    }
    if (G > L.P) G = L.P;
    const uint64_t nitems = G * ipp, nwords = G * L.WPP;
    if (!fastdiv_ok(nitems + kThreads, ipp) || !fastdiv_ok(ipp, ipr) || !fastdiv_ok(nwords + kThreads, L.WPP))
        return false;
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW;
    a->LH = (uint32_t)L.LH; a->LW = (uint32_t)L.LW; a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP;
    a->G = (uint32_t)G; a->ipr = (uint32_t)ipr; a->ipp = (uint32_t)ipp;
    uint32_t S = 1;
    while (S < 64 && (uint64_t)S * 2 <= ipp) S *= 2;
    a->S = S;
    a->xs_floats = (uint32_t)((G * L.HW + 3) / 4 * 4);
    a->items_cap = (uint32_t)((nitems + 3) / 4 * 4);
    a->vec_load = vec_load;
    a->d_ipp = make_fastdiv((uint32_t)ipp);
    a->d_ipr = make_fastdiv((uint32_t)ipr);
    a->d_wpp = make_fastdiv((uint32_t)L.WPP);
    *lds = 16ull * G + 4ull * a->xs_floats + 8ull * a->items_cap;
    *grid = (uint32_t)((L.P + G - 1) / G);
    *vec_out = vec;
    return *lds <= kLdsMax;
}

}  // namespace

// ------------------------------------------------------------------ C ABI

extern "C" {

int division_abi_version(void) { return 1; }

size_t division_packed_bytes(int64_t N, int64_t C, int64_t H, int64_t W, int B, int b, division_dtype dt) {
    Layout L;
    if (make_layout(N, C, H, W, B, b, (int)dt, &L) != DIVISION_OK) return 0;
    return L.total;
}

int division_packed_layout(int64_t N, int64_t C, int64_t H, int64_t W, int B, int b, division_dtype dt,
                           size_t* codes_off, size_t* codes_bytes, size_t* meta_off, size_t* meta_bytes,
                           size_t* lfc_off, size_t* lfc_bytes) {
    if (!codes_off || !codes_bytes || !meta_off || !meta_bytes || !lfc_off || !lfc_bytes) return DIVISION_EINVAL;
    Layout L;
    if (make_layout(N, C, H, W, B, b, (int)dt, &L) != DIVISION_OK) return DIVISION_EINVAL;
    *codes_off = L.codes_off; *codes_bytes = L.codes_bytes;
    *meta_off = L.meta_off;   *meta_bytes = L.meta_bytes;
    *lfc_off = L.lfc_off;     *lfc_bytes = L.lfc_bytes;
    return DIVISION_OK;
}

int division_compress(const void* x, int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt,
                      int B, int b, uint64_t seed, void* packed, size_t packed_capacity, void* hip_stream) {
    if (!x || !packed) return DIVISION_EINVAL;
    Layout L;
    const int rc = make_layout(N, C, H, W, B, b, (int)dt, &L);
    if (rc != DIVISION_OK) return rc;
    if (packed_capacity < L.total) return DIVISION_ESIZE;
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    if (((uintptr_t)x % es) != 0 || ((uintptr_t)packed % 16) != 0) return DIVISION_EALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char* pk = static_cast<char*>(packed);
    const uint32_t seed_a = mix32((uint32_t)(seed & 0xffffffffu) ^ 0x243F6A88u);
    const uint32_t seed_c = mix32((uint32_t)(seed >> 32) ^ 0x85A308D3u);

    TileArgs a{};
    size_t lds = 0;
    uint32_t grid = 0;
    int vec = 1;
    hipError_t err;
    if (plan_tile(L, H, W, B, es, x, &a, &grid, &lds, &vec)) {
        a.pads = make_pads(pk, L);
        a.x = x;
        a.codes = reinterpret_cast<uint32_t*>(pk + L.codes_off);
        a.meta = reinterpret_cast<float*>(pk + L.meta_off);
        a.lfc = pk + L.lfc_off;
        a.seed_a = seed_a; a.seed_c = seed_c;
        if (dt == DIVISION_F32)
            err = b == 2 ? launch_tile<float, 2>(B, vec, a, grid, lds, st) : launch_tile<float, 4>(B, vec, a, grid, lds, st);
        else
            err = b == 2 ? launch_tile<bf16_t, 2>(B, vec, a, grid, lds, st) : launch_tile<bf16_t, 4>(B, vec, a, grid, lds, st);
    } else {
        AnyArgs g{};
        g.pads = make_pads(pk, L);
        g.x = x;
        g.codes = reinterpret_cast<uint32_t*>(pk + L.codes_off);
        g.meta = reinterpret_cast<float*>(pk + L.meta_off);
        g.lfc = pk + L.lfc_off;
        g.P = (uint32_t)L.P; g.H = (uint32_t)H; g.W = (uint32_t)W; g.HW = (uint32_t)L.HW;
        g.LH = (uint32_t)L.LH; g.LW = (uint32_t)L.LW; g.nb = (uint32_t)L.nb; g.WPP = (uint32_t)L.WPP; g.B = (uint32_t)B;
        g.seed_a = seed_a; g.seed_c = seed_c;
        const dim3 gr((uint32_t)L.P), bl(kThreads);
        if (dt == DIVISION_F32) {
            if (b == 2) hipLaunchKernelGGL((compress_any<float, 2>), gr, bl, 0, st, g);
            else hipLaunchKernelGGL((compress_any<float, 4>), gr, bl, 0, st, g);
        } else {
            if (b == 2) hipLaunchKernelGGL((compress_any<bf16_t, 2>), gr, bl, 0, st, g);
            else hipLaunchKernelGGL((compress_any<bf16_t, 4>), gr, bl, 0, st, g);
        }
        err = hipGetLastError();
    }
    return err == hipSuccess ? DIVISION_OK : DIVISION_EHIP;
}

int division_decompress(const void* packed, size_t packed_bytes, int64_t N, int64_t C, int64_t H, int64_t W,
                        division_dtype dt, int B, int b, void* xhat, void* hip_stream) {
    if (!xhat || !packed) return DIVISION_EINVAL;
    Layout L;
    const int rc = make_layout(N, C, H, W, B, b, (int)dt, &L);
    if (rc != DIVISION_OK) return rc;
    if (packed_bytes < L.total) return DIVISION_ESIZE;
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    if (((uintptr_t)xhat % es) != 0 || ((uintptr_t)packed % 16) != 0) return DIVISION_EALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const char* pk = static_cast<const char*>(packed);

    DecArgs a{};
    a.codes = reinterpret_cast<const uint32_t*>(pk + L.codes_off);
    a.meta = reinterpret_cast<const float*>(pk + L.meta_off);
    a.lfc = pk + L.lfc_off;
    a.xhat = xhat;
    a.P = (uint32_t)L.P; a.H = (uint32_t)H; a.W = (uint32_t)W; a.HW = (uint32_t)L.HW;
    a.LH = (uint32_t)L.LH; a.LW = (uint32_t)L.LW; a.nb = (uint32_t)L.nb; a.WPP = (uint32_t)L.WPP; a.B = (uint32_t)B;
    a.d_B = make_fastdiv((uint32_t)B);
    a.d_W = make_fastdiv((uint32_t)W);
    a.d_HW = make_fastdiv((uint32_t)L.HW);
    const bool small_idx = fastdiv_ok((uint64_t)H, (uint64_t)B) && fastdiv_ok((uint64_t)W, (uint64_t)B);
    const bool out_vec_aligned = ((uintptr_t)xhat % (4 * es)) == 0;
    const uint64_t target = 16ull * 4 * kThreads;      // elements per workgroup

    void (*kern)(DecArgs) = nullptr;
    uint32_t grid = 0;
    // fast path: rows are whole vectors that sit inside one block
    if (W % 4 == 0 && B % 4 == 0 && small_idx && out_vec_aligned) {
        a.q4 = (uint32_t)(L.HW / 4);
        a.w4 = (uint32_t)(W / 4);
        uint64_t G = (target / 4 + a.q4 - 1) / a.q4;
        if (G > L.P) G = L.P;
        while (G > 1 && !fastdiv_ok(G * a.q4 + kThreads, a.q4)) --G;
        if (fastdiv_ok(G * a.q4 + kThreads, a.q4) && fastdiv_ok(a.q4, a.w4)) {
            a.G = (uint32_t)G;
            a.d_q4 = make_fastdiv(a.q4);
            a.d_w4 = make_fastdiv(a.w4);
            grid = (uint32_t)((L.P + G - 1) / G);
            if (dt == DIVISION_F32) kern = b == 2 ? decompress_rowvec<float, 2> : decompress_rowvec<float, 4>;
            else kern = b == 2 ? decompress_rowvec<bf16_t, 2> : decompress_rowvec<bf16_t, 4>;
        }
    }
    // general path: flat run of G planes, G*HW a multiple of 4
    if (!kern && small_idx && out_vec_aligned && fastdiv_ok(L.HW, (uint64_t)W)) {
        const uint64_t unit = 4 / gcd_u64(4, L.HW);
        uint64_t G = (target + L.HW - 1) / L.HW;
        G = (G + unit - 1) / unit * unit;
        if (G > L.P) G = L.P;
        if (fastdiv_ok(G * L.HW + 4ull * kThreads, L.HW)) {
            a.G = (uint32_t)G;
            grid = (uint32_t)((L.P + G - 1) / G);
            if (dt == DIVISION_F32) kern = b == 2 ? decompress_flat<float, 2> : decompress_flat<float, 4>;
            else kern = b == 2 ? decompress_flat<bf16_t, 2> : decompress_flat<bf16_t, 4>;
        }
    }
    if (!kern) {
        a.G = 1;
        grid = (uint32_t)L.P;
        if (dt == DIVISION_F32) kern = b == 2 ? decompress_scalar<float, 2> : decompress_scalar<float, 4>;
        else kern = b == 2 ? decompress_scalar<bf16_t, 2> : decompress_scalar<bf16_t, 4>;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), 0, st, a);
    return hipGetLastError() == hipSuccess ? DIVISION_OK : DIVISION_EHIP;
}

}  // extern "C"
