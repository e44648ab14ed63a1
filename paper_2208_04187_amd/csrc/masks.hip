// 1-bit mask operators for AMD MI355X (gfx950): the Relu and Dropout operators of
// "DIVISION: Memory Efficient Training via Dual Activation Precision" (appendix on
// operator compression, Algorithms "Relu operator" and "Dropout operator").
//
//   forward:   V = sgn(H) (Relu) or V ~ Bernoulli(1 - p) (Dropout); out = V (.) H;
//              V is cached one bit per element (N^2/8 bytes per channel).
//   backward:  grad_in = V (.) grad_out.
//
// Pure streaming kernels: one 16-byte vector per lane and step, the lane's 4 (fp32) or
// 8 (bf16) mask bits are merged over 8 or 4 adjacent lanes with DPP and leave as whole
// 32-bit words.  Mask layout: bit i%32 of word i/32, pad bits zero.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/division.h"

namespace {

constexpr int kThreads = 256;
constexpr int kVecPerThread = 4;                  // 16-byte vectors a thread handles, kThreads apart
constexpr uint32_t kWeyl = 0x9E3779B9u;
constexpr uint64_t kDropoutStream = 0xD509A5B3C2E1F047ull;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 32-bit xorshift-multiply finaliser (shifts 16/15/16): the codec's random source
__host__ __device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du;
    x ^= x >> 15; x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// random word of element pair j of a stream segment with keys (k1, k2)
__device__ __forceinline__ uint32_t pair_word(uint32_t k1, uint32_t k2, uint32_t j) {
    uint32_t x = k1 + j * kWeyl;
    x ^= x >> 16; x *= 0x7feb352du;
    x = x ^ (x >> 15) ^ k2; x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, false);
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each 8 lanes

// element helpers: T = float or uint16_t (bf16 bit pattern); values pass through bit for bit
template <typename T> struct Tr;
template <> struct Tr<float> {
    static constexpr int EPV = 4;
    static __device__ __forceinline__ bool positive(uint32_t bits) { return __uint_as_float(bits) > 0.0f; }
};
template <> struct Tr<uint16_t> {
    static constexpr int EPV = 8;
    static __device__ __forceinline__ bool positive(uint32_t bits) { return __uint_as_float(bits << 16) > 0.0f; }
};

// the EPV "is positive" bits of one vector (bit e = element e)
template <typename T>
__device__ __forceinline__ uint32_t positive_bits(u32x4 q) {
    uint32_t m = 0;
    if constexpr (sizeof(T) == 4) {
        m |= Tr<T>::positive(q.x) ? 1u : 0u; m |= Tr<T>::positive(q.y) ? 2u : 0u;
        m |= Tr<T>::positive(q.z) ? 4u : 0u; m |= Tr<T>::positive(q.w) ? 8u : 0u;
    } else {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            m |= Tr<T>::positive(w[k] & 0xffffu) ? (1u << (2 * k)) : 0u;
            m |= Tr<T>::positive(w[k] >> 16) ? (2u << (2 * k)) : 0u;
        }
    }
    return m;
}

// keeps the elements of a vector whose bit is set, +0 elsewhere
template <typename T>
__device__ __forceinline__ u32x4 select_bits(u32x4 q, uint32_t m) {
    u32x4 o;
    if constexpr (sizeof(T) == 4) {
        o.x = (m & 1u) ? q.x : 0u; o.y = (m & 2u) ? q.y : 0u;
        o.z = (m & 4u) ? q.z : 0u; o.w = (m & 8u) ? q.w : 0u;
    } else {
        uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t keep = ((m >> (2 * k)) & 1u ? 0x0000ffffu : 0u) | ((m >> (2 * k + 1)) & 1u ? 0xffff0000u : 0u);
            w[k] &= keep;
        }
        o.x = w[0]; o.y = w[1]; o.z = w[2]; o.w = w[3];
    }
    return o;
}

// Dropout's keep bits of the EPV elements starting at element e0 (a multiple of EPV):
// element i keeps its value iff the 16 random bits of element (i mod 2^32) of stream
// segment i >> 32 are >= T.
template <typename T>
__device__ __forceinline__ uint32_t keep_bits(uint64_t e0, uint32_t seed_a, uint32_t seed_c, uint32_t thr) {
    constexpr int EPV = Tr<T>::EPV;
    const uint32_t seg = (uint32_t)(e0 >> 32);
    const uint32_t k1 = mix32(seg ^ seed_a);
    const uint32_t k2 = mix32(k1 + seed_c);
    const uint32_t j0 = (uint32_t)e0 >> 1;
    uint32_t m = 0;
#pragma unroll
    for (int k = 0; k < EPV / 2; ++k) {
        const uint32_t w = pair_word(k1, k2, j0 + (uint32_t)k);
        m |= ((w & 0xffffu) >= thr ? 1u : 0u) << (2 * k);
        m |= ((w >> 16) >= thr ? 2u : 0u) << (2 * k);
    }
    return m;
}

// merges the per-lane bit groups of 32/EPV adjacent lanes into the 32-bit mask word they
// share (every lane of the group ends up with the whole word); all lanes must be active
template <typename T>
__device__ __forceinline__ uint32_t merge_word(uint32_t m, uint32_t lane) {
    constexpr int EPV = Tr<T>::EPV;
    constexpr uint32_t LPW = 32 / EPV;               // lanes per word: 8 (fp32) or 4 (bf16)
    uint32_t v = m << (EPV * (lane & (LPW - 1)));
    v |= dpp_u32<kDppXor1>(v);
    v |= dpp_u32<kDppXor2>(v);
    if constexpr (LPW == 8) v |= dpp_u32<kDppHalfMirror>(v);
    return v;
}

struct MaskArgs {
    const void* in;        // x (forward) or grad_out (backward)
    void* out;             // y or grad_in
    uint32_t* mask;
    uint64_t n;            // elements
    uint64_t nwords;       // mask words = ceil(n / 32)
    uint32_t vec;          // in and out are 16-byte aligned: whole vectors move with 16-byte accesses
    uint32_t seed_a, seed_c, thr;      // dropout only
};

// MODE 0: Relu forward, 1: Dropout forward, 2: backward (mask is read)
template <typename T, int MODE>
__global__ void __launch_bounds__(kThreads) mask_kernel(MaskArgs a) {
    constexpr int EPV = Tr<T>::EPV;
    constexpr uint32_t LPW = 32 / EPV;
    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const T* in = static_cast<const T*>(a.in);
    T* out = static_cast<T*>(a.out);
    const uint64_t v0 = (uint64_t)blockIdx.x * (kThreads * kVecPerThread) + tid;
#pragma unroll
    for (int u = 0; u < kVecPerThread; ++u) {
        const uint64_t vi = v0 + (uint64_t)u * kThreads;       // the lane's vector
        const uint64_t e0 = vi * EPV;
        const bool whole = e0 + EPV <= a.n;
        const bool fast = whole && a.vec;
        u32x4 q = {0u, 0u, 0u, 0u};
        if (fast) {
            q = *reinterpret_cast<const u32x4*>(in + e0);
        } else if (e0 < a.n) {
            // ragged last vector, or unaligned buffers: element by element
            uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int e = 0; e < EPV; ++e)
                if (e0 + e < a.n) {
                    if constexpr (sizeof(T) == 4) w[e] = __float_as_uint(in[e0 + e]);
                    else w[e / 2] |= (uint32_t)in[e0 + e] << (16 * (e & 1));
                }
            q.x = w[0]; q.y = w[1]; q.z = w[2]; q.w = w[3];
        }
        uint32_t m;
        if constexpr (MODE == 0) m = positive_bits<T>(q);
        else if constexpr (MODE == 1) m = keep_bits<T>(e0, a.seed_a, a.seed_c, a.thr);
        else {
            const uint64_t wi = vi / LPW;
            const uint32_t word = wi < a.nwords ? a.mask[wi] : 0u;
            m = (word >> (EPV * (uint32_t)(vi & (LPW - 1)))) & ((1u << EPV) - 1u);
        }
        // bits of elements past the end are zero
        if (!whole) m &= e0 < a.n ? (1u << (uint32_t)(a.n - e0)) - 1u : 0u;
        const u32x4 o = select_bits<T>(q, m);
        if (fast) {
            *reinterpret_cast<u32x4*>(out + e0) = o;
        } else if (e0 < a.n) {
            const uint32_t w[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
            for (int e = 0; e < EPV; ++e)
                if (e0 + e < a.n) {
                    if constexpr (sizeof(T) == 4) out[e0 + e] = __uint_as_float(w[e]);
                    else out[e0 + e] = (uint16_t)(w[e / 2] >> (16 * (e & 1)));
                }
        }
        if constexpr (MODE != 2) {
            const uint32_t word = merge_word<T>(m, lane);
            const uint64_t wi = vi / LPW;
            if ((lane & (LPW - 1)) == 0 && wi < a.nwords) a.mask[wi] = word;
        }
    }
}

int launch(int mode, const void* in, int64_t n, division_dtype dt, void* out, void* mask, size_t mask_bytes,
           float p, uint64_t seed, void* hip_stream) {
    if (n < 0 || (dt != DIVISION_F32 && dt != DIVISION_BF16)) return DIVISION_EINVAL;
    if (n == 0) return DIVISION_OK;                 // nothing to do; the pointers may be null
    if (!in || !out || !mask) return DIVISION_EINVAL;
    if (n > (int64_t)1 << 40) return DIVISION_ERANGE;
    if (mask_bytes < division_mask_bytes(n)) return DIVISION_ESIZE;
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    if (((uintptr_t)in % es) != 0 || ((uintptr_t)out % es) != 0 || ((uintptr_t)mask % 4) != 0) return DIVISION_EALIGN;
    MaskArgs a{};
    a.in = in; a.out = out; a.mask = static_cast<uint32_t*>(mask);
    a.n = (uint64_t)n; a.nwords = ((uint64_t)n + 31) / 32;
    a.vec = ((uintptr_t)in % 16) == 0 && ((uintptr_t)out % 16) == 0;
    if (mode == 1) {
        const uint64_t s = seed ^ kDropoutStream;
        a.seed_a = mix32((uint32_t)(s & 0xffffffffu) ^ 0x243F6A88u);
        a.seed_c = mix32((uint32_t)(s >> 32) ^ 0x85A308D3u);
        // T = floor(p * 65536 + 0.5) in binary64, clipped to [0, 65536]; NaN drops nothing
        const double t = (double)p * 65536.0 + 0.5;
        a.thr = !(t >= 1.0) ? 0u : t >= 65537.0 ? 65536u : (uint32_t)t;
    }
    const uint64_t epv = 16 / es;
    const uint64_t nvec = ((uint64_t)n + epv - 1) / epv;
    const uint64_t per_block = (uint64_t)kThreads * kVecPerThread;
    const uint32_t grid = (uint32_t)((nvec + per_block - 1) / per_block);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    void (*kern)(MaskArgs);
    if (dt == DIVISION_F32) kern = mode == 0 ? mask_kernel<float, 0> : mode == 1 ? mask_kernel<float, 1> : mask_kernel<float, 2>;
    else kern = mode == 0 ? mask_kernel<uint16_t, 0> : mode == 1 ? mask_kernel<uint16_t, 1> : mask_kernel<uint16_t, 2>;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), 0, st, a);
    return hipGetLastError() == hipSuccess ? DIVISION_OK : DIVISION_EHIP;
}

// ------------------------------------------------------------------ Max-Pooling layer, kernel = stride = k

struct PoolArgs {
    const void* in;        // x (forward) or grad_out (backward)
    void* out;             // y or grad_in
    uint32_t* mask;
    uint32_t P, H, W, HW, OH, OW, k;
    uint32_t band;         // output rows a workgroup handles
    uint32_t bands;        // bands per plane
};

__global__ void __launch_bounds__(kThreads) zero_words(uint32_t* p, uint64_t n) {
    for (uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kThreads) p[i] = 0u;
}

template <typename T> __device__ __forceinline__ float as_float(T v);
template <> __device__ __forceinline__ float as_float<float>(float v) { return v; }
template <> __device__ __forceinline__ float as_float<uint16_t>(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

// Forward: a workgroup takes a band of output rows of one plane.  Every thread scans whole
// windows (first maximum in row-major order wins), writes the maxima and sets the location bits
// in an LDS image of the band's slice of the mask; the slice then leaves as whole words, the two
// words it may share with neighbouring slices by atomic OR (the mask is cleared beforehand).
template <typename T, bool K2>
__global__ void __launch_bounds__(kThreads) maxpool_forward_kernel(PoolArgs a) {
    extern __shared__ uint32_t words[];
    const uint32_t tid = threadIdx.x;
    const uint32_t p = blockIdx.x / a.bands;
    const uint32_t oi0 = (blockIdx.x - p * a.bands) * a.band;
    const uint32_t oi1 = min(a.OH, oi0 + a.band);
    const uint64_t start = (uint64_t)p * a.HW + (uint64_t)oi0 * a.k * a.W;      // first bit of the slice
    const uint64_t end = (uint64_t)p * a.HW + (uint64_t)oi1 * a.k * a.W;        // one past its last bit
    const uint64_t w0 = start >> 5;
    const uint32_t nwords = (uint32_t)(((end - 1) >> 5) - w0) + 1u;
    for (uint32_t w = tid; w < nwords; w += kThreads) words[w] = 0u;
    __syncthreads();

    const T* xp = static_cast<const T*>(a.in) + (size_t)p * a.HW;
    T* yp = static_cast<T*>(a.out) + (size_t)p * a.OH * a.OW;
    const uint32_t nout = (oi1 - oi0) * a.OW;
    for (uint32_t o = tid; o < nout; o += kThreads) {
        const uint32_t r = o / a.OW;
        const uint32_t oj = o - r * a.OW;
        const uint32_t oi = oi0 + r;
        const uint32_t base = oi * a.k * a.W + oj * a.k;
        uint32_t best = base;
        T bt;
        if (K2) {
            // 2 x 2 window, rows of two adjacent elements each in one load (W even, x aligned to two elements)
            struct alignas(2 * sizeof(T)) Pair { T a, b; };
            const Pair r0 = *reinterpret_cast<const Pair*>(xp + base);
            const Pair r1 = *reinterpret_cast<const Pair*>(xp + base + a.W);
            bt = r0.a;
            float bv = as_float<T>(bt);
            if (as_float<T>(r0.b) > bv) { bv = as_float<T>(r0.b); bt = r0.b; best = base + 1; }
            if (as_float<T>(r1.a) > bv) { bv = as_float<T>(r1.a); bt = r1.a; best = base + a.W; }
            if (as_float<T>(r1.b) > bv) { bv = as_float<T>(r1.b); bt = r1.b; best = base + a.W + 1; }
        } else {
            bt = xp[base];
            float bv = as_float<T>(bt);
            for (uint32_t wr = 0; wr < a.k; ++wr)
                for (uint32_t wc = 0; wc < a.k; ++wc) {
                    const uint32_t idx = base + wr * a.W + wc;
                    const T t = xp[idx];
                    const float v = as_float<T>(t);
                    if (v > bv) { bv = v; bt = t; best = idx; }
                }
        }
        yp[oi * a.OW + oj] = bt;
        const uint32_t bit = (uint32_t)((uint64_t)p * a.HW + best - (w0 << 5));
        atomicOr(&words[bit >> 5], 1u << (bit & 31u));
    }
    __syncthreads();
    for (uint32_t w = tid; w < nwords; w += kThreads) {
        const uint32_t v = words[w];
        if (w == 0 || w == nwords - 1) { if (v) atomicOr(&a.mask[w0 + w], v); }
        else a.mask[w0 + w] = v;
    }
}

// Forward, k = 2 on rows of whole 8-element pieces (W % 8 == 0, H * W a multiple of 32, 16-byte aligned
// x): a thread takes four adjacent windows, i.e. eight consecutive elements of two rows (two 16-byte loads
// per row for 4-byte elements, one for 2-byte ones), writes their four maxima with one store and the eight
// location bits of each row as one byte of the LDS image of the band's mask slice: bytes have one owner, so
// there is no atomic, and a band of an even number of output rows is whole mask words, so the slice leaves
// with plain stores and the mask needs no clearing beforehand.  The last band of a plane also writes the
// (zero) bits of an odd last row.
template <typename T>
__global__ void __launch_bounds__(kThreads) maxpool2_forward_fast(PoolArgs a) {
    extern __shared__ uint32_t words[];
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    constexpr uint32_t EPV = 16 / sizeof(T);             // elements per 16-byte load
    const uint32_t tid = threadIdx.x;
    const uint32_t p = blockIdx.x / a.bands;
    const uint32_t bnd = blockIdx.x - p * a.bands;
    const uint32_t oi0 = bnd * a.band;
    const uint32_t oi1 = min(a.OH, oi0 + a.band);
    const uint32_t r0 = 2u * oi0;
    const uint32_t r1 = bnd + 1 == a.bands ? a.H : 2u * oi1;                 // input rows [r0, r1) belong to this band
    const uint64_t w0 = ((uint64_t)p * a.HW + (uint64_t)r0 * a.W) >> 5;      // first word of the slice (whole words)
    const uint32_t nwords = (r1 - r0) * a.W / 32u;
    for (uint32_t w = tid; w < nwords; w += kThreads) words[w] = 0u;
    __syncthreads();
    uint8_t* bytes = reinterpret_cast<uint8_t*>(words);
    const T* xp = static_cast<const T*>(a.in) + (size_t)p * a.HW;
    T* yp = static_cast<T*>(a.out) + (size_t)p * a.OH * a.OW;
    const uint32_t ow4 = a.OW / 4u;
    const uint32_t n4 = (oi1 - oi0) * ow4;
    for (uint32_t o4 = tid; o4 < n4; o4 += kThreads) {
        const uint32_t r = o4 / ow4;
        const uint32_t oj4 = o4 - r * ow4;
        const uint32_t oi = oi0 + r;
        const uint32_t base = 2u * oi * a.W + oj4 * 8u;                    // first of the eight elements, upper row
        uint32_t e0[8], e1[8];                                              // the two rows as fp32 bit patterns
        if constexpr (sizeof(T) == 4) {
            const u32x4 a0 = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xp + base));
            const u32x4 a1 = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xp + base + 4));
            const u32x4 b0 = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xp + base + a.W));
            const u32x4 b1 = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xp + base + a.W + 4));
            e0[0] = a0.x; e0[1] = a0.y; e0[2] = a0.z; e0[3] = a0.w; e0[4] = a1.x; e0[5] = a1.y; e0[6] = a1.z; e0[7] = a1.w;
            e1[0] = b0.x; e1[1] = b0.y; e1[2] = b0.z; e1[3] = b0.w; e1[4] = b1.x; e1[5] = b1.y; e1[6] = b1.z; e1[7] = b1.w;
        } else {
            const u32x4 a0 = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xp + base));
            const u32x4 b0 = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xp + base + a.W));
            const uint32_t wa[4] = {a0.x, a0.y, a0.z, a0.w}, wb[4] = {b0.x, b0.y, b0.z, b0.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                e0[2 * j] = wa[j] << 16; e0[2 * j + 1] = wa[j] & 0xffff0000u;
                e1[2 * j] = wb[j] << 16; e1[2 * j + 1] = wb[j] & 0xffff0000u;
            }
        }
        (void)EPV;
        uint32_t m[4], byte0 = 0, byte1 = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // first maximum in row-major order: a later element wins only if it compares greater
            uint32_t best = e0[2 * j], loc = 0;
            if (__uint_as_float(e0[2 * j + 1]) > __uint_as_float(best)) { best = e0[2 * j + 1]; loc = 1; }
            if (__uint_as_float(e1[2 * j]) > __uint_as_float(best)) { best = e1[2 * j]; loc = 2; }
            if (__uint_as_float(e1[2 * j + 1]) > __uint_as_float(best)) { best = e1[2 * j + 1]; loc = 3; }
            m[j] = best;
            byte0 |= (loc < 2 ? 1u << loc : 0u) << (2 * j);
            byte1 |= (loc >= 2 ? 1u << (loc - 2) : 0u) << (2 * j);
        }
        if constexpr (sizeof(T) == 4) {
            __builtin_nontemporal_store(u32x4{m[0], m[1], m[2], m[3]}, reinterpret_cast<u32x4*>(yp + oi * a.OW + oj4 * 4u));
        } else {
            __builtin_nontemporal_store(u32x2{(m[0] >> 16) | (m[1] & 0xffff0000u), (m[2] >> 16) | (m[3] & 0xffff0000u)},
                                        reinterpret_cast<u32x2*>(yp + oi * a.OW + oj4 * 4u));
        }
        const uint32_t b0i = (2u * r * a.W + oj4 * 8u) >> 3;               // byte of the slice that holds the upper row's eight bits
        bytes[b0i] = (uint8_t)byte0;
        bytes[b0i + (a.W >> 3)] = (uint8_t)byte1;
    }
    __syncthreads();
    for (uint32_t w = tid; w < nwords; w += kThreads) a.mask[w0 + w] = words[w];
}

// Backward: grad_in = V (.) (1_{k x k} (x) grad_out).  VEC = 4: a thread takes four consecutive
// elements of one row per step (W % 4 == 0, grad_in 16-byte resp. 8-byte aligned): one 16-byte
// store, one mask word read.  VEC = 1: element by element.
template <typename T, int VEC>
__global__ void __launch_bounds__(kThreads) maxpool_backward_kernel(PoolArgs a) {
    const uint32_t p = blockIdx.y;
    const T* gp = static_cast<const T*>(a.in) + (size_t)p * a.OH * a.OW;
    T* op = static_cast<T*>(a.out) + (size_t)p * a.HW;
    const uint64_t bit0 = (uint64_t)p * a.HW;
    const uint32_t nv = a.HW / VEC;
    for (uint32_t vi = blockIdx.x * kThreads + threadIdx.x; vi < nv; vi += gridDim.x * kThreads) {
        const uint32_t i = vi * VEC;
        const uint64_t bit = bit0 + i;
        // HW % 4 == 0 when VEC == 4, so the four bits never straddle a word
        const uint32_t bits = (a.mask[bit >> 5] >> (uint32_t)(bit & 31u)) & ((1u << VEC) - 1u);
        const uint32_t r = i / a.W;
        const uint32_t c = i - r * a.W;
        const uint32_t oi = r / a.k;
        const T* grow = gp + oi * a.OW;
        T v[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const uint32_t oj = (c + e) / a.k;
            v[e] = 0;
            if (((bits >> e) & 1u) && oi < a.OH && oj < a.OW) v[e] = grow[oj];
        }
        if constexpr (VEC == 4) {
            struct alignas(4 * sizeof(T)) Quad { T q[4]; };
            Quad o; o.q[0] = v[0]; o.q[1] = v[1]; o.q[2] = v[2]; o.q[3] = v[3];
            *reinterpret_cast<Quad*>(op + i) = o;
        } else {
            op[i] = v[0];
        }
    }
}

// Backward, k = 2 on rows of whole 4-element pieces (W % 4 == 0, 16-byte aligned grad_in, 8-byte aligned
// grad_out): a thread rebuilds four consecutive elements of one row, which lie under two adjacent windows:
// one mask word, one load of the two output gradients, one non-temporal 16-byte store; a workgroup of
// one... four wavefronts writes 4 KB and ends (what a write stream wants here).
template <typename T>
__global__ void __launch_bounds__(kThreads) maxpool2_backward_fast(PoolArgs a) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const uint32_t p = blockIdx.y;
    const T* gp = static_cast<const T*>(a.in) + (size_t)p * a.OH * a.OW;
    T* op = static_cast<T*>(a.out) + (size_t)p * a.HW;
    const uint32_t vi = blockIdx.x * kThreads + threadIdx.x;
    if (vi >= a.HW / 4u) return;
    const uint32_t w4 = a.W / 4u;
    const uint32_t r = vi / w4;
    const uint32_t c = (vi - r * w4) * 4u;
    const uint64_t bit = (uint64_t)p * a.HW + (uint64_t)vi * 4u;
    const uint32_t bits = (a.mask[bit >> 5] >> (uint32_t)(bit & 31u)) & 15u;
    // a row past the last whole window has no bits set: any row's gradients will do for the address
    const uint32_t oi = min(r >> 1, a.OH - 1u);
    const T* g = gp + oi * a.OW + (c >> 1);
    uint32_t g0, g1;                                   // the two gradients as raw element bits
    if constexpr (sizeof(T) == 4) {
        const u32x2 v = *reinterpret_cast<const u32x2*>(g);
        g0 = v.x; g1 = v.y;
    } else {
        const uint32_t v = *reinterpret_cast<const uint32_t*>(g);
        g0 = v & 0xffffu; g1 = v >> 16;
    }
    const uint32_t o0 = bits & 1u ? g0 : 0u, o1 = bits & 2u ? g0 : 0u, o2 = bits & 4u ? g1 : 0u, o3 = bits & 8u ? g1 : 0u;
    if constexpr (sizeof(T) == 4) __builtin_nontemporal_store(u32x4{o0, o1, o2, o3}, reinterpret_cast<u32x4*>(op + (size_t)vi * 4u));
    else __builtin_nontemporal_store(u32x2{o0 | (o1 << 16), o2 | (o3 << 16)}, reinterpret_cast<u32x2*>(op + (size_t)vi * 4u));
}

int pool_args(bool forward, const void* in, void* out, const void* mask, int64_t N, int64_t C, int64_t H, int64_t W,
              division_dtype dt, int k, size_t mask_bytes, PoolArgs* a) {
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || k < 1 || (dt != DIVISION_F32 && dt != DIVISION_BF16)) return DIVISION_EINVAL;
    // the pooled-size buffer (y / grad_out) may be null when there is no whole window
    const bool no_window = H / k == 0 || W / k == 0;
    if (!mask || (!in && !(no_window && !forward)) || (!out && !(no_window && forward))) return DIVISION_EINVAL;
    const uint64_t P = (uint64_t)N * (uint64_t)C, HW = (uint64_t)H * (uint64_t)W;
    if (N > 0x7fffffff || C > 0x7fffffff || H > 0x7fffffff || W > 0x7fffffff || P > 0x7fffffffull || HW > 0x7fffffffull ||
        P * HW > (1ull << 40) || k > 0x7fff)
        return DIVISION_ERANGE;
    if (mask_bytes < division_mask_bytes((int64_t)(P * HW))) return DIVISION_ESIZE;
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    if (((uintptr_t)in % es) != 0 || ((uintptr_t)out % es) != 0 || ((uintptr_t)mask % 4) != 0) return DIVISION_EALIGN;
    a->in = in; a->out = out; a->mask = static_cast<uint32_t*>(const_cast<void*>(mask));
    a->P = (uint32_t)P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)HW;
    a->OH = (uint32_t)(H / k); a->OW = (uint32_t)(W / k); a->k = (uint32_t)k;
    return DIVISION_OK;
}

}  // namespace

extern "C" {

size_t division_mask_bytes(int64_t n) { return n < 0 ? 0 : (size_t)((n + 31) / 32) * 4u; }

int division_relu_forward(const void* x, int64_t n, division_dtype dt, void* y, void* mask, size_t mask_capacity,
                          void* hip_stream) {
    return launch(0, x, n, dt, y, mask, mask_capacity, 0.0f, 0, hip_stream);
}

int division_dropout_forward(const void* x, int64_t n, division_dtype dt, float p, uint64_t seed, void* y, void* mask,
                             size_t mask_capacity, void* hip_stream) {
    return launch(1, x, n, dt, y, mask, mask_capacity, p, seed, hip_stream);
}

int division_mask_backward(const void* mask, size_t mask_bytes, const void* grad_out, int64_t n, division_dtype dt,
                           void* grad_in, void* hip_stream) {
    return launch(2, grad_out, n, dt, grad_in, const_cast<void*>(mask), mask_bytes, 0.0f, 0, hip_stream);
}

int division_maxpool_forward(const void* x, int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt, int k,
                             void* y, void* mask, size_t mask_capacity, void* hip_stream) {
    PoolArgs a{};
    const int rc = pool_args(true, x, y, mask, N, C, H, W, dt, k, mask_capacity, &a);
    if (rc != DIVISION_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const size_t esz = dt == DIVISION_BF16 ? 2 : 4;
    if (k == 2 && a.OH > 0 && a.W % 8 == 0 && a.HW % 32 == 0 && ((uintptr_t)x % 16) == 0 && ((uintptr_t)y % (4 * esz)) == 0) {
        // bands of an even number of output rows (whole mask words), at most 64 Ki bits, enough of them to fill the machine
#ifndef DIVISION_POOL_WG_BYTES
#define DIVISION_POOL_WG_BYTES 8192
#endif
        // about 8 KB of x per workgroup (short-lived workgroups, many of them), at most 64 Ki mask bits
        uint32_t band = (uint32_t)(DIVISION_POOL_WG_BYTES / (2ull * a.W * esz)) & ~1u;
        if (band < 2) band = 2;
        if (2ull * band * a.W > 65536) band = (uint32_t)(65536 / (2ull * a.W)) & ~1u;
        if (band < 2) band = 0;
        if (band >= 2) {
            a.band = band;
            a.bands = (a.OH + band - 1) / band;
            const uint64_t grid = (uint64_t)a.P * a.bands;
            // the last band of a plane also holds an odd last row
            const size_t lds = ((size_t)(band + 1) * 2 * a.W) / 8 + 16;
            if (grid <= 0x7fffffffull) {
                void (*kern)(PoolArgs) = dt == DIVISION_F32 ? maxpool2_forward_fast<float> : maxpool2_forward_fast<uint16_t>;
                hipLaunchKernelGGL(kern, dim3((uint32_t)grid), dim3(kThreads), lds, st, a);
                return hipGetLastError() == hipSuccess ? DIVISION_OK : DIVISION_EHIP;
            }
        }
    }
    const uint64_t nwords = ((uint64_t)a.P * a.HW + 31) / 32;
    const uint32_t zgrid = (uint32_t)((nwords + kThreads * 8ull - 1) / (kThreads * 8ull));
    hipLaunchKernelGGL(zero_words, dim3(zgrid < 1 ? 1 : zgrid), dim3(kThreads), 0, st, a.mask, nwords);
    if (hipGetLastError() != hipSuccess) return DIVISION_EHIP;
    if (a.OH == 0 || a.OW == 0) return DIVISION_OK;          // no whole window: empty output, all-zero mask
    // a band's slice of the mask lives in LDS: at most 64 Ki bits (+ the two edge words)
    const uint64_t row_bits = (uint64_t)a.k * a.W;
    if (row_bits > 65536) return DIVISION_ERANGE;
    uint32_t band = (uint32_t)(65536 / row_bits);
    if (band > a.OH) band = a.OH;
    // small planes: fewer rows per band than fit, so that the launch still has enough workgroups
    while (band > 1 && (uint64_t)a.P * ((a.OH + band - 1) / band) < 2048) band = (band + 1) / 2;
    a.band = band;
    a.bands = (a.OH + band - 1) / band;
    const uint64_t grid = (uint64_t)a.P * a.bands;
    if (grid > 0x7fffffffull) return DIVISION_ERANGE;
    const size_t lds = 4 * ((size_t)band * row_bits / 32 + 2);
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    const bool k2 = k == 2 && a.W % 2 == 0 && ((uintptr_t)x % (2 * es)) == 0;       // a.HW is even then
    void (*kern)(PoolArgs);
    if (dt == DIVISION_F32) kern = k2 ? maxpool_forward_kernel<float, true> : maxpool_forward_kernel<float, false>;
    else kern = k2 ? maxpool_forward_kernel<uint16_t, true> : maxpool_forward_kernel<uint16_t, false>;
    hipLaunchKernelGGL(kern, dim3((uint32_t)grid), dim3(kThreads), lds, st, a);
    return hipGetLastError() == hipSuccess ? DIVISION_OK : DIVISION_EHIP;
}

int division_maxpool_backward(const void* mask, size_t mask_bytes, const void* grad_out, int64_t N, int64_t C,
                              int64_t H, int64_t W, division_dtype dt, int k, void* grad_in, void* hip_stream) {
    PoolArgs a{};
    const int rc = pool_args(false, grad_out, grad_in, mask, N, C, H, W, dt, k, mask_bytes, &a);
    if (rc != DIVISION_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const size_t esz = dt == DIVISION_BF16 ? 2 : 4;
    if (k == 2 && a.OH > 0 && a.OW > 0 && a.W % 4 == 0 && ((uintptr_t)grad_in % (4 * esz)) == 0 && ((uintptr_t)grad_out % (2 * esz)) == 0 &&
        a.P <= 65535u) {
        void (*fast)(PoolArgs) = dt == DIVISION_F32 ? maxpool2_backward_fast<float> : maxpool2_backward_fast<uint16_t>;
        hipLaunchKernelGGL(fast, dim3((a.HW / 4 + kThreads - 1) / kThreads, a.P), dim3(kThreads), 0, st, a);
        return hipGetLastError() == hipSuccess ? DIVISION_OK : DIVISION_EHIP;
    }
    const bool vec4 = a.W % 4 == 0 && ((uintptr_t)grad_in % (4 * esz)) == 0;
    void (*kern)(PoolArgs);
    if (dt == DIVISION_F32) kern = vec4 ? maxpool_backward_kernel<float, 4> : maxpool_backward_kernel<float, 1>;
    else kern = vec4 ? maxpool_backward_kernel<uint16_t, 4> : maxpool_backward_kernel<uint16_t, 1>;
    const uint32_t per = vec4 ? 4u : 1u;
    uint32_t gx = (a.HW / per + kThreads * 2u - 1) / (kThreads * 2u);
    if (gx < 1) gx = 1;
    if (gx > 4096) gx = 4096;
    // grid.y takes a slice of planes per launch; a multiple of 32 planes, so that every slice's
    // first mask bit starts a word
    constexpr uint32_t kSlice = 65504;
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    for (uint32_t p0 = 0; p0 < a.P; p0 += kSlice) {
        PoolArgs b = a;
        const uint32_t np = a.P - p0 < kSlice ? a.P - p0 : kSlice;
        b.in = static_cast<const char*>(a.in) + (size_t)p0 * a.OH * a.OW * es;
        b.out = static_cast<char*>(a.out) + (size_t)p0 * a.HW * es;
        b.mask = a.mask + ((uint64_t)p0 * a.HW) / 32;
        hipLaunchKernelGGL(kern, dim3(gx, np), dim3(kThreads), 0, st, b);
        if (hipGetLastError() != hipSuccess) return DIVISION_EHIP;
    }
    return DIVISION_OK;
}

}  // extern "C"
