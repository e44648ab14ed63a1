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
// Work decomposition (one GPU; (sample, channel) planes are independent; except in compress_plane
// and compress_any every element of x is read from HBM exactly once, and no intermediate tensor
// touches HBM).  The host picks the first kernel of this list that covers the shape:
//   compress_line    1-D maps (one row) whose block is a power-of-two number of 16-byte vectors: planes
//                    in registers, block sums by DPP (before compress_regs for 2-byte elements and
//                    planes below 2048 elements, after it otherwise)
//   compress_regs    planes of 2K-3K / 8K-13K / up to 53K elements (56x56, 112x112, 224x224; 3-D maps of
//                    those sizes), B = 4, 8 (template) or 12, 16 (from the arguments): one plane per
//                    workgroup of one / four / sixteen wavefronts, the plane stays in registers from
//                    load to codes
//   compress_lane    one-block planes with an odd element count (7x7): a lane per plane
//   compress_items   planes of at most 64 pooling items (28x28, 14x14, CIFAR shapes), B = 4, 8: a lane
//                    per pooling item, loaded straight from global memory, DPP reductions
//   compress_units   2-D planes of 256 to about 27K elements whose rows or blocks are not whole 16-byte vectors
//                    (odd widths: 27x27, 55x55, 147x147; B = 18): four consecutive elements per lane step
//                    whatever the width, the block of each element looked up in a table made once per
//                    workgroup, the plane parked in LDS for the block sums, next plane's loads in flight
//   compress_wave    other planes up to 17 KB, B = 4, 8: one wavefront per chunk of planes staged in LDS
//   compress_tile    other planes up to 156 KB, B = 4, 8: four wavefronts per chunk staged in LDS
//   compress_one     planes that are a single block (B = 64 on 56x56 and below): flat vectors in registers
//   compress_rows    any block size, 3-D maps: chunk staged in LDS, vectors kept in registers for Quant
//   compress_plane   planes beyond LDS with vector rows and blocks (video volumes, image-sized maps):
//                    a workgroup per plane, two vector passes over x
//   compress_any     everything else (giant planes with odd extents): scalar, slow
//   decompress_rowvec / _table / _words / _flat / _lane / _scalar: streaming, the packed slice of a
//                    workgroup staged in LDS, one 16-byte non-temporal store per lane step (_words:
//                    small planes of odd width, the chunk rebuilt in LDS word by word first)
//   decompress_units the counterpart of compress_units (odd widths from 512 elements per plane up): four
//                    consecutive elements per lane step, block table made once per workgroup, the next
//                    plane's codes and LFC in flight
// The kernels with a _3d twin take N x C x D x H x W maps with B x B x B blocks (Appendix D).
// Every kernel takes a table of up to 8 maps of one shape (blockIdx.y picks the map).
// Element / cache types: float, bf16_t, f32c16_t (fp32 map, tuple cached as bfloat16).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <stdio.h>
#include <stdlib.h>
#include <type_traits>
#include <vector>
#include "../../include/division.h"

// The kernels are instantiated per element / cache type (float, bf16_t, f32c16_t).  To build the
// library in parallel this file can be compiled three times with -DDIVISION_PART=0, 1, 2: each part
// instantiates the kernels of one type behind three bridge functions, part 0 also holds the C ABI.
// Without the macro one translation unit holds everything.
#if !defined(DIVISION_PART)
#define DIVISION_HOST 1
#define DIVISION_HAS_F32 1
#define DIVISION_HAS_BF16 1
#define DIVISION_HAS_C16 1
#else
#define DIVISION_HOST (DIVISION_PART == 0)
#define DIVISION_HAS_F32 (DIVISION_PART == 0)
#define DIVISION_HAS_BF16 (DIVISION_PART == 1)
#define DIVISION_HAS_C16 (DIVISION_PART == 2)
#endif
// launch descriptors travel through the bridges as untyped pointers (their types live in the
// unnamed namespace of each part; the parts are built from this one source, so the layouts agree)
#define DIVISION_BRIDGE __attribute__((visibility("hidden")))
DIVISION_BRIDGE hipError_t division_bridge_compress_f32(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_compress_bf16(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_compress_c16(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_decompress_f32(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_decompress_bf16(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_decompress_c16(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_relu_f32(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_relu_bf16(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_relu_c16(const void* launch, int b);

namespace {

constexpr int kThreads = 256;              // 4 wavefronts of 64
constexpr uint32_t kLdsTarget = 40u << 10; // preferred LDS bytes per workgroup (4 groups per CU)
constexpr uint32_t kRowsLdsTarget = 40u << 10; // same for compress_rows
constexpr uint32_t kLdsMax = 156u << 10;   // hard limit per workgroup (160 KB per CU)
constexpr uint32_t kWeyl = 0x9E3779B9u;
// cache policy of the loads of x: default.  x is read exactly once, but marking
// the loads non-temporal (2) measured 4 % slower on the whole step.
constexpr int kLoadAux = 0;

// ------------------------------------------------------------------ helpers

struct bf16_t { uint16_t v; };
// an fp32 map whose H^L, delta and Delta are cached as bfloat16 (the paper's format): same
// element as float, different cache layout; a type of its own so that the choice costs nothing
// at run time
struct f32c16_t { float v; };
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
template <> struct Elem<f32c16_t> {
    static __device__ __forceinline__ float load(const f32c16_t* p, size_t i) { return p[i].v; }
    static __device__ __forceinline__ void store(f32c16_t* p, size_t i, float v) { p[i].v = v; }
    static __device__ __forceinline__ float round(float v) { return v; }
};
template <typename T> constexpr uint32_t kC16 = 0;
template <> constexpr uint32_t kC16<f32c16_t> = 1;
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

// ---- the paper's cached format (c16): fp32 maps whose H^L, delta and Delta are cached as bfloat16

// largest bfloat16 <= f and smallest bfloat16 >= f (finite f)
__device__ __forceinline__ float bf16_floor_f(float f) {
    const uint32_t u = __float_as_uint(f);
    uint32_t t = u & 0xffff0000u;                                    // toward zero
    if ((u & 0x80000000u) && (u & 0xffffu)) t += 0x10000u;           // negative: one step away from zero
    return __uint_as_float(t);
}
__device__ __forceinline__ float bf16_ceil_f(float f) {
    const uint32_t u = __float_as_uint(f);
    uint32_t t = u & 0xffff0000u;
    if (!(u & 0x80000000u) && (u & 0xffffu)) t += 0x10000u;
    return __uint_as_float(t);
}

// Scale of one plane from its residual extremes.  Plain: delta = min, Delta, inv as plane_scale.
// c16: the quantiser has to use the very values the decoder will read and every residual has to
// stay inside their code range, so delta = min rounded DOWN to bfloat16, Delta =
// fl(fl(max - delta) / L) rounded UP to bfloat16, inv = fl(1 / Delta).
__device__ __forceinline__ void plane_scale_any(float mn, float mx, float Lf, uint32_t c16,
                                                float& delta, float& Delta, float& inv) {
    if (!c16) {
        delta = mn;
        plane_scale(mn, mx, Lf, Delta, inv);
        return;
    }
    delta = bf16_floor_f(mn);
    const float range = mx - delta;
    if (range >= 0x1p-90f && range <= 3.4028234663852886e38f) {
        Delta = bf16_ceil_f(range / Lf);
        inv = 1.0f / Delta;
    } else {
        Delta = 0.0f;
        inv = 0.0f;
    }
}

// (delta, Delta) of plane p: two floats, or two bfloat16 in one word (c16)
__device__ __forceinline__ void meta_store(float* meta, uint32_t p, float delta, float Delta, uint32_t c16) {
    if (c16) reinterpret_cast<uint32_t*>(meta)[p] = (__float_as_uint(delta) >> 16) | (__float_as_uint(Delta) & 0xffff0000u);
    else reinterpret_cast<float2*>(meta)[p] = make_float2(delta, Delta);
}
__device__ __forceinline__ float2 meta_load(const float* meta, uint32_t p, uint32_t c16) {
    if (c16) {
        const uint32_t w = reinterpret_cast<const uint32_t*>(meta)[p];
        return make_float2(__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u));
    }
    return reinterpret_cast<const float2*>(meta)[p];
}

// H^L: stored in the element type of x, or as bfloat16 (c16; x is fp32 then)
template <typename T>
__device__ __forceinline__ float lfc_round(float v, uint32_t c16) {
    return (sizeof(T) == 2 || c16) ? bf16_bits_to_float(float_to_bf16_bits(v)) : v;
}
template <typename T>
__device__ __forceinline__ void lfc_store(void* base, size_t idx, float v, uint32_t c16) {
    if (sizeof(T) == 2 || c16) static_cast<uint16_t*>(base)[idx] = (uint16_t)float_to_bf16_bits(v);
    else static_cast<float*>(base)[idx] = v;
}
template <typename T>
__device__ __forceinline__ float lfc_load(const void* base, size_t idx, uint32_t c16) {
    if (sizeof(T) == 2 || c16) return bf16_bits_to_float(static_cast<const uint16_t*>(base)[idx]);
    return static_cast<const float*>(base)[idx];
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

// One launch serves up to kMaxBatch tensors of one shape (blockIdx.y picks the
// tensor): fewer, longer kernels, so less of a step is spent filling and
// draining the machine.
constexpr int kMaxBatch = 8;
struct CompTab { const void* x[kMaxBatch]; void* pk[kMaxBatch]; uint32_t seed_a[kMaxBatch], seed_c[kMaxBatch]; };
struct DecTab { const void* pk[kMaxBatch]; void* xhat[kMaxBatch]; };

// Offsets of the regions inside a packed buffer, and the byte ranges between /
// after them that must read as zero (each shorter than 16 bytes).
struct Regions { size_t meta_off, lfc_off; size_t pad_off[3]; uint32_t pad_len[3]; };

// this workgroup's tensor
struct CompPtrs { const void* x; uint32_t* codes; float* meta; void* lfc; uint32_t seed_a, seed_c; };
__device__ __forceinline__ CompPtrs comp_ptrs(const CompTab& tab, const Regions& rg, uint32_t tid) {
    const uint32_t ti = blockIdx.y;
    char* pk = static_cast<char*>(tab.pk[ti]);
    if (blockIdx.x == 0 && tid < 48) {
        const uint32_t k = tid >> 4, j = tid & 15u;
        if (j < rg.pad_len[k]) pk[rg.pad_off[k] + j] = 0;
    }
    CompPtrs pt;
    pt.x = tab.x[ti];
    pt.codes = reinterpret_cast<uint32_t*>(pk);
    pt.meta = reinterpret_cast<float*>(pk + rg.meta_off);
    pt.lfc = pk + rg.lfc_off;
    pt.seed_a = tab.seed_a[ti];
    pt.seed_c = tab.seed_c[ti];
    return pt;
}
struct DecPtrs { const uint32_t* codes; const float* meta; const void* lfc; void* xhat; };
__device__ __forceinline__ DecPtrs dec_ptrs(const DecTab& tab, const Regions& rg) {
    const uint32_t ti = blockIdx.y;
    const char* pk = static_cast<const char*>(tab.pk[ti]);
    DecPtrs pt;
    pt.codes = reinterpret_cast<const uint32_t*>(pk);
    pt.meta = reinterpret_cast<const float*>(pk + rg.meta_off);
    pt.lfc = pk + rg.lfc_off;
    pt.xhat = tab.xhat[ti];
    return pt;
}

struct TileArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, H, W, HW, LH, LW, nb, WPP;
    uint32_t G;          // planes per workgroup
    uint32_t ipr;        // item slots per block row (padded to the items-per-block count)
    uint32_t ipp;        // item slots per plane = LH * ipr
    uint32_t S;          // lanes cooperating on one plane's min/max (power of two <= 64)
    uint32_t xs_floats;  // LDS floats reserved for the chunk (multiple of 4)
    uint32_t items_cap;  // LDS floats reserved per item array
    uint32_t vec_load;   // chunk starts are 16-byte aligned
    FastDiv d_ipp, d_ipr, d_wpp;
};

// ------------------------------------------------------------------ synchronisation

// Orders LDS traffic between the lanes of ONE wavefront.  The LDS unit serves
// a wavefront's instructions in issue order, so no wait is needed; the fence
// only stops the compiler from moving LDS accesses across this point.  Unlike
// __syncthreads() it does not wait for outstanding global loads and stores.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Workgroup barrier that publishes LDS writes only: waits for this wave's LDS
// operations (lgkmcnt), not for its global loads and stores (vmcnt), then
// joins the barrier.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_s_waitcnt(0xc07f);      // lgkmcnt(0), vmcnt and expcnt untouched
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ------------------------------------------------------------------ cross-lane helpers (DPP)

// value of another lane of the same 16-lane row; all lanes must be active
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    const uint64_t u = __double_as_longlong(v);
    const uint32_t lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)u, CTRL, 0xf, 0xf, false);
    const uint32_t hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(u >> 32), CTRL, 0xf, 0xf, false);
    return __longlong_as_double(((uint64_t)hi << 32) | lo);
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each 8 lanes
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside each 16 lanes

// sum over aligned groups of N lanes (N = 1, 2, 4, 8), result in every lane of the group
template <int N>
__device__ __forceinline__ double group_sum(double v) {
    if constexpr (N >= 2) v += dpp_f64<kDppXor1>(v);
    if constexpr (N >= 4) v += dpp_f64<kDppXor2>(v);
    if constexpr (N >= 8) v += dpp_f64<kDppHalfMirror>(v);
    return v;
}

// min / max over aligned groups of S lanes (S a power of two <= 64, uniform
// in the wave), result in every lane of the group
__device__ __forceinline__ void group_minmax(uint32_t S, float& mn, float& mx) {
    if (S >= 2)  { mn = fminf(mn, dpp_f32<kDppXor1>(mn)); mx = fmaxf(mx, dpp_f32<kDppXor1>(mx)); }
    if (S >= 4)  { mn = fminf(mn, dpp_f32<kDppXor2>(mn)); mx = fmaxf(mx, dpp_f32<kDppXor2>(mx)); }
    if (S >= 8)  { mn = fminf(mn, dpp_f32<kDppHalfMirror>(mn)); mx = fmaxf(mx, dpp_f32<kDppHalfMirror>(mx)); }
    if (S >= 16) { mn = fminf(mn, dpp_f32<kDppMirror>(mn)); mx = fmaxf(mx, dpp_f32<kDppMirror>(mx)); }
    if (S >= 32) {
        const int imn = __float_as_int(mn), imx = __float_as_int(mx);
        const float n0 = __int_as_float(__builtin_amdgcn_readlane(imn, 0)), n1 = __int_as_float(__builtin_amdgcn_readlane(imn, 16));
        const float n2 = __int_as_float(__builtin_amdgcn_readlane(imn, 32)), n3 = __int_as_float(__builtin_amdgcn_readlane(imn, 48));
        const float x0 = __int_as_float(__builtin_amdgcn_readlane(imx, 0)), x1 = __int_as_float(__builtin_amdgcn_readlane(imx, 16));
        const float x2 = __int_as_float(__builtin_amdgcn_readlane(imx, 32)), x3 = __int_as_float(__builtin_amdgcn_readlane(imx, 48));
        if (S == 64) {
            mn = fminf(fminf(n0, n1), fminf(n2, n3));
            mx = fmaxf(fmaxf(x0, x1), fmaxf(x2, x3));
        } else {
            const bool upper = (threadIdx.x & 32u) != 0;
            mn = upper ? fminf(n2, n3) : fminf(n0, n1);
            mx = upper ? fmaxf(x2, x3) : fmaxf(x0, x1);
        }
    }
}

// ------------------------------------------------------------------ compress, LDS tile

// One pair of elements -> two codes pushed into the packed word (element
// 2j+1 first, then 2j: words are built from the last element down, so that
// element 0 ends in the low bits).  Exact integer evaluation of
// floor(t + r/2^16): T = trunc(t * 2^(32-BITS)), sum = T + (r << (16-BITS)),
// code = top BITS bits of sum.  For BITS <= 4, t <= L(1 + 3 ulp) and r < 2^16 keep the
// sum below 2^32, so no clamp is needed.
template <int BITS>
__device__ __forceinline__ uint32_t push_pair(uint32_t acc, float h0, float h1, float delta, float invs,
                                              uint32_t xw, uint32_t k2, uint32_t rscale) {
    uint32_t x = xw;
    x ^= x >> 16; x *= 0x7feb352du;
    x = x ^ (x >> 15) ^ k2; x *= 0x846ca68bu;
    // final x ^= x >> 16: the high half is unchanged, the low half becomes lo ^ hi
    const uint32_t xl = x ^ (x >> 16);
    uint32_t T1 = (uint32_t)((h1 - delta) * invs);
    uint32_t T0 = (uint32_t)((h0 - delta) * invs);
    if constexpr (BITS == 8) {
        // t may exceed L by a few ulp; with 8-bit codes an ulp of 255 is as large as the random
        // term's step (2^-16), so the sum could wrap: clamp t to L first (the code is L either way)
        T1 = min(T1, 255u << 24);
        T0 = min(T0, 255u << 24);
    }
    uint32_t s1, s0;
    asm("v_mad_u32_u16 %0, %1, %2, %3 op_sel:[1,0,0,0]" : "=v"(s1) : "v"(x), "s"(rscale), "v"(T1));
    asm("v_mad_u32_u16 %0, %1, %2, %3 op_sel:[0,0,0,0]" : "=v"(s0) : "v"(xl), "s"(rscale), "v"(T0));
    acc = __builtin_amdgcn_alignbit(acc, s1, 32 - BITS);
    acc = __builtin_amdgcn_alignbit(acc, s0, 32 - BITS);
    return acc;
}

// T: element type; BITS: code width; B: block size (4 or 8); VEC: elements per
// LDS vector access in the pooling phase (W % VEC == 0, B % VEC == 0);
// NT: threads per workgroup (64 or 256).
template <typename T, int BITS, int B, int VEC, int NT>
__global__ void __launch_bounds__(NT) compress_tile(TileArgs a) {
    extern __shared__ float4 smem4[];
    float4* params = smem4;                                   // [G] (delta, inv scaled, k1, k2)
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
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, tid);

    // ---- phase 0: chunk -> LDS (fp32); coalesced 16-byte loads, up to 8 in flight per lane
    {
        const T* src = static_cast<const T*>(pt.x) + (size_t)p0 * a.HW;
        constexpr uint32_t EPV = 16 / sizeof(T);
        constexpr int U = 8;
        const uint32_t nv = a.vec_load ? n / EPV : 0;
        const u32x4* src4 = reinterpret_cast<const u32x4*>(src);
        for (uint32_t v0 = 0; v0 < nv; v0 += U * NT) {
            u32x4 q[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t v = v0 + u * NT + tid;
                if (v < nv) q[u] = __builtin_nontemporal_load(src4 + v);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t v = v0 + u * NT + tid;
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
        for (uint32_t e = nv * EPV + tid; e < n; e += NT) xs[e] = Elem<T>::load(src, e);
    }
    lds_barrier();

    // ---- phase 1: block means (Sec. 4.1 AveragePooling), residual in place
    // item = (plane g, block row bi, slot s): B rows x VEC columns of one block;
    // the IPB items of a block sit in adjacent lanes
    const uint32_t nitems = Gc * a.ipp;
    for (uint32_t it0 = 0; it0 < nitems; it0 += NT) {
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
        S = group_sum<IPB>(S);

        const uint32_t bj = s / IPB;
        const uint32_t rows = min((uint32_t)B, a.H - min(a.H, r0));
        const uint32_t cols = min((uint32_t)B, a.W - min(a.W, bj * B));
        const uint32_t cnt = max(rows * cols, 1u);
        // exact sum / count, one rounding to fp32, then to the storage type
        float m;
        if ((cnt & (cnt - 1)) == 0) m = (float)(S * (1.0 / (double)cnt));   // power of two: exact scaling
        else m = (float)(S / (double)cnt);
        const float lfc = lfc_round<T>(m, kC16<T>);
        if (valid && (s % IPB) == 0)
            lfc_store<T>(pt.lfc, (size_t)(p0 + g) * a.nb + bi * a.LW + bj, lfc, kC16<T>);

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
    lds_barrier();

    // ---- phase 2: per-plane min / max, scale of Eq. (quantization), keys
    {
        const uint32_t S = a.S;
        const uint32_t groups = NT / S;
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
            group_minmax(S, mn, mx);
            if (live && sub == 0) {
                float delta, Delta, inv;
                plane_scale_any(mn, mx, Lf, kC16<T>, delta, Delta, inv);
                const uint32_t p = p0 + g;
                meta_store(pt.meta, p, delta, Delta, kC16<T>);
                const uint32_t k1 = mix32(p ^ pt.seed_a);
                const uint32_t k2 = mix32(k1 + pt.seed_c);
                params[g] = make_float4(delta, inv * (float)(1u << (32 - BITS)), __uint_as_float(k1), __uint_as_float(k2));
            }
        }
    }
    lds_barrier();

    // ---- phase 3: Quant of Eq. (quantization) + packing, one word per lane
    {
        const uint32_t nwords = Gc * a.WPP;
        const bool hw4 = (a.HW & 3u) == 0;
        const uint32_t rscale = 1u << (16 - BITS);
        for (uint32_t wi = tid; wi < nwords; wi += NT) {
            const uint32_t g = fdiv(wi, a.d_wpp);
            const uint32_t k = wi - g * a.WPP;
            const float4 pr = params[g];
            const float delta = pr.x, invs = pr.y;
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
            const uint32_t xw0 = k1 + (k * (CPW / 2)) * kWeyl;
            uint32_t word = 0;
#pragma unroll
            for (int j = CPW / 2 - 1; j >= 0; --j)
                word = push_pair<BITS>(word, h[2 * j], h[2 * j + 1], delta, invs, xw0 + (uint32_t)j * kWeyl, k2, rscale);
            pt.codes[(size_t)(p0 + g) * a.WPP + k] = word;
        }
    }
}

// ------------------------------------------------------------------ compress, one wavefront per chunk

struct WaveArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, H, W, HW, LH, LW, nb, WPP;
    uint32_t G;          // planes per wavefront (one workgroup = one wavefront)
    uint32_t ipr;        // item slots per block row (padded to the items-per-block count)
    uint32_t ipp;        // item slots per plane = LH * ipr
    uint32_t ippp;       // ipp padded: next power of two if <= 64, else next multiple of 64
    uint32_t ippp_log2;  // log2(ippp) when ippp <= 64
    uint32_t vec_load;   // chunk starts are 16-byte aligned
    FastDiv d_ipr, d_wpp;
};

// (float)(S / cnt) for a small positive integer cnt, the way the reference
// definition rounds it (binary64 quotient, then one rounding to binary32),
// without a binary64 division in the common case: q = S * (1/cnt) is within
// 2 ulp of the binary64 quotient, so both round to the same binary32 value
// unless q lies within a few ulp of a binary32 rounding midpoint (the 29
// mantissa bits a binary32 drops close to 1000...0); only then, for the whole
// wavefront, the true division runs.
__device__ __forceinline__ float mean_of(double S, uint32_t cnt) {
    if ((cnt & (cnt - 1)) == 0) return (float)(S * (1.0 / (double)cnt));     // power of two: exact scaling
    const double q = S * (1.0 / (double)cnt);
    const uint32_t low = (uint32_t)__double_as_longlong(q) & 0x1fffffffu;
    const uint32_t dist = low > 0x10000000u ? low - 0x10000000u : 0x10000000u - low;
    if (__builtin_expect(__any(dist < 16u), 0)) return (float)(S / (double)cnt);
    return (float)q;
}

// Sec. 4.1 for one pooling item: B rows x VEC columns of one block, read from
// LDS; the IPB items of a block sit in adjacent lanes.  Writes the block's LFC,
// overwrites x by the residual, folds the item's residual min / max into
// (hmin, hmax).  Lanes without an item work on item 0 of the chunk and have
// their effects masked.  Rows past the map (ragged last block row, FULLROWS
// false) re-read row 0 of the item: a duplicate changes neither min nor max,
// its residual is written back to the very value row 0 gets, and its row sum
// is left out of the block sum.
// What a lane needs to know about its pooling item apart from the plane: the
// same in every round, so it is worked out once per wavefront.
struct ItemGeom {
    uint32_t off;      // element offset of the item's first row inside its plane
    uint32_t lfc_idx;  // index of the item's block in the plane's LFC
    uint32_t nrows;    // rows of the block that exist (1..B)
    uint32_t cnt;      // elements of the block (rows * columns)
    bool in_plane;     // the slot holds an item (not padding)
    bool writes_lfc;   // first item of its block
};

template <int B, int VEC>
__device__ __forceinline__ ItemGeom item_geom(const WaveArgs& a, uint32_t rem) {
    constexpr int IPB = B / VEC;
    ItemGeom gm;
    const uint32_t bi = fdiv(rem, a.d_ipr);
    const uint32_t s = rem - bi * a.ipr;
    const uint32_t col0 = s * VEC;
    const uint32_t r0 = bi * B;
    const uint32_t bj = s / IPB;
    gm.in_plane = rem < a.ipp && col0 < a.W;
    gm.off = gm.in_plane ? r0 * a.W + col0 : 0u;
    gm.nrows = gm.in_plane ? min((uint32_t)B, a.H - r0) : 1u;
    const uint32_t rows = min((uint32_t)B, a.H - min(a.H, r0));
    const uint32_t cols = min((uint32_t)B, a.W - min(a.W, bj * B));
    gm.cnt = max(rows * cols, 1u);
    gm.lfc_idx = bi * a.LW + bj;
    gm.writes_lfc = gm.in_plane && (s % IPB) == 0;
    return gm;
}

template <typename T, int B, int VEC, bool FULLROWS>
__device__ __forceinline__ void pool_item(float* xs, const WaveArgs& a, void* lfc_base, size_t lfc_plane, uint32_t g, const ItemGeom& gm,
                                          bool live, float& hmin, float& hmax) {
    constexpr int IPB = B / VEC;
    const bool valid = live && gm.in_plane;
    const uint32_t base = valid ? g * a.HW + gm.off : 0u;
    const uint32_t nrows = FULLROWS ? (uint32_t)B : (valid ? gm.nrows : 1u);

    float v[B][VEC];
    uint32_t off[B];
    double S = 0.0;
#pragma unroll
    for (int rr = 0; rr < B; ++rr) {
        const bool ok = FULLROWS || (uint32_t)rr < nrows;
        off[rr] = base + (ok ? rr : 0) * a.W;
        const float* src = xs + off[rr];
        if constexpr (VEC == 4) {
            float4 q = *reinterpret_cast<const float4*>(src);
            v[rr][0] = q.x; v[rr][1] = q.y; v[rr][2] = q.z; v[rr][3] = q.w;
        } else if constexpr (VEC == 2) {
            float2 q = *reinterpret_cast<const float2*>(src);
            v[rr][0] = q.x; v[rr][1] = q.y;
        } else {
            v[rr][0] = src[0];
        }
        double rs = (double)v[rr][0];
#pragma unroll
        for (int c = 1; c < VEC; ++c) rs += (double)v[rr][c];
        S += ok ? rs : 0.0;
    }
    S = valid ? S : 0.0;
    S = group_sum<IPB>(S);

    // exact sum / count, one rounding to fp32, then to the storage type
    const float lfc = lfc_round<T>(mean_of(S, gm.cnt), kC16<T>);
    if (live && gm.writes_lfc) lfc_store<T>(lfc_base, lfc_plane + gm.lfc_idx, lfc, kC16<T>);

    // H^H = H - UpSampling(H^L), written back over x
    float mn = __builtin_inff(), mx = -__builtin_inff();
    float h[B][VEC];
#pragma unroll
    for (int rr = 0; rr < B; ++rr)
#pragma unroll
        for (int c = 0; c < VEC; ++c) {
            h[rr][c] = v[rr][c] - lfc;
            mn = fminf(mn, h[rr][c]);
            mx = fmaxf(mx, h[rr][c]);
        }
    if (valid) {
#pragma unroll
        for (int rr = 0; rr < B; ++rr) {
            float* dst = xs + off[rr];
            if constexpr (VEC == 4) *reinterpret_cast<float4*>(dst) = make_float4(h[rr][0], h[rr][1], h[rr][2], h[rr][3]);
            else if constexpr (VEC == 2) *reinterpret_cast<float2*>(dst) = make_float2(h[rr][0], h[rr][1]);
            else dst[0] = h[rr][0];
        }
        hmin = fminf(hmin, mn);
        hmax = fmaxf(hmax, mx);
    }
}

// staging registers of one chunk: up to 16 coalesced 16-byte loads per lane
struct ChunkRegs { u32x4 q[16]; };

// Issues all loads of the chunk.  Buffer addressing: lane*16 plus a scalar offset, reads past the chunk return
// zero, so there is no per-lane address arithmetic and no bounds branch.
template <typename T>
__device__ __forceinline__ void chunk_load(ChunkRegs& r, const WaveArgs& a, const void* x, uint32_t chunk, uint32_t lane) {
    const uint32_t p0 = chunk * a.G;
    const uint32_t Gc = min(a.G, a.P - p0);
    constexpr uint32_t EPV = 16 / sizeof(T);
    const uint32_t nv = Gc * a.HW / EPV;
    const T* src = static_cast<const T*>(x) + (size_t)p0 * a.HW;
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(src), 0, (int)(nv * 16u), 0x00020000);
    const uint32_t voff = lane * 16u;
#pragma unroll
    for (int u = 0; u < 16; ++u)
        if ((uint32_t)u * 64u < nv) r.q[u] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, u * 1024u, kLoadAux);
}

template <typename T>
__device__ __forceinline__ void chunk_to_lds(const ChunkRegs& r, float* xs, uint32_t nv, uint32_t lane) {
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const uint32_t v = u * 64 + lane;
        if (v < nv) {
            if constexpr (sizeof(T) == 4) {
                reinterpret_cast<u32x4*>(xs)[v] = r.q[u];
            } else {
                const u32x4 q = r.q[u];
                float4 lo, hi;
                lo.x = __uint_as_float(q.x << 16); lo.y = __uint_as_float(q.x & 0xffff0000u);
                lo.z = __uint_as_float(q.y << 16); lo.w = __uint_as_float(q.y & 0xffff0000u);
                hi.x = __uint_as_float(q.z << 16); hi.y = __uint_as_float(q.z & 0xffff0000u);
                hi.z = __uint_as_float(q.w << 16); hi.w = __uint_as_float(q.w & 0xffff0000u);
                reinterpret_cast<float4*>(xs)[2 * v] = lo;
                reinterpret_cast<float4*>(xs)[2 * v + 1] = hi;
            }
        }
    }
}

// A workgroup is ONE wavefront and owns one chunk of G whole planes: no phase
// needs a cross-wave barrier, and a CU keeps a dozen independent wavefronts in
// different phases in flight, so that the HBM loads of some overlap the
// arithmetic of others (measured faster than persistent wavefronts that
// prefetch their next chunk, which ran in lock step).
template <typename T, int BITS, int B, int VEC>
__global__ void __launch_bounds__(64) compress_wave(WaveArgs a) {
    extern __shared__ float4 smem4[];
    float4* params = smem4;                                   // [G] (delta, inv scaled, k1, k2)
    float* xs = reinterpret_cast<float*>(smem4 + a.G);        // [G*HW] x, later the residual h

    constexpr int CPW = 32 / BITS;        // codes per word
    constexpr int PPW = CPW / 2;          // element pairs per word
    constexpr float Lf = float((1 << BITS) - 1);
    constexpr uint32_t EPV = 16 / sizeof(T);
    const uint32_t lane = threadIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, lane);

    const uint32_t chunk = blockIdx.x;
    const uint32_t p0 = chunk * a.G;
    const uint32_t Gc = min(a.G, a.P - p0);
    const uint32_t n = Gc * a.HW;
    {
        // ---- phase 0: chunk -> LDS (fp32): every load is issued before the first LDS write
        const uint32_t nv = a.vec_load ? n / EPV : 0;
        if (a.vec_load) {
            ChunkRegs regs;
            chunk_load<T>(regs, a, pt.x, chunk, lane);
            chunk_to_lds<T>(regs, xs, nv, lane);
        }
        const T* src = static_cast<const T*>(pt.x) + (size_t)p0 * a.HW;
        for (uint32_t e = nv * EPV + lane; e < n; e += 64) xs[e] = Elem<T>::load(src, e);
        wave_sync();

        // ---- phases 1+2: pooling items, then the plane's min / max and scale.
        // ippp <= 64: a round covers 64/ippp whole planes; else a plane takes ippp/64 rounds.
        {
            const bool small = a.ippp <= 64;
            const uint32_t ppr = small ? 64u >> a.ippp_log2 : 1u;       // planes per round
            const uint32_t rpp = small ? 1u : a.ippp >> 6;               // rounds per plane
            const uint32_t S = small ? a.ippp : 64u;
            const uint32_t gsub = small ? lane >> a.ippp_log2 : 0u;
            const uint32_t sub = lane & (S - 1);
            const bool fullrows = (a.H % B) == 0;
            const ItemGeom geom0 = item_geom<B, VEC>(a, sub);      // the lane's item when a plane fits one round
            for (uint32_t g0 = 0; g0 < Gc; g0 += ppr) {
                const uint32_t g = g0 + gsub;
                const bool live = g < Gc;
                const size_t lfc_plane = (size_t)(p0 + g) * a.nb;      // the plane's first LFC element
                float mn = __builtin_inff(), mx = -__builtin_inff();
                if (small) {
                    if (fullrows) pool_item<T, B, VEC, true>(xs, a, pt.lfc, lfc_plane, g, geom0, live, mn, mx);
                    else pool_item<T, B, VEC, false>(xs, a, pt.lfc, lfc_plane, g, geom0, live, mn, mx);
                } else {
                    for (uint32_t t = 0; t < rpp; ++t) {
                        const ItemGeom gm = item_geom<B, VEC>(a, t * 64 + sub);
                        if (fullrows) pool_item<T, B, VEC, true>(xs, a, pt.lfc, lfc_plane, g, gm, live, mn, mx);
                        else pool_item<T, B, VEC, false>(xs, a, pt.lfc, lfc_plane, g, gm, live, mn, mx);
                    }
                }
                group_minmax(S, mn, mx);
                if (live && sub == 0) params[g] = make_float4(mn, mx, 0.0f, 0.0f);
            }
        }
        wave_sync();

        // ---- phase 2: one lane per plane: scale of Eq. (quantization) and the plane's keys
        for (uint32_t g = lane; g < Gc; g += 64) {
            const float4 mm = params[g];
            float delta, Delta, inv;
            plane_scale_any(mm.x, mm.y, Lf, kC16<T>, delta, Delta, inv);
            const uint32_t p = p0 + g;
            const uint32_t k1 = mix32(p ^ pt.seed_a);
            const uint32_t k2 = mix32(k1 + pt.seed_c);
            meta_store(pt.meta, p, delta, Delta, kC16<T>);
            params[g] = make_float4(delta, inv * (float)(1u << (32 - BITS)), __uint_as_float(k1), __uint_as_float(k2));
        }
        wave_sync();

        // ---- phase 3: Quant of Eq. (quantization) + packing
        {
            const uint32_t nwords = Gc * a.WPP;
            const bool hw4 = (a.HW & 3u) == 0;
            const uint32_t rscale = 1u << (16 - BITS);
            // a short last round is done pair-per-lane instead of word-per-lane
            const uint32_t tailw = nwords & 63u;
            const bool pair_tail = tailw != 0 && tailw * PPW <= 64;
            const uint32_t nfull = pair_tail ? nwords - tailw : nwords;
            for (uint32_t wi = lane; wi < nfull; wi += 64) {
                const uint32_t g = fdiv(wi, a.d_wpp);
                const uint32_t k = wi - g * a.WPP;
                const float4 pr = params[g];
                const float delta = pr.x, invs = pr.y;
                const uint32_t k1 = __float_as_uint(pr.z), k2 = __float_as_uint(pr.w);
                const uint32_t e0 = k * CPW;
                const uint32_t left = a.HW - e0;
                const float* hp = xs + g * a.HW + e0;
                // A ragged last word reads past its plane (into the next plane or the
                // LDS slack behind the chunk); those codes are cleared below.
                float h[CPW];
                if (hw4) {
#pragma unroll
                    for (int q = 0; q < CPW / 4; ++q) {
                        float4 f = reinterpret_cast<const float4*>(hp)[q];
                        h[4 * q] = f.x; h[4 * q + 1] = f.y; h[4 * q + 2] = f.z; h[4 * q + 3] = f.w;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < CPW; ++e) h[e] = hp[e];
                }
                const uint32_t xw0 = k1 + (k * PPW) * kWeyl;
                uint32_t word = 0;
#pragma unroll
                for (int j = PPW - 1; j >= 0; --j)
                    word = push_pair<BITS>(word, h[2 * j], h[2 * j + 1], delta, invs, xw0 + (uint32_t)j * kWeyl, k2, rscale);
                if (left < (uint32_t)CPW) word &= (1u << (left * BITS)) - 1u;      // pad bits are zero
                pt.codes[(size_t)(p0 + g) * a.WPP + k] = word;
            }
            if (pair_tail) {
                // lane = one element pair of the last words; PPW adjacent lanes build one word
                const uint32_t wi = nfull + lane / PPW;
                const uint32_t pw = lane % PPW;
                const bool act = wi < nwords;
                uint32_t part = 0;
                uint32_t g = 0, k = 0;
                if (act) {
                    g = fdiv(wi, a.d_wpp);
                    k = wi - g * a.WPP;
                    const float4 pr = params[g];
                    const float delta = pr.x, invs = pr.y;
                    const uint32_t k1 = __float_as_uint(pr.z), k2 = __float_as_uint(pr.w);
                    const uint32_t e0 = k * CPW + 2 * pw;
                    const float* hp = xs + g * a.HW;
                    const float h0 = e0 < a.HW ? hp[e0] : delta;
                    const float h1 = e0 + 1 < a.HW ? hp[e0 + 1] : delta;
                    const uint32_t two = push_pair<BITS>(0u, h0, h1, delta, invs, k1 + (k * PPW + pw) * kWeyl, k2, rscale);
                    part = two << (pw * 2 * BITS);
                }
                part |= __builtin_amdgcn_update_dpp(0, (int)part, kDppXor1, 0xf, 0xf, false);
                if constexpr (PPW >= 4) part |= __builtin_amdgcn_update_dpp(0, (int)part, kDppXor2, 0xf, 0xf, false);
                if constexpr (PPW == 8) part |= __builtin_amdgcn_update_dpp(0, (int)part, kDppHalfMirror, 0xf, 0xf, false);
                if (act && pw == 0) pt.codes[(size_t)(p0 + g) * a.WPP + k] = part;
            }
        }
    }
}

// ------------------------------------------------------------------ compress, items straight from global memory

struct ItemsArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, H, W, HW, LW, nb, WPP;
    uint32_t ipr;        // item slots per block row (padded to the items-per-block count)
    uint32_t ipp;        // item slots per plane = LH * ipr (<= 64)
    uint32_t S;          // lanes per plane: ipp rounded up to a power of two
    uint32_t S_log2;
    uint32_t ppr;        // planes per round = 64 / S
    uint32_t rpw;        // rounds a workgroup handles one after the other
    uint32_t nrounds;    // ceil(P / ppr)
    FastDiv d_ipr;
};

// Small planes (at most 64 pooling items, e.g. 28x28 and 14x14 with B = 8): one
// wavefront per round of 64/S whole planes, and x never goes through LDS.  A
// lane owns one pooling item (B rows x VEC columns of one block) and loads it
// straight from global memory, one VEC-wide load per row; the items of a block
// and of a plane sit in adjacent lanes, so the block sum (binary64) and the
// plane's min / max are DPP reductions and every lane ends up with its plane's
// scale.  The item is quantised out of the registers; its VEC codes per row are
// OR-ed into the round's packed words in LDS (cleared first, so pad bits stay
// zero), which then leave as whole coalesced words.  R = rows an item holds: B, or 1 for
// maps of a single row (1-D maps), whose items would otherwise carry B - 1 masked rows.
template <typename T, int BITS, int B, int VEC, int R>
__global__ void __launch_bounds__(64) compress_items(ItemsArgs a) {
    constexpr int IPB = B / VEC;          // items per block (power of two)
    constexpr int CPW = 32 / BITS;        // codes per word
    constexpr float Lf = float((1 << BITS) - 1);
    extern __shared__ float4 smem4[];
    uint32_t* cw = reinterpret_cast<uint32_t*>(smem4);        // [ppr * WPP] packed words of the round

    const uint32_t lane = threadIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, lane);

    // the lane's item: the same in every round
    const uint32_t g = lane >> a.S_log2;                      // plane of the round
    const uint32_t sub = lane & (a.S - 1);
    const uint32_t bi = fdiv(sub, a.d_ipr);
    const uint32_t sl = sub - bi * a.ipr;
    const uint32_t col0 = sl * VEC, r0 = bi * B, bj = sl / IPB;
    const bool in_plane = sub < a.ipp && col0 < a.W;
    const uint32_t off = in_plane ? r0 * a.W + col0 : 0u;     // first element of the item inside its plane
    const uint32_t nrows = in_plane ? min((uint32_t)B, a.H - r0) : 1u;
    const uint32_t cnt = max(min((uint32_t)B, a.H - min(a.H, r0)) * min((uint32_t)B, a.W - min(a.W, bj * B)), 1u);
    const uint32_t lfc_idx = bi * a.LW + bj;
    const bool writes_lfc = in_plane && (sl % IPB) == 0;
    const bool fullrows = R == 1 || (a.H % B) == 0;
    const uint32_t rscale = 1u << (16 - BITS);
    const uint32_t xoff = (off / 2u) * kWeyl;                 // pair counter of the item's first row
    const uint32_t rowW = (a.W / 2u) * kWeyl;                 // pair counter distance between rows
    const uint32_t rwords = a.ppr * a.WPP;

    const uint32_t rend = min(a.nrounds, (blockIdx.x + 1) * a.rpw);
    for (uint32_t round = blockIdx.x * a.rpw; round < rend; ++round) {
        const uint32_t p0 = round * a.ppr;
        const uint32_t Gc = min(a.ppr, a.P - p0);
        const bool live = g < Gc;
        const bool valid = live && in_plane;

        // ---- load the item: rows past the map re-read row 0 (no effect on min / max, left out of the sum);
        // lanes without an item read item 0 of the round and have their effects masked
        float v[R][VEC];
        {
            const T* src = static_cast<const T*>(pt.x) + (size_t)p0 * a.HW;
            const __amdgpu_buffer_rsrc_t rsrc =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(src), 0, (int)(Gc * a.HW * sizeof(T)), 0x00020000);
            const uint32_t base = (valid ? g * a.HW + off : 0u) * (uint32_t)sizeof(T);
            const uint32_t rowb = a.W * (uint32_t)sizeof(T);
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                const uint32_t vo = fullrows ? base : base + ((uint32_t)rr < nrows ? rr * rowb : 0u);
                const uint32_t so = fullrows ? rr * rowb : 0u;
                if constexpr (sizeof(T) == 4 && VEC == 4) {
                    const u32x4 q = __builtin_amdgcn_raw_buffer_load_b128(rsrc, vo, so, kLoadAux);
                    v[rr][0] = __uint_as_float(q.x); v[rr][1] = __uint_as_float(q.y);
                    v[rr][2] = __uint_as_float(q.z); v[rr][3] = __uint_as_float(q.w);
                } else if constexpr (sizeof(T) == 4 && VEC == 2) {
                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                    const u32x2 q = __builtin_amdgcn_raw_buffer_load_b64(rsrc, vo, so, kLoadAux);
                    v[rr][0] = __uint_as_float(q.x); v[rr][1] = __uint_as_float(q.y);
                } else if constexpr (VEC == 4) {
                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                    const u32x2 q = __builtin_amdgcn_raw_buffer_load_b64(rsrc, vo, so, kLoadAux);
                    v[rr][0] = __uint_as_float(q.x << 16); v[rr][1] = __uint_as_float(q.x & 0xffff0000u);
                    v[rr][2] = __uint_as_float(q.y << 16); v[rr][3] = __uint_as_float(q.y & 0xffff0000u);
                } else {
                    const uint32_t q = __builtin_amdgcn_raw_buffer_load_b32(rsrc, vo, so, kLoadAux);
                    v[rr][0] = __uint_as_float(q << 16); v[rr][1] = __uint_as_float(q & 0xffff0000u);
                }
            }
        }
        // the round's packed words start at zero
        for (uint32_t w = lane; w < rwords; w += 64) cw[w] = 0u;

        // ---- Sec. 4.1 AveragePooling: block sum in binary64 over the block's adjacent lanes
        double Sm = 0.0;
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            double rs = (double)v[rr][0];
#pragma unroll
            for (int c = 1; c < VEC; ++c) rs += (double)v[rr][c];
            Sm += (fullrows || (uint32_t)rr < nrows) ? rs : 0.0;
        }
        Sm = valid ? Sm : 0.0;
        Sm = group_sum<IPB>(Sm);
        const float lfc = lfc_round<T>(mean_of(Sm, cnt), kC16<T>);
        if (valid && writes_lfc) lfc_store<T>(pt.lfc, (size_t)(p0 + g) * a.nb + lfc_idx, lfc, kC16<T>);

        // ---- residual H^H = H - UpSampling(H^L) in place, plane min / max
        float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
        for (int rr = 0; rr < R; ++rr)
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                v[rr][c] = v[rr][c] - lfc;
                mn = fminf(mn, v[rr][c]);
                mx = fmaxf(mx, v[rr][c]);
            }
        mn = valid ? mn : __builtin_inff();
        mx = valid ? mx : -__builtin_inff();
        group_minmax(a.S, mn, mx);

        // ---- scale of Eq. (quantization), keys, meta: every lane of the plane computes the same values
        float delta, Delta, inv;
        plane_scale_any(mn, mx, Lf, kC16<T>, delta, Delta, inv);
        const float invs = inv * (float)(1u << (32 - BITS));
        const uint32_t p = p0 + g;
        const uint32_t k1 = mix32(p ^ pt.seed_a);
        const uint32_t k2 = mix32(k1 + pt.seed_c);
        if (live && sub == 0) meta_store(pt.meta, p, delta, Delta, kC16<T>);
        wave_sync();                                           // the zeroed words precede the ORs below

        // ---- Quant + packing: the VEC codes of a row are OR-ed into their word (a row part never straddles words)
        {
            const uint32_t xw0 = k1 + xoff;
            uint32_t* const pw = cw + g * a.WPP;
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                const uint32_t xw = xw0 + (uint32_t)rr * rowW;
                uint32_t c;
                if constexpr (VEC == 4) {
                    c = push_pair<BITS>(0u, v[rr][2], v[rr][3], delta, invs, xw + kWeyl, k2, rscale);
                    c = push_pair<BITS>(c, v[rr][0], v[rr][1], delta, invs, xw, k2, rscale);
                } else {
                    c = push_pair<BITS>(0u, v[rr][0], v[rr][1], delta, invs, xw, k2, rscale);
                }
                const uint32_t i = off + (uint32_t)rr * a.W;              // element index inside the plane
                if (valid && (fullrows || (uint32_t)rr < nrows))
                    __hip_atomic_fetch_or(pw + i / CPW, c << ((i % CPW) * BITS), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
        wave_sync();
        {
            uint32_t* dst = pt.codes + (size_t)p0 * a.WPP;
            const uint32_t nw = Gc * a.WPP;
            for (uint32_t w = lane; w < nw; w += 64) dst[w] = cw[w];
        }
        wave_sync();                                           // the words are cleared again by the next round
    }
}

// ------------------------------------------------------------------ one-block planes, a lane per plane

struct LaneArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, HW, WPP;
    uint32_t nrounds;    // ceil(P / 64): a round is 64 planes, one per lane
    uint32_t rpw;        // rounds a workgroup handles one after the other
    uint32_t vec_load;   // x is 16-byte aligned (a round starts on a 16-byte boundary)
};

// Planes that are a single block (H <= B and W <= B, e.g. 7x7 with B = 8) with
// an odd number of elements: one wavefront per round of 64 planes.  The round
// (64*HW contiguous elements) is loaded with coalesced 16-byte loads and parked
// in LDS; then lane g owns plane g outright: it reads its HW elements with a
// stride of HW words (odd, so the 64 lanes hit 64 different banks), sums them in
// binary64 in index order, takes min / max, and in a second pass quantises its
// plane pair by pair into its WPP words.  No cross-lane step at all.
template <typename T, int BITS>
__global__ void __launch_bounds__(64) compress_lane(LaneArgs a) {
    constexpr int CPW = 32 / BITS;        // codes per word
    constexpr int PPW = CPW / 2;          // element pairs per word
    constexpr uint32_t EPV = 16 / sizeof(T);
    constexpr float Lf = float((1 << BITS) - 1);
    extern __shared__ float4 smem4[];
    float* xs = reinterpret_cast<float*>(smem4);              // [64 * HW (+3)]

    const uint32_t lane = threadIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, lane);
    const uint32_t rscale = 1u << (16 - BITS);
    const float* mine = xs + lane * a.HW;

    const uint32_t rend = min(a.nrounds, (blockIdx.x + 1) * a.rpw);
    for (uint32_t round = blockIdx.x * a.rpw; round < rend; ++round) {
        const uint32_t p0 = round * 64u;
        const uint32_t Gc = min(64u, a.P - p0);
        const uint32_t n = Gc * a.HW;
        const bool live = lane < Gc;
        const T* src = static_cast<const T*>(pt.x) + (size_t)p0 * a.HW;

        // ---- the round -> LDS as fp32; vectors past its end read as zero
        const uint32_t nv = a.vec_load ? n / EPV : 0u;
        if (a.vec_load) {
            const __amdgpu_buffer_rsrc_t rsrc =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(src), 0, (int)(nv * 16u), 0x00020000);
            u32x4 q[16];
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if ((uint32_t)u * 64u < nv) q[u] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane * 16u, u * 1024, kLoadAux);
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const uint32_t vi = lane + 64u * u;
                if ((uint32_t)u * 64u < nv && vi < nv) {
                    if constexpr (sizeof(T) == 4) {
                        reinterpret_cast<u32x4*>(xs)[vi] = q[u];
                    } else {
                        float4* d = reinterpret_cast<float4*>(xs) + 2 * vi;
                        d[0] = make_float4(__uint_as_float(q[u].x << 16), __uint_as_float(q[u].x & 0xffff0000u),
                                           __uint_as_float(q[u].y << 16), __uint_as_float(q[u].y & 0xffff0000u));
                        d[1] = make_float4(__uint_as_float(q[u].z << 16), __uint_as_float(q[u].z & 0xffff0000u),
                                           __uint_as_float(q[u].w << 16), __uint_as_float(q[u].w & 0xffff0000u));
                    }
                }
            }
        }
        for (uint32_t e = nv * EPV + lane; e < n; e += 64) xs[e] = Elem<T>::load(src, e);
        wave_sync();

        // ---- Sec. 4.1 AveragePooling over the whole plane, min / max of x.  x -> fl(x - m) is
        // monotone, so the residual's extremes are fl(min x - m) and fl(max x - m).
        // Lanes past the last plane work on plane 0 of the round and store nothing.
        const float* pl = live ? mine : xs;
        double S = 0.0;
        float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll 7
        for (uint32_t e = 0; e < a.HW; ++e) {
            const float v = pl[e];
            S += (double)v;
            mn = fminf(mn, v);
            mx = fmaxf(mx, v);
        }
        const float lfc = lfc_round<T>(mean_of(S, a.HW), kC16<T>);
        const float hmn = mn - lfc, hmx = mx - lfc;
        float delta, Delta, inv;
        plane_scale_any(hmn, hmx, Lf, kC16<T>, delta, Delta, inv);
        const float invs = inv * (float)(1u << (32 - BITS));
        const uint32_t p = p0 + lane;
        const uint32_t k1 = mix32(p ^ pt.seed_a);
        const uint32_t k2 = mix32(k1 + pt.seed_c);
        if (live) {
            lfc_store<T>(pt.lfc, p, lfc, kC16<T>);
            meta_store(pt.meta, p, delta, Delta, kC16<T>);
        }

        // ---- residual, Quant of Eq. (quantization), packing: whole words, then the ragged last one
        uint32_t* cdst = pt.codes + (size_t)p * a.WPP;
        const uint32_t wfull = a.HW / CPW;
        for (uint32_t w = 0; w < wfull; ++w) {
            const float* hp = pl + w * CPW;
            const uint32_t xw0 = k1 + (w * PPW) * kWeyl;
            uint32_t word = 0;
#pragma unroll
            for (int j = PPW - 1; j >= 0; --j)
                word = push_pair<BITS>(word, hp[2 * j] - lfc, hp[2 * j + 1] - lfc, delta, invs, xw0 + (uint32_t)j * kWeyl, k2, rscale);
            if (live) cdst[w] = word;
        }
        const uint32_t left = a.HW - wfull * CPW;              // 0 .. CPW-1 elements in the last word
        if (left) {
            const float* hp = pl + wfull * CPW;
            const uint32_t xw0 = k1 + (wfull * PPW) * kWeyl;
            uint32_t word = 0;
            // pairs from the last one down; an odd `left` pairs its last element with a repeat of itself
            for (int j = (int)((left - 1) / 2); j >= 0; --j) {
                const float h0 = hp[2 * j] - lfc;
                const float h1 = hp[min((uint32_t)(2 * j + 1), left - 1)] - lfc;
                word = push_pair<BITS>(word, h0, h1, delta, invs, xw0 + (uint32_t)j * kWeyl, k2, rscale);
            }
            word &= (1u << (left * BITS)) - 1u;                 // pad bits are zero
            if (live) cdst[wfull] = word;
        }
        wave_sync();      // LDS is reused by the next round
    }
}

// ------------------------------------------------------------------ compress, plane held in registers

struct RegsArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, H, W, HW, LH, LW, nb, WPP;
    uint32_t q4;         // units (4 consecutive elements) per plane = H*W/4
    uint32_t w4;         // units per row = W/4
    uint32_t ppw;        // planes a workgroup handles one after the other
    uint32_t B;          // block size, read by the instance for any B (template argument 0) only
    FastDiv d_w4, d_LW, d_B, d_upb;      // d_upb divides by B / 4
    void* y;             // relu_compress_regs: the activation's output map and its 1-bit mask (one map per launch)
    uint32_t* mask;
    uint32_t D;          // compress_regs_3d: depth slices; H, LH then count the rows / block rows of ONE slice
    FastDiv d_H, d_slice;    // divide by H and by LH * LW
};

constexpr int kRegUnits = 13;     // units per lane: planes of up to 13 * (threads per workgroup) units

// Large planes (56x56 with one wavefront, 112x112 with four): the plane never
// goes through LDS.  Lane `tid` keeps units tid, tid+NT, tid+2NT, ... (the
// layout of the coalesced 16-byte loads) in registers from the load to the
// packed codes; LDS carries only one binary64 sum per unit and one LFC value
// per block (~7 KB per wavefront), so occupancy is set by registers, not LDS.
// A unit lies inside one block (W % 4 == 0, B % 4 == 0), which block is the
// same for every plane and is worked out once per workgroup.
// B = 0 is the instance for any block size that is a multiple of 4 (12, 16, 64 of the paper's
// sweep): the block size comes from the arguments, the loops over a block's unit sums run to
// their bounds instead of being unrolled, and rounds of units past the plane are skipped, so
// that planes far below 13 units per lane are worth taking too.
// RELU: x is the input of a Relu operator (Appendix, Relu listing) whose output y is the map to
// cache: y = x where x > 0 else +0 is written out, its 1-bit mask too (H*W a multiple of 32: a
// plane's mask is whole words, a word is the eight units of eight neighbouring lanes), and y is
// what gets compressed, without a second trip through HBM.
// ND = 3: planes of D x H x W elements with blocks of B x B x B (Appendix D); a unit's block and the
// units of a block are found with the depth as a third coordinate, everything else is the same.
template <typename T, int BITS, int B, int NW, bool RELU, int ND = 2>
__device__ __forceinline__ void compress_regs_body(const RegsArgs& a) {
    constexpr int NT = 64 * NW;
    constexpr int K = kRegUnits;
    constexpr int UPB = B / 4;            // units per block row
    constexpr float Lf = float((1 << BITS) - 1);
    extern __shared__ float4 smem4[];
    double* usum = reinterpret_cast<double*>(smem4);                  // [K*NT] per-unit sums
    float* lfcs = reinterpret_cast<float*>(usum + K * NT);            // [nb + 1], last = NaN sentinel
    float* red = lfcs + ((a.nb + 1 + 3) & ~3u);                        // [2*NW] cross-wave min / max
    double* zsum = reinterpret_cast<double*>(red + 2 * NW + 2);       // [nb*B] (3-D maps) one sum per block and depth slice

    const uint32_t tid = threadIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, tid);

    // which block each of the lane's units belongs to (nb = sentinel for units past the plane)
    uint32_t blk[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t f = tid + NT * k;
        const uint32_t row = fdiv(f, a.d_w4);          // row, counted over all depth slices
        const uint32_t c4 = f - row * a.w4;
        if constexpr (ND == 3) {
            const uint32_t z = fdiv(row, a.d_H);
            blk[k] = f < a.q4 ? ((z / B) * a.LH + (row - z * a.H) / B) * a.LW + c4 / UPB : a.nb;
        } else if constexpr (B != 0) blk[k] = f < a.q4 ? (row / B) * a.LW + c4 / UPB : a.nb;
        else blk[k] = f < a.q4 ? fdiv(row, a.d_B) * a.LW + fdiv(c4, a.d_upb) : a.nb;
    }
    if (tid == 0) lfcs[a.nb] = __builtin_nanf("");
    bool full_blocks = false;
    if constexpr (B != 0) full_blocks = (a.H % B) == 0 && (a.W % B) == 0 && (ND == 2 || (a.D % B) == 0);
    // rounds of units a plane has (uniform); the one- and four-wavefront instances for B = 4 and 8
    // always run all K (their planes fill at least eight of them)
    auto round_live = [&](int k) -> bool { return (B != 0 && NW != 16 && ND == 2) || (uint32_t)(NT * k) < a.q4; };

    const uint32_t pbeg = blockIdx.x * a.ppw;
    const uint32_t pend = min(a.P, pbeg + a.ppw);
    for (uint32_t p = pbeg; p < pend; ++p) {
        // ---- load the plane: coalesced, bounds-checked (units past the plane read as zero)
        float x[K][4];
        {
            const T* src = static_cast<const T*>(pt.x) + (size_t)p * a.HW;
            const __amdgpu_buffer_rsrc_t rsrc =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(src), 0, (int)(a.HW * sizeof(T)), 0x00020000);
#pragma unroll
            for (int k = 0; k < K; ++k) {
                if (!round_live(k)) {
                    x[k][0] = x[k][1] = x[k][2] = x[k][3] = 0.0f;
                    continue;
                }
                if constexpr (sizeof(T) == 4) {
                    const u32x4 q = __builtin_amdgcn_raw_buffer_load_b128(rsrc, tid * 16u, k * NT * 16, kLoadAux);
                    x[k][0] = __uint_as_float(q.x); x[k][1] = __uint_as_float(q.y);
                    x[k][2] = __uint_as_float(q.z); x[k][3] = __uint_as_float(q.w);
                } else {
                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                    const u32x2 q = __builtin_amdgcn_raw_buffer_load_b64(rsrc, tid * 8u, k * NT * 8, kLoadAux);
                    x[k][0] = __uint_as_float(q.x << 16); x[k][1] = __uint_as_float(q.x & 0xffff0000u);
                    x[k][2] = __uint_as_float(q.y << 16); x[k][3] = __uint_as_float(q.y & 0xffff0000u);
                }
            }
        }
        if constexpr (RELU) {
            T* ydst = static_cast<T*>(a.y) + (size_t)p * a.HW;
            const __amdgpu_buffer_rsrc_t yrs =
                __builtin_amdgcn_make_buffer_rsrc(ydst, 0, (int)(a.HW * sizeof(T)), 0x00020000);
            const __amdgpu_buffer_rsrc_t mrs =
                __builtin_amdgcn_make_buffer_rsrc(a.mask + (size_t)p * (a.HW / 32), 0, (int)(a.HW / 8), 0x00020000);
#pragma unroll
            for (int k = 0; k < K; ++k) {
                if (!round_live(k)) continue;
                uint32_t nib = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool pos = x[k][e] > 0.0f;
                    nib |= (pos ? 1u : 0u) << e;
                    x[k][e] = pos ? x[k][e] : 0.0f;
                }
                // stores past the plane are dropped by the buffer bound
                if constexpr (sizeof(T) == 4) {
                    u32x4 o;
                    o.x = __float_as_uint(x[k][0]); o.y = __float_as_uint(x[k][1]);
                    o.z = __float_as_uint(x[k][2]); o.w = __float_as_uint(x[k][3]);
                    __builtin_amdgcn_raw_buffer_store_b128(o, yrs, tid * 16u, k * NT * 16, 0);
                } else {
                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                    u32x2 o;
                    o.x = (__float_as_uint(x[k][0]) >> 16) | (__float_as_uint(x[k][1]) & 0xffff0000u);
                    o.y = (__float_as_uint(x[k][2]) >> 16) | (__float_as_uint(x[k][3]) & 0xffff0000u);
                    __builtin_amdgcn_raw_buffer_store_b64(o, yrs, tid * 8u, k * NT * 8, 0);
                }
                uint32_t w = nib << (4u * (tid & 7u));
                w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, kDppXor1, 0xf, 0xf, false);
                w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, kDppXor2, 0xf, 0xf, false);
                w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, kDppHalfMirror, 0xf, 0xf, false);
                if ((tid & 7u) == 0) __builtin_amdgcn_raw_buffer_store_b32(w, mrs, (tid >> 3) * 4u, k * (NT / 8) * 4, 0);
            }
        }
        // ---- Sec. 4.1 AveragePooling, step 1: one binary64 sum per unit
#pragma unroll
        for (int k = 0; k < K; ++k)
            if (round_live(k)) usum[tid + NT * k] = ((double)x[k][0] + (double)x[k][1]) + ((double)x[k][2] + (double)x[k][3]);
        if constexpr (NW == 1) wave_sync(); else lds_barrier();

        if constexpr (ND == 3) {
            // ---- step 2a (3-D maps): a lane per (block, depth slice) adds that slice's B x UPB unit sums
            for (uint32_t t2 = tid; t2 < a.nb * B; t2 += NT) {
                const uint32_t t = t2 / B, z = t2 - t * B;
                const uint32_t bd = fdiv(t, a.d_slice);
                const uint32_t rem = t - bd * (a.LH * a.LW);
                const uint32_t bi3 = fdiv(rem, a.d_LW);
                const uint32_t bj3 = rem - bi3 * a.LW;
                const uint32_t deps = min((uint32_t)B, a.D - bd * B);
                const uint32_t rows = min((uint32_t)B, a.H - bi3 * B);
                const uint32_t units = min((uint32_t)UPB, a.w4 - bj3 * UPB);
                double Sz = 0.0;
                if (z < deps) {
                    const double* us = usum + ((bd * B + z) * a.H + bi3 * B) * a.w4 + bj3 * UPB;
#pragma unroll
                    for (int rr = 0; rr < B; ++rr)
#pragma unroll
                        for (int u = 0; u < UPB; ++u) {
                            const bool ok = (uint32_t)rr < rows && (uint32_t)u < units;
                            const double v = us[ok ? rr * a.w4 + u : 0u];
                            Sz += ok ? v : 0.0;
                        }
                }
                zsum[t2] = Sz;
            }
            if constexpr (NW == 1) wave_sync(); else lds_barrier();
        }
        // ---- step 2: a lane per block adds the block's unit sums in a fixed order
        for (uint32_t t = tid; t < a.nb; t += NT) {
            const uint32_t bi = fdiv(t, a.d_LW);
            const uint32_t bj = t - bi * a.LW;
            double S = 0.0;
            uint32_t cnt;
            if constexpr (B == 0) {
                const uint32_t upb = a.B / 4;
                const uint32_t rows = min(a.B, a.H - bi * a.B);
                const uint32_t units = min(upb, a.w4 - bj * upb);
                const double* us = usum + bi * a.B * a.w4 + bj * upb;
                // four reads at a time (units past the block re-read its first and add nothing), so
                // that several reads go out together
                for (uint32_t rr = 0; rr < rows; ++rr) {
                    for (uint32_t ub = 0; ub < units; ub += 4) {
#pragma unroll
                        for (uint32_t u = 0; u < 4; ++u) {
                            const bool ok = ub + u < units;
                            const double v = us[ok ? rr * a.w4 + ub + u : 0u];
                            S += ok ? v : 0.0;
                        }
                    }
                }
                cnt = rows * units * 4;
            }
            const uint32_t u0 = bi * B * a.w4 + bj * UPB;
            if constexpr (ND == 3) {
                // t = (bd * LH + bi3) * LW + bj: the block's units are B slices x B rows x UPB units
                const uint32_t bd = fdiv(t, a.d_slice);
                const uint32_t rem = t - bd * (a.LH * a.LW);
                const uint32_t bi3 = fdiv(rem, a.d_LW);
                const uint32_t bj3 = rem - bi3 * a.LW;
                const uint32_t deps = min((uint32_t)B, a.D - bd * B);
                const uint32_t rows = min((uint32_t)B, a.H - bi3 * B);
                const uint32_t units = min((uint32_t)UPB, a.w4 - bj3 * UPB);
#pragma unroll
                for (int z = 0; z < B; ++z) S += zsum[t * B + z];          // slices past the map hold 0
                cnt = deps * rows * units * 4;
            } else if constexpr (B == 0) {
            } else if (full_blocks) {
#pragma unroll
                for (int rr = 0; rr < B; ++rr)
#pragma unroll
                    for (int u = 0; u < UPB; ++u) S += usum[u0 + rr * a.w4 + u];
                cnt = B * B;
            } else {
                const uint32_t rows = min((uint32_t)B, a.H - bi * B);
                const uint32_t units = min((uint32_t)UPB, a.w4 - bj * UPB);
#pragma unroll
                for (int rr = 0; rr < B; ++rr)
#pragma unroll
                    for (int u = 0; u < UPB; ++u) {
                        const bool ok = (uint32_t)rr < rows && (uint32_t)u < units;
                        const double v = usum[ok ? u0 + rr * a.w4 + u : u0];
                        S += ok ? v : 0.0;
                    }
                cnt = rows * units * 4;
            }
            const float lfc = lfc_round<T>(mean_of(S, cnt), kC16<T>);
            lfcs[t] = lfc;
            lfc_store<T>(pt.lfc, (size_t)p * a.nb + t, lfc, kC16<T>);
        }
        if constexpr (NW == 1) wave_sync(); else lds_barrier();

        // ---- residual H^H = H - UpSampling(H^L) in place, plane min / max.
        // Units past the plane take the NaN sentinel: their residual is NaN,
        // which min / max skip.
        float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (!round_live(k)) continue;
            const float lfc = lfcs[blk[k]];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x[k][e] = x[k][e] - lfc;
                mn = fminf(mn, x[k][e]);
                mx = fmaxf(mx, x[k][e]);
            }
        }
        group_minmax(64, mn, mx);
        if constexpr (NW > 1) {
            if ((tid & 63u) == 0) { red[2 * (tid >> 6)] = mn; red[2 * (tid >> 6) + 1] = mx; }
            lds_barrier();
#pragma unroll
            for (int w = 0; w < NW; ++w) { mn = fminf(mn, red[2 * w]); mx = fmaxf(mx, red[2 * w + 1]); }
        }

        // ---- scale of Eq. (quantization), keys, meta
        float delta, Delta, inv;
        plane_scale_any(mn, mx, Lf, kC16<T>, delta, Delta, inv);
        const float invs = inv * (float)(1u << (32 - BITS));
        const uint32_t k1 = mix32(p ^ pt.seed_a);
        const uint32_t k2 = mix32(k1 + pt.seed_c);
        if (tid == 0) meta_store(pt.meta, p, delta, Delta, kC16<T>);

        // ---- Quant + packing: a unit is two element pairs = 4 codes (one byte for b = 2, a word for b = 8)
        {
            const uint32_t rscale = 1u << (16 - BITS);
            constexpr uint32_t CB = BITS / 2;                         // code bytes per unit (1, 2 or 4)
            uint8_t* cbase = reinterpret_cast<uint8_t*>(pt.codes) + (size_t)p * a.WPP * 4;
            const __amdgpu_buffer_rsrc_t crs =
                __builtin_amdgcn_make_buffer_rsrc(cbase, 0, (int)(a.q4 * CB), 0x00020000);
            const uint32_t xw0 = k1 + (2u * tid) * kWeyl;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                if (!round_live(k)) continue;
                const uint32_t xw = xw0 + (uint32_t)(2 * NT * k) * kWeyl;
                uint32_t c = push_pair<BITS>(0u, x[k][2], x[k][3], delta, invs, xw + kWeyl, k2, rscale);
                c = push_pair<BITS>(c, x[k][0], x[k][1], delta, invs, xw, k2, rscale);
                // stores past the plane's code bytes are dropped by the buffer bound
                if constexpr (CB == 1) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)c, crs, tid, k * NT, 0);
                else if constexpr (CB == 2) __builtin_amdgcn_raw_buffer_store_b16((uint16_t)c, crs, tid * 2u, k * NT * 2, 0);
                else __builtin_amdgcn_raw_buffer_store_b32(c, crs, tid * 4u, k * NT * 4, 0);
            }
            // pad bytes of the plane's last word are zero
            const uint32_t padb = a.WPP * 4 - a.q4 * CB;
            if (tid < padb) cbase[a.q4 * CB + tid] = 0;
        }
        if constexpr (NW == 1) wave_sync(); else lds_barrier();      // usum, lfcs and red are reused
    }
}

template <typename T, int BITS, int B, int NW>
__global__ void __launch_bounds__(64 * NW) compress_regs(RegsArgs a) { compress_regs_body<T, BITS, B, NW, false>(a); }
template <typename T, int BITS, int B, int NW>
__global__ void __launch_bounds__(64 * NW) relu_compress_regs(RegsArgs a) { compress_regs_body<T, BITS, B, NW, true>(a); }
template <typename T, int BITS, int B, int NW>
__global__ void __launch_bounds__(64 * NW) compress_regs_3d(RegsArgs a) { compress_regs_body<T, BITS, B, NW, false, 3>(a); }

// ------------------------------------------------------------------ compress, plane in registers, any width

struct UnitsArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, H, W, HW, LW, nb, WPP, B;
    uint32_t q4;         // units (4 consecutive elements) per plane, the last one may be partly past it
    uint32_t q4p;        // q4 rounded up to whole rounds of the plane's lanes
    uint32_t nitem;      // nb * B row segments
    uint32_t S, S_log2;  // instance NW = 0: lanes per plane (8, 16 or 32), 64 / S planes per wavefront
    uint32_t reg_bytes;  // LDS bytes of one plane's region (a multiple of 16)
    uint32_t nrounds;    // rounds of planes the grid walks over: P, or P / (64 / S) rounded up (NW = 0)
    FastDiv d_W, d_B, d_LW;
};

// Planes whose rows or blocks are not whole 16-byte vectors (odd widths: 55 x 55, 27 x 27,
// 147 x 147; block sizes such as 18): the register kernel's structure with the block found per
// element instead of per unit.  A unit is four consecutive elements of the plane whatever the
// width (planes start on 4-byte boundaries, which is all a 16-byte buffer load needs); lane l of
// the S lanes of a plane takes units l, l+S, ...  Which block each element belongs to is the same
// for every plane: worked out once per workgroup and kept as the LDS byte offset of the block's
// LFC, two offsets per register.  The plane is parked in LDS (the next plane's loads go out right
// after and fly during the rest); a lane per (block, row of the block) adds its row segment in
// binary64 (lanes of one block read rows W floats apart: no bank conflicts for odd W), a lane per
// block adds its rows; the residual goes back to LDS and is quantised from there.  Elements of
// the last unit past the plane take the NaN sentinel like whole units past it.
// NW = 1 .. 16: the NW wavefronts of the workgroup share one plane (S = 64 * NW).  NW = 0: small
// planes (below 512 elements), S = 8, 16 or 32 lanes per plane and 64 / S planes per wavefront,
// each with its own LDS region; reductions stay inside the S lanes.
constexpr int kUnitsK = 8;        // units, and row segments, per lane

template <typename T, int BITS, int NW>
__global__ void __launch_bounds__(NW ? 64 * NW : 64) compress_units(UnitsArgs a) {
    constexpr bool SUB = NW == 0;
    constexpr int NT = SUB ? 64 : 64 * NW;
    constexpr int K = kUnitsK;
    constexpr float Lf = float((1 << BITS) - 1);
    constexpr uint32_t UB = 4 * sizeof(T);                                 // bytes of a unit in x
    typedef uint32_t raw_t __attribute__((ext_vector_type(sizeof(T))));     // a unit as loaded: 16 or 8 bytes
    const uint32_t tid = threadIdx.x;
    const uint32_t S = SUB ? a.S : (uint32_t)NT;                          // lanes per plane
    const uint32_t l = SUB ? tid & (S - 1u) : tid;                        // lane among them
    const uint32_t g = SUB ? tid >> a.S_log2 : 0u;                        // which plane of the round
    const uint32_t G = SUB ? 64u >> a.S_log2 : 1u;                        // planes per round
    extern __shared__ float4 smem4[];
    char* region = reinterpret_cast<char*>(smem4) + g * a.reg_bytes;
    float4* xs4 = reinterpret_cast<float4*>(region);                      // [q4p] the plane, later its residual
    float* xs = reinterpret_cast<float*>(region);
    double* rsum = reinterpret_cast<double*>(xs + 4 * a.q4p);             // [nitem] row-segment sums
    float* lfcs = reinterpret_cast<float*>(rsum + a.nitem);               // [nb + 1], last = NaN sentinel
    float* red = lfcs + ((a.nb + 1 + 3) & ~3u);                           // [2*NW] cross-wave min / max
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, tid);
    auto sync = [&]() { if constexpr (NW <= 1) wave_sync(); else lds_barrier(); };
    // rounds of units a plane has (uniform); units of the last round past the plane are worked on like
    // the others: they load zeros or a neighbour's elements and take the NaN sentinel
    auto round_live = [&](int k) -> bool { return S * (uint32_t)k < a.q4; };

    // 2-byte elements, odd planes of an odd element count: the plane starts in the middle of a dword.
    // Its loads then start one element early (every load stays dword-aligned and inside dwords that hold
    // elements of the map) and land in LDS one element lower.  The same for all planes a lane works on:
    // the grid is even or every workgroup has one plane (NW >= 1); a round is an even number of planes (NW = 0).
    const uint32_t shift = sizeof(T) == 2 ? ((blockIdx.x * G + g) * a.HW) & 1u : 0u;
    const uint32_t shift0 = SUB ? 0u : shift;                             // of the round's first plane

    // LDS byte offset of the LFC of each element's block (4 * nb = the sentinel for elements past the plane)
    uint32_t lo[K][2];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        uint32_t off[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t e = 4u * (l + S * k) + j;
            const uint32_t r = fdiv(e, a.d_W);
            const uint32_t c = e - r * a.W;
            off[j] = 4u * (e < a.HW ? fdiv(r, a.d_B) * a.LW + fdiv(c, a.d_B) : a.nb);
        }
        lo[k][0] = off[0] | (off[1] << 16);
        lo[k][1] = off[2] | (off[3] << 16);
    }
    // the row segments of the lane (item i = block * B + row of the block): where the segment starts in
    // the plane, and in the top bits how many elements it has (0: a row past the map, or no item)
    uint32_t it[K];
#pragma unroll
    for (int m = 0; m < K; ++m) {
        const uint32_t i = l + S * m;
        const uint32_t t = fdiv(i, a.d_B), rr = i - t * a.B;
        const uint32_t bi = fdiv(t, a.d_LW), bj = t - bi * a.LW;
        const uint32_t r = bi * a.B + rr;
        const uint32_t bw = min(a.B, a.W - bj * a.B);
        it[m] = (i < a.nitem && r < a.H) ? (r * a.W + bj * a.B) | (bw << 20) : 0u;
    }
    if (l == 0) lfcs[a.nb] = __builtin_nanf("");
    const uint32_t tail = a.HW & 3u;          // elements of the last unit inside the plane (0: all four)

    // the loads of a round of planes: coalesced, all in flight at once; dwords past the round's last
    // plane read as zero
    raw_t q[K];
    auto issue_loads = [&](uint32_t rd) {
        const uint32_t pf = rd * G;                                      // the round's first plane
        const uint32_t np = min(G, a.P - pf);
        const T* src = static_cast<const T*>(pt.x) + ((size_t)pf * a.HW - shift0);
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<T*>(src), 0, (int)((((np * a.HW + shift0) * sizeof(T)) + 3u) & ~3u), 0x00020000);
        const uint32_t voff = (g * a.HW - (shift - shift0)) * (uint32_t)sizeof(T) + l * UB;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (!round_live(k)) continue;
            if constexpr (sizeof(T) == 4) q[k] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, (int)(S * k * UB), kLoadAux);
            else q[k] = __builtin_amdgcn_raw_buffer_load_b64(rsrc, voff, (int)(S * k * UB), kLoadAux);
        }
    };

    // a workgroup takes rounds blockIdx.x, blockIdx.x + gridDim.x, ...: the tables above are made once
    if (blockIdx.x < a.nrounds) issue_loads(blockIdx.x);
    for (uint32_t rd = blockIdx.x; rd < a.nrounds; rd += gridDim.x) {
        const uint32_t p = rd * G + g;
        const bool pv = p < a.P;                                          // (NW = 0) the last round may have fewer planes
        // ---- park the plane in LDS as fp32, then start the next round's loads: they fly while this one is worked on
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (!round_live(k)) continue;
            float4 v;
            if constexpr (sizeof(T) == 4) {
                v = make_float4(__uint_as_float(q[k].x), __uint_as_float(q[k].y), __uint_as_float(q[k].z), __uint_as_float(q[k].w));
            } else {
                v = make_float4(__uint_as_float(q[k].x << 16), __uint_as_float(q[k].x & 0xffff0000u),
                                __uint_as_float(q[k].y << 16), __uint_as_float(q[k].y & 0xffff0000u));
            }
            if (sizeof(T) == 2 && shift) {
                float* d = xs + 4u * (l + S * k);
                if (l + S * k != 0) d[-1] = v.x;
                d[0] = v.y; d[1] = v.z; d[2] = v.w;
            } else {
                xs4[l + S * k] = v;
            }
        }
        if (rd + gridDim.x < a.nrounds) issue_loads(rd + gridDim.x);
        sync();

        // ---- Sec. 4.1 AveragePooling, step 1: a lane per (block, row) adds the row's elements inside the block
#pragma unroll
        for (int m = 0; m < K; ++m) {
            if (S * (uint32_t)m >= a.nitem) continue;
            const uint32_t bw = it[m] >> 20;
            const float* src = xs + (it[m] & 0xfffffu);
            double Sr = 0.0;
            uint32_t c = 0;
            for (; c + 8 <= bw; c += 8) {
                float v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = src[c + j];
#pragma unroll
                for (int j = 0; j < 8; ++j) Sr += (double)v[j];
            }
            if (c + 4 <= bw) {
                const float v0 = src[c], v1 = src[c + 1], v2 = src[c + 2], v3 = src[c + 3];
                Sr += (double)v0; Sr += (double)v1; Sr += (double)v2; Sr += (double)v3;
                c += 4;
            }
            for (; c < bw; ++c) Sr += (double)src[c];
            if (l + S * m < a.nitem) rsum[l + S * m] = Sr;
        }
        sync();

        // ---- step 2: a lane per block adds its rows from the top down
        for (uint32_t t = l; t < a.nb; t += S) {
            const uint32_t bi = fdiv(t, a.d_LW), bj = t - bi * a.LW;
            const uint32_t rows = min(a.B, a.H - bi * a.B);
            const uint32_t bw = min(a.B, a.W - bj * a.B);
            double Sb = 0.0;
            for (uint32_t rr = 0; rr < rows; ++rr) Sb += rsum[t * a.B + rr];
            const float lfc = lfc_round<T>(mean_of(Sb, rows * bw), kC16<T>);
            lfcs[t] = lfc;
            if (pv) lfc_store<T>(pt.lfc, (size_t)p * a.nb + t, lfc, kC16<T>);
        }
        sync();

        // ---- residual H^H = H - UpSampling(H^L), written back over the plane; plane min / max (NaN
        // residuals of elements past the plane are skipped by min / max)
        float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (!round_live(k)) continue;
            const char* lb = reinterpret_cast<const char*>(lfcs);
            float4 v = xs4[l + S * k];
            v.x -= *reinterpret_cast<const float*>(lb + (lo[k][0] & 0xffffu));
            v.y -= *reinterpret_cast<const float*>(lb + (lo[k][0] >> 16));
            v.z -= *reinterpret_cast<const float*>(lb + (lo[k][1] & 0xffffu));
            v.w -= *reinterpret_cast<const float*>(lb + (lo[k][1] >> 16));
            xs4[l + S * k] = v;
            mn = fminf(fminf(mn, v.x), fminf(v.y, fminf(v.z, v.w)));
            mx = fmaxf(fmaxf(mx, v.x), fmaxf(v.y, fmaxf(v.z, v.w)));
        }
        if constexpr (SUB) {
            group_minmax(S, mn, mx);
        } else {
            group_minmax(64, mn, mx);
            if constexpr (NW > 1) {
                if ((tid & 63u) == 0) { red[2 * (tid >> 6)] = mn; red[2 * (tid >> 6) + 1] = mx; }
                lds_barrier();
#pragma unroll
                for (int w = 0; w < NW; ++w) { mn = fminf(mn, red[2 * w]); mx = fmaxf(mx, red[2 * w + 1]); }
            }
        }

        // ---- scale of Eq. (quantization), keys, meta
        float delta, Delta, inv;
        plane_scale_any(mn, mx, Lf, kC16<T>, delta, Delta, inv);
        const float invs = inv * (float)(1u << (32 - BITS));
        const uint32_t k1 = mix32(p ^ pt.seed_a);
        const uint32_t k2 = mix32(k1 + pt.seed_c);
        if (l == 0 && pv) meta_store(pt.meta, p, delta, Delta, kC16<T>);

        // ---- Quant + packing: a unit is two element pairs = 4 codes; a lane reads back the residuals it wrote
        {
            const uint32_t rscale = 1u << (16 - BITS);
            constexpr uint32_t CB = BITS / 2;                         // code bytes per unit (1, 2 or 4)
            // NW >= 1: the buffer ends with the plane's last unit, so that stores of units past the plane
            // are dropped; NW = 0: it ends with the round's last plane, units past a plane are skipped
            const uint32_t pf = rd * G;
            uint8_t* cround = reinterpret_cast<uint8_t*>(pt.codes) + (size_t)pf * a.WPP * 4;
            const __amdgpu_buffer_rsrc_t crs = __builtin_amdgcn_make_buffer_rsrc(
                cround, 0, (int)(SUB ? min(G, a.P - pf) * a.WPP * 4u : a.q4 * CB), 0x00020000);
            const uint32_t cvoff = g * a.WPP * 4u + l * CB;
            const uint32_t xw0 = k1 + (2u * l) * kWeyl;
            const uint32_t tailmask = tail ? (1u << (tail * BITS)) - 1u : 0xffffffffu;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                if (!round_live(k)) continue;
                const float4 v = xs4[l + S * k];
                const uint32_t xw = xw0 + (2u * S * (uint32_t)k) * kWeyl;
                uint32_t c = push_pair<BITS>(0u, v.z, v.w, delta, invs, xw + kWeyl, k2, rscale);
                c = push_pair<BITS>(c, v.x, v.y, delta, invs, xw, k2, rscale);
                // the last unit's elements past the plane leave zero bits
                if (l + S * k + 1 == a.q4) c &= tailmask;
                if (SUB && l + S * k >= a.q4) continue;
                if constexpr (CB == 1) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)c, crs, cvoff, (int)(S * k), 0);
                else if constexpr (CB == 2) __builtin_amdgcn_raw_buffer_store_b16((uint16_t)c, crs, cvoff, (int)(S * k * 2), 0);
                else __builtin_amdgcn_raw_buffer_store_b32(c, crs, cvoff, (int)(S * k * 4), 0);
            }
            // pad bytes of the plane's last word are zero
            const uint32_t padb = a.WPP * 4 - a.q4 * CB;
            if (l < padb && pv) cround[(size_t)g * a.WPP * 4 + a.q4 * CB + l] = 0;
        }
        sync();      // xs, rsum, lfcs and red are reused
    }
}

// the elements of one 16-byte vector of x as fp32
template <typename T>
__device__ __forceinline__ void unpack_vec(const u32x4& q, float (&x)[16 / sizeof(T)]) {
    if constexpr (sizeof(T) == 4) {
        x[0] = __uint_as_float(q.x); x[1] = __uint_as_float(q.y); x[2] = __uint_as_float(q.z); x[3] = __uint_as_float(q.w);
    } else {
        x[0] = __uint_as_float(q.x << 16); x[1] = __uint_as_float(q.x & 0xffff0000u);
        x[2] = __uint_as_float(q.y << 16); x[3] = __uint_as_float(q.y & 0xffff0000u);
        x[4] = __uint_as_float(q.z << 16); x[5] = __uint_as_float(q.z & 0xffff0000u);
        x[6] = __uint_as_float(q.w << 16); x[7] = __uint_as_float(q.w & 0xffff0000u);
    }
}

// ------------------------------------------------------------------ compress, planes that are one block

struct OneArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, HW, WPP;
    uint32_t qv;         // 16-byte vectors per plane
    uint32_t S, S_log2;  // lanes per plane (power of two, at most 64)
    uint32_t ppw;        // planes per wavefront = 64 / S
    uint32_t upb, upb_log2;  // compress_line: vectors per block (power of two, at most S); nb = blocks per plane
    uint32_t nb;
};

constexpr int kOneUnits = 13;     // vectors per lane: planes of up to 13 * 64 vectors

// sum over aligned groups of S lanes (S a power of two <= 64, uniform in the wave) in a fixed
// order, result in every lane of the group; all lanes must be active
__device__ __forceinline__ double group_sum_any(uint32_t S, double v) {
    if (S >= 2)  v += dpp_f64<kDppXor1>(v);
    if (S >= 4)  v += dpp_f64<kDppXor2>(v);
    if (S >= 8)  v += dpp_f64<kDppHalfMirror>(v);
    if (S >= 16) v += dpp_f64<kDppMirror>(v);
    if (S >= 32) {
        const uint64_t u = (uint64_t)__double_as_longlong(v);
        const int lo = (int)(uint32_t)u, hi = (int)(uint32_t)(u >> 32);
        auto row = [&](int lane) -> double {
            const uint32_t l = (uint32_t)__builtin_amdgcn_readlane(lo, lane), h = (uint32_t)__builtin_amdgcn_readlane(hi, lane);
            return __longlong_as_double((long long)(((uint64_t)h << 32) | l));
        };
        const double r0 = row(0), r1 = row(16), r2 = row(32), r3 = row(48);
        if (S == 64) v = (r0 + r1) + (r2 + r3);
        else v = (threadIdx.x & 32u) ? r2 + r3 : r0 + r1;
    }
    return v;
}

// The block covers the whole plane (B at least every extent of the map: the later layers of a
// network, or a block size like 64 on maps of 56 x 56 and below): H^L is the plane's mean, rows
// and columns play no part, and the plane is a flat run of 16-byte vectors.  One wavefront per
// 64 / S planes; the S lanes of a plane keep its vectors in registers (vector u in lane u mod S),
// sums and extremes are reductions over those lanes, the codes leave as one to eight bytes per
// vector.  LDS is not used.
template <typename T, int BITS>
__global__ void __launch_bounds__(64) compress_one(OneArgs a) {
    constexpr int K = kOneUnits;
    constexpr uint32_t EPV = 16 / sizeof(T);
    constexpr uint32_t CBV = EPV * BITS / 8;
    constexpr float Lf = float((1 << BITS) - 1);
    const uint32_t tid = threadIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, tid);
    const uint32_t sub = tid & (a.S - 1u);
    const uint32_t p = blockIdx.x * a.ppw + (tid >> a.S_log2);
    const bool live = p < a.P;
    const uint32_t pc = live ? p : a.P - 1u;          // lanes past the last plane redo it; their stores are masked
    const u32x4* src = reinterpret_cast<const u32x4*>(static_cast<const T*>(pt.x) + (size_t)pc * a.HW);

    u32x4 q[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t u = sub + (uint32_t)k * a.S;
        if (u < a.qv) q[k] = __builtin_nontemporal_load(src + u);
    }
    // ---- Sec. 4.1 AveragePooling with one window: the mean of the plane
    double S = 0.0;
    float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t u = sub + (uint32_t)k * a.S;
        if (u < a.qv) {
            float f[EPV];
            unpack_vec<T>(q[k], f);
            double s4 = ((double)f[0] + (double)f[1]) + ((double)f[2] + (double)f[3]);
            mn = fminf(mn, fminf(fminf(f[0], f[1]), fminf(f[2], f[3])));
            mx = fmaxf(mx, fmaxf(fmaxf(f[0], f[1]), fmaxf(f[2], f[3])));
            if constexpr (EPV == 8) {
                s4 += ((double)f[4] + (double)f[5]) + ((double)f[6] + (double)f[7]);
                mn = fminf(mn, fminf(fminf(f[4], f[5]), fminf(f[6], f[7])));
                mx = fmaxf(mx, fmaxf(fmaxf(f[4], f[5]), fmaxf(f[6], f[7])));
            }
            S += s4;
        }
    }
    S = group_sum_any(a.S, S);
    const float lfc = lfc_round<T>(mean_of(S, a.HW), kC16<T>);
    // ---- extremes of the residual (x -> fl(x - m) is monotone), scale of Eq. (quantization), keys
    mn = mn - lfc;
    mx = mx - lfc;
    group_minmax(a.S, mn, mx);
    float delta, Delta, inv;
    plane_scale_any(mn, mx, Lf, kC16<T>, delta, Delta, inv);
    const float invs = inv * (float)(1u << (32 - BITS));
    const uint32_t k1 = mix32(pc ^ pt.seed_a);
    const uint32_t k2 = mix32(k1 + pt.seed_c);
    uint8_t* cbase = reinterpret_cast<uint8_t*>(pt.codes) + (size_t)pc * a.WPP * 4;
    if (live && sub == 0) {
        meta_store(pt.meta, p, delta, Delta, kC16<T>);
        lfc_store<T>(pt.lfc, (size_t)p, lfc, kC16<T>);
        const uint32_t padb = a.WPP * 4 - a.qv * CBV;                 // pad bytes of the last word are zero
        for (uint32_t t = 0; t < padb; ++t) cbase[a.qv * CBV + t] = 0;
    }
    // ---- residual, Quant, packing
    const uint32_t rscale = 1u << (16 - BITS);
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t u = sub + (uint32_t)k * a.S;
        if (live && u < a.qv) {
            float h[EPV];
            unpack_vec<T>(q[k], h);
#pragma unroll
            for (uint32_t e = 0; e < EPV; ++e) h[e] = h[e] - lfc;
            const uint32_t xw0 = k1 + (u * (EPV / 2)) * kWeyl;
            uint8_t* dst = cbase + u * CBV;
            if constexpr (CBV <= 4) {
                uint32_t c = 0;
#pragma unroll
                for (int j = EPV / 2 - 1; j >= 0; --j)
                    c = push_pair<BITS>(c, h[2 * j], h[2 * j + 1], delta, invs, xw0 + (uint32_t)j * kWeyl, k2, rscale);
                if constexpr (CBV == 1) *dst = (uint8_t)c;
                else if constexpr (CBV == 2) *reinterpret_cast<uint16_t*>(dst) = (uint16_t)c;
                else *reinterpret_cast<uint32_t*>(dst) = c;
            } else {
                uint32_t lo = 0, hi = 0;
                hi = push_pair<BITS>(hi, h[6], h[7], delta, invs, xw0 + 3u * kWeyl, k2, rscale);
                hi = push_pair<BITS>(hi, h[4], h[5], delta, invs, xw0 + 2u * kWeyl, k2, rscale);
                lo = push_pair<BITS>(lo, h[2], h[3], delta, invs, xw0 + kWeyl, k2, rscale);
                lo = push_pair<BITS>(lo, h[0], h[1], delta, invs, xw0, k2, rscale);
                reinterpret_cast<uint32_t*>(dst)[0] = lo;
                reinterpret_cast<uint32_t*>(dst)[1] = hi;
            }
        }
    }
}

// 1-D maps (Appendix D, AveragePooling1D: Minibatch x Channel x N, the maps of linear and
// transformer layers) whose block is a power-of-two number of 16-byte vectors (B = 4, 8, 16, 32, 64
// for fp32): laid out like compress_one, the `upb` vectors of a block sit in neighbouring lanes of
// one round, so a block's sum is a DPP reduction over those lanes and its LFC stays in a register.
// No LDS.
template <typename T, int BITS>
__global__ void __launch_bounds__(64) compress_line(OneArgs a) {
    constexpr int K = kOneUnits;
    constexpr uint32_t EPV = 16 / sizeof(T);
    constexpr uint32_t CBV = EPV * BITS / 8;
    constexpr float Lf = float((1 << BITS) - 1);
    const uint32_t tid = threadIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, tid);
    const uint32_t sub = tid & (a.S - 1u);
    const uint32_t p = blockIdx.x * a.ppw + (tid >> a.S_log2);
    const bool live = p < a.P;
    const uint32_t pc = live ? p : a.P - 1u;          // lanes past the last plane redo it; their stores are masked
    const u32x4* src = reinterpret_cast<const u32x4*>(static_cast<const T*>(pt.x) + (size_t)pc * a.HW);

    u32x4 q[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t u = sub + (uint32_t)k * a.S;
        if (u < a.qv) q[k] = __builtin_nontemporal_load(src + u);
    }
    // ---- AveragePooling1D: block sums over the lanes of a block, residual extremes of the plane
    float lfcv[K];
    float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
    for (int k = 0; k < K; ++k) {
        if ((uint32_t)k * a.S >= a.qv) { lfcv[k] = 0.0f; continue; }          // uniform: no vector of this round exists
        const uint32_t u = sub + (uint32_t)k * a.S;
        const bool valid = u < a.qv;
        float f[EPV];
        double s4 = 0.0;
        if (valid) {
            unpack_vec<T>(q[k], f);
            s4 = ((double)f[0] + (double)f[1]) + ((double)f[2] + (double)f[3]);
            if constexpr (EPV == 8) s4 += ((double)f[4] + (double)f[5]) + ((double)f[6] + (double)f[7]);
        }
        const double Sb = group_sum_any(a.upb, s4);
        const uint32_t ustart = u & ~(a.upb - 1u);
        const uint32_t nvec = valid ? min(a.upb, a.qv - ustart) : 1u;           // the last block may be short
        const float lfc = lfc_round<T>(mean_of(Sb, nvec * EPV), kC16<T>);
        lfcv[k] = lfc;
        if (valid) {
#pragma unroll
            for (uint32_t e = 0; e < EPV; ++e) {
                const float h = f[e] - lfc;
                mn = fminf(mn, h);
                mx = fmaxf(mx, h);
            }
            if (live && u == ustart) lfc_store<T>(pt.lfc, (size_t)p * a.nb + (u >> a.upb_log2), lfc, kC16<T>);
        }
    }
    group_minmax(a.S, mn, mx);
    float delta, Delta, inv;
    plane_scale_any(mn, mx, Lf, kC16<T>, delta, Delta, inv);
    const float invs = inv * (float)(1u << (32 - BITS));
    const uint32_t k1 = mix32(pc ^ pt.seed_a);
    const uint32_t k2 = mix32(k1 + pt.seed_c);
    uint8_t* cbase = reinterpret_cast<uint8_t*>(pt.codes) + (size_t)pc * a.WPP * 4;
    if (live && sub == 0) {
        meta_store(pt.meta, p, delta, Delta, kC16<T>);
        const uint32_t padb = a.WPP * 4 - a.qv * CBV;                 // pad bytes of the last word are zero
        for (uint32_t t = 0; t < padb; ++t) cbase[a.qv * CBV + t] = 0;
    }
    // ---- residual, Quant, packing
    const uint32_t rscale = 1u << (16 - BITS);
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t u = sub + (uint32_t)k * a.S;
        if (live && u < a.qv) {
            float h[EPV];
            unpack_vec<T>(q[k], h);
#pragma unroll
            for (uint32_t e = 0; e < EPV; ++e) h[e] = h[e] - lfcv[k];
            const uint32_t xw0 = k1 + (u * (EPV / 2)) * kWeyl;
            uint8_t* dst = cbase + u * CBV;
            if constexpr (CBV <= 4) {
                uint32_t c = 0;
#pragma unroll
                for (int j = EPV / 2 - 1; j >= 0; --j)
                    c = push_pair<BITS>(c, h[2 * j], h[2 * j + 1], delta, invs, xw0 + (uint32_t)j * kWeyl, k2, rscale);
                if constexpr (CBV == 1) *dst = (uint8_t)c;
                else if constexpr (CBV == 2) *reinterpret_cast<uint16_t*>(dst) = (uint16_t)c;
                else *reinterpret_cast<uint32_t*>(dst) = c;
            } else {
                uint32_t lo = 0, hi = 0;
                hi = push_pair<BITS>(hi, h[6], h[7], delta, invs, xw0 + 3u * kWeyl, k2, rscale);
                hi = push_pair<BITS>(hi, h[4], h[5], delta, invs, xw0 + 2u * kWeyl, k2, rscale);
                lo = push_pair<BITS>(lo, h[2], h[3], delta, invs, xw0 + kWeyl, k2, rscale);
                lo = push_pair<BITS>(lo, h[0], h[1], delta, invs, xw0, k2, rscale);
                reinterpret_cast<uint32_t*>(dst)[0] = lo;
                reinterpret_cast<uint32_t*>(dst)[1] = hi;
            }
        }
    }
}

// ------------------------------------------------------------------ compress, any block size, chunk in LDS

struct RowsArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, H, W, HW, LH, LW, nb, WPP, B;      // H, LH: rows / block rows over all depth slices of a 3-D map
    uint32_t D, Hs, LHs; // depth, rows and block rows of one depth slice (D = 1, Hs = H, LHs = LH for a 2-D map)
    uint32_t G;          // planes per workgroup
    uint32_t xs_floats;  // LDS floats reserved for the chunk (multiple of 4, + slack for ragged last words)
    uint32_t vec_load;   // chunk starts are 16-byte aligned
    uint32_t keep;       // the chunk is at most kRowsKeep 16-byte vectors per lane, each inside one row: lanes keep what they load
    uint32_t vecblk;     // keep, and the block size is a multiple of the vector too: a vector lies in one block
    uint32_t qv;         // 16-byte vectors per plane (when keep)
    FastDiv d_W, d_B, d_LW, d_HLW, d_nb, d_wpp, d_Hs, d_LHs, d_qv;
};

constexpr int kRowsKeep = 13;     // 16-byte vectors a lane of compress_rows holds in registers

// One 16-byte vector of x (EPV consecutive elements of one row: W is a multiple of EPV) -> its
// EPV * BITS / 8 code bytes.  f = vector index inside the plane, lp = the plane's LFC values (LDS),
// pr = (delta, scaled inv, k1, k2) of the plane, plane_codes = the plane's packed words.
// Args carries W, LW, Hs, LHs and the dividers d_W, d_B, d_Hs.
template <typename T, int BITS, int ND, typename Args>
__device__ __forceinline__ void quant_vector(const Args& a, const u32x4& q, uint32_t f, const float4 pr, const float* lp,
                                             uint8_t* plane_codes) {
    constexpr uint32_t EPV = 16 / sizeof(T);
    constexpr uint32_t CBV = EPV * BITS / 8;
    const uint32_t rscale = 1u << (16 - BITS);
    const uint32_t k1 = __float_as_uint(pr.z), k2 = __float_as_uint(pr.w);
    float h[EPV];
    unpack_vec<T>(q, h);
    const uint32_t i0 = f * EPV;
    const uint32_t r = fdiv(i0, a.d_W);                  // row, counted over all depth slices of a 3-D map
    const uint32_t c0 = i0 - r * a.W;
    uint32_t brow;
    if constexpr (ND == 3) {
        const uint32_t z = fdiv(r, a.d_Hs);
        brow = fdiv(z, a.d_B) * a.LHs + fdiv(r - z * a.Hs, a.d_B);
    } else {
        brow = fdiv(r, a.d_B);
    }
    const float* lrow = lp + brow * a.LW;
#pragma unroll
    for (uint32_t e = 0; e < EPV; ++e) h[e] = h[e] - lrow[fdiv(c0 + e, a.d_B)];
    const uint32_t xw0 = k1 + (f * (EPV / 2)) * kWeyl;
    uint8_t* dst = plane_codes + f * CBV;
    if constexpr (CBV <= 4) {
        uint32_t c = 0;
#pragma unroll
        for (int j = EPV / 2 - 1; j >= 0; --j)
            c = push_pair<BITS>(c, h[2 * j], h[2 * j + 1], pr.x, pr.y, xw0 + (uint32_t)j * kWeyl, k2, rscale);
        if constexpr (CBV == 1) *dst = (uint8_t)c;
        else if constexpr (CBV == 2) *reinterpret_cast<uint16_t*>(dst) = (uint16_t)c;
        else *reinterpret_cast<uint32_t*>(dst) = c;
    } else {
        // eight 8-bit codes: two words
        uint32_t lo = 0, hi = 0;
        hi = push_pair<BITS>(hi, h[6], h[7], pr.x, pr.y, xw0 + 3u * kWeyl, k2, rscale);
        hi = push_pair<BITS>(hi, h[4], h[5], pr.x, pr.y, xw0 + 2u * kWeyl, k2, rscale);
        lo = push_pair<BITS>(lo, h[2], h[3], pr.x, pr.y, xw0 + kWeyl, k2, rscale);
        lo = push_pair<BITS>(lo, h[0], h[1], pr.x, pr.y, xw0, k2, rscale);
        reinterpret_cast<uint32_t*>(dst)[0] = lo;
        reinterpret_cast<uint32_t*>(dst)[1] = hi;
    }
}

// Any block size B (the paper's sweep uses 12, 16, 18 and 64 besides 8).  A workgroup of four
// wavefronts stages a chunk of G planes in LDS with coalesced loads, then
//   1. a lane per (row, block column): binary64 sum, min and max of that row segment;
//   2. a lane per block: adds its rows' partial sums in row order -> LFC, and the extremes of the
//      block's residual (x -> fl(x - m) is monotone, so they are fl(min x - m), fl(max x - m));
//   3. a lane per plane: min / max over its blocks, scale, keys, meta;
//   4. a lane per packed word: residual against the block's LFC, quantise, pack.
// When rows are whole 16-byte vectors and the chunk is at most kRowsKeep of them per lane (the usual
// case) the lanes keep the vectors they loaded in registers and step 4 runs on those: a vector's
// codes leave as one to eight bytes, and x is read from LDS by the pooling steps only.
// ND = 3: the plane is a 3-D map (Appendix D) of D slices of Hs rows, blocks of B x B x B; its D*Hs
// rows are staged and summed as rows like those of a 2-D map, a block adds the rows of its B slices.
template <typename T, int BITS, int ND>
__device__ __forceinline__ void compress_rows_body(const RowsArgs& a) {
    extern __shared__ float4 smem4[];
    float4* params = smem4;                                                   // [G] (delta, inv scaled, k1, k2)
    float* xs = reinterpret_cast<float*>(smem4 + a.G);                        // [xs_floats] the chunk as fp32
    float4* rowp = reinterpret_cast<float4*>(xs + a.xs_floats);               // [G*H*LW] (sum lo, sum hi, min, max)
    float* lfcs = reinterpret_cast<float*>(rowp + a.G * a.H * a.LW);          // [G*nb]
    float2* bext = reinterpret_cast<float2*>(lfcs + ((a.G * a.nb + 1u) & ~1u)); // [G*nb] residual extremes per block

    constexpr int CPW = 32 / BITS;
    constexpr int PPW = CPW / 2;
    constexpr float Lf = float((1 << BITS) - 1);
    const uint32_t tid = threadIdx.x;
    const uint32_t p0 = blockIdx.x * a.G;
    const uint32_t Gc = min(a.G, a.P - p0);
    const uint32_t n = Gc * a.HW;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, tid);

    // ---- chunk -> LDS (fp32): coalesced 16-byte loads, all of a lane's in flight at once (up to
    // kRowsKeep, kept for step 4) or eight at a time
    constexpr uint32_t EPV = 16 / sizeof(T);
    const uint32_t nv = a.vec_load ? n / EPV : 0;
    const bool keep = a.keep != 0;                      // uniform
    u32x4 kept[kRowsKeep];
    {
        const T* src = static_cast<const T*>(pt.x) + (size_t)p0 * a.HW;
        const u32x4* src4 = reinterpret_cast<const u32x4*>(src);
        auto to_lds = [&](const u32x4& q, uint32_t v) {
            if constexpr (sizeof(T) == 4) {
                reinterpret_cast<u32x4*>(xs)[v] = q;
            } else {
                float f[8];
                unpack_vec<T>(q, f);
                reinterpret_cast<float4*>(xs)[2 * v] = make_float4(f[0], f[1], f[2], f[3]);
                reinterpret_cast<float4*>(xs)[2 * v + 1] = make_float4(f[4], f[5], f[6], f[7]);
            }
        };
        if (keep) {
#pragma unroll
            for (int k = 0; k < kRowsKeep; ++k) {
                const uint32_t v = k * kThreads + tid;
                if (v < nv) kept[k] = __builtin_nontemporal_load(src4 + v);
            }
            if (a.vecblk) {
                // a vector lies inside one block: LDS takes its sum, min and max instead of its elements
#pragma unroll
                for (int k = 0; k < kRowsKeep; ++k) {
                    const uint32_t v = k * kThreads + tid;
                    if (v < nv) {
                        float f[EPV];
                        unpack_vec<T>(kept[k], f);
                        double S = ((double)f[0] + (double)f[1]) + ((double)f[2] + (double)f[3]);
                        float mn = fminf(fminf(f[0], f[1]), fminf(f[2], f[3]));
                        float mx = fmaxf(fmaxf(f[0], f[1]), fmaxf(f[2], f[3]));
                        if constexpr (EPV == 8) {
                            S += ((double)f[4] + (double)f[5]) + ((double)f[6] + (double)f[7]);
                            mn = fminf(mn, fminf(fminf(f[4], f[5]), fminf(f[6], f[7])));
                            mx = fmaxf(mx, fmaxf(fmaxf(f[4], f[5]), fmaxf(f[6], f[7])));
                        }
                        const uint64_t sb = (uint64_t)__double_as_longlong(S);
                        reinterpret_cast<float4*>(xs)[v] =
                            make_float4(__uint_as_float((uint32_t)sb), __uint_as_float((uint32_t)(sb >> 32)), mn, mx);
                    }
                }
            } else {
#pragma unroll
                for (int k = 0; k < kRowsKeep; ++k) {
                    const uint32_t v = k * kThreads + tid;
                    if (v < nv) to_lds(kept[k], v);
                }
            }
        } else {
            constexpr int U = 8;
            for (uint32_t v0 = 0; v0 < nv; v0 += U * kThreads) {
                u32x4 q[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint32_t v = v0 + u * kThreads + tid;
                    if (v < nv) q[u] = __builtin_nontemporal_load(src4 + v);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint32_t v = v0 + u * kThreads + tid;
                    if (v < nv) to_lds(q[u], v);
                }
            }
            for (uint32_t e = nv * EPV + tid; e < n; e += kThreads) xs[e] = Elem<T>::load(src, e);
        }
    }
    lds_barrier();

    // ---- 1. row segments (Sec. 4.1 AveragePooling, first half)
    const uint32_t HLW = a.H * a.LW;
    for (uint32_t s = tid; s < Gc * HLW; s += kThreads) {
        const uint32_t g = fdiv(s, a.d_HLW);
        const uint32_t rem = s - g * HLW;
        const uint32_t r = fdiv(rem, a.d_LW);
        const uint32_t bj = rem - r * a.LW;
        const uint32_t c0 = bj * a.B;
        const uint32_t cols = min(a.B, a.W - c0);
        double S = 0.0;
        float mn = __builtin_inff(), mx = -__builtin_inff();
        if (a.vecblk) {
            // the segment is whole vectors: add their sums
            const float4* rec = reinterpret_cast<const float4*>(xs) + (g * a.HW + r * a.W + c0) / EPV;
            for (uint32_t u = 0; u < cols / EPV; ++u) {
                const float4 q = rec[u];
                S += __longlong_as_double((long long)(((uint64_t)__float_as_uint(q.y) << 32) | __float_as_uint(q.x)));
                mn = fminf(mn, q.z);
                mx = fmaxf(mx, q.w);
            }
        } else {
            const float* row = xs + g * a.HW + r * a.W + c0;
            for (uint32_t c = 0; c < cols; ++c) {
                const float v = row[c];
                S += (double)v;
                mn = fminf(mn, v);
                mx = fmaxf(mx, v);
            }
        }
        const uint64_t sb = (uint64_t)__double_as_longlong(S);
        rowp[s] = make_float4(__uint_as_float((uint32_t)sb), __uint_as_float((uint32_t)(sb >> 32)), mn, mx);
    }
    lds_barrier();

    // ---- 2. blocks: LFC and the extremes of the block's residual.  All lanes of a wavefront run
    // the loop body (mean_of votes across the wavefront); slots past the chunk redo block 0.
    const uint32_t nblk = Gc * a.nb;
    for (uint32_t t0 = 0; t0 < nblk; t0 += kThreads) {
        const uint32_t t = t0 + tid;
        const bool live = t < nblk;
        const uint32_t tt = live ? t : 0u;
        const uint32_t g = fdiv(tt, a.d_nb);
        const uint32_t blk = tt - g * a.nb;
        const uint32_t bq = fdiv(blk, a.d_LW);                  // block row, counted over all depth slices
        const uint32_t bj = blk - bq * a.LW;
        uint32_t bd = 0, bi = bq;
        if constexpr (ND == 3) { bd = fdiv(bq, a.d_LHs); bi = bq - bd * a.LHs; }
        const uint32_t r0 = bi * a.B;
        const uint32_t rows = min(a.B, a.Hs - r0);
        const uint32_t cols = min(a.B, a.W - bj * a.B);
        const uint32_t z0 = bd * a.B;
        const uint32_t deps = ND == 3 ? min(a.B, a.D - z0) : 1u;
        double S = 0.0;
        float mn = __builtin_inff(), mx = -__builtin_inff();
        for (uint32_t z = 0; z < deps; ++z) {
            const float4* rp = rowp + g * HLW + ((z0 + z) * a.Hs + r0) * a.LW + bj;
#pragma unroll 4
            for (uint32_t rr = 0; rr < rows; ++rr) {
                const float4 q = rp[rr * a.LW];
                S += __longlong_as_double((long long)(((uint64_t)__float_as_uint(q.y) << 32) | __float_as_uint(q.x)));
                mn = fminf(mn, q.z);
                mx = fmaxf(mx, q.w);
            }
        }
        const float lfc = lfc_round<T>(mean_of(S, deps * rows * cols), kC16<T>);
        if (live) {
            lfcs[t] = lfc;
            lfc_store<T>(pt.lfc, (size_t)p0 * a.nb + t, lfc, kC16<T>);
            bext[t] = make_float2(mn - lfc, mx - lfc);
        }
    }
    lds_barrier();

    // ---- 3. planes: scale of Eq. (quantization), keys, meta.  Sixteen lanes share a plane's blocks.
    for (uint32_t g0 = 0; g0 < Gc; g0 += kThreads / 16) {
        const uint32_t g = g0 + (tid >> 4);
        float mn = __builtin_inff(), mx = -__builtin_inff();
        if (g < Gc) {
            for (uint32_t j = tid & 15u; j < a.nb; j += 16) {
                const float2 e = bext[g * a.nb + j];
                mn = fminf(mn, e.x);
                mx = fmaxf(mx, e.y);
            }
        }
        group_minmax(16, mn, mx);
        if (g >= Gc || (tid & 15u) != 0) continue;
        float delta, Delta, inv;
        plane_scale_any(mn, mx, Lf, kC16<T>, delta, Delta, inv);
        const uint32_t p = p0 + g;
        const uint32_t k1 = mix32(p ^ pt.seed_a);
        const uint32_t k2 = mix32(k1 + pt.seed_c);
        meta_store(pt.meta, p, delta, Delta, kC16<T>);
        params[g] = make_float4(delta, inv * (float)(1u << (32 - BITS)), __uint_as_float(k1), __uint_as_float(k2));
    }
    lds_barrier();

    // ---- 4. residual, Quant of Eq. (quantization), packing: one word per lane and step.
    // Adjacent lanes own adjacent words, CPW floats apart in LDS: were all lanes to read their
    // k-th pair at once they would meet in 64 / CPW banks.  Lane l therefore starts at pair
    // `rot` = (l / (64 / CPW)) mod PPW and goes round its word; the pairs are pushed in that
    // cyclic order and the word is rotated into place at the end.
    const uint32_t rscale = 1u << (16 - BITS);
    if (keep) {
        // the lane's own vectors: EPV consecutive elements of one plane each, EPV * BITS / 8 code bytes
        constexpr uint32_t CBV = EPV * BITS / 8;
        uint8_t* cbase = reinterpret_cast<uint8_t*>(pt.codes) + (size_t)p0 * a.WPP * 4;
#pragma unroll
        for (int k = 0; k < kRowsKeep; ++k) {
            const uint32_t v = k * kThreads + tid;
            if (v < nv) {
                const uint32_t g = fdiv(v, a.d_qv);
                const uint32_t f = v - g * a.qv;                 // vector index inside the plane
                quant_vector<T, BITS, ND>(a, kept[k], f, params[g], lfcs + g * a.nb, cbase + (size_t)g * a.WPP * 4);
            }
        }
        // pad bytes of every plane's last word are zero
        const uint32_t padb = a.WPP * 4 - a.qv * CBV;
        for (uint32_t t = tid; t < Gc * padb; t += kThreads) {
            const uint32_t g = t / padb;
            cbase[(size_t)g * a.WPP * 4 + a.qv * CBV + (t - g * padb)] = 0;
        }
        return;
    }
    const uint32_t nwords = Gc * a.WPP;
    const uint32_t rot = (tid / (64u / CPW)) & (uint32_t)(PPW - 1);
    for (uint32_t wi = tid; wi < nwords; wi += kThreads) {
        const uint32_t g = fdiv(wi, a.d_wpp);
        const uint32_t k = wi - g * a.WPP;
        const float4 pr = params[g];
        const uint32_t k1 = __float_as_uint(pr.z), k2 = __float_as_uint(pr.w);
        const uint32_t e0 = k * CPW;
        const uint32_t left = a.HW - e0;                       // elements of the plane from e0 on (>= 1)
        const float* xp = xs + g * a.HW;
        const float* lp = lfcs + g * a.nb;
        const uint32_t xw0 = k1 + (k * PPW) * kWeyl;
        uint32_t word = 0;
#pragma unroll
        for (int t = PPW - 1; t >= 0; --t) {
            const uint32_t j = (rot + (uint32_t)t) & (uint32_t)(PPW - 1);
            float h[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                // a ragged last word repeats the plane's last element; those codes are cleared below
                const uint32_t i = e0 + min(2u * j + (uint32_t)e, left - 1u);
                const uint32_t r = fdiv(i, a.d_W);
                const uint32_t c = i - r * a.W;
                uint32_t brow;
                if constexpr (ND == 3) {
                    const uint32_t z = fdiv(r, a.d_Hs);
                    brow = fdiv(z, a.d_B) * a.LHs + fdiv(r - z * a.Hs, a.d_B);
                } else {
                    brow = fdiv(r, a.d_B);
                }
                h[e] = xp[i] - lp[brow * a.LW + fdiv(c, a.d_B)];
            }
            word = push_pair<BITS>(word, h[0], h[1], pr.x, pr.y, xw0 + j * kWeyl, k2, rscale);
        }
        // pushed from pair rot+PPW-1 down to pair rot (mod PPW): pair rot sits in the low bits
        word = __builtin_amdgcn_alignbit(word, word, (32u - rot * 2u * BITS) & 31u);
        if (left < (uint32_t)CPW) word &= (1u << (left * BITS)) - 1u;          // pad bits are zero
        pt.codes[(size_t)(p0 + g) * a.WPP + k] = word;
    }
}

template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) compress_rows(RowsArgs a) { compress_rows_body<T, BITS, 2>(a); }
template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) compress_rows_3d(RowsArgs a) { compress_rows_body<T, BITS, 3>(a); }

// ------------------------------------------------------------------ compress, planes beyond LDS

struct PlaneArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, W, HW, LW, nb, WPP, B;
    uint32_t D, Hs, LHs;     // depth slices, rows and block rows of one slice (D = 1 for a 2-D map)
    uint32_t nitem;          // D * LHs * LW: blocks of one depth slice each
    uint32_t qv;             // 16-byte vectors per plane
    FastDiv d_W, d_B, d_Hs, d_LW, d_LHs, d_slice;      // d_slice divides by LHs * LW
};

// Planes too large for LDS (the 3-D maps of video models, 2-D maps from 200 x 200 up): one
// workgroup per plane, x is read twice, both times with 16-byte loads (rows and blocks are whole
// vectors here).
//   A. a lane per (depth slice, block): sum, min and max of the block's elements in that slice;
//      neighbouring lanes read neighbouring row segments;
//   B. a lane per block: adds its slices -> LFC (LDS and packed buffer), residual extremes;
//   C. range of the plane, scale of Eq. (quantization), keys, meta;
//   D. a lane per vector: residual against the LFC, Quant, code bytes out (the second read of x
//      comes out of the caches as far as they hold the plane).
template <typename T, int BITS, int ND>
__device__ __forceinline__ void compress_plane_body(const PlaneArgs& a) {
    extern __shared__ float4 smem4[];
    float4* part = smem4;                                          // [nitem] (sum lo, sum hi, min, max)
    float* lfcs = reinterpret_cast<float*>(part + a.nitem);       // [nb]
    float* red = lfcs + ((a.nb + 3u) & ~3u);                       // [2 * kThreads / 64] + 4 params
    constexpr uint32_t EPV = 16 / sizeof(T);
    constexpr uint32_t CBV = EPV * BITS / 8;
    constexpr float Lf = float((1 << BITS) - 1);
    const uint32_t tid = threadIdx.x;
    const uint32_t p = blockIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, tid);
    const u32x4* xv = reinterpret_cast<const u32x4*>(static_cast<const T*>(pt.x) + (size_t)p * a.HW);
    const uint32_t wv = a.W / EPV;                                 // vectors per row
    const uint32_t slice = a.LHs * a.LW;

    // ---- A. blocks of one slice (Sec. 4.1 / Appendix D AveragePooling, first half)
    for (uint32_t it = tid; it < a.nitem; it += kThreads) {
        const uint32_t z = fdiv(it, a.d_slice);
        const uint32_t rem = it - z * slice;
        const uint32_t bi = fdiv(rem, a.d_LW);
        const uint32_t bj = rem - bi * a.LW;
        const uint32_t r0 = bi * a.B, c0 = bj * a.B;
        const uint32_t rows = min(a.B, a.Hs - r0);
        const uint32_t nvec = min(a.B, a.W - c0) / EPV;
        const u32x4* src = xv + (size_t)(z * a.Hs + r0) * wv + c0 / EPV;
        double S = 0.0;
        float mn = __builtin_inff(), mx = -__builtin_inff();
        for (uint32_t rr = 0; rr < rows; ++rr) {
            for (uint32_t u = 0; u < nvec; ++u) {
                float f[EPV];
                unpack_vec<T>(src[(size_t)rr * wv + u], f);
                S += ((double)f[0] + (double)f[1]) + ((double)f[2] + (double)f[3]);
                mn = fminf(mn, fminf(fminf(f[0], f[1]), fminf(f[2], f[3])));
                mx = fmaxf(mx, fmaxf(fmaxf(f[0], f[1]), fmaxf(f[2], f[3])));
                if constexpr (EPV == 8) {
                    S += ((double)f[4] + (double)f[5]) + ((double)f[6] + (double)f[7]);
                    mn = fminf(mn, fminf(fminf(f[4], f[5]), fminf(f[6], f[7])));
                    mx = fmaxf(mx, fmaxf(fmaxf(f[4], f[5]), fmaxf(f[6], f[7])));
                }
            }
        }
        const uint64_t sb = (uint64_t)__double_as_longlong(S);
        part[it] = make_float4(__uint_as_float((uint32_t)sb), __uint_as_float((uint32_t)(sb >> 32)), mn, mx);
    }
    lds_barrier();

    // ---- B. blocks: LFC and residual extremes.  All lanes of a wavefront run the loop body
    // (mean_of votes across the wavefront); slots past the plane redo block 0.
    float mn = __builtin_inff(), mx = -__builtin_inff();
    for (uint32_t t0 = 0; t0 < a.nb; t0 += kThreads) {
        const uint32_t t = t0 + tid;
        const bool live = t < a.nb;
        const uint32_t blk = live ? t : 0u;
        const uint32_t bd = fdiv(blk, a.d_slice);
        const uint32_t rem = blk - bd * slice;
        const uint32_t bi = fdiv(rem, a.d_LW);
        const uint32_t bj = rem - bi * a.LW;
        const uint32_t rows = min(a.B, a.Hs - bi * a.B);
        const uint32_t cols = min(a.B, a.W - bj * a.B);
        const uint32_t z0 = bd * a.B;
        const uint32_t deps = min(a.B, a.D - z0);
        double S = 0.0;
        float bmn = __builtin_inff(), bmx = -__builtin_inff();
#pragma unroll 4
        for (uint32_t z = 0; z < deps; ++z) {
            const float4 q = part[(z0 + z) * slice + rem];
            S += __longlong_as_double((long long)(((uint64_t)__float_as_uint(q.y) << 32) | __float_as_uint(q.x)));
            bmn = fminf(bmn, q.z);
            bmx = fmaxf(bmx, q.w);
        }
        const float lfc = lfc_round<T>(mean_of(S, deps * rows * cols), kC16<T>);
        if (live) {
            lfcs[t] = lfc;
            lfc_store<T>(pt.lfc, (size_t)p * a.nb + t, lfc, kC16<T>);
            mn = fminf(mn, bmn - lfc);               // x -> fl(x - m) is monotone
            mx = fmaxf(mx, bmx - lfc);
        }
    }

    // ---- C. range of the plane, scale, keys, meta
    group_minmax(64, mn, mx);
    if ((tid & 63u) == 0) { red[2 * (tid >> 6)] = mn; red[2 * (tid >> 6) + 1] = mx; }
    lds_barrier();
    if (tid == 0) {
        for (uint32_t w = 0; w < kThreads / 64; ++w) { mn = fminf(mn, red[2 * w]); mx = fmaxf(mx, red[2 * w + 1]); }
        float delta, Delta, inv;
        plane_scale_any(mn, mx, Lf, kC16<T>, delta, Delta, inv);
        meta_store(pt.meta, p, delta, Delta, kC16<T>);
        const uint32_t k1 = mix32(p ^ pt.seed_a);
        const uint32_t k2 = mix32(k1 + pt.seed_c);
        float4* prm = reinterpret_cast<float4*>(red + 2 * (kThreads / 64));
        *prm = make_float4(delta, inv * (float)(1u << (32 - BITS)), __uint_as_float(k1), __uint_as_float(k2));
    }
    lds_barrier();
    const float4 pr = *reinterpret_cast<const float4*>(red + 2 * (kThreads / 64));

    // ---- D. residual, Quant, packing: a vector per lane and step, four steps in flight
    uint8_t* cbase = reinterpret_cast<uint8_t*>(pt.codes) + (size_t)p * a.WPP * 4;
    constexpr int U = 4;
    for (uint32_t v0 = 0; v0 < a.qv; v0 += U * kThreads) {
        u32x4 q[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t v = v0 + u * kThreads + tid;
            if (v < a.qv) q[u] = xv[v];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t v = v0 + u * kThreads + tid;
            if (v < a.qv) quant_vector<T, BITS, ND>(a, q[u], v, pr, lfcs, cbase);
        }
    }
    const uint32_t padb = a.WPP * 4 - a.qv * CBV;                  // pad bytes of the last word are zero
    if (tid < padb) cbase[a.qv * CBV + tid] = 0;
}

template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) compress_plane(PlaneArgs a) { compress_plane_body<T, BITS, 2>(a); }
template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) compress_plane_3d(PlaneArgs a) { compress_plane_body<T, BITS, 3>(a); }

// ------------------------------------------------------------------ compress, any shape (slow)

struct AnyArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, H, W, HW, LH, LW, nb, WPP, B;      // H, LH: rows / block rows of one depth slice
    uint32_t D;                                     // depth slices (1 for a 2-D map)
};

// One workgroup per plane; x is re-read from global memory in each pass.
// ND = 3: planes of D x H x W elements with blocks of B x B x B (Appendix D).
template <typename T, int BITS, int ND>
__device__ __forceinline__ void compress_any_body(const AnyArgs& a) {
    __shared__ float red_min[kThreads], red_max[kThreads];
    __shared__ float4 sh_params;
    constexpr int CPW = 32 / BITS;
    constexpr float Lf = float((1 << BITS) - 1);
    const uint32_t tid = threadIdx.x;
    const uint32_t p = blockIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, tid);
    const T* xp = static_cast<const T*>(pt.x) + (size_t)p * a.HW;
    const size_t lfc0 = (size_t)p * a.nb;      // this plane's first LFC element

    // pass A: block means; block min/max of the residual follow from the
    // block min/max of x because x -> fl(x - m) is monotone
    float mn = __builtin_inff(), mx = -__builtin_inff();
    for (uint32_t blk = tid; blk < a.nb; blk += kThreads) {
        const uint32_t bq = blk / a.LW, bj = blk - bq * a.LW;
        uint32_t bd = 0, bi = bq;
        if constexpr (ND == 3) { bd = bq / a.LH; bi = bq - bd * a.LH; }
        const uint32_t r1 = min(a.H, (bi + 1) * a.B), c1 = min(a.W, (bj + 1) * a.B);
        const uint32_t z1 = ND == 3 ? min(a.D, (bd + 1) * a.B) : 1u;
        double S = 0.0;
        float xmin = __builtin_inff(), xmax = -__builtin_inff();
        uint32_t cnt = 0;
        for (uint32_t z = bd * a.B; z < z1; ++z)
            for (uint32_t r = bi * a.B; r < r1; ++r)
                for (uint32_t c = bj * a.B; c < c1; ++c) {
                    const float v = Elem<T>::load(xp, ((size_t)z * a.H + r) * a.W + c);
                    S += (double)v; xmin = fminf(xmin, v); xmax = fmaxf(xmax, v); ++cnt;
                }
        const float lfc = lfc_round<T>((float)(S / (double)cnt), kC16<T>);
        lfc_store<T>(pt.lfc, lfc0 + blk, lfc, kC16<T>);
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
        float delta, Delta, inv;
        plane_scale_any(red_min[0], red_max[0], Lf, kC16<T>, delta, Delta, inv);
        meta_store(pt.meta, p, delta, Delta, kC16<T>);
        const uint32_t k1 = mix32(p ^ pt.seed_a);
        const uint32_t k2 = mix32(k1 + pt.seed_c);
        sh_params = make_float4(delta, inv * 65536.0f, __uint_as_float(k1), __uint_as_float(k2));
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
            uint32_t brow;
            if constexpr (ND == 3) {
                const uint32_t z = r / a.H;
                brow = (z / a.B) * a.LH + (r - z * a.H) / a.B;
            } else {
                brow = r / a.B;
            }
            // written by this workgroup in pass A; visible after the barrier above
            const float lfc = lfc_load<T>(pt.lfc, lfc0 + brow * a.LW + c / a.B, kC16<T>);
            const float h = Elem<T>::load(xp, i) - lfc;
            const uint32_t w = pair_word(k1 + (i >> 1) * kWeyl, k2);
            const uint32_t q = (i & 1u) ? quant<1>(h, delta, inv16, w) : quant<0>(h, delta, inv16, w);
            word |= min(q, (1u << BITS) - 1u) << (e * BITS);      // t may exceed L by a few ulp
        }
        pt.codes[(size_t)p * a.WPP + k] = word;
    }
}

template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) compress_any(AnyArgs a) { compress_any_body<T, BITS, 2>(a); }
template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) compress_any_3d(AnyArgs a) { compress_any_body<T, BITS, 3>(a); }

// ------------------------------------------------------------------ decompress

struct DecArgs {
    DecTab tab;
    Regions rg;
    uint32_t P, H, W, HW, LH, LW, nb, WPP, B;
    uint32_t G;          // planes per workgroup
    uint32_t q4;         // HW / 4
    uint32_t w4;         // W / 4
    uint32_t Hs, LHs;    // 3-D maps: rows and block rows of one depth slice (H counts the rows of all slices)
    uint32_t pair8;      // 2-byte elements, W a multiple of 8, output 16-byte aligned: a lane step writes 8 elements
    uint32_t out_off;    // decompress_words: byte offset of the staged output in LDS
    FastDiv d_q4, d_w4, d_B, d_W, d_HW, d_Hs, d_wpp;
};

// Index of the first block of the block row that holds row r; for a 3-D map (Appendix D,
// UpSampling3D) r counts the rows of all depth slices.
template <int ND>
__device__ __forceinline__ uint32_t lfc_row(const DecArgs& a, uint32_t r) {
    if constexpr (ND == 3) {
        const uint32_t z = fdiv(r, a.d_Hs);
        return (fdiv(z, a.d_B) * a.LHs + fdiv(r - z * a.Hs, a.d_B)) * a.LW;
    } else {
        return fdiv(r, a.d_B) * a.LW;
    }
}

// Sec. 4.2: hh = Delta*q + delta ; reconstruction: xhat = lfc + hh (three fp32 ops)
__device__ __forceinline__ float dequant(uint32_t q, float Delta, float delta, float lfc) {
    float hh = (float)q * Delta;
    hh = hh + delta;
    return lfc + hh;
}

// Four reconstructed elements leave with one store.  The map is written once
// and not read again by this library, so the stores are non-temporal: they do
// not displace what the neighbouring kernels keep in the caches (3.5 % on the
// whole compress + decompress step).  Build with -DDIVISION_TEMPORAL_STORE when
// the consumer of the map runs right behind and should find it in the
// last-level cache.
template <typename T>
__device__ __forceinline__ void store4(T* dst, size_t i, float a, float b, float c, float d) {
#ifndef DIVISION_TEMPORAL_STORE
    if constexpr (sizeof(T) == 4) {
        f32x4 v; v.x = a; v.y = b; v.z = c; v.w = d;
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(dst + i));
    } else {
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        u32x2 o;
        o.x = float_to_bf16_bits(a) | (float_to_bf16_bits(b) << 16);
        o.y = float_to_bf16_bits(c) | (float_to_bf16_bits(d) << 16);
        __builtin_nontemporal_store(o, reinterpret_cast<u32x2*>(dst + i));
    }
#else
    if constexpr (sizeof(T) == 4) {
        *reinterpret_cast<float4*>(dst + i) = make_float4(a, b, c, d);
    } else {
        uint2 o;
        o.x = float_to_bf16_bits(a) | (float_to_bf16_bits(b) << 16);
        o.y = float_to_bf16_bits(c) | (float_to_bf16_bits(d) << 16);
        *reinterpret_cast<uint2*>(dst + i) = o;
    }
#endif
}

// Copies this workgroup's slices of the three packed regions (codes, meta, LFC
// of planes p0 .. p0+Gc-1: about 8 % of the output volume) into LDS with
// coalesced loads, so that the streaming loop below depends on LDS latency
// only and its 16-byte stores go out back to back.
template <typename T>
__device__ __forceinline__ void stage_packed(const DecArgs& a, const DecPtrs& pt, uint32_t p0, uint32_t Gc, uint32_t* s_codes,
                                             float2* s_meta, T* s_lfc, uint32_t tid) {
    const uint32_t nw = Gc * a.WPP;
    const uint32_t* src = pt.codes + (size_t)p0 * a.WPP;
    if ((((size_t)p0 * a.WPP) & 3u) == 0) {
        const uint32_t nq = nw >> 2;
        for (uint32_t i = tid; i < nq; i += kThreads)
            reinterpret_cast<u32x4*>(s_codes)[i] = reinterpret_cast<const u32x4*>(src)[i];
        for (uint32_t i = (nq << 2) + tid; i < nw; i += kThreads) s_codes[i] = src[i];
    } else {
        for (uint32_t i = tid; i < nw; i += kThreads) s_codes[i] = src[i];
    }
    for (uint32_t i = tid; i < Gc; i += kThreads) s_meta[i] = meta_load(pt.meta, p0 + i, kC16<T>);
    const uint32_t nl = Gc * a.nb;
    if (sizeof(T) == 4 && kC16<T>) {
        // bfloat16 H^L of an fp32 map: widened here, so that the streaming loops read floats as ever
        const uint16_t* lsrc = static_cast<const uint16_t*>(pt.lfc) + (size_t)p0 * a.nb;
        for (uint32_t i = tid; i < nl; i += kThreads) reinterpret_cast<float*>(s_lfc)[i] = bf16_bits_to_float(lsrc[i]);
    } else {
        const T* lsrc = static_cast<const T*>(pt.lfc) + (size_t)p0 * a.nb;
        for (uint32_t i = tid; i < nl; i += kThreads) s_lfc[i] = lsrc[i];
    }
    lds_barrier();
}

// LDS carve-up shared by the two streaming kernels (the host sizes it the same way)
template <typename T>
__device__ __forceinline__ void dec_lds(const DecArgs& a, uint32_t*& s_codes, float2*& s_meta, T*& s_lfc) {
    extern __shared__ float4 smem4[];
    s_codes = reinterpret_cast<uint32_t*>(smem4);
    s_meta = reinterpret_cast<float2*>(s_codes + ((a.G * a.WPP + 3u) & ~3u));
    s_lfc = reinterpret_cast<T*>(s_meta + a.G);
}

// W % 4 == 0 and B % 4 == 0: the four elements of a vector lie in one row and
// share one LFC value.  A workgroup streams G whole planes.
template <typename T, int BITS, int ND>
__device__ __forceinline__ void decompress_rowvec_body(const DecArgs& a) {
    const DecPtrs pt = dec_ptrs(a.tab, a.rg);
    uint32_t* s_codes; float2* s_meta; T* s_lfc;
    dec_lds<T>(a, s_codes, s_meta, s_lfc);
    const uint32_t tid = threadIdx.x;
    const uint32_t p0 = blockIdx.x * a.G;
    const uint32_t Gc = min(a.G, a.P - p0);
    stage_packed<T>(a, pt, p0, Gc, s_codes, s_meta, s_lfc, tid);
    const uint32_t nvec = Gc * a.q4;
    constexpr uint32_t Lq = (1u << BITS) - 1u;
    T* out = static_cast<T*>(pt.xhat) + (size_t)p0 * a.HW;
    if constexpr (sizeof(T) == 2) {
        if (a.pair8) {
            // two neighbouring vectors of one row per lane step: one 16-byte store
            for (uint32_t vi = 2 * tid; vi < nvec; vi += 2 * kThreads) {
                const uint32_t g = fdiv(vi, a.d_q4);
                const uint32_t fi = vi - g * a.q4;                     // even
                const float2 dd = s_meta[g];
                uint32_t lo, hi;                                       // codes of elements 0-3 and 4-7
                if constexpr (BITS == 2) {
                    lo = reinterpret_cast<const uint16_t*>(s_codes)[(g * a.WPP * 4 + fi) >> 1];
                    hi = lo >> 8;
                } else if constexpr (BITS == 4) {
                    lo = s_codes[(g * a.WPP * 2 + fi) >> 1];
                    hi = lo >> 16;
                } else {
                    lo = s_codes[g * a.WPP + fi];
                    hi = s_codes[g * a.WPP + fi + 1];
                }
                const uint32_t r = fdiv(fi, a.d_w4);
                const uint32_t c = (fi - r * a.w4) * 4;
                const T* lrow = s_lfc + g * a.nb + lfc_row<ND>(a, r);
                const float l0 = Elem<T>::load(lrow, fdiv(c, a.d_B)), l1 = Elem<T>::load(lrow, fdiv(c + 4, a.d_B));
                uint32_t w[4];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    w[e] = float_to_bf16_bits(dequant((lo >> (2 * e * BITS)) & Lq, dd.y, dd.x, l0)) |
                           (float_to_bf16_bits(dequant((lo >> ((2 * e + 1) * BITS)) & Lq, dd.y, dd.x, l0)) << 16);
                    w[2 + e] = float_to_bf16_bits(dequant((hi >> (2 * e * BITS)) & Lq, dd.y, dd.x, l1)) |
                               (float_to_bf16_bits(dequant((hi >> ((2 * e + 1) * BITS)) & Lq, dd.y, dd.x, l1)) << 16);
                }
                u32x4 o; o.x = w[0]; o.y = w[1]; o.z = w[2]; o.w = w[3];
#ifndef DIVISION_TEMPORAL_STORE
                __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(out + (size_t)vi * 4));
#else
                *reinterpret_cast<u32x4*>(out + (size_t)vi * 4) = o;
#endif
            }
            return;
        }
    }
    for (uint32_t vi = tid; vi < nvec; vi += kThreads) {
        const uint32_t g = fdiv(vi, a.d_q4);
        const uint32_t fi = vi - g * a.q4;        // vector index inside the plane
        const float2 dd = s_meta[g];
        uint32_t c4;                               // the four codes, BITS apart from bit 0
        if constexpr (BITS == 2) c4 = reinterpret_cast<const uint8_t*>(s_codes)[g * a.WPP * 4 + fi];
        else if constexpr (BITS == 4) c4 = reinterpret_cast<const uint16_t*>(s_codes)[g * a.WPP * 2 + fi];
        else c4 = s_codes[g * a.WPP + fi];
        const uint32_t r = fdiv(fi, a.d_w4);
        const uint32_t c = (fi - r * a.w4) * 4;
        const float lfc = Elem<T>::load(s_lfc, g * a.nb + lfc_row<ND>(a, r) + fdiv(c, a.d_B));
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = dequant((c4 >> (e * BITS)) & Lq, dd.y, dd.x, lfc);
        store4(out, (size_t)vi * 4, o[0], o[1], o[2], o[3]);
    }
}

template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) decompress_rowvec(DecArgs a) { decompress_rowvec_body<T, BITS, 2>(a); }
template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) decompress_rowvec_3d(DecArgs a) { decompress_rowvec_body<T, BITS, 3>(a); }

// H*W a multiple of 4 and at most 255 blocks per plane: the LFC index of every
// element of a plane is looked up in a table (one byte per element, four per
// vector) that the workgroup builds once in LDS, so the streaming loop has no
// row / column arithmetic.  A workgroup streams G whole planes.
template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) decompress_table(DecArgs a) {
    const DecPtrs pt = dec_ptrs(a.tab, a.rg);
    uint32_t* s_codes; float2* s_meta; T* s_lfc;
    dec_lds<T>(a, s_codes, s_meta, s_lfc);
    uint32_t* s_tab = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(s_lfc) + ((a.G * a.nb * sizeof(T) + 15u) & ~15u));
    constexpr uint32_t Lq = (1u << BITS) - 1u;
    const uint32_t tid = threadIdx.x;
    const uint32_t p0 = blockIdx.x * a.G;
    const uint32_t Gc = min(a.G, a.P - p0);
    for (uint32_t fi = tid; fi < a.q4; fi += kThreads) {
        uint32_t r = fdiv(fi * 4, a.d_W);
        uint32_t c = fi * 4 - r * a.W;
        uint32_t t = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            t |= (fdiv(r, a.d_B) * a.LW + fdiv(c, a.d_B)) << (8 * e);
            if (++c == a.W) { c = 0; ++r; }
        }
        s_tab[fi] = t;
    }
    stage_packed<T>(a, pt, p0, Gc, s_codes, s_meta, s_lfc, tid);      // ends with a barrier
    const uint32_t nvec = Gc * a.q4;
    T* out = static_cast<T*>(pt.xhat) + (size_t)p0 * a.HW;
    for (uint32_t vi = tid; vi < nvec; vi += kThreads) {
        const uint32_t g = fdiv(vi, a.d_q4);
        const uint32_t fi = vi - g * a.q4;
        const float2 dd = s_meta[g];
        uint32_t c4;
        if constexpr (BITS == 2) c4 = reinterpret_cast<const uint8_t*>(s_codes)[g * a.WPP * 4 + fi];
        else if constexpr (BITS == 4) c4 = reinterpret_cast<const uint16_t*>(s_codes)[g * a.WPP * 2 + fi];
        else c4 = s_codes[g * a.WPP + fi];
        const uint32_t t = s_tab[fi];
        const T* lp = s_lfc + g * a.nb;
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            o[e] = dequant((c4 >> (e * BITS)) & Lq, dd.y, dd.x, Elem<T>::load(lp, (t >> (8 * e)) & 0xffu));
        store4(out, (size_t)vi * 4, o[0], o[1], o[2], o[3]);
    }
}

// Any W, H, B: a workgroup streams G whole planes as one flat run of elements,
// four consecutive elements per lane step; every element finds its own plane,
// row, column and block.  G*HW is a multiple of 4 whenever G < P remains, so
// vector stores stay aligned; the ragged end of the last chunk is scalar.
template <typename T, int BITS, int ND>
__device__ __forceinline__ void decompress_flat_body(const DecArgs& a) {
    const DecPtrs pt = dec_ptrs(a.tab, a.rg);
    uint32_t* s_codes; float2* s_meta; T* s_lfc;
    dec_lds<T>(a, s_codes, s_meta, s_lfc);
    constexpr uint32_t CPW = 32 / BITS;
    constexpr uint32_t Lq = (1u << BITS) - 1u;
    const uint32_t tid = threadIdx.x;
    const uint32_t p0 = blockIdx.x * a.G;
    const uint32_t Gc = min(a.G, a.P - p0);
    stage_packed<T>(a, pt, p0, Gc, s_codes, s_meta, s_lfc, tid);
    const uint32_t n = Gc * a.HW;
    T* out = static_cast<T*>(pt.xhat) + (size_t)p0 * a.HW;
    const bool one_block = a.nb == 1;             // map smaller than the block: LFC is one value per plane
    for (uint32_t e0 = tid * 4; e0 < n; e0 += kThreads * 4) {
        uint32_t g = fdiv(e0, a.d_HW);
        uint32_t i = e0 - g * a.HW;
        float o[4];
        if (one_block && e0 + 4 <= n && a.HW >= 4) {
            // at most one plane boundary inside the vector: elements before it use
            // plane g, the others plane g+1 (which exists because e0+4 <= n)
            const uint32_t n0 = min(4u, a.HW - i);
            const uint32_t g1 = n0 < 4 ? g + 1 : g;
            const float2 da = s_meta[g], db = s_meta[g1];
            const float la = Elem<T>::load(s_lfc, g), lb = Elem<T>::load(s_lfc, g1);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool first = (uint32_t)e < n0;
                const uint32_t idx = first ? i + e : (uint32_t)e - n0;
                const uint32_t w = s_codes[(first ? g : g1) * a.WPP + idx / CPW];
                const uint32_t q = (w >> ((idx % CPW) * BITS)) & Lq;
                o[e] = dequant(q, first ? da.y : db.y, first ? da.x : db.x, first ? la : lb);
            }
            store4(out, e0, o[0], o[1], o[2], o[3]);
            continue;
        }
        if (!one_block && i + 4 <= a.HW && (i % CPW) + 4 <= CPW) {
            // the four elements share plane, scale and code word
            const float2 dd = s_meta[g];
            const uint32_t w = s_codes[g * a.WPP + i / CPW] >> ((i % CPW) * BITS);
            const T* lp = s_lfc + g * a.nb;
            uint32_t r = fdiv(i, a.d_W);
            uint32_t c = i - r * a.W;
            uint32_t rowoff = lfc_row<ND>(a, r);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lfc = Elem<T>::load(lp, rowoff + fdiv(c, a.d_B));
                o[e] = dequant((w >> (e * BITS)) & Lq, dd.y, dd.x, lfc);
                if (++c == a.W) { c = 0; ++r; rowoff = lfc_row<ND>(a, r); }
            }
            store4(out, e0, o[0], o[1], o[2], o[3]);
            continue;
        }
        uint32_t r = fdiv(i, a.d_W);
        uint32_t c = i - r * a.W;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o[e] = 0.0f;
            if (e0 + e < n) {
                const float2 dd = s_meta[g];
                const uint32_t q = (s_codes[g * a.WPP + i / CPW] >> ((i % CPW) * BITS)) & Lq;
                const float lfc = Elem<T>::load(s_lfc, g * a.nb + lfc_row<ND>(a, r) + fdiv(c, a.d_B));
                o[e] = dequant(q, dd.y, dd.x, lfc);
                ++i;
                if (++c == a.W) { c = 0; ++r; }
                if (i == a.HW) { i = 0; r = 0; c = 0; ++g; }
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

template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) decompress_flat(DecArgs a) { decompress_flat_body<T, BITS, 2>(a); }
template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) decompress_flat_3d(DecArgs a) { decompress_flat_body<T, BITS, 3>(a); }

// Maps whose rows are not whole vectors (odd widths, odd plane sizes) with several blocks per
// plane: the chunk of G planes is rebuilt in LDS first, a lane per packed word (the word's
// elements lie in one plane; the lane walks them with a running row and column, starting at a
// lane-dependent element so that the lanes of a wavefront write to different banks), then leaves
// with aligned 16-byte stores like the other streaming kernels (G*HW is a multiple of 4 except in
// the last chunk, whose ragged end is scalar).
template <typename T, int BITS, int ND>
__device__ __forceinline__ void decompress_words_body(const DecArgs& a) {
    const DecPtrs pt = dec_ptrs(a.tab, a.rg);
    uint32_t* s_codes; float2* s_meta; T* s_lfc;
    dec_lds<T>(a, s_codes, s_meta, s_lfc);
    extern __shared__ float4 smem4[];
    float* s_out = reinterpret_cast<float*>(reinterpret_cast<char*>(smem4) + a.out_off);
    constexpr uint32_t CPW = 32 / BITS;
    constexpr uint32_t Lq = (1u << BITS) - 1u;
    const uint32_t tid = threadIdx.x;
    const uint32_t p0 = blockIdx.x * a.G;
    const uint32_t Gc = min(a.G, a.P - p0);
    stage_packed<T>(a, pt, p0, Gc, s_codes, s_meta, s_lfc, tid);      // ends with a barrier

    // ---- Sec. 4.2 and the reconstruction equation, a packed word per lane and step
    const uint32_t nwords = Gc * a.WPP;
    const uint32_t rot = (tid / (64u / CPW)) & (CPW - 1u);           // lanes CPW floats apart share a bank
    for (uint32_t wi = tid; wi < nwords; wi += kThreads) {
        const uint32_t g = fdiv(wi, a.d_wpp);
        const uint32_t k = wi - g * a.WPP;
        const uint32_t word = s_codes[wi];
        const float2 dd = s_meta[g];
        const T* lp = s_lfc + g * a.nb;
        float* op = s_out + g * a.HW;
        const uint32_t i0 = k * CPW;
        const uint32_t cnt = min(CPW, a.HW - i0);                   // elements of the plane in this word
        // start at element `rot` of the word, go to its end, then from its first element up to rot
        uint32_t e = rot;
        uint32_t r = fdiv(i0 + e, a.d_W);
        uint32_t c = i0 + e - r * a.W;
        uint32_t rowoff = lfc_row<ND>(a, r);
#pragma unroll
        for (uint32_t step = 0; step < CPW; ++step) {
            if (e < cnt) {
                const float lfc = Elem<T>::load(lp, rowoff + fdiv(c, a.d_B));
                op[i0 + e] = dequant((word >> (e * BITS)) & Lq, dd.y, dd.x, lfc);
            }
            ++e;
            if (e == CPW) {                                          // wrap to the word's first element
                e = 0;
                r = fdiv(i0, a.d_W);
                c = i0 - r * a.W;
                rowoff = lfc_row<ND>(a, r);
            } else if (++c == a.W) {
                c = 0;
                ++r;
                rowoff = lfc_row<ND>(a, r);
            }
        }
    }
    lds_barrier();

    // ---- out: 16-byte stores of the rebuilt chunk
    const uint32_t n = Gc * a.HW;
    T* out = static_cast<T*>(pt.xhat) + (size_t)p0 * a.HW;
    const uint32_t nvec = n >> 2;
    for (uint32_t v = tid; v < nvec; v += kThreads) {
        const float4 o = reinterpret_cast<const float4*>(s_out)[v];
        store4(out, (size_t)v * 4, o.x, o.y, o.z, o.w);
    }
    for (uint32_t t = (nvec << 2) + tid; t < n; t += kThreads) Elem<T>::store(out, t, s_out[t]);
}

template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) decompress_words(DecArgs a) { decompress_words_body<T, BITS, 2>(a); }
template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) decompress_words_3d(DecArgs a) { decompress_words_body<T, BITS, 3>(a); }

// 2-D planes whose rows or blocks are not whole vectors (odd widths), the counterpart of compress_units:
// a lane step rebuilds four consecutive elements of the plane whatever the width and writes them with
// one store (planes start on 4-byte boundaries).  Which block each element belongs to is the same for
// every plane: a table of LDS offsets made once per workgroup, which then takes planes blockIdx.x,
// blockIdx.x + gridDim.x, ...  A plane's LFC goes through LDS (two buffers, one barrier per plane);
// the next plane's codes, LFC and meta are loaded while the current one is rebuilt.
constexpr int kUnitsLfc = 4;      // LFC values a lane stages per plane: planes of up to 4 * threads blocks
template <typename T, int BITS, int NW>
__global__ void __launch_bounds__(64 * NW) decompress_units(DecArgs a) {
    constexpr int NT = 64 * NW;
    constexpr int K = kUnitsK;
    constexpr int KL = kUnitsLfc;
    constexpr uint32_t CB = BITS / 2;                  // code bytes per unit
    constexpr uint32_t Lq = (1u << BITS) - 1u;
    extern __shared__ float4 smem4[];
    float* lbuf = reinterpret_cast<float*>(smem4);     // [2][nbp]
    const uint32_t nbp = (a.nb + 3u) & ~3u;
    const DecPtrs pt = dec_ptrs(a.tab, a.rg);
    const uint32_t tid = threadIdx.x;
    auto round_live = [&](int k) -> bool { return (uint32_t)(NT * k) < a.q4; };

    // 2-byte elements, odd planes of an odd element count: the plane starts in the middle of a dword.
    // Its units then start one element early, so that every store is dword-aligned; the element before
    // the plane and those past it are left alone.  The same for all planes of the workgroup: the grid is
    // even then, or every workgroup has one plane.
    const uint32_t shift = sizeof(T) == 2 ? (blockIdx.x * a.HW) & 1u : 0u;

    // LDS byte offset of the LFC of each element's block (elements outside the plane: block 0, never stored)
    uint32_t lo[K][2];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        uint32_t off[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t e = 4u * (tid + NT * k) + j - shift;       // wraps for the element before the plane
            const uint32_t r = fdiv(e, a.d_W);
            const uint32_t c = e - r * a.W;
            off[j] = e < a.HW ? 4u * (fdiv(r, a.d_B) * a.LW + fdiv(c, a.d_B)) : 0u;
        }
        lo[k][0] = off[0] | (off[1] << 16);
        lo[k][1] = off[2] | (off[3] << 16);
    }
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    uint32_t codes[K];
    u32x2 wide[sizeof(T) == 2 ? K : 1];                // shifted units: the two code words a unit's codes lie in
    float lf[KL];
    float2 dd;
    auto issue_loads = [&](uint32_t p) {
        const __amdgpu_buffer_rsrc_t crs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint32_t*>(pt.codes) + (size_t)p * a.WPP, 0, (int)(a.q4 * CB), 0x00020000);
        if constexpr (sizeof(T) == 2) {
            if (shift) {
                // codes of elements 4f-1 .. 4f+2: 4 * BITS bits from bit (4f-1) * BITS of the plane's code words
                const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc(
                    const_cast<uint32_t*>(pt.codes) + (size_t)p * a.WPP, 0, (int)(a.WPP * 4u), 0x00020000);
#pragma unroll
                for (int k = 0; k < K; ++k) {
                    if (!round_live(k)) continue;
                    const uint32_t f = tid + NT * k;
                    const uint32_t bit = f ? (4u * f - 1u) * BITS : 0u;
                    wide[k] = __builtin_amdgcn_raw_buffer_load_b64(wrs, (bit >> 5) * 4u, 0, 0);
                }
            }
        }
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (!round_live(k) || shift) continue;
            if constexpr (CB == 1) codes[k] = __builtin_amdgcn_raw_buffer_load_b8(crs, tid, k * NT, 0);
            else if constexpr (CB == 2) codes[k] = __builtin_amdgcn_raw_buffer_load_b16(crs, tid * 2u, k * NT * 2, 0);
            else codes[k] = __builtin_amdgcn_raw_buffer_load_b32(crs, tid * 4u, k * NT * 4, 0);
        }
#pragma unroll
        for (int m = 0; m < KL; ++m) {
            const uint32_t t = tid + NT * m;
            if ((uint32_t)(NT * m) < a.nb) lf[m] = t < a.nb ? lfc_load<T>(pt.lfc, (size_t)p * a.nb + t, kC16<T>) : 0.0f;
        }
        dd = meta_load(pt.meta, p, kC16<T>);
    };

    if (blockIdx.x < a.P) issue_loads(blockIdx.x);
    uint32_t flip = 0;
    for (uint32_t p = blockIdx.x; p < a.P; p += gridDim.x, flip ^= 1u) {
        float* lfcs = lbuf + flip * nbp;
#pragma unroll
        for (int m = 0; m < KL; ++m) {
            const uint32_t t = tid + NT * m;
            if ((uint32_t)(NT * m) < a.nb && t < a.nb) lfcs[t] = lf[m];
        }
        uint32_t c4[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            c4[k] = 0u;
            if (!round_live(k)) continue;
            if constexpr (sizeof(T) == 2) {
                if (shift) {
                    const uint32_t f = tid + NT * k;
                    const uint32_t bit = f ? (4u * f - 1u) * BITS : 0u;
                    const uint32_t c = __builtin_amdgcn_alignbit(wide[k].y, wide[k].x, bit & 31u);
                    c4[k] = f ? c : c << BITS;             // unit 0: the slot before the plane, then elements 0, 1, 2
                    continue;
                }
            }
            c4[k] = codes[k];
        }
        const float2 sc = dd;
        if (p + gridDim.x < a.P) issue_loads(p + gridDim.x);
        if constexpr (NW == 1) wave_sync(); else lds_barrier();

        T* out = static_cast<T*>(pt.xhat) + (size_t)p * a.HW;       // element e of the plane at out[e]
        const char* lb = reinterpret_cast<const char*>(lfcs);
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (!round_live(k)) continue;
            const uint32_t f = tid + NT * k;
            float o[4];
            o[0] = dequant(c4[k] & Lq, sc.y, sc.x, *reinterpret_cast<const float*>(lb + (lo[k][0] & 0xffffu)));
            o[1] = dequant((c4[k] >> BITS) & Lq, sc.y, sc.x, *reinterpret_cast<const float*>(lb + (lo[k][0] >> 16)));
            o[2] = dequant((c4[k] >> (2 * BITS)) & Lq, sc.y, sc.x, *reinterpret_cast<const float*>(lb + (lo[k][1] & 0xffffu)));
            o[3] = dequant((c4[k] >> (3 * BITS)) & Lq, sc.y, sc.x, *reinterpret_cast<const float*>(lb + (lo[k][1] >> 16)));
            const uint32_t e0 = 4u * f - shift;                  // the unit's first element (wraps for unit 0 of a shifted plane)
            if (e0 + 4u <= a.HW && (shift == 0u || f != 0u)) {
                store4(out - shift, (size_t)f * 4, o[0], o[1], o[2], o[3]);
            } else {
                // a unit that reaches outside the plane (the last one when H*W is not a multiple of 4,
                // the first one of a shifted plane): element by element
#pragma unroll
                for (uint32_t j = 0; j < 4; ++j) {
                    const uint32_t e = e0 + j;
                    if (e < a.HW) Elem<T>::store(out, e, o[j]);
                }
            }
        }
    }
}

// planes too large for the 32-bit index tricks above: one element per thread step
template <typename T, int BITS, int ND>
__device__ __forceinline__ void decompress_scalar_body(const DecArgs& a) {
    const DecPtrs pt = dec_ptrs(a.tab, a.rg);
    constexpr uint32_t CPW = 32 / BITS;
    constexpr uint32_t Lq = (1u << BITS) - 1u;
    const uint32_t p = blockIdx.x;
    const float2 dd = meta_load(pt.meta, p, kC16<T>);
    const size_t lfc0 = (size_t)p * a.nb;
    const uint32_t* cp = pt.codes + (size_t)p * a.WPP;
    T* out = static_cast<T*>(pt.xhat) + (size_t)p * a.HW;
    for (uint32_t i = threadIdx.x; i < a.HW; i += kThreads) {
        const uint32_t r = i / a.W, c = i - r * a.W;
        const uint32_t q = (cp[i / CPW] >> ((i % CPW) * BITS)) & Lq;
        uint32_t brow;
        if constexpr (ND == 3) {
            const uint32_t z = r / a.Hs;
            brow = (z / a.B) * a.LHs + (r - z * a.Hs) / a.B;
        } else {
            brow = r / a.B;
        }
        const float lfc = lfc_load<T>(pt.lfc, lfc0 + brow * a.LW + c / a.B, kC16<T>);
        Elem<T>::store(out, i, dequant(q, dd.y, dd.x, lfc));
    }
}

template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) decompress_scalar(DecArgs a) { decompress_scalar_body<T, BITS, 2>(a); }
template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) decompress_scalar_3d(DecArgs a) { decompress_scalar_body<T, BITS, 3>(a); }

// ------------------------------------------------------------------ host side

// One-block planes with an odd number of elements (the shapes compress_lane
// takes): one wavefront per round of 64 planes, lane g reconstructs plane g from
// its WPP code words into LDS (stride HW words, odd: no bank conflicts), then the
// round leaves with coalesced 16-byte stores.  a.G = rounds per workgroup.
template <typename T, int BITS>
__global__ void __launch_bounds__(64) decompress_lane(DecArgs a) {
    constexpr int CPW = 32 / BITS;
    constexpr uint32_t Lmask = (1u << BITS) - 1u;
    extern __shared__ float4 smem4[];
    float* xs = reinterpret_cast<float*>(smem4);              // [64 * HW (+3)]
    const uint32_t lane = threadIdx.x;
    const DecPtrs pt = dec_ptrs(a.tab, a.rg);
    const uint32_t nrounds = (a.P + 63u) / 64u;
    float* mine = xs + lane * a.HW;
    const bool out_vec = (reinterpret_cast<uintptr_t>(pt.xhat) % (4 * sizeof(T))) == 0;

    const uint32_t rend = min(nrounds, (blockIdx.x + 1) * a.G);
    for (uint32_t round = blockIdx.x * a.G; round < rend; ++round) {
        const uint32_t p0 = round * 64u;
        const uint32_t Gc = min(64u, a.P - p0);
        const uint32_t p = lane < Gc ? p0 + lane : p0;        // lanes past the last plane redo plane p0 (never stored)
        const float2 dd = meta_load(pt.meta, p, kC16<T>);
        const float lfc = lfc_load<T>(pt.lfc, p, kC16<T>);
        const uint32_t* cp = pt.codes + (size_t)p * a.WPP;
        const uint32_t wfull = a.HW / CPW;
        for (uint32_t w = 0; w < wfull; ++w) {
            const uint32_t word = cp[w];
#pragma unroll
            for (int j = 0; j < CPW; ++j) mine[w * CPW + j] = dequant((word >> (j * BITS)) & Lmask, dd.y, dd.x, lfc);
        }
        const uint32_t left = a.HW - wfull * CPW;
        if (left) {
            const uint32_t word = cp[wfull];
            for (uint32_t j = 0; j < left; ++j) mine[wfull * CPW + j] = dequant((word >> (j * BITS)) & Lmask, dd.y, dd.x, lfc);
        }
        wave_sync();

        const uint32_t n = Gc * a.HW;
        T* out = static_cast<T*>(pt.xhat) + (size_t)p0 * a.HW;
        const uint32_t nv = out_vec ? n / 4u : 0u;
        for (uint32_t vi = lane; vi < nv; vi += 64) {
            const float4 f = reinterpret_cast<const float4*>(xs)[vi];
            store4(out, (size_t)vi * 4, f.x, f.y, f.z, f.w);
        }
        for (uint32_t e = nv * 4u + lane; e < n; e += 64) Elem<T>::store(out, e, xs[e]);
        wave_sync();      // LDS is reused by the next round
    }
}

struct Layout {
    uint64_t P, HW, LD, LH, LW, nb, WPP;      // HW = elements per plane (D*H*W), nb = LD*LH*LW blocks
    size_t codes_off, codes_bytes, meta_off, meta_bytes, lfc_off, lfc_bytes, total;
};

size_t align16(size_t v) { return (v + 15u) & ~(size_t)15u; }

// A plane is D x H x W elements (Appendix D: 3-D maps); D = 1 for the 2-D maps of Sec. 4.1.
int make_layout(int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int B, int b, int dt, Layout* L) {
    if (N <= 0 || C <= 0 || D <= 0 || H <= 0 || W <= 0 || B < 1 || (b != 2 && b != 4 && b != 8)) return DIVISION_EINVAL;
    if (dt != DIVISION_F32 && dt != DIVISION_BF16 && dt != DIVISION_F32_C16) return DIVISION_EINVAL;
    const uint64_t lim31 = 0x7fffffffull;
    if ((uint64_t)N > lim31 || (uint64_t)C > lim31 || (uint64_t)D > lim31 || (uint64_t)H > lim31 || (uint64_t)W > lim31)
        return DIVISION_ERANGE;
    L->P = (uint64_t)N * (uint64_t)C;
    if ((uint64_t)D * (uint64_t)H > lim31) return DIVISION_ERANGE;
    L->HW = (uint64_t)D * (uint64_t)H * (uint64_t)W;
    if (L->P > lim31 || L->HW > lim31 || L->P * L->HW > (1ull << 40)) return DIVISION_ERANGE;
    L->LD = ((uint64_t)D + B - 1) / B;
    L->LH = ((uint64_t)H + B - 1) / B;
    L->LW = ((uint64_t)W + B - 1) / B;
    L->nb = L->LD * L->LH * L->LW;
    const uint64_t cpw = 32 / b;
    L->WPP = (L->HW + cpw - 1) / cpw;
    const size_t lfc_es = dt == DIVISION_F32 ? 4 : 2;          // H^L: element type of x, bfloat16 in the cached-as-bf16 mode
    const size_t meta_es = dt == DIVISION_F32_C16 ? 4 : 8;      // (delta, Delta) per plane
    L->codes_off = 0;
    L->codes_bytes = (size_t)(4 * L->P * L->WPP);
    L->meta_off = align16(L->codes_bytes);
    L->meta_bytes = (size_t)(meta_es * L->P);
    L->lfc_off = align16(L->meta_off + L->meta_bytes);
    L->lfc_bytes = (size_t)(lfc_es * L->P * L->nb);
    L->total = align16(L->lfc_off + L->lfc_bytes);
    return DIVISION_OK;
}

uint64_t gcd_u64(uint64_t a, uint64_t b) { while (b) { uint64_t t = a % b; a = b; b = t; } return a; }

// fdiv(n, d) is exact while n*d < 2^32
bool fastdiv_ok(uint64_t n_max, uint64_t d) { return n_max * d < (1ull << 32); }

Regions make_regions(const Layout& L) {
    Regions rg;
    rg.meta_off = L.meta_off;
    rg.lfc_off = L.lfc_off;
    rg.pad_off[0] = L.codes_off + L.codes_bytes; rg.pad_len[0] = (uint32_t)(L.meta_off - rg.pad_off[0]);
    rg.pad_off[1] = L.meta_off + L.meta_bytes;   rg.pad_len[1] = (uint32_t)(L.lfc_off - rg.pad_off[1]);
    rg.pad_off[2] = L.lfc_off + L.lfc_bytes;     rg.pad_len[2] = (uint32_t)(L.total - rg.pad_off[2]);
    return rg;
}

// Preferred LDS footprint of one wavefront's chunk in compress_wave (small chunks = many wavefronts
// per CU; 8.7 KB measured best over the ResNet-50 set); a single plane of up to kWavePlaneMax bytes is
// taken whatever the preference says.
constexpr uint32_t kWaveChunkLds = 8704u;
constexpr uint32_t kWavePlaneMax = 17u << 10;

int num_cus() {
    static int n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
            v = 256;
        return v;
    }();
    return n;
}

// dynamic LDS above the default limit needs a one-time opt-in per kernel
template <typename Args>
hipError_t allow_large_lds(void (*kern)(Args), size_t lds) {
    if (lds <= 48u * 1024u) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax);
}

template <typename T, int BITS, int B>
hipError_t launch_tile_vec(int vec, const TileArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    void (*kern)(TileArgs) = vec == 4 ? compress_tile<T, BITS, B, 4, 256>
                           : vec == 2 ? compress_tile<T, BITS, B, 2, 256>
                                      : compress_tile<T, BITS, B, 1, 256>;
    hipError_t e = allow_large_lds(kern, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, a);
    return hipGetLastError();
}

template <typename T, int BITS>
hipError_t launch_tile(int B, int vec, const TileArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    return B == 8 ? launch_tile_vec<T, BITS, 8>(vec, a, grid, lds, st)
                  : launch_tile_vec<T, BITS, 4>(vec, a, grid, lds, st);
}

template <typename T, int BITS, int B>
hipError_t launch_wave_vec(int vec, const WaveArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    void (*kern)(WaveArgs) = vec == 4 ? compress_wave<T, BITS, B, 4>
                           : vec == 2 ? compress_wave<T, BITS, B, 2>
                                      : compress_wave<T, BITS, B, 1>;
    hipLaunchKernelGGL(kern, grid, dim3(64), lds, st, a);
    return hipGetLastError();
}

template <typename T, int BITS>
hipError_t launch_wave(int B, int vec, const WaveArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    return B == 8 ? launch_wave_vec<T, BITS, 8>(vec, a, grid, lds, st)
                  : launch_wave_vec<T, BITS, 4>(vec, a, grid, lds, st);
}

// Fills the plane-in-registers compress plan; false when the shape is not covered.
bool plan_regs(const Layout& L, int64_t D, int64_t H, int64_t W, int B, size_t es, const void* x,
               RegsArgs* a, uint32_t* grid, size_t* lds, int* nw_out) {
    if (B % 4 != 0 || W % 4 != 0) return false;
    if (D > 1 && B != 8) return false;            // 3-D maps: the B = 8 instances only
    if (((uintptr_t)x % (4 * es)) != 0) return false;
    const uint64_t q4 = L.HW / 4;
    const bool any_b = B != 4 && B != 8;          // the instance that reads B from its arguments
    int nw;
    if (any_b) {
        // a lane adds the unit sums of its block one after the other: at most 64 of them (blocks of
        // up to 16 x 16, longer ones on maps of few rows), several blocks per plane
        const uint64_t brows = (uint64_t)B < (uint64_t)H ? (uint64_t)B : (uint64_t)H;
        if (brows * ((uint64_t)B / 4) > 64 || L.nb == 1) return false;
        if (q4 >= 512 && q4 <= (uint64_t)kRegUnits * 64) nw = 1;
        else if (q4 > (uint64_t)kRegUnits * 64 && q4 <= (uint64_t)kRegUnits * 256) nw = 4;
        else return false;
    } else if (q4 >= 512 && q4 <= (uint64_t)kRegUnits * 64) nw = 1;
    else if (q4 >= (D > 1 ? (uint64_t)kRegUnits * 64 + 1 : 2048) && q4 <= (uint64_t)kRegUnits * 256) nw = 4;
    else if (q4 > (uint64_t)kRegUnits * 256 && q4 <= (uint64_t)kRegUnits * 1024) nw = 16;   // image-sized planes: 1024 threads, one workgroup per CU
    else return false;
    const uint64_t nt = 64ull * nw, w4 = (uint64_t)W / 4;
    if (!fastdiv_ok(kRegUnits * nt, w4) || !fastdiv_ok(L.nb + nt, L.LW) || L.HW * es >= (1ull << 31)) return false;
    if (!fastdiv_ok((uint64_t)H, (uint64_t)B) || !fastdiv_ok(w4, (uint64_t)B / 4)) return false;
    if (!fastdiv_ok((uint64_t)D * (uint64_t)H, (uint64_t)H) || !fastdiv_ok(L.nb + nt, L.LH * L.LW)) return false;
    a->D = (uint32_t)D;
    a->d_H = make_fastdiv((uint32_t)H);
    a->d_slice = make_fastdiv((uint32_t)(L.LH * L.LW));
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW;
    a->LH = (uint32_t)L.LH; a->LW = (uint32_t)L.LW; a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP;
    a->q4 = (uint32_t)q4; a->w4 = (uint32_t)w4;
    a->ppw = 1;      // one plane per workgroup measured best (more workgroups, better balance)
    a->B = (uint32_t)B;
    a->d_w4 = make_fastdiv((uint32_t)w4);
    a->d_LW = make_fastdiv((uint32_t)L.LW);
    a->d_B = make_fastdiv((uint32_t)B);
    a->d_upb = make_fastdiv((uint32_t)B / 4);
    *lds = 8ull * kRegUnits * nt + 4ull * ((L.nb + 1 + 3) & ~3ull) + 8ull * nw + 16 + (D > 1 ? 8ull * L.nb * B + 16 : 0);
    *grid = (uint32_t)((L.P + a->ppw - 1) / a->ppw);
    *nw_out = nw;
    return *lds <= (nw == 16 ? (size_t)kLdsMax : (size_t)(60u * 1024u));
}

template <typename T, int BITS>
hipError_t launch_regs(int B, int nw, const RegsArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    void (*kern)(RegsArgs);
    if (a.D > 1) kern = nw == 1 ? compress_regs_3d<T, BITS, 8, 1> : nw == 4 ? compress_regs_3d<T, BITS, 8, 4> : compress_regs_3d<T, BITS, 8, 16>;
    else if (nw == 1) kern = B == 8 ? compress_regs<T, BITS, 8, 1> : B == 4 ? compress_regs<T, BITS, 4, 1> : compress_regs<T, BITS, 0, 1>;
    else if (nw == 4) kern = B == 8 ? compress_regs<T, BITS, 8, 4> : B == 4 ? compress_regs<T, BITS, 4, 4> : compress_regs<T, BITS, 0, 4>;
    else kern = B == 8 ? compress_regs<T, BITS, 8, 16> : compress_regs<T, BITS, 4, 16>;
    const hipError_t e = allow_large_lds(kern, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, dim3(64 * nw), lds, st, a);
    return hipGetLastError();
}

// Fills the plan of the register kernel for any width; false when the shape is not covered: 2-D maps
// of at most 8 x 1024 units that fit LDS beside their row sums (up to about 163 x 163 elements).
constexpr uint64_t kUnitsMin = 128;       // units per plane from which a plane gets a whole wavefront or more
constexpr uint64_t kUnitsSubMin = 64;     // units per plane from which the instance with 16 or 32 lanes per plane is used
                                          // (17 x 17: 1.7 -> 2.3 TB/s; 13 x 13 and 15 x 15 are no faster than in compress_wave)
bool plan_units(const Layout& L, int64_t D, int64_t H, int64_t W, int B, size_t es, const void* x,
                UnitsArgs* a, uint32_t* grid, size_t* lds, int* nw_out) {
    if (D != 1 || H == 1 || ((uintptr_t)x % 4) != 0) return false;
    // small planes of even width under B = 4 and 8 are the wavefront kernel's (pairs of elements per
    // lane): measured faster there
    if ((B == 4 || B == 8) && W % 2 == 0 && 4ull * L.HW + 16ull <= kWavePlaneMax) return false;
    const uint64_t q4 = (L.HW + 3) / 4;
    if (L.nb > 16383 || B > 4095) return false;              // LFC offsets are kept as 16-bit byte offsets
    const uint64_t nitem = L.nb * (uint64_t)B;
    int nw = 1;
    uint64_t S = 64;                                          // lanes per plane
    if (q4 < kUnitsMin) {
        // small planes: 8, 16 or 32 lanes each, several planes per wavefront
        if (q4 < kUnitsSubMin) return false;
        S = 8;
        while (S < 64 && (q4 > (uint64_t)kUnitsK * S || nitem > (uint64_t)kUnitsK * S)) S *= 2;
        nw = S < 64 ? 0 : 1;
    }
    if (nw) {
        while (nw < 16 && (q4 > (uint64_t)kUnitsK * 64 * nw || nitem > (uint64_t)kUnitsK * 64 * nw)) nw *= 2;
        S = 64ull * nw;
    }
    if (q4 > (uint64_t)kUnitsK * S || nitem > (uint64_t)kUnitsK * S) return false;       // 8 units and 8 row segments per lane
    const uint64_t q4p = (q4 + S - 1) / S * S;
    if (!fastdiv_ok(4ull * kUnitsK * S + 4, (uint64_t)W) || !fastdiv_ok(4ull * kUnitsK * S + 4, (uint64_t)B) ||
        !fastdiv_ok(nitem + S, (uint64_t)B) || !fastdiv_ok(L.nb + S, L.LW))
        return false;
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW;
    a->LW = (uint32_t)L.LW; a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP; a->B = (uint32_t)B;
    a->q4 = (uint32_t)q4; a->q4p = (uint32_t)q4p; a->nitem = (uint32_t)nitem;
    a->S = (uint32_t)S;
    a->S_log2 = 0;
    while ((1ull << a->S_log2) < S) ++a->S_log2;
    a->d_W = make_fastdiv((uint32_t)W);
    a->d_B = make_fastdiv((uint32_t)B);
    a->d_LW = make_fastdiv((uint32_t)L.LW);
    const uint64_t G = nw ? 1 : 64 / S;                       // planes per round
    const uint64_t reg = (16ull * q4p + 8ull * nitem + 4ull * ((L.nb + 1 + 3) & ~3ull) + 8ull * (nw ? nw : 1) + 16 + 15) & ~15ull;
    a->reg_bytes = (uint32_t)reg;
    a->nrounds = (uint32_t)((L.P + G - 1) / G);
    *lds = reg * G;
    if (*lds > (size_t)kLdsMax) return false;
    // as many workgroups as the machine holds at once (LDS, and 16 wavefronts per CU), each taking every
    // grid-th round of planes
    const uint64_t wpg = nw ? (uint64_t)nw : 1;               // wavefronts per workgroup
    uint64_t per_cu = (160ull << 10) / *lds;
    if (per_cu > 16ull / wpg) per_cu = 16ull / wpg;
    if (per_cu < 1) per_cu = 1;
    uint64_t g = (uint64_t)num_cus() * per_cu;
    g += g & 1;            // even: with 2-byte elements the planes of a workgroup then start alike within a dword
    *grid = (uint32_t)(g < a->nrounds ? g : a->nrounds);
    *nw_out = nw;
    return true;
}

template <typename T, int BITS>
hipError_t launch_units(int nw, const UnitsArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    void (*kern)(UnitsArgs) = nw == 0 ? compress_units<T, BITS, 0> : nw == 1 ? compress_units<T, BITS, 1>
                            : nw == 2 ? compress_units<T, BITS, 2> : nw == 4 ? compress_units<T, BITS, 4>
                            : nw == 8 ? compress_units<T, BITS, 8> : compress_units<T, BITS, 16>;
    const hipError_t e = allow_large_lds(kern, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, dim3(nw ? 64 * nw : 64), lds, st, a);
    return hipGetLastError();
}

// one-block planes with an odd element count: the shapes the lane-per-plane kernels take
bool lane_shape(const Layout& L) { return L.nb == 1 && (L.HW & 1) == 1 && L.HW <= 64; }

// Fills the lane-per-plane compress plan; false when the shape is not covered.
bool plan_lane(const Layout& L, size_t es, const void* x, LaneArgs* a, uint32_t* grid, size_t* lds) {
    if (!lane_shape(L)) return false;
    a->P = (uint32_t)L.P; a->HW = (uint32_t)L.HW; a->WPP = (uint32_t)L.WPP;
    a->nrounds = (uint32_t)((L.P + 63) / 64);
    a->vec_load = ((uintptr_t)x % 16) == 0;
    uint32_t rpw = 2;
    while (rpw > 1 && a->nrounds / rpw < 32u * (uint32_t)num_cus()) --rpw;
    a->rpw = rpw;
    *lds = 4ull * (64ull * L.HW + 4) + 16 * (es == 2 ? 1 : 0);
    *grid = (a->nrounds + rpw - 1) / rpw;
    return true;
}

// Fills the items-from-global compress plan (small planes); false when the shape is not covered.
bool plan_items(const Layout& L, int64_t H, int64_t W, int B, size_t es, const void* x,
                ItemsArgs* a, uint32_t* grid, size_t* lds, int* vec_out) {
    if ((B != 4 && B != 8) || W % 2 != 0) return false;
    const int vec = W % 4 == 0 ? 4 : 2;
    if (((uintptr_t)x % (vec * es)) != 0) return false;
    const uint64_t ipb = (uint64_t)B / vec;
    const uint64_t slots = (uint64_t)W / vec;
    const uint64_t ipr = (slots + ipb - 1) / ipb * ipb;
    const uint64_t ipp = L.LH * ipr;
    if (ipp > 64) return false;
    uint64_t S = 1, lg = 0;
    while (S < ipp) { S *= 2; ++lg; }
    const uint64_t ppr = 64 / S;
    if (ppr * L.WPP * 4 > 32u * 1024u || ppr * L.HW * es >= (1ull << 31)) return false;
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW;
    a->LW = (uint32_t)L.LW; a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP;
    a->ipr = (uint32_t)ipr; a->ipp = (uint32_t)ipp; a->S = (uint32_t)S; a->S_log2 = (uint32_t)lg;
    a->ppr = (uint32_t)ppr;
    a->nrounds = (uint32_t)((L.P + ppr - 1) / ppr);
    a->d_ipr = make_fastdiv((uint32_t)ipr);
    uint32_t rpw = 2;
    while (rpw > 1 && a->nrounds / rpw < 32u * (uint32_t)num_cus()) --rpw;
    a->rpw = rpw;
    *lds = 4ull * ppr * L.WPP + 16;
    *grid = (a->nrounds + rpw - 1) / rpw;
    *vec_out = vec;
    return true;
}

template <typename T, int BITS>
hipError_t launch_items(int B, int vec, const ItemsArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    void (*kern)(ItemsArgs);
    if (a.H == 1) {
        if (B == 8) kern = vec == 4 ? compress_items<T, BITS, 8, 4, 1> : compress_items<T, BITS, 8, 2, 1>;
        else kern = vec == 4 ? compress_items<T, BITS, 4, 4, 1> : compress_items<T, BITS, 4, 2, 1>;
    } else {
        if (B == 8) kern = vec == 4 ? compress_items<T, BITS, 8, 4, 8> : compress_items<T, BITS, 8, 2, 8>;
        else kern = vec == 4 ? compress_items<T, BITS, 4, 4, 4> : compress_items<T, BITS, 4, 2, 4>;
    }
    hipLaunchKernelGGL(kern, grid, dim3(64), lds, st, a);
    return hipGetLastError();
}

// Fills the one-wavefront compress plan; false when the shape is not covered.
bool plan_wave(const Layout& L, int64_t H, int64_t W, int B, int b, size_t es, const void* x,
               WaveArgs* a, uint32_t* grid, size_t* lds, int* vec_out) {
    if (B != 4 && B != 8) return false;
    const uint64_t per_plane = 4ull * L.HW + 16ull;
    if (per_plane > kWavePlaneMax) return false;
    const int vec = (W % 4 == 0) ? 4 : (W % 2 == 0) ? 2 : 1;
    const uint32_t ipb = (uint32_t)B / (uint32_t)vec;
    const uint64_t slots = ((uint64_t)W + vec - 1) / vec;
    const uint64_t ipr = (slots + ipb - 1) / ipb * ipb;
    const uint64_t ipp = L.LH * ipr;
    uint64_t ippp = 1, lg = 0;
    if (ipp <= 64) { while (ippp < ipp) { ippp *= 2; ++lg; } }
    else ippp = (ipp + 63) / 64 * 64;
    uint64_t Gmax = kWaveChunkLds / per_plane;
    if (Gmax < 1) Gmax = 1;
    if (Gmax > L.P) Gmax = L.P;
    const uint64_t unit = 16 / gcd_u64(16, L.HW * es);
    uint32_t vec_load = ((uintptr_t)x % 16) == 0;
    if (vec_load && unit > 1 && Gmax < unit && Gmax < L.P) {
        if (unit * per_plane <= kWavePlaneMax) Gmax = unit; else vec_load = 0;
    }
    const uint64_t step = vec_load ? unit : 1;
    // pick the G that wastes the fewest lanes in partly filled rounds
    const uint64_t cpw = 32 / b, ppw = cpw / 2;
    const double c1 = 4.5 * B * vec, c3 = 8.5 * (double)cpw;
    uint64_t G = 0;
    double best = 0;
    for (uint64_t g = step; g <= Gmax; g += step) {
        const double r1 = ipp <= 64 ? (double)((g + 64 / ippp - 1) / (64 / ippp)) : (double)(g * (ippp / 64));
        const uint64_t nw = g * L.WPP, tw = nw % 64;
        const double r3 = (double)(nw / 64) + (tw == 0 ? 0.0 : tw * ppw <= 64 ? 0.25 : 1.0);
        const double per_elt = (r1 * c1 + r3 * c3 + 2.0) / (double)(g * L.HW);
        if (G == 0 || per_elt < best * 0.97) { G = g; best = per_elt; }
    }
    if (G == 0) G = Gmax;          // Gmax == P < unit: a single chunk, aligned at its start
    if (!fastdiv_ok(ippp, ipr) || !fastdiv_ok(G * L.WPP + 64, L.WPP)) return false;
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW;
    a->LH = (uint32_t)L.LH; a->LW = (uint32_t)L.LW; a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP;
    a->G = (uint32_t)G; a->ipr = (uint32_t)ipr; a->ipp = (uint32_t)ipp;
    a->ippp = (uint32_t)ippp; a->ippp_log2 = (uint32_t)lg;
    a->vec_load = vec_load;
    a->d_ipr = make_fastdiv((uint32_t)ipr);
    a->d_wpp = make_fastdiv((uint32_t)L.WPP);
    *lds = 16ull * G + 4ull * ((G * L.HW + 3) / 4 * 4) + 64;      // 16 floats of slack for ragged last words
    // the staging registers hold 16 x 64 vectors of 16 bytes
    if (vec_load && G * L.HW * es > 16ull * 1024ull) return false;
    *grid = (uint32_t)((L.P + G - 1) / G);
    *vec_out = vec;
    return true;
}

// Fills the one-block plan: the block covers the plane, which is whole 16-byte vectors, at most
// kOneUnits per lane of a wavefront.
bool plan_one(const Layout& L, size_t es, const void* x, OneArgs* a, uint32_t* grid) {
    const uint64_t epv = 16 / es;
    if (L.nb != 1 || ((uintptr_t)x % 16) != 0 || L.HW % epv != 0) return false;
    const uint64_t qv = L.HW / epv;
    if (qv > (uint64_t)kOneUnits * 64) return false;
    // lanes per plane: the smallest power of two from 8 up (a plane's lanes then read 128 contiguous
    // bytes per round) that keeps the plane within kOneUnits rounds
    uint32_t best_S = 0, best_log = 0;
    for (uint32_t lg = 3; lg <= 6; ++lg) {
        const uint64_t S = 1ull << lg;
        if ((qv + S - 1) / S <= (uint64_t)kOneUnits) { best_S = (uint32_t)S; best_log = lg; break; }
    }
    a->P = (uint32_t)L.P; a->HW = (uint32_t)L.HW; a->WPP = (uint32_t)L.WPP;
    a->qv = (uint32_t)qv;
    a->S = best_S; a->S_log2 = best_log;
    a->ppw = 64u / best_S;
    *grid = (uint32_t)((L.P + a->ppw - 1) / a->ppw);
    return true;
}

// single-block planes of whole vectors: compress_one's, ahead of the kernels for general shapes
bool one_shape(const Layout& L, size_t es, const void* x) {
    OneArgs tmp{};
    uint32_t g = 0;
    return plan_one(L, es, x, &tmp, &g);
}

// Fills the plan of compress_line: a 1-D map (one row) of whole 16-byte vectors, several blocks per
// plane, a block a power-of-two number of vectors, at most kOneUnits vectors per lane.
bool plan_line(const Layout& L, int64_t D, int64_t H, int B, size_t es, const void* x, OneArgs* a, uint32_t* grid) {
    const uint64_t epv = 16 / es;
    if (D != 1 || H != 1 || L.nb < 2 || ((uintptr_t)x % 16) != 0 || L.HW % epv != 0 || (uint64_t)B % epv != 0) return false;
    const uint64_t qv = L.HW / epv, upb = (uint64_t)B / epv;
    if ((upb & (upb - 1)) != 0 || upb > 64 || qv > (uint64_t)kOneUnits * 64) return false;
    uint32_t upb_log = 0;
    while ((1ull << upb_log) < upb) ++upb_log;
    // lanes per plane: the smallest power of two that is a block, at least 8 (a plane's lanes then read
    // 128 contiguous bytes per round) and keeps the plane within kOneUnits rounds: few lanes per plane
    // mean many planes per wavefront to share its fixed costs (measured: 8 or 16 lanes beat both the
    // choice with the fewest idle lane slots and wider ones)
    uint32_t best_S = 0, best_log = 0;
    for (uint32_t lg = upb_log > 3 ? upb_log : 3; lg <= 6; ++lg) {
        const uint64_t S = 1ull << lg;
        if ((qv + S - 1) / S <= (uint64_t)kOneUnits) { best_S = (uint32_t)S; best_log = lg; break; }
    }
    if (best_S == 0) return false;
    a->P = (uint32_t)L.P; a->HW = (uint32_t)L.HW; a->WPP = (uint32_t)L.WPP;
    a->qv = (uint32_t)qv;
    a->S = best_S; a->S_log2 = best_log;
    a->ppw = 64u / best_S;
    a->upb = (uint32_t)upb; a->upb_log2 = upb_log;
    a->nb = (uint32_t)L.nb;
    *grid = (uint32_t)((L.P + a->ppw - 1) / a->ppw);
    return true;
}

// 1-D maps the register kernel would take as well: compress_line is the faster one for 2-byte
// elements (it loads 16 bytes per lane, the register kernel 8); for fp32 the register kernel is (by 5-10 %)
bool line_first(const Layout& L, size_t es) { return es == 2 || L.HW / 4 < 512; }

// Fills the any-block-size compress plan; false when a plane does not fit LDS or the 32-bit index tricks.
// Hs = rows of one depth slice, D = depth slices (1 for a 2-D map).
bool plan_rows(const Layout& L, int64_t D, int64_t Hs, int64_t W, int B, int b, size_t es, const void* x,
               RowsArgs* a, uint32_t* grid, size_t* lds) {
    (void)b;
    const int64_t H = D * Hs;                       // rows of all slices
    if ((uint64_t)B > L.HW + 64) return false;      // keeps fdiv(r, B) exact; such a B is "one block" anyway: see below
    const uint64_t per_plane = 4ull * L.HW + 16ull * (uint64_t)H * L.LW + 12ull * L.nb + 16ull;
    if (per_plane + 256 > kLdsMax) return false;
    if (!fastdiv_ok(L.HW, (uint64_t)W) || !fastdiv_ok((uint64_t)(H > W ? H : W), (uint64_t)B)) return false;
    if (!fastdiv_ok((uint64_t)H, (uint64_t)Hs) || !fastdiv_ok(L.LD * L.LH, L.LH)) return false;
    uint64_t G = kRowsLdsTarget / per_plane;
    if (G < 1) G = 1;
    if (G > L.P) G = L.P;
    // chunk starts on 16-byte boundaries when G is a multiple of `unit`
    const uint64_t unit = 16 / gcd_u64(16, L.HW * es);
    uint32_t vec_load = ((uintptr_t)x % 16) == 0;
    if (vec_load && G % unit != 0) {
        if (G > unit) G -= G % unit;
        else if (unit * per_plane + 256 <= kLdsMax && unit <= L.P) G = unit;
        else if (G < L.P) vec_load = 0;
    }
    const uint64_t HLW = (uint64_t)H * L.LW;
    if (!fastdiv_ok(G * HLW + kThreads, HLW) || !fastdiv_ok(HLW, L.LW) || !fastdiv_ok(G * L.nb + kThreads, L.nb) ||
        !fastdiv_ok(L.nb, L.LW) || !fastdiv_ok(G * L.WPP + kThreads, L.WPP))
        return false;
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW;
    a->LH = (uint32_t)(L.LD * L.LH); a->LW = (uint32_t)L.LW; a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP; a->B = (uint32_t)B;
    a->D = (uint32_t)D; a->Hs = (uint32_t)Hs; a->LHs = (uint32_t)L.LH;
    a->G = (uint32_t)G;
    a->xs_floats = (uint32_t)((G * L.HW + 3) / 4 * 4);
    a->vec_load = vec_load;
    const uint64_t epv = 16 / es;
    a->keep = vec_load && (uint64_t)W % epv == 0 && G * (L.HW / epv) <= (uint64_t)kRowsKeep * kThreads;
    a->vecblk = a->keep && (uint64_t)B % epv == 0;
    a->qv = (uint32_t)(L.HW / epv);
    a->d_qv = make_fastdiv(a->qv ? a->qv : 1u);
    a->d_W = make_fastdiv((uint32_t)W);
    a->d_B = make_fastdiv((uint32_t)B);
    a->d_Hs = make_fastdiv((uint32_t)Hs);
    a->d_LHs = make_fastdiv((uint32_t)L.LH);
    a->d_LW = make_fastdiv((uint32_t)L.LW);
    a->d_HLW = make_fastdiv((uint32_t)HLW);
    a->d_nb = make_fastdiv((uint32_t)L.nb);
    a->d_wpp = make_fastdiv((uint32_t)L.WPP);
    *lds = 16ull * G + 4ull * a->xs_floats + 16ull * G * HLW + 4ull * ((G * L.nb + 1) & ~1ull) + 8ull * G * L.nb + 16;
    *grid = (uint32_t)((L.P + G - 1) / G);
    return *lds <= kLdsMax;
}

// Fills the workgroup-per-plane plan for planes beyond LDS; false when rows or blocks are not whole
// 16-byte vectors or the per-slice partial sums do not fit LDS.
bool plan_plane(const Layout& L, int64_t D, int64_t Hs, int64_t W, int B, size_t es, const void* x,
                PlaneArgs* a, uint32_t* grid, size_t* lds) {
    const uint64_t epv = 16 / es;
    if (((uintptr_t)x % 16) != 0 || (uint64_t)W % epv != 0 || (uint64_t)B % epv != 0) return false;
    const uint64_t H = (uint64_t)D * (uint64_t)Hs;
    const uint64_t slice = L.LH * L.LW;
    const uint64_t nitem = (uint64_t)D * slice;
    const uint64_t need = 16ull * nitem + 4ull * ((L.nb + 3) & ~3ull) + 8ull * (kThreads / 64) + 16 + 16;
    if (need > kLdsMax) return false;
    if (!fastdiv_ok(L.HW, (uint64_t)W) || !fastdiv_ok(H > (uint64_t)W ? H : (uint64_t)W, (uint64_t)B) ||
        !fastdiv_ok(H, (uint64_t)Hs) || !fastdiv_ok(nitem + kThreads, slice) || !fastdiv_ok(slice, L.LW))
        return false;
    a->P = (uint32_t)L.P; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW; a->LW = (uint32_t)L.LW;
    a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP; a->B = (uint32_t)B;
    a->D = (uint32_t)D; a->Hs = (uint32_t)Hs; a->LHs = (uint32_t)L.LH;
    a->nitem = (uint32_t)nitem;
    a->qv = (uint32_t)(L.HW / epv);
    a->d_W = make_fastdiv((uint32_t)W);
    a->d_B = make_fastdiv((uint32_t)B);
    a->d_Hs = make_fastdiv((uint32_t)Hs);
    a->d_LW = make_fastdiv((uint32_t)L.LW);
    a->d_LHs = make_fastdiv((uint32_t)L.LH);
    a->d_slice = make_fastdiv((uint32_t)slice);
    *lds = need;
    *grid = (uint32_t)L.P;
    return true;
}

// Fills the tiled-compress launch plan; false when the shape is not covered.
bool plan_tile(const Layout& L, int64_t H, int64_t W, int B, int b, size_t es, const void* x,
               TileArgs* a, uint32_t* grid, size_t* lds, int* vec_out, int* nt_out) {
    if (B != 4 && B != 8) return false;
    const int vec = (W % 4 == 0) ? 4 : (W % 2 == 0) ? 2 : 1;
    const uint32_t ipb = (uint32_t)B / (uint32_t)vec;
    const uint64_t slots = ((uint64_t)W + vec - 1) / vec;
    const uint64_t ipr = (slots + ipb - 1) / ipb * ipb;
    const uint64_t ipp = L.LH * ipr;
    const uint64_t per_plane = 4ull * L.HW + 8ull * ipp + 16ull;
    if (per_plane + 64 > kLdsMax) return false;
    const int nt = 256;
    uint64_t Gmax = kLdsTarget / per_plane;
    if (Gmax < 1) Gmax = 1;
    if (Gmax > L.P) Gmax = L.P;
    // chunk starts stay 16-byte aligned when G * (bytes per plane) is a multiple of 16
    const uint64_t unit = 16 / gcd_u64(16, L.HW * es);
    uint32_t vec_load = ((uintptr_t)x % 16) == 0;
    if (vec_load && unit > 1 && Gmax < unit && Gmax < L.P) {
        if (unit * per_plane + 64 <= kLdsMax) Gmax = unit; else vec_load = 0;
    }
    const uint64_t step = vec_load ? unit : 1;
    // pick the G whose last, partly filled wavefront pass wastes the fewest lanes
    const double c1 = 4.0 * B * vec, c3 = 7.5 * (32 / b);
    uint64_t G = 0;
    double best = 0;
    for (uint64_t g = step; g <= Gmax; g += step) {
        const double cost = (double)((g * ipp + 63) / 64) * c1 + (double)((g * L.WPP + 63) / 64) * c3;
        const double per_elt = cost / (double)(g * L.HW);
        if (G == 0 || per_elt < best * 0.98) { G = g; best = per_elt; }
    }
    if (G == 0) G = Gmax;          // Gmax == P < unit: a single chunk, aligned at its start
    const uint64_t nitems = G * ipp, nwords = G * L.WPP;
    if (!fastdiv_ok(nitems + 256, ipp) || !fastdiv_ok(ipp, ipr) || !fastdiv_ok(nwords + 256, L.WPP))
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
    *nt_out = nt;
    return *lds <= kLdsMax;
}

// LDS bytes of the streaming decompress kernels for G planes per workgroup
size_t dec_lds_bytes(const Layout& L, size_t es, uint64_t G) {
    return 4ull * ((G * L.WPP + 3) & ~(uint64_t)3) + 8ull * G + es * G * L.nb + 16;
}
constexpr size_t kDecLdsMax = 60u << 10;

// Planes per workgroup of the streaming decompress kernels: about 32 KB of output, in whole 128-byte
// lines where that is possible within twice the target, so that no line is shared by two
// workgroups.  Measured inside a whole compress + decompress step over the ResNet-50 set: 24-48 KB
// is the flat optimum (64 KB: 0.5-1 % slower, 12 KB: 4 % slower, 6 KB: 12 %).  A decompress kernel
// timed on its own, launch after launch, prefers 12 KB by 15 %, but not between other kernels.
// `mult`: G must be a multiple of it (flat kernel: whole 4-element vectors).
constexpr uint64_t kDecChunkBytes = 32768;
uint64_t dec_planes(const Layout& L, size_t es, uint64_t mult) {
    const uint64_t target = kDecChunkBytes / es;
    uint64_t G = (target + L.HW / 2) / L.HW;
    if (G < 1) G = 1;
    uint64_t unit = 128 / gcd_u64(128, L.HW * es);
    unit = unit / gcd_u64(unit, mult) * mult;
    if (unit * L.HW > 2 * target) unit = mult;
    G = (G + unit / 2) / unit * unit;
    if (G < unit) G = unit;
    if (G > L.P) G = L.P;
    return G;
}

// Fills the decompress launch plan; returns 0 (row vectors), 3 (block table), 6 (four consecutive elements
// per lane step, any width), 5 (word by word through LDS), 1 (flat), 4 (lane per plane) or 2 (scalar).
// Hs = rows of one depth slice, D = depth slices (1 for a 2-D map; the table kernel takes 2-D maps only).
int plan_decompress(const Layout& L, int64_t D, int64_t Hs, int64_t W, int B, size_t es, const void* xhat,
                    DecArgs* a, uint32_t* grid) {
    const int64_t H = D * Hs;
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW;
    a->LH = (uint32_t)(L.LD * L.LH); a->LW = (uint32_t)L.LW; a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP; a->B = (uint32_t)B;
    a->Hs = (uint32_t)Hs; a->LHs = (uint32_t)L.LH;
    a->d_B = make_fastdiv((uint32_t)B);
    a->d_W = make_fastdiv((uint32_t)W);
    a->d_HW = make_fastdiv((uint32_t)L.HW);
    a->d_Hs = make_fastdiv((uint32_t)Hs);
    const bool small_idx = fastdiv_ok((uint64_t)H, (uint64_t)B) && fastdiv_ok((uint64_t)W, (uint64_t)B) &&
                           fastdiv_ok((uint64_t)H, (uint64_t)Hs);
    const bool out_vec_aligned = ((uintptr_t)xhat % (4 * es)) == 0;
    // one-block planes with an odd element count: a lane per plane, 64 planes per round
    if (lane_shape(L)) {
        const uint32_t nrounds = (uint32_t)((L.P + 63) / 64);
        uint32_t rpw = 2;
        while (rpw > 1 && nrounds / rpw < 32u * (uint32_t)num_cus()) --rpw;
        a->G = rpw;
        *grid = (nrounds + rpw - 1) / rpw;
        return 4;
    }
    // fast path: rows are whole vectors that sit inside one block
    if (W % 4 == 0 && B % 4 == 0 && small_idx && out_vec_aligned) {
        a->q4 = (uint32_t)(L.HW / 4);
        a->w4 = (uint32_t)(W / 4);
        uint64_t G = dec_planes(L, es, 1);
        while (G > 1 && !fastdiv_ok(G * a->q4 + kThreads, a->q4)) --G;
        if (fastdiv_ok(G * a->q4 + kThreads, a->q4) && fastdiv_ok(a->q4, a->w4) && dec_lds_bytes(L, es, G) <= kDecLdsMax) {
            a->G = (uint32_t)G;
            a->d_q4 = make_fastdiv(a->q4);
            a->d_w4 = make_fastdiv(a->w4);
            a->pair8 = es == 2 && W % 8 == 0 && ((uintptr_t)xhat % 16) == 0;
            *grid = (uint32_t)((L.P + G - 1) / G);
            return 0;
        }
    }
    // planes of whole vectors with few blocks: LFC indices from a table in LDS
    if (D == 1 && L.HW % 4 == 0 && L.nb > 1 && L.nb <= 255 && small_idx && out_vec_aligned && fastdiv_ok(L.HW, (uint64_t)W)) {
        a->q4 = (uint32_t)(L.HW / 4);
        uint64_t G = dec_planes(L, es, 1);
        while (G > 1 && !fastdiv_ok(G * a->q4 + kThreads, a->q4)) --G;
        if (fastdiv_ok(G * a->q4 + kThreads, a->q4) && dec_lds_bytes(L, es, G) + 4ull * a->q4 + 16 <= kDecLdsMax) {
            a->G = (uint32_t)G;
            a->d_q4 = make_fastdiv(a->q4);
            *grid = (uint32_t)((L.P + G - 1) / G);
            return 3;
        }
    }
    // 2-D planes of 512 elements and more whose rows or blocks are not whole vectors: four consecutive
    // elements per lane step, planes starting on 4-byte boundaries
    if (D == 1 && Hs > 1 && small_idx && ((uintptr_t)xhat % 4) == 0 && L.nb <= 16383) {
        const uint64_t q4 = (L.HW + 3) / 4;
        int nw = 1;
        while (nw < 16 && (q4 > (uint64_t)kUnitsK * 64 * nw || L.nb > (uint64_t)kUnitsLfc * 64 * nw)) nw *= 2;
        const uint64_t nt = 64ull * nw;
        if (q4 >= kUnitsMin && q4 <= (uint64_t)kUnitsK * nt && L.nb <= (uint64_t)kUnitsLfc * nt &&
            fastdiv_ok(4ull * kUnitsK * nt + 4, (uint64_t)W) && fastdiv_ok(4ull * kUnitsK * nt + 4, (uint64_t)B)) {
            a->q4 = (uint32_t)q4;
            a->G = (uint32_t)nw;                  // wavefronts per workgroup
            uint64_t g = (uint64_t)num_cus() * (16ull / nw);
            g += g & 1;
            *grid = (uint32_t)(g < L.P ? g : L.P);
            return 6;
        }
    }
    // several blocks per plane, rows not whole vectors: rebuilt in LDS word by word
    if (L.nb > 1 && small_idx && out_vec_aligned && fastdiv_ok(L.HW, (uint64_t)W)) {
        const uint64_t unit = 4 / gcd_u64(4, L.HW);
        uint64_t G = dec_planes(L, 4, unit);          // the chunk is staged as fp32 whatever the element type
        const uint64_t staged = (dec_lds_bytes(L, es, G) + 15) & ~15ull;
        if (fastdiv_ok(G * L.WPP + kThreads, L.WPP) && staged + 4ull * ((G * L.HW + 3) & ~3ull) <= kDecLdsMax) {
            a->G = (uint32_t)G;
            a->out_off = (uint32_t)staged;
            a->d_wpp = make_fastdiv((uint32_t)L.WPP);
            *grid = (uint32_t)((L.P + G - 1) / G);
            return 5;
        }
    }
    // general path: flat run of G planes, G*HW a multiple of 4
    if (small_idx && out_vec_aligned && fastdiv_ok(L.HW, (uint64_t)W)) {
        const uint64_t unit = 4 / gcd_u64(4, L.HW);
        const uint64_t G = dec_planes(L, es, unit);
        if (fastdiv_ok(G * L.HW + 4ull * kThreads, L.HW) && dec_lds_bytes(L, es, G) <= kDecLdsMax) {
            a->G = (uint32_t)G;
            *grid = (uint32_t)((L.P + G - 1) / G);
            return 1;
        }
    }
    a->G = 1;
    *grid = (uint32_t)L.P;
    return 2;
}

// calls f(T{}, std::integral_constant<int, BITS>{}) for the element / cache type and code width of a call
// calls f(std::integral_constant<int, BITS>{}) for the code width of a call
template <typename F>
hipError_t with_bits(int b, F&& f) {
    return b == 2 ? f(std::integral_constant<int, 2>{}) : b == 4 ? f(std::integral_constant<int, 4>{})
                                                                  : f(std::integral_constant<int, 8>{});
}

enum CompKind { REGS, LANE, LINE, ITEMS, UNITS, WAVE, TILE, ONE, ROWS, PLANE, ANY };

// everything a compress launch needs once the plan is made (the arguments of the kernel that was picked)
struct CompLaunch {
    int kind, B, vec, nt, nw, flat;
    uint32_t gx, gy;
    size_t lds;
    hipStream_t st;
    TileArgs a; WaveArgs wa; RegsArgs ra; ItemsArgs ia; LaneArgs la; RowsArgs wa2; PlaneArgs pa; OneArgs oa; AnyArgs g; UnitsArgs ua;
};
struct DecLaunch {
    int kind, flat, nw;
    uint32_t gx, gy;
    size_t lds;
    hipStream_t st;
    DecArgs a;
};

template <typename T>
hipError_t do_compress(const CompLaunch& c, int b) {
    const dim3 gd(c.gx, c.gy);
    hipStream_t st = c.st;
    const size_t lds = c.lds;
    const bool flat = c.flat != 0;
    return with_bits(b, [&](auto bits) -> hipError_t {
        constexpr int BITS = decltype(bits)::value;
        switch (c.kind) {
            case REGS: return launch_regs<T, BITS>(c.B, c.nw, c.ra, gd, lds, st);
            case ITEMS: return launch_items<T, BITS>(c.B, c.vec, c.ia, gd, lds, st);
            case UNITS: return launch_units<T, BITS>(c.nw, c.ua, gd, lds, st);
            case WAVE: return launch_wave<T, BITS>(c.B, c.vec, c.wa, gd, lds, st);
            case TILE: return launch_tile<T, BITS>(c.B, c.vec, c.a, gd, lds, st);
            case LANE: hipLaunchKernelGGL((compress_lane<T, BITS>), gd, dim3(64), lds, st, c.la); return hipGetLastError();
            case ONE: hipLaunchKernelGGL((compress_one<T, BITS>), gd, dim3(64), 0, st, c.oa); return hipGetLastError();
            case LINE: hipLaunchKernelGGL((compress_line<T, BITS>), gd, dim3(64), 0, st, c.oa); return hipGetLastError();
            case ROWS: {
                void (*kern)(RowsArgs) = flat ? compress_rows<T, BITS> : compress_rows_3d<T, BITS>;
                const hipError_t e = allow_large_lds(kern, lds);
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL(kern, gd, dim3(kThreads), lds, st, c.wa2);
                return hipGetLastError();
            }
            case PLANE: {
                void (*kern)(PlaneArgs) = flat ? compress_plane<T, BITS> : compress_plane_3d<T, BITS>;
                const hipError_t e = allow_large_lds(kern, lds);
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL(kern, gd, dim3(kThreads), lds, st, c.pa);
                return hipGetLastError();
            }
            default: {
                void (*kern)(AnyArgs) = flat ? compress_any<T, BITS> : compress_any_3d<T, BITS>;
                hipLaunchKernelGGL(kern, gd, dim3(kThreads), 0, st, c.g);
                return hipGetLastError();
            }
        }
    });
}

template <typename T>
hipError_t do_decompress(const DecLaunch& c, int b) {
    return with_bits(b, [&](auto bits) -> hipError_t {
        constexpr int BITS = decltype(bits)::value;
        const int kind = c.kind;
        void (*kern)(DecArgs);
        if (kind == 6) {
            kern = c.nw == 1 ? decompress_units<T, BITS, 1> : c.nw == 2 ? decompress_units<T, BITS, 2>
                 : c.nw == 4 ? decompress_units<T, BITS, 4> : c.nw == 8 ? decompress_units<T, BITS, 8>
                                                                        : decompress_units<T, BITS, 16>;
            hipLaunchKernelGGL(kern, dim3(c.gx, c.gy), dim3(64 * c.nw), c.lds, c.st, c.a);
            return hipGetLastError();
        }
        if (c.flat)
            kern = kind == 0 ? decompress_rowvec<T, BITS> : kind == 3 ? decompress_table<T, BITS>
                 : kind == 5 ? decompress_words<T, BITS> : kind == 1 ? decompress_flat<T, BITS>
                 : kind == 4 ? decompress_lane<T, BITS> : decompress_scalar<T, BITS>;
        else
            kern = kind == 0 ? decompress_rowvec_3d<T, BITS> : kind == 5 ? decompress_words_3d<T, BITS>
                 : kind == 1 ? decompress_flat_3d<T, BITS>
                 : kind == 4 ? decompress_lane<T, BITS> : decompress_scalar_3d<T, BITS>;
        const hipError_t e = allow_large_lds(kern, c.lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3(c.gx, c.gy), dim3(kind == 4 ? 64 : kThreads), c.lds, c.st, c.a);
        return hipGetLastError();
    });
}

// the Relu + compress kernel of the register kernel's planes (one map per launch; c.ra carries y and mask)
template <typename T>
hipError_t do_relu(const CompLaunch& c, int b) {
    return with_bits(b, [&](auto bits) -> hipError_t {
        constexpr int BITS = decltype(bits)::value;
        void (*kern)(RegsArgs);
        if (c.nw == 1) kern = c.B == 8 ? relu_compress_regs<T, BITS, 8, 1> : relu_compress_regs<T, BITS, 4, 1>;
        else kern = c.B == 8 ? relu_compress_regs<T, BITS, 8, 4> : relu_compress_regs<T, BITS, 4, 4>;
        hipLaunchKernelGGL(kern, dim3(c.gx, 1), dim3(64 * c.nw), c.lds, c.st, c.ra);
        return hipGetLastError();
    });
}

hipError_t bridge_compress(division_dtype dt, const CompLaunch& c, int b) {
    return dt == DIVISION_F32 ? division_bridge_compress_f32(&c, b)
         : dt == DIVISION_BF16 ? division_bridge_compress_bf16(&c, b) : division_bridge_compress_c16(&c, b);
}
hipError_t bridge_decompress(division_dtype dt, const DecLaunch& c, int b) {
    return dt == DIVISION_F32 ? division_bridge_decompress_f32(&c, b)
         : dt == DIVISION_BF16 ? division_bridge_decompress_bf16(&c, b) : division_bridge_decompress_c16(&c, b);
}
hipError_t bridge_relu(division_dtype dt, const CompLaunch& c, int b) {
    return dt == DIVISION_F32 ? division_bridge_relu_f32(&c, b)
         : dt == DIVISION_BF16 ? division_bridge_relu_bf16(&c, b) : division_bridge_relu_c16(&c, b);
}

// A 3-D map with a dimension of extent 1 is a 2-D map with the same flat element order, the same
// blocks and the same packed buffer: D x 1 x W -> D x W, D x H x 1 -> D x H.  (1 x H x W needs nothing.)
void squeeze_dims(int64_t& D, int64_t& H, int64_t& W) {
    if (D > 1 && H == 1) { H = D; D = 1; }
    else if (D > 1 && W == 1) { W = H; H = D; D = 1; }
}

// A plane that is a single block has the same cached tuple under every block size that covers it:
// small 2-D planes are handed to the kernels specialised for B = 4 and B = 8.
int covering_block(const Layout& L, int64_t D, int64_t H, int64_t W, int B) {
    if (L.nb != 1 || D != 1) return B;
    const int64_t m = H > W ? H : W;
    return m <= 4 ? 4 : m <= 8 ? 8 : B;
}

int packed_layout_impl(int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int B, int b, division_dtype dt,
                       size_t* codes_off, size_t* codes_bytes, size_t* meta_off, size_t* meta_bytes,
                       size_t* lfc_off, size_t* lfc_bytes) {
    if (!codes_off || !codes_bytes || !meta_off || !meta_bytes || !lfc_off || !lfc_bytes) return DIVISION_EINVAL;
    Layout L;
    if (make_layout(N, C, D, H, W, B, b, (int)dt, &L) != DIVISION_OK) return DIVISION_EINVAL;
    *codes_off = L.codes_off; *codes_bytes = L.codes_bytes;
    *meta_off = L.meta_off;   *meta_bytes = L.meta_bytes;
    *lfc_off = L.lfc_off;     *lfc_bytes = L.lfc_bytes;
    return DIVISION_OK;
}

int compress_impl(int count, const void* const* x, void* const* packed, const uint64_t* seeds,
                  int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, division_dtype dt,
                  int B, int b, size_t packed_capacity, void* hip_stream) {
    if (count < 0 || (count > 0 && (!x || !packed || !seeds))) return DIVISION_EINVAL;
    squeeze_dims(D, H, W);
    Layout L;
    const int rc = make_layout(N, C, D, H, W, B, b, (int)dt, &L);
    if (rc != DIVISION_OK) return rc;
    B = covering_block(L, D, H, W, B);
    if (packed_capacity < L.total) return DIVISION_ESIZE;
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    uintptr_t all_x = 0;            // alignment of the batch = alignment of the OR of its pointers
    for (int i = 0; i < count; ++i) {
        if (!x[i] || !packed[i]) return DIVISION_EINVAL;
        if (((uintptr_t)x[i] % es) != 0 || ((uintptr_t)packed[i] % 16) != 0) return DIVISION_EALIGN;
        all_x |= (uintptr_t)x[i];
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const void* xa = reinterpret_cast<const void*>(all_x ? all_x : 16);
    const Regions rg = make_regions(L);

    for (int i0 = 0; i0 < count; i0 += kMaxBatch) {
        const int cnt = count - i0 < kMaxBatch ? count - i0 : kMaxBatch;
        CompTab tab{};
        for (int i = 0; i < cnt; ++i) {
            tab.x[i] = x[i0 + i];
            tab.pk[i] = packed[i0 + i];
            tab.seed_a[i] = mix32((uint32_t)(seeds[i0 + i] & 0xffffffffu) ^ 0x243F6A88u);
            tab.seed_c[i] = mix32((uint32_t)(seeds[i0 + i] >> 32) ^ 0x85A308D3u);
        }
        TileArgs a{};
        WaveArgs wa{};
        RegsArgs ra{};
        ItemsArgs ia{};
        LaneArgs la{};
        RowsArgs wa2{};
        PlaneArgs pa{};
        OneArgs oa{};
        AnyArgs g{};
        UnitsArgs ua{};
        size_t lds = 0;
        uint32_t grid = 0;
        int vec = 1, nt = 64, nw = 1;
        CompKind kind;
        const bool flat = D == 1;               // the register, item, wavefront and tile kernels take 2-D maps
        if (line_first(L, es) && plan_line(L, D, H, B, es, xa, &oa, &grid)) { kind = LINE; oa.tab = tab; oa.rg = rg; lds = 0; }
        else if (plan_regs(L, D, H, W, B, es, xa, &ra, &grid, &lds, &nw)) { kind = REGS; ra.tab = tab; ra.rg = rg; }
        else if (plan_lane(L, es, xa, &la, &grid, &lds)) { kind = LANE; la.tab = tab; la.rg = rg; }
        else if (plan_line(L, D, H, B, es, xa, &oa, &grid)) { kind = LINE; oa.tab = tab; oa.rg = rg; lds = 0; }
        else if (flat && plan_items(L, H, W, B, es, xa, &ia, &grid, &lds, &vec)) { kind = ITEMS; ia.tab = tab; ia.rg = rg; }
        else if (!one_shape(L, es, xa) && plan_units(L, D, H, W, B, es, xa, &ua, &grid, &lds, &nw)) { kind = UNITS; ua.tab = tab; ua.rg = rg; }
        else if (flat && plan_wave(L, H, W, B, b, es, xa, &wa, &grid, &lds, &vec)) {
            kind = WAVE; wa.tab = tab; wa.rg = rg;
        } else if (flat && plan_tile(L, H, W, B, b, es, xa, &a, &grid, &lds, &vec, &nt)) { kind = TILE; a.tab = tab; a.rg = rg; }
        else if (plan_one(L, es, xa, &oa, &grid)) { kind = ONE; oa.tab = tab; oa.rg = rg; lds = 0; }
        else if (plan_rows(L, D, H, W, B, b, es, xa, &wa2, &grid, &lds)) { kind = ROWS; wa2.tab = tab; wa2.rg = rg; }
        else if (plan_plane(L, D, H, W, B, es, xa, &pa, &grid, &lds)) { kind = PLANE; pa.tab = tab; pa.rg = rg; }
        else {
            kind = ANY;
            g.tab = tab; g.rg = rg;
            g.P = (uint32_t)L.P; g.H = (uint32_t)H; g.W = (uint32_t)W; g.HW = (uint32_t)L.HW; g.D = (uint32_t)D;
            g.LH = (uint32_t)L.LH; g.LW = (uint32_t)L.LW; g.nb = (uint32_t)L.nb; g.WPP = (uint32_t)L.WPP; g.B = (uint32_t)B;
            grid = (uint32_t)L.P;
        }
        CompLaunch c{};
        c.kind = kind; c.B = B; c.vec = vec; c.nt = nt; c.nw = nw; c.flat = flat;
        c.gx = grid; c.gy = (uint32_t)cnt; c.lds = lds; c.st = st;
        c.a = a; c.wa = wa; c.ra = ra; c.ia = ia; c.la = la; c.wa2 = wa2; c.pa = pa; c.oa = oa; c.g = g; c.ua = ua;
        const hipError_t err = bridge_compress(dt, c, b);
        if (err != hipSuccess) return DIVISION_EHIP;
    }
    return DIVISION_OK;
}

int decompress_impl(int count, const void* const* packed, void* const* xhat, size_t packed_bytes,
                    int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, division_dtype dt,
                    int B, int b, void* hip_stream) {
    if (count < 0 || (count > 0 && (!packed || !xhat))) return DIVISION_EINVAL;
    squeeze_dims(D, H, W);
    Layout L;
    const int rc = make_layout(N, C, D, H, W, B, b, (int)dt, &L);
    if (rc != DIVISION_OK) return rc;
    B = covering_block(L, D, H, W, B);
    if (packed_bytes < L.total) return DIVISION_ESIZE;
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    uintptr_t all_out = 0;
    for (int i = 0; i < count; ++i) {
        if (!xhat[i] || !packed[i]) return DIVISION_EINVAL;
        if (((uintptr_t)xhat[i] % es) != 0 || ((uintptr_t)packed[i] % 16) != 0) return DIVISION_EALIGN;
        all_out |= (uintptr_t)xhat[i];
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const Regions rg = make_regions(L);

    for (int i0 = 0; i0 < count; i0 += kMaxBatch) {
        const int cnt = count - i0 < kMaxBatch ? count - i0 : kMaxBatch;
        DecArgs a{};
        uint32_t grid = 0;
        const int kind = plan_decompress(L, D, H, W, B, es, reinterpret_cast<const void*>(all_out ? all_out : 16), &a, &grid);
        for (int i = 0; i < cnt; ++i) { a.tab.pk[i] = packed[i0 + i]; a.tab.xhat[i] = xhat[i0 + i]; }
        a.rg = rg;
        // LDS of the streaming kernels: staged codes, meta and LFC of G planes (+ the block table)
        size_t lds = 0;
        if (kind == 4) lds = 4ull * (64ull * L.HW + 4);
        else if (kind == 6) lds = 8ull * ((L.nb + 3) & ~3ull);
        else if (kind == 5) lds = a.out_off + 4ull * ((a.G * L.HW + 3) & ~3ull);
        else if (kind != 2) lds = dec_lds_bytes(L, es, a.G) + (kind == 3 ? 4ull * a.q4 + 16 : 0);
        DecLaunch c{};
        c.kind = kind; c.flat = D == 1; c.nw = kind == 6 ? (int)a.G : 0; c.gx = grid; c.gy = (uint32_t)cnt; c.lds = lds; c.st = st; c.a = a;
        if (bridge_decompress(dt, c, b) != hipSuccess) return DIVISION_EHIP;
    }
    return DIVISION_OK;
}

int kernel_name_impl(int direction, const void* data, int64_t N, int64_t C, int64_t D, int64_t H, int64_t W,
                     division_dtype dt, int B, int b, char* out, size_t cap) {
    if (!out || cap == 0) return DIVISION_EINVAL;
    squeeze_dims(D, H, W);
    Layout L;
    const int rc = make_layout(N, C, D, H, W, B, b, (int)dt, &L);
    if (rc != DIVISION_OK) return rc;
    B = covering_block(L, D, H, W, B);
    const bool flat = D == 1;
    const char* sfx = flat ? "" : "_3d";
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    const char* tn = dt == DIVISION_BF16 ? "bf16_t" : dt == DIVISION_F32_C16 ? "f32c16_t" : "float";
    int n;
    if (direction == 0) {
        TileArgs a{}; WaveArgs wa{}; RegsArgs ra{}; ItemsArgs ia{}; LaneArgs la{}; RowsArgs wa2{}; PlaneArgs pa{}; OneArgs oa{}; UnitsArgs ua{}; size_t lds = 0; uint32_t grid = 0; int vec = 1, nt = 64, nw = 1;
        if (line_first(L, es) && plan_line(L, D, H, B, es, data, &oa, &grid))
            n = snprintf(out, cap, "compress_line<%s, %d>", tn, b);
        else if (plan_regs(L, D, H, W, B, es, data, &ra, &grid, &lds, &nw))
            n = snprintf(out, cap, "compress_regs%s<%s, %d, %d, %d>", sfx, tn, b, (B == 4 || B == 8) ? B : 0, nw);
        else if (plan_lane(L, es, data, &la, &grid, &lds))
            n = snprintf(out, cap, "compress_lane<%s, %d>", tn, b);
        else if (plan_line(L, D, H, B, es, data, &oa, &grid))
            n = snprintf(out, cap, "compress_line<%s, %d>", tn, b);
        else if (flat && plan_items(L, H, W, B, es, data, &ia, &grid, &lds, &vec))
            n = snprintf(out, cap, "compress_items<%s, %d, %d, %d, %d>", tn, b, B, vec, H == 1 ? 1 : B);
        else if (!one_shape(L, es, data) && plan_units(L, D, H, W, B, es, data, &ua, &grid, &lds, &nw))
            n = snprintf(out, cap, "compress_units<%s, %d, %d>", tn, b, nw);
        else if (flat && plan_wave(L, H, W, B, b, es, data, &wa, &grid, &lds, &vec))
            n = snprintf(out, cap, "compress_wave<%s, %d, %d, %d>", tn, b, B, vec);
        else if (flat && plan_tile(L, H, W, B, b, es, data, &a, &grid, &lds, &vec, &nt))
            n = snprintf(out, cap, "compress_tile<%s, %d, %d, %d, %d>", tn, b, B, vec, nt);
        else if (plan_one(L, es, data, &oa, &grid))
            n = snprintf(out, cap, "compress_one<%s, %d>", tn, b);
        else if (plan_rows(L, D, H, W, B, b, es, data, &wa2, &grid, &lds))
            n = snprintf(out, cap, "compress_rows%s<%s, %d>", sfx, tn, b);
        else if (plan_plane(L, D, H, W, B, es, data, &pa, &grid, &lds))
            n = snprintf(out, cap, "compress_plane%s<%s, %d>", sfx, tn, b);
        else
            n = snprintf(out, cap, "compress_any%s<%s, %d>", sfx, tn, b);
    } else {
        DecArgs a{}; uint32_t grid = 0;
        const int kind = plan_decompress(L, D, H, W, B, es, data, &a, &grid);
        if (kind == 6)
            n = snprintf(out, cap, "decompress_units<%s, %d, %d>", tn, b, (int)a.G);
        else
            n = snprintf(out, cap, "%s%s<%s, %d>", kind == 0 ? "decompress_rowvec" : kind == 3 ? "decompress_table" : kind == 5 ? "decompress_words" : kind == 1 ? "decompress_flat" : kind == 4 ? "decompress_lane" : "decompress_scalar",
                         kind == 4 ? "" : sfx, tn, b);
    }
    return (n < 0 || (size_t)n >= cap) ? DIVISION_ESIZE : DIVISION_OK;
}

}  // namespace

// ------------------------------------------------------------------ bridges: the kernels of one type each

#if DIVISION_HAS_F32
hipError_t division_bridge_compress_f32(const void* c, int b) { return do_compress<float>(*static_cast<const CompLaunch*>(c), b); }
hipError_t division_bridge_decompress_f32(const void* c, int b) { return do_decompress<float>(*static_cast<const DecLaunch*>(c), b); }
hipError_t division_bridge_relu_f32(const void* c, int b) { return do_relu<float>(*static_cast<const CompLaunch*>(c), b); }
#endif
#if DIVISION_HAS_BF16
hipError_t division_bridge_compress_bf16(const void* c, int b) { return do_compress<bf16_t>(*static_cast<const CompLaunch*>(c), b); }
hipError_t division_bridge_decompress_bf16(const void* c, int b) { return do_decompress<bf16_t>(*static_cast<const DecLaunch*>(c), b); }
hipError_t division_bridge_relu_bf16(const void* c, int b) { return do_relu<bf16_t>(*static_cast<const CompLaunch*>(c), b); }
#endif
#if DIVISION_HAS_C16
hipError_t division_bridge_compress_c16(const void* c, int b) { return do_compress<f32c16_t>(*static_cast<const CompLaunch*>(c), b); }
hipError_t division_bridge_decompress_c16(const void* c, int b) { return do_decompress<f32c16_t>(*static_cast<const DecLaunch*>(c), b); }
hipError_t division_bridge_relu_c16(const void* c, int b) { return do_relu<f32c16_t>(*static_cast<const CompLaunch*>(c), b); }
#endif

// ------------------------------------------------------------------ C ABI

#if DIVISION_HOST
extern "C" {

int division_abi_version(void) { return 1; }

size_t division_packed_bytes(int64_t N, int64_t C, int64_t H, int64_t W, int B, int b, division_dtype dt) {
    Layout L;
    if (make_layout(N, C, 1, H, W, B, b, (int)dt, &L) != DIVISION_OK) return 0;
    return L.total;
}

size_t division_packed_bytes_3d(int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int B, int b, division_dtype dt) {
    Layout L;
    if (make_layout(N, C, D, H, W, B, b, (int)dt, &L) != DIVISION_OK) return 0;
    return L.total;
}

int division_packed_layout(int64_t N, int64_t C, int64_t H, int64_t W, int B, int b, division_dtype dt,
                           size_t* codes_off, size_t* codes_bytes, size_t* meta_off, size_t* meta_bytes,
                           size_t* lfc_off, size_t* lfc_bytes) {
    return packed_layout_impl(N, C, 1, H, W, B, b, dt, codes_off, codes_bytes, meta_off, meta_bytes, lfc_off, lfc_bytes);
}

int division_packed_layout_3d(int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int B, int b, division_dtype dt,
                              size_t* codes_off, size_t* codes_bytes, size_t* meta_off, size_t* meta_bytes,
                              size_t* lfc_off, size_t* lfc_bytes) {
    return packed_layout_impl(N, C, D, H, W, B, b, dt, codes_off, codes_bytes, meta_off, meta_bytes, lfc_off, lfc_bytes);
}

int division_compress_batch(int count, const void* const* x, void* const* packed, const uint64_t* seeds,
                            int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt,
                            int B, int b, size_t packed_capacity, void* hip_stream) {
    return compress_impl(count, x, packed, seeds, N, C, 1, H, W, dt, B, b, packed_capacity, hip_stream);
}

int division_compress(const void* x, int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt,
                      int B, int b, uint64_t seed, void* packed, size_t packed_capacity, void* hip_stream) {
    if (!x || !packed) return DIVISION_EINVAL;
    return compress_impl(1, &x, &packed, &seed, N, C, 1, H, W, dt, B, b, packed_capacity, hip_stream);
}

int division_compress_3d(const void* x, int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, division_dtype dt,
                         int B, int b, uint64_t seed, void* packed, size_t packed_capacity, void* hip_stream) {
    if (!x || !packed) return DIVISION_EINVAL;
    return compress_impl(1, &x, &packed, &seed, N, C, D, H, W, dt, B, b, packed_capacity, hip_stream);
}

int division_decompress_batch(int count, const void* const* packed, void* const* xhat, size_t packed_bytes,
                              int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt,
                              int B, int b, void* hip_stream) {
    return decompress_impl(count, packed, xhat, packed_bytes, N, C, 1, H, W, dt, B, b, hip_stream);
}

int division_decompress(const void* packed, size_t packed_bytes, int64_t N, int64_t C, int64_t H, int64_t W,
                        division_dtype dt, int B, int b, void* xhat, void* hip_stream) {
    if (!xhat || !packed) return DIVISION_EINVAL;
    return decompress_impl(1, &packed, &xhat, packed_bytes, N, C, 1, H, W, dt, B, b, hip_stream);
}

int division_decompress_3d(const void* packed, size_t packed_bytes, int64_t N, int64_t C, int64_t D, int64_t H, int64_t W,
                           division_dtype dt, int B, int b, void* xhat, void* hip_stream) {
    if (!xhat || !packed) return DIVISION_EINVAL;
    return decompress_impl(1, &packed, &xhat, packed_bytes, N, C, D, H, W, dt, B, b, hip_stream);
}

int division_relu_compress(const void* x, int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt,
                           int B, int b, uint64_t seed, void* y, void* mask, size_t mask_capacity,
                           void* packed, size_t packed_capacity, void* hip_stream) {
    if (!x || !y || !mask || !packed) return DIVISION_EINVAL;
    Layout L;
    const int rc = make_layout(N, C, 1, H, W, B, b, (int)dt, &L);
    if (rc != DIVISION_OK) return rc;
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    const int64_t n = (int64_t)(L.P * L.HW);
    if (mask_capacity < division_mask_bytes(n) || packed_capacity < L.total) return DIVISION_ESIZE;
    if (((uintptr_t)x % es) != 0 || ((uintptr_t)y % es) != 0 || ((uintptr_t)mask % 4) != 0 || ((uintptr_t)packed % 16) != 0)
        return DIVISION_EALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    // fused: the planes the register kernel takes, when a plane's mask is whole words
    RegsArgs ra{};
    uint32_t grid = 0;
    size_t lds = 0;
    int nw = 1;
    const void* both = reinterpret_cast<const void*>((uintptr_t)x | (uintptr_t)y);
    if (L.HW % 32 == 0 && (B == 4 || B == 8) && plan_regs(L, 1, H, W, B, es, both, &ra, &grid, &lds, &nw) && nw <= 4) {
        ra.tab.x[0] = x;
        ra.tab.pk[0] = packed;
        ra.tab.seed_a[0] = mix32((uint32_t)(seed & 0xffffffffu) ^ 0x243F6A88u);
        ra.tab.seed_c[0] = mix32((uint32_t)(seed >> 32) ^ 0x85A308D3u);
        ra.rg = make_regions(L);
        ra.y = y;
        ra.mask = static_cast<uint32_t*>(mask);
        CompLaunch c{};
        c.B = B; c.nw = nw; c.gx = grid; c.gy = 1; c.lds = lds; c.st = st; c.ra = ra;
        const hipError_t err = bridge_relu(dt, c, b);
        return err == hipSuccess ? DIVISION_OK : DIVISION_EHIP;
    }
    // other shapes: the operator, then the codec on its output
    const int r1 = division_relu_forward(x, n, dt == DIVISION_F32_C16 ? DIVISION_F32 : dt, y, mask, mask_capacity, hip_stream);
    if (r1 != DIVISION_OK) return r1;
    const void* yin = y;
    return compress_impl(1, &yin, &packed, &seed, N, C, 1, H, W, dt, B, b, packed_capacity, hip_stream);
}

int division_relu_compress_fused(int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt, int B, int b) {
    Layout L;
    if (make_layout(N, C, 1, H, W, B, b, (int)dt, &L) != DIVISION_OK) return 0;
    RegsArgs ra{};
    uint32_t grid = 0;
    size_t lds = 0;
    int nw = 1;
    return L.HW % 32 == 0 && (B == 4 || B == 8) &&
           plan_regs(L, 1, H, W, B, dt == DIVISION_BF16 ? 2 : 4, reinterpret_cast<const void*>((uintptr_t)16), &ra, &grid, &lds, &nw) && nw <= 4;
}

// Both directions of the descriptor-array calls: validates every map, then serves the maps that
// share a shape and parameters together, in order of first appearance.
static int run_maps(int count, const division_map* maps, void* hip_stream, bool compress) {
    if (count < 0 || (count > 0 && !maps)) return DIVISION_EINVAL;
    for (int i = 0; i < count; ++i) {
        const division_map& m = maps[i];
        Layout L;
        const int rc = make_layout(m.N, m.C, m.D, m.H, m.W, m.B, m.b, (int)m.dt, &L);
        if (rc != DIVISION_OK) return rc;
        if (!m.packed || (compress ? !m.x : !m.xhat)) return DIVISION_EINVAL;
        if (m.packed_bytes < L.total) return DIVISION_ESIZE;
        const size_t es = m.dt == DIVISION_BF16 ? 2 : 4;
        const void* data = compress ? m.x : m.xhat;
        if (((uintptr_t)data % es) != 0 || ((uintptr_t)m.packed % 16) != 0) return DIVISION_EALIGN;
    }
    auto same = [](const division_map& p, const division_map& q) {
        return p.N == q.N && p.C == q.C && p.D == q.D && p.H == q.H && p.W == q.W && p.dt == q.dt && p.B == q.B && p.b == q.b;
    };
    std::vector<char> done((size_t)count, 0);
    std::vector<const void*> in;
    std::vector<void*> out;
    std::vector<uint64_t> seeds;
    for (int i = 0; i < count; ++i) {
        if (done[(size_t)i]) continue;
        in.clear(); out.clear(); seeds.clear();
        size_t cap = ~(size_t)0;
        for (int j = i; j < count; ++j) {
            if (done[(size_t)j] || !same(maps[i], maps[j])) continue;
            done[(size_t)j] = 1;
            in.push_back(compress ? maps[j].x : maps[j].packed);
            out.push_back(compress ? maps[j].packed : maps[j].xhat);
            seeds.push_back(maps[j].seed);
            if (maps[j].packed_bytes < cap) cap = maps[j].packed_bytes;
        }
        const division_map& m = maps[i];
        const int rc = compress
            ? compress_impl((int)in.size(), in.data(), out.data(), seeds.data(), m.N, m.C, m.D, m.H, m.W, m.dt, m.B, m.b, cap, hip_stream)
            : decompress_impl((int)in.size(), in.data(), out.data(), cap, m.N, m.C, m.D, m.H, m.W, m.dt, m.B, m.b, hip_stream);
        if (rc != DIVISION_OK) return rc;
    }
    return DIVISION_OK;
}

int division_compress_maps(int count, const division_map* maps, void* hip_stream) {
    return run_maps(count, maps, hip_stream, true);
}

int division_decompress_maps(int count, const division_map* maps, void* hip_stream) {
    return run_maps(count, maps, hip_stream, false);
}

int division_kernel_name(int direction, const void* data, int64_t N, int64_t C, int64_t H, int64_t W,
                         division_dtype dt, int B, int b, char* out, size_t cap) {
    return kernel_name_impl(direction, data, N, C, 1, H, W, dt, B, b, out, cap);
}

int division_kernel_name_3d(int direction, const void* data, int64_t N, int64_t C, int64_t D, int64_t H, int64_t W,
                            division_dtype dt, int B, int b, char* out, size_t cap) {
    return kernel_name_impl(direction, data, N, C, D, H, W, dt, B, b, out, cap);
}

}  // extern "C"
#endif  // DIVISION_HOST
