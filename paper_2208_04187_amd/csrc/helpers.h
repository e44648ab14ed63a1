// Part of division.hip (included inside its unnamed namespace, in this order): element types, fast division, scale and meta helpers, pointer tables, wavefront synchronisation, DPP reductions.

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
// Quotient by a runtime divisor d through one multiply-high: exact while numerator * d < 2^32 (the host checks it
// with fastdiv_ok).  The divisor 1 has no 32-bit multiplier: its m is 0 and `one` is all ones, so that the quotient
// needs no test (a test on m, uniform as it is, became a scalar branch per division: 13 in decompress_stream, 228
// in compress_units, each ending a basic block in the middle of the loads; without them decompress_stream runs
// 1.5-2.5 % faster).  fdiv_tested is the form with the test, kept for the one loop that measured faster with it.
struct FastDiv { uint32_t one, m; };
__device__ __forceinline__ uint32_t fdiv(uint32_t n, FastDiv f) { return __umulhi(n, f.m) | (n & f.one); }
__device__ __forceinline__ uint32_t fdiv_tested(uint32_t n, FastDiv f) { return f.m ? __umulhi(n, f.m) : n; }
static FastDiv make_fastdiv(uint32_t d) {
    FastDiv f; f.one = d <= 1 ? 0xffffffffu : 0u; f.m = d <= 1 ? 0u : (uint32_t)((1ull << 32) / d) + 1u; return f;
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
// fl(fl(max - delta) / L) rounded UP to bfloat16, inv = fl(1 / Delta); Delta = inv = 0 when the
// range is below 2^-90, not finite, or Delta would not be a finite bfloat16.
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
        // L = 1 and a range beyond the largest bfloat16: no finite step to cache, the plane is degenerate
        const bool finite = Delta <= 3.3895313892515355e38f;
        inv = finite ? 1.0f / Delta : 0.0f;
        Delta = finite ? Delta : 0.0f;
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

// Which unit of work (a plane, a chunk of planes) workgroup b of n takes.  Workgroups are dealt to
// the eight XCDs round-robin by their index, and each XCD has its own L2.  A compress workgroup
// writes a few hundred bytes into each of three regions (codes, meta, H^L), far less than a cache
// line per region for small planes, so with the plain order b -> b the lines of those regions are
// written piecewise from eight L2s.  Here the workgroups of one XCD (equal b % 8) take runs of 64
// consecutive units instead, so that every line of the packed buffer is completed inside one L2
// and leaves it whole (a read stream with the writes of compress_regs: 5.63 -> 5.81 TB/s).  The
// last n % 512 units keep the plain order.
__device__ __forceinline__ uint32_t xcd_run_index(uint32_t b, uint32_t n) {
    constexpr uint32_t X = 8, R = 64;
    const uint32_t full = n - n % (X * R);
    if (b >= full) return b;
    const uint32_t x = b % X, j = b / X;
    return ((j / R) * X + x) * R + (j % R);
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

// A bounds-checked 16-byte buffer store whose offset sits in the vector operand only.  A VALU write to
// the data registers of a store of more than 8 bytes needs wait states behind the store; the
// compiler counts them for buffer stores WITHOUT a scalar offset register only.  With the offset
// split as (lane part in the VGPR, round part in an SGPR) a kernel here stored, now and then, the NEXT
// vector's first dword for the last four lanes of a row of sixteen: the instruction right behind the
// store had overwritten the first data register.  Keeping the scalar offset at the constant 0 makes
// the compiler see the hazard and keep its distance.
__device__ __forceinline__ void store_b128_checked(u32x4 v, __amdgpu_buffer_rsrc_t rsrc, uint32_t byte_offset, int aux) {
    if (aux == 2) __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, byte_offset, 0, 2);
    else __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, byte_offset, 0, 0);
}

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

// value of another lane of the same 16-lane row; all lanes must be active.  bound_ctrl is set: the
// permutations used here never read outside the row, and with it the compiler need not initialise
// the destination (two fewer instructions per 64-bit exchange)
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    const uint64_t u = __double_as_longlong(v);
    const uint32_t lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)u, CTRL, 0xf, 0xf, true);
    const uint32_t hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(u >> 32), CTRL, 0xf, 0xf, true);
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
