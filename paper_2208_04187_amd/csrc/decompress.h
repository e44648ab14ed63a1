// Part of division.hip (included inside its unnamed namespace, in this order): the decompress kernels.

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
template <int ND, bool TESTED = false>
__device__ __forceinline__ uint32_t lfc_row(const DecArgs& a, uint32_t r) {
    auto div = [](uint32_t n, FastDiv f) { return TESTED ? fdiv_tested(n, f) : fdiv(n, f); };
    if constexpr (ND == 3) {
        const uint32_t z = div(r, a.d_Hs);
        return (div(z, a.d_B) * a.LHs + div(r - z * a.Hs, a.d_B)) * a.LW;
    } else {
        return div(r, a.d_B) * a.LW;
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
// whole compress + decompress step).
template <typename T>
__device__ __forceinline__ void store4(T* dst, size_t i, float a, float b, float c, float d) {
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
    const uint32_t nq = (((size_t)p0 * a.WPP) & 3u) == 0 ? nw >> 2 : 0u;       // 16-byte vectors of code words
    const uint32_t nl = Gc * a.nb;
    constexpr bool widen = sizeof(T) == 4 && kC16<T>;      // bfloat16 H^L of an fp32 map: widened here, the streaming loops read floats
    typedef typename std::conditional<widen, uint16_t, T>::type LT;
    const LT* lsrc = static_cast<const LT*>(pt.lfc) + (size_t)p0 * a.nb;
    auto put_lfc = [&](uint32_t i, LT v) {
        if constexpr (widen) reinterpret_cast<float*>(s_lfc)[i] = bf16_bits_to_float(v);
        else s_lfc[i] = v;
    };
    // the first piece of each of the four slices is fetched before any of them is waited for (one
    // latency instead of four: a loop that loads and parks, then the next, waits once per loop)
    const uint32_t iw = (nq << 2) + tid;
    const bool hq = tid < nq, hw = iw < nw, hm = tid < Gc, hl = tid < nl;
    u32x4 q0{0u, 0u, 0u, 0u};
    uint32_t w0 = 0;
    float2 m0 = make_float2(0.0f, 0.0f);
    LT l0{};
    if (hq) q0 = reinterpret_cast<const u32x4*>(src)[tid];
    if (hw) w0 = src[iw];
    if (hm) m0 = meta_load(pt.meta, p0 + tid, kC16<T>);
    if (hl) l0 = lsrc[tid];
    if (hq) reinterpret_cast<u32x4*>(s_codes)[tid] = q0;
    if (hw) s_codes[iw] = w0;
    if (hm) s_meta[tid] = m0;
    if (hl) put_lfc(tid, l0);
    // what is left of larger slices
    for (uint32_t i = tid + kThreads; i < nq; i += kThreads)
        reinterpret_cast<u32x4*>(s_codes)[i] = reinterpret_cast<const u32x4*>(src)[i];
    for (uint32_t i = iw + kThreads; i < nw; i += kThreads) s_codes[i] = src[i];
    for (uint32_t i = tid + kThreads; i < Gc; i += kThreads) s_meta[i] = meta_load(pt.meta, p0 + i, kC16<T>);
    for (uint32_t i = tid + kThreads; i < nl; i += kThreads) put_lfc(i, lsrc[i]);
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
                // (the divisions of this loop keep their test for the divisor 1: measured 1 % faster on the
                // 256 x 256 x 56 x 56 bfloat16 map than without)
                const uint32_t g = fdiv_tested(vi, a.d_q4);
                const uint32_t fi = vi - g * a.q4;                     // even
                const float2 dd = s_meta[g];
                uint32_t lo, hi;                                       // codes of elements 0-3 and 4-7
                if constexpr (BITS == 1) {
                    lo = reinterpret_cast<const uint8_t*>(s_codes)[g * a.WPP * 4 + (fi >> 1)];
                    hi = lo >> 4;
                } else if constexpr (BITS == 2) {
                    lo = reinterpret_cast<const uint16_t*>(s_codes)[(g * a.WPP * 4 + fi) >> 1];
                    hi = lo >> 8;
                } else if constexpr (BITS == 4) {
                    lo = s_codes[(g * a.WPP * 2 + fi) >> 1];
                    hi = lo >> 16;
                } else {
                    lo = s_codes[g * a.WPP + fi];
                    hi = s_codes[g * a.WPP + fi + 1];
                }
                const uint32_t r = fdiv_tested(fi, a.d_w4);
                const uint32_t c = (fi - r * a.w4) * 4;
                const T* lrow = s_lfc + g * a.nb + lfc_row<ND, true>(a, r);
                const float l0 = Elem<T>::load(lrow, fdiv_tested(c, a.d_B)), l1 = Elem<T>::load(lrow, fdiv_tested(c + 4, a.d_B));
                uint32_t w[4];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    w[e] = float_to_bf16_bits(dequant((lo >> (2 * e * BITS)) & Lq, dd.y, dd.x, l0)) |
                           (float_to_bf16_bits(dequant((lo >> ((2 * e + 1) * BITS)) & Lq, dd.y, dd.x, l0)) << 16);
                    w[2 + e] = float_to_bf16_bits(dequant((hi >> (2 * e * BITS)) & Lq, dd.y, dd.x, l1)) |
                               (float_to_bf16_bits(dequant((hi >> ((2 * e + 1) * BITS)) & Lq, dd.y, dd.x, l1)) << 16);
                }
                u32x4 o; o.x = w[0]; o.y = w[1]; o.z = w[2]; o.w = w[3];
                __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(out + (size_t)vi * 4));
            }
            return;
        }
    }
    for (uint32_t vi = tid; vi < nvec; vi += kThreads) {
        const uint32_t g = fdiv(vi, a.d_q4);
        const uint32_t fi = vi - g * a.q4;        // vector index inside the plane
        const float2 dd = s_meta[g];
        uint32_t c4;                               // the four codes, BITS apart from bit 0
        if constexpr (BITS == 1) c4 = reinterpret_cast<const uint8_t*>(s_codes)[g * a.WPP * 4 + (fi >> 1)] >> ((fi & 1u) * 4u);
        else if constexpr (BITS == 2) c4 = reinterpret_cast<const uint8_t*>(s_codes)[g * a.WPP * 4 + fi];
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

// The row-vector case again (W % 4 == 0, B % 4 == 0, 4-byte elements) without staging and without a
// barrier: a workgroup is ONE wavefront that rebuilds kStreamK * 64 consecutive 16-byte vectors of the
// map (4 KB for kStreamK = 4), wherever the plane boundaries fall.  Each lane finds the plane, row and
// block of its vectors, loads their code byte / half-word / word, their plane's (delta, Delta) and their
// block's H^L straight from the packed buffer (all of its lines are shared by many lanes and rounds, so
// nearly all of these loads are cache hits), and stores.  All loads of the chunk are issued before the
// first store.  Short-lived one-wavefront workgroups that write a few KB each are what the memory
// system takes fastest (a write-only stream: 6.4 - 6.7 TB/s in 4 KB pieces, 5.5 in 32 KB ones), and with
// no barrier the latency of the packed reads is hidden by the other wavefronts of the CU.
constexpr int kStreamK = DIVISION_STREAM_K;
template <typename T, int BITS, int ND>
__device__ __forceinline__ void decompress_stream_body(const DecArgs& a) {
    static_assert(sizeof(T) == 4, "4-byte elements");
    constexpr int K = kStreamK;
    constexpr uint32_t Lq = (1u << BITS) - 1u;
    constexpr uint32_t CBY = BITS / 2;                                  // code bytes per vector
    const DecPtrs pt = dec_ptrs(a.tab, a.rg);
    const uint32_t lane = threadIdx.x;
    // first vector of the chunk, counted over the whole map: its plane g0 and its place r0 inside the
    // plane (uniform; the quotient by a binary64 reciprocal, then put right)
    const uint64_t v0 = (uint64_t)blockIdx.x * (64u * K);
    const uint64_t nvec = (uint64_t)a.P * a.q4;
    uint32_t g0 = (uint32_t)((double)v0 * (1.0 / (double)a.q4));
    int64_t r0 = (int64_t)(v0 - (uint64_t)g0 * a.q4);
    if (r0 < 0) { --g0; r0 += a.q4; }
    if (r0 >= (int64_t)a.q4) { ++g0; r0 -= a.q4; }
    g0 = __builtin_amdgcn_readfirstlane(g0);
    const uint32_t t0 = __builtin_amdgcn_readfirstlane((uint32_t)r0);

    uint32_t code[K];
    float2 dd[K];
    float lfc[K];
    const uint8_t* cbase = reinterpret_cast<const uint8_t*>(pt.codes);
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t t = t0 + 64u * k + lane;                           // < q4 + 64 K
        const uint32_t dg = fdiv(t, a.d_q4);
        const uint32_t fi = t - dg * a.q4;                                // vector inside its plane
        const uint32_t g = min(g0 + dg, a.P - 1u);                         // vectors past the map re-read its last plane
        const uint32_t r = fdiv(fi, a.d_w4);
        const uint32_t c = (fi - r * a.w4) * 4u;
        const uint32_t blk = lfc_row<ND>(a, r) + fdiv(c, a.d_B);
        const uint8_t* cp = cbase + (size_t)g * a.WPP * 4u + (BITS == 1 ? (size_t)(fi >> 1) : (size_t)fi * CBY);
        if constexpr (BITS == 1) code[k] = (uint32_t)*cp >> ((fi & 1u) * 4u);     // four 1-bit codes: half a byte
        else if constexpr (BITS == 2) code[k] = *cp;
        else if constexpr (BITS == 4) code[k] = *reinterpret_cast<const uint16_t*>(cp);
        else code[k] = *reinterpret_cast<const uint32_t*>(cp);
        dd[k] = meta_load(pt.meta, g, kC16<T>);
        lfc[k] = lfc_load<T>(pt.lfc, (size_t)g * a.nb + blk, kC16<T>);
    }
    T* out = static_cast<T*>(pt.xhat) + v0 * 4u;
    const uint64_t left = nvec - v0;                                      // vectors from the chunk's start to the map's end
    const __amdgpu_buffer_rsrc_t ors = __builtin_amdgcn_make_buffer_rsrc(
        out, 0, (int)(left < 64u * K ? (uint32_t)left * 16u : 64u * K * 16u), 0x00020000);
#pragma unroll
    for (int k = 0; k < K; ++k) {
        u32x4 o;
        o.x = __float_as_uint(dequant(code[k] & Lq, dd[k].y, dd[k].x, lfc[k]));
        o.y = __float_as_uint(dequant((code[k] >> BITS) & Lq, dd[k].y, dd[k].x, lfc[k]));
        o.z = __float_as_uint(dequant((code[k] >> (2 * BITS)) & Lq, dd[k].y, dd[k].x, lfc[k]));
        o.w = __float_as_uint(dequant((code[k] >> (3 * BITS)) & Lq, dd[k].y, dd[k].x, lfc[k]));
        store_b128_checked(o, ors, lane * 16u + (uint32_t)(k * 1024), DIVISION_STREAM_STORE_AUX);   // past the map: dropped
    }
}
template <typename T, int BITS>
__global__ void __launch_bounds__(64) decompress_stream(DecArgs a) { if constexpr (sizeof(T) == 4) decompress_stream_body<T, BITS, 2>(a); }
template <typename T, int BITS>
__global__ void __launch_bounds__(64) decompress_stream_3d(DecArgs a) { if constexpr (sizeof(T) == 4) decompress_stream_body<T, BITS, 3>(a); }

// The stream kernel for maps whose rows, blocks or planes are not whole vectors (odd widths, any B; 4-byte
// elements): a workgroup is again ONE wavefront that rebuilds kStreamK * 64 consecutive, aligned 16-byte
// vectors of the map wherever rows and planes end, without LDS or barrier.  A vector's four elements may
// lie in two rows and in two planes (planes have at least 4 elements): each element finds its own plane,
// row, column and block; the vector's codes are the 4 * BITS bits from its first element's place in its
// plane's code words (two words, funnel-shifted), continued with the first bits of the next plane where
// the plane ends inside the vector; (delta, Delta) of both planes and the H^L of each element's block come
// straight from the packed buffer (cache hits: all lanes of a chunk share a few lines).  Vectors past the
// map re-read its last plane and their stores are dropped by the buffer bound, dword by dword, so a map
// whose element count is not a multiple of 4 ends with a partly stored vector.
// quotient by a divisor of at least 2 (the host checks it, and that numerator * divisor < 2^32): fdiv without
// its term for the divisor 1
__device__ __forceinline__ uint32_t udiv2(uint32_t n, FastDiv f) { return __umulhi(n, f.m); }
// offset of row r's first block among a plane's H^L values (r counts the rows of all depth slices)
template <int ND>
__device__ __forceinline__ uint32_t lfc_row2(const DecArgs& a, uint32_t r) {
    if constexpr (ND == 3) {
        const uint32_t z = udiv2(r, a.d_Hs);
        return (udiv2(z, a.d_B) * a.LHs + udiv2(r - z * a.Hs, a.d_B)) * a.LW;
    } else {
        return udiv2(r, a.d_B) * a.LW;
    }
}
template <typename T, int BITS, int ND>
__device__ __forceinline__ void decompress_stream_any_body(const DecArgs& a) {
    static_assert(sizeof(T) == 4, "4-byte elements");
    constexpr int K = kStreamK;
    constexpr uint32_t Lq = (1u << BITS) - 1u;
    constexpr uint32_t LB = kC16<T> ? 2u : 4u, MB = kC16<T> ? 4u : 8u;     // bytes of one H^L value, of one (delta, Delta)
    const DecPtrs pt = dec_ptrs(a.tab, a.rg);
    const uint32_t lane = threadIdx.x;
    // first element of the chunk, counted over the whole map: its plane g0 and its place t0 inside the plane
    const uint64_t e0 = (uint64_t)blockIdx.x * (256u * K);
    const uint64_t ntot = (uint64_t)a.P * a.HW;
    uint32_t g0 = (uint32_t)((double)e0 * (1.0 / (double)a.HW));
    int64_t r0 = (int64_t)(e0 - (uint64_t)g0 * a.HW);
    if (r0 < 0) { --g0; r0 += a.HW; }
    if (r0 >= (int64_t)a.HW) { ++g0; r0 -= a.HW; }
    g0 = __builtin_amdgcn_readfirstlane(g0);
    const uint32_t t0 = __builtin_amdgcn_readfirstlane((uint32_t)r0);
    // the three regions of the packed buffer through bounds-checked buffers with 32-bit offsets (the host
    // checks that each is below 4 GiB); the word behind the last plane's code words reads as zero
    const __amdgpu_buffer_rsrc_t crs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(pt.codes), 0, (int)(a.P * a.WPP * 4u), 0x00020000);
    const __amdgpu_buffer_rsrc_t mrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(pt.meta), 0, (int)(a.P * MB), 0x00020000);
    const __amdgpu_buffer_rsrc_t lrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(pt.lfc), 0, (int)(a.P * a.nb * LB), 0x00020000);

    uint32_t lo[K], hi[K], nx[K], sh[K], n0[K], lw[K][4];
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
    u32x2 ma[K], mb[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        // (products of two numbers below 2^24 use the full-rate 24-bit multiply; the host checks the sizes)
        const uint32_t t = t0 + 4u * (64u * k + lane);                    // < HW + 256 K
        const uint32_t dg = udiv2(t, a.d_HW);
        const uint32_t i = t - __umul24(dg, a.HW);                        // the vector's first element inside its plane
        const uint32_t g = min(g0 + dg, a.P - 1u);                         // vectors past the map re-read its last plane
        const uint32_t g1 = min(g + 1u, a.P - 1u);
        n0[k] = min(4u, a.HW - i);                                        // elements of the vector that lie in plane g
        const uint32_t bit = i * BITS;
        sh[k] = bit & 31u;
        // One load of three words: the two the vector's codes may lie in and the one behind them.  Where the plane
        // ends inside the vector its codes end in the plane's last word, and the next plane's first word is the
        // second or the third of the three.  (Behind the map's last plane the words read as zero and are not used.)
        const uint32_t wi = bit >> 5;
        const u32x3 cw3 = __builtin_amdgcn_raw_buffer_load_b96(crs, (__umul24(g, a.WPP) + wi) * 4u, 0, 0);
        lo[k] = cw3.x;
        hi[k] = cw3.y;
        nx[k] = wi + 1u == a.WPP ? cw3.y : cw3.z;
        // (delta, Delta) of the plane and of the next one lie side by side (the last plane has no next one: zeros)
        if constexpr (kC16<T>) {
            const u32x2 m2 = __builtin_amdgcn_raw_buffer_load_b64(mrs, g * 4u, 0, 0);
            ma[k].x = m2.x; mb[k].x = m2.y;
        } else {
            const u32x4 m4 = __builtin_amdgcn_raw_buffer_load_b128(mrs, g * 8u, 0, 0);
            ma[k] = u32x2{m4.x, m4.y}; mb[k] = u32x2{m4.z, m4.w};
        }
        if constexpr (ND == 0) {
            // one block per plane: H^L of the plane and of the next one lie side by side, one load
            if constexpr (kC16<T>) {
                lw[k][0] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(lrs, g * 2u, 0, 0) << 16;     // (2-byte values: a 4-byte load
                lw[k][1] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(lrs, g * 2u + 2u, 0, 0) << 16; // of both would not be aligned)
            } else {
                const u32x2 l2 = __builtin_amdgcn_raw_buffer_load_b64(lrs, g * 4u, 0, 0);
                lw[k][0] = l2.x; lw[k][1] = l2.y;
            }
            continue;
        }
        // Row r and column c of the first element.  W >= 4: the vector leaves its row at most once; B >= 4: what
        // lies behind the row's end (columns 0-2 of the next row, or of row 0 of the next plane) is in block
        // column 0, and inside the row the block column grows by at most one.  Byte offsets of the H^L values:
        // oa (the first element's block), ob (block column 0 of the next row), oc (block 0 of the next plane).
        const uint32_t r = udiv2(i, a.d_W);
        const uint32_t c = i - __umul24(r, a.W);
        const uint32_t bc = udiv2(c, a.d_B);
        const uint32_t crem = c - __umul24(bc, a.B);                      // column inside its block
        uint32_t rt0, rt1;
        if constexpr (ND == 2) {
            const uint32_t rb = udiv2(r, a.d_B);
            const uint32_t rrem = r - __umul24(rb, a.B);
            rt0 = __umul24(rb, a.LW);
            rt1 = rt0 + (rrem + 1u >= a.B ? a.LW : 0u);
        } else {
            rt0 = lfc_row2<ND>(a, r);
            rt1 = lfc_row2<ND>(a, r + 1u);
        }
        const uint32_t pg = __umul24(g, a.nb);
        const uint32_t oa = (pg + rt0 + bc) * LB, ob = (pg + rt1) * LB, oc = __umul24(g1, a.nb) * LB;
        // (three loads instead of four, the middle elements picking among them, measured 5-15 % slower: the
        // selects cost more than the load)
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) {
            const bool first = j < n0[k];
            const bool wrap = c + j >= a.W;
            const uint32_t in_row = oa + (crem + j >= a.B ? LB : 0u);
            const uint32_t off = first ? (wrap ? ob : in_row) : oc;
            if constexpr (kC16<T>) lw[k][j] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(lrs, off, 0, 0) << 16;
            else lw[k][j] = __builtin_amdgcn_raw_buffer_load_b32(lrs, off, 0, 0);
        }
    }
    T* out = static_cast<T*>(pt.xhat) + e0;
    const uint64_t left = ntot - e0;                                      // elements from the chunk's start to the map's end
    const __amdgpu_buffer_rsrc_t ors = __builtin_amdgcn_make_buffer_rsrc(
        out, 0, (int)(left < 256u * K ? (uint32_t)left * 4u : 256u * K * 4u), 0x00020000);
#pragma unroll
    for (int k = 0; k < K; ++k) {
        uint32_t c = __builtin_amdgcn_alignbit(hi[k], lo[k], sh[k]);
        // the plane's last n0 codes, then the next plane's first ones: 64-bit shifts, so that n0 = 4 (a shift by the
        // whole word) needs no test (a test would let the compiler move the load of nx behind it, after a wait)
        const uint32_t nb0 = n0[k] * BITS;
        c = (c & (uint32_t)((1ull << nb0) - 1ull)) | (uint32_t)((uint64_t)nx[k] << nb0);
        float2 da, db;
        if constexpr (kC16<T>) {
            da = make_float2(__uint_as_float(ma[k].x << 16), __uint_as_float(ma[k].x & 0xffff0000u));
            db = make_float2(__uint_as_float(mb[k].x << 16), __uint_as_float(mb[k].x & 0xffff0000u));
        } else {
            da = make_float2(__uint_as_float(ma[k].x), __uint_as_float(ma[k].y));
            db = make_float2(__uint_as_float(mb[k].x), __uint_as_float(mb[k].y));
        }
        uint32_t ov[4];
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) {
            const bool first = j < n0[k];
            const uint32_t lfcw = ND == 0 ? (first ? lw[k][0] : lw[k][1]) : lw[k][j];
            ov[j] = __float_as_uint(dequant((c >> (j * BITS)) & Lq, first ? da.y : db.y, first ? da.x : db.x, __uint_as_float(lfcw)));
        }
        u32x4 o; o.x = ov[0]; o.y = ov[1]; o.z = ov[2]; o.w = ov[3];
        store_b128_checked(o, ors, lane * 16u + (uint32_t)(k * 1024), DIVISION_STREAM_STORE_AUX);   // past the map: dropped
    }
}
template <typename T, int BITS>
__global__ void __launch_bounds__(64) decompress_stream_any(DecArgs a) { if constexpr (sizeof(T) == 4) decompress_stream_any_body<T, BITS, 2>(a); }
template <typename T, int BITS>
__global__ void __launch_bounds__(64) decompress_stream_any_3d(DecArgs a) { if constexpr (sizeof(T) == 4) decompress_stream_any_body<T, BITS, 3>(a); }
// planes that are one block (any number of map dimensions): no rows or columns, H^L is the plane's
template <typename T, int BITS>
__global__ void __launch_bounds__(64) decompress_stream_one(DecArgs a) { if constexpr (sizeof(T) == 4) decompress_stream_any_body<T, BITS, 0>(a); }

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
        if constexpr (BITS == 1) c4 = reinterpret_cast<const uint8_t*>(s_codes)[g * a.WPP * 4 + (fi >> 1)] >> ((fi & 1u) * 4u);
        else if constexpr (BITS == 2) c4 = reinterpret_cast<const uint8_t*>(s_codes)[g * a.WPP * 4 + fi];
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

// Planes (2-D or 3-D maps) whose rows or blocks are not whole vectors (odd widths), the counterpart of compress_units:
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

    // Planes whose element count is not a multiple of 4 start 1, 2 or 3 elements past a unit boundary of
    // the map.  Their units then start that many elements early: every store is a whole, aligned unit of
    // the map (16 bytes for 4-byte elements: a write-only probe runs at 5.9 TB/s there and at 4.6 TB/s
    // with 16-byte stores at 4-byte-aligned addresses; 2-byte elements need it, a store in the middle of
    // a dword is not possible), the elements before the plane and those past it are left alone.  The
    // same for all planes of the workgroup: the grid is a multiple of 4, or every workgroup has one plane.
    const uint32_t shift = (blockIdx.x * a.HW) & 3u;

    // LDS byte offset of the LFC of each element's block (elements outside the plane: block 0, never stored)
    uint32_t lo[K][2];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        uint32_t off[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t e = 4u * (tid + NT * k) + j - shift;       // wraps for the element before the plane
            const uint32_t ra = fdiv(e, a.d_W);                       // row, counted over all depth slices
            const uint32_t c = e - ra * a.W;
            const uint32_t z = fdiv(ra, a.d_Hs);
            const uint32_t r = ra - z * a.Hs;
            off[j] = e < a.HW ? 4u * ((fdiv(z, a.d_B) * a.LHs + fdiv(r, a.d_B)) * a.LW + fdiv(c, a.d_B)) : 0u;
        }
        lo[k][0] = off[0] | (off[1] << 16);
        lo[k][1] = off[2] | (off[3] << 16);
    }
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    u32x2 wide[K];      // .x: the unit's codes as loaded; shifted units: the two code words the unit's codes lie in
    float lf[KL];
    float2 dd;
    auto issue_loads = [&](uint32_t p) {
        const __amdgpu_buffer_rsrc_t crs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint32_t*>(pt.codes) + (size_t)p * a.WPP, 0, (int)(a.WPP * 4u), 0x00020000);
        if (shift) {
            // codes of elements 4f-shift .. 4f-shift+3: 4 * BITS bits from bit (4f-shift) * BITS of the plane's code words
            const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<uint32_t*>(pt.codes) + (size_t)p * a.WPP, 0, (int)(a.WPP * 4u), 0x00020000);
#pragma unroll
            for (int k = 0; k < K; ++k) {
                if (!round_live(k)) continue;
                const uint32_t f = tid + NT * k;
                const uint32_t bit = f ? (4u * f - shift) * BITS : 0u;
                wide[k] = __builtin_amdgcn_raw_buffer_load_b64(wrs, (bit >> 5) * 4u, 0, 0);
            }
        }
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (!round_live(k) || shift) continue;
            if constexpr (BITS == 1) wide[k].x = __builtin_amdgcn_raw_buffer_load_b8(crs, (tid + (uint32_t)(NT * k)) >> 1, 0, 0);   // two units per byte
            else if constexpr (CB == 1) wide[k].x = __builtin_amdgcn_raw_buffer_load_b8(crs, tid, k * NT, 0);
            else if constexpr (CB == 2) wide[k].x = __builtin_amdgcn_raw_buffer_load_b16(crs, tid * 2u, k * NT * 2, 0);
            else wide[k].x = __builtin_amdgcn_raw_buffer_load_b32(crs, tid * 4u, k * NT * 4, 0);
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
            if (shift) {
                const uint32_t f = tid + NT * k;
                const uint32_t bit = f ? (4u * f - shift) * BITS : 0u;
                const uint32_t c = __builtin_amdgcn_alignbit(wide[k].y, wide[k].x, bit & 31u);
                c4[k] = f ? c : c << (shift * BITS);       // unit 0: the slots before the plane, then its first elements
                continue;
            }
            c4[k] = BITS == 1 ? wide[k].x >> ((tid & 1u) * 4u) : wide[k].x;
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
