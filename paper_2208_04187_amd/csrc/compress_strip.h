// Part of division.hip (included inside its unnamed namespace, in this order): compress_strip.

// ------------------------------------------------------------------ compress, a strip of 28 or 32 elements per lane

struct StripArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, H, HW, WPP, nb;
    uint32_t nrounds;    // ceil(P / planes per round)
    void* y;             // relu_compress_strip: the activation's output map and its 1-bit mask (one map per launch);
    uint32_t* mask;      // a round's elements are a multiple of 32 then: its mask bits are whole words
};

// Geometry of the strip kernel for planes of width W under block size B (both compile-time).
template <int W, int B>
struct StripGeom {
    static_assert(W == 28 || W == 14 || W == 32 || W == 16, "strip widths");
    static constexpr int E = (W == 28 || W == 14) ? 28 : 32;   // elements per lane: seven or eight 16-byte units
    static constexpr int RPL = E / W;                           // rows per lane (1 or 2)
    static constexpr int S = 32 / (RPL * RPL);                  // lane slots per plane: 32 rows, or 8 x 2 rows
    static constexpr int G = 64 / S;                            // planes per round
    static constexpr int NSEG = (W + B - 1) / B;                // blocks per block row = columns of the pooled map
    static constexpr int LBR = B / RPL;                         // lanes per block row
    static constexpr bool kDpp = LBR == 2 || LBR == 4 || LBR == 8;   // the lanes of a block row are an aligned DPP group
    static_assert(B % RPL == 0, "a lane's rows lie in one block row");
};

// Small planes of a fixed width (28 x 28 and 14 x 14 of a ResNet on ImageNet, 32 x 32 and 16 x 16 on
// CIFAR) under a fixed block size (8, and the 12, 16 and 18 of the block-size sweep of Sec. 5): a
// lane owns a strip of 28 or 32 consecutive elements of its plane, i.e. one row of a 28- or 32-wide
// map or two rows of a 14- or 16-wide one, seven or eight 16-byte units, and keeps it in registers
// from the pooling to the codes.  Which block each element of the strip belongs to is known at
// compile time.  The lanes of a plane sit side by side (32 slots for up to 32 rows, 8 slots for up
// to 16 rows; 2 resp. 8 planes per wavefront).  Block sums (binary64): when the lanes of a block
// row are an aligned group of 4 or 8 (B = 8) they are DPP reductions and every lane ends up with
// its own blocks' H^L; for the other block sizes a lane parks its strip's share of each block in
// LDS, a lane per block adds the shares of the block's rows in row order, and the lanes read the
// H^L values back.  The plane's extremes are DPP reductions either way: no per-element lookup.
//
// Memory side: the round (all its planes are contiguous) is read with coalesced 16-byte loads that
// are issued before anything else and land in LDS in the map's own order; each lane then takes its
// strip out of LDS (a stride of 28 or 32 words).  The codes of a unit go back to LDS as one byte /
// half-word / word and leave as whole coalesced words.
// One round per workgroup of one wavefront.
//
// RELU: x is the input of a Relu operator (Appendix, Relu listing) whose output y is the map to
// cache.  The operator is applied to the round as it arrives, in the coalesced order of the loads:
// y leaves from the same registers (16-byte stores), the mask bits of a lane's unit are merged
// over eight adjacent lanes (DPP OR) and leave as whole words; the codec then runs on y.
template <typename T, int BITS, int W, int B, bool RELU>
__device__ __forceinline__ void compress_strip_body(const StripArgs& a) {
    using Geo = StripGeom<W, B>;
    constexpr int E = Geo::E, S = Geo::S, G = Geo::G, NSEG = Geo::NSEG, LBR = Geo::LBR, RPL = Geo::RPL;
    constexpr int UPL = E / 4;                  // units per lane
    constexpr int CB = BITS / 2;                // code bytes per 4-element unit
    constexpr float Lf = float((1 << BITS) - 1);
    extern __shared__ float4 smem4[];
    float* xs = reinterpret_cast<float*>(smem4);                     // [UPL * 64 units] the round, later its code words
    double* part = reinterpret_cast<double*>(xs + UPL * 64 * 4);      // [64 * NSEG] a strip's share of each block of its block row
    float* lfcs = reinterpret_cast<float*>(part + 64 * NSEG);        // [G * nb <= 64] H^L of the round
    (void)part; (void)lfcs; (void)RPL;

    const uint32_t lane = threadIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, lane);
    const uint32_t round = xcd_run_index(blockIdx.x, a.nrounds);
    const uint32_t p0 = round * G;
    const uint32_t Gc = min((uint32_t)G, a.P - p0);

    // ---- the round's loads first: coalesced, bounds-checked (units past the round read as zero)
    u32x4 q[UPL];
    {
        const T* src = static_cast<const T*>(pt.x) + (size_t)p0 * a.HW;
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(src), 0, (int)(Gc * a.HW * sizeof(T)), 0x00020000);
#pragma unroll
        for (int k = 0; k < UPL; ++k) {
            if constexpr (sizeof(T) == 4) {
                q[k] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane * 16u, k * 1024, kLoadAux);
            } else {
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                const u32x2 h = __builtin_amdgcn_raw_buffer_load_b64(rsrc, lane * 8u, k * 512, kLoadAux);
                q[k] = u32x4{h.x << 16, h.x & 0xffff0000u, h.y << 16, h.y & 0xffff0000u};
            }
        }
    }
    if constexpr (RELU) {
        T* ydst = static_cast<T*>(a.y) + (size_t)p0 * a.HW;
        const __amdgpu_buffer_rsrc_t yrs =
            __builtin_amdgcn_make_buffer_rsrc(ydst, 0, (int)(Gc * a.HW * sizeof(T)), 0x00020000);
        // G * HW is a multiple of 32, so the round's mask starts at a word; a last, shorter round
        // ends the mask, whose final word has zero pad bits (elements past the round were read as zero)
        const uint32_t mwords = (Gc * a.HW + 31u) / 32u;
        const __amdgpu_buffer_rsrc_t mrs =
            __builtin_amdgcn_make_buffer_rsrc(a.mask + (size_t)round * (G * a.HW / 32u), 0, (int)(mwords * 4u), 0x00020000);
#pragma unroll
        for (int k = 0; k < UPL; ++k) {
            uint32_t nib = 0;
            uint32_t v[4] = {q[k].x, q[k].y, q[k].z, q[k].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool pos = __uint_as_float(v[e]) > 0.0f;
                nib |= (pos ? 1u : 0u) << e;
                v[e] = pos ? v[e] : 0u;
            }
            q[k] = u32x4{v[0], v[1], v[2], v[3]};
            // stores past the round are dropped by the buffer bound
            if constexpr (sizeof(T) == 4) {
                store_b128_checked(q[k], yrs, lane * 16u + (uint32_t)(k * 1024), 0);
            } else {
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                u32x2 o;
                o.x = (v[0] >> 16) | (v[1] & 0xffff0000u);
                o.y = (v[2] >> 16) | (v[3] & 0xffff0000u);
                __builtin_amdgcn_raw_buffer_store_b64(o, yrs, lane * 8u, k * 512, 0);
            }
            uint32_t w = nib << (4u * (lane & 7u));
            w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, kDppXor1, 0xf, 0xf, false);
            w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, kDppXor2, 0xf, 0xf, false);
            w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, kDppHalfMirror, 0xf, 0xf, false);
            if ((lane & 7u) == 0) __builtin_amdgcn_raw_buffer_store_b32(w, mrs, (lane >> 3) * 4u, k * 32, 0);
        }
    }
    // the lane's place: plane g of the round, strip sl of the plane
    const uint32_t g = lane / S, sl = lane % S;
    const bool live = g < Gc;
    const bool valid = live && sl * E < a.HW;
    const uint32_t bi = sl / LBR;                                      // block row of the strip
    const uint32_t rows = min((uint32_t)B, a.H - min(a.H, bi * (uint32_t)B));   // rows of that block row that exist
    const uint32_t p = p0 + g;
    const uint32_t k1 = mix32(p ^ pt.seed_a);
    const uint32_t k2 = mix32(k1 + pt.seed_c);
    const uint32_t rscale = 1u << (16 - BITS);
    const uint32_t xv = G * a.HW / 4u;                                // units of a whole round
#pragma unroll
    for (int k = 0; k < UPL; ++k)
        if (lane + 64u * k < xv) reinterpret_cast<u32x4*>(xs)[lane + 64 * k] = q[k];
    wave_sync();

    // ---- the strip; lanes without one take strip 0 of the round and have their effects masked
    float x[E];
    {
        const float4* sp = reinterpret_cast<const float4*>(xs + (valid ? g * a.HW + sl * E : 0u));
#pragma unroll
        for (int u = 0; u < UPL; ++u) {
            const float4 v = sp[u];
            x[4 * u] = v.x; x[4 * u + 1] = v.y; x[4 * u + 2] = v.z; x[4 * u + 3] = v.w;
        }
    }

    // ---- Sec. 4.1 AveragePooling: the strip's share of each block of its block row, then the
    // block row's lanes together (binary64, fixed order)
    double Sm[NSEG];
#pragma unroll
    for (int s = 0; s < NSEG; ++s) Sm[s] = 0.0;
#pragma unroll
    for (int e = 0; e < E; ++e) Sm[(e % W) / B] += (double)x[e];
    float lfc[NSEG];
    if constexpr (Geo::kDpp) {
#pragma unroll
        for (int s = 0; s < NSEG; ++s) {
            const double Sb = group_sum<LBR>(valid ? Sm[s] : 0.0);
            const uint32_t cols = (uint32_t)(W - B * s < B ? W - B * s : B);     // a constant once the loop is unrolled
            lfc[s] = lfc_round<T>(mean_of(Sb, max(rows, 1u) * cols), kC16<T>);
        }
        if (valid && sl % LBR == 0) {
#pragma unroll
            for (int s = 0; s < NSEG; ++s) lfc_store<T>(pt.lfc, (size_t)p * a.nb + bi * NSEG + s, lfc[s], kC16<T>);
        }
    } else {
        // the shares of a plane's strips lie one after the other: [plane of the round][strip][block column]
#pragma unroll
        for (int s = 0; s < NSEG; ++s) part[lane * NSEG + s] = valid ? Sm[s] : 0.0;
        wave_sync();
        // a lane per block of the round adds the shares of the block's strips in row order
        const uint32_t nbr = Gc * a.nb;                                   // at most 64 (the host checks G * nb)
        if (lane < nbr) {
            const uint32_t bg = lane / a.nb, t = lane - bg * a.nb;       // plane of the round, block of the plane
            const uint32_t tbi = t / NSEG, s = t - tbi * NSEG;
            const uint32_t brows = min((uint32_t)B, a.H - tbi * (uint32_t)B);    // >= 1: the block exists
            const uint32_t nstrips = (brows + RPL - 1) / RPL;
            const double* ps = part + (bg * S + tbi * LBR) * NSEG + s;
            double Sb = 0.0;
            for (uint32_t i = 0; i < nstrips; ++i) Sb += ps[i * NSEG];
            const uint32_t cols = min((uint32_t)B, (uint32_t)W - s * (uint32_t)B);
            const float m = lfc_round<T>(mean_of(Sb, brows * cols), kC16<T>);
            lfcs[lane] = m;
            lfc_store<T>(pt.lfc, (size_t)(p0 + bg) * a.nb + t, m, kC16<T>);
        }
        wave_sync();
#pragma unroll
        for (int s = 0; s < NSEG; ++s) lfc[s] = lfcs[valid ? g * a.nb + bi * NSEG + s : 0u];
    }

    // ---- residual H^H = H - UpSampling(H^L) in place, the plane's extremes
    float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
    for (int e = 0; e < E; ++e) {
        x[e] = x[e] - lfc[(e % W) / B];
        mn = fminf(mn, x[e]);
        mx = fmaxf(mx, x[e]);
    }
    mn = valid ? mn : __builtin_inff();
    mx = valid ? mx : -__builtin_inff();
    group_minmax(S, mn, mx);

    // ---- scale of Eq. (quantization): every lane of the plane computes the same values
    float delta, Delta, inv;
    plane_scale_any(mn, mx, Lf, kC16<T>, delta, Delta, inv);
    const float invs = inv * (float)(1u << (32 - BITS));
    if (live && sl == 0) meta_store(pt.meta, p, delta, Delta, kC16<T>);

    // ---- Quant + packing: a unit's four codes are one byte (b = 2), half-word or word of the plane's
    // code bytes; they are collected in LDS (over the round, which every lane has taken out by now)
    wave_sync();
    uint32_t* cw = reinterpret_cast<uint32_t*>(xs);
    const uint32_t nwords = Gc * a.WPP;
    {
        // pad bytes of a plane's last word stay zero
        const u32x4 z{0u, 0u, 0u, 0u};
        for (uint32_t i = lane; i * 4u < nwords; i += 64) reinterpret_cast<u32x4*>(cw)[i] = z;
    }
    wave_sync();
    {
        uint8_t* cb = reinterpret_cast<uint8_t*>(cw) + g * a.WPP * 4u + sl * (uint32_t)(UPL * CB);
        const uint32_t xw0 = k1 + (sl * (uint32_t)(E / 2)) * kWeyl;
        uint32_t strip_bits = 0;                                       // 1-bit codes: the strip's E codes
        (void)cb; (void)strip_bits;
#pragma unroll
        for (int u = 0; u < UPL; ++u) {
            const uint32_t xw = xw0 + (uint32_t)(2 * u) * kWeyl;
            uint32_t c = push_pair<BITS>(0u, x[4 * u + 2], x[4 * u + 3], delta, invs, xw + kWeyl, k2, rscale);
            c = push_pair<BITS>(c, x[4 * u], x[4 * u + 1], delta, invs, xw, k2, rscale);
            if constexpr (BITS == 1) strip_bits |= c << (4 * u);
            else if (valid) {
                if constexpr (CB == 1) cb[u] = (uint8_t)c;
                else if constexpr (CB == 2) reinterpret_cast<uint16_t*>(cb)[u] = (uint16_t)c;
                else reinterpret_cast<uint32_t*>(cb)[u] = c;
            }
        }
        if constexpr (BITS == 1) {
            // a strip's E bits start at bit sl * E of the plane's code words, for E = 28 in the middle of a
            // byte: the lanes OR their bits into the (cleared) words, one or two words per strip
            if (valid) {
                uint32_t* pw = cw + g * a.WPP;
                const uint32_t bit = sl * (uint32_t)E, sh = bit & 31u;
                __hip_atomic_fetch_or(pw + (bit >> 5), strip_bits << sh, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                if (sh + (uint32_t)E > 32u)
                    __hip_atomic_fetch_or(pw + (bit >> 5) + 1u, strip_bits >> (32u - sh), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
    }
    wave_sync();
    {
        uint32_t* dst = pt.codes + (size_t)p0 * a.WPP;
        for (uint32_t w = lane; w < nwords; w += 64) dst[w] = cw[w];
    }
}

template <typename T, int BITS, int W, int B>
__global__ void __launch_bounds__(64) compress_strip(StripArgs a) { compress_strip_body<T, BITS, W, B, false>(a); }
template <typename T, int BITS, int W, int B>
__global__ void __launch_bounds__(64) relu_compress_strip(StripArgs a) { compress_strip_body<T, BITS, W, B, true>(a); }
