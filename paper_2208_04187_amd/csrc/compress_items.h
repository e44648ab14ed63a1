// Part of division.hip (included inside its unnamed namespace, in this order): compress_items.

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
    void* y;             // relu_compress_items: the activation's output map and its 1-bit mask (one map per launch);
    uint32_t* mask;      // rpw * ppr * HW is a multiple of 32 then: a workgroup's mask bits are whole words
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
// RELU: x is the input of a Relu operator (Appendix, Relu listing) whose output y is the map to
// cache: y = x where x > 0 else +0 is written out row by row as it was loaded, and y is what gets
// compressed.  The 1-bit mask (bit i of the whole map = x_i > 0) of the planes a workgroup handles
// is OR-ed together in LDS and leaves as whole words when the workgroup is done.
template <typename T, int BITS, int B, int VEC, int R, bool RELU>
__device__ __forceinline__ void compress_items_body(const ItemsArgs& a) {
    constexpr int IPB = B / VEC;          // items per block (power of two)
    constexpr int CPW = 32 / BITS;        // codes per word
    constexpr float Lf = float((1 << BITS) - 1);
    extern __shared__ float4 smem4[];
    uint32_t* cw = reinterpret_cast<uint32_t*>(smem4);        // [ppr * WPP] packed words of the round
    uint32_t* mw = cw + ((a.ppr * a.WPP + 3u) & ~3u);         // RELU: [rpw * ppr * HW / 32] mask words of the workgroup

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

    const uint32_t wg = xcd_run_index(blockIdx.x, gridDim.x);   // which run of rpw rounds this workgroup takes
    const uint32_t rend = min(a.nrounds, (wg + 1) * a.rpw);
    const uint32_t mbits = a.rpw * a.ppr * a.HW;               // RELU: mask bits of a workgroup (a multiple of 32)
    if constexpr (RELU) {
        for (uint32_t w = lane; w < mbits / 32u; w += 64) mw[w] = 0u;
        wave_sync();
    }
    for (uint32_t round = wg * a.rpw; round < rend; ++round) {
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
                    const u32x4 q = __builtin_amdgcn_raw_buffer_load_b128(rsrc, vo, so, kLoadReuse);
                    v[rr][0] = __uint_as_float(q.x); v[rr][1] = __uint_as_float(q.y);
                    v[rr][2] = __uint_as_float(q.z); v[rr][3] = __uint_as_float(q.w);
                } else if constexpr (sizeof(T) == 4 && VEC == 2) {
                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                    const u32x2 q = __builtin_amdgcn_raw_buffer_load_b64(rsrc, vo, so, kLoadReuse);
                    v[rr][0] = __uint_as_float(q.x); v[rr][1] = __uint_as_float(q.y);
                } else if constexpr (VEC == 4) {
                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                    const u32x2 q = __builtin_amdgcn_raw_buffer_load_b64(rsrc, vo, so, kLoadReuse);
                    v[rr][0] = __uint_as_float(q.x << 16); v[rr][1] = __uint_as_float(q.x & 0xffff0000u);
                    v[rr][2] = __uint_as_float(q.y << 16); v[rr][3] = __uint_as_float(q.y & 0xffff0000u);
                } else {
                    const uint32_t q = __builtin_amdgcn_raw_buffer_load_b32(rsrc, vo, so, kLoadReuse);
                    v[rr][0] = __uint_as_float(q << 16); v[rr][1] = __uint_as_float(q & 0xffff0000u);
                }
            }
        }
        // the round's packed words start at zero
        for (uint32_t w = lane; w < rwords; w += 64) cw[w] = 0u;
        if constexpr (RELU) {
            // y = Relu(x) back to memory the way x came in, the mask bits of the rows into LDS
            T* ydst = static_cast<T*>(a.y) + (size_t)p0 * a.HW;
            const __amdgpu_buffer_rsrc_t yrs =
                __builtin_amdgcn_make_buffer_rsrc(ydst, 0, (int)(Gc * a.HW * sizeof(T)), 0x00020000);
            const uint32_t base = (g * a.HW + off) * (uint32_t)sizeof(T);
            const uint32_t rowb = a.W * (uint32_t)sizeof(T);
            const uint32_t bit0 = (round - wg * a.rpw) * a.ppr * a.HW + g * a.HW + off;    // of the item's first row
#pragma unroll
            for (int rr = 0; rr < R; ++rr) {
                uint32_t bits = 0;
#pragma unroll
                for (int c = 0; c < VEC; ++c) {
                    const bool pos = v[rr][c] > 0.0f;
                    bits |= (pos ? 1u : 0u) << c;
                    v[rr][c] = pos ? v[rr][c] : 0.0f;
                }
                if (!valid || !(fullrows || (uint32_t)rr < nrows)) continue;
                const uint32_t vo = base + (uint32_t)rr * rowb;
                if constexpr (sizeof(T) == 4 && VEC == 4) {
                    u32x4 o;
                    o.x = __float_as_uint(v[rr][0]); o.y = __float_as_uint(v[rr][1]);
                    o.z = __float_as_uint(v[rr][2]); o.w = __float_as_uint(v[rr][3]);
                    __builtin_amdgcn_raw_buffer_store_b128(o, yrs, vo, 0, 0);
                } else if constexpr (sizeof(T) == 4 && VEC == 2) {
                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                    u32x2 o;
                    o.x = __float_as_uint(v[rr][0]); o.y = __float_as_uint(v[rr][1]);
                    __builtin_amdgcn_raw_buffer_store_b64(o, yrs, vo, 0, 0);
                } else if constexpr (VEC == 4) {
                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                    u32x2 o;
                    o.x = (__float_as_uint(v[rr][0]) >> 16) | (__float_as_uint(v[rr][1]) & 0xffff0000u);
                    o.y = (__float_as_uint(v[rr][2]) >> 16) | (__float_as_uint(v[rr][3]) & 0xffff0000u);
                    __builtin_amdgcn_raw_buffer_store_b64(o, yrs, vo, 0, 0);
                } else {
                    __builtin_amdgcn_raw_buffer_store_b32((__float_as_uint(v[rr][0]) >> 16) | (__float_as_uint(v[rr][1]) & 0xffff0000u),
                                                          yrs, vo, 0, 0);
                }
                const uint32_t e = bit0 + (uint32_t)rr * a.W;          // VEC bits inside one word (e is a multiple of VEC)
                if (bits) __hip_atomic_fetch_or(mw + e / 32u, bits << (e % 32u), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }

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
    if constexpr (RELU) {
        // the workgroup's mask words: bits [wg * mbits, ...) of the map, as far as the map goes
        const uint64_t first = (uint64_t)wg * mbits;
        const uint64_t total = (uint64_t)a.P * a.HW;
        const uint32_t nbits = (uint32_t)min((uint64_t)mbits, total - first);
        uint32_t* dst = a.mask + first / 32u;
        for (uint32_t w = lane; w < (nbits + 31u) / 32u; w += 64) dst[w] = mw[w];
    }
}

template <typename T, int BITS, int B, int VEC, int R>
__global__ void __launch_bounds__(64) compress_items(ItemsArgs a) { compress_items_body<T, BITS, B, VEC, R, false>(a); }
template <typename T, int BITS, int B, int VEC>
__global__ void __launch_bounds__(64) relu_compress_items(ItemsArgs a) { compress_items_body<T, BITS, B, VEC, B, true>(a); }
