// Part of division.hip (included inside its unnamed namespace, after compress_strip.h): compress_rowstrip.

// ------------------------------------------------------------------ compress, a row of an odd-width plane per lane

// Geometry for planes of an odd width W (13, 15, 17, 27, 35, 55: maps of AlexNet and Inception-v3).
template <int W>
struct RowStripGeom {
    static_assert(W % 2 == 1 && W <= 64, "odd widths up to 64");
    static constexpr int S = W <= 16 ? 16 : W <= 32 ? 32 : 64;   // lane slots per plane = rows a plane may have
    static constexpr int G = 64 / S;                             // planes per round
    static constexpr int LPL = (G * S * W + 255) / 256;          // 16-byte units a lane loads: a round of G planes of S rows
    static constexpr int NP = (W + 1) / 2;                       // element pairs a row touches
};

// The strip kernel for planes whose rows are not whole 16-byte vectors: a lane owns one ROW of W
// elements (W odd, compile-time) and keeps it in registers from the pooling to the codes; the lanes
// of a plane sit side by side (16, 32 or 64 slots), B = 4 or 8 rows of a block row are an aligned DPP
// group, so block sums and the plane's extremes are DPP reductions as in compress_strip.  The round
// (its planes are contiguous) is read with coalesced 16-byte loads into LDS in the map's own order
// (a round starts on a 4-byte boundary at least, which is all a buffer load needs); a lane takes
// its row out with scalar LDS reads (stride W words, odd: no bank conflicts inside a plane).
//
// Codes: the random word of Eq. (quantization)'s stochastic rounding belongs to a PAIR of elements
// (2j, 2j+1) of the plane, and with W odd every other row starts in the middle of a pair.  A lane
// therefore quantises the NP = (W+1)/2 pairs its row touches: its W elements shifted by the parity
// of its first element, the one slot that belongs to the neighbouring row filled with delta (code 0).
// Its (W+1) * BITS code bits start at an even element of the plane, anywhere in a word: they are
// built as words from bit 0, shifted as one string and OR-ed into the plane's cleared code words in
// LDS (the neighbour's bits of a shared word arrive by its own OR), which then leave as whole
// coalesced words.  One round per workgroup of one wavefront.
template <typename T, int BITS, int W, int B>
__global__ void __launch_bounds__(64) compress_rowstrip(StripArgs a) {
    using Geo = RowStripGeom<W>;
    constexpr int S = Geo::S, G = Geo::G, LPL = Geo::LPL, NP = Geo::NP;
    constexpr int NSEG = (W + B - 1) / B;       // blocks per block row
    constexpr int PPW = 16 / BITS;              // element pairs per code word
    constexpr int NWD = (NP + PPW - 1) / PPW;   // code words a row's pairs fill when they start at bit 0
    static_assert(B == 4 || B == 8, "block rows are DPP groups");
    constexpr float Lf = float((1 << BITS) - 1);
    extern __shared__ float4 smem4[];
    float* xs = reinterpret_cast<float*>(smem4);                     // the round, later its code words

    const uint32_t lane = threadIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, lane);
    const uint32_t round = xcd_run_index(blockIdx.x, a.nrounds);
    const uint32_t p0 = round * G;
    const uint32_t Gc = min((uint32_t)G, a.P - p0);

    // ---- the round's loads first: coalesced, bounds-checked (units past the round read as zero)
    u32x4 q[LPL];
    {
        const T* src = static_cast<const T*>(pt.x) + (size_t)p0 * a.HW;
        // the range ends with the dword that holds the round's last element (2-byte elements, an odd number of
        // them: the bounds check is per dword, and the dword's other half is the next plane's first element or
        // the two bytes behind the map, inside the same aligned dword)
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(src), 0, (int)((Gc * a.HW * sizeof(T) + 3u) & ~3u), 0x00020000);
#pragma unroll
        for (int k = 0; k < LPL; ++k) {
            if constexpr (sizeof(T) == 4) {
                q[k] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane * 16u + (uint32_t)(k * 1024), 0, kLoadAux);
            } else {
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                const u32x2 h = __builtin_amdgcn_raw_buffer_load_b64(rsrc, lane * 8u + (uint32_t)(k * 512), 0, kLoadAux);
                q[k] = u32x4{h.x << 16, h.x & 0xffff0000u, h.y << 16, h.y & 0xffff0000u};
            }
        }
    }
    // the lane's place: plane g of the round, row sl of the plane
    const uint32_t g = lane / S, sl = lane % S;
    const bool live = g < Gc;
    const bool valid = live && sl < a.H;
    const uint32_t bi = sl / B;                                        // block row of the row
    const uint32_t rows = min((uint32_t)B, a.H - min(a.H, bi * (uint32_t)B));   // rows of that block row that exist
    const uint32_t p = p0 + g;
    const uint32_t k1 = mix32(p ^ pt.seed_a);
    const uint32_t k2 = mix32(k1 + pt.seed_c);
    const uint32_t rscale = 1u << (16 - BITS);
    const uint32_t xv = (G * a.HW + 3u) / 4u;                          // units of a whole round (the host sized LDS for them)
#pragma unroll
    for (int k = 0; k < LPL; ++k)
        if (lane + 64u * k < xv) reinterpret_cast<u32x4*>(xs)[lane + 64 * k] = q[k];
    wave_sync();

    // ---- the row; lanes without one take row 0 of the round and have their effects masked
    float x[W];
    {
        const float* sp = xs + (valid ? g * a.HW + sl * (uint32_t)W : 0u);
#pragma unroll
        for (int e = 0; e < W; ++e) x[e] = sp[e];
    }

    // ---- Sec. 4.1 AveragePooling: the row's share of each block of its block row, then the block
    // row's lanes together (binary64, fixed order)
    double Sm[NSEG];
#pragma unroll
    for (int s = 0; s < NSEG; ++s) Sm[s] = 0.0;
#pragma unroll
    for (int e = 0; e < W; ++e) Sm[e / B] += (double)x[e];
    float lfc[NSEG];
#pragma unroll
    for (int s = 0; s < NSEG; ++s) {
        const double Sb = group_sum<B>(valid ? Sm[s] : 0.0);
        const uint32_t cols = (uint32_t)(W - B * s < B ? W - B * s : B);     // a constant once the loop is unrolled
        lfc[s] = lfc_round<T>(mean_of(Sb, max(rows, 1u) * cols), kC16<T>);
    }
    if (valid && sl % B == 0) {
#pragma unroll
        for (int s = 0; s < NSEG; ++s) lfc_store<T>(pt.lfc, (size_t)p * a.nb + bi * NSEG + s, lfc[s], kC16<T>);
    }

    // ---- residual H^H = H - UpSampling(H^L) in place, the plane's extremes
    float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
    for (int e = 0; e < W; ++e) {
        x[e] = x[e] - lfc[e / B];
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

    // ---- Quant + packing (every lane has taken its row out of LDS by now)
    wave_sync();
    uint32_t* cw = reinterpret_cast<uint32_t*>(xs);
    const uint32_t nwords = Gc * a.WPP;
    {
        const u32x4 z{0u, 0u, 0u, 0u};
        for (uint32_t i = lane; i * 4u < nwords; i += 64) reinterpret_cast<u32x4*>(cw)[i] = z;
    }
    wave_sync();
    {
        const uint32_t f0 = sl * (uint32_t)W;            // the row's first element in the plane
        const bool odd = (f0 & 1u) != 0;                 // it is the second element of its pair
        const uint32_t j0 = f0 >> 1;                     // first pair the row touches
        uint32_t w[NWD];
#pragma unroll
        for (int wi = 0; wi < NWD; ++wi) {
            uint32_t acc = 0;
#pragma unroll
            for (int pj = PPW - 1; pj >= 0; --pj) {
                const int jj = wi * PPW + pj;
                if (jj >= NP) continue;
                // slots 2jj and 2jj+1 of the row's pairs: elements 2jj - odd and 2jj + 1 - odd of the row
                const float e_even = 2 * jj < W ? x[2 * jj < W ? 2 * jj : 0] : delta;               // slot 2jj, row starts a pair
                const float e_odd0 = 2 * jj >= 1 ? x[2 * jj >= 1 ? 2 * jj - 1 : 0] : delta;         // slot 2jj, row starts mid-pair
                const float f_even = 2 * jj + 1 < W ? x[2 * jj + 1 < W ? 2 * jj + 1 : 0] : delta;   // slot 2jj+1
                const float f_odd0 = x[2 * jj < W ? 2 * jj : 0];                                    // slot 2jj+1, mid-pair (2jj <= W-1)
                const float h0 = odd ? e_odd0 : e_even;
                const float h1 = odd ? f_odd0 : f_even;
                acc = push_pair<BITS>(acc, h0, h1, delta, invs, k1 + (j0 + (uint32_t)jj) * kWeyl, k2, rscale);
            }
            w[wi] = acc;
        }
        if (valid) {
            const uint32_t bit = 2u * j0 * (uint32_t)BITS;           // where the row's string starts in the plane's code bits
            const uint32_t sh = bit & 31u;
            uint32_t* pw = cw + g * a.WPP + (bit >> 5);
#pragma unroll
            for (int i = 0; i <= NWD; ++i) {
                const uint64_t two = ((uint64_t)(i < NWD ? w[i < NWD ? i : 0] : 0u) << 32) | (i > 0 ? w[i > 0 ? i - 1 : 0] : 0u);
                const uint32_t v = (uint32_t)(two >> (32u - sh));
                // a word that is all zero adds nothing (the slots past the row's own elements are zero)
                if (v != 0u) __hip_atomic_fetch_or(pw + i, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
    }
    wave_sync();
    {
        uint32_t* dst = pt.codes + (size_t)p0 * a.WPP;
        for (uint32_t wd = lane; wd < nwords; wd += 64) dst[wd] = cw[wd];
    }
}
