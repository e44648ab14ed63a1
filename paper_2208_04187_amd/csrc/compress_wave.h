// Part of division.hip (included inside its unnamed namespace, in this order): compress_wave.

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

// (float)(S / cnt) for a positive integer cnt, the way the reference definition rounds it
// (binary64 quotient, then one rounding to binary32), without a binary64 division in the common
// case.  q = fl(S * fl(1/cnt)) carries two roundings of relative size 2^-53 each, so it lies within
// 2^-52 |S/cnt| <= 2 ulp of the exact quotient, i.e. within 3 ulp of the binary64 quotient
// d = fl(S/cnt) (half an ulp from the exact one, plus q's own grid).  q and d round to the same
// binary32 unless a rounding boundary of binary32 lies between them.  For a normal binary32 result
// those boundaries are the binary64 numbers whose low 29 bits read 1000...0 (and, for d itself to
// land on the other side, nothing closer than that): if the low 29 bits of q are at least 16 ulp
// from that pattern, no boundary is within 16 ulp of q, d is within 3, so both round alike.
// A nonzero q below 2^-126 rounds to a subnormal binary32, which drops more than 29 bits, so the
// pattern test does not see its boundaries: it takes the division.  (q >= 2^-126 > d cannot
// disagree: d is then within 3 ulp below 2^-126, q's low bits are near zero, both round to 2^-126.)
// S is a sum of binary32 values, at least 2^-149 in magnitude when nonzero, so neither q nor d is
// a subnormal binary64; cnt < 2^32 is exact in binary64.  mean_rule_divides says whether q may
// stand in for d; it is host code too, so that a test can run the rule without a GPU.
__host__ __device__ __forceinline__ bool mean_rule_divides(double q) {
    uint64_t bits;
    __builtin_memcpy(&bits, &q, sizeof bits);
    const uint32_t low = (uint32_t)bits & 0x1fffffffu;
    const uint32_t dist = low > 0x10000000u ? low - 0x10000000u : 0x10000000u - low;
    const bool subnormal = q != 0.0 && __builtin_fabs(q) < 0x1p-126;
    return dist < 16u || subnormal;
}
__host__ __device__ __forceinline__ bool mean_count_is_power_of_two(uint32_t cnt) { return (cnt & (cnt - 1)) == 0; }

// The rule on the device: when any lane of the wavefront needs the division, all take it.
// rcp must be the binary64 quotient 1.0 / cnt (a kernel that needs the mean of many blocks of one size
// divides once and passes it in).
__device__ __forceinline__ float mean_with_rcp(double S, uint32_t cnt, double rcp) {
    if (mean_count_is_power_of_two(cnt)) return (float)(S * rcp);     // exact scaling
    const double q = S * rcp;
    if (__builtin_expect(__any(mean_rule_divides(q)), 0)) return (float)(S / (double)cnt);
    return (float)q;
}
__device__ __forceinline__ float mean_of(double S, uint32_t cnt) { return mean_with_rcp(S, cnt, 1.0 / (double)cnt); }

// The rule for one value on the host (what a lane whose neighbours do not ask for the division computes).
inline float mean_of_host(double S, uint32_t cnt, int* divided) {
    *divided = 0;
    if (mean_count_is_power_of_two(cnt)) return (float)(S * (1.0 / (double)cnt));
    const double q = S * (1.0 / (double)cnt);
    if (mean_rule_divides(q)) { *divided = 1; return (float)(S / (double)cnt); }
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
