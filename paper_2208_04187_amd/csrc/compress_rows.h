// Part of division.hip (included inside its unnamed namespace, in this order): compress_rows (2-D and 3-D).

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
