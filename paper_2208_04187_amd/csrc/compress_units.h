// Part of division.hip (included inside its unnamed namespace, in this order): compress_units.

// ------------------------------------------------------------------ compress, plane in registers, any width

struct UnitsArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, H, W, HW, LW, nb, WPP, B;      // H = rows of one depth slice
    uint32_t D, LH, Bz;  // depth slices (1: a 2-D map), block rows per slice, depth of a block (B, or 1 for 2-D maps)
    uint32_t q4;         // units (4 consecutive elements) per plane, the last one may be partly past it
    uint32_t q4p;        // q4 rounded up to whole rounds of the plane's lanes
    uint32_t nitem;      // nb * Bz * B row segments
    uint32_t S, S_log2;  // instance NW = 0: lanes per plane (8, 16 or 32), 64 / S planes per wavefront
    uint32_t reg_bytes;  // LDS bytes of one plane's region (a multiple of 16)
    uint32_t nrounds;    // rounds of planes the grid walks over: P, or P / (64 / S) rounded up (NW = 0)
    FastDiv d_W, d_B, d_LW, d_H, d_BBz, d_slice;      // d_BBz divides by Bz * B, d_slice by LH * LW
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
// 3-D maps (Appendix D): planes of D x H x W elements with blocks of B x B x B; an element's block
// and the row segments of a block are found with the depth as a third coordinate, the rest is the same.
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
            const uint32_t ra = fdiv(e, a.d_W);                       // row, counted over all depth slices
            const uint32_t c = e - ra * a.W;
            const uint32_t z = fdiv(ra, a.d_H);
            const uint32_t r = ra - z * a.H;
            off[j] = 4u * (e < a.HW ? (fdiv(z, a.d_B) * a.LH + fdiv(r, a.d_B)) * a.LW + fdiv(c, a.d_B) : a.nb);
        }
        lo[k][0] = off[0] | (off[1] << 16);
        lo[k][1] = off[2] | (off[3] << 16);
    }
    // the row segments of the lane (item i = (block * Bz + slice of the block) * B + row of the block):
    // where the segment starts in the plane, and in the top bits how many elements it has (0: a row or
    // slice past the map, or no item)
    uint32_t it[K];
#pragma unroll
    for (int m = 0; m < K; ++m) {
        const uint32_t i = l + S * m;
        const uint32_t t = fdiv(i, a.d_BBz), rem = i - t * (a.Bz * a.B);
        const uint32_t zz = fdiv(rem, a.d_B), rr = rem - zz * a.B;
        const uint32_t bd = fdiv(t, a.d_slice), t2 = t - bd * (a.LH * a.LW);
        const uint32_t bi = fdiv(t2, a.d_LW), bj = t2 - bi * a.LW;
        const uint32_t z = bd * a.B + zz, r = bi * a.B + rr;
        const uint32_t bw = min(a.B, a.W - bj * a.B);
        it[m] = (i < a.nitem && z < a.D && r < a.H) ? ((z * a.H + r) * a.W + bj * a.B) | (bw << 20) : 0u;
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

        // ---- step 2: a lane per block adds its rows, slice by slice from the top down
        for (uint32_t t = l; t < a.nb; t += S) {
            const uint32_t bd = fdiv(t, a.d_slice), t2 = t - bd * (a.LH * a.LW);
            const uint32_t bi = fdiv(t2, a.d_LW), bj = t2 - bi * a.LW;
            const uint32_t deps = min(a.Bz, a.D - bd * a.B);
            const uint32_t rows = min(a.B, a.H - bi * a.B);
            const uint32_t bw = min(a.B, a.W - bj * a.B);
            double Sb = 0.0;
            for (uint32_t zz = 0; zz < deps; ++zz)
                for (uint32_t rr = 0; rr < rows; ++rr) Sb += rsum[(t * a.Bz + zz) * a.B + rr];
            const float lfc = lfc_round<T>(mean_of(Sb, deps * rows * bw), kC16<T>);
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
            constexpr uint32_t CB = BITS / 2;                         // code bytes per unit (1, 2 or 4; 1-bit codes: half a byte)
            const uint32_t cbytes = BITS == 1 ? (a.q4 + 1u) / 2u : a.q4 * CB;    // code bytes of a plane
            // NW >= 1: the buffer ends with the plane's last unit, so that stores of units past the plane
            // are dropped; NW = 0: it ends with the round's last plane, units past a plane are skipped
            const uint32_t pf = rd * G;
            uint8_t* cround = reinterpret_cast<uint8_t*>(pt.codes) + (size_t)pf * a.WPP * 4;
            const __amdgpu_buffer_rsrc_t crs = __builtin_amdgcn_make_buffer_rsrc(
                cround, 0, (int)(SUB ? min(G, a.P - pf) * a.WPP * 4u : cbytes), 0x00020000);
            const uint32_t cvoff = g * a.WPP * 4u + l * CB;
            const uint32_t cvoff1 = (l & 1u) ? 0x80000000u : g * a.WPP * 4u + (l >> 1);     // 1-bit codes: the odd lane stores nothing
            (void)cvoff1;
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
                if constexpr (BITS == 1) {
                    // the four codes of a unit are half a byte: the even lane of a pair stores the byte of both
                    // units (a unit past the plane contributes zeros, the odd lane's store is dropped)
                    const bool in = l + S * k < a.q4;
                    c = in ? c : 0u;
                    c |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)c, 0xB1, 0xf, 0xf, true) << 4;   // quad_perm [1,0,3,2]
                    __builtin_amdgcn_raw_buffer_store_b8((uint8_t)c, crs, in ? cvoff1 + (uint32_t)(S * k / 2) : 0x80000000u, 0, 0);
                    continue;
                }
                if (SUB && l + S * k >= a.q4) continue;
                if constexpr (CB == 1) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)c, crs, cvoff, (int)(S * k), 0);
                else if constexpr (CB == 2) __builtin_amdgcn_raw_buffer_store_b16((uint16_t)c, crs, cvoff, (int)(S * k * 2), 0);
                else __builtin_amdgcn_raw_buffer_store_b32(c, crs, cvoff, (int)(S * k * 4), 0);
            }
            // pad bytes of the plane's last word are zero
            const uint32_t padb = a.WPP * 4 - cbytes;
            if (l < padb && pv) cround[(size_t)g * a.WPP * 4 + cbytes + l] = 0;
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
