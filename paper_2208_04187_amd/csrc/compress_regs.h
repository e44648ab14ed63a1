// Part of division.hip (included inside its unnamed namespace, in this order): compress_regs (2-D and 3-D) and relu_compress_regs.

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
// FULL: every one of the K rounds holds units of the plane, so no round is tested (a uniform test per
// round puts each round into a basic block of its own that waits for every load; the instances that
// must test because their planes may be short get a second copy of the body for planes that are not).
template <typename T, int BITS, int B, int NW, bool RELU, int ND = 2, bool FULL = false>
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

    uint32_t blk[K];
    bool full_blocks = false;
    if constexpr (B != 0) full_blocks = (a.H % B) == 0 && (a.W % B) == 0 && (ND == 2 || (a.D % B) == 0);
    const uint32_t tid = threadIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, tid);
    // rounds of units a plane has (uniform); the one- and four-wavefront instances for B = 4 and 8
    // always run all K (their planes fill at least eight of them)
    auto round_live = [&](int k) -> bool { return FULL || (B != 0 && NW != 16 && ND == 2) || (uint32_t)(NT * k) < a.q4; };

    // One plane per workgroup (more workgroups, better balance than several planes each).  Which
    // plane: see xcd_run_index.
    const uint32_t p = xcd_run_index(blockIdx.x, a.P);
    {
        // ---- load the plane first of all: coalesced, bounds-checked (units past the plane read as
        // zero).  Everything the workgroup has to set up (the block of each unit, the sentinel)
        // runs while the loads are in flight.
        float x[K][4];
        {
            const T* src = static_cast<const T*>(pt.x) + (size_t)p * a.HW;
            const __amdgpu_buffer_rsrc_t rsrc =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(src), 0, (int)(a.HW * sizeof(T)), 0x00020000);
            u32x4 q[K];
#pragma unroll
            for (int k = 0; k < K; ++k) {
                q[k] = u32x4{0u, 0u, 0u, 0u};
                if (!round_live(k)) continue;
                if constexpr (sizeof(T) == 4) {
                    q[k] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, tid * 16u, k * NT * 16, kLoadAux);
                } else {
                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                    const u32x2 h = __builtin_amdgcn_raw_buffer_load_b64(rsrc, tid * 8u, k * NT * 8, kLoadAux);
                    q[k].x = h.x; q[k].y = h.y;
                }
            }
            // which block each of the lane's units belongs to (nb = sentinel for units past the plane)
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const uint32_t f = tid + NT * k;
                const uint32_t row = fdiv(f, a.d_w4);          // row, counted over all depth slices
                const uint32_t c4 = f - row * a.w4;
                uint32_t bk;
                if constexpr (ND == 3) {
                    const uint32_t z = fdiv(row, a.d_H);
                    bk = ((z / B) * a.LH + (row - z * a.H) / B) * a.LW + c4 / UPB;
                } else if constexpr (B != 0) bk = (row / B) * a.LW + c4 / UPB;
                else bk = fdiv(row, a.d_B) * a.LW + fdiv(c4, a.d_upb);
                blk[k] = f < a.q4 ? bk : a.nb;
            }
            if (tid == 0) lfcs[a.nb] = __builtin_nanf("");
#pragma unroll
            for (int k = 0; k < K; ++k) {
                if constexpr (sizeof(T) == 4) {
                    x[k][0] = __uint_as_float(q[k].x); x[k][1] = __uint_as_float(q[k].y);
                    x[k][2] = __uint_as_float(q[k].z); x[k][3] = __uint_as_float(q[k].w);
                } else {
                    x[k][0] = __uint_as_float(q[k].x << 16); x[k][1] = __uint_as_float(q[k].x & 0xffff0000u);
                    x[k][2] = __uint_as_float(q[k].y << 16); x[k][3] = __uint_as_float(q[k].y & 0xffff0000u);
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
                    // the whole offset in the vector operand (see store_b128_checked)
                    store_b128_checked(o, yrs, tid * 16u + (uint32_t)(k * NT * 16), 0);
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
            constexpr uint32_t CB = BITS / 2;                         // code bytes per unit (1, 2 or 4; 1-bit codes: half a byte)
            const uint32_t cbytes = BITS == 1 ? (a.q4 + 1u) / 2u : a.q4 * CB;    // code bytes of the plane
            uint8_t* cbase = reinterpret_cast<uint8_t*>(pt.codes) + (size_t)p * a.WPP * 4;
            const __amdgpu_buffer_rsrc_t crs =
                __builtin_amdgcn_make_buffer_rsrc(cbase, 0, (int)cbytes, 0x00020000);
            const uint32_t xw0 = k1 + (2u * tid) * kWeyl;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                if (!round_live(k)) continue;
                const uint32_t xw = xw0 + (uint32_t)(2 * NT * k) * kWeyl;
                uint32_t c = push_pair<BITS>(0u, x[k][2], x[k][3], delta, invs, xw + kWeyl, k2, rscale);
                c = push_pair<BITS>(c, x[k][0], x[k][1], delta, invs, xw, k2, rscale);
                // stores past the plane's code bytes are dropped by the buffer bound
                if constexpr (BITS == 1) {
                    // the four codes of a unit are half a byte: the even lane of a pair stores the byte of
                    // both units (the odd lane's store is dropped; a unit past the plane contributes zeros)
                    c = tid + (uint32_t)(k * NT) < a.q4 ? c : 0u;
                    const uint32_t up = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)c, 0xB1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]
                    __builtin_amdgcn_raw_buffer_store_b8((uint8_t)(c | (up << 4)), crs, (tid & 1u) ? 0x80000000u : (tid >> 1) + (uint32_t)(k * (NT / 2)), 0, 0);
                } else if constexpr (CB == 1) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)c, crs, tid, k * NT, 0);
                else if constexpr (CB == 2) __builtin_amdgcn_raw_buffer_store_b16((uint16_t)c, crs, tid * 2u, k * NT * 2, 0);
                else __builtin_amdgcn_raw_buffer_store_b32(c, crs, tid * 4u, k * NT * 4, 0);
            }
            // pad bytes of the plane's last word are zero
            const uint32_t padb = a.WPP * 4 - cbytes;
            if (tid < padb) cbase[cbytes + tid] = 0;
        }
    }
}

template <typename T, int BITS, int B, int NW>
__global__ void __launch_bounds__(64 * NW) compress_regs(RegsArgs a) {
    if constexpr (B == 0 || NW == 16) {
        if ((uint32_t)(64 * NW * (kRegUnits - 1)) < a.q4) compress_regs_body<T, BITS, B, NW, false, 2, true>(a);
        else compress_regs_body<T, BITS, B, NW, false, 2, false>(a);
    } else {
        compress_regs_body<T, BITS, B, NW, false>(a);
    }
}
template <typename T, int BITS, int B, int NW>
__global__ void __launch_bounds__(64 * NW) relu_compress_regs(RegsArgs a) { compress_regs_body<T, BITS, B, NW, true>(a); }
template <typename T, int BITS, int B, int NW>
__global__ void __launch_bounds__(64 * NW) compress_regs_3d(RegsArgs a) {
    if ((uint32_t)(64 * NW * (kRegUnits - 1)) < a.q4) compress_regs_body<T, BITS, B, NW, false, 3, true>(a);
    else compress_regs_body<T, BITS, B, NW, false, 3, false>(a);
}
