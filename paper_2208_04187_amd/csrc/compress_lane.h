// Part of division.hip (included inside its unnamed namespace, in this order): compress_lane.

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

    const uint32_t wg = xcd_run_index(blockIdx.x, gridDim.x);   // which run of rpw rounds this workgroup takes
    const uint32_t rend = min(a.nrounds, (wg + 1) * a.rpw);
    for (uint32_t round = wg * a.rpw; round < rend; ++round) {
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
