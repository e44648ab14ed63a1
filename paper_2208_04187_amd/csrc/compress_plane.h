// Part of division.hip (included inside its unnamed namespace, in this order): compress_plane (2-D and 3-D).

// ------------------------------------------------------------------ compress, planes beyond LDS

struct PlaneArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, W, HW, LW, nb, WPP, B;
    uint32_t D, Hs, LHs;     // depth slices, rows and block rows of one slice (D = 1 for a 2-D map)
    uint32_t nitem;          // D * LHs * LW: blocks of one depth slice each
    uint32_t qv;             // 16-byte vectors per plane
    FastDiv d_W, d_B, d_Hs, d_LW, d_LHs, d_slice;      // d_slice divides by LHs * LW
};

// Planes too large for LDS (the 3-D maps of video models, 2-D maps from 200 x 200 up): one
// workgroup per plane, x is read twice, both times with 16-byte loads (rows and blocks are whole
// vectors here).
//   A. a lane per (depth slice, block): sum, min and max of the block's elements in that slice;
//      neighbouring lanes read neighbouring row segments;
//   B. a lane per block: adds its slices -> LFC (LDS and packed buffer), residual extremes;
//   C. range of the plane, scale of Eq. (quantization), keys, meta;
//   D. a lane per vector: residual against the LFC, Quant, code bytes out (the second read of x
//      comes out of the caches as far as they hold the plane).
template <typename T, int BITS, int ND>
__device__ __forceinline__ void compress_plane_body(const PlaneArgs& a) {
    extern __shared__ float4 smem4[];
    float4* part = smem4;                                          // [nitem] (sum lo, sum hi, min, max)
    float* lfcs = reinterpret_cast<float*>(part + a.nitem);       // [nb]
    float* red = lfcs + ((a.nb + 3u) & ~3u);                       // [2 * kThreads / 64] + 4 params
    constexpr uint32_t EPV = 16 / sizeof(T);
    constexpr uint32_t CBV = EPV * BITS / 8;
    constexpr float Lf = float((1 << BITS) - 1);
    const uint32_t tid = threadIdx.x;
    const uint32_t p = blockIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, tid);
    const u32x4* xv = reinterpret_cast<const u32x4*>(static_cast<const T*>(pt.x) + (size_t)p * a.HW);
    const uint32_t wv = a.W / EPV;                                 // vectors per row
    const uint32_t slice = a.LHs * a.LW;

    // ---- A. blocks of one slice (Sec. 4.1 / Appendix D AveragePooling, first half)
    for (uint32_t it = tid; it < a.nitem; it += kThreads) {
        const uint32_t z = fdiv(it, a.d_slice);
        const uint32_t rem = it - z * slice;
        const uint32_t bi = fdiv(rem, a.d_LW);
        const uint32_t bj = rem - bi * a.LW;
        const uint32_t r0 = bi * a.B, c0 = bj * a.B;
        const uint32_t rows = min(a.B, a.Hs - r0);
        const uint32_t nvec = min(a.B, a.W - c0) / EPV;
        const u32x4* src = xv + (size_t)(z * a.Hs + r0) * wv + c0 / EPV;
        double S = 0.0;
        float mn = __builtin_inff(), mx = -__builtin_inff();
        for (uint32_t rr = 0; rr < rows; ++rr) {
            for (uint32_t u = 0; u < nvec; ++u) {
                float f[EPV];
                unpack_vec<T>(src[(size_t)rr * wv + u], f);
                S += ((double)f[0] + (double)f[1]) + ((double)f[2] + (double)f[3]);
                mn = fminf(mn, fminf(fminf(f[0], f[1]), fminf(f[2], f[3])));
                mx = fmaxf(mx, fmaxf(fmaxf(f[0], f[1]), fmaxf(f[2], f[3])));
                if constexpr (EPV == 8) {
                    S += ((double)f[4] + (double)f[5]) + ((double)f[6] + (double)f[7]);
                    mn = fminf(mn, fminf(fminf(f[4], f[5]), fminf(f[6], f[7])));
                    mx = fmaxf(mx, fmaxf(fmaxf(f[4], f[5]), fmaxf(f[6], f[7])));
                }
            }
        }
        const uint64_t sb = (uint64_t)__double_as_longlong(S);
        part[it] = make_float4(__uint_as_float((uint32_t)sb), __uint_as_float((uint32_t)(sb >> 32)), mn, mx);
    }
    lds_barrier();

    // ---- B. blocks: LFC and residual extremes.  All lanes of a wavefront run the loop body
    // (mean_of votes across the wavefront); slots past the plane redo block 0.
    float mn = __builtin_inff(), mx = -__builtin_inff();
    for (uint32_t t0 = 0; t0 < a.nb; t0 += kThreads) {
        const uint32_t t = t0 + tid;
        const bool live = t < a.nb;
        const uint32_t blk = live ? t : 0u;
        const uint32_t bd = fdiv(blk, a.d_slice);
        const uint32_t rem = blk - bd * slice;
        const uint32_t bi = fdiv(rem, a.d_LW);
        const uint32_t bj = rem - bi * a.LW;
        const uint32_t rows = min(a.B, a.Hs - bi * a.B);
        const uint32_t cols = min(a.B, a.W - bj * a.B);
        const uint32_t z0 = bd * a.B;
        const uint32_t deps = min(a.B, a.D - z0);
        double S = 0.0;
        float bmn = __builtin_inff(), bmx = -__builtin_inff();
#pragma unroll 4
        for (uint32_t z = 0; z < deps; ++z) {
            const float4 q = part[(z0 + z) * slice + rem];
            S += __longlong_as_double((long long)(((uint64_t)__float_as_uint(q.y) << 32) | __float_as_uint(q.x)));
            bmn = fminf(bmn, q.z);
            bmx = fmaxf(bmx, q.w);
        }
        const float lfc = lfc_round<T>(mean_of(S, deps * rows * cols), kC16<T>);
        if (live) {
            lfcs[t] = lfc;
            lfc_store<T>(pt.lfc, (size_t)p * a.nb + t, lfc, kC16<T>);
            mn = fminf(mn, bmn - lfc);               // x -> fl(x - m) is monotone
            mx = fmaxf(mx, bmx - lfc);
        }
    }

    // ---- C. range of the plane, scale, keys, meta
    group_minmax(64, mn, mx);
    if ((tid & 63u) == 0) { red[2 * (tid >> 6)] = mn; red[2 * (tid >> 6) + 1] = mx; }
    lds_barrier();
    if (tid == 0) {
        for (uint32_t w = 0; w < kThreads / 64; ++w) { mn = fminf(mn, red[2 * w]); mx = fmaxf(mx, red[2 * w + 1]); }
        float delta, Delta, inv;
        plane_scale_any(mn, mx, Lf, kC16<T>, delta, Delta, inv);
        meta_store(pt.meta, p, delta, Delta, kC16<T>);
        const uint32_t k1 = mix32(p ^ pt.seed_a);
        const uint32_t k2 = mix32(k1 + pt.seed_c);
        float4* prm = reinterpret_cast<float4*>(red + 2 * (kThreads / 64));
        *prm = make_float4(delta, inv * (float)(1u << (32 - BITS)), __uint_as_float(k1), __uint_as_float(k2));
    }
    lds_barrier();
    const float4 pr = *reinterpret_cast<const float4*>(red + 2 * (kThreads / 64));

    // ---- D. residual, Quant, packing: a vector per lane and step, four steps in flight
    uint8_t* cbase = reinterpret_cast<uint8_t*>(pt.codes) + (size_t)p * a.WPP * 4;
    constexpr int U = 4;
    for (uint32_t v0 = 0; v0 < a.qv; v0 += U * kThreads) {
        u32x4 q[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t v = v0 + u * kThreads + tid;
            if (v < a.qv) q[u] = xv[v];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t v = v0 + u * kThreads + tid;
            if (v < a.qv) quant_vector<T, BITS, ND>(a, q[u], v, pr, lfcs, cbase);
        }
    }
    const uint32_t padb = a.WPP * 4 - a.qv * CBV;                  // pad bytes of the last word are zero
    if (tid < padb) cbase[a.qv * CBV + tid] = 0;
}

template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) compress_plane(PlaneArgs a) { compress_plane_body<T, BITS, 2>(a); }
template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) compress_plane_3d(PlaneArgs a) { compress_plane_body<T, BITS, 3>(a); }
