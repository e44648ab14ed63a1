// Part of division.hip (included inside its unnamed namespace, in this order): push_pair (Quant of a pair of elements) and compress_tile.

// ------------------------------------------------------------------ compress, LDS tile

// One pair of elements -> two codes pushed into the packed word (element
// 2j+1 first, then 2j: words are built from the last element down, so that
// element 0 ends in the low bits).  Exact integer evaluation of
// floor(t + r/2^16): T = trunc(t * 2^(32-BITS)), sum = T + (r << (16-BITS)),
// code = top BITS bits of sum.  For BITS <= 4, t <= L(1 + 3 ulp) and r < 2^16 keep the
// sum below 2^32, so no clamp is needed.
template <int BITS>
__device__ __forceinline__ uint32_t push_pair(uint32_t acc, float h0, float h1, float delta, float invs,
                                              uint32_t xw, uint32_t k2, uint32_t rscale) {
    uint32_t x = xw;
    x ^= x >> 16; x *= 0x7feb352du;
    x = x ^ (x >> 15) ^ k2; x *= 0x846ca68bu;
    // final x ^= x >> 16: the high half is unchanged, the low half becomes lo ^ hi
    const uint32_t xl = x ^ (x >> 16);
    uint32_t T1 = (uint32_t)((h1 - delta) * invs);
    uint32_t T0 = (uint32_t)((h0 - delta) * invs);
    if constexpr (BITS == 8) {
        // t may exceed L by a few ulp; with 8-bit codes an ulp of 255 is as large as the random
        // term's step (2^-16), so the sum could wrap: clamp t to L first (the code is L either way)
        T1 = min(T1, 255u << 24);
        T0 = min(T0, 255u << 24);
    }
    uint32_t s1, s0;
    asm("v_mad_u32_u16 %0, %1, %2, %3 op_sel:[1,0,0,0]" : "=v"(s1) : "v"(x), "s"(rscale), "v"(T1));
    asm("v_mad_u32_u16 %0, %1, %2, %3 op_sel:[0,0,0,0]" : "=v"(s0) : "v"(xl), "s"(rscale), "v"(T0));
    acc = __builtin_amdgcn_alignbit(acc, s1, 32 - BITS);
    acc = __builtin_amdgcn_alignbit(acc, s0, 32 - BITS);
    return acc;
}

// T: element type; BITS: code width; B: block size (4 or 8); VEC: elements per
// LDS vector access in the pooling phase (W % VEC == 0, B % VEC == 0);
// NT: threads per workgroup (64 or 256).
template <typename T, int BITS, int B, int VEC, int NT>
__global__ void __launch_bounds__(NT) compress_tile(TileArgs a) {
    extern __shared__ float4 smem4[];
    float4* params = smem4;                                   // [G] (delta, inv scaled, k1, k2)
    float* xs = reinterpret_cast<float*>(smem4 + a.G);        // [G*HW] x, later the residual h
    float* item_min = xs + a.xs_floats;                       // [items_cap]
    float* item_max = item_min + a.items_cap;                 // [items_cap]

    constexpr int IPB = B / VEC;          // pooling items per block (power of two)
    constexpr int CPW = 32 / BITS;        // codes per word
    constexpr float Lf = float((1 << BITS) - 1);
    const uint32_t tid = threadIdx.x;
    const uint32_t p0 = blockIdx.x * a.G;
    const uint32_t Gc = min(a.G, a.P - p0);
    const uint32_t n = Gc * a.HW;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, tid);

    // ---- phase 0: chunk -> LDS (fp32); coalesced 16-byte loads, up to 8 in flight per lane
    {
        const T* src = static_cast<const T*>(pt.x) + (size_t)p0 * a.HW;
        constexpr uint32_t EPV = 16 / sizeof(T);
        constexpr int U = 8;
        const uint32_t nv = a.vec_load ? n / EPV : 0;
        const u32x4* src4 = reinterpret_cast<const u32x4*>(src);
        for (uint32_t v0 = 0; v0 < nv; v0 += U * NT) {
            u32x4 q[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t v = v0 + u * NT + tid;
                if (v < nv) q[u] = __builtin_nontemporal_load(src4 + v);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t v = v0 + u * NT + tid;
                if (v < nv) {
                    if constexpr (sizeof(T) == 4) {
                        reinterpret_cast<u32x4*>(xs)[v] = q[u];
                    } else {
                        float4 lo, hi;
                        lo.x = __uint_as_float(q[u].x << 16); lo.y = __uint_as_float(q[u].x & 0xffff0000u);
                        lo.z = __uint_as_float(q[u].y << 16); lo.w = __uint_as_float(q[u].y & 0xffff0000u);
                        hi.x = __uint_as_float(q[u].z << 16); hi.y = __uint_as_float(q[u].z & 0xffff0000u);
                        hi.z = __uint_as_float(q[u].w << 16); hi.w = __uint_as_float(q[u].w & 0xffff0000u);
                        reinterpret_cast<float4*>(xs)[2 * v] = lo;
                        reinterpret_cast<float4*>(xs)[2 * v + 1] = hi;
                    }
                }
            }
        }
        for (uint32_t e = nv * EPV + tid; e < n; e += NT) xs[e] = Elem<T>::load(src, e);
    }
    lds_barrier();

    // ---- phase 1: block means (Sec. 4.1 AveragePooling), residual in place
    // item = (plane g, block row bi, slot s): B rows x VEC columns of one block;
    // the IPB items of a block sit in adjacent lanes
    const uint32_t nitems = Gc * a.ipp;
    for (uint32_t it0 = 0; it0 < nitems; it0 += NT) {
        const uint32_t it = it0 + tid;
        const uint32_t g = fdiv(it, a.d_ipp);
        const uint32_t rem = it - g * a.ipp;
        const uint32_t bi = fdiv(rem, a.d_ipr);
        const uint32_t s = rem - bi * a.ipr;
        const uint32_t col0 = s * VEC;
        const uint32_t r0 = bi * B;
        const bool valid = it < nitems && col0 < a.W;
        const uint32_t base = g * a.HW + r0 * a.W + col0;

        float v[B][VEC];
        double S = 0.0;
#pragma unroll
        for (int rr = 0; rr < B; ++rr) {
            const bool ok = valid && (r0 + rr < a.H);
#pragma unroll
            for (int c = 0; c < VEC; ++c) v[rr][c] = 0.0f;
            if (ok) {
                const float* src = xs + base + rr * a.W;
                if constexpr (VEC == 4) {
                    float4 q = *reinterpret_cast<const float4*>(src);
                    v[rr][0] = q.x; v[rr][1] = q.y; v[rr][2] = q.z; v[rr][3] = q.w;
                } else if constexpr (VEC == 2) {
                    float2 q = *reinterpret_cast<const float2*>(src);
                    v[rr][0] = q.x; v[rr][1] = q.y;
                } else {
                    v[rr][0] = src[0];
                }
            }
#pragma unroll
            for (int c = 0; c < VEC; ++c) S += (double)v[rr][c];
        }
        S = group_sum<IPB>(S);

        const uint32_t bj = s / IPB;
        const uint32_t rows = min((uint32_t)B, a.H - min(a.H, r0));
        const uint32_t cols = min((uint32_t)B, a.W - min(a.W, bj * B));
        const uint32_t cnt = max(rows * cols, 1u);
        // exact sum / count, one rounding to fp32, then to the storage type
        float m;
        if ((cnt & (cnt - 1)) == 0) m = (float)(S * (1.0 / (double)cnt));   // power of two: exact scaling
        else m = (float)(S / (double)cnt);
        const float lfc = lfc_round<T>(m, kC16<T>);
        if (valid && (s % IPB) == 0)
            lfc_store<T>(pt.lfc, (size_t)(p0 + g) * a.nb + bi * a.LW + bj, lfc, kC16<T>);

        // Sec. 4.1: H^H = H - UpSampling(H^L); written back over x
        float hmin = __builtin_inff(), hmax = -__builtin_inff();
#pragma unroll
        for (int rr = 0; rr < B; ++rr) {
            const bool ok = valid && (r0 + rr < a.H);
            if (ok) {
                float h[VEC];
#pragma unroll
                for (int c = 0; c < VEC; ++c) {
                    h[c] = v[rr][c] - lfc;
                    hmin = fminf(hmin, h[c]);
                    hmax = fmaxf(hmax, h[c]);
                }
                float* dst = xs + base + rr * a.W;
                if constexpr (VEC == 4) *reinterpret_cast<float4*>(dst) = make_float4(h[0], h[1], h[2], h[3]);
                else if constexpr (VEC == 2) *reinterpret_cast<float2*>(dst) = make_float2(h[0], h[1]);
                else dst[0] = h[0];
            }
        }
        if (it < nitems) { item_min[it] = hmin; item_max[it] = hmax; }
    }
    lds_barrier();

    // ---- phase 2: per-plane min / max, scale of Eq. (quantization), keys
    {
        const uint32_t S = a.S;
        const uint32_t groups = NT / S;
        const uint32_t sub = tid & (S - 1);
        for (uint32_t g0 = 0; g0 < Gc; g0 += groups) {
            const uint32_t g = g0 + tid / S;
            const bool live = g < Gc;
            float mn = __builtin_inff(), mx = -__builtin_inff();
            if (live) {
                const uint32_t b0 = g * a.ipp;
                for (uint32_t k = sub; k < a.ipp; k += S) {
                    mn = fminf(mn, item_min[b0 + k]);
                    mx = fmaxf(mx, item_max[b0 + k]);
                }
            }
            group_minmax(S, mn, mx);
            if (live && sub == 0) {
                float delta, Delta, inv;
                plane_scale_any(mn, mx, Lf, kC16<T>, delta, Delta, inv);
                const uint32_t p = p0 + g;
                meta_store(pt.meta, p, delta, Delta, kC16<T>);
                const uint32_t k1 = mix32(p ^ pt.seed_a);
                const uint32_t k2 = mix32(k1 + pt.seed_c);
                params[g] = make_float4(delta, inv * (float)(1u << (32 - BITS)), __uint_as_float(k1), __uint_as_float(k2));
            }
        }
    }
    lds_barrier();

    // ---- phase 3: Quant of Eq. (quantization) + packing, one word per lane
    {
        const uint32_t nwords = Gc * a.WPP;
        const bool hw4 = (a.HW & 3u) == 0;
        const uint32_t rscale = 1u << (16 - BITS);
        for (uint32_t wi = tid; wi < nwords; wi += NT) {
            const uint32_t g = fdiv(wi, a.d_wpp);
            const uint32_t k = wi - g * a.WPP;
            const float4 pr = params[g];
            const float delta = pr.x, invs = pr.y;
            const uint32_t k1 = __float_as_uint(pr.z), k2 = __float_as_uint(pr.w);
            const uint32_t e0 = k * CPW;
            const uint32_t left = a.HW - e0;
            const float* hp = xs + g * a.HW + e0;
            float h[CPW];
            if (hw4 && left >= (uint32_t)CPW) {
#pragma unroll
                for (int q = 0; q < CPW / 4; ++q) {
                    float4 f = reinterpret_cast<const float4*>(hp)[q];
                    h[4 * q] = f.x; h[4 * q + 1] = f.y; h[4 * q + 2] = f.z; h[4 * q + 3] = f.w;
                }
            } else {
                // ragged tail: elements past the plane take h = delta -> t = 0 -> code 0
#pragma unroll
                for (int e = 0; e < CPW; ++e) h[e] = (uint32_t)e < left ? hp[e] : delta;
            }
            const uint32_t xw0 = k1 + (k * (CPW / 2)) * kWeyl;
            uint32_t word = 0;
#pragma unroll
            for (int j = CPW / 2 - 1; j >= 0; --j)
                word = push_pair<BITS>(word, h[2 * j], h[2 * j + 1], delta, invs, xw0 + (uint32_t)j * kWeyl, k2, rscale);
            pt.codes[(size_t)(p0 + g) * a.WPP + k] = word;
        }
    }
}
