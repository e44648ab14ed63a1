// Part of division.hip (included inside its unnamed namespace, in this order): compress_any (2-D and 3-D).

// ------------------------------------------------------------------ compress, any shape (slow)

struct AnyArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, H, W, HW, LH, LW, nb, WPP, B;      // H, LH: rows / block rows of one depth slice
    uint32_t D;                                     // depth slices (1 for a 2-D map)
};

// One workgroup per plane; x is re-read from global memory in each pass.
// ND = 3: planes of D x H x W elements with blocks of B x B x B (Appendix D).
template <typename T, int BITS, int ND>
__device__ __forceinline__ void compress_any_body(const AnyArgs& a) {
    __shared__ float red_min[kThreads], red_max[kThreads];
    __shared__ float4 sh_params;
    constexpr int CPW = 32 / BITS;
    constexpr float Lf = float((1 << BITS) - 1);
    const uint32_t tid = threadIdx.x;
    const uint32_t p = blockIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, tid);
    const T* xp = static_cast<const T*>(pt.x) + (size_t)p * a.HW;
    const size_t lfc0 = (size_t)p * a.nb;      // this plane's first LFC element

    // pass A: block means; block min/max of the residual follow from the
    // block min/max of x because x -> fl(x - m) is monotone
    float mn = __builtin_inff(), mx = -__builtin_inff();
    for (uint32_t blk = tid; blk < a.nb; blk += kThreads) {
        const uint32_t bq = blk / a.LW, bj = blk - bq * a.LW;
        uint32_t bd = 0, bi = bq;
        if constexpr (ND == 3) { bd = bq / a.LH; bi = bq - bd * a.LH; }
        const uint32_t r1 = min(a.H, (bi + 1) * a.B), c1 = min(a.W, (bj + 1) * a.B);
        const uint32_t z1 = ND == 3 ? min(a.D, (bd + 1) * a.B) : 1u;
        double S = 0.0;
        float xmin = __builtin_inff(), xmax = -__builtin_inff();
        uint32_t cnt = 0;
        for (uint32_t z = bd * a.B; z < z1; ++z)
            for (uint32_t r = bi * a.B; r < r1; ++r)
                for (uint32_t c = bj * a.B; c < c1; ++c) {
                    const float v = Elem<T>::load(xp, ((size_t)z * a.H + r) * a.W + c);
                    S += (double)v; xmin = fminf(xmin, v); xmax = fmaxf(xmax, v); ++cnt;
                }
        const float lfc = lfc_round<T>((float)(S / (double)cnt), kC16<T>);
        lfc_store<T>(pt.lfc, lfc0 + blk, lfc, kC16<T>);
        mn = fminf(mn, xmin - lfc);
        mx = fmaxf(mx, xmax - lfc);
    }
    red_min[tid] = mn; red_max[tid] = mx;
    __syncthreads();
    for (uint32_t off = kThreads / 2; off > 0; off >>= 1) {
        if (tid < off) {
            red_min[tid] = fminf(red_min[tid], red_min[tid + off]);
            red_max[tid] = fmaxf(red_max[tid], red_max[tid + off]);
        }
        __syncthreads();
    }
    if (tid == 0) {
        float delta, Delta, inv;
        plane_scale_any(red_min[0], red_max[0], Lf, kC16<T>, delta, Delta, inv);
        meta_store(pt.meta, p, delta, Delta, kC16<T>);
        const uint32_t k1 = mix32(p ^ pt.seed_a);
        const uint32_t k2 = mix32(k1 + pt.seed_c);
        sh_params = make_float4(delta, inv * 65536.0f, __uint_as_float(k1), __uint_as_float(k2));
    }
    __syncthreads();
    const float delta = sh_params.x, inv16 = sh_params.y;
    const uint32_t k1 = __float_as_uint(sh_params.z), k2 = __float_as_uint(sh_params.w);

    // pass B: quantise and pack, one word per thread
    for (uint32_t k = tid; k < a.WPP; k += kThreads) {
        uint32_t word = 0;
        for (int e = 0; e < CPW; ++e) {
            const uint32_t i = k * CPW + e;
            if (i >= a.HW) break;
            const uint32_t r = i / a.W, c = i - r * a.W;
            uint32_t brow;
            if constexpr (ND == 3) {
                const uint32_t z = r / a.H;
                brow = (z / a.B) * a.LH + (r - z * a.H) / a.B;
            } else {
                brow = r / a.B;
            }
            // written by this workgroup in pass A; visible after the barrier above
            const float lfc = lfc_load<T>(pt.lfc, lfc0 + brow * a.LW + c / a.B, kC16<T>);
            const float h = Elem<T>::load(xp, i) - lfc;
            const uint32_t w = pair_word(k1 + (i >> 1) * kWeyl, k2);
            const uint32_t q = (i & 1u) ? quant<1>(h, delta, inv16, w) : quant<0>(h, delta, inv16, w);
            word |= min(q, (1u << BITS) - 1u) << (e * BITS);      // t may exceed L by a few ulp
        }
        pt.codes[(size_t)p * a.WPP + k] = word;
    }
}

template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) compress_any(AnyArgs a) { compress_any_body<T, BITS, 2>(a); }
template <typename T, int BITS>
__global__ void __launch_bounds__(kThreads) compress_any_3d(AnyArgs a) { compress_any_body<T, BITS, 3>(a); }
