// Part of division.hip (included inside its unnamed namespace, in this order): compress_one and compress_line.

// ------------------------------------------------------------------ compress, planes that are one block

struct OneArgs {
    CompTab tab;
    Regions rg;
    uint32_t P, HW, WPP;
    uint32_t qv;         // 16-byte vectors per plane
    uint32_t S, S_log2;  // lanes per plane (power of two, at most 64)
    uint32_t ppw;        // planes per wavefront = 64 / S
    uint32_t upb, upb_log2;  // compress_line: vectors per block (power of two, at most S); nb = blocks per plane
    uint32_t nb;
    uint32_t K;          // rounds of the instance to launch (3, 6, 12 or 13): not read by the kernels
    uint32_t NG;         // compress_line: groups of 64 / S planes per wavefront (1, or 12 / rounds per plane for tiny planes)
};

constexpr int kOneUnits = 13;     // vectors per lane: planes of up to 13 * 64 vectors

// sum over aligned groups of S lanes (S a power of two <= 64, uniform in the wave) in a fixed
// order, result in every lane of the group; all lanes must be active
__device__ __forceinline__ double group_sum_any(uint32_t S, double v) {
    if (S >= 2)  v += dpp_f64<kDppXor1>(v);
    if (S >= 4)  v += dpp_f64<kDppXor2>(v);
    if (S >= 8)  v += dpp_f64<kDppHalfMirror>(v);
    if (S >= 16) v += dpp_f64<kDppMirror>(v);
    if (S >= 32) {
        const uint64_t u = (uint64_t)__double_as_longlong(v);
        const int lo = (int)(uint32_t)u, hi = (int)(uint32_t)(u >> 32);
        auto row = [&](int lane) -> double {
            const uint32_t l = (uint32_t)__builtin_amdgcn_readlane(lo, lane), h = (uint32_t)__builtin_amdgcn_readlane(hi, lane);
            return __longlong_as_double((long long)(((uint64_t)h << 32) | l));
        };
        const double r0 = row(0), r1 = row(16), r2 = row(32), r3 = row(48);
        if (S == 64) v = (r0 + r1) + (r2 + r3);
        else v = (threadIdx.x & 32u) ? r2 + r3 : r0 + r1;
    }
    return v;
}

// The block covers the whole plane (B at least every extent of the map: the later layers of a
// network, or a block size like 64 on maps of 56 x 56 and below): H^L is the plane's mean, rows
// and columns play no part, and the plane is a flat run of 16-byte vectors.  One wavefront per
// 64 / S planes; the S lanes of a plane keep its vectors in registers (vector u in lane u mod S),
// sums and extremes are reductions over those lanes, the codes leave as one to eight bytes per
// vector.  LDS is not used.
// K: rounds the instance runs (3, 4, 6 or 13; the host picks lanes per plane and K so that a plane has at
// most K rounds of vectors and few of the K * S lane slots stay empty).  No round is tested at run time:
// a uniform test per round splits the code into blocks that each wait for every load (measured: 50 ->
// 40 us on 64 x 256 x 56 x 56); a round past the plane loads nothing (its offsets are out of range) and
// works on zeros that are masked.
template <typename T, int BITS, int K>
__global__ void __launch_bounds__(64) compress_one(OneArgs a) {
    constexpr uint32_t EPV = 16 / sizeof(T);
    constexpr uint32_t CBV = EPV * BITS / 8;
    constexpr bool HALF = EPV * BITS == 4;                // 1-bit codes of a 4-element vector: half a byte
    constexpr float Lf = float((1 << BITS) - 1);
    constexpr uint32_t kDrop = 0x80000000u;              // an offset past every buffer here: the access is dropped
    const uint32_t tid = threadIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, tid);
    const uint32_t sub = tid & (a.S - 1u), pl = tid >> a.S_log2;
    const uint32_t p0 = xcd_run_index(blockIdx.x, gridDim.x) * a.ppw;
    const uint32_t Gc = min(a.ppw, a.P - p0);
    const uint32_t p = p0 + pl;
    const bool live = pl < Gc;

    // the planes of a wavefront are contiguous: one bounds-checked buffer, no branch that depends on a
    // lane (a vector past its plane's end reads the neighbour's data or zero and is masked below)
    u32x4 q[K];
    {
        const T* src = static_cast<const T*>(pt.x) + (size_t)p0 * a.HW;
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(src), 0, (int)(Gc * a.HW * sizeof(T)), 0x00020000);
        const uint32_t off0 = live ? (pl * a.qv + sub) * 16u : kDrop;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            // a vector past the plane's end is not fetched (offset out of range: it reads as zero)
            const uint32_t u = sub + (uint32_t)k * a.S;
            q[k] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, u < a.qv ? off0 + (uint32_t)k * a.S * 16u : kDrop, 0, kLoadAux);
        }
    }
    // ---- Sec. 4.1 AveragePooling with one window: the mean of the plane
    double S = 0.0;
    float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const bool valid = sub + (uint32_t)k * a.S < a.qv;
        float f[EPV];
        unpack_vec<T>(q[k], f);
        double s4 = ((double)f[0] + (double)f[1]) + ((double)f[2] + (double)f[3]);
        float vmn = fminf(fminf(f[0], f[1]), fminf(f[2], f[3]));
        float vmx = fmaxf(fmaxf(f[0], f[1]), fmaxf(f[2], f[3]));
        if constexpr (EPV == 8) {
            s4 += ((double)f[4] + (double)f[5]) + ((double)f[6] + (double)f[7]);
            vmn = fminf(vmn, fminf(fminf(f[4], f[5]), fminf(f[6], f[7])));
            vmx = fmaxf(vmx, fmaxf(fmaxf(f[4], f[5]), fmaxf(f[6], f[7])));
        }
        S += valid ? s4 : 0.0;
        mn = fminf(mn, valid ? vmn : __builtin_inff());
        mx = fmaxf(mx, valid ? vmx : -__builtin_inff());
    }
    S = group_sum_any(a.S, S);
    const float lfc = lfc_round<T>(mean_of(S, a.HW), kC16<T>);
    // ---- extremes of the residual (x -> fl(x - m) is monotone), scale of Eq. (quantization), keys
    mn = mn - lfc;
    mx = mx - lfc;
    group_minmax(a.S, mn, mx);
    float delta, Delta, inv;
    plane_scale_any(mn, mx, Lf, kC16<T>, delta, Delta, inv);
    const float invs = inv * (float)(1u << (32 - BITS));
    const uint32_t k1 = mix32(p ^ pt.seed_a);
    const uint32_t k2 = mix32(k1 + pt.seed_c);
    uint8_t* cwave = reinterpret_cast<uint8_t*>(pt.codes) + (size_t)p0 * a.WPP * 4;
    if (live && sub == 0) {
        meta_store(pt.meta, p, delta, Delta, kC16<T>);
        lfc_store<T>(pt.lfc, (size_t)p, lfc, kC16<T>);
        uint8_t* cbase = cwave + (size_t)pl * a.WPP * 4;
        const uint32_t cbytes = HALF ? (a.qv + 1u) / 2u : a.qv * CBV;
        const uint32_t padb = a.WPP * 4 - cbytes;                     // pad bytes of the last word are zero
        for (uint32_t t = 0; t < padb; ++t) cbase[cbytes + t] = 0;
    }
    // ---- residual, Quant, packing
    const __amdgpu_buffer_rsrc_t crs = __builtin_amdgcn_make_buffer_rsrc(cwave, 0, (int)(Gc * a.WPP * 4u), 0x00020000);
    const uint32_t rscale = 1u << (16 - BITS);
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t u = sub + (uint32_t)k * a.S;
        const uint32_t co = live && u < a.qv ? pl * a.WPP * 4u + u * CBV : kDrop;
        float h[EPV];
        unpack_vec<T>(q[k], h);
#pragma unroll
        for (uint32_t e = 0; e < EPV; ++e) h[e] = h[e] - lfc;
        const uint32_t xw0 = k1 + (u * (EPV / 2)) * kWeyl;
        if constexpr (CBV <= 4) {
            uint32_t c = 0;
#pragma unroll
            for (int j = EPV / 2 - 1; j >= 0; --j)
                c = push_pair<BITS>(c, h[2 * j], h[2 * j + 1], delta, invs, xw0 + (uint32_t)j * kWeyl, k2, rscale);
            if constexpr (HALF) {
                // the even lane of a pair stores the byte of both vectors (a vector past the plane gives zeros)
                c = co != kDrop ? c : 0u;
                c |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)c, 0xB1, 0xf, 0xf, true) << 4;     // quad_perm [1,0,3,2]
                __builtin_amdgcn_raw_buffer_store_b8((uint8_t)c, crs, co != kDrop && (sub & 1u) == 0 ? pl * a.WPP * 4u + (u >> 1) : kDrop, 0, 0);
            } else if constexpr (CBV == 1) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)c, crs, co, 0, 0);
            else if constexpr (CBV == 2) __builtin_amdgcn_raw_buffer_store_b16((uint16_t)c, crs, co, 0, 0);
            else __builtin_amdgcn_raw_buffer_store_b32(c, crs, co, 0, 0);
        } else {
            uint32_t lo = 0, hi = 0;
            hi = push_pair<BITS>(hi, h[6], h[7], delta, invs, xw0 + 3u * kWeyl, k2, rscale);
            hi = push_pair<BITS>(hi, h[4], h[5], delta, invs, xw0 + 2u * kWeyl, k2, rscale);
            lo = push_pair<BITS>(lo, h[2], h[3], delta, invs, xw0 + kWeyl, k2, rscale);
            lo = push_pair<BITS>(lo, h[0], h[1], delta, invs, xw0, k2, rscale);
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            __builtin_amdgcn_raw_buffer_store_b64(u32x2{lo, hi}, crs, co, 0, 0);
        }
    }
}

// 1-D maps (Appendix D, AveragePooling1D: Minibatch x Channel x N, the maps of linear and
// transformer layers) whose block is a power-of-two number of 16-byte vectors (B = 4, 8, 16, 32, 64
// for fp32): laid out like compress_one, the `upb` vectors of a block sit in neighbouring lanes of
// one round, so a block's sum is a DPP reduction over those lanes and its LFC stays in a register.
// No LDS.  The planes of a wavefront are contiguous: their vectors are read through one bounds-checked
// buffer (a lane whose vector lies past its plane reads its neighbour's data or zero and is masked in
// the arithmetic), codes and H^L leave through bounds-checked buffer stores with the offset pushed out
// of range where nothing is to be written: no branch depends on a lane or on the round, loads and
// rounds are straight-line code that the compiler is free to interleave.  K as in compress_one.
constexpr int kLineUnits = 13;
// NG > 1: planes of at most R = K / NG rounds (a few hundred bytes each): a wavefront takes NG groups of
// 64 / S planes one after the other, all their loads issued first, so that it has K vectors per lane in
// flight like the instances for larger planes (two or three would not cover the memory latency).
template <typename T, int BITS, int K, int NG = 1>
__global__ void __launch_bounds__(64) compress_line(OneArgs a) {
    constexpr int R = K / NG;
    static_assert(R * NG == K, "whole groups");
    constexpr uint32_t EPV = 16 / sizeof(T);
    constexpr uint32_t CBV = EPV * BITS / 8;
    constexpr bool HALF = EPV * BITS == 4;                // 1-bit codes of a 4-element vector: half a byte
    constexpr float Lf = float((1 << BITS) - 1);
    constexpr uint32_t kDrop = 0x80000000u;              // an offset past every buffer here (and no wrap when a round's offset is added): the access is dropped
    const uint32_t tid = threadIdx.x;
    const CompPtrs pt = comp_ptrs(a.tab, a.rg, tid);
    const uint32_t sub = tid & (a.S - 1u);
    const uint32_t ppw = a.ppw * NG;                     // planes of the wavefront
    const uint32_t p0 = xcd_run_index(blockIdx.x, gridDim.x) * ppw;
    const uint32_t Gc = min(ppw, a.P - p0);

    u32x4 q[K];
    {
        const T* src = static_cast<const T*>(pt.x) + (size_t)p0 * a.HW;
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(src), 0, (int)(Gc * a.HW * sizeof(T)), 0x00020000);
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const uint32_t pl = (uint32_t)g * a.ppw + (tid >> a.S_log2);
            const uint32_t off0 = pl < Gc ? (pl * a.qv + sub) * 16u : kDrop;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                // no round is tested (see compress_one); a vector past the plane's end is not fetched
                const uint32_t u = sub + (uint32_t)r * a.S;
                q[g * R + r] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, u < a.qv ? off0 + (uint32_t)r * a.S * 16u : kDrop, 0, kLoadAux);
            }
        }
    }
    // every block but the plane's last has upb vectors: their reciprocals are taken once, not per round
    const uint32_t cnt_full = a.upb * EPV, cnt_last = (a.qv - (a.nb - 1u) * a.upb) * EPV;
    const double rcp_full = 1.0 / (double)cnt_full, rcp_last = 1.0 / (double)cnt_last;
    uint8_t* cwave = reinterpret_cast<uint8_t*>(pt.codes) + (size_t)p0 * a.WPP * 4;
    const __amdgpu_buffer_rsrc_t crs = __builtin_amdgcn_make_buffer_rsrc(cwave, 0, (int)(Gc * a.WPP * 4u), 0x00020000);
    constexpr uint32_t LB = (sizeof(T) == 2 || kC16<T>) ? 2u : 4u;          // bytes of a cached H^L value
    const __amdgpu_buffer_rsrc_t lrs = __builtin_amdgcn_make_buffer_rsrc(
        static_cast<uint8_t*>(pt.lfc) + (size_t)p0 * a.nb * LB, 0, (int)(Gc * a.nb * LB), 0x00020000);
    const uint32_t rscale = 1u << (16 - BITS);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
    const uint32_t pl = (uint32_t)g * a.ppw + (tid >> a.S_log2);
    const uint32_t p = p0 + pl;
    const bool live = pl < Gc;
    // ---- AveragePooling1D: block sums over the lanes of a block, residual extremes of the plane
    float lfcv[R];
    float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const uint32_t u = sub + (uint32_t)k * a.S;
        const bool valid = u < a.qv;
        float f[EPV];
        unpack_vec<T>(q[g * R + k], f);
        double s4 = ((double)f[0] + (double)f[1]) + ((double)f[2] + (double)f[3]);
        if constexpr (EPV == 8) s4 += ((double)f[4] + (double)f[5]) + ((double)f[6] + (double)f[7]);
        s4 = valid ? s4 + 0.0 : 0.0;                  // a block of negative zeros sums to +0, as a sum from 0 does
        const double Sb = group_sum_any(a.upb, s4);
        const uint32_t ustart = u & ~(a.upb - 1u);
        const bool last = ustart + a.upb >= a.qv;                              // the last block may be short
        const float lfc = lfc_round<T>(mean_with_rcp(Sb, last ? cnt_last : cnt_full, last ? rcp_last : rcp_full), kC16<T>);
        lfcv[k] = lfc;
        float hmn = __builtin_inff(), hmx = -__builtin_inff();
#pragma unroll
        for (uint32_t e = 0; e < EPV; ++e) {
            const float h = f[e] - lfc;
            hmn = fminf(hmn, h);
            hmx = fmaxf(hmx, h);
        }
        mn = fminf(mn, valid ? hmn : __builtin_inff());
        mx = fmaxf(mx, valid ? hmx : -__builtin_inff());
    }
    group_minmax(a.S, mn, mx);
    float delta, Delta, inv;
    plane_scale_any(mn, mx, Lf, kC16<T>, delta, Delta, inv);
    const float invs = inv * (float)(1u << (32 - BITS));
    const uint32_t k1 = mix32(p ^ pt.seed_a);
    const uint32_t k2 = mix32(k1 + pt.seed_c);
    if (live && sub == 0) {
        meta_store(pt.meta, p, delta, Delta, kC16<T>);
        uint8_t* cbase = cwave + (size_t)pl * a.WPP * 4;
        const uint32_t cbytes = HALF ? (a.qv + 1u) / 2u : a.qv * CBV;
        const uint32_t padb = a.WPP * 4 - cbytes;                     // pad bytes of the last word are zero
        for (uint32_t t = 0; t < padb; ++t) cbase[cbytes + t] = 0;
    }
    // ---- residual, Quant, packing
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const uint32_t u = sub + (uint32_t)k * a.S;
        const bool wr = live && u < a.qv;
        {
            // H^L of the block whose first vector this is
            const uint32_t lo = wr && (u & (a.upb - 1u)) == 0 ? (pl * a.nb + (u >> a.upb_log2)) * LB : kDrop;
            if constexpr (LB == 2) __builtin_amdgcn_raw_buffer_store_b16((uint16_t)float_to_bf16_bits(lfcv[k]), lrs, lo, 0, 0);
            else __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(lfcv[k]), lrs, lo, 0, 0);
        }
        float h[EPV];
        unpack_vec<T>(q[g * R + k], h);
#pragma unroll
        for (uint32_t e = 0; e < EPV; ++e) h[e] = h[e] - lfcv[k];
        const uint32_t xw0 = k1 + (u * (EPV / 2)) * kWeyl;
        const uint32_t co = wr ? pl * a.WPP * 4u + u * CBV : kDrop;
        if constexpr (CBV <= 4) {
            uint32_t c = 0;
#pragma unroll
            for (int j = EPV / 2 - 1; j >= 0; --j)
                c = push_pair<BITS>(c, h[2 * j], h[2 * j + 1], delta, invs, xw0 + (uint32_t)j * kWeyl, k2, rscale);
            if constexpr (HALF) {
                c = wr ? c : 0u;
                c |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)c, 0xB1, 0xf, 0xf, true) << 4;     // quad_perm [1,0,3,2]
                __builtin_amdgcn_raw_buffer_store_b8((uint8_t)c, crs, wr && (sub & 1u) == 0 ? pl * a.WPP * 4u + (u >> 1) : kDrop, 0, 0);
            } else if constexpr (CBV == 1) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)c, crs, co, 0, 0);
            else if constexpr (CBV == 2) __builtin_amdgcn_raw_buffer_store_b16((uint16_t)c, crs, co, 0, 0);
            else __builtin_amdgcn_raw_buffer_store_b32(c, crs, co, 0, 0);
        } else {
            uint32_t lo = 0, hi = 0;
            hi = push_pair<BITS>(hi, h[6], h[7], delta, invs, xw0 + 3u * kWeyl, k2, rscale);
            hi = push_pair<BITS>(hi, h[4], h[5], delta, invs, xw0 + 2u * kWeyl, k2, rscale);
            lo = push_pair<BITS>(lo, h[2], h[3], delta, invs, xw0 + kWeyl, k2, rscale);
            lo = push_pair<BITS>(lo, h[0], h[1], delta, invs, xw0, k2, rscale);
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            __builtin_amdgcn_raw_buffer_store_b64(u32x2{lo, hi}, crs, co, 0, 0);
        }
    }
    }
}
