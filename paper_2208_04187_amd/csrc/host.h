// Part of division.hip (included inside its unnamed namespace, in this order): packed layout, launch plans, launches, the implementation behind the C ABI.

// ------------------------------------------------------------------ host side

struct Layout {
    uint64_t P, HW, LD, LH, LW, nb, WPP;      // HW = elements per plane (D*H*W), nb = LD*LH*LW blocks
    size_t codes_off, codes_bytes, meta_off, meta_bytes, lfc_off, lfc_bytes, total;
};

size_t align16(size_t v) { return (v + 15u) & ~(size_t)15u; }

// A plane is D x H x W elements (Appendix D: 3-D maps); D = 1 for the 2-D maps of Sec. 4.1.
int make_layout(int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int B, int b, int dt, Layout* L) {
    if (N <= 0 || C <= 0 || D <= 0 || H <= 0 || W <= 0 || B < 1 || (b != 1 && b != 2 && b != 4 && b != 8)) return DIVISION_EINVAL;
    if (dt != DIVISION_F32 && dt != DIVISION_BF16 && dt != DIVISION_F32_C16) return DIVISION_EINVAL;
    const uint64_t lim31 = 0x7fffffffull;
    if ((uint64_t)N > lim31 || (uint64_t)C > lim31 || (uint64_t)D > lim31 || (uint64_t)H > lim31 || (uint64_t)W > lim31)
        return DIVISION_ERANGE;
    L->P = (uint64_t)N * (uint64_t)C;
    if ((uint64_t)D * (uint64_t)H > lim31) return DIVISION_ERANGE;
    L->HW = (uint64_t)D * (uint64_t)H * (uint64_t)W;
    if (L->P > lim31 || L->HW > lim31 || L->P * L->HW > (1ull << 40)) return DIVISION_ERANGE;
    L->LD = ((uint64_t)D + B - 1) / B;
    L->LH = ((uint64_t)H + B - 1) / B;
    L->LW = ((uint64_t)W + B - 1) / B;
    L->nb = L->LD * L->LH * L->LW;
    const uint64_t cpw = 32 / b;
    L->WPP = (L->HW + cpw - 1) / cpw;
    const size_t lfc_es = dt == DIVISION_F32 ? 4 : 2;          // H^L: element type of x, bfloat16 in the cached-as-bf16 mode
    const size_t meta_es = dt == DIVISION_F32_C16 ? 4 : 8;      // (delta, Delta) per plane
    L->codes_off = 0;
    L->codes_bytes = (size_t)(4 * L->P * L->WPP);
    L->meta_off = align16(L->codes_bytes);
    L->meta_bytes = (size_t)(meta_es * L->P);
    L->lfc_off = align16(L->meta_off + L->meta_bytes);
    L->lfc_bytes = (size_t)(lfc_es * L->P * L->nb);
    L->total = align16(L->lfc_off + L->lfc_bytes);
    return DIVISION_OK;
}

uint64_t gcd_u64(uint64_t a, uint64_t b) { while (b) { uint64_t t = a % b; a = b; b = t; } return a; }

// fdiv(n, d) is exact while n*d < 2^32
bool fastdiv_ok(uint64_t n_max, uint64_t d) { return n_max * d < (1ull << 32); }

Regions make_regions(const Layout& L) {
    Regions rg;
    rg.meta_off = L.meta_off;
    rg.lfc_off = L.lfc_off;
    rg.pad_off[0] = L.codes_off + L.codes_bytes; rg.pad_len[0] = (uint32_t)(L.meta_off - rg.pad_off[0]);
    rg.pad_off[1] = L.meta_off + L.meta_bytes;   rg.pad_len[1] = (uint32_t)(L.lfc_off - rg.pad_off[1]);
    rg.pad_off[2] = L.lfc_off + L.lfc_bytes;     rg.pad_len[2] = (uint32_t)(L.total - rg.pad_off[2]);
    return rg;
}

// Preferred LDS footprint of one wavefront's chunk in compress_wave (small chunks = many wavefronts
// per CU; 8.7 KB measured best over the ResNet-50 set); a single plane of up to kWavePlaneMax bytes is
// taken whatever the preference says.
constexpr uint32_t kWaveChunkLds = 8704u;
constexpr uint32_t kWavePlaneMax = 17u << 10;

// Compute units of the current device (sizes the grids of the kernels that walk over planes).  Asked
// once per device and kept: a table of constants of the machine, not state of a call.
int num_cus() {
    constexpr int kMaxDev = 64;
    static std::atomic<int> cus[kMaxDev];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return 256;
    int v = cus[dev].load(std::memory_order_relaxed);
    if (v > 0) return v;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    cus[dev].store(v, std::memory_order_relaxed);
    return v;
}

// dynamic LDS above the default limit needs a one-time opt-in per kernel
template <typename Args>
hipError_t allow_large_lds(void (*kern)(Args), size_t lds) {
    if (lds <= 48u * 1024u) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax);
}

template <typename T, int BITS, int B>
hipError_t launch_tile_vec(int vec, const TileArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    void (*kern)(TileArgs) = vec == 4 ? compress_tile<T, BITS, B, 4, 256>
                           : vec == 2 ? compress_tile<T, BITS, B, 2, 256>
                                      : compress_tile<T, BITS, B, 1, 256>;
    hipError_t e = allow_large_lds(kern, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, a);
    return hipGetLastError();
}

template <typename T, int BITS>
hipError_t launch_tile(int B, int vec, const TileArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    return B == 8 ? launch_tile_vec<T, BITS, 8>(vec, a, grid, lds, st)
                  : launch_tile_vec<T, BITS, 4>(vec, a, grid, lds, st);
}

template <typename T, int BITS, int B>
hipError_t launch_wave_vec(int vec, const WaveArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    void (*kern)(WaveArgs) = vec == 4 ? compress_wave<T, BITS, B, 4>
                           : vec == 2 ? compress_wave<T, BITS, B, 2>
                                      : compress_wave<T, BITS, B, 1>;
    hipLaunchKernelGGL(kern, grid, dim3(64), lds, st, a);
    return hipGetLastError();
}

template <typename T, int BITS>
hipError_t launch_wave(int B, int vec, const WaveArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    return B == 8 ? launch_wave_vec<T, BITS, 8>(vec, a, grid, lds, st)
                  : launch_wave_vec<T, BITS, 4>(vec, a, grid, lds, st);
}

// Fills the plane-in-registers compress plan; false when the shape is not covered.
bool plan_regs(const Layout& L, int64_t D, int64_t H, int64_t W, int B, size_t es, const void* x,
               RegsArgs* a, uint32_t* grid, size_t* lds, int* nw_out) {
    if (B % 4 != 0 || W % 4 != 0) return false;
    if (D > 1 && B != 8) return false;            // 3-D maps: the B = 8 instances only
    if (((uintptr_t)x % (4 * es)) != 0) return false;
    const uint64_t q4 = L.HW / 4;
    const bool any_b = B != 4 && B != 8;          // the instance that reads B from its arguments
    int nw;
    if (any_b) {
        // a lane adds the unit sums of its block one after the other: at most 64 of them (blocks of
        // up to 16 x 16, longer ones on maps of few rows), several blocks per plane
        const uint64_t brows = (uint64_t)B < (uint64_t)H ? (uint64_t)B : (uint64_t)H;
        if (brows * ((uint64_t)B / 4) > 64 || L.nb == 1) return false;
        if (q4 >= 512 && q4 <= (uint64_t)kRegUnits * 64) nw = 1;
        else if (q4 > (uint64_t)kRegUnits * 64 && q4 <= (uint64_t)kRegUnits * 256) nw = 4;
        else return false;
    } else if (q4 >= 512 && q4 <= (uint64_t)kRegUnits * 64) nw = 1;
    else if (q4 >= (D > 1 ? (uint64_t)kRegUnits * 64 + 1 : 2048) && q4 <= (uint64_t)kRegUnits * 256) nw = 4;
    else if (q4 > (uint64_t)kRegUnits * 256 && q4 <= (uint64_t)kRegUnits * 1024) nw = 16;   // image-sized planes: 1024 threads, one workgroup per CU
    else return false;
    const uint64_t nt = 64ull * nw, w4 = (uint64_t)W / 4;
    if (!fastdiv_ok(kRegUnits * nt, w4) || !fastdiv_ok(L.nb + nt, L.LW) || L.HW * es >= (1ull << 31)) return false;
    if (!fastdiv_ok((uint64_t)H, (uint64_t)B) || !fastdiv_ok(w4, (uint64_t)B / 4)) return false;
    if (!fastdiv_ok((uint64_t)D * (uint64_t)H, (uint64_t)H) || !fastdiv_ok(L.nb + nt, L.LH * L.LW)) return false;
    a->D = (uint32_t)D;
    a->d_H = make_fastdiv((uint32_t)H);
    a->d_slice = make_fastdiv((uint32_t)(L.LH * L.LW));
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW;
    a->LH = (uint32_t)L.LH; a->LW = (uint32_t)L.LW; a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP;
    a->q4 = (uint32_t)q4; a->w4 = (uint32_t)w4;
    a->ppw = 1;      // one plane per workgroup measured best (more workgroups, better balance)
    a->B = (uint32_t)B;
    a->d_w4 = make_fastdiv((uint32_t)w4);
    a->d_LW = make_fastdiv((uint32_t)L.LW);
    a->d_B = make_fastdiv((uint32_t)B);
    a->d_upb = make_fastdiv((uint32_t)B / 4);
    *lds = 8ull * kRegUnits * nt + 4ull * ((L.nb + 1 + 3) & ~3ull) + 8ull * nw + 16 + (D > 1 ? 8ull * L.nb * B + 16 : 0);
    *grid = (uint32_t)((L.P + a->ppw - 1) / a->ppw);
    *nw_out = nw;
    return *lds <= (nw == 16 ? (size_t)kLdsMax : (size_t)(60u * 1024u));
}

template <typename T, int BITS>
hipError_t launch_regs(int B, int nw, const RegsArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    void (*kern)(RegsArgs);
    if (a.D > 1) kern = nw == 1 ? compress_regs_3d<T, BITS, 8, 1> : nw == 4 ? compress_regs_3d<T, BITS, 8, 4> : compress_regs_3d<T, BITS, 8, 16>;
    else if (nw == 1) kern = B == 8 ? compress_regs<T, BITS, 8, 1> : B == 4 ? compress_regs<T, BITS, 4, 1> : compress_regs<T, BITS, 0, 1>;
    else if (nw == 4) kern = B == 8 ? compress_regs<T, BITS, 8, 4> : B == 4 ? compress_regs<T, BITS, 4, 4> : compress_regs<T, BITS, 0, 4>;
    else kern = B == 8 ? compress_regs<T, BITS, 8, 16> : compress_regs<T, BITS, 4, 16>;
    const hipError_t e = allow_large_lds(kern, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, dim3(64 * nw), lds, st, a);
    return hipGetLastError();
}

// Fills the plan of the register kernel for any width; false when the shape is not covered: 2-D maps
// of at most 8 x 1024 units that fit LDS beside their row sums (up to about 163 x 163 elements).
constexpr uint64_t kUnitsMin = 128;       // units per plane from which a plane gets a whole wavefront or more
constexpr uint64_t kUnitsSubMin = 64;     // units per plane from which the instance with 16 or 32 lanes per plane is used
                                          // (17 x 17: 1.7 -> 2.3 TB/s; 13 x 13 and 15 x 15 are no faster than in compress_wave)
bool plan_units(const Layout& L, int64_t D, int64_t H, int64_t W, int B, size_t es, const void* x,
                UnitsArgs* a, uint32_t* grid, size_t* lds, int* nw_out) {
    if (H == 1 || ((uintptr_t)x % 4) != 0) return false;
    // small planes of even width under B = 4 and 8 are the wavefront kernel's (pairs of elements per
    // lane): measured faster there
    if (D == 1 && (B == 4 || B == 8) && W % 2 == 0 && 4ull * L.HW + 16ull <= kWavePlaneMax) return false;
    const uint64_t q4 = (L.HW + 3) / 4;
    if (L.nb > 16383 || B > 4095) return false;              // LFC offsets are kept as 16-bit byte offsets
    // 2-D planes below 2048 elements with whole-vector rows: compress_rows keeps their vectors in registers
    // and is the faster one (28 x 28 under B = 12: 43 us against 49)
    if (D == 1 && W % 4 == 0 && q4 < 512) return false;
    const uint64_t Bz = D > 1 ? (uint64_t)B : 1;              // depth of a block
    const uint64_t nitem = L.nb * Bz * (uint64_t)B;
    int nw = 1;
    uint64_t S = 64;                                          // lanes per plane
    if (q4 < kUnitsMin) {
        // small planes: 8, 16 or 32 lanes each, several planes per wavefront
        if (q4 < kUnitsSubMin) return false;
        S = 8;
        while (S < 64 && (q4 > (uint64_t)kUnitsK * S || nitem > (uint64_t)kUnitsK * S)) S *= 2;
        nw = S < 64 ? 0 : 1;
    }
    if (nw) {
        while (nw < 16 && (q4 > (uint64_t)kUnitsK * 64 * nw || nitem > (uint64_t)kUnitsK * 64 * nw)) nw *= 2;
        S = 64ull * nw;
    }
    if (q4 > (uint64_t)kUnitsK * S || nitem > (uint64_t)kUnitsK * S) return false;       // 8 units and 8 row segments per lane
    const uint64_t q4p = (q4 + S - 1) / S * S;
    if (!fastdiv_ok(4ull * kUnitsK * S + 4, (uint64_t)W) || !fastdiv_ok(4ull * kUnitsK * S + 4, (uint64_t)B) ||
        !fastdiv_ok(nitem + S, (uint64_t)B * Bz) || !fastdiv_ok(L.nb + S, L.LH * L.LW) ||
        !fastdiv_ok(4ull * kUnitsK * S + 4, (uint64_t)H))
        return false;
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW;
    a->LW = (uint32_t)L.LW; a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP; a->B = (uint32_t)B;
    a->D = (uint32_t)D; a->LH = (uint32_t)L.LH; a->Bz = (uint32_t)Bz;
    a->d_H = make_fastdiv((uint32_t)H);
    a->d_BBz = make_fastdiv((uint32_t)(Bz * (uint64_t)B));
    a->d_slice = make_fastdiv((uint32_t)(L.LH * L.LW));
    a->q4 = (uint32_t)q4; a->q4p = (uint32_t)q4p; a->nitem = (uint32_t)nitem;
    a->S = (uint32_t)S;
    a->S_log2 = 0;
    while ((1ull << a->S_log2) < S) ++a->S_log2;
    a->d_W = make_fastdiv((uint32_t)W);
    a->d_B = make_fastdiv((uint32_t)B);
    a->d_LW = make_fastdiv((uint32_t)L.LW);
    const uint64_t G = nw ? 1 : 64 / S;                       // planes per round
    const uint64_t reg = (16ull * q4p + 8ull * nitem + 4ull * ((L.nb + 1 + 3) & ~3ull) + 8ull * (nw ? nw : 1) + 16 + 15) & ~15ull;
    a->reg_bytes = (uint32_t)reg;
    a->nrounds = (uint32_t)((L.P + G - 1) / G);
    *lds = reg * G;
    if (*lds > (size_t)kLdsMax) return false;
    // as many workgroups as the machine holds at once (LDS, and 16 wavefronts per CU), each taking every
    // grid-th round of planes
    const uint64_t wpg = nw ? (uint64_t)nw : 1;               // wavefronts per workgroup
    uint64_t per_cu = (160ull << 10) / *lds;
    if (per_cu > 16ull / wpg) per_cu = 16ull / wpg;
    if (per_cu < 1) per_cu = 1;
    uint64_t g = (uint64_t)num_cus() * per_cu;
    g += g & 1;            // even: with 2-byte elements the planes of a workgroup then start alike within a dword
    *grid = (uint32_t)(g < a->nrounds ? g : a->nrounds);
    *nw_out = nw;
    return true;
}

template <typename T, int BITS>
hipError_t launch_units(int nw, const UnitsArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    void (*kern)(UnitsArgs) = nw == 0 ? compress_units<T, BITS, 0> : nw == 1 ? compress_units<T, BITS, 1>
                            : nw == 2 ? compress_units<T, BITS, 2> : nw == 4 ? compress_units<T, BITS, 4>
                                                                             : compress_units<T, BITS, 8>;
    // 1-bit codes have no instance of sixteen wavefronts (its lane pairing does not fit the 128 registers
    // a lane of 1024 threads has): the planner sends those planes elsewhere
    if constexpr (BITS != 1) { if (nw == 16) kern = compress_units<T, BITS, 16>; }
    else if (nw == 16) return hipErrorInvalidValue;
    const hipError_t e = allow_large_lds(kern, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, dim3(nw ? 64 * nw : 64), lds, st, a);
    return hipGetLastError();
}

// one-block planes with an odd element count: the shapes the lane-per-plane kernels take
bool lane_shape(const Layout& L) { return L.nb == 1 && (L.HW & 1) == 1 && L.HW <= 64; }

// Fills the lane-per-plane compress plan; false when the shape is not covered.
bool plan_lane(const Layout& L, size_t es, const void* x, LaneArgs* a, uint32_t* grid, size_t* lds) {
    if (!lane_shape(L)) return false;
    a->P = (uint32_t)L.P; a->HW = (uint32_t)L.HW; a->WPP = (uint32_t)L.WPP;
    a->nrounds = (uint32_t)((L.P + 63) / 64);
    a->vec_load = ((uintptr_t)x % 16) == 0;
    uint32_t rpw = 2;
    while (rpw > 1 && a->nrounds / rpw < 32u * (uint32_t)num_cus()) --rpw;
    a->rpw = rpw;
    *lds = 4ull * (64ull * L.HW + 4) + 16 * (es == 2 ? 1 : 0);
    *grid = (a->nrounds + rpw - 1) / rpw;
    return true;
}

// Fills the items-from-global compress plan (small planes); false when the shape is not covered.
bool plan_items(const Layout& L, int64_t H, int64_t W, int B, size_t es, const void* x,
                ItemsArgs* a, uint32_t* grid, size_t* lds, int* vec_out) {
    if ((B != 4 && B != 8) || W % 2 != 0) return false;
    const int vec = W % 4 == 0 ? 4 : 2;
    if (((uintptr_t)x % (vec * es)) != 0) return false;
    const uint64_t ipb = (uint64_t)B / vec;
    const uint64_t slots = (uint64_t)W / vec;
    const uint64_t ipr = (slots + ipb - 1) / ipb * ipb;
    const uint64_t ipp = L.LH * ipr;
    if (ipp > 64) return false;
    uint64_t S = 1, lg = 0;
    while (S < ipp) { S *= 2; ++lg; }
    const uint64_t ppr = 64 / S;
    if (ppr * L.WPP * 4 > 32u * 1024u || ppr * L.HW * es >= (1ull << 31)) return false;
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW;
    a->LW = (uint32_t)L.LW; a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP;
    a->ipr = (uint32_t)ipr; a->ipp = (uint32_t)ipp; a->S = (uint32_t)S; a->S_log2 = (uint32_t)lg;
    a->ppr = (uint32_t)ppr;
    a->nrounds = (uint32_t)((L.P + ppr - 1) / ppr);
    a->d_ipr = make_fastdiv((uint32_t)ipr);
    uint32_t rpw = 2;
    while (rpw > 1 && a->nrounds / rpw < 32u * (uint32_t)num_cus()) --rpw;
    a->rpw = rpw;
    *lds = 4ull * ppr * L.WPP + 16;
    *grid = (a->nrounds + rpw - 1) / rpw;
    *vec_out = vec;
    return true;
}

// Fills the strip kernel's plan: 2-D maps of width 28 or 32 (at most 32 rows) or 14 or 16 (an even number
// of rows, at most 16), 16-byte aligned, under a block size the kernel has an instance for: 8 on 28 / 14
// (the items kernel keeps 32 / 16 under B = 8), 12, 16 (where a plane has several blocks) and 18 of the
// block-size sweep; false when the shape is not covered.  *width = 100 * W + B names the instance.
bool plan_strip(const Layout& L, int64_t H, int64_t W, int B, size_t es, const void* x,
                StripArgs* a, uint32_t* grid, size_t* lds, int* width) {
    if (((uintptr_t)x % (4 * es)) != 0) return false;
    uint64_t G, upl;
    if ((W == 28 || W == 32) && H <= 32) { G = 2; upl = W == 28 ? 7 : 8; }
    else if ((W == 14 || W == 16) && H % 2 == 0 && H <= 16) { G = 8; upl = W == 14 ? 7 : 8; }
    else return false;
    const bool wide = W == 28 || W == 32;
    bool have;
    switch (B) {
        case 4: have = W == 32 || W == 16; break;
        case 8: have = true; break;
        case 12: have = true; break;
        case 16: have = wide; break;
        case 18: have = wide; break;
        default: have = false;
    }
    if (!have) return false;
    const uint64_t nseg = ((uint64_t)W + B - 1) / B;
    const bool dpp = B == 4 || B == 8;
    if (L.LW != nseg || (!dpp && G * L.nb > 64)) return false;
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->HW = (uint32_t)L.HW; a->WPP = (uint32_t)L.WPP; a->nb = (uint32_t)L.nb;
    a->nrounds = (uint32_t)((L.P + G - 1) / G);
    *grid = a->nrounds;
    // the round; for the block sizes whose block rows are no DPP group also the strips' shares and the round's H^L
    *lds = dpp ? 4ull * G * L.HW + 16 : upl * 1024 + 64 * nseg * 8 + 256 + 16;
    *width = (int)(100 * W + B);
    return true;
}

template <typename T, int BITS>
hipError_t launch_strip(int width, const StripArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    void (*kern)(StripArgs);
    switch (width) {
        case 2808: kern = compress_strip<T, BITS, 28, 8>; break;
        case 1408: kern = compress_strip<T, BITS, 14, 8>; break;
        case 3208: kern = compress_strip<T, BITS, 32, 8>; break;
        case 1608: kern = compress_strip<T, BITS, 16, 8>; break;
        case 3204: kern = compress_strip<T, BITS, 32, 4>; break;
        case 1604: kern = compress_strip<T, BITS, 16, 4>; break;
        case 2812: kern = compress_strip<T, BITS, 28, 12>; break;
        case 2816: kern = compress_strip<T, BITS, 28, 16>; break;
        case 2818: kern = compress_strip<T, BITS, 28, 18>; break;
        case 3212: kern = compress_strip<T, BITS, 32, 12>; break;
        case 3216: kern = compress_strip<T, BITS, 32, 16>; break;
        case 3218: kern = compress_strip<T, BITS, 32, 18>; break;
        case 1412: kern = compress_strip<T, BITS, 14, 12>; break;
        case 1612: kern = compress_strip<T, BITS, 16, 12>; break;
        default: return hipErrorInvalidValue;
    }
    hipLaunchKernelGGL(kern, grid, dim3(64), lds, st, a);
    return hipGetLastError();
}

// Fills the plan of the row-per-lane strip kernel: 2-D maps of an odd width it has an instance for (13, 15,
// 17, 27, 35, 55) with at most 16 (13, 15), 32 (17, 27) or 64 rows, under B = 8 or 4, 16-byte aligned.
// *width = 100 * W + B names the instance.
bool plan_rowstrip(const Layout& L, int64_t H, int64_t W, int B, size_t es, const void* x,
                   StripArgs* a, uint32_t* grid, size_t* lds, int* width) {
    if (((uintptr_t)x % 16) != 0) return false;
    uint64_t S;
    if (W == 13 || W == 15) S = 16;
    else if (W == 17 || W == 27) S = 32;
    else if (W == 35 || W == 55) S = 64;
    else return false;
    if ((B != 8 && B != 4) || H < 2 || (uint64_t)H > S) return false;
    const uint64_t G = 64 / S;
    if (L.LW != ((uint64_t)W + B - 1) / B) return false;
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->HW = (uint32_t)L.HW; a->WPP = (uint32_t)L.WPP; a->nb = (uint32_t)L.nb;
    a->nrounds = (uint32_t)((L.P + G - 1) / G);
    *grid = a->nrounds;
    *lds = 16ull * ((G * L.HW + 3) / 4) + 16;          // the round in whole 16-byte units
    *width = (int)(100 * W + B);
    return true;
}

template <typename T, int BITS>
hipError_t launch_rowstrip(int width, const StripArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    void (*kern)(StripArgs);
    switch (width) {
        case 1308: kern = compress_rowstrip<T, BITS, 13, 8>; break;
        case 1304: kern = compress_rowstrip<T, BITS, 13, 4>; break;
        case 1508: kern = compress_rowstrip<T, BITS, 15, 8>; break;
        case 1504: kern = compress_rowstrip<T, BITS, 15, 4>; break;
        case 1708: kern = compress_rowstrip<T, BITS, 17, 8>; break;
        case 1704: kern = compress_rowstrip<T, BITS, 17, 4>; break;
        case 2708: kern = compress_rowstrip<T, BITS, 27, 8>; break;
        case 2704: kern = compress_rowstrip<T, BITS, 27, 4>; break;
        case 3508: kern = compress_rowstrip<T, BITS, 35, 8>; break;
        case 3504: kern = compress_rowstrip<T, BITS, 35, 4>; break;
        case 5508: kern = compress_rowstrip<T, BITS, 55, 8>; break;
        case 5504: kern = compress_rowstrip<T, BITS, 55, 4>; break;
        default: return hipErrorInvalidValue;
    }
    hipLaunchKernelGGL(kern, grid, dim3(64), lds, st, a);
    return hipGetLastError();
}

// The Relu + compress instance of the strip kernel; a round's mask bits must be whole words.
bool plan_relu_strip(const Layout& L, int64_t H, int64_t W, int B, size_t es, const void* xy,
                     StripArgs* a, uint32_t* grid, size_t* lds, int* width) {
    // the instances whose block sums are DPP reductions: B = 8 on every strip width, B = 4 on 32 / 16
    if ((B != 8 && B != 4) || !plan_strip(L, H, W, B, es, xy, a, grid, lds, width)) return false;
    const uint64_t G = (W == 28 || W == 32) ? 2 : 8;
    return (G * L.HW) % 32 == 0;
}

template <typename T, int BITS>
hipError_t launch_relu_strip(int width, const StripArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    void (*kern)(StripArgs);
    switch (width) {
        case 2808: kern = relu_compress_strip<T, BITS, 28, 8>; break;
        case 1408: kern = relu_compress_strip<T, BITS, 14, 8>; break;
        case 3208: kern = relu_compress_strip<T, BITS, 32, 8>; break;
        case 1608: kern = relu_compress_strip<T, BITS, 16, 8>; break;
        case 3204: kern = relu_compress_strip<T, BITS, 32, 4>; break;
        case 1604: kern = relu_compress_strip<T, BITS, 16, 4>; break;
        default: return hipErrorInvalidValue;
    }
    hipLaunchKernelGGL(kern, grid, dim3(64), lds, st, a);
    return hipGetLastError();
}

template <typename T, int BITS>
hipError_t launch_items(int B, int vec, const ItemsArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    void (*kern)(ItemsArgs);
    if (a.H == 1) {
        if (B == 8) kern = vec == 4 ? compress_items<T, BITS, 8, 4, 1> : compress_items<T, BITS, 8, 2, 1>;
        else kern = vec == 4 ? compress_items<T, BITS, 4, 4, 1> : compress_items<T, BITS, 4, 2, 1>;
    } else {
        if (B == 8) kern = vec == 4 ? compress_items<T, BITS, 8, 4, 8> : compress_items<T, BITS, 8, 2, 8>;
        else kern = vec == 4 ? compress_items<T, BITS, 4, 4, 4> : compress_items<T, BITS, 4, 2, 4>;
    }
    hipLaunchKernelGGL(kern, grid, dim3(64), lds, st, a);
    return hipGetLastError();
}

// The Relu + compress instance of the items kernel (2-D maps, items of B rows).
template <typename T, int BITS>
hipError_t launch_relu_items(int B, int vec, const ItemsArgs& a, dim3 grid, size_t lds, hipStream_t st) {
    void (*kern)(ItemsArgs);
    if (B == 8) kern = vec == 4 ? relu_compress_items<T, BITS, 8, 4> : relu_compress_items<T, BITS, 8, 2>;
    else kern = vec == 4 ? relu_compress_items<T, BITS, 4, 4> : relu_compress_items<T, BITS, 4, 2>;
    hipLaunchKernelGGL(kern, grid, dim3(64), lds, st, a);
    return hipGetLastError();
}

// Plan of the fused Relu + compress call on the shapes of the items kernel: the rounds a workgroup
// handles are rounded up until its mask bits are whole words.  False when the shape is not covered.
bool plan_relu_items(const Layout& L, int64_t H, int64_t W, int B, size_t es, const void* xy,
                     ItemsArgs* a, uint32_t* grid, size_t* lds, int* vec_out) {
    if (H == 1 || !plan_items(L, H, W, B, es, xy, a, grid, lds, vec_out)) return false;
    uint32_t m = 1;
    while (((uint64_t)m * a->ppr * L.HW) % 32 != 0) ++m;              // at most 16: H*W is even here
    a->rpw = (a->rpw + m - 1) / m * m;
    const uint64_t mbits = (uint64_t)a->rpw * a->ppr * L.HW;
    *lds = 4ull * (((uint64_t)a->ppr * L.WPP + 3) & ~3ull) + mbits / 8 + 16;
    *grid = (a->nrounds + a->rpw - 1) / a->rpw;
    return *lds <= 60u * 1024u;
}

// Fills the one-wavefront compress plan; false when the shape is not covered.
bool plan_wave(const Layout& L, int64_t H, int64_t W, int B, int b, size_t es, const void* x,
               WaveArgs* a, uint32_t* grid, size_t* lds, int* vec_out) {
    if (B != 4 && B != 8) return false;
    const uint64_t per_plane = 4ull * L.HW + 16ull;
    if (per_plane > kWavePlaneMax) return false;
    const int vec = (W % 4 == 0) ? 4 : (W % 2 == 0) ? 2 : 1;
    const uint32_t ipb = (uint32_t)B / (uint32_t)vec;
    const uint64_t slots = ((uint64_t)W + vec - 1) / vec;
    const uint64_t ipr = (slots + ipb - 1) / ipb * ipb;
    const uint64_t ipp = L.LH * ipr;
    uint64_t ippp = 1, lg = 0;
    if (ipp <= 64) { while (ippp < ipp) { ippp *= 2; ++lg; } }
    else ippp = (ipp + 63) / 64 * 64;
    uint64_t Gmax = kWaveChunkLds / per_plane;
    if (Gmax < 1) Gmax = 1;
    if (Gmax > L.P) Gmax = L.P;
    const uint64_t unit = 16 / gcd_u64(16, L.HW * es);
    uint32_t vec_load = ((uintptr_t)x % 16) == 0;
    if (vec_load && unit > 1 && Gmax < unit && Gmax < L.P) {
        if (unit * per_plane <= kWavePlaneMax) Gmax = unit; else vec_load = 0;
    }
    const uint64_t step = vec_load ? unit : 1;
    // pick the G that wastes the fewest lanes in partly filled rounds
    const uint64_t cpw = 32 / b, ppw = cpw / 2;
    const double c1 = 4.5 * B * vec, c3 = 8.5 * (double)cpw;
    uint64_t G = 0;
    double best = 0;
    for (uint64_t g = step; g <= Gmax; g += step) {
        const double r1 = ipp <= 64 ? (double)((g + 64 / ippp - 1) / (64 / ippp)) : (double)(g * (ippp / 64));
        const uint64_t nw = g * L.WPP, tw = nw % 64;
        const double r3 = (double)(nw / 64) + (tw == 0 ? 0.0 : tw * ppw <= 64 ? 0.25 : 1.0);
        const double per_elt = (r1 * c1 + r3 * c3 + 2.0) / (double)(g * L.HW);
        if (G == 0 || per_elt < best * 0.97) { G = g; best = per_elt; }
    }
    if (G == 0) G = Gmax;          // Gmax == P < unit: a single chunk, aligned at its start
    if (!fastdiv_ok(ippp, ipr) || !fastdiv_ok(G * L.WPP + 64, L.WPP)) return false;
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW;
    a->LH = (uint32_t)L.LH; a->LW = (uint32_t)L.LW; a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP;
    a->G = (uint32_t)G; a->ipr = (uint32_t)ipr; a->ipp = (uint32_t)ipp;
    a->ippp = (uint32_t)ippp; a->ippp_log2 = (uint32_t)lg;
    a->vec_load = vec_load;
    a->d_ipr = make_fastdiv((uint32_t)ipr);
    a->d_wpp = make_fastdiv((uint32_t)L.WPP);
    *lds = 16ull * G + 4ull * ((G * L.HW + 3) / 4 * 4) + 64;      // 16 floats of slack for ragged last words
    // the staging registers hold 16 x 64 vectors of 16 bytes
    if (vec_load && G * L.HW * es > 16ull * 1024ull) return false;
    *grid = (uint32_t)((L.P + G - 1) / G);
    *vec_out = vec;
    return true;
}

// Lanes per plane S (a power of two from min_log up) and rounds K of the instance (3, 4, 6 or 13) for
// planes of qv vectors: the pair that leaves the fewest of the K * S lane slots empty; among equals
// the one with more rounds (fewer, longer-lived lanes per plane measured better than many short ones).
bool pick_lanes_and_rounds(uint64_t qv, uint32_t min_log, uint32_t* S_out, uint32_t* log_out, uint32_t* K_out) {
    uint64_t best = 0;
    for (uint32_t lg = min_log; lg <= 6; ++lg) {
        const uint64_t S = 1ull << lg, R = (qv + S - 1) / S;
        if (R > 13) continue;
        const uint64_t K = R <= 3 ? 3 : R <= 4 ? 4 : R <= 6 ? 6 : 13;
        const uint64_t slots = K * S;
        if (best == 0 || slots < best || (slots == best && K > *K_out)) { best = slots; *S_out = (uint32_t)S; *log_out = lg; *K_out = (uint32_t)K; }
    }
    return best != 0;
}

// Fills the one-block plan: the block covers the plane, which is whole 16-byte vectors, at most
// kOneUnits per lane of a wavefront.
bool plan_one(const Layout& L, size_t es, const void* x, OneArgs* a, uint32_t* grid) {
    const uint64_t epv = 16 / es;
    if (L.nb != 1 || ((uintptr_t)x % 16) != 0 || L.HW % epv != 0) return false;
    const uint64_t qv = L.HW / epv;
    if (qv > (uint64_t)kOneUnits * 64) return false;
    // lanes per plane: a power of two from 4 up (a plane's lanes then read 64 contiguous bytes per round)
    uint32_t best_S = 0, best_log = 0, K = 0;
    if (!pick_lanes_and_rounds(qv, 2, &best_S, &best_log, &K)) return false;
    a->P = (uint32_t)L.P; a->HW = (uint32_t)L.HW; a->WPP = (uint32_t)L.WPP;
    a->qv = (uint32_t)qv;
    a->S = best_S; a->S_log2 = best_log;
    a->ppw = 64u / best_S;
    a->K = K;
    a->NG = 1;
    *grid = (uint32_t)((L.P + a->ppw - 1) / a->ppw);
    return true;
}

// single-block planes of whole vectors: compress_one's, ahead of the kernels for general shapes
bool one_shape(const Layout& L, size_t es, const void* x) {
    OneArgs tmp{};
    uint32_t g = 0;
    return plan_one(L, es, x, &tmp, &g);
}

// Fills the plan of compress_line: a 1-D map (one row) of whole 16-byte vectors, several blocks per
// plane, a block a power-of-two number of vectors, at most kOneUnits vectors per lane.
bool plan_line(const Layout& L, int64_t D, int64_t H, int B, size_t es, const void* x, OneArgs* a, uint32_t* grid) {
    const uint64_t epv = 16 / es;
    if (D != 1 || H != 1 || L.nb < 2 || ((uintptr_t)x % 16) != 0 || L.HW % epv != 0 || (uint64_t)B % epv != 0) return false;
    const uint64_t qv = L.HW / epv, upb = (uint64_t)B / epv;
    if ((upb & (upb - 1)) != 0 || upb > 64 || qv > (uint64_t)kLineUnits * 64) return false;
    uint32_t upb_log = 0;
    while ((1ull << upb_log) < upb) ++upb_log;
    // lanes per plane: a power of two that holds a block, at least 8 (a plane's lanes then read 128
    // contiguous bytes per round)
    uint32_t best_S = 0, best_log = 0, K = 0;
    if (!pick_lanes_and_rounds(qv, upb_log > 3 ? upb_log : 3, &best_S, &best_log, &K)) return false;
    // planes of at most three rounds: twelve rounds of several plane groups per wavefront
    const uint32_t R = (uint32_t)((qv + best_S - 1) / best_S);
    a->NG = K == 3 ? 12u / R : 1u;
    a->K = K == 3 ? 12u : K;
    a->P = (uint32_t)L.P; a->HW = (uint32_t)L.HW; a->WPP = (uint32_t)L.WPP;
    a->qv = (uint32_t)qv;
    a->S = best_S; a->S_log2 = best_log;
    a->ppw = 64u / best_S;
    a->upb = (uint32_t)upb; a->upb_log2 = upb_log;
    a->nb = (uint32_t)L.nb;
    *grid = (uint32_t)((L.P + (uint64_t)a->ppw * a->NG - 1) / ((uint64_t)a->ppw * a->NG));
    return true;
}

// 1-D maps the register kernel would take as well: compress_line is the faster one for 2-byte
// elements (it loads 16 bytes per lane, the register kernel 8); for fp32 the register kernel is (by 5-10 %)
bool line_first(const Layout& L, size_t es) { return es == 2 || L.HW / 4 < 512; }

// Fills the any-block-size compress plan; false when a plane does not fit LDS or the 32-bit index tricks.
// Hs = rows of one depth slice, D = depth slices (1 for a 2-D map).
bool plan_rows(const Layout& L, int64_t D, int64_t Hs, int64_t W, int B, int b, size_t es, const void* x,
               RowsArgs* a, uint32_t* grid, size_t* lds) {
    (void)b;
    const int64_t H = D * Hs;                       // rows of all slices
    if ((uint64_t)B > L.HW + 64) return false;      // keeps fdiv(r, B) exact; such a B is "one block" anyway: see below
    const uint64_t per_plane = 4ull * L.HW + 16ull * (uint64_t)H * L.LW + 12ull * L.nb + 16ull;
    if (per_plane + 256 > kLdsMax) return false;
    if (!fastdiv_ok(L.HW, (uint64_t)W) || !fastdiv_ok((uint64_t)(H > W ? H : W), (uint64_t)B)) return false;
    if (!fastdiv_ok((uint64_t)H, (uint64_t)Hs) || !fastdiv_ok(L.LD * L.LH, L.LH)) return false;
    uint64_t G = kRowsLdsTarget / per_plane;
    if (G < 1) G = 1;
    if (G > L.P) G = L.P;
    // chunk starts on 16-byte boundaries when G is a multiple of `unit`
    const uint64_t unit = 16 / gcd_u64(16, L.HW * es);
    uint32_t vec_load = ((uintptr_t)x % 16) == 0;
    if (vec_load && G % unit != 0) {
        if (G > unit) G -= G % unit;
        else if (unit * per_plane + 256 <= kLdsMax && unit <= L.P) G = unit;
        else if (G < L.P) vec_load = 0;
    }
    const uint64_t HLW = (uint64_t)H * L.LW;
    if (!fastdiv_ok(G * HLW + kThreads, HLW) || !fastdiv_ok(HLW, L.LW) || !fastdiv_ok(G * L.nb + kThreads, L.nb) ||
        !fastdiv_ok(L.nb, L.LW) || !fastdiv_ok(G * L.WPP + kThreads, L.WPP))
        return false;
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW;
    a->LH = (uint32_t)(L.LD * L.LH); a->LW = (uint32_t)L.LW; a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP; a->B = (uint32_t)B;
    a->D = (uint32_t)D; a->Hs = (uint32_t)Hs; a->LHs = (uint32_t)L.LH;
    a->G = (uint32_t)G;
    a->xs_floats = (uint32_t)((G * L.HW + 3) / 4 * 4);
    a->vec_load = vec_load;
    const uint64_t epv = 16 / es;
    a->keep = vec_load && (uint64_t)W % epv == 0 && G * (L.HW / epv) <= (uint64_t)kRowsKeep * kThreads;
    a->vecblk = a->keep && (uint64_t)B % epv == 0;
    a->qv = (uint32_t)(L.HW / epv);
    a->d_qv = make_fastdiv(a->qv ? a->qv : 1u);
    a->d_W = make_fastdiv((uint32_t)W);
    a->d_B = make_fastdiv((uint32_t)B);
    a->d_Hs = make_fastdiv((uint32_t)Hs);
    a->d_LHs = make_fastdiv((uint32_t)L.LH);
    a->d_LW = make_fastdiv((uint32_t)L.LW);
    a->d_HLW = make_fastdiv((uint32_t)HLW);
    a->d_nb = make_fastdiv((uint32_t)L.nb);
    a->d_wpp = make_fastdiv((uint32_t)L.WPP);
    *lds = 16ull * G + 4ull * a->xs_floats + 16ull * G * HLW + 4ull * ((G * L.nb + 1) & ~1ull) + 8ull * G * L.nb + 16;
    *grid = (uint32_t)((L.P + G - 1) / G);
    return *lds <= kLdsMax;
}

// Fills the workgroup-per-plane plan for planes beyond LDS; false when rows or blocks are not whole
// 16-byte vectors or the per-slice partial sums do not fit LDS.
bool plan_plane(const Layout& L, int64_t D, int64_t Hs, int64_t W, int B, size_t es, const void* x,
                PlaneArgs* a, uint32_t* grid, size_t* lds) {
    const uint64_t epv = 16 / es;
    if (((uintptr_t)x % 16) != 0 || (uint64_t)W % epv != 0 || (uint64_t)B % epv != 0) return false;
    const uint64_t H = (uint64_t)D * (uint64_t)Hs;
    const uint64_t slice = L.LH * L.LW;
    const uint64_t nitem = (uint64_t)D * slice;
    const uint64_t need = 16ull * nitem + 4ull * ((L.nb + 3) & ~3ull) + 8ull * (kThreads / 64) + 16 + 16;
    if (need > kLdsMax) return false;
    if (!fastdiv_ok(L.HW, (uint64_t)W) || !fastdiv_ok(H > (uint64_t)W ? H : (uint64_t)W, (uint64_t)B) ||
        !fastdiv_ok(H, (uint64_t)Hs) || !fastdiv_ok(nitem + kThreads, slice) || !fastdiv_ok(slice, L.LW))
        return false;
    a->P = (uint32_t)L.P; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW; a->LW = (uint32_t)L.LW;
    a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP; a->B = (uint32_t)B;
    a->D = (uint32_t)D; a->Hs = (uint32_t)Hs; a->LHs = (uint32_t)L.LH;
    a->nitem = (uint32_t)nitem;
    a->qv = (uint32_t)(L.HW / epv);
    a->d_W = make_fastdiv((uint32_t)W);
    a->d_B = make_fastdiv((uint32_t)B);
    a->d_Hs = make_fastdiv((uint32_t)Hs);
    a->d_LW = make_fastdiv((uint32_t)L.LW);
    a->d_LHs = make_fastdiv((uint32_t)L.LH);
    a->d_slice = make_fastdiv((uint32_t)slice);
    *lds = need;
    *grid = (uint32_t)L.P;
    return true;
}

// Fills the tiled-compress launch plan; false when the shape is not covered.
bool plan_tile(const Layout& L, int64_t H, int64_t W, int B, int b, size_t es, const void* x,
               TileArgs* a, uint32_t* grid, size_t* lds, int* vec_out, int* nt_out) {
    if (B != 4 && B != 8) return false;
    const int vec = (W % 4 == 0) ? 4 : (W % 2 == 0) ? 2 : 1;
    const uint32_t ipb = (uint32_t)B / (uint32_t)vec;
    const uint64_t slots = ((uint64_t)W + vec - 1) / vec;
    const uint64_t ipr = (slots + ipb - 1) / ipb * ipb;
    const uint64_t ipp = L.LH * ipr;
    const uint64_t per_plane = 4ull * L.HW + 8ull * ipp + 16ull;
    if (per_plane + 64 > kLdsMax) return false;
    const int nt = 256;
    uint64_t Gmax = kLdsTarget / per_plane;
    if (Gmax < 1) Gmax = 1;
    if (Gmax > L.P) Gmax = L.P;
    // chunk starts stay 16-byte aligned when G * (bytes per plane) is a multiple of 16
    const uint64_t unit = 16 / gcd_u64(16, L.HW * es);
    uint32_t vec_load = ((uintptr_t)x % 16) == 0;
    if (vec_load && unit > 1 && Gmax < unit && Gmax < L.P) {
        if (unit * per_plane + 64 <= kLdsMax) Gmax = unit; else vec_load = 0;
    }
    const uint64_t step = vec_load ? unit : 1;
    // pick the G whose last, partly filled wavefront pass wastes the fewest lanes
    const double c1 = 4.0 * B * vec, c3 = 7.5 * (32 / b);
    uint64_t G = 0;
    double best = 0;
    for (uint64_t g = step; g <= Gmax; g += step) {
        const double cost = (double)((g * ipp + 63) / 64) * c1 + (double)((g * L.WPP + 63) / 64) * c3;
        const double per_elt = cost / (double)(g * L.HW);
        if (G == 0 || per_elt < best * 0.98) { G = g; best = per_elt; }
    }
    if (G == 0) G = Gmax;          // Gmax == P < unit: a single chunk, aligned at its start
    const uint64_t nitems = G * ipp, nwords = G * L.WPP;
    if (!fastdiv_ok(nitems + 256, ipp) || !fastdiv_ok(ipp, ipr) || !fastdiv_ok(nwords + 256, L.WPP))
        return false;
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW;
    a->LH = (uint32_t)L.LH; a->LW = (uint32_t)L.LW; a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP;
    a->G = (uint32_t)G; a->ipr = (uint32_t)ipr; a->ipp = (uint32_t)ipp;
    uint32_t S = 1;
    while (S < 64 && (uint64_t)S * 2 <= ipp) S *= 2;
    a->S = S;
    a->xs_floats = (uint32_t)((G * L.HW + 3) / 4 * 4);
    a->items_cap = (uint32_t)((nitems + 3) / 4 * 4);
    a->vec_load = vec_load;
    a->d_ipp = make_fastdiv((uint32_t)ipp);
    a->d_ipr = make_fastdiv((uint32_t)ipr);
    a->d_wpp = make_fastdiv((uint32_t)L.WPP);
    *lds = 16ull * G + 4ull * a->xs_floats + 8ull * a->items_cap;
    *grid = (uint32_t)((L.P + G - 1) / G);
    *vec_out = vec;
    *nt_out = nt;
    return *lds <= kLdsMax;
}

// LDS bytes of the streaming decompress kernels for G planes per workgroup
size_t dec_lds_bytes(const Layout& L, size_t es, uint64_t G) {
    return 4ull * ((G * L.WPP + 3) & ~(uint64_t)3) + 8ull * G + es * G * L.nb + 16;
}
constexpr size_t kDecLdsMax = 60u << 10;

// Planes per workgroup of the streaming decompress kernels: about 32 KB of output, in whole 128-byte
// lines where that is possible within twice the target, so that no line is shared by two
// workgroups.  Measured inside a whole compress + decompress step over the ResNet-50 set: 24-48 KB
// is the flat optimum (64 KB: 0.5-1 % slower, 12 KB: 4 % slower, 6 KB: 12 %).  A decompress kernel
// timed on its own, launch after launch, prefers 12 KB by 15 %, but not between other kernels.
// `mult`: G must be a multiple of it (flat kernel: whole 4-element vectors).
#ifndef DIVISION_DEC_CHUNK
#define DIVISION_DEC_CHUNK 32768
#endif
constexpr uint64_t kDecChunkBytes = DIVISION_DEC_CHUNK;
uint64_t dec_planes(const Layout& L, size_t es, uint64_t mult) {
    const uint64_t target = kDecChunkBytes / es;
    uint64_t G = (target + L.HW / 2) / L.HW;
    if (G < 1) G = 1;
    uint64_t unit = 128 / gcd_u64(128, L.HW * es);
    unit = unit / gcd_u64(unit, mult) * mult;
    if (unit * L.HW > 2 * target) unit = mult;
    G = (G + unit / 2) / unit * unit;
    if (G < unit) G = unit;
    if (G > L.P) G = L.P;
    return G;
}

// Fills the decompress launch plan; returns 7 (row vectors of 4-byte elements, a wavefront per chunk), 0 (row vectors), 3 (block table),
// 8 (4-byte elements of any width, a wavefront per chunk), 6 (four consecutive elements
// per lane step, any width), 5 (word by word through LDS), 1 (flat), 4 (lane per plane) or 2 (scalar).
// Hs = rows of one depth slice, D = depth slices (1 for a 2-D map; the table kernel takes 2-D maps only).
int plan_decompress(const Layout& L, int64_t D, int64_t Hs, int64_t W, int B, size_t es, const void* xhat,
                    DecArgs* a, uint32_t* grid) {
    const int64_t H = D * Hs;
    a->P = (uint32_t)L.P; a->H = (uint32_t)H; a->W = (uint32_t)W; a->HW = (uint32_t)L.HW;
    a->LH = (uint32_t)(L.LD * L.LH); a->LW = (uint32_t)L.LW; a->nb = (uint32_t)L.nb; a->WPP = (uint32_t)L.WPP; a->B = (uint32_t)B;
    a->Hs = (uint32_t)Hs; a->LHs = (uint32_t)L.LH;
    a->d_B = make_fastdiv((uint32_t)B);
    a->d_W = make_fastdiv((uint32_t)W);
    a->d_HW = make_fastdiv((uint32_t)L.HW);
    a->d_Hs = make_fastdiv((uint32_t)Hs);
    const bool small_idx = fastdiv_ok((uint64_t)H, (uint64_t)B) && fastdiv_ok((uint64_t)W, (uint64_t)B) &&
                           fastdiv_ok((uint64_t)H, (uint64_t)Hs);
    const bool out_vec_aligned = ((uintptr_t)xhat % (4 * es)) == 0;
    // one-block planes with an odd element count: a lane per plane, 64 planes per round
    if (lane_shape(L)) {
        const uint32_t nrounds = (uint32_t)((L.P + 63) / 64);
        uint32_t rpw = 2;
        while (rpw > 1 && nrounds / rpw < 32u * (uint32_t)num_cus()) --rpw;
        a->G = rpw;
        *grid = (nrounds + rpw - 1) / rpw;
        return 4;
    }
    // 4-byte elements, one block per plane (not those of the lane kernel above, which measured the same on 7 x 7, nor those of the row-vector stream kernel below): a wavefront per
    // chunk of aligned vectors, H^L is the plane's
    if (es == 4 && L.nb == 1 && !(W % 4 == 0 && B % 4 == 0) && L.HW >= 4 && L.HW < (1ull << 24) && L.P < (1ull << 24) && out_vec_aligned &&
        L.P * L.WPP * 4 < (1ull << 31) && L.P * 8 < (1ull << 31)) {
        const uint64_t chunk = 256ull * kStreamK;                       // elements
        const uint64_t ntot = L.P * L.HW;
        if (fastdiv_ok(L.HW + chunk + 4, L.HW) && (ntot + chunk - 1) / chunk < (1ull << 31) && ntot < (1ull << 42)) {
            *grid = (uint32_t)((ntot + chunk - 1) / chunk);
            return 9;
        }
    }
    // fast path: rows are whole vectors that sit inside one block
    if (W % 4 == 0 && B % 4 == 0 && small_idx && out_vec_aligned) {
        a->q4 = (uint32_t)(L.HW / 4);
        a->w4 = (uint32_t)(W / 4);
        // 4-byte elements: one wavefront per 64 * kStreamK vectors, no staging
        const uint64_t chunk = 64ull * kStreamK;
        const uint64_t nvec = L.P * (L.HW / 4);
        if (es == 4 && fastdiv_ok(a->q4 + chunk, a->q4) && fastdiv_ok(a->q4, a->w4) && (nvec + chunk - 1) / chunk < (1ull << 31) &&
            nvec < (1ull << 40)) {
            a->d_q4 = make_fastdiv(a->q4);
            a->d_w4 = make_fastdiv(a->w4);
            *grid = (uint32_t)((nvec + chunk - 1) / chunk);
            return 7;
        }
        uint64_t G = dec_planes(L, es, 1);
        while (G > 1 && !fastdiv_ok(G * a->q4 + kThreads, a->q4)) --G;
        if (fastdiv_ok(G * a->q4 + kThreads, a->q4) && fastdiv_ok(a->q4, a->w4) && dec_lds_bytes(L, es, G) <= kDecLdsMax) {
            a->G = (uint32_t)G;
            a->d_q4 = make_fastdiv(a->q4);
            a->d_w4 = make_fastdiv(a->w4);
            a->pair8 = es == 2 && W % 8 == 0 && ((uintptr_t)xhat % 16) == 0;
            *grid = (uint32_t)((L.P + G - 1) / G);
            return 0;
        }
    }
    // planes of whole vectors with few blocks: LFC indices from a table in LDS
    if (D == 1 && L.HW % 4 == 0 && L.nb > 1 && L.nb <= 255 && small_idx && out_vec_aligned && fastdiv_ok(L.HW, (uint64_t)W)) {
        a->q4 = (uint32_t)(L.HW / 4);
        uint64_t G = dec_planes(L, es, 1);
        while (G > 1 && !fastdiv_ok(G * a->q4 + kThreads, a->q4)) --G;
        if (fastdiv_ok(G * a->q4 + kThreads, a->q4) && dec_lds_bytes(L, es, G) + 4ull * a->q4 + 16 <= kDecLdsMax) {
            a->G = (uint32_t)G;
            a->d_q4 = make_fastdiv(a->q4);
            *grid = (uint32_t)((L.P + G - 1) / G);
            return 3;
        }
    }
    // 4-byte elements, rows, blocks or planes that are not whole vectors: a wavefront per chunk of aligned vectors,
    // every element finds its own plane and block
    // (several blocks per plane: one-block planes are the flat kernel's, measured faster there; B >= 4 and W >= 4: a
    // vector then leaves its row and its block column at most once, and no division is by 1; plane and plane count
    // below 2^24 for the 24-bit multiplies; the three regions of the packed buffer within 32-bit byte offsets)
    if (es == 4 && L.nb > 1 && W >= 4 && B >= 4 && (D == 1 || Hs >= 2) && L.HW < (1ull << 24) && L.P < (1ull << 24) && small_idx && out_vec_aligned && fastdiv_ok(L.HW, (uint64_t)W) &&
        fastdiv_ok((uint64_t)H + 1, (uint64_t)B) && L.P * L.WPP * 4 < (1ull << 31) && L.P * L.nb * 4 < (1ull << 31) && L.P * 8 < (1ull << 31)) {
        const uint64_t chunk = 256ull * kStreamK;                       // elements
        const uint64_t ntot = L.P * L.HW;
        if (fastdiv_ok(L.HW + chunk + 4, L.HW) && (ntot + chunk - 1) / chunk < (1ull << 31) && ntot < (1ull << 42)) {
            *grid = (uint32_t)((ntot + chunk - 1) / chunk);
            return 8;
        }
    }
    // planes (2-D or 3-D) of 512 elements and more whose rows or blocks are not whole vectors: four consecutive
    // elements per lane step, planes starting on 4-byte boundaries
    if (Hs > 1 && small_idx && ((uintptr_t)xhat % 4) == 0 && L.nb <= 16383) {
        // units per plane, counting the one more that a plane starting 3 elements past a unit boundary takes
        const uint64_t q4 = (L.HW + (L.HW % 4 ? 6 : 0)) / 4;
        int nw = 1;
        while (nw < 16 && (q4 > (uint64_t)kUnitsK * 64 * nw || L.nb > (uint64_t)kUnitsLfc * 64 * nw)) nw *= 2;
        const uint64_t nt = 64ull * nw;
        if (q4 >= kUnitsMin && q4 <= (uint64_t)kUnitsK * nt && L.nb <= (uint64_t)kUnitsLfc * nt &&
            fastdiv_ok(4ull * kUnitsK * nt + 4, (uint64_t)W) && fastdiv_ok(4ull * kUnitsK * nt + 4, (uint64_t)B) &&
            fastdiv_ok(4ull * kUnitsK * nt + 4, (uint64_t)Hs)) {
            a->q4 = (uint32_t)q4;
            a->G = (uint32_t)nw;                  // wavefronts per workgroup
            uint64_t g = (uint64_t)num_cus() * (16ull / nw);
            g = (g + 3) & ~3ull;        // the planes of a workgroup start alike within a unit of the map
            *grid = (uint32_t)(g < L.P ? g : L.P);
            return 6;
        }
    }
    // several blocks per plane, rows not whole vectors: rebuilt in LDS word by word
    if (L.nb > 1 && small_idx && out_vec_aligned && fastdiv_ok(L.HW, (uint64_t)W)) {
        const uint64_t unit = 4 / gcd_u64(4, L.HW);
        uint64_t G = dec_planes(L, 4, unit);          // the chunk is staged as fp32 whatever the element type
        const uint64_t staged = (dec_lds_bytes(L, es, G) + 15) & ~15ull;
        if (fastdiv_ok(G * L.WPP + kThreads, L.WPP) && staged + 4ull * ((G * L.HW + 3) & ~3ull) <= kDecLdsMax) {
            a->G = (uint32_t)G;
            a->out_off = (uint32_t)staged;
            a->d_wpp = make_fastdiv((uint32_t)L.WPP);
            *grid = (uint32_t)((L.P + G - 1) / G);
            return 5;
        }
    }
    // general path: flat run of G planes, G*HW a multiple of 4
    if (small_idx && out_vec_aligned && fastdiv_ok(L.HW, (uint64_t)W)) {
        const uint64_t unit = 4 / gcd_u64(4, L.HW);
        const uint64_t G = dec_planes(L, es, unit);
        if (fastdiv_ok(G * L.HW + 4ull * kThreads, L.HW) && dec_lds_bytes(L, es, G) <= kDecLdsMax) {
            a->G = (uint32_t)G;
            *grid = (uint32_t)((L.P + G - 1) / G);
            return 1;
        }
    }
    a->G = 1;
    *grid = (uint32_t)L.P;
    return 2;
}

// calls f(T{}, std::integral_constant<int, BITS>{}) for the element / cache type and code width of a call
// calls f(std::integral_constant<int, BITS>{}) for the code width of a call
template <typename F>
hipError_t with_bits(int b, F&& f) {
    return b == 2 ? f(std::integral_constant<int, 2>{}) : b == 4 ? f(std::integral_constant<int, 4>{})
                                                                  : f(std::integral_constant<int, 8>{});
}

enum CompKind { REGS, LANE, LINE, STRIP, ROWSTRIP, ITEMS, UNITS, WAVE, TILE, ONE, ROWS, PLANE, ANY };

// everything a compress launch needs once the plan is made (the arguments of the kernel that was picked)
struct CompLaunch {
    int kind, B, vec, nt, nw, flat;
    uint32_t gx, gy;
    size_t lds;
    hipStream_t st;
    TileArgs a; WaveArgs wa; RegsArgs ra; ItemsArgs ia; LaneArgs la; RowsArgs wa2; PlaneArgs pa; OneArgs oa; AnyArgs g; UnitsArgs ua; StripArgs sa;
};
struct DecLaunch {
    int kind, flat, nw;
    uint32_t gx, gy;
    size_t lds;
    hipStream_t st;
    DecArgs a;
};

template <typename T, int BITS>
hipError_t launch_one(const OneArgs& a, dim3 gd, hipStream_t st) {
    void (*kern)(OneArgs) = a.K == 3 ? compress_one<T, BITS, 3> : a.K == 4 ? compress_one<T, BITS, 4> : a.K == 6 ? compress_one<T, BITS, 6> : compress_one<T, BITS, 13>;
    hipLaunchKernelGGL(kern, gd, dim3(64), 0, st, a);
    return hipGetLastError();
}
template <typename T, int BITS>
hipError_t launch_line(const OneArgs& a, dim3 gd, hipStream_t st) {
    void (*kern)(OneArgs) = a.K == 12 ? (a.NG == 12 ? compress_line<T, BITS, 12, 12> : a.NG == 6 ? compress_line<T, BITS, 12, 6> : compress_line<T, BITS, 12, 4>)
                          : a.K == 4 ? compress_line<T, BITS, 4> : a.K == 6 ? compress_line<T, BITS, 6> : compress_line<T, BITS, 13>;
    hipLaunchKernelGGL(kern, gd, dim3(64), 0, st, a);
    return hipGetLastError();
}

template <typename T>
hipError_t do_compress(const CompLaunch& c, int b) {
    const dim3 gd(c.gx, c.gy);
    hipStream_t st = c.st;
    const size_t lds = c.lds;
    const bool flat = c.flat != 0;
    if (b == 1) {
        // 1-bit codes: the kernels that have an instance for them (the planner picks nothing else)
        switch (c.kind) {
            case REGS: return launch_regs<T, 1>(c.B, c.nw, c.ra, gd, lds, st);
            case STRIP: return launch_strip<T, 1>(c.vec, c.sa, gd, lds, st);
            case ROWSTRIP: return launch_rowstrip<T, 1>(c.vec, c.sa, gd, lds, st);
            case LANE: hipLaunchKernelGGL((compress_lane<T, 1>), gd, dim3(64), lds, st, c.la); return hipGetLastError();
            case ITEMS: return launch_items<T, 1>(c.B, c.vec, c.ia, gd, lds, st);
            case UNITS: return launch_units<T, 1>(c.nw, c.ua, gd, lds, st);
            case ONE: return launch_one<T, 1>(c.oa, gd, st);
            case LINE: return launch_line<T, 1>(c.oa, gd, st);
            case TILE: return launch_tile<T, 1>(c.B, c.vec, c.a, gd, lds, st);
            default: {
                void (*kern)(AnyArgs) = flat ? compress_any<T, 1> : compress_any_3d<T, 1>;
                hipLaunchKernelGGL(kern, gd, dim3(kThreads), 0, st, c.g);
                return hipGetLastError();
            }
        }
    }
    return with_bits(b, [&](auto bits) -> hipError_t {
        constexpr int BITS = decltype(bits)::value;
        switch (c.kind) {
            case REGS: return launch_regs<T, BITS>(c.B, c.nw, c.ra, gd, lds, st);
            case STRIP: return launch_strip<T, BITS>(c.vec, c.sa, gd, lds, st);
            case ROWSTRIP: return launch_rowstrip<T, BITS>(c.vec, c.sa, gd, lds, st);
            case ITEMS: return launch_items<T, BITS>(c.B, c.vec, c.ia, gd, lds, st);
            case UNITS: return launch_units<T, BITS>(c.nw, c.ua, gd, lds, st);
            case WAVE: return launch_wave<T, BITS>(c.B, c.vec, c.wa, gd, lds, st);
            case TILE: return launch_tile<T, BITS>(c.B, c.vec, c.a, gd, lds, st);
            case LANE: hipLaunchKernelGGL((compress_lane<T, BITS>), gd, dim3(64), lds, st, c.la); return hipGetLastError();
            case ONE: return launch_one<T, BITS>(c.oa, gd, st);
            case LINE: return launch_line<T, BITS>(c.oa, gd, st);
            case ROWS: {
                void (*kern)(RowsArgs) = flat ? compress_rows<T, BITS> : compress_rows_3d<T, BITS>;
                const hipError_t e = allow_large_lds(kern, lds);
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL(kern, gd, dim3(kThreads), lds, st, c.wa2);
                return hipGetLastError();
            }
            case PLANE: {
                void (*kern)(PlaneArgs) = flat ? compress_plane<T, BITS> : compress_plane_3d<T, BITS>;
                const hipError_t e = allow_large_lds(kern, lds);
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL(kern, gd, dim3(kThreads), lds, st, c.pa);
                return hipGetLastError();
            }
            default: {
                void (*kern)(AnyArgs) = flat ? compress_any<T, BITS> : compress_any_3d<T, BITS>;
                hipLaunchKernelGGL(kern, gd, dim3(kThreads), 0, st, c.g);
                return hipGetLastError();
            }
        }
    });
}

template <typename T>
hipError_t do_decompress(const DecLaunch& c, int b) {
    // every decompress kernel has an instance for 1-bit codes too
    auto launch = [&](auto bits) -> hipError_t {
        constexpr int BITS = decltype(bits)::value;
        const int kind = c.kind;
        void (*kern)(DecArgs);
        if (kind == 7 || kind == 8 || kind == 9) {
            if (kind == 7) kern = c.flat ? decompress_stream<T, BITS> : decompress_stream_3d<T, BITS>;
            else if (kind == 9) kern = decompress_stream_one<T, BITS>;
            else kern = c.flat ? decompress_stream_any<T, BITS> : decompress_stream_any_3d<T, BITS>;
            hipLaunchKernelGGL(kern, dim3(c.gx, c.gy), dim3(64), 0, c.st, c.a);
            return hipGetLastError();
        }
        if (kind == 6) {
            kern = c.nw == 1 ? decompress_units<T, BITS, 1> : c.nw == 2 ? decompress_units<T, BITS, 2>
                 : c.nw == 4 ? decompress_units<T, BITS, 4> : c.nw == 8 ? decompress_units<T, BITS, 8>
                                                                        : decompress_units<T, BITS, 16>;
            hipLaunchKernelGGL(kern, dim3(c.gx, c.gy), dim3(64 * c.nw), c.lds, c.st, c.a);
            return hipGetLastError();
        }
        if (c.flat)
            kern = kind == 0 ? decompress_rowvec<T, BITS> : kind == 3 ? decompress_table<T, BITS>
                 : kind == 5 ? decompress_words<T, BITS> : kind == 1 ? decompress_flat<T, BITS>
                 : kind == 4 ? decompress_lane<T, BITS> : decompress_scalar<T, BITS>;
        else
            kern = kind == 0 ? decompress_rowvec_3d<T, BITS> : kind == 5 ? decompress_words_3d<T, BITS>
                 : kind == 1 ? decompress_flat_3d<T, BITS>
                 : kind == 4 ? decompress_lane<T, BITS> : decompress_scalar_3d<T, BITS>;
        const hipError_t e = allow_large_lds(kern, c.lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3(c.gx, c.gy), dim3(kind == 4 ? 64 : kThreads), c.lds, c.st, c.a);
        return hipGetLastError();
    };
    return b == 1 ? launch(std::integral_constant<int, 1>{}) : with_bits(b, launch);
}

// the Relu + compress kernels: the register kernel's planes (c.ra carries y and mask), c.kind == STRIP the
// strip kernel's (c.sa) or, c.kind == ITEMS, the items kernel's (c.ia); one map per launch
template <typename T>
hipError_t do_relu(const CompLaunch& c, int b) {
    return with_bits(b, [&](auto bits) -> hipError_t {
        constexpr int BITS = decltype(bits)::value;
        if (c.kind == ITEMS) return launch_relu_items<T, BITS>(c.B, c.vec, c.ia, dim3(c.gx, 1), c.lds, c.st);
        if (c.kind == STRIP) return launch_relu_strip<T, BITS>(c.vec, c.sa, dim3(c.gx, 1), c.lds, c.st);
        void (*kern)(RegsArgs);
        if (c.nw == 1) kern = c.B == 8 ? relu_compress_regs<T, BITS, 8, 1> : relu_compress_regs<T, BITS, 4, 1>;
        else kern = c.B == 8 ? relu_compress_regs<T, BITS, 8, 4> : relu_compress_regs<T, BITS, 4, 4>;
        hipLaunchKernelGGL(kern, dim3(c.gx, 1), dim3(64 * c.nw), c.lds, c.st, c.ra);
        return hipGetLastError();
    });
}

hipError_t bridge_compress(division_dtype dt, const CompLaunch& c, int b) {
    return dt == DIVISION_F32 ? division_bridge_compress_f32(&c, b)
         : dt == DIVISION_BF16 ? division_bridge_compress_bf16(&c, b) : division_bridge_compress_c16(&c, b);
}
hipError_t bridge_decompress(division_dtype dt, const DecLaunch& c, int b) {
    return dt == DIVISION_F32 ? division_bridge_decompress_f32(&c, b)
         : dt == DIVISION_BF16 ? division_bridge_decompress_bf16(&c, b) : division_bridge_decompress_c16(&c, b);
}
hipError_t bridge_relu(division_dtype dt, const CompLaunch& c, int b) {
    return dt == DIVISION_F32 ? division_bridge_relu_f32(&c, b)
         : dt == DIVISION_BF16 ? division_bridge_relu_bf16(&c, b) : division_bridge_relu_c16(&c, b);
}

// A 3-D map with a dimension of extent 1 is a 2-D map with the same flat element order, the same
// blocks and the same packed buffer: D x 1 x W -> D x W, D x H x 1 -> D x H.  (1 x H x W needs nothing.)
void squeeze_dims(int64_t& D, int64_t& H, int64_t& W) {
    if (D > 1 && H == 1) { H = D; D = 1; }
    else if (D > 1 && W == 1) { W = H; H = D; D = 1; }
}

// A plane that is a single block has the same cached tuple under every block size that covers it:
// small 2-D planes are handed to the kernels specialised for B = 4 and B = 8.
int covering_block(const Layout& L, int64_t D, int64_t H, int64_t W, int B) {
    if (L.nb != 1 || D != 1) return B;
    const int64_t m = H > W ? H : W;
    return m <= 4 ? 4 : m <= 8 ? 8 : B;
}

int packed_layout_impl(int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int B, int b, division_dtype dt,
                       size_t* codes_off, size_t* codes_bytes, size_t* meta_off, size_t* meta_bytes,
                       size_t* lfc_off, size_t* lfc_bytes) {
    if (!codes_off || !codes_bytes || !meta_off || !meta_bytes || !lfc_off || !lfc_bytes) return DIVISION_EINVAL;
    Layout L;
    if (make_layout(N, C, D, H, W, B, b, (int)dt, &L) != DIVISION_OK) return DIVISION_EINVAL;
    *codes_off = L.codes_off; *codes_bytes = L.codes_bytes;
    *meta_off = L.meta_off;   *meta_bytes = L.meta_bytes;
    *lfc_off = L.lfc_off;     *lfc_bytes = L.lfc_bytes;
    return DIVISION_OK;
}

int compress_impl(int count, const void* const* x, void* const* packed, const uint64_t* seeds,
                  int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, division_dtype dt,
                  int B, int b, size_t packed_capacity, void* hip_stream) {
    if (count < 0 || (count > 0 && (!x || !packed || !seeds))) return DIVISION_EINVAL;
    squeeze_dims(D, H, W);
    Layout L;
    const int rc = make_layout(N, C, D, H, W, B, b, (int)dt, &L);
    if (rc != DIVISION_OK) return rc;
    B = covering_block(L, D, H, W, B);
    if (packed_capacity < L.total) return DIVISION_ESIZE;
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    uintptr_t all_x = 0;            // alignment of the batch = alignment of the OR of its pointers
    for (int i = 0; i < count; ++i) {
        if (!x[i] || !packed[i]) return DIVISION_EINVAL;
        if (((uintptr_t)x[i] % es) != 0 || ((uintptr_t)packed[i] % 16) != 0) return DIVISION_EALIGN;
        all_x |= (uintptr_t)x[i];
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const void* xa = reinterpret_cast<const void*>(all_x ? all_x : 16);
    const Regions rg = make_regions(L);

    for (int i0 = 0; i0 < count; i0 += kMaxBatch) {
        const int cnt = count - i0 < kMaxBatch ? count - i0 : kMaxBatch;
        CompTab tab{};
        for (int i = 0; i < cnt; ++i) {
            tab.x[i] = x[i0 + i];
            tab.pk[i] = packed[i0 + i];
            tab.seed_a[i] = mix32((uint32_t)(seeds[i0 + i] & 0xffffffffu) ^ 0x243F6A88u);
            tab.seed_c[i] = mix32((uint32_t)(seeds[i0 + i] >> 32) ^ 0x85A308D3u);
        }
        TileArgs a{};
        WaveArgs wa{};
        RegsArgs ra{};
        ItemsArgs ia{};
        LaneArgs la{};
        RowsArgs wa2{};
        PlaneArgs pa{};
        OneArgs oa{};
        AnyArgs g{};
        UnitsArgs ua{};
        StripArgs sa{};
        size_t lds = 0;
        uint32_t grid = 0;
        int vec = 1, nt = 64, nw = 1;
        CompKind kind;
        const bool flat = D == 1;               // the register, item, wavefront and tile kernels take 2-D maps
        auto use_any = [&]() {
            kind = ANY;
            g.tab = tab; g.rg = rg;
            g.P = (uint32_t)L.P; g.H = (uint32_t)H; g.W = (uint32_t)W; g.HW = (uint32_t)L.HW; g.D = (uint32_t)D;
            g.LH = (uint32_t)L.LH; g.LW = (uint32_t)L.LW; g.nb = (uint32_t)L.nb; g.WPP = (uint32_t)L.WPP; g.B = (uint32_t)B;
            grid = (uint32_t)L.P;
        };
        // 1-bit codes (Q = 1) have no instance of the wave, rows and plane kernels, nor of the units kernel with
        // sixteen wavefronts: the wave kernel's shapes go to the tile kernel, the others to the general kernel
        const bool wide = b != 1;
        if (line_first(L, es) && plan_line(L, D, H, B, es, xa, &oa, &grid)) { kind = LINE; oa.tab = tab; oa.rg = rg; lds = 0; }
        else if (plan_regs(L, D, H, W, B, es, xa, &ra, &grid, &lds, &nw)) { kind = REGS; ra.tab = tab; ra.rg = rg; }
        else if (plan_lane(L, es, xa, &la, &grid, &lds)) { kind = LANE; la.tab = tab; la.rg = rg; }
        else if (plan_line(L, D, H, B, es, xa, &oa, &grid)) { kind = LINE; oa.tab = tab; oa.rg = rg; lds = 0; }
        else if (flat && plan_strip(L, H, W, B, es, xa, &sa, &grid, &lds, &vec)) { kind = STRIP; sa.tab = tab; sa.rg = rg; }
        else if (flat && plan_rowstrip(L, H, W, B, es, xa, &sa, &grid, &lds, &vec)) { kind = ROWSTRIP; sa.tab = tab; sa.rg = rg; }
        else if (flat && plan_items(L, H, W, B, es, xa, &ia, &grid, &lds, &vec)) { kind = ITEMS; ia.tab = tab; ia.rg = rg; }
        else if (!one_shape(L, es, xa) && plan_units(L, D, H, W, B, es, xa, &ua, &grid, &lds, &nw) && (wide || nw != 16)) { kind = UNITS; ua.tab = tab; ua.rg = rg; }
        else if (wide && flat && plan_wave(L, H, W, B, b, es, xa, &wa, &grid, &lds, &vec)) {
            kind = WAVE; wa.tab = tab; wa.rg = rg;
        } else if (flat && plan_tile(L, H, W, B, b, es, xa, &a, &grid, &lds, &vec, &nt)) { kind = TILE; a.tab = tab; a.rg = rg; }
        else if (plan_one(L, es, xa, &oa, &grid)) { kind = ONE; oa.tab = tab; oa.rg = rg; lds = 0; }
        else if (wide && plan_rows(L, D, H, W, B, b, es, xa, &wa2, &grid, &lds)) { kind = ROWS; wa2.tab = tab; wa2.rg = rg; }
        else if (wide && plan_plane(L, D, H, W, B, es, xa, &pa, &grid, &lds)) { kind = PLANE; pa.tab = tab; pa.rg = rg; }
        else use_any();
        CompLaunch c{};
        c.kind = kind; c.B = B; c.vec = vec; c.nt = nt; c.nw = nw; c.flat = flat;
        c.gx = grid; c.gy = (uint32_t)cnt; c.lds = lds; c.st = st;
        c.sa = sa; c.a = a; c.wa = wa; c.ra = ra; c.ia = ia; c.la = la; c.wa2 = wa2; c.pa = pa; c.oa = oa; c.g = g; c.ua = ua;
        const hipError_t err = bridge_compress(dt, c, b);
        if (err != hipSuccess) return DIVISION_EHIP;
    }
    return DIVISION_OK;
}

int decompress_impl(int count, const void* const* packed, void* const* xhat, size_t packed_bytes,
                    int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, division_dtype dt,
                    int B, int b, void* hip_stream) {
    if (count < 0 || (count > 0 && (!packed || !xhat))) return DIVISION_EINVAL;
    squeeze_dims(D, H, W);
    Layout L;
    const int rc = make_layout(N, C, D, H, W, B, b, (int)dt, &L);
    if (rc != DIVISION_OK) return rc;
    B = covering_block(L, D, H, W, B);
    if (packed_bytes < L.total) return DIVISION_ESIZE;
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    uintptr_t all_out = 0;
    for (int i = 0; i < count; ++i) {
        if (!xhat[i] || !packed[i]) return DIVISION_EINVAL;
        if (((uintptr_t)xhat[i] % es) != 0 || ((uintptr_t)packed[i] % 16) != 0) return DIVISION_EALIGN;
        all_out |= (uintptr_t)xhat[i];
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const Regions rg = make_regions(L);

    for (int i0 = 0; i0 < count; i0 += kMaxBatch) {
        const int cnt = count - i0 < kMaxBatch ? count - i0 : kMaxBatch;
        DecArgs a{};
        uint32_t grid = 0;
        const int kind = plan_decompress(L, D, H, W, B, es, reinterpret_cast<const void*>(all_out ? all_out : 16), &a, &grid);
        for (int i = 0; i < cnt; ++i) { a.tab.pk[i] = packed[i0 + i]; a.tab.xhat[i] = xhat[i0 + i]; }
        a.rg = rg;
        // LDS of the streaming kernels: staged codes, meta and LFC of G planes (+ the block table)
        size_t lds = 0;
        if (kind == 4) lds = 4ull * (64ull * L.HW + 4);
        else if (kind == 6) lds = 8ull * ((L.nb + 3) & ~3ull);
        else if (kind == 7 || kind == 8 || kind == 9) lds = 0;
        else if (kind == 5) lds = a.out_off + 4ull * ((a.G * L.HW + 3) & ~3ull);
        else if (kind != 2) lds = dec_lds_bytes(L, es, a.G) + (kind == 3 ? 4ull * a.q4 + 16 : 0);
        DecLaunch c{};
        c.kind = kind; c.flat = D == 1; c.nw = kind == 6 ? (int)a.G : 0; c.gx = grid; c.gy = (uint32_t)cnt; c.lds = lds; c.st = st; c.a = a;
        if (bridge_decompress(dt, c, b) != hipSuccess) return DIVISION_EHIP;
    }
    return DIVISION_OK;
}

int kernel_name_impl(int direction, const void* data, int64_t N, int64_t C, int64_t D, int64_t H, int64_t W,
                     division_dtype dt, int B, int b, char* out, size_t cap) {
    if (!out || cap == 0) return DIVISION_EINVAL;
    squeeze_dims(D, H, W);
    Layout L;
    const int rc = make_layout(N, C, D, H, W, B, b, (int)dt, &L);
    if (rc != DIVISION_OK) return rc;
    B = covering_block(L, D, H, W, B);
    const bool flat = D == 1;
    const char* sfx = flat ? "" : "_3d";
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    const char* tn = dt == DIVISION_BF16 ? "bf16_t" : dt == DIVISION_F32_C16 ? "f32c16_t" : "float";
    int n;
    if (direction == 0) {
        const bool wide = b != 1;        // as in compress_impl
        TileArgs a{}; WaveArgs wa{}; RegsArgs ra{}; ItemsArgs ia{}; LaneArgs la{}; RowsArgs wa2{}; PlaneArgs pa{}; OneArgs oa{}; UnitsArgs ua{}; StripArgs sa{}; size_t lds = 0; uint32_t grid = 0; int vec = 1, nt = 64, nw = 1;
        if (line_first(L, es) && plan_line(L, D, H, B, es, data, &oa, &grid))
            n = snprintf(out, cap, "compress_line<%s, %d, %u, %u>", tn, b, oa.K, oa.NG);
        else if (plan_regs(L, D, H, W, B, es, data, &ra, &grid, &lds, &nw))
            n = snprintf(out, cap, "compress_regs%s<%s, %d, %d, %d>", sfx, tn, b, (B == 4 || B == 8) ? B : 0, nw);
        else if (plan_lane(L, es, data, &la, &grid, &lds))
            n = snprintf(out, cap, "compress_lane<%s, %d>", tn, b);
        else if (plan_line(L, D, H, B, es, data, &oa, &grid))
            n = snprintf(out, cap, "compress_line<%s, %d, %u, %u>", tn, b, oa.K, oa.NG);
        else if (flat && plan_strip(L, H, W, B, es, data, &sa, &grid, &lds, &vec))
            n = snprintf(out, cap, "compress_strip<%s, %d, %d, %d>", tn, b, vec / 100, vec % 100);
        else if (flat && plan_rowstrip(L, H, W, B, es, data, &sa, &grid, &lds, &vec))
            n = snprintf(out, cap, "compress_rowstrip<%s, %d, %d, %d>", tn, b, vec / 100, vec % 100);
        else if (flat && plan_items(L, H, W, B, es, data, &ia, &grid, &lds, &vec))
            n = snprintf(out, cap, "compress_items<%s, %d, %d, %d, %d>", tn, b, B, vec, H == 1 ? 1 : B);
        else if (!one_shape(L, es, data) && plan_units(L, D, H, W, B, es, data, &ua, &grid, &lds, &nw) && (wide || nw != 16))
            n = snprintf(out, cap, "compress_units<%s, %d, %d>", tn, b, nw);
        else if (wide && flat && plan_wave(L, H, W, B, b, es, data, &wa, &grid, &lds, &vec))
            n = snprintf(out, cap, "compress_wave<%s, %d, %d, %d>", tn, b, B, vec);
        else if (flat && plan_tile(L, H, W, B, b, es, data, &a, &grid, &lds, &vec, &nt))
            n = snprintf(out, cap, "compress_tile<%s, %d, %d, %d, %d>", tn, b, B, vec, nt);
        else if (plan_one(L, es, data, &oa, &grid))
            n = snprintf(out, cap, "compress_one<%s, %d, %u>", tn, b, oa.K);
        else if (wide && plan_rows(L, D, H, W, B, b, es, data, &wa2, &grid, &lds))
            n = snprintf(out, cap, "compress_rows%s<%s, %d>", sfx, tn, b);
        else if (wide && plan_plane(L, D, H, W, B, es, data, &pa, &grid, &lds))
            n = snprintf(out, cap, "compress_plane%s<%s, %d>", sfx, tn, b);
        else
            n = snprintf(out, cap, "compress_any%s<%s, %d>", sfx, tn, b);
    } else {
        DecArgs a{}; uint32_t grid = 0;
        const int kind = plan_decompress(L, D, H, W, B, es, data, &a, &grid);
        if (kind == 6)
            n = snprintf(out, cap, "decompress_units<%s, %d, %d>", tn, b, (int)a.G);
        else if (kind == 7)
            n = snprintf(out, cap, "decompress_stream%s<%s, %d>", sfx, tn, b);
        else if (kind == 8)
            n = snprintf(out, cap, "decompress_stream_any%s<%s, %d>", sfx, tn, b);
        else if (kind == 9)
            n = snprintf(out, cap, "decompress_stream_one<%s, %d>", tn, b);
        else
            n = snprintf(out, cap, "%s%s<%s, %d>", kind == 0 ? "decompress_rowvec" : kind == 3 ? "decompress_table" : kind == 5 ? "decompress_words" : kind == 1 ? "decompress_flat" : kind == 4 ? "decompress_lane" : "decompress_scalar",
                         kind == 4 ? "" : sfx, tn, b);
    }
    return (n < 0 || (size_t)n >= cap) ? DIVISION_ESIZE : DIVISION_OK;
}
