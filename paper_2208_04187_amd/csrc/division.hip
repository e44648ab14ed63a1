// DIVISION activation codec for AMD MI355X (gfx950): HIP kernels and C ABI.
//
// Paper: "DIVISION: Memory Efficient Training via Dual Activation Precision".
//   compress   = Sec. 4.1  (AveragePooling -> residual against UpSampling ->
//                           Quant of Eq. (quantization) -> cache the tuple)
//   decompress = Sec. 4.2  (Dequant, then the reconstruction equation)
//
// Compile with -ffp-contract=off: the codec's fp32 steps are single IEEE
// operations (sub, mul, add), never fused, so that codes are reproducible.
//
// Work decomposition (one GPU; (sample, channel) planes are independent; except in compress_plane
// and compress_any every element of x is read from HBM exactly once, and no intermediate tensor
// touches HBM).  The host picks the first kernel of this list that covers the shape:
//   compress_line    1-D maps (one row) whose block is a power-of-two number of 16-byte vectors: planes
//                    in registers, block sums by DPP (before compress_regs for 2-byte elements and
//                    planes below 2048 elements, after it otherwise)
//   compress_regs    planes of 2K-3K / 8K-13K / up to 53K elements (56x56, 112x112, 224x224; 3-D maps of
//                    those sizes), B = 4, 8 (template) or 12, 16 (from the arguments): one plane per
//                    workgroup of one / four / sixteen wavefronts, the plane stays in registers from
//                    load to codes
//   compress_lane    one-block planes with an odd element count (7x7): a lane per plane
//   compress_strip   planes of width 28 / 32 (up to 32 rows) or 14 / 16 (up to 16 rows) under B = 8 (28, 14) and the
//                    12, 16, 18 of the block-size sweep: a lane per strip of 28 or 32 consecutive elements (one
//                    or two rows), the round read with coalesced loads and handed out through LDS, extremes by
//                    DPP, block sums by DPP (B = 8) or through LDS (relu_compress_strip: B = 8 with a Relu
//                    applied to the round as its loads arrive)
//   compress_rowstrip  planes of an odd width with an instance (13, 15, 17, 27, 35, 55) under B = 8 or 4: the strip
//                    kernel with a row per lane; rows start in the middle of an element pair every other time, so a
//                    lane quantises the pairs its row touches and ORs its code bits into the plane's words in LDS
//   compress_items   planes of at most 64 pooling items (28x28, 14x14, CIFAR shapes), B = 4, 8: a lane per
//                    pooling item, loaded straight from global memory, DPP reductions (relu_compress_items:
//                    the same with a Relu applied to the rows as they arrive)
//   compress_units   planes (2-D or 3-D maps) of 256 to about 27K elements whose rows or blocks are not whole
//                    16-byte vectors (odd widths: 27x27, 55x55, 147x147; B = 18): four consecutive elements per lane step
//                    whatever the width, the block of each element looked up in a table made once per
//                    workgroup, the plane parked in LDS for the block sums, next plane's loads in flight
//   compress_wave    other planes up to 17 KB, B = 4, 8: one wavefront per chunk of planes staged in LDS
//   compress_tile    other planes up to 156 KB, B = 4, 8: four wavefronts per chunk staged in LDS
//   compress_one     planes that are a single block (B = 64 on 56x56 and below): flat vectors in registers
//   compress_rows    any block size, small 3-D maps: chunk staged in LDS, vectors kept in registers for Quant
//   compress_plane   planes beyond LDS with vector rows and blocks (video volumes, image-sized maps):
//                    a workgroup per plane, two vector passes over x
//   compress_any     everything else (giant planes with odd extents): scalar, slow
//   decompress_stream / decompress_stream_any / decompress_stream_one: 4-byte elements, one wavefront per 4 KB chunk of aligned vectors, no LDS:
//                    rows of whole vectors inside one block (_stream), or any width where a vector may span two rows
//                    and two planes (_stream_any: each element finds its plane and block, six loads per vector;
//                    _stream_one: planes that are one block)
//   decompress_rowvec / _table / _words / _flat / _lane / _scalar: streaming, the packed slice of a
//                    workgroup staged in LDS, one 16-byte non-temporal store per lane step (_words:
//                    small planes of odd width, the chunk rebuilt in LDS word by word first)
//   decompress_units the counterpart of compress_units (odd widths from 512 elements per plane up): four
//                    consecutive elements per lane step, block table made once per workgroup, the next
//                    plane's codes and LFC in flight
// Code widths: 2, 4 and 8 bits in every kernel; 1 bit (four codes of a unit = half a byte) in compress_regs,
// compress_strip, compress_rowstrip, compress_lane, compress_items, compress_units (up to 8 wavefronts), compress_one,
// compress_line, compress_tile, compress_any and in
// every decompress kernel.
// The kernels with a _3d twin take N x C x D x H x W maps with B x B x B blocks (Appendix D).
// Every kernel takes a table of up to 8 maps of one shape (blockIdx.y picks the map).
// Element / cache types: float, bf16_t, f32c16_t (fp32 map, tuple cached as bfloat16).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <stdio.h>
#include <stdlib.h>
#include <atomic>
#include <type_traits>
#include <vector>
#include "../../include/division.h"

// The kernels are instantiated per element / cache type (float, bf16_t, f32c16_t).  To build the
// library in parallel this file can be compiled three times with -DDIVISION_PART=0, 1, 2: each part
// instantiates the kernels of one type behind three bridge functions, part 0 also holds the C ABI.
// Without the macro one translation unit holds everything.
#if !defined(DIVISION_PART)
#define DIVISION_HOST 1
#define DIVISION_HAS_F32 1
#define DIVISION_HAS_BF16 1
#define DIVISION_HAS_C16 1
#else
#define DIVISION_HOST (DIVISION_PART == 0)
#define DIVISION_HAS_F32 (DIVISION_PART == 0)
#define DIVISION_HAS_BF16 (DIVISION_PART == 1)
#define DIVISION_HAS_C16 (DIVISION_PART == 2)
#endif
// launch descriptors travel through the bridges as untyped pointers (their types live in the
// unnamed namespace of each part; the parts are built from this one source, so the layouts agree)
#define DIVISION_BRIDGE __attribute__((visibility("hidden")))
DIVISION_BRIDGE hipError_t division_bridge_compress_f32(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_compress_bf16(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_compress_c16(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_decompress_f32(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_decompress_bf16(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_decompress_c16(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_relu_f32(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_relu_bf16(const void* launch, int b);
DIVISION_BRIDGE hipError_t division_bridge_relu_c16(const void* launch, int b);

namespace {

constexpr int kThreads = 256;              // 4 wavefronts of 64
constexpr uint32_t kLdsTarget = 40u << 10; // preferred LDS bytes per workgroup (4 groups per CU)
constexpr uint32_t kRowsLdsTarget = 40u << 10; // same for compress_rows
constexpr uint32_t kLdsMax = 156u << 10;   // hard limit per workgroup (160 KB per CU)
constexpr uint32_t kWeyl = 0x9E3779B9u;
// Cache policy of the loads of x (the aux operand of the buffer loads: bit 1 = nt).  A kernel whose
// wavefronts read whole contiguous runs, every line once, marks its loads non-temporal: a read-only
// stream of this shape measured 6.4 -> 7.0 TB/s that way, and x no longer displaces the packed
// buffers from the last-level cache.  A kernel whose lanes read rows of a few bytes each
// (compress_items) touches every line several times and needs the default policy: it ran 15 %
// slower with non-temporal loads.
#ifndef DIVISION_LOAD_AUX
#define DIVISION_LOAD_AUX 2
#endif
constexpr int kLoadAux = DIVISION_LOAD_AUX;
constexpr int kLoadReuse = 0;
#ifndef DIVISION_STREAM_K
#define DIVISION_STREAM_K 4
#endif
#ifndef DIVISION_STREAM_STORE_AUX
#define DIVISION_STREAM_STORE_AUX 2
#endif

#include "helpers.h"
#include "compress_tile.h"
#include "compress_wave.h"
#include "compress_items.h"
#include "compress_strip.h"
#include "compress_rowstrip.h"
#include "compress_lane.h"
#include "compress_regs.h"
#include "compress_units.h"
#include "compress_one.h"
#include "compress_rows.h"
#include "compress_plane.h"
#include "compress_any.h"
#include "decompress.h"
#include "host.h"

}  // namespace

// ------------------------------------------------------------------ bridges: the kernels of one type each

#if DIVISION_HAS_F32
hipError_t division_bridge_compress_f32(const void* c, int b) { return do_compress<float>(*static_cast<const CompLaunch*>(c), b); }
hipError_t division_bridge_decompress_f32(const void* c, int b) { return do_decompress<float>(*static_cast<const DecLaunch*>(c), b); }
hipError_t division_bridge_relu_f32(const void* c, int b) { return do_relu<float>(*static_cast<const CompLaunch*>(c), b); }
#endif
#if DIVISION_HAS_BF16
hipError_t division_bridge_compress_bf16(const void* c, int b) { return do_compress<bf16_t>(*static_cast<const CompLaunch*>(c), b); }
hipError_t division_bridge_decompress_bf16(const void* c, int b) { return do_decompress<bf16_t>(*static_cast<const DecLaunch*>(c), b); }
hipError_t division_bridge_relu_bf16(const void* c, int b) { return do_relu<bf16_t>(*static_cast<const CompLaunch*>(c), b); }
#endif
#if DIVISION_HAS_C16
hipError_t division_bridge_compress_c16(const void* c, int b) { return do_compress<f32c16_t>(*static_cast<const CompLaunch*>(c), b); }
hipError_t division_bridge_decompress_c16(const void* c, int b) { return do_decompress<f32c16_t>(*static_cast<const DecLaunch*>(c), b); }
hipError_t division_bridge_relu_c16(const void* c, int b) { return do_relu<f32c16_t>(*static_cast<const CompLaunch*>(c), b); }
#endif

// ------------------------------------------------------------------ C ABI

#if DIVISION_HOST
extern "C" {

int division_abi_version(void) { return 1; }

size_t division_packed_bytes(int64_t N, int64_t C, int64_t H, int64_t W, int B, int b, division_dtype dt) {
    Layout L;
    if (make_layout(N, C, 1, H, W, B, b, (int)dt, &L) != DIVISION_OK) return 0;
    return L.total;
}

size_t division_packed_bytes_3d(int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int B, int b, division_dtype dt) {
    Layout L;
    if (make_layout(N, C, D, H, W, B, b, (int)dt, &L) != DIVISION_OK) return 0;
    return L.total;
}

int division_packed_layout(int64_t N, int64_t C, int64_t H, int64_t W, int B, int b, division_dtype dt,
                           size_t* codes_off, size_t* codes_bytes, size_t* meta_off, size_t* meta_bytes,
                           size_t* lfc_off, size_t* lfc_bytes) {
    return packed_layout_impl(N, C, 1, H, W, B, b, dt, codes_off, codes_bytes, meta_off, meta_bytes, lfc_off, lfc_bytes);
}

int division_packed_layout_3d(int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int B, int b, division_dtype dt,
                              size_t* codes_off, size_t* codes_bytes, size_t* meta_off, size_t* meta_bytes,
                              size_t* lfc_off, size_t* lfc_bytes) {
    return packed_layout_impl(N, C, D, H, W, B, b, dt, codes_off, codes_bytes, meta_off, meta_bytes, lfc_off, lfc_bytes);
}

int division_compress_batch(int count, const void* const* x, void* const* packed, const uint64_t* seeds,
                            int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt,
                            int B, int b, size_t packed_capacity, void* hip_stream) {
    return compress_impl(count, x, packed, seeds, N, C, 1, H, W, dt, B, b, packed_capacity, hip_stream);
}

int division_compress(const void* x, int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt,
                      int B, int b, uint64_t seed, void* packed, size_t packed_capacity, void* hip_stream) {
    if (!x || !packed) return DIVISION_EINVAL;
    return compress_impl(1, &x, &packed, &seed, N, C, 1, H, W, dt, B, b, packed_capacity, hip_stream);
}

int division_compress_3d(const void* x, int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, division_dtype dt,
                         int B, int b, uint64_t seed, void* packed, size_t packed_capacity, void* hip_stream) {
    if (!x || !packed) return DIVISION_EINVAL;
    return compress_impl(1, &x, &packed, &seed, N, C, D, H, W, dt, B, b, packed_capacity, hip_stream);
}

int division_decompress_batch(int count, const void* const* packed, void* const* xhat, size_t packed_bytes,
                              int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt,
                              int B, int b, void* hip_stream) {
    return decompress_impl(count, packed, xhat, packed_bytes, N, C, 1, H, W, dt, B, b, hip_stream);
}

int division_decompress(const void* packed, size_t packed_bytes, int64_t N, int64_t C, int64_t H, int64_t W,
                        division_dtype dt, int B, int b, void* xhat, void* hip_stream) {
    if (!xhat || !packed) return DIVISION_EINVAL;
    return decompress_impl(1, &packed, &xhat, packed_bytes, N, C, 1, H, W, dt, B, b, hip_stream);
}

int division_decompress_3d(const void* packed, size_t packed_bytes, int64_t N, int64_t C, int64_t D, int64_t H, int64_t W,
                           division_dtype dt, int B, int b, void* xhat, void* hip_stream) {
    if (!xhat || !packed) return DIVISION_EINVAL;
    return decompress_impl(1, &packed, &xhat, packed_bytes, N, C, D, H, W, dt, B, b, hip_stream);
}

int division_relu_compress(const void* x, int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt,
                           int B, int b, uint64_t seed, void* y, void* mask, size_t mask_capacity,
                           void* packed, size_t packed_capacity, void* hip_stream) {
    if (!x || !y || !mask || !packed) return DIVISION_EINVAL;
    Layout L;
    const int rc = make_layout(N, C, 1, H, W, B, b, (int)dt, &L);
    if (rc != DIVISION_OK) return rc;
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    const int64_t n = (int64_t)(L.P * L.HW);
    if (mask_capacity < division_mask_bytes(n) || packed_capacity < L.total) return DIVISION_ESIZE;
    if (((uintptr_t)x % es) != 0 || ((uintptr_t)y % es) != 0 || ((uintptr_t)mask % 4) != 0 || ((uintptr_t)packed % 16) != 0)
        return DIVISION_EALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    // fused: the planes the register kernel takes, when a plane's mask is whole words
    RegsArgs ra{};
    uint32_t grid = 0;
    size_t lds = 0;
    int nw = 1;
    const void* both = reinterpret_cast<const void*>((uintptr_t)x | (uintptr_t)y);
    if (b != 1 && L.HW % 32 == 0 && (B == 4 || B == 8) && plan_regs(L, 1, H, W, B, es, both, &ra, &grid, &lds, &nw) && nw <= 4) {
        ra.tab.x[0] = x;
        ra.tab.pk[0] = packed;
        ra.tab.seed_a[0] = mix32((uint32_t)(seed & 0xffffffffu) ^ 0x243F6A88u);
        ra.tab.seed_c[0] = mix32((uint32_t)(seed >> 32) ^ 0x85A308D3u);
        ra.rg = make_regions(L);
        ra.y = y;
        ra.mask = static_cast<uint32_t*>(mask);
        CompLaunch c{};
        c.kind = REGS; c.B = B; c.nw = nw; c.gx = grid; c.gy = 1; c.lds = lds; c.st = st; c.ra = ra;
        const hipError_t err = bridge_relu(dt, c, b);
        return err == hipSuccess ? DIVISION_OK : DIVISION_EHIP;
    }
    // fused too: the 28- and 14-wide planes of the strip kernel
    StripArgs sa{};
    int vec = 1;
    const int Bc = covering_block(L, 1, H, W, B);
    if (b != 1 && plan_relu_strip(L, H, W, Bc, es, both, &sa, &grid, &lds, &vec)) {
        sa.tab.x[0] = x;
        sa.tab.pk[0] = packed;
        sa.tab.seed_a[0] = mix32((uint32_t)(seed & 0xffffffffu) ^ 0x243F6A88u);
        sa.tab.seed_c[0] = mix32((uint32_t)(seed >> 32) ^ 0x85A308D3u);
        sa.rg = make_regions(L);
        sa.y = y;
        sa.mask = static_cast<uint32_t*>(mask);
        CompLaunch c{};
        c.kind = STRIP; c.B = Bc; c.vec = vec; c.gx = grid; c.gy = 1; c.lds = lds; c.st = st; c.sa = sa;
        const hipError_t err = bridge_relu(dt, c, b);
        return err == hipSuccess ? DIVISION_OK : DIVISION_EHIP;
    }
    // and the other small planes of the items kernel (the CIFAR shapes)
    ItemsArgs ia{};
    if (b != 1 && (Bc == 4 || Bc == 8) && plan_relu_items(L, H, W, Bc, es, both, &ia, &grid, &lds, &vec)) {
        ia.tab.x[0] = x;
        ia.tab.pk[0] = packed;
        ia.tab.seed_a[0] = mix32((uint32_t)(seed & 0xffffffffu) ^ 0x243F6A88u);
        ia.tab.seed_c[0] = mix32((uint32_t)(seed >> 32) ^ 0x85A308D3u);
        ia.rg = make_regions(L);
        ia.y = y;
        ia.mask = static_cast<uint32_t*>(mask);
        CompLaunch c{};
        c.kind = ITEMS; c.B = Bc; c.vec = vec; c.gx = grid; c.gy = 1; c.lds = lds; c.st = st; c.ia = ia;
        const hipError_t err = bridge_relu(dt, c, b);
        return err == hipSuccess ? DIVISION_OK : DIVISION_EHIP;
    }
    // other shapes: the operator, then the codec on its output
    const int r1 = division_relu_forward(x, n, dt == DIVISION_F32_C16 ? DIVISION_F32 : dt, y, mask, mask_capacity, hip_stream);
    if (r1 != DIVISION_OK) return r1;
    const void* yin = y;
    return compress_impl(1, &yin, &packed, &seed, N, C, 1, H, W, dt, B, b, packed_capacity, hip_stream);
}

int division_relu_compress_fused(int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt, int B, int b) {
    Layout L;
    if (make_layout(N, C, 1, H, W, B, b, (int)dt, &L) != DIVISION_OK || b == 1) return 0;
    RegsArgs ra{};
    uint32_t grid = 0;
    size_t lds = 0;
    int nw = 1;
    const size_t es = dt == DIVISION_BF16 ? 2 : 4;
    const void* aligned = reinterpret_cast<const void*>((uintptr_t)16);
    if (L.HW % 32 == 0 && (B == 4 || B == 8) && plan_regs(L, 1, H, W, B, es, aligned, &ra, &grid, &lds, &nw) && nw <= 4) return 1;
    StripArgs sa{};
    int vec = 1;
    const int Bc = covering_block(L, 1, H, W, B);
    if (plan_relu_strip(L, H, W, Bc, es, aligned, &sa, &grid, &lds, &vec)) return 1;
    ItemsArgs ia{};
    return (Bc == 4 || Bc == 8) && plan_relu_items(L, H, W, Bc, es, aligned, &ia, &grid, &lds, &vec);
}

// Both directions of the descriptor-array calls: validates every map, then serves the maps that
// share a shape and parameters together, in order of first appearance.
static int run_maps(int count, const division_map* maps, void* hip_stream, bool compress) {
    if (count < 0 || (count > 0 && !maps)) return DIVISION_EINVAL;
    for (int i = 0; i < count; ++i) {
        const division_map& m = maps[i];
        Layout L;
        const int rc = make_layout(m.N, m.C, m.D, m.H, m.W, m.B, m.b, (int)m.dt, &L);
        if (rc != DIVISION_OK) return rc;
        if (!m.packed || (compress ? !m.x : !m.xhat)) return DIVISION_EINVAL;
        if (m.packed_bytes < L.total) return DIVISION_ESIZE;
        const size_t es = m.dt == DIVISION_BF16 ? 2 : 4;
        const void* data = compress ? m.x : m.xhat;
        if (((uintptr_t)data % es) != 0 || ((uintptr_t)m.packed % 16) != 0) return DIVISION_EALIGN;
    }
    auto same = [](const division_map& p, const division_map& q) {
        return p.N == q.N && p.C == q.C && p.D == q.D && p.H == q.H && p.W == q.W && p.dt == q.dt && p.B == q.B && p.b == q.b;
    };
    std::vector<char> done((size_t)count, 0);
    std::vector<const void*> in;
    std::vector<void*> out;
    std::vector<uint64_t> seeds;
    for (int i = 0; i < count; ++i) {
        if (done[(size_t)i]) continue;
        in.clear(); out.clear(); seeds.clear();
        size_t cap = ~(size_t)0;
        for (int j = i; j < count; ++j) {
            if (done[(size_t)j] || !same(maps[i], maps[j])) continue;
            done[(size_t)j] = 1;
            in.push_back(compress ? maps[j].x : maps[j].packed);
            out.push_back(compress ? maps[j].packed : maps[j].xhat);
            seeds.push_back(maps[j].seed);
            if (maps[j].packed_bytes < cap) cap = maps[j].packed_bytes;
        }
        const division_map& m = maps[i];
        const int rc = compress
            ? compress_impl((int)in.size(), in.data(), out.data(), seeds.data(), m.N, m.C, m.D, m.H, m.W, m.dt, m.B, m.b, cap, hip_stream)
            : decompress_impl((int)in.size(), in.data(), out.data(), cap, m.N, m.C, m.D, m.H, m.W, m.dt, m.B, m.b, hip_stream);
        if (rc != DIVISION_OK) return rc;
    }
    return DIVISION_OK;
}

int division_compress_maps(int count, const division_map* maps, void* hip_stream) {
    return run_maps(count, maps, hip_stream, true);
}

int division_decompress_maps(int count, const division_map* maps, void* hip_stream) {
    return run_maps(count, maps, hip_stream, false);
}

int division_kernel_name(int direction, const void* data, int64_t N, int64_t C, int64_t H, int64_t W,
                         division_dtype dt, int B, int b, char* out, size_t cap) {
    return kernel_name_impl(direction, data, N, C, 1, H, W, dt, B, b, out, cap);
}

float division_block_mean_rule(double block_sum, uint32_t count, int* divided) {
    int d = 0;
    const float m = count ? mean_of_host(block_sum, count, &d) : 0.0f;
    if (divided) *divided = d;
    return m;
}

int division_kernel_name_3d(int direction, const void* data, int64_t N, int64_t C, int64_t D, int64_t H, int64_t W,
                            division_dtype dt, int B, int b, char* out, size_t cap) {
    return kernel_name_impl(direction, data, N, C, D, H, W, dt, B, b, out, cap);
}

}  // extern "C"
#endif  // DIVISION_HOST
