/*
 * division.h -- C ABI of the DIVISION activation codec for AMD MI355X (gfx950).
 *
 * The codec is the per-layer hot path of "DIVISION: Memory Efficient Training
 * via Dual Activation Precision": in the forward pass every cached activation
 * map H (NCHW) is replaced by the tuple (H^L, V^H, Delta, delta) of Sec. 4.1,
 * in the backward pass the map is rebuilt from that tuple as in Sec. 4.2.
 *
 * All tensor pointers are DEVICE pointers (HIP global memory) unless a
 * comment says "host".  The library allocates nothing, keeps no state between
 * calls that any result depends on (it remembers the compute-unit count of each
 * device it has seen and which kernels it has allowed a large LDS footprint),
 * and never synchronises: every kernel is enqueued on the caller's stream and
 * the call returns at once.  Calls act on the current device of the calling
 * thread.  Buffers stay owned by the caller and
 * must remain valid until the stream has passed the call.
 *
 * Packed buffer layout (little endian; P = N*C planes, one plane = one
 * (sample, channel) map of H*W elements; LH = ceil(H/B), LW = ceil(W/B);
 * CPW = 32/b codes per word; WPP = ceil(H*W/CPW) words per plane):
 *
 *   codes  at byte 0                      uint32 [P][WPP]
 *          element i = r*W + c of a plane sits in word i / CPW at bit
 *          (i % CPW) * b; pad bits are zero.
 *   meta   at align16(end of codes)       float  [P][2] = (delta_p, Delta_p)
 *          (DIVISION_F32_C16: bfloat16 [P][2])
 *   lfc    at align16(end of meta)        T      [P][LH][LW], T = element type
 *          (DIVISION_F32_C16: bfloat16)
 *   total  = align16(end of lfc)          == division_packed_bytes(...)
 */
#ifndef DIVISION_H
#define DIVISION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Element type of x and of the reconstructed map, and how the tuple is cached:
 *   DIVISION_F32      x fp32;  H^L fp32, (delta, Delta) fp32
 *   DIVISION_BF16     x bf16;  H^L bf16, (delta, Delta) fp32
 *   DIVISION_F32_C16  x fp32;  H^L, delta and Delta cached as bfloat16: the format of Sec. 4.1
 *                     (N^2 Q/8 + 4 bytes per channel for V^H, delta, Delta; H^L 0.8 % of the map
 *                     at B = 8).  delta is the plane minimum rounded DOWN to bfloat16 and Delta
 *                     is fl(fl(max - delta)/L) rounded UP, so that the cached values bracket every
 *                     residual and the quantiser uses exactly what the decoder reads.
 * (The mask operators below take DIVISION_F32 or DIVISION_BF16 only.)
 */
typedef enum { DIVISION_F32 = 0, DIVISION_BF16 = 1, DIVISION_F32_C16 = 2 } division_dtype;

/* Return codes of every int-returning entry point. */
enum {
    DIVISION_OK     = 0,
    DIVISION_EINVAL = 1,  /* null pointer, N/C/H/W <= 0, B < 1, b not in {1,2,4,8}, unknown dtype */
    DIVISION_ESIZE  = 2,  /* packed buffer smaller than division_packed_bytes(...)             */
    DIVISION_EALIGN = 3,  /* x / xhat not aligned to the element size, packed not to 16 bytes  */
    DIVISION_ERANGE = 4,  /* N*C or H*W above 2^31-1, or N*C*H*W above 2^40                    */
    DIVISION_EHIP   = 5   /* a kernel launch failed; hipGetLastError() holds the detail        */
};

/*
 * Size in bytes of the cached tuple (H^L, V^H, Delta, delta) of one NCHW map
 * (Sec. 4.1, last paragraph; the paper's per-channel accounting N^2 Q/8 + 4
 * bytes plus the pooled map, here with fp32 (delta, Delta) and word-padded
 * codes).  Host-only arithmetic; returns 0 for invalid arguments.
 */
size_t division_packed_bytes(int64_t N, int64_t C, int64_t H, int64_t W,
                             int B, int b, division_dtype dt);

/*
 * Byte offset and size of the three regions of the packed buffer, i.e. of the
 * members of the cached tuple of Sec. 4.1 (last paragraph): codes = V^H packed
 * at b bits (the N^2 Q/8 bytes per channel of that passage, padded to whole
 * words), meta = (delta, Delta) of Eq. (quantization) per plane, lfc = H^L,
 * the pooled map of ceil(H/B) x ceil(W/B) means per plane (Appendix D gives
 * the pooled shape for B | N; the border windows are the footnote's N < B
 * rule applied per edge).  The layout itself is stated at the top of this
 * file.  Host-only; out pointers are host pointers, none may be null.
 * Returns DIVISION_OK or DIVISION_EINVAL.
 */
int division_packed_layout(int64_t N, int64_t C, int64_t H, int64_t W,
                           int B, int b, division_dtype dt,
                           size_t *codes_off, size_t *codes_bytes,
                           size_t *meta_off, size_t *meta_bytes,
                           size_t *lfc_off, size_t *lfc_bytes);

/*
 * Forward-pass compression (Sec. 4.1; Algorithm 1, the four steps after the
 * layer's forward: AveragePooling, residual against UpSampling, Quant, Cache).
 *
 *   x       device, read only, N*C*H*W elements of type dt, dense NCHW.
 *   B       pooling window = stride (the paper's block size B), >= 1.  Maps
 *           smaller than B are pooled to 1x1 (footnote of Sec. 4.1); when B
 *           does not divide H or W the border windows average their valid
 *           elements only.
 *   b       bits per HFC code (the paper's Q): 1, 2, 4 or 8.  2, 4 and 8 have fast compress kernels
 *           for every shape; 1 has them under B = 4 and 8 (and for the ResNet-50, CIFAR and token
 *           maps under any B) and is compressed by the general kernel (slow) for other block sizes on
 *           small planes, planes beyond LDS and small 3-D maps.  Decompression is fast for every b.
 *   seed    selects the stochastic-rounding stream of Eq. (quantization); the
 *           output is a pure function of (x, shape, dt, B, b, seed) and does
 *           not depend on the launch geometry or the device.
 *   packed  device, written in full (pad bits and pad bytes zero), at least
 *           division_packed_bytes(...) bytes, 16-byte aligned; must not
 *           overlap x.
 *   hip_stream  a hipStream_t passed as void* (NULL = the default stream).
 *
 * Per plane: H^L = block means (stored in type dt); H^H = x - nearest
 * up-sampling of the stored H^L; delta = min H^H, Delta = (max H^H - delta) /
 * (2^b - 1); code = floor(t + u) with t = (H^H - delta) * (2^b - 1)/(max-delta)
 * and u uniform in [0,1) with 16 random bits per element.  A plane whose
 * residual range is below 2^-90 (or beyond the largest binary32) gets Delta = 0
 * and all-zero codes.  Zeros keep a sign: a block of -0 has mean +0, and the
 * minimum of residuals +0 and -0 is -0 (the order of IEEE 754 minimum), so the
 * stored bytes do not depend on where in a plane a zero stands.  Subnormal
 * inputs and means are kept, not flushed.
 * NaN or infinite inputs give unspecified codes (no error is raised).
 */
int division_compress(const void *x, int64_t N, int64_t C, int64_t H, int64_t W,
                      division_dtype dt, int B, int b, uint64_t seed,
                      void *packed, size_t packed_capacity, void *hip_stream);

/*
 * Backward-pass decompression (Sec. 4.2 and the reconstruction equation;
 * Algorithm 1, the Dequant and UpSampling+add steps):
 *   xhat = UpSampling(H^L) + (Delta * V^H + delta), rounded to type dt.
 *
 *   packed  device, read only, as written by division_compress with the same
 *           (N, C, H, W, dt, B, b); packed_bytes is the size of that buffer.
 *   xhat    device, N*C*H*W elements of type dt, written in full; must not
 *           overlap packed.
 */
int division_decompress(const void *packed, size_t packed_bytes,
                        int64_t N, int64_t C, int64_t H, int64_t W,
                        division_dtype dt, int B, int b,
                        void *xhat, void *hip_stream);

/*
 * The same two operations over `count` maps of ONE shape (Algorithm 1 runs the
 * forward-pass compression once per layer and the backward-pass decompression
 * once per layer; layers whose maps share (N, C, H, W, dt, B, b) can be served
 * together).  Tensor i gives exactly the bytes that the single-map call with
 * (x[i], seeds[i], packed[i]) resp. (packed[i], xhat[i]) gives; up to 8 maps
 * share one kernel launch, so the machine is filled and drained once for all
 * of them.
 *
 *   x, packed, xhat   HOST arrays of `count` DEVICE pointers, read during the
 *                     call only; the same requirements as above hold for every
 *                     pointed-to buffer, and no two output buffers may overlap.
 *   seeds             HOST array of `count` seeds.
 *   packed_capacity / packed_bytes   size of EACH packed buffer.
 *
 * count == 0 is a no-op (DIVISION_OK); count < 0 or a null array or a null
 * entry is DIVISION_EINVAL.  Arguments are checked for the whole batch before
 * anything is launched.
 */
int division_compress_batch(int count, const void *const *x, void *const *packed,
                            const uint64_t *seeds,
                            int64_t N, int64_t C, int64_t H, int64_t W,
                            division_dtype dt, int B, int b,
                            size_t packed_capacity, void *hip_stream);

int division_decompress_batch(int count, const void *const *packed, void *const *xhat,
                              size_t packed_bytes,
                              int64_t N, int64_t C, int64_t H, int64_t W,
                              division_dtype dt, int B, int b, void *hip_stream);

/*
 * 1-bit masks of the Relu and Dropout operators (appendix on operator
 * compression; Algorithms "Relu operator" and "Dropout operator"): the forward
 * pass caches V, one bit per element (N^2/8 bytes per channel), instead of the
 * activation; the backward pass needs nothing else.
 *
 * Mask layout: bit i%32 of the 32-bit word i/32 holds V of element i (flat
 * index, any tensor shape); pad bits of the last word are zero.
 * division_mask_bytes(n) = 4*ceil(n/32) (host-only; 0 for n < 0).
 *
 *   x, y, grad_out, grad_in   device, n elements of type dt, aligned to the
 *           element size (16-byte alignment of both buffers of a call enables
 *           the fast path).  y may be x itself and grad_in may be grad_out
 *           itself (in place); other overlaps are not allowed.
 *   mask    device, 4-byte aligned, at least division_mask_bytes(n) bytes;
 *           written in full by the forward calls, read by the backward call.
 *
 * division_relu_forward:    V = sgn(x) (1 where x > 0), y = V (.) x.
 * division_dropout_forward: V ~ Bernoulli(1 - p) element-wise, y = V (.) x, no
 *           rescaling (as in the listing; fold 1/(1-p) into a neighbouring
 *           layer).  V is a pure function of (n, p, seed): element i is kept
 *           iff its 16 random bits are >= floor(p*65536 + 0.5).
 * division_mask_backward:   grad_in = V (.) grad_out (both operators).
 * Where V = 0 the result is +0 whatever the operand.  Values pass through bit
 * for bit.  n == 0 is a no-op (the pointers may then be null).  Errors as above (EINVAL, ESIZE, EALIGN,
 * ERANGE for n > 2^40, EHIP).
 */
size_t division_mask_bytes(int64_t n);

int division_relu_forward(const void *x, int64_t n, division_dtype dt,
                          void *y, void *mask, size_t mask_capacity, void *hip_stream);

int division_dropout_forward(const void *x, int64_t n, division_dtype dt, float p, uint64_t seed,
                             void *y, void *mask, size_t mask_capacity, void *hip_stream);

int division_mask_backward(const void *mask, size_t mask_bytes, const void *grad_out, int64_t n,
                           division_dtype dt, void *grad_in, void *hip_stream);

/*
 * Max-Pooling layer with kernel size = stride = k (appendix on operator
 * compression, Algorithm "Max-Pooling layer"): the forward pass returns the
 * pooled map and caches V, which marks where each window's maximum sits in the
 * input, one bit per INPUT element (layout as above, flat NCHW index); the
 * backward pass is grad_in = V (.) (1_{k x k} (x) grad_out).
 *
 *   x, grad_in   device, N*C*H*W elements of type dt.
 *   y, grad_out  device, N*C*floor(H/k)*floor(W/k) elements; rows and columns
 *                past the last whole window belong to no window (V = 0 there,
 *                zero gradient).  No buffer may overlap another.
 *   mask         device, 4-byte aligned, division_mask_bytes(N*C*H*W) bytes.
 * Exactly one element per window is marked: the first maximum in row-major
 * order inside the window.  Values pass through bit for bit; where V = 0 the
 * gradient is +0.  k*W above 65536, N*C or H*W above 2^31-1 or N*C*H*W above
 * 2^40 give DIVISION_ERANGE.
 */
int division_maxpool_forward(const void *x, int64_t N, int64_t C, int64_t H, int64_t W,
                             division_dtype dt, int k, void *y, void *mask, size_t mask_capacity,
                             void *hip_stream);

int division_maxpool_backward(const void *mask, size_t mask_bytes, const void *grad_out,
                              int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt, int k,
                              void *grad_in, void *hip_stream);

/*
 * Profiling aid (host-only): writes the name of the kernel template instance
 * that division_compress (direction 0, data = x) or division_decompress
 * (direction 1, data = xhat) would launch for these arguments, as it appears
 * in a kernel trace, e.g. "compress_tile<float, 2, 8, 4>".  The choice depends
 * on the shape, the block size and the 16-byte alignment of `data` (which may
 * be null: treated as aligned).  out is a host buffer of cap bytes.
 * Returns DIVISION_OK, or DIVISION_ESIZE when cap is too small.
 */
int division_kernel_name(int direction, const void *data,
                         int64_t N, int64_t C, int64_t H, int64_t W,
                         division_dtype dt, int B, int b, char *out, size_t cap);

/*
 * 3-D activation maps (Appendix D: AveragePooling3D / UpSampling3D, the Quant of
 * Eq. (quantization) unchanged).  x is an N x C x D x H x W tensor, contiguous in
 * that order; a plane is the D*H*W elements of one (sample, channel) pair, the
 * blocks are B x B x B (clipped at the far faces, ceil(D/B) x ceil(H/B) x
 * ceil(W/B) of them, stored in that order), element i of a plane is its
 * row-major index ((d*H + h)*W + w) for the code position and the random
 * numbers.  The packed buffer has the layout of the 2-D one with HW = D*H*W
 * and the block count above.  D = 1 gives exactly the 2-D calls; so does a
 * volume with H = 1 or W = 1 (D x W resp. D x H maps).  Pointers, alignment,
 * ownership, stream and error codes as for division_compress /
 * division_decompress; D*H and D*H*W above 2^31-1 give DIVISION_ERANGE.
 */
size_t division_packed_bytes_3d(int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int B, int b,
                                division_dtype dt);

int division_packed_layout_3d(int64_t N, int64_t C, int64_t D, int64_t H, int64_t W, int B, int b,
                              division_dtype dt, size_t *codes_off, size_t *codes_bytes, size_t *meta_off,
                              size_t *meta_bytes, size_t *lfc_off, size_t *lfc_bytes);

int division_compress_3d(const void *x, int64_t N, int64_t C, int64_t D, int64_t H, int64_t W,
                         division_dtype dt, int B, int b, uint64_t seed, void *packed,
                         size_t packed_capacity, void *hip_stream);

int division_decompress_3d(const void *packed, size_t packed_bytes, int64_t N, int64_t C, int64_t D,
                           int64_t H, int64_t W, division_dtype dt, int B, int b, void *xhat,
                           void *hip_stream);

/*
 * The Relu operator fused with the compression of its output (a conv-BN-Relu block caches the
 * Relu's 1-bit mask for the Relu's own backward pass and the Relu's output, compressed, for the
 * next layer's: Appendix, Relu listing, and Sec. 4.1).  Equivalent to division_relu_forward(x -> y,
 * mask) followed by division_compress(y -> packed), with the same outputs bit for bit; for the
 * shapes division_relu_compress_fused reports (B = 4 or 8, 16-byte aligned x and y; planes of
 * 2048-3328 or 8192-13312 elements in whole 32-element mask words, the 28- / 32-wide planes of
 * at most 32 rows and the 14- / 16-wide ones of at most 16 under B = 8 (32, 16: also B = 4), and
 * the other small planes of at most 64 pooling items of B rows by 2 or 4 columns) one kernel does both and y does not travel through HBM a second time.  Other shapes run the two
 * kernels one after the other.  y may be x itself (in place); arguments as for the two calls it replaces.
 */
int division_relu_compress(const void *x, int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt,
                           int B, int b, uint64_t seed, void *y, void *mask, size_t mask_capacity,
                           void *packed, size_t packed_capacity, void *hip_stream);

/* 1 when division_relu_compress runs as one kernel for this shape (aligned pointers assumed), else 0
 * (host-only). */
int division_relu_compress_fused(int64_t N, int64_t C, int64_t H, int64_t W, division_dtype dt, int B, int b);

/*
 * A whole step in one call: the maps a forward (backward) pass caches (rebuilds), of any mix of
 * shapes, element types, block sizes and code widths (Algorithm 1 loops over the layers; this
 * call takes the loop's maps as an array of descriptors).  Map i gives exactly the bytes the
 * single-map call with its fields gives.  Maps that agree in (N, C, D, H, W, dt, B, b) are
 * served together, up to 8 per kernel launch, in the order of their first appearance.
 *
 *   maps   HOST array of `count` descriptors, read during the call only.
 *          x       device, the map (compress only; ignored by decompress)
 *          packed  device, the cached tuple: written by compress (capacity
 *                  packed_bytes), read by decompress (size packed_bytes)
 *          xhat    device, the rebuilt map (decompress only; ignored by compress)
 *          D       depth of a 3-D map, 1 for 2-D and 1-D maps
 *          seed    stochastic-rounding stream of the map (compress only)
 *
 * All descriptors are checked before anything is launched; the first invalid one decides the
 * error code.  count == 0 is a no-op; count < 0 or maps == NULL with count > 0 is DIVISION_EINVAL.
 */
typedef struct division_map {
    const void *x;
    void *packed;
    void *xhat;
    size_t packed_bytes;
    int64_t N, C, D, H, W;
    division_dtype dt;
    int B, b;
    uint64_t seed;
} division_map;

int division_compress_maps(int count, const division_map *maps, void *hip_stream);

int division_decompress_maps(int count, const division_map *maps, void *hip_stream);

/* division_kernel_name for the 3-D calls. */
int division_kernel_name_3d(int direction, const void *data, int64_t N, int64_t C, int64_t D, int64_t H,
                            int64_t W, division_dtype dt, int B, int b, char *out, size_t cap);

/*
 * Test aid (host-only, no GPU needed): the block mean of Sec. 4.1 (AveragePooling) as the compress
 * kernels evaluate it.  The definition is (float)(block_sum / count): the exact sum of the block's
 * elements, held in binary64, divided in binary64, rounded once to binary32.  The kernels multiply
 * by the reciprocal of count instead and fall back to the division when the product lies close to
 * a rounding boundary of binary32 or below the smallest normal binary32; this function runs that
 * very rule (same source) on the host, so that it can be checked against the definition for every
 * count.  *divided (may be null) receives 1 when the division was taken.  count == 0 returns 0.
 */
float division_block_mean_rule(double block_sum, uint32_t count, int *divided);

/* Version of this ABI (host-only). */
int division_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DIVISION_H */
