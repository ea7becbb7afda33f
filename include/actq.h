/*
 * actq.h -- C ABI of libactq: per-group stochastic quantization of saved
 * activations for activation-compressed training (ActNN, arXiv 2104.14129),
 * written for one AMD MI355X (gfx950).
 *
 * The tensor is viewed as N samples x D features, sample-major and contiguous
 * (Sec. 4.1: an activation H in R^{N x D}).  Each sample is cut into
 * ng = ceil(D / G) groups of G consecutive features; groups never cross a
 * sample, because the bit-width b_n is a per-sample quantity (Sec. 4.2).  The
 * last group of a sample may be ragged when G does not divide D.
 *
 * Conventions shared by every call
 *   - Return value: 0 (ACTQ_OK) or a negative actq_status.  A human-readable
 *     text for the last failure on the calling thread is returned by
 *     actq_last_error().
 *   - "device" pointers are HIP device memory, "host" pointers ordinary memory.
 *     The caller owns every buffer; the library allocates nothing, keeps no
 *     state between calls and never frees or retains a pointer.
 *   - Device calls are asynchronous on the HIP stream passed as `stream`
 *     (a hipStream_t cast to void*, NULL = the default stream) and never
 *     synchronise.  All argument validation happens on the host before any
 *     launch; a call that fails validation launches nothing.
 *   - Inputs must be finite.  Non-finite inputs are memory-safe but the codes
 *     they produce are unspecified.
 *   - Supported group size: G = 256.  Supported widths: every b_n from 1 to 8.
 *   - x / out must be aligned to 16 bytes, packed to 16 bytes, header and offsets to 8,
 *     bits (device) to 4.
 */
#ifndef ACTQ_H
#define ACTQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum actq_status {
    ACTQ_OK = 0,
    ACTQ_EINVAL = -1,      /* bad argument (null, size, alignment, G, dtype, bits) */
    ACTQ_EINFEASIBLE = -2, /* allocate_bits: budget below the narrowest allowed width */
    ACTQ_EHIP = -3         /* the HIP runtime refused the launch                   */
} actq_status;

typedef enum actq_dtype {
    ACTQ_F32 = 0, /* IEEE binary32 */
    ACTQ_F16 = 1  /* IEEE binary16; widened exactly to binary32 before any arithmetic */
} actq_dtype;

/* Per-group header kept beside the codes. */
typedef enum actq_header_format {
    ACTQ_HDR_F32 = 0, /* (Z, R/B) in binary32: 8 bytes per group, 0.25 bit per element at G = 256 */
    ACTQ_HDR_BF16 = 1, /* (Z, R) in bfloat16 as in Sec. 4.1: 4 bytes per group, 0.125 bit per
                         element.  Z is rounded down to bfloat16 and R = max - Z is rounded up, so
                         every element still scales into [0, B]; a degenerate group stores R = 0 */
    ACTQ_HDR_TENSOR = 2 /* one pair (Z, R) in binary32 for the whole tensor, 8 bytes in all: the
                           per-tensor baseline the paper compares with (Sec. 4.1, Sec. 6.1).  The
                           pair is an INPUT of actq_quantize_pack, written beforehand by
                           actq_tensor_stats (or by the caller: it must cover every element) */
} actq_header_format;

/* Library version, major*10000 + minor*100 + patch. */
int actq_version(void);

/* Hex digest of the sources and build flags this binary was compiled from (set by the build
 * script; "unknown" for a hand build).  The Python binding compares it with the digest of the
 * sources beside it, so that an edited kernel is never tested against a stale binary.  The
 * pointer is to static storage. */
const char* actq_source_hash(void);

/* Text of the last error raised on this thread ("" if none).  The pointer stays
 * valid until the next failing call on the same thread. */
const char* actq_last_error(void);

/*
 * Size of the compressed store (the "bit stream" of Sec. 5.1; the layout is
 * this library's, the paper does not give one).
 *
 * Sample n occupies ng * G * b_n / 8 bytes starting at byte
 * offsets_host[n] = sum_{m<n} ng * G * b_m / 8; *total_host receives the sum
 * over all samples.  Inside a sample, group g starts at g * G * b_n / 8 and the
 * code of in-group element j occupies bits [j*b_n, j*b_n + b_n) of the group's
 * stream, where stream bit k is bit (k mod 8) of byte floor(k / 8): an LSB-first
 * linear bit stream.  A code whose width does not divide 8 may straddle two
 * bytes; a group always ends on a byte (32*b_n bytes).  The padding codes of a
 * ragged last group are zero.
 *
 * bits_host [N]    host, in   : b_n in 1..8
 * offsets_host [N] host, out  : may be NULL when only the total is wanted
 * total_host       host, out  : may be NULL
 * Errors: ACTQ_EINVAL on N <= 0, D <= 0, unsupported G, a width outside
 * 1..8, or both outputs NULL.
 */
int actq_packed_bytes(int64_t N, int64_t D, int32_t G, const uint8_t* bits_host,
                      uint64_t* offsets_host, uint64_t* total_host);

/* Bytes of the header for N*ng groups in format hf (host arithmetic only; 8 for ACTQ_HDR_TENSOR). */
int actq_header_bytes(int64_t N, int64_t D, int32_t G, actq_header_format hf, uint64_t* bytes_host);

/*
 * Per-group zero point Z = min and range R = max - min (Sec. 4.1).
 *
 * x      device, in  : N*D elements of dtype `dt`
 * gmin   device, out : [N*ng] float, Z of every group; -0.0 is stored as +0.0
 * grange device, out : [N*ng] float, R = max - min rounded to nearest; a zero range is +0.0
 * Only the valid elements of a ragged group take part.
 * Errors: ACTQ_EINVAL on a null or misaligned pointer, N or D out of range
 * (N < 2^32, D < 2^34), unsupported G or dtype; ACTQ_EHIP if the launch fails.
 */
int actq_group_stats(const void* x, actq_dtype dt, int64_t N, int64_t D, int32_t G,
                     float* gmin, float* grange, void* stream);

/*
 * Forward pass: scale, round stochastically, pack (Sec. 4.1, Sec. 5.1), in one
 * pass over x.
 *
 * For a group with zero point Z and range R and a sample with b bits,
 * B = 2^b - 1:  inv = B / R,  scale = R / B  (binary32, round to nearest);
 * a group whose R is zero, or whose B / R overflows, has inv = scale = 0.
 * For every element: u = min((x - Z) * inv, B), two separately rounded
 * binary32 operations, then stochastic rounding (ceil(u) with probability
 * u - floor(u), floor(u) otherwise) driven by uniform noise from Philox4x32-10
 * (Salmon et al., SC'11) keyed by `seed`, so a call is exactly reproducible.
 * With d the feature index inside sample n:
 *   noise_bits = 24: counter (d>>2, n, lo32(tag), hi32(tag)), element d takes
 *                    output word d&3, noise = (word >> 8) * 2^-24, and
 *                    code = floor(u) + [noise < u - floor(u)];
 *   noise_bits = 16: counter (d>>3, n, lo32(tag), hi32(tag)), element d takes
 *                    word (d>>1)&3, low half if d is even, high half if odd,
 *                    noise = half * 2^-16, and code = floor(u + noise), the sum
 *                    being one binary32 addition rounded to nearest.  Over the
 *                    65,536 noise values the code is ceil(u) with a probability
 *                    within 2^-16 of frac(u) (the noise grid and the rounding of
 *                    the sum both stay inside that bound), an integer u keeps its
 *                    code, and the code never exceeds B.  This is the fast mode:
 *                    one generator call serves eight elements.
 * key = (lo32(seed), hi32(seed)).  `tag` separates tensors (layers) that share
 * a seed.  Requires N < 2^32 and D < 2^34.
 *
 * x        device, in  : N*D elements of dtype `dt`
 * bits     device, in  : [N] widths b_n in 1..8
 * offsets  device, in  : [N] byte offsets as produced by actq_packed_bytes
 * packed   device, out : the bit stream; `packed_capacity` bytes are writable
 * header   device, out : [N*ng] groups in format hf: {float Z, float scale} or
 *                        {uint16 Z, uint16 R} (bfloat16 bit patterns), 8-byte aligned;
 *                        with ACTQ_HDR_TENSOR it is device, IN: one {float Z, float R}
 *
 * bits and offsets live on the device, so the host cannot check them: a sample
 * whose width is not in 1..8 or whose byte range would leave
 * [0, packed_capacity) is skipped (no byte of its output is written).
 * Errors: ACTQ_EINVAL on a null or misaligned pointer, sizes out of range,
 * unsupported G, dtype, noise_bits or header format, or a capacity below one bit
 * per element; ACTQ_EHIP if the launch fails.
 */
int actq_quantize_pack(const void* x, actq_dtype dt, int64_t N, int64_t D, int32_t G,
                       const uint8_t* bits, const uint64_t* offsets,
                       uint64_t seed, uint64_t tag, int32_t noise_bits,
                       void* packed, uint64_t packed_capacity, void* header,
                       actq_header_format hf, void* stream);

/*
 * Backward pass: unpack and dequantize (Sec. 4.1): h^ = code * scale + Z,
 * evaluated as one fused multiply-add in binary32; binary16 output is the
 * round-to-nearest-even conversion of that value.
 *
 * With the bfloat16 header the step is recomputed as scale = R / B (one
 * binary32 division) before the multiply-add.
 *
 * packed  device, in  : bit stream written by actq_quantize_pack
 * header  device, in  : as written by actq_quantize_pack with the same hf
 * bits, offsets       : as for actq_quantize_pack; a sample that fails the same
 *                       checks against `packed_capacity` is skipped
 * out     device, out : N*D elements of dtype `out_dt`
 * Errors: as for actq_quantize_pack.
 */
int actq_unpack_dequantize(const void* packed, uint64_t packed_capacity,
                           const void* header, actq_header_format hf, const uint8_t* bits,
                           const uint64_t* offsets, int64_t N, int64_t D, int32_t G,
                           void* out, actq_dtype out_dt, void* stream);

/*
 * Range and zero point of a whole tensor (the single-group quantizer of Sec. 4.1's
 * comparison): zr[0] = Z = min over all n elements (-0.0 stored as +0.0),
 * zr[1] = R = max - min rounded to nearest.  The pair is the header of
 * ACTQ_HDR_TENSOR.  Three small launches on `stream`; the result does not depend
 * on the order in which the hardware combines partial results.
 *
 * x  device, in  : n elements of dtype dt, 16-byte aligned, n in [1, 2^40)
 * zr device, out : two floats, 8-byte aligned
 */
int actq_tensor_stats(const void* x, actq_dtype dt, int64_t n, float* zr, void* stream);

/*
 * Per-sample sensitivity of a linear layer (Sec. 4.2, Eq. (8) and the sentence
 * after Prob. (9)): w_n = (G / 6) * ||grad_n||^2 * sum_g R_ng^2, the input of
 * actq_allocate_bits.  It reads only the group ranges written by
 * actq_group_stats (1/256 of the tensor), one block per sample, binary32 sums in
 * a fixed order.
 *
 * grange device, in  : [N*ng] float
 * grad2  device, in  : [N] float, the squared gradient norms (or their running
 *                      estimate, Sec. 4.3); NULL means 1
 * w      device, out : [N] float
 * Errors: ACTQ_EINVAL on a null or misaligned pointer (grad2 may be null) or
 * N, ng outside [1, 2^32); ACTQ_EHIP if the launch fails.
 */
int actq_sample_sensitivity(const float* grange, int64_t N, int64_t ng, int32_t G,
                            const float* grad2, float* w, void* stream);

/* Sets of allowed widths for the allocator: bit b set means b bits is allowed. */
#define ACTQ_WIDTHS_POW2 0x116u /* {1, 2, 4, 8}: a code never straddles a byte */
#define ACTQ_WIDTHS_ALL 0x1FEu  /* {1, ..., 8}: the one-bit-at-a-time greedy of Sec. 4.3 */

/*
 * Greedy solution of the bit-allocation problem (Sec. 4.2, Prob. (9); greedy
 * with a binary heap as in Sec. 4.3): minimise sum_i w_i / B_i^2 subject to
 * sum_i D_i * b_i <= budget_bits, B_i = 2^{b_i} - 1.
 *
 * Every item starts at the widest allowed width.  A move lowers one item to the
 * next narrower allowed width, b_hi -> b_lo.  Its price is the variance it adds
 * per bit it frees,
 *   key = (double)w_i * c / (double)D_i,
 *   c = (1/B_lo^2 - 1/B_hi^2) / (b_hi - b_lo)   evaluated in double,
 * and while the budget is exceeded the move with the smallest (key, i) is
 * applied.  The header cost of the groups is not part of the budget.
 *
 * w        host, in  : [M] sensitivities, finite and >= 0
 * D        host, in  : [M] element counts, > 0
 * widths             : non-empty subset of bits 1..8, e.g. ACTQ_WIDTHS_POW2
 * bits_out host, out : [M]
 * Errors: ACTQ_EINVAL on bad arguments; ACTQ_EINFEASIBLE when even the narrowest
 * allowed width everywhere exceeds the budget (bits_out is then all narrowest).
 */
int actq_allocate_bits(const float* w, const int64_t* D, int64_t M,
                       int64_t budget_bits, uint32_t widths, uint8_t* bits_out);

/*
 * The same allocation computed on the device, so that a step needs no host
 * round trip between the statistics and the quantizer (Sec. 4.3 runs the
 * allocator inside the training step).  The result equals actq_allocate_bits
 * bit for bit: the greedy's answer is fixed by the price of its last move, which
 * one workgroup finds by radix selection over the 64-bit price patterns; moves
 * of exactly that price are applied in (i, step) order.  It also writes the byte
 * offsets that actq_packed_bytes would compute for the chosen widths.
 *
 * w        device, in  : [M] sensitivities
 * D_items  device, in  : [M] element counts, or NULL: every item has D elements
 * D                    : element count per item when D_items is NULL (else ignored)
 * G                    : group size used for the offsets (256)
 * bits     device, out : [M]
 * offsets  device, out : [M] offsets[i] = sum_{j<i} ceil(D_j / G) * G * b_j / 8
 * result   device, out : [2] result[0] = total bytes of the bit stream,
 *                        result[1] = ACTQ_OK, ACTQ_EINVAL (some w not finite or
 *                        negative, or a D_items entry outside (0, 2^34)) or
 *                        ACTQ_EINFEASIBLE; in both failure cases every item gets
 *                        the narrowest width, so the outputs stay usable
 * Requires sum_i 8 * D_i < 2^63.  Asynchronous on `stream`; the return value covers
 * only the host-side checks and the launch.
 */
int actq_allocate_bits_device(const float* w, const int64_t* D_items, int64_t D, int64_t M,
                              int32_t G, int64_t budget_bits, uint32_t widths,
                              uint8_t* bits, uint64_t* offsets, int64_t* result, void* stream);

/*
 * Several tensors per launch.  A network saves dozens of activations of very
 * different sizes per step (Sec. 5.1: every layer keeps a compressed context);
 * these calls do the work of the single-tensor calls for up to
 * ACTQ_MAX_TENSORS_PER_CALL tensors in one launch, with identical results.
 * All tensors of a call share N, the dtype, the header format, the seed and the
 * bit stream buffer (`packed`, with each tensor's own offsets array addressing
 * it); tensor i draws its noise with tag + i.  Every D must be a multiple of
 * G = 256 (tensors with ragged groups go through the single-tensor calls).
 * The launch is sized for the largest tensor of the call (the surplus blocks of
 * smaller ones exit at once), so a call should group tensors of similar size.
 *
 * The descriptor array lives in HOST memory and is copied into the launch; the
 * pointers inside are device pointers with the alignment rules of the
 * single-tensor calls.  Fields a call does not use may be NULL.
 */
#define ACTQ_MAX_TENSORS_PER_CALL 40
typedef struct actq_tensor {
    const void* x;           /* in : N*D elements (group_stats_multi, quantize_pack_multi)   */
    void* out;               /* out: N*D elements (unpack_dequantize_multi)                  */
    float* gmin;             /* out: [N*ng] (group_stats_multi)                              */
    float* grange;           /* out: [N*ng] (group_stats_multi)                              */
    void* header;            /* out of quantize_pack_multi, in of unpack_dequantize_multi    */
    const uint8_t* bits;     /* in : [N] widths (quantize, dequantize)                       */
    const uint64_t* offsets; /* in : [N] byte offsets into `packed` (quantize, dequantize)   */
    int64_t D;               /* features per sample, a multiple of 256                       */
} actq_tensor;

int actq_group_stats_multi(const actq_tensor* tensors_host, int32_t count, actq_dtype dt,
                           int64_t N, int32_t G, void* stream);
int actq_quantize_pack_multi(const actq_tensor* tensors_host, int32_t count, actq_dtype dt,
                             int64_t N, int32_t G, uint64_t seed, uint64_t tag, int32_t noise_bits,
                             void* packed, uint64_t packed_capacity, actq_header_format hf,
                             void* stream);
int actq_unpack_dequantize_multi(const actq_tensor* tensors_host, int32_t count,
                                 const void* packed, uint64_t packed_capacity,
                                 actq_header_format hf, int64_t N, int32_t G, actq_dtype out_dt,
                                 void* stream);

/*
 * Exact context of a ReLU layer (appendix, "Activation Layers"): one bit per
 * element, f'(x) = [x > 0], nothing approximated.
 *
 * Forward: y[i] = x[i] where x[i] > 0, +0 elsewhere; bit i of the stream (bit
 * i mod 8 of byte floor(i / 8), the layout of 1-bit codes) is [x[i] > 0].  The
 * stream is padded with zero bits to a whole number of 256-bit groups:
 * actq_relu_mask_bytes(n) = ceil(n / 256) * 32 bytes.
 * Backward: grad_x[i] = grad_y[i] where bit i is set, +0 elsewhere.
 *
 * x, y           device : n elements of dtype dt; y may be the same buffer as x
 * grad_y, grad_x device : likewise; grad_x may be the same buffer as grad_y
 * mask           device : actq_relu_mask_bytes(n) bytes
 * All three 16-byte aligned; n in [1, 2^40).
 */
int actq_relu_mask_bytes(int64_t n, uint64_t* bytes_host);
int actq_relu_forward(const void* x, actq_dtype dt, int64_t n, void* y, uint8_t* mask, void* stream);
int actq_relu_backward(const uint8_t* mask, const void* grad_y, actq_dtype dt, int64_t n,
                       void* grad_x, void* stream);

/*
 * Exact context of a max-pooling layer (appendix, "Pooling Layers", "Max
 * Pooling"): for every output location the position k of the maximum inside
 * its window, 0 <= k < kh*kw <= 256, in 8 bits.
 *
 * The tensors are `planes` (= batch * channels) row-major images, H x W in,
 * OH x OW out with OH = floor((H + 2*ph - dh*(kh-1) - 1) / sh) + 1 (likewise
 * OW), as returned by actq_pool2d_output_size.  Window position k = a*kw + b
 * is input row sh*i - ph + dh*a, column sw*j - pw + dw*b; padded positions
 * never win; among equal values the smallest k wins.
 * Backward: grad_x of an input location is the sum, in binary32 and in
 * ascending (i, j), of the grad_y whose stored position points at it; a stored
 * position that points outside the image is ignored.
 *
 * x, grad_x  device : planes*H*W elements;  y, grad_y : planes*OH*OW elements
 * argmax     device : planes*OH*OW bytes
 * Errors: ACTQ_EINVAL on a window of more than 256 positions, padding above
 * half the window size, a window larger than the padded image, non-positive
 * sizes, strides or dilations, planes*H*W >= 2^40, or misaligned tensors.
 */
int actq_pool2d_output_size(int32_t H, int32_t W, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                            int32_t ph, int32_t pw, int32_t dh, int32_t dw,
                            int32_t* OH_host, int32_t* OW_host);
int actq_maxpool2d_forward(const void* x, actq_dtype dt, int64_t planes, int32_t H, int32_t W,
                           int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw,
                           int32_t dh, int32_t dw, void* y, uint8_t* argmax, void* stream);
int actq_maxpool2d_backward(const uint8_t* argmax, const void* grad_y, actq_dtype dt, int64_t planes,
                            int32_t H, int32_t W, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                            int32_t ph, int32_t pw, int32_t dh, int32_t dw, void* grad_x,
                            void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ACTQ_H */
