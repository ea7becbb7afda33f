// Internal declarations shared by the host-side API file and the kernel file of libactq.
#ifndef ACTQ_INTERNAL_H
#define ACTQ_INTERNAL_H

#include <cstdint>
#include <cstring>

#include <hip/hip_runtime.h>

#include "actq.h"

namespace actq {

constexpr int kGroup = 256;  // the one supported group size: one wavefront x 4 elements

// A sensitivity is valid if it is finite and not negative (-0.0 counts as zero).  Decided on the
// bit pattern: this library is compiled under the assumption that its floating-point data holds
// no NaN, which lets the compiler fold away a NaN test written as a comparison.
__host__ __device__ inline bool valid_sensitivity_bits(uint32_t bits)
{
    const bool finite = (bits & 0x7f800000u) != 0x7f800000u;   // exponent all ones: infinity or NaN
    const bool negative = (bits >> 31) != 0 && bits != 0x80000000u;
    return finite && !negative;
}

// Records a message for actq_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// The allowed widths of the allocator, widest first, with the price of every step down.
struct Ladder {
    int count;        // number of allowed widths, 1..8
    int width[8];     // width[0] > width[1] > ... ; unused entries are 0
    double price[7];  // price[r]: step width[r] -> width[r+1]
};
bool make_ladder(uint32_t widths, Ladder* out);

// Exact n / d for 0 <= n < 2^31 by one multiply-high, an add and a shift (division by an
// invariant integer after Granlund and Montgomery): with s = ceil(log2 d) and
// m = floor(2^32 (2^s - d) / d) + 1,  n / d = (mulhi(n, m) + n) >> s.
struct FastDiv {
    uint32_t m, s;
};

inline FastDiv make_fastdiv(uint32_t d)
{
    uint32_t s = 0;
    while ((uint64_t(1) << s) < d) ++s;
    FastDiv f;
    f.m = static_cast<uint32_t>(((uint64_t(1) << 32) * ((uint64_t(1) << s) - d)) / d + 1);
    f.s = s;
    return f;
}

// Launchers (kernels file).  Arguments are already validated.  Each returns ACTQ_OK or
// ACTQ_EHIP after recording the HIP error text.
int launch_group_stats(const void* x, int dtype, int64_t N, int64_t D, float* gmin,
                       float* grange, void* stream);
int launch_quantize_pack(const void* x, int dtype, int64_t N, int64_t D, const uint8_t* bits,
                         const uint64_t* offsets, uint64_t seed, uint64_t tag, int noise_bits,
                         void* packed, uint64_t capacity, void* header, int hdr, void* stream);
int launch_unpack_dequantize(const void* packed, uint64_t capacity, const void* header, int hdr,
                             const uint8_t* bits, const uint64_t* offsets, int64_t N,
                             int64_t D, void* out, int out_dtype, void* stream);
int launch_group_stats_multi(const actq_tensor* tensors, int32_t count, int dtype, int64_t N, void* stream);
int launch_quantize_pack_multi(const actq_tensor* tensors, int32_t count, int dtype, int64_t N, uint64_t seed,
                               uint64_t tag, int noise_bits, void* packed, uint64_t capacity, int hdr, void* stream);
int launch_unpack_dequantize_multi(const actq_tensor* tensors, int32_t count, const void* packed, uint64_t capacity,
                                   int hdr, int64_t N, int out_dtype, void* stream);
int launch_tensor_stats(const void* x, int dtype, int64_t n, float* zr, void* stream);
int launch_sample_sensitivity(const float* grange, int64_t N, int64_t ng, int32_t G,
                              const float* grad2, float* w, void* stream);
int launch_allocate_bits(const float* w, const int64_t* D_items, int64_t D, int64_t M, int64_t budget_bits,
                         const Ladder& lad, uint8_t* bits, uint64_t* offsets, int64_t* result, void* stream);

// Geometry of a 2-D pooling window, validated, with the output size worked out.
struct PoolShape {
    int32_t H, W, OH, OW;
    int32_t kh, kw, sh, sw, ph, pw, dh, dw;
};

// Launchers of the exact layer contexts (context kernels file).
int launch_relu_forward(const void* x, int dtype, int64_t n, void* y, uint8_t* mask, void* stream);
int launch_relu_backward(const uint8_t* mask, const void* grad_y, int dtype, int64_t n, void* grad_x, void* stream);
int launch_maxpool2d_forward(const void* x, int dtype, int64_t planes, const PoolShape& p, void* y,
                             uint8_t* argmax, void* stream);
int launch_maxpool2d_backward(const uint8_t* argmax, const void* grad_y, int dtype, int64_t planes,
                              const PoolShape& p, void* grad_x, void* stream);

}  // namespace actq

#endif
