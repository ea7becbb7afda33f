// Host side of libactq: argument validation, size arithmetic, the greedy bit allocator,
// and the extern "C" entry points declared in actq.h.  Nothing here touches the GPU
// except through the launchers of the kernel file.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <queue>
#include <utility>
#include <vector>

#include "actq_internal.h"

namespace actq {

static thread_local char g_error[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

static bool width_ok(unsigned b) { return b >= 1 && b <= 8; }

static bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Shape checks common to the three device calls.
static int check_view(const char* who, int64_t N, int64_t D, int32_t G)
{
    if (N <= 0 || D <= 0) return fail(ACTQ_EINVAL, "%s: N and D must be positive (N=%lld, D=%lld)", who, (long long)N, (long long)D);
    if (G != kGroup) return fail(ACTQ_EINVAL, "%s: unsupported group size G=%d (only %d)", who, G, kGroup);
    if (N >= (int64_t(1) << 32)) return fail(ACTQ_EINVAL, "%s: N must be below 2^32", who);
    if (D >= (int64_t(1) << 34)) return fail(ACTQ_EINVAL, "%s: D must be below 2^34", who);
    int64_t ng = (D + G - 1) / G;
    // total groups and total elements must fit the 64-bit index arithmetic comfortably
    if (N > (int64_t(1) << 62) / (ng * G)) return fail(ACTQ_EINVAL, "%s: N*D too large", who);
    return ACTQ_OK;
}

static int check_header(const char* who, int hf)
{
    if (hf != ACTQ_HDR_F32 && hf != ACTQ_HDR_BF16 && hf != ACTQ_HDR_TENSOR) return fail(ACTQ_EINVAL, "%s: unknown header format %d", who, hf);
    return ACTQ_OK;
}

static int check_dtype(const char* who, int dt)
{
    if (dt != ACTQ_F32 && dt != ACTQ_F16) return fail(ACTQ_EINVAL, "%s: unknown dtype %d", who, dt);
    return ACTQ_OK;
}

}  // namespace actq

using namespace actq;

namespace actq {

// Allowed widths, widest first, and for every step down the variance it adds per bit it
// frees, for a unit of w / D: (1/B_low^2 - 1/B_high^2) / (b_high - b_low), in double.
bool make_ladder(uint32_t widths, Ladder* out)
{
    if ((widths & ~0x1FEu) != 0 || (widths & 0x1FEu) == 0) return false;
    out->count = 0;
    for (int b = 8; b >= 1; --b)
        if ((widths >> b) & 1u) out->width[out->count++] = b;
    for (int r = 0; r + 1 < out->count; ++r) {
        const int hi = out->width[r], lo = out->width[r + 1];
        const double Bh = static_cast<double>((1 << hi) - 1), Bl = static_cast<double>((1 << lo) - 1);
        out->price[r] = (1.0 / (Bl * Bl) - 1.0 / (Bh * Bh)) / static_cast<double>(hi - lo);
    }
    for (int r = out->count; r < 8; ++r) out->width[r] = 0;
    for (int r = (out->count > 0 ? out->count - 1 : 0); r < 7; ++r) out->price[r] = 0.0;
    return true;
}

}  // namespace actq

extern "C" {

int actq_version(void) { return 400; }

#ifndef ACTQ_SOURCE_HASH
#define ACTQ_SOURCE_HASH "unknown"
#endif
// the digest follows a fixed marker, so that it can also be read from the file without loading it
static const char g_source_digest[] = "actq-source-digest:" ACTQ_SOURCE_HASH;
const char* actq_source_hash(void) { return g_source_digest + sizeof("actq-source-digest:") - 1; }

int actq_header_bytes(int64_t N, int64_t D, int32_t G, actq_header_format hf, uint64_t* bytes_host)
{
    if (int rc = check_view("actq_header_bytes", N, D, G)) return rc;
    if (int rc = check_header("actq_header_bytes", hf)) return rc;
    if (!bytes_host) return fail(ACTQ_EINVAL, "actq_header_bytes: null output");
    const uint64_t ng = static_cast<uint64_t>((D + G - 1) / G);
    *bytes_host = hf == ACTQ_HDR_TENSOR ? 8u : static_cast<uint64_t>(N) * ng * (hf == ACTQ_HDR_BF16 ? 4u : 8u);
    return ACTQ_OK;
}

const char* actq_last_error(void) { return g_error; }

int actq_packed_bytes(int64_t N, int64_t D, int32_t G, const uint8_t* bits_host,
                      uint64_t* offsets_host, uint64_t* total_host)
{
    if (int rc = check_view("actq_packed_bytes", N, D, G)) return rc;
    if (!bits_host) return fail(ACTQ_EINVAL, "actq_packed_bytes: bits_host is null");
    if (!offsets_host && !total_host) return fail(ACTQ_EINVAL, "actq_packed_bytes: both outputs are null");
    const uint64_t ng = static_cast<uint64_t>((D + G - 1) / G);
    const uint64_t group_bytes_per_bit = static_cast<uint64_t>(G) / 8;
    for (int64_t n = 0; n < N; ++n)
        if (!width_ok(bits_host[n]))
            return fail(ACTQ_EINVAL, "actq_packed_bytes: bits[%lld]=%u is not in 1..8", (long long)n, bits_host[n]);
    uint64_t acc = 0;
    for (int64_t n = 0; n < N; ++n) {
        if (offsets_host) offsets_host[n] = acc;
        acc += ng * group_bytes_per_bit * bits_host[n];
    }
    if (total_host) *total_host = acc;
    return ACTQ_OK;
}

int actq_group_stats(const void* x, actq_dtype dt, int64_t N, int64_t D, int32_t G,
                     float* gmin, float* grange, void* stream)
{
    if (int rc = check_view("actq_group_stats", N, D, G)) return rc;
    if (int rc = check_dtype("actq_group_stats", dt)) return rc;
    if (!x || !gmin || !grange) return fail(ACTQ_EINVAL, "actq_group_stats: null pointer");
    if (!aligned(x, 16)) return fail(ACTQ_EINVAL, "actq_group_stats: x must be 16-byte aligned");
    if (!aligned(gmin, 4) || !aligned(grange, 4)) return fail(ACTQ_EINVAL, "actq_group_stats: outputs must be 4-byte aligned");
    return launch_group_stats(x, dt, N, D, gmin, grange, stream);
}

int actq_quantize_pack(const void* x, actq_dtype dt, int64_t N, int64_t D, int32_t G,
                       const uint8_t* bits, const uint64_t* offsets, uint64_t seed,
                       uint64_t tag, int32_t noise_bits, void* packed,
                       uint64_t packed_capacity, void* header, actq_header_format hf, void* stream)
{
    if (int rc = check_view("actq_quantize_pack", N, D, G)) return rc;
    if (int rc = check_header("actq_quantize_pack", hf)) return rc;
    if (int rc = check_dtype("actq_quantize_pack", dt)) return rc;
    if (!x || !bits || !offsets || !packed || !header) return fail(ACTQ_EINVAL, "actq_quantize_pack: null pointer");
    if (noise_bits != 24 && noise_bits != 16) return fail(ACTQ_EINVAL, "actq_quantize_pack: noise_bits must be 24 or 16, got %d", noise_bits);
    if (!aligned(x, 16)) return fail(ACTQ_EINVAL, "actq_quantize_pack: x must be 16-byte aligned");
    if (!aligned(packed, 16)) return fail(ACTQ_EINVAL, "actq_quantize_pack: packed must be 16-byte aligned");
    if (!aligned(header, 8)) return fail(ACTQ_EINVAL, "actq_quantize_pack: header must be 8-byte aligned");
    if (!aligned(offsets, 8)) return fail(ACTQ_EINVAL, "actq_quantize_pack: offsets must be 8-byte aligned");
    if (!aligned(bits, 4)) return fail(ACTQ_EINVAL, "actq_quantize_pack: bits must be 4-byte aligned");
    const uint64_t ng = static_cast<uint64_t>((D + G - 1) / G);
    if (packed_capacity < static_cast<uint64_t>(N) * ng * (G / 8))
        return fail(ACTQ_EINVAL, "actq_quantize_pack: packed_capacity %llu is below one bit per element", (unsigned long long)packed_capacity);
    return launch_quantize_pack(x, dt, N, D, bits, offsets, seed, tag, noise_bits, packed,
                                packed_capacity, header, hf, stream);
}

int actq_unpack_dequantize(const void* packed, uint64_t packed_capacity, const void* header,
                           actq_header_format hf, const uint8_t* bits, const uint64_t* offsets,
                           int64_t N, int64_t D, int32_t G, void* out, actq_dtype out_dt, void* stream)
{
    if (int rc = check_view("actq_unpack_dequantize", N, D, G)) return rc;
    if (int rc = check_header("actq_unpack_dequantize", hf)) return rc;
    if (int rc = check_dtype("actq_unpack_dequantize", out_dt)) return rc;
    if (!packed || !header || !bits || !offsets || !out) return fail(ACTQ_EINVAL, "actq_unpack_dequantize: null pointer");
    if (!aligned(out, 16)) return fail(ACTQ_EINVAL, "actq_unpack_dequantize: out must be 16-byte aligned");
    if (!aligned(packed, 16)) return fail(ACTQ_EINVAL, "actq_unpack_dequantize: packed must be 16-byte aligned");
    if (!aligned(header, 8)) return fail(ACTQ_EINVAL, "actq_unpack_dequantize: header must be 8-byte aligned");
    if (!aligned(offsets, 8)) return fail(ACTQ_EINVAL, "actq_unpack_dequantize: offsets must be 8-byte aligned");
    if (!aligned(bits, 4)) return fail(ACTQ_EINVAL, "actq_unpack_dequantize: bits must be 4-byte aligned");
    return launch_unpack_dequantize(packed, packed_capacity, header, hf, bits, offsets, N, D, out,
                                    out_dt, stream);
}

int actq_sample_sensitivity(const float* grange, int64_t N, int64_t ng, int32_t G,
                            const float* grad2, float* w, void* stream)
{
    if (!grange || !w) return fail(ACTQ_EINVAL, "actq_sample_sensitivity: null pointer");
    if (N <= 0 || ng <= 0 || N >= (int64_t(1) << 32) || ng >= (int64_t(1) << 32))
        return fail(ACTQ_EINVAL, "actq_sample_sensitivity: N and ng must be positive and below 2^32");
    if (G <= 0) return fail(ACTQ_EINVAL, "actq_sample_sensitivity: G must be positive");
    if (!aligned(grange, 4) || !aligned(w, 4) || !aligned(grad2, 4))
        return fail(ACTQ_EINVAL, "actq_sample_sensitivity: arrays must be 4-byte aligned");
    return launch_sample_sensitivity(grange, N, ng, G, grad2, w, stream);
}

// Greedy allocator of Sec. 4.3 over the allowed widths, widest first.  The heap holds, for
// every item that can still be lowered, the price of its next move; ties go to the lowest
// item index.  An item's successive prices never decrease (its cost is convex in the width),
// so popping the cheapest move and pushing the item's next one visits moves in globally
// sorted order.
int actq_allocate_bits(const float* w, const int64_t* D, int64_t M, int64_t budget_bits,
                       uint32_t widths, uint8_t* bits_out)
{
    if (!w || !D || !bits_out) return fail(ACTQ_EINVAL, "actq_allocate_bits: null pointer");
    if (M <= 0) return fail(ACTQ_EINVAL, "actq_allocate_bits: M must be positive");
    if (budget_bits < 0) return fail(ACTQ_EINVAL, "actq_allocate_bits: negative budget");
    actq::Ladder lad;
    if (!actq::make_ladder(widths, &lad))
        return fail(ACTQ_EINVAL, "actq_allocate_bits: widths mask 0x%x must be a non-empty subset of bits 1..8", widths);
    __int128 used = 0;
    for (int64_t i = 0; i < M; ++i) {
        uint32_t pattern;
        std::memcpy(&pattern, &w[i], sizeof pattern);
        if (!valid_sensitivity_bits(pattern))
            return fail(ACTQ_EINVAL, "actq_allocate_bits: w[%lld] must be finite and >= 0", (long long)i);
        if (D[i] <= 0) return fail(ACTQ_EINVAL, "actq_allocate_bits: D[%lld] must be positive", (long long)i);
        used += static_cast<__int128>(D[i]) * lad.width[0];
    }
    auto price = [&](int64_t i, int rung) {
        return (static_cast<double>(w[i]) * lad.price[rung]) / static_cast<double>(D[i]);
    };
    std::vector<uint8_t> rung(static_cast<size_t>(M), 0);  // position of every item on the ladder
    auto finish = [&]() {
        for (int64_t i = 0; i < M; ++i) bits_out[i] = static_cast<uint8_t>(lad.width[rung[i]]);
    };
    const __int128 budget = budget_bits;
    if (used <= budget) { finish(); return ACTQ_OK; }

    using Move = std::pair<double, int64_t>;  // (price, item): lexicographic order is the rule
    std::vector<Move> init;
    if (lad.count > 1) {
        init.reserve(static_cast<size_t>(M));
        for (int64_t i = 0; i < M; ++i) init.emplace_back(price(i, 0), i);
    }
    std::priority_queue<Move, std::vector<Move>, std::greater<Move>> heap(std::greater<Move>(), std::move(init));
    while (used > budget) {
        if (heap.empty()) {
            finish();
            return fail(ACTQ_EINFEASIBLE, "actq_allocate_bits: budget %lld is below %d bit(s) per element",
                        (long long)budget_bits, lad.width[lad.count - 1]);
        }
        const int64_t i = heap.top().second;
        heap.pop();
        const int r = rung[i];
        used -= static_cast<__int128>(D[i]) * (lad.width[r] - lad.width[r + 1]);
        rung[i] = static_cast<uint8_t>(r + 1);
        if (r + 2 < lad.count) heap.emplace(price(i, r + 1), i);
    }
    finish();
    return ACTQ_OK;
}

int actq_allocate_bits_device(const float* w, const int64_t* D_items, int64_t D, int64_t M, int32_t G,
                              int64_t budget_bits, uint32_t widths, uint8_t* bits, uint64_t* offsets,
                              int64_t* result, void* stream)
{
    if (!w || !bits || !offsets || !result) return fail(ACTQ_EINVAL, "actq_allocate_bits_device: null pointer");
    if (M <= 0 || M >= (int64_t(1) << 31)) return fail(ACTQ_EINVAL, "actq_allocate_bits_device: M must be in [1, 2^31)");
    if (G != kGroup) return fail(ACTQ_EINVAL, "actq_allocate_bits_device: unsupported group size G=%d (supported: %d)", G, kGroup);
    if (!D_items && (D <= 0 || D >= (int64_t(1) << 34)))
        return fail(ACTQ_EINVAL, "actq_allocate_bits_device: D must be in [1, 2^34) when D_items is null");
    if (!D_items && static_cast<__int128>(D) * M * 8 >= (static_cast<__int128>(1) << 63))
        return fail(ACTQ_EINVAL, "actq_allocate_bits_device: 8 * M * D must stay below 2^63");
    if (budget_bits < 0) return fail(ACTQ_EINVAL, "actq_allocate_bits_device: negative budget");
    if (!aligned(w, 4) || !aligned(D_items, 8) || !aligned(offsets, 8) || !aligned(result, 8))
        return fail(ACTQ_EINVAL, "actq_allocate_bits_device: w must be 4-byte aligned, D_items, offsets and result 8-byte aligned");
    actq::Ladder lad;
    if (!actq::make_ladder(widths, &lad))
        return fail(ACTQ_EINVAL, "actq_allocate_bits_device: widths mask 0x%x must be a non-empty subset of bits 1..8", widths);
    return launch_allocate_bits(w, D_items, D, M, budget_bits, lad, bits, offsets, result, stream);
}

// Checks shared by the multi-tensor calls: which == 0 stats, 1 quantize, 2 dequantize.
static int check_multi(const char* who, const actq_tensor* t, int32_t count, int dt, int64_t N, int32_t G, int which,
                       const void* packed, int hf)
{
    if (int rc = check_dtype(who, dt)) return rc;
    if (!t) return fail(ACTQ_EINVAL, "%s: tensors_host is null", who);
    if (count < 1 || count > ACTQ_MAX_TENSORS_PER_CALL)
        return fail(ACTQ_EINVAL, "%s: count must be in [1, %d]", who, ACTQ_MAX_TENSORS_PER_CALL);
    if (which != 0) {
        if (int rc = check_header(who, hf)) return rc;
        if (!packed || !aligned(packed, 16)) return fail(ACTQ_EINVAL, "%s: packed must be non-null and 16-byte aligned", who);
    }
    for (int32_t i = 0; i < count; ++i) {
        if (int rc = check_view(who, N, t[i].D, G)) return rc;
        if (t[i].D % G != 0) return fail(ACTQ_EINVAL, "%s: tensor %d: D must be a multiple of %d", who, i, G);
        const void* data = which == 2 ? t[i].out : t[i].x;
        if (!data || !aligned(data, 16)) return fail(ACTQ_EINVAL, "%s: tensor %d: data pointer must be non-null and 16-byte aligned", who, i);
        if (which == 0) {
            if (!t[i].gmin || !t[i].grange || !aligned(t[i].gmin, 4) || !aligned(t[i].grange, 4))
                return fail(ACTQ_EINVAL, "%s: tensor %d: gmin and grange must be non-null and 4-byte aligned", who, i);
        } else {
            if (!t[i].header || !aligned(t[i].header, 8)) return fail(ACTQ_EINVAL, "%s: tensor %d: header must be non-null and 8-byte aligned", who, i);
            if (!t[i].bits || !aligned(t[i].bits, 4)) return fail(ACTQ_EINVAL, "%s: tensor %d: bits must be non-null and 4-byte aligned", who, i);
            if (!t[i].offsets || !aligned(t[i].offsets, 8)) return fail(ACTQ_EINVAL, "%s: tensor %d: offsets must be non-null and 8-byte aligned", who, i);
        }
    }
    return ACTQ_OK;
}

int actq_group_stats_multi(const actq_tensor* tensors_host, int32_t count, actq_dtype dt, int64_t N, int32_t G,
                           void* stream)
{
    if (int rc = check_multi("actq_group_stats_multi", tensors_host, count, dt, N, G, 0, nullptr, 0)) return rc;
    return launch_group_stats_multi(tensors_host, count, dt, N, stream);
}

int actq_quantize_pack_multi(const actq_tensor* tensors_host, int32_t count, actq_dtype dt, int64_t N, int32_t G,
                             uint64_t seed, uint64_t tag, int32_t noise_bits, void* packed,
                             uint64_t packed_capacity, actq_header_format hf, void* stream)
{
    if (int rc = check_multi("actq_quantize_pack_multi", tensors_host, count, dt, N, G, 1, packed, hf)) return rc;
    if (noise_bits != 24 && noise_bits != 16)
        return fail(ACTQ_EINVAL, "actq_quantize_pack_multi: noise_bits must be 24 or 16, got %d", noise_bits);
    return launch_quantize_pack_multi(tensors_host, count, dt, N, seed, tag, noise_bits, packed, packed_capacity, hf, stream);
}

int actq_unpack_dequantize_multi(const actq_tensor* tensors_host, int32_t count, const void* packed,
                                 uint64_t packed_capacity, actq_header_format hf, int64_t N, int32_t G,
                                 actq_dtype out_dt, void* stream)
{
    if (int rc = check_multi("actq_unpack_dequantize_multi", tensors_host, count, out_dt, N, G, 2, packed, hf)) return rc;
    return launch_unpack_dequantize_multi(tensors_host, count, packed, packed_capacity, hf, N, out_dt, stream);
}

int actq_tensor_stats(const void* x, actq_dtype dt, int64_t n, float* zr, void* stream)
{
    if (int rc = check_dtype("actq_tensor_stats", dt)) return rc;
    if (!x || !zr) return fail(ACTQ_EINVAL, "actq_tensor_stats: null pointer");
    if (n <= 0 || n >= (int64_t(1) << 40)) return fail(ACTQ_EINVAL, "actq_tensor_stats: n must be in [1, 2^40)");
    if (!aligned(x, 16)) return fail(ACTQ_EINVAL, "actq_tensor_stats: x must be 16-byte aligned");
    if (!aligned(zr, 8)) return fail(ACTQ_EINVAL, "actq_tensor_stats: zr must be 8-byte aligned");
    return launch_tensor_stats(x, dt, n, zr, stream);
}

int actq_relu_mask_bytes(int64_t n, uint64_t* bytes_host)
{
    if (n <= 0 || !bytes_host) return fail(ACTQ_EINVAL, "actq_relu_mask_bytes: n must be positive and bytes_host non-null");
    *bytes_host = static_cast<uint64_t>((n + 255) / 256) * 32;
    return ACTQ_OK;
}

static int check_elementwise(const char* who, const void* a, const void* b, const void* mask, int dt, int64_t n)
{
    if (int rc = check_dtype(who, dt)) return rc;
    if (!a || !b || !mask) return fail(ACTQ_EINVAL, "%s: null pointer", who);
    if (n <= 0 || n >= (int64_t(1) << 40)) return fail(ACTQ_EINVAL, "%s: n must be in [1, 2^40)", who);
    if (!aligned(a, 16) || !aligned(b, 16) || !aligned(mask, 16))
        return fail(ACTQ_EINVAL, "%s: tensors and mask must be 16-byte aligned", who);
    return ACTQ_OK;
}

int actq_relu_forward(const void* x, actq_dtype dt, int64_t n, void* y, uint8_t* mask, void* stream)
{
    if (int rc = check_elementwise("actq_relu_forward", x, y, mask, dt, n)) return rc;
    return launch_relu_forward(x, dt, n, y, mask, stream);
}

int actq_relu_backward(const uint8_t* mask, const void* grad_y, actq_dtype dt, int64_t n, void* grad_x,
                       void* stream)
{
    if (int rc = check_elementwise("actq_relu_backward", grad_y, grad_x, mask, dt, n)) return rc;
    return launch_relu_backward(mask, grad_y, dt, n, grad_x, stream);
}

static int make_pool_shape(const char* who, int32_t H, int32_t W, int32_t kh, int32_t kw, int32_t sh, int32_t sw,
                           int32_t ph, int32_t pw, int32_t dh, int32_t dw, PoolShape* p)
{
    if (H <= 0 || W <= 0) return fail(ACTQ_EINVAL, "%s: H and W must be positive", who);
    if (kh <= 0 || kw <= 0 || static_cast<int64_t>(kh) * kw > 256)
        return fail(ACTQ_EINVAL, "%s: window %d x %d must have 1..256 positions (8-bit context)", who, kh, kw);
    if (sh <= 0 || sw <= 0 || dh <= 0 || dw <= 0) return fail(ACTQ_EINVAL, "%s: strides and dilations must be positive", who);
    if (ph < 0 || pw < 0 || 2 * ph > kh || 2 * pw > kw)
        return fail(ACTQ_EINVAL, "%s: padding must be between 0 and half the window size", who);
    const int64_t eh = static_cast<int64_t>(dh) * (kh - 1) + 1, ew = static_cast<int64_t>(dw) * (kw - 1) + 1;
    if (H + 2 * static_cast<int64_t>(ph) < eh || W + 2 * static_cast<int64_t>(pw) < ew)
        return fail(ACTQ_EINVAL, "%s: the window does not fit the padded input", who);
    if (eh > (int64_t(1) << 20) || ew > (int64_t(1) << 20) || H > (1 << 24) || W > (1 << 24) ||
        sh > (1 << 20) || sw > (1 << 20))
        return fail(ACTQ_EINVAL, "%s: geometry too large", who);
    if (static_cast<int64_t>(H) * W >= (int64_t(1) << 31) ||
        (static_cast<int64_t>(H) + 2 * ph) * (static_cast<int64_t>(W) + 2 * pw) >= (int64_t(1) << 31))
        return fail(ACTQ_EINVAL, "%s: one image must have fewer than 2^31 locations", who);
    p->H = H; p->W = W;
    p->kh = kh; p->kw = kw; p->sh = sh; p->sw = sw; p->ph = ph; p->pw = pw; p->dh = dh; p->dw = dw;
    p->OH = static_cast<int32_t>((H + 2 * static_cast<int64_t>(ph) - eh) / sh + 1);
    p->OW = static_cast<int32_t>((W + 2 * static_cast<int64_t>(pw) - ew) / sw + 1);
    return ACTQ_OK;
}

int actq_pool2d_output_size(int32_t H, int32_t W, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph,
                            int32_t pw, int32_t dh, int32_t dw, int32_t* OH_host, int32_t* OW_host)
{
    if (!OH_host || !OW_host) return fail(ACTQ_EINVAL, "actq_pool2d_output_size: null output");
    PoolShape p;
    if (int rc = make_pool_shape("actq_pool2d_output_size", H, W, kh, kw, sh, sw, ph, pw, dh, dw, &p)) return rc;
    *OH_host = p.OH;
    *OW_host = p.OW;
    return ACTQ_OK;
}

static int check_pool_call(const char* who, const void* a, const void* b, const void* arg, int dt, int64_t planes,
                           const PoolShape& p)
{
    if (int rc = check_dtype(who, dt)) return rc;
    if (!a || !b || !arg) return fail(ACTQ_EINVAL, "%s: null pointer", who);
    if (planes <= 0 || static_cast<__int128>(planes) * p.H * p.W >= (static_cast<__int128>(1) << 40))
        return fail(ACTQ_EINVAL, "%s: planes * H * W must be in [1, 2^40)", who);
    const uintptr_t elem = dt == ACTQ_F32 ? 4 : 2;
    if (!aligned(a, elem) || !aligned(b, elem)) return fail(ACTQ_EINVAL, "%s: tensors must be aligned to their element size", who);
    return ACTQ_OK;
}

int actq_maxpool2d_forward(const void* x, actq_dtype dt, int64_t planes, int32_t H, int32_t W, int32_t kh,
                           int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw, int32_t dh, int32_t dw,
                           void* y, uint8_t* argmax, void* stream)
{
    PoolShape p;
    if (int rc = make_pool_shape("actq_maxpool2d_forward", H, W, kh, kw, sh, sw, ph, pw, dh, dw, &p)) return rc;
    if (int rc = check_pool_call("actq_maxpool2d_forward", x, y, argmax, dt, planes, p)) return rc;
    return launch_maxpool2d_forward(x, dt, planes, p, y, argmax, stream);
}

int actq_maxpool2d_backward(const uint8_t* argmax, const void* grad_y, actq_dtype dt, int64_t planes, int32_t H,
                            int32_t W, int32_t kh, int32_t kw, int32_t sh, int32_t sw, int32_t ph, int32_t pw,
                            int32_t dh, int32_t dw, void* grad_x, void* stream)
{
    PoolShape p;
    if (int rc = make_pool_shape("actq_maxpool2d_backward", H, W, kh, kw, sh, sw, ph, pw, dh, dw, &p)) return rc;
    if (int rc = check_pool_call("actq_maxpool2d_backward", grad_y, grad_x, argmax, dt, planes, p)) return rc;
    return launch_maxpool2d_backward(argmax, grad_y, dt, planes, p, grad_x, stream);
}

}  // extern "C"
