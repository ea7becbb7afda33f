// HIP kernels of libactq for gfx950 (MI355X): per-group min/range, stochastic rounding
// with Philox4x32-10 noise, bit-stream packing, and unpack + dequantize (ActNN,
// Sec. 4.1 and Sec. 5.1).
//
// Work decomposition.  The group size is 256 = one 64-lane wavefront x 4 consecutive
// elements per lane, so one 128-bit load per lane brings in a whole group, and the
// min / max of a group is a wavefront reduction with no LDS traffic.  A *tile* is
// kTileGroups consecutive groups of one sample; tiles never cross a sample, so the
// width b_n is uniform over a tile and every branch on it is divergence-free.  A
// wavefront owns a run of consecutive tiles (a contiguous span of HBM) and exits.
//
// This file must be compiled with -ffp-contract=off: the scaling step is a subtraction
// and a multiplication that are rounded separately.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "actq_internal.h"

namespace actq {
namespace {

constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;
constexpr int kBlock = kWave * kWavesPerBlock;
constexpr int kTileGroups = 4;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------
// Cross-lane helpers (DPP within a row of 16 lanes, v_readlane across rows).

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v)
{
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xf, 0xf, false));
}

constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7-i inside each 8 lanes
constexpr int kDppMirror = 0x140;      // lane i <-> 15-i inside each 16 lanes

// min / max of a value over the wavefront, returned in every lane.  Inputs are finite.
__device__ __forceinline__ float wave_min(float v)
{
    v = fminf(v, dpp_f32<kDppXor1>(v));
    v = fminf(v, dpp_f32<kDppXor2>(v));
    v = fminf(v, dpp_f32<kDppHalfMirror>(v));
    v = fminf(v, dpp_f32<kDppMirror>(v));
    const int iv = __float_as_int(v);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(iv, 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(iv, 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(iv, 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(iv, 48));
    return fminf(fminf(r0, r1), fminf(r2, r3));
}

__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_f32<kDppXor1>(v));
    v = fmaxf(v, dpp_f32<kDppXor2>(v));
    v = fmaxf(v, dpp_f32<kDppHalfMirror>(v));
    v = fmaxf(v, dpp_f32<kDppMirror>(v));
    const int iv = __float_as_int(v);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(iv, 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(iv, 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(iv, 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(iv, 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// ------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11), state in registers.

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t prod_a = static_cast<uint64_t>(c0) * 0xD2511F53u;
        const uint64_t prod_b = static_cast<uint64_t>(c2) * 0xCD9E8D57u;
        const uint32_t y0 = static_cast<uint32_t>(prod_b >> 32) ^ c1 ^ k0;
        const uint32_t y2 = static_cast<uint32_t>(prod_a >> 32) ^ c3 ^ k1;
        c1 = static_cast<uint32_t>(prod_b);
        c3 = static_cast<uint32_t>(prod_a);
        c0 = y0;
        c2 = y2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0;
    out[1] = c1;
    out[2] = c2;
    out[3] = c3;
}

// ------------------------------------------------------------------------------------
// Loading four consecutive elements of one lane, widened to binary32.

template <typename T>
struct Io;

template <>
struct Io<float> {
    static __device__ __forceinline__ void load4(const float* p, float (&v)[4])
    {
        const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
    static __device__ __forceinline__ float load1(const float* p) { return *p; }
    static __device__ __forceinline__ void store4(float* p, const float (&v)[4])
    {
        f32x4 t;
        t.x = v[0]; t.y = v[1]; t.z = v[2]; t.w = v[3];
        __builtin_nontemporal_store(t, reinterpret_cast<f32x4*>(p));
    }
    static __device__ __forceinline__ void store1(float* p, float v) { *p = v; }
};

template <>
struct Io<_Float16> {
    static __device__ __forceinline__ void load4(const _Float16* p, float (&v)[4])
    {
        const f16x4 t = __builtin_nontemporal_load(reinterpret_cast<const f16x4*>(p));
        v[0] = static_cast<float>(t.x); v[1] = static_cast<float>(t.y);
        v[2] = static_cast<float>(t.z); v[3] = static_cast<float>(t.w);
    }
    static __device__ __forceinline__ float load1(const _Float16* p) { return static_cast<float>(*p); }
    // binary32 -> binary16, round to nearest even, of a value that has already been rounded
    // to binary32.  The empty asm keeps the compiler from merging the conversion into the
    // producing multiply-add (a mixed-precision fma rounds once, straight to binary16, and
    // differs from the two-step result in rare half-way cases).
    static __device__ __forceinline__ _Float16 narrow(float v)
    {
        asm("" : "+v"(v));
        return static_cast<_Float16>(v);
    }
    static __device__ __forceinline__ void store4(_Float16* p, const float (&v)[4])
    {
        f16x4 t;
        t.x = narrow(v[0]); t.y = narrow(v[1]); t.z = narrow(v[2]); t.w = narrow(v[3]);
        __builtin_nontemporal_store(t, reinterpret_cast<f16x4*>(p));
    }
    static __device__ __forceinline__ void store1(_Float16* p, float v) { *p = narrow(v); }
};

// Geometry shared by the kernels.  All of it is wavefront-uniform.
struct Geometry {
    int64_t D;              // features per sample
    uint32_t ng;            // groups per sample
    uint32_t tiles_per_sample;
    uint32_t tiles;         // N * tiles_per_sample
    uint32_t tiles_per_wave;
};

struct TileCursor {
    uint32_t n;   // sample
    uint32_t g0;  // first group of the tile inside the sample
};

// Loads the lane's four elements of group g (sample base xs).  VEC: the group is full
// and 16-byte (8 for binary16) aligned.  Otherwise every element is guarded; elements
// past D read as +inf in lo[] and -inf in hi[] so that they drop out of min and max.
template <typename T, bool VEC>
__device__ __forceinline__ void load_group(const T* xs, int64_t d0, int64_t D, float (&v)[4],
                                           bool (&ok)[4])
{
    if (VEC) {
        Io<T>::load4(xs + d0, v);
        ok[0] = ok[1] = ok[2] = ok[3] = true;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            ok[k] = d0 + k < D;
            v[k] = ok[k] ? Io<T>::load1(xs + d0 + k) : 0.0f;
        }
    }
}

template <bool VEC>
__device__ __forceinline__ void lane_min_max(const float (&v)[4], const bool (&ok)[4], float& lo, float& hi)
{
    if (VEC) {
        lo = fminf(fminf(v[0], v[1]), fminf(v[2], v[3]));
        hi = fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3]));
    } else {
        lo = __builtin_inff();
        hi = -__builtin_inff();
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            lo = ok[k] ? fminf(lo, v[k]) : lo;
            hi = ok[k] ? fmaxf(hi, v[k]) : hi;
        }
    }
}

__device__ __forceinline__ uint32_t wave_index()
{
    const uint32_t w = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    return static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(w)));
}

// ------------------------------------------------------------------------------------
// Sec. 4.1: Z = min, R = max - min per group.

template <typename T, bool VEC>
__global__ __launch_bounds__(kBlock) void group_stats_kernel(const T* __restrict__ x, Geometry geo,
                                                             float* __restrict__ gmin,
                                                             float* __restrict__ grange)
{
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t first = wave_index() * geo.tiles_per_wave;
    if (first >= geo.tiles) return;
    const uint32_t last = min(first + geo.tiles_per_wave, geo.tiles);
    uint32_t n = first / geo.tiles_per_sample;
    uint32_t g0 = (first - n * geo.tiles_per_sample) * kTileGroups;
    for (uint32_t tile = first; tile < last; ++tile) {
        const T* xs = x + static_cast<int64_t>(n) * geo.D;
        const int groups = static_cast<int>(min(static_cast<uint32_t>(kTileGroups), geo.ng - g0));
        float v[kTileGroups][4];
        bool ok[kTileGroups][4];
#pragma unroll
        for (int u = 0; u < kTileGroups; ++u)
            if (u < groups)
                load_group<T, VEC>(xs, (static_cast<int64_t>(g0 + u) << 8) + lane * 4, geo.D, v[u], ok[u]);
#pragma unroll
        for (int u = 0; u < kTileGroups; ++u) {
            if (u < groups) {
                float lo, hi;
                lane_min_max<VEC>(v[u], ok[u], lo, hi);
                const float mn = wave_min(lo) + 0.0f;  // -0.0 -> +0.0
                const float mx = wave_max(hi);
                if (lane == 0) {
                    const int64_t gi = static_cast<int64_t>(n) * geo.ng + g0 + u;
                    gmin[gi] = mn;
                    grange[gi] = mx - mn;
                }
            }
        }
        g0 += kTileGroups;
        if (g0 >= geo.ng) { g0 = 0; ++n; }
    }
}

// ------------------------------------------------------------------------------------
// Sec. 4.1 + Sec. 5.1: scale, round stochastically, pack.

// OR of `piece << (bits_per_lane * (lane % lanes_per_word))` over each cluster of lanes
// that share a 32-bit word of the stream; every lane of the cluster receives the word.
template <int B>
__device__ __forceinline__ uint32_t gather_word(uint32_t piece, int lane)
{
    constexpr int lanes_per_word = 8 / B;  // 4*B bits per lane
    if (lanes_per_word == 1) return piece;
    uint32_t w = piece << ((lane & (lanes_per_word - 1)) * (4 * B));
    w |= dpp_u32<kDppXor1>(w);
    if (lanes_per_word >= 4) w |= dpp_u32<kDppXor2>(w);
    if (lanes_per_word >= 8) w |= dpp_u32<kDppHalfMirror>(w);
    return w;
}

template <typename T, int NOISE_BITS, bool VEC, int B>
__device__ __forceinline__ void quantize_tile(const T* xs, int64_t D, uint32_t n, uint32_t g0,
                                              int groups, uint32_t ng, int lane, uint32_t k0,
                                              uint32_t k1, uint32_t tag0, uint32_t tag1,
                                              uint8_t* __restrict__ dst_sample,
                                              float* __restrict__ header)
{
    constexpr float kB = static_cast<float>((1 << B) - 1);
    float v[kTileGroups][4];
    bool ok[kTileGroups][4];
#pragma unroll
    for (int u = 0; u < kTileGroups; ++u)
        if (u < groups)
            load_group<T, VEC>(xs, (static_cast<int64_t>(g0 + u) << 8) + lane * 4, D, v[u], ok[u]);

#pragma unroll
    for (int u = 0; u < kTileGroups; ++u) {
        if (u >= groups) continue;
        const uint32_t g = g0 + u;
        float lo, hi;
        lane_min_max<VEC>(v[u], ok[u], lo, hi);
        const float mn = wave_min(lo) + 0.0f;
        const float range = wave_max(hi) - mn;
        float inv = kB / range;
        float scale = range / kB;
        if (!(range != 0.0f) || !__builtin_isfinite(inv)) {
            inv = 0.0f;
            scale = 0.0f;
        }
        if (lane == 0) {
            f32x2 h;
            h.x = mn;
            h.y = scale;
            *reinterpret_cast<f32x2*>(header + 2 * (static_cast<int64_t>(n) * ng + g)) = h;
        }

        // noise: one Philox call covers 4 (24-bit) or 8 (16-bit) consecutive features
        uint32_t r[4];
        const uint32_t d0 = (g << 8) + lane * 4;  // feature index of the lane's first element, < 2^34 / ... see launcher
        uint32_t rnd[4];
        if (NOISE_BITS == 24) {
            philox4x32_10((g << 6) + lane, n, tag0, tag1, k0, k1, r);
#pragma unroll
            for (int k = 0; k < 4; ++k) rnd[k] = r[k] >> 8;
        } else {
            philox4x32_10((g << 5) + (lane >> 1), n, tag0, tag1, k0, k1, r);
            const uint32_t wa = (lane & 1) ? r[2] : r[0];
            const uint32_t wb = (lane & 1) ? r[3] : r[1];
            rnd[0] = wa & 0xffffu;
            rnd[1] = wa >> 16;
            rnd[2] = wb & 0xffffu;
            rnd[3] = wb >> 16;
        }
        (void)d0;
        constexpr float kNoiseScale = NOISE_BITS == 24 ? 5.9604644775390625e-08f : 1.52587890625e-05f;

        uint32_t piece = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float centred = v[u][k] - mn;
            float uu = centred * inv;
            uu = fminf(uu, kB);
            const float fl = floorf(uu);
            const float frac = uu - fl;
            const float noise = static_cast<float>(rnd[k]) * kNoiseScale;
            uint32_t q = static_cast<uint32_t>(fl) + (noise < frac ? 1u : 0u);
            if (!VEC) q = ok[u][k] ? q : 0u;
            piece |= q << (k * B);
        }
        const uint32_t word = gather_word<B>(piece, lane);
        constexpr int lanes_per_word = 8 / B;
        if ((lane & (lanes_per_word - 1)) == 0) {
            uint32_t* dst = reinterpret_cast<uint32_t*>(dst_sample + static_cast<uint64_t>(g) * (32 * B));
            dst[lane / lanes_per_word] = word;
        }
    }
}

template <typename T, int NOISE_BITS, bool VEC>
__global__ __launch_bounds__(kBlock) void quantize_pack_kernel(
    const T* __restrict__ x, Geometry geo, const uint8_t* __restrict__ bits,
    const uint64_t* __restrict__ offsets, uint32_t k0, uint32_t k1, uint32_t tag0, uint32_t tag1,
    uint8_t* __restrict__ packed, uint64_t capacity, float* __restrict__ header)
{
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t first = wave_index() * geo.tiles_per_wave;
    if (first >= geo.tiles) return;
    const uint32_t last = min(first + geo.tiles_per_wave, geo.tiles);
    uint32_t n = first / geo.tiles_per_sample;
    uint32_t g0 = (first - n * geo.tiles_per_sample) * kTileGroups;
    for (uint32_t tile = first; tile < last; ++tile) {
        const T* xs = x + static_cast<int64_t>(n) * geo.D;
        const int groups = static_cast<int>(min(static_cast<uint32_t>(kTileGroups), geo.ng - g0));
        const uint32_t b = bits[n];
        const uint64_t off = offsets[n];
        const uint64_t bytes = static_cast<uint64_t>(geo.ng) * 32u * b;
        // a sample whose width or byte range is invalid is skipped, nothing is written
        const bool fits = (off & 3u) == 0 && off <= capacity && bytes <= capacity - off;
        if (fits) {
            uint8_t* dst = packed + off;
            switch (b) {
                case 1: quantize_tile<T, NOISE_BITS, VEC, 1>(xs, geo.D, n, g0, groups, geo.ng, lane, k0, k1, tag0, tag1, dst, header); break;
                case 2: quantize_tile<T, NOISE_BITS, VEC, 2>(xs, geo.D, n, g0, groups, geo.ng, lane, k0, k1, tag0, tag1, dst, header); break;
                case 4: quantize_tile<T, NOISE_BITS, VEC, 4>(xs, geo.D, n, g0, groups, geo.ng, lane, k0, k1, tag0, tag1, dst, header); break;
                case 8: quantize_tile<T, NOISE_BITS, VEC, 8>(xs, geo.D, n, g0, groups, geo.ng, lane, k0, k1, tag0, tag1, dst, header); break;
                default: break;
            }
        }
        g0 += kTileGroups;
        if (g0 >= geo.ng) { g0 = 0; ++n; }
    }
}

// ------------------------------------------------------------------------------------
// Sec. 4.1: h^ = code * scale + Z.

template <typename T, bool VEC, int B>
__device__ __forceinline__ void dequantize_tile(const uint8_t* __restrict__ src_sample,
                                                const float* __restrict__ header, T* os, int64_t D,
                                                uint32_t n, uint32_t g0, int groups, uint32_t ng,
                                                int lane)
{
    constexpr int lanes_per_word = 8 / B;
    constexpr uint32_t code_mask = (1u << B) - 1u;
    uint32_t word[kTileGroups];
    f32x2 hd[kTileGroups];
#pragma unroll
    for (int u = 0; u < kTileGroups; ++u) {
        if (u >= groups) continue;
        const uint32_t g = g0 + u;
        const uint32_t* src = reinterpret_cast<const uint32_t*>(src_sample + static_cast<uint64_t>(g) * (32 * B));
        word[u] = __builtin_nontemporal_load(src + lane / lanes_per_word);
        hd[u] = *reinterpret_cast<const f32x2*>(header + 2 * (static_cast<int64_t>(n) * ng + g));
    }
#pragma unroll
    for (int u = 0; u < kTileGroups; ++u) {
        if (u >= groups) continue;
        const uint32_t g = g0 + u;
        const uint32_t piece = word[u] >> ((lane & (lanes_per_word - 1)) * (4 * B));
        float o[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t q = (piece >> (k * B)) & code_mask;
            o[k] = __builtin_fmaf(static_cast<float>(q), hd[u].y, hd[u].x);
        }
        const int64_t d0 = (static_cast<int64_t>(g) << 8) + lane * 4;
        if (VEC) {
            Io<T>::store4(os + d0, o);
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (d0 + k < D) Io<T>::store1(os + d0 + k, o[k]);
        }
    }
}

template <typename T, bool VEC>
__global__ __launch_bounds__(kBlock) void unpack_dequantize_kernel(
    const uint8_t* __restrict__ packed, uint64_t capacity, const float* __restrict__ header,
    const uint8_t* __restrict__ bits, const uint64_t* __restrict__ offsets, Geometry geo,
    T* __restrict__ out)
{
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t first = wave_index() * geo.tiles_per_wave;
    if (first >= geo.tiles) return;
    const uint32_t last = min(first + geo.tiles_per_wave, geo.tiles);
    uint32_t n = first / geo.tiles_per_sample;
    uint32_t g0 = (first - n * geo.tiles_per_sample) * kTileGroups;
    for (uint32_t tile = first; tile < last; ++tile) {
        T* os = out + static_cast<int64_t>(n) * geo.D;
        const int groups = static_cast<int>(min(static_cast<uint32_t>(kTileGroups), geo.ng - g0));
        const uint32_t b = bits[n];
        const uint64_t off = offsets[n];
        const uint64_t bytes = static_cast<uint64_t>(geo.ng) * 32u * b;
        const bool fits = (off & 3u) == 0 && off <= capacity && bytes <= capacity - off;
        if (fits) {
            const uint8_t* src = packed + off;
            switch (b) {
                case 1: dequantize_tile<T, VEC, 1>(src, header, os, geo.D, n, g0, groups, geo.ng, lane); break;
                case 2: dequantize_tile<T, VEC, 2>(src, header, os, geo.D, n, g0, groups, geo.ng, lane); break;
                case 4: dequantize_tile<T, VEC, 4>(src, header, os, geo.D, n, g0, groups, geo.ng, lane); break;
                case 8: dequantize_tile<T, VEC, 8>(src, header, os, geo.D, n, g0, groups, geo.ng, lane); break;
                default: break;
            }
        }
        g0 += kTileGroups;
        if (g0 >= geo.ng) { g0 = 0; ++n; }
    }
}

// ------------------------------------------------------------------------------------
// Host-side launch geometry.

int make_geometry(const char* who, int64_t N, int64_t D, Geometry* geo, dim3* grid)
{
    const int64_t ng = (D + kGroup - 1) / kGroup;
    const int64_t tps = (ng + kTileGroups - 1) / kTileGroups;
    const int64_t tiles = N * tps;
    if (tiles >= (int64_t(1) << 31)) return fail(ACTQ_EINVAL, "%s: tensor too large for one launch (%lld tiles)", who, (long long)tiles);
    geo->D = D;
    geo->ng = static_cast<uint32_t>(ng);
    geo->tiles_per_sample = static_cast<uint32_t>(tps);
    geo->tiles = static_cast<uint32_t>(tiles);
    // enough wavefronts to fill 256 CUs several times over, at most 8 tiles (32 KiB of
    // binary32 input) per wavefront
    int64_t tpw = tiles / (256 * 4 * 16);
    if (tpw < 1) tpw = 1;
    if (tpw > 8) tpw = 8;
    geo->tiles_per_wave = static_cast<uint32_t>(tpw);
    const int64_t waves = (tiles + tpw - 1) / tpw;
    *grid = dim3(static_cast<unsigned>((waves + kWavesPerBlock - 1) / kWavesPerBlock));
    return ACTQ_OK;
}

int check_launch(const char* who)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ACTQ_EHIP, "%s: launch failed: %s", who, hipGetErrorString(e));
    return ACTQ_OK;
}

// Vector path: every group is full and every sample base keeps the 128-bit alignment.
bool vector_ok(int64_t D) { return D % kGroup == 0; }

}  // namespace

int launch_group_stats(const void* x, int dtype, int64_t N, int64_t D, float* gmin, float* grange,
                       void* stream)
{
    Geometry geo;
    dim3 grid;
    if (int rc = make_geometry("actq_group_stats", N, D, &geo, &grid)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool vec = vector_ok(D);
    if (dtype == ACTQ_F32) {
        auto* p = static_cast<const float*>(x);
        if (vec) group_stats_kernel<float, true><<<grid, kBlock, 0, s>>>(p, geo, gmin, grange);
        else group_stats_kernel<float, false><<<grid, kBlock, 0, s>>>(p, geo, gmin, grange);
    } else {
        auto* p = static_cast<const _Float16*>(x);
        if (vec) group_stats_kernel<_Float16, true><<<grid, kBlock, 0, s>>>(p, geo, gmin, grange);
        else group_stats_kernel<_Float16, false><<<grid, kBlock, 0, s>>>(p, geo, gmin, grange);
    }
    return check_launch("actq_group_stats");
}

template <typename T>
static void launch_quantize_typed(const T* x, const Geometry& geo, dim3 grid, hipStream_t s, bool vec,
                                  int noise_bits, const uint8_t* bits, const uint64_t* offsets,
                                  uint64_t seed, uint64_t tag, uint8_t* packed, uint64_t capacity,
                                  float* header)
{
    const uint32_t k0 = static_cast<uint32_t>(seed), k1 = static_cast<uint32_t>(seed >> 32);
    const uint32_t t0 = static_cast<uint32_t>(tag), t1 = static_cast<uint32_t>(tag >> 32);
    if (noise_bits == 24) {
        if (vec) quantize_pack_kernel<T, 24, true><<<grid, kBlock, 0, s>>>(x, geo, bits, offsets, k0, k1, t0, t1, packed, capacity, header);
        else quantize_pack_kernel<T, 24, false><<<grid, kBlock, 0, s>>>(x, geo, bits, offsets, k0, k1, t0, t1, packed, capacity, header);
    } else {
        if (vec) quantize_pack_kernel<T, 16, true><<<grid, kBlock, 0, s>>>(x, geo, bits, offsets, k0, k1, t0, t1, packed, capacity, header);
        else quantize_pack_kernel<T, 16, false><<<grid, kBlock, 0, s>>>(x, geo, bits, offsets, k0, k1, t0, t1, packed, capacity, header);
    }
}

int launch_quantize_pack(const void* x, int dtype, int64_t N, int64_t D, const uint8_t* bits,
                         const uint64_t* offsets, uint64_t seed, uint64_t tag, int noise_bits,
                         void* packed, uint64_t capacity, float* header, void* stream)
{
    Geometry geo;
    dim3 grid;
    if (int rc = make_geometry("actq_quantize_pack", N, D, &geo, &grid)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool vec = vector_ok(D);
    if (dtype == ACTQ_F32)
        launch_quantize_typed(static_cast<const float*>(x), geo, grid, s, vec, noise_bits, bits, offsets, seed, tag, static_cast<uint8_t*>(packed), capacity, header);
    else
        launch_quantize_typed(static_cast<const _Float16*>(x), geo, grid, s, vec, noise_bits, bits, offsets, seed, tag, static_cast<uint8_t*>(packed), capacity, header);
    return check_launch("actq_quantize_pack");
}

int launch_unpack_dequantize(const void* packed, uint64_t capacity, const float* header,
                             const uint8_t* bits, const uint64_t* offsets, int64_t N, int64_t D,
                             void* out, int out_dtype, void* stream)
{
    Geometry geo;
    dim3 grid;
    if (int rc = make_geometry("actq_unpack_dequantize", N, D, &geo, &grid)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool vec = vector_ok(D);
    auto* pk = static_cast<const uint8_t*>(packed);
    if (out_dtype == ACTQ_F32) {
        auto* o = static_cast<float*>(out);
        if (vec) unpack_dequantize_kernel<float, true><<<grid, kBlock, 0, s>>>(pk, capacity, header, bits, offsets, geo, o);
        else unpack_dequantize_kernel<float, false><<<grid, kBlock, 0, s>>>(pk, capacity, header, bits, offsets, geo, o);
    } else {
        auto* o = static_cast<_Float16*>(out);
        if (vec) unpack_dequantize_kernel<_Float16, true><<<grid, kBlock, 0, s>>>(pk, capacity, header, bits, offsets, geo, o);
        else unpack_dequantize_kernel<_Float16, false><<<grid, kBlock, 0, s>>>(pk, capacity, header, bits, offsets, geo, o);
    }
    return check_launch("actq_unpack_dequantize");
}

}  // namespace actq
