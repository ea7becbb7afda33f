// HIP kernels of libactq for gfx950 (MI355X): per-group min/range, stochastic rounding
// with Philox4x32-10 noise, bit-stream packing, and unpack + dequantize (ActNN,
// Sec. 4.1 and Sec. 5.1).
//
// Work decomposition.  The group size is 256 = one 64-lane wavefront x 4 consecutive
// elements per lane, so one 128-bit load per lane brings in a whole group.  A *tile* is
// four consecutive groups of one sample (4 KiB of binary32 input, four loads in flight per
// lane); tiles never cross a sample, so the width b_n is uniform over a tile and every
// branch on it is divergence-free.  One wavefront handles one tile and exits: on this part
// many short-lived wavefronts stream HBM faster than a few long-lived ones.
//
// The path is bound by HBM only if the integer work of the noise generator stays hidden,
// so the per-group bookkeeping is kept off the vector ALU as far as possible:
//   * the min and max of the four groups are reduced *together*: eight partial values per
//     lane are folded by a transposing butterfly (v_permlane32_swap, v_permlane16_swap,
//     DPP row_ror:8) that halves the number of live values at every step, so the whole
//     tile costs 18 cross-lane operations instead of 48, and group g's result lands in
//     row g (lanes 16g..16g+15) of the wavefront;
//   * the two IEEE divisions per group (B / R and R / B) are therefore done once per tile,
//     each row working on its own group, and broadcast with v_readlane;
//   * packed codes go through a wavefront-private LDS slice so that the bit stream leaves
//     as one fully coalesced store per tile whatever the width.
// The quantizer has two more kernels for the cases that carry the traffic (full groups, binary32
// header; see quantize_run_f16 and quantize_tile_f32): there the tile is loaded in address order,
// dealt through the LDS so that a lane holds a contiguous piece of one group, and the lane keeps
// its noise, its share of the reduction and its bytes of the bit stream to itself.
//
// Beyond the arithmetic, four things about the memory system decide the speed (all measured
// on tensors that do not fit the caches):
//   * small writes that reach HBM in the middle of a read stream are expensive out of all
//     proportion (the statistics, 0.8 % of the bytes, cost 10 % of the time): they are issued
//     as ordinary cached stores and the tiles are dealt to the eight XCDs in long runs, so that
//     whole lines of them collect in one L2 (wave_unit);
//   * a write stream is fastest when every XCD writes every eighth 4 KiB page of it (the
//     dequantizer's order), and a branch between the loads and the stores of a wavefront makes
//     the compiler serialise the stores (dequantize_groups);
//   * the scalar loads at the start of a wavefront are issued in batches (ACTQ_SCALAR_BATCH*);
//   * loads must cover whole cache lines per instruction: four 128-bit loads whose lanes are 64
//     bytes apart cost the binary16 quantizer a third of its time (quantize_run_f16).
//
// This file must be compiled with -ffp-contract=off: the scaling step is a subtraction
// and a multiplication that are rounded separately.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "actq_internal.h"

namespace actq {
namespace {

constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;
constexpr int kBlock = kWave * kWavesPerBlock;
constexpr int kTileGroups = 4;
constexpr int kMaxMulti = ACTQ_MAX_TENSORS_PER_CALL;  // tensors of one multi-tensor launch

// Launch shapes of the multi-tensor kernels (which also serve single binary32 tensors of full
// groups).  Each value was chosen by A/B runs on the 53-tensor ResNet-50 sweep at batch 256,
// alternatives in brackets.
constexpr int kDqGroupsF32 = 4;         // dequantizer: groups per wavefront, binary32 output [2, 1: slower]
constexpr int kDqGroupsF16 = 8;         //              binary16 output: the same 4 KiB per wavefront
constexpr int kDqBlock = 256;           //              threads per block [512 alike; 1024, 128, 64 slower]
constexpr bool kDqVectorHeader = true;  //              group headers by lane-uniform vector loads [scalar loads: 10 % slower on cold data]
constexpr int kDqXcdMap = 1;            //              tiles dealt to the XCDs modulo 8 [plain order: 13 % slower]
constexpr int kDqRun = 1;
constexpr int kGsTiles = 1;             // statistics: tiles per wavefront [2: slower]
constexpr int kGsBlock = 256;           //             threads per block [64 .. 1024: alike or slower]
constexpr int kGsXcdMap = 0;
constexpr int kGsRun = 16;              //             consecutive workgroups' tiles per XCD [1: 5 % slower; 8, 32 near; not powers of two: slower]
constexpr int kQpXcdMap = 0;            // quantizer [tiles modulo 8: slower]
constexpr int kQpRun = 16;              //           [1: 3 % slower; 32 alike]

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

// ------------------------------------------------------------------------------------
// Cross-lane helpers (DPP within a row of 16 lanes, v_readlane across rows).

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v)
{
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xf, 0xf, true));
}

constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7-i inside each 8 lanes
constexpr int kDppXor8 = 0x128;        // row_ror:8, lane i <-> i^8 inside each 16 lanes

typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

// min over lanes {l, l^32} of a (kept in lanes 0..31) and of b (kept in lanes 32..63)
__device__ __forceinline__ float fold32(float a, float b)
{
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return fminf(__uint_as_float(r.x), __uint_as_float(r.y));
}

// min over lanes {l, l^16} of a (kept in rows 0 and 2) and of b (kept in rows 1 and 3)
__device__ __forceinline__ float fold16(float a, float b)
{
    const u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return fminf(__uint_as_float(r.x), __uint_as_float(r.y));
}

// Joint reduction of the four groups of a tile.  lo[u] / hi[u] are the lane-local minimum
// and maximum of group u.  On return every lane of row u (lanes 16u..16u+15) holds the
// wavefront-wide minimum and maximum of group u.  Inputs are finite.
__device__ __forceinline__ void tile_min_max(const float (&lo)[4], const float (&hi)[4], int lane,
                                             float& row_min, float& row_max)
{
    // max(x) = -min(-x): all eight values are folded with min; value 2u is lo[u], 2u+1 is -hi[u]
    float c[4];
    c[0] = fold32(lo[0], lo[2]);    // values 0 | 4
    c[1] = fold32(-hi[0], -hi[2]);  // values 1 | 5
    c[2] = fold32(lo[1], lo[3]);    // values 2 | 6
    c[3] = fold32(-hi[1], -hi[3]);  // values 3 | 7
    float d[2];
    d[0] = fold16(c[0], c[2]);      // value (lane>>4)*2
    d[1] = fold16(c[1], c[3]);      // value (lane>>4)*2 + 1
    const bool upper = (lane & 8) != 0;
    const float keep = upper ? d[1] : d[0];
    const float give = upper ? d[0] : d[1];
    float e = fminf(keep, dpp_f32<kDppXor8>(give));  // value lane>>3, still to fold over lane bits 0..2
    e = fminf(e, dpp_f32<kDppXor1>(e));
    e = fminf(e, dpp_f32<kDppXor2>(e));
    e = fminf(e, dpp_f32<kDppHalfMirror>(e));
    const float other = dpp_f32<kDppXor8>(e);
    row_min = upper ? other : e;
    row_max = -(upper ? e : other);
}

// ------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11), state in registers.  The two three-way exclusive-ors
// of a round are one gfx950 three-input bit operation each (truth table 0x96 = a ^ b ^ c).

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t prod_a = static_cast<uint64_t>(c0) * 0xD2511F53u;
        const uint64_t prod_b = static_cast<uint64_t>(c2) * 0xCD9E8D57u;
        const uint32_t y0 = __builtin_amdgcn_bitop3_b32(static_cast<uint32_t>(prod_b >> 32), c1, k0, 0x96);
        const uint32_t y2 = __builtin_amdgcn_bitop3_b32(static_cast<uint32_t>(prod_a >> 32), c3, k1, 0x96);
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

// Launch geometry.  grid.x covers the tiles of one sample, grid.y * grid.z the samples, so
// no kernel ever divides a linear index.  Everything here is wavefront-uniform.
struct Geometry {
    int64_t D;                  // features per sample
    uint32_t N;                 // samples
    uint32_t ng;                // groups per sample
    uint32_t tiles_per_sample;  // ceil(ng / 4)
    uint32_t grid_y;            // samples per grid.z slice
    uint32_t hdr_mode;          // header: 0 = (Z, R/B) binary32, 1 = (Z, R) bfloat16, 2 = one (Z, R) for the tensor
};

// Tile (inside its sample) and sample of this wavefront; false if it has no work.  One tile per
// wavefront: measured on the stage-1 tensor, longer runs (2, 4, 8 tiles) lose a few per cent, and a
// loop around the tile code keeps the compiler from scheduling it as freely.
__device__ __forceinline__ bool wave_work(const Geometry& geo, uint32_t& n, uint32_t& tile)
{
    const uint32_t wave = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6)));
    n = blockIdx.z * geo.grid_y + blockIdx.y;
    tile = blockIdx.x * kWavesPerBlock + wave;
    return n < geo.N && tile < geo.tiles_per_sample;
}

// Loads the lane's four elements of up to four groups.  VEC: every group of the tensor is
// full and 16-byte (8 for binary16) aligned.  Otherwise every element is guarded.
template <typename T, bool VEC>
__device__ __forceinline__ void load_tile(const T* xs, uint32_t g0, int groups, int lane, int64_t D,
                                          float (&v)[kTileGroups][4], bool (&ok)[kTileGroups][4])
{
#pragma unroll
    for (int u = 0; u < kTileGroups; ++u) {
        const int64_t d0 = (static_cast<int64_t>(g0 + u) << 8) + lane * 4;
        if (VEC) {
            // A group past the end of the sample re-reads the tile's first group (valid memory;
            // its results are never stored): the loads stay unconditional and all four are
            // issued back to back.
            const int64_t d_safe = u < groups ? d0 : (static_cast<int64_t>(g0) << 8) + lane * 4;
            Io<T>::load4(xs + d_safe, v[u]);
            ok[u][0] = ok[u][1] = ok[u][2] = ok[u][3] = true;
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                ok[u][k] = u < groups && d0 + k < D;
                v[u][k] = ok[u][k] ? Io<T>::load1(xs + d0 + k) : 0.0f;
            }
        }
    }
}

// Lane-local minimum and maximum of each group.  Guarded-out elements drop out; a group
// with no valid element in this lane yields (+inf, -inf).
template <bool VEC>
__device__ __forceinline__ void lane_min_max(const float (&v)[kTileGroups][4], const bool (&ok)[kTileGroups][4],
                                             float (&lo)[kTileGroups], float (&hi)[kTileGroups])
{
#pragma unroll
    for (int u = 0; u < kTileGroups; ++u) {
        if (VEC) {
            lo[u] = fminf(fminf(v[u][0], v[u][1]), fminf(v[u][2], v[u][3]));
            hi[u] = fmaxf(fmaxf(v[u][0], v[u][1]), fmaxf(v[u][2], v[u][3]));
        } else {
            lo[u] = __builtin_inff();
            hi[u] = -__builtin_inff();
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                lo[u] = ok[u][k] ? fminf(lo[u], v[u][k]) : lo[u];
                hi[u] = ok[u][k] ? fmaxf(hi[u], v[u][k]) : hi[u];
            }
        }
    }
}

// Loads through the constant address space: for memory that no kernel of this library writes
// while it reads it (widths, offsets, and the headers in the dequantizer).  A wavefront-uniform
// load of this kind goes through the scalar data path whatever the compiler can prove about
// aliasing, which keeps four loads per tile off the vector memory pipeline.
template <typename V>
__device__ __forceinline__ V load_readonly(const V* p)
{
    typedef const V __attribute__((address_space(4))) * constant_ptr;
    return *(constant_ptr)(reinterpret_cast<uintptr_t>(p));
}

// True if the sample's byte range [off, off + bytes) is 32-byte aligned and inside the stream.
__device__ __forceinline__ bool range_ok(uint64_t off, uint64_t bytes, uint64_t capacity)
{
    return (off & 31u) == 0 && off <= capacity && bytes <= capacity - off;
}

// Width of sample n through the scalar data path: the 32-bit word that holds bits[n] (the
// array is 4-byte aligned, so the word shares a page with bits[n] and the load cannot fault
// even when N is not a multiple of four), then a shift.
__device__ __forceinline__ uint32_t load_width(const uint8_t* __restrict__ bits, uint32_t n)
{
    const uint32_t word = load_readonly(reinterpret_cast<const uint32_t*>(bits) + (n >> 2));
    return (word >> ((n & 3u) * 8u)) & 0xffu;
}

// bfloat16 header (Sec. 4.1, last paragraph): the zero point is rounded down and the range,
// taken from the rounded zero point, is rounded up, so every element still scales into [0, B].
// Both return the 16 bits of the bfloat16 value.
__device__ __forceinline__ uint32_t bf16_floor_bits(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u >> 16) + (((u & 0xffffu) != 0 && (u >> 31) != 0) ? 1u : 0u);
}

__device__ __forceinline__ uint32_t bf16_ceil_bits(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u >> 16) + (((u & 0xffffu) != 0 && (u >> 31) == 0) ? 1u : 0u);
}

// (Z, scale = R / B) of group `index` from either header format.
// Header of group `index` as (Z, step R / B).  HDR: 0 = stored as such in binary32; 1 = (Z, R) in
// bfloat16; 2 = one (Z, R) pair in binary32 for the whole tensor, the step being 0 when R is 0
// or B / R overflows (the degenerate rule of the quantizer).
// A zero the compiler cannot see through, in a vector register: added to a wavefront-uniform
// index it keeps the load on the vector memory path.
__device__ __forceinline__ uint32_t vector_zero()
{
    uint32_t z;
    asm volatile("v_mov_b32 %0, 0" : "=v"(z));
    return z;
}

// The same header through the vector memory path: every lane loads the same address.
template <int HDR>
__device__ __forceinline__ f32x2 load_header_vector(const void* __restrict__ header, int64_t index, float kB, uint32_t vzero)
{
    if (HDR == 2) {
        const f32x2 zr = static_cast<const f32x2*>(header)[vzero];
        f32x2 h;
        h.x = zr.x;
        h.y = (zr.y != 0.0f && __builtin_isfinite(kB / zr.y)) ? zr.y / kB : 0.0f;
        return h;
    }
    if (HDR == 1) {
        const uint32_t w = static_cast<const uint32_t*>(header)[index + vzero];
        f32x2 h;
        h.x = __uint_as_float(w << 16);
        h.y = __uint_as_float(w & 0xffff0000u) / kB;
        return h;
    }
    return static_cast<const f32x2*>(header)[index + vzero];
}

template <int HDR>
__device__ __forceinline__ f32x2 load_header(const void* __restrict__ header, int64_t index, float kB)
{
    if (HDR == 2) {
        const f32x2 zr = load_readonly(static_cast<const f32x2*>(header));
        f32x2 h;
        h.x = zr.x;
        h.y = (zr.y != 0.0f && __builtin_isfinite(kB / zr.y)) ? zr.y / kB : 0.0f;
        return h;
    }
    if (HDR == 1) {
        const uint32_t w = load_readonly(static_cast<const uint32_t*>(header) + index);
        f32x2 h;
        h.x = __uint_as_float(w << 16);
        h.y = __uint_as_float(w & 0xffff0000u) / kB;  // IEEE division, as the step R / B is defined
        return h;
    }
    return load_readonly(static_cast<const f32x2*>(header) + index);
}

// ------------------------------------------------------------------------------------
// Sec. 4.1: Z = min, R = max - min per group.

template <typename T, bool VEC>
__global__ __launch_bounds__(kBlock) void group_stats_kernel(const T* __restrict__ x, Geometry geo,
                                                             float* __restrict__ gmin,
                                                             float* __restrict__ grange)
{
    const int lane = threadIdx.x & (kWave - 1);
    uint32_t n, tile;
    if (!wave_work(geo, n, tile)) return;
    const T* xs = x + static_cast<int64_t>(n) * geo.D;
    const uint32_t g0 = tile * kTileGroups;
    const int groups = static_cast<int>(min(static_cast<uint32_t>(kTileGroups), geo.ng - g0));
    float v[kTileGroups][4];
    bool ok[kTileGroups][4];
    load_tile<T, VEC>(xs, g0, groups, lane, geo.D, v, ok);
    float lo[kTileGroups], hi[kTileGroups];
    lane_min_max<VEC>(v, ok, lo, hi);
    float mn, mx;
    tile_min_max(lo, hi, lane, mn, mx);
    mn += 0.0f;  // -0.0 -> +0.0
    const int row = lane >> 4;
    if ((lane & 15) == 0 && row < groups) {
        const int64_t gi = static_cast<int64_t>(n) * geo.ng + g0 + row;
        gmin[gi] = mn;
        grange[gi] = (mx - mn) + 0.0f;  // a zero range is +0.0 whichever zeros the extremes were
    }
}

// ------------------------------------------------------------------------------------
// Sec. 4.1 + Sec. 5.1: scale, round stochastically, pack.

// Orders the compiler's view of a wavefront-private LDS hand-over (write by one lane, read
// by another lane of the same wavefront).  The hardware executes one wavefront's LDS
// instructions in order, so no instruction is emitted.
__device__ __forceinline__ void wave_lds_handover()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Noise words for the lane's four elements of each group of the tile, as integers on a grid
// of 2^NOISE_BITS points.
template <int NOISE_BITS>
__device__ __forceinline__ void tile_noise(uint32_t n, uint32_t g0, int lane, uint32_t k0, uint32_t k1,
                                           uint32_t tag0, uint32_t tag1, uint32_t (&rnd)[kTileGroups][4])
{
    if (NOISE_BITS == 24) {
        // counter = feature index / 4: one call per lane per group
#pragma unroll
        for (int u = 0; u < kTileGroups; ++u) {
            uint32_t r[4];
            philox4x32_10(((g0 + u) << 6) + lane, n, tag0, tag1, k0, k1, r);
#pragma unroll
            for (int k = 0; k < 4; ++k) rnd[u][k] = r[k] >> 8;
        }
    } else {
        // counter = feature index / 8: one call serves two neighbouring lanes of one group.
        // Even lanes generate for group 2p, odd lanes for group 2p+1, and the pair trades
        // the halves it does not need, so each lane makes one call per two groups.
        const bool odd = (lane & 1) != 0;
#pragma unroll
        for (int p = 0; p < kTileGroups / 2; ++p) {
            uint32_t r[4];
            philox4x32_10(((g0 + 2 * p + (odd ? 1u : 0u)) << 5) + (lane >> 1), n, tag0, tag1, k0, k1, r);
            // the partner needs words 2,3 of an even lane's call and words 0,1 of an odd lane's
            const uint32_t got0 = dpp_u32<kDppXor1>(odd ? r[0] : r[2]);
            const uint32_t got1 = dpp_u32<kDppXor1>(odd ? r[1] : r[3]);
            const uint32_t a0 = odd ? got0 : r[0], a1 = odd ? got1 : r[1];  // group 2p
            const uint32_t b0 = odd ? r[2] : got0, b1 = odd ? r[3] : got1;  // group 2p+1
            rnd[2 * p][0] = a0 & 0xffffu; rnd[2 * p][1] = a0 >> 16;
            rnd[2 * p][2] = a1 & 0xffffu; rnd[2 * p][3] = a1 >> 16;
            rnd[2 * p + 1][0] = b0 & 0xffffu; rnd[2 * p + 1][1] = b0 >> 16;
            rnd[2 * p + 1][2] = b1 & 0xffffu; rnd[2 * p + 1][3] = b1 >> 16;
        }
    }
}

// The lane's share of one tile: four elements of each of up to four groups, widened to
// binary32, and which of them exist.
struct TileRegs {
    float v[kTileGroups][4];
    bool ok[kTileGroups][4];
};

template <int NOISE_BITS, bool VEC, int B>
__device__ __forceinline__ void encode_tile(const TileRegs& td, const uint32_t (&rnd)[kTileGroups][4],
                                            float row_min, float row_max, uint32_t n, uint32_t g0,
                                            int groups, uint32_t ng, int lane,
                                            uint8_t* __restrict__ dst_sample,
                                            void* __restrict__ header, uint32_t hdr_mode, uint32_t* stage)
{
    constexpr float kB = static_cast<float>((1 << B) - 1);
    constexpr float kNoiseGrid = 16777216.0f;  // 24-bit noise is compared as an integer with frac * 2^24
    const bool hdr_bf16 = hdr_mode == 1, hdr_tensor = hdr_mode == 2;
    float mn = row_min;
    float range;
    uint32_t zb = 0, rb = 0;
    if (hdr_tensor) {
        // one (Z, R) for the whole tensor, given by the caller: the group's own extremes are not used
        const f32x2 zr = static_cast<const f32x2*>(header)[0];
        mn = zr.x;
        range = zr.y;
    } else if (hdr_bf16) {
        zb = bf16_floor_bits(mn);
        mn = __uint_as_float(zb << 16);
        rb = bf16_ceil_bits(row_max - mn);
        range = __uint_as_float(rb << 16);
        if (!__builtin_isfinite(range)) range = 0.0f;  // rounding up overflowed: degenerate
    } else {
        range = row_max - mn;
    }
    float inv = kB / range;
    float scale = range / kB;
    if (!(range != 0.0f) || !__builtin_isfinite(inv)) {  // constant group, or B / R overflows
        inv = 0.0f;
        scale = 0.0f;
        rb = 0;
    }
    const int row = lane >> 4;
    if (!hdr_tensor && (lane & 15) == 0 && row < groups) {
        const int64_t gi = static_cast<int64_t>(n) * ng + g0 + row;
        if (hdr_bf16) {
            static_cast<uint32_t*>(header)[gi] = zb | (rb << 16);
        } else {
            f32x2 h;
            h.x = mn;
            h.y = scale;
            // an ordinary (cached) store: the 8-byte pairs of neighbouring tiles meet in the L2 and
            // leave as whole lines; as non-temporal stores they reached HBM piecemeal (+2 % on the sweep)
            static_cast<f32x2*>(header)[gi] = h;
        }
    }

    uint32_t piece[kTileGroups];
#pragma unroll
    for (int u = 0; u < kTileGroups; ++u) {
        const float mn_u = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(mn), 16 * u));
        const float inv_u = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(inv), 16 * u));
        piece[u] = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float centred = td.v[u][k] - mn_u;
            float scaled = centred * inv_u;
            scaled = fminf(scaled, kB);  // the two roundings can overshoot B by an ulp
            uint32_t q;
            if (NOISE_BITS == 16) {
                // add and floor: noise * 2^-16 is exact, so the fma is the single binary32
                // addition u + noise; the sum is non-negative, truncation = floor
                q = static_cast<uint32_t>(__builtin_fmaf(static_cast<float>(rnd[u][k]), 1.52587890625e-05f, scaled));
            } else {
                const float frac = __builtin_amdgcn_fractf(scaled);  // exact for scaled >= 0
                q = static_cast<uint32_t>(scaled);                   // truncation = floor
                q += (static_cast<float>(rnd[u][k]) < frac * kNoiseGrid) ? 1u : 0u;
            }
            if (!VEC) q = td.ok[u][k] ? q : 0u;
            piece[u] |= q << (k * B);
        }
    }

    // the bit stream of the tile is 4 * 32 * B contiguous bytes
    uint8_t* dst_tile = dst_sample + static_cast<uint64_t>(g0) * (32 * B);
    if (B == 8) {
#pragma unroll
        for (int u = 0; u < kTileGroups; ++u)
            if (u < groups)
                __builtin_nontemporal_store(piece[u], reinterpret_cast<uint32_t*>(dst_tile) + u * 64 + lane);
    } else if (B == 4) {
        uint16_t* s16 = reinterpret_cast<uint16_t*>(stage);
#pragma unroll
        for (int u = 0; u < kTileGroups; ++u) s16[u * 64 + lane] = static_cast<uint16_t>(piece[u]);
        wave_lds_handover();
        const u32x2 w = reinterpret_cast<const u32x2*>(stage)[lane];
        if (lane * 8 < groups * 128)
            __builtin_nontemporal_store(w, reinterpret_cast<u32x2*>(dst_tile) + lane);
    } else if (B == 2) {
        uint8_t* s8 = reinterpret_cast<uint8_t*>(stage);
#pragma unroll
        for (int u = 0; u < kTileGroups; ++u) s8[u * 64 + lane] = static_cast<uint8_t>(piece[u]);
        wave_lds_handover();
        const uint32_t w = stage[lane];
        if (lane * 4 < groups * 64)
            __builtin_nontemporal_store(w, reinterpret_cast<uint32_t*>(dst_tile) + lane);
    } else if (B != 1) {
        // B = 3, 5, 6, 7: a lane's 4*B bits start at bit 4*B*lane of the group and may cross a
        // 32-bit word.  The lanes OR their bits into the zeroed slice, which then leaves as
        // whole words.
#pragma unroll
        for (int j = 0; j < 4; ++j) stage[j * 64 + lane] = 0u;
        wave_lds_handover();
#pragma unroll
        for (int u = 0; u < kTileGroups; ++u) {
            const uint32_t bit = static_cast<uint32_t>(u) * (256u * B) + static_cast<uint32_t>(lane) * (4u * B);
            const uint32_t word = bit >> 5, shift = bit & 31u;
            __hip_atomic_fetch_or(stage + word, piece[u] << shift, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
            if (shift + 4u * B > 32u)
                __hip_atomic_fetch_or(stage + word + 1, piece[u] >> (32u - shift), __ATOMIC_RELAXED,
                                      __HIP_MEMORY_SCOPE_WAVEFRONT);
        }
        wave_lds_handover();
#pragma unroll
        for (int j = 0; j * 64 < 32 * B; ++j) {
            const int idx = j * 64 + lane;
            if (idx < groups * 8 * B)
                __builtin_nontemporal_store(stage[idx], reinterpret_cast<uint32_t*>(dst_tile) + idx);
        }
    } else {
        // B == 1: a lane holds a nibble per group; neighbours merge into a byte first
        const uint32_t nib = piece[0] | (piece[1] << 8) | (piece[2] << 16) | (piece[3] << 24);
        const uint32_t both = nib | (dpp_u32<kDppXor1>(nib) << 4);  // valid in even lanes
        uint8_t* s8 = reinterpret_cast<uint8_t*>(stage);
        if ((lane & 1) == 0) {
#pragma unroll
            for (int u = 0; u < kTileGroups; ++u) s8[u * 32 + (lane >> 1)] = static_cast<uint8_t>(both >> (8 * u));
        }
        wave_lds_handover();
        const uint16_t w = reinterpret_cast<const uint16_t*>(stage)[lane];
        if (lane * 2 < groups * 32)
            __builtin_nontemporal_store(w, reinterpret_cast<uint16_t*>(dst_tile) + lane);
    }
    wave_lds_handover();  // the slice is reused by the next tile of this wavefront
}

// Geometry of the quantizer's launch.
struct StreamGeometry {
    int64_t D;
    uint32_t N;
    uint32_t ng;
    uint32_t tiles_per_sample;
    uint32_t hdr_mode;        // header: 0 = (Z, R/B) binary32 per group, 1 = (Z, R) bfloat16 per group, 2 = one (Z, R) given
};

// The tile of a wavefront, with the scalar facts of its sample.
struct Cursor {
    uint32_t n, t;   // sample, tile inside the sample
    uint32_t b;      // width of the sample
    uint64_t off;    // byte offset of the sample in the bit stream
};

template <typename T, bool VEC>
__device__ __forceinline__ void fetch(const T* __restrict__ x, const StreamGeometry& geo,
                                      const uint8_t* __restrict__ bits, const uint64_t* __restrict__ offsets,
                                      int lane, Cursor& c, TileRegs& r)
{
    const int groups = static_cast<int>(min(static_cast<uint32_t>(kTileGroups), geo.ng - c.t * kTileGroups));
    load_tile<T, VEC>(x + static_cast<int64_t>(c.n) * geo.D, c.t * kTileGroups, groups, lane, geo.D, r.v, r.ok);
    c.b = load_width(bits, c.n);
    c.off = load_readonly(offsets + c.n);
}

template <int NOISE_BITS, bool VEC>
__device__ __forceinline__ void quantize_one(const TileRegs& r, const Cursor& c, const StreamGeometry& geo,
                                             int lane, uint32_t k0, uint32_t k1, uint32_t tag0, uint32_t tag1,
                                             uint8_t* __restrict__ packed, uint64_t capacity,
                                             void* __restrict__ header, uint32_t* stage)
{
    const uint32_t g0 = c.t * kTileGroups;
    const int groups = static_cast<int>(min(static_cast<uint32_t>(kTileGroups), geo.ng - g0));
    uint32_t rnd[kTileGroups][4];
    tile_noise<NOISE_BITS>(c.n, g0, lane, k0, k1, tag0, tag1, rnd);
    float lo[kTileGroups], hi[kTileGroups];
    lane_min_max<VEC>(r.v, r.ok, lo, hi);
    float row_min, row_max;
    tile_min_max(lo, hi, lane, row_min, row_max);
    row_min += 0.0f;  // -0.0 -> +0.0
    // Pin the order: the tile's HBM loads and the noise come before the wavefront looks at the
    // sample's width and offset.  Without this the early exit below is hoisted to the top and a
    // fresh wavefront first sits through dependent scalar loads before it issues any HBM load.
    uint32_t b = c.b, off_lo = static_cast<uint32_t>(c.off), off_hi = static_cast<uint32_t>(c.off >> 32);
    asm volatile("" : "+v"(row_min), "+v"(b), "+v"(off_lo), "+v"(off_hi));
    b = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(b)));
    const uint64_t off = static_cast<uint64_t>(static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(off_lo)))) |
                         (static_cast<uint64_t>(static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(off_hi)))) << 32);
    // a sample whose width or byte range is invalid is skipped, nothing is written
    const uint64_t bytes = static_cast<uint64_t>(geo.ng) * 32u * b;
    if ((off & 31u) != 0 || off > capacity || bytes > capacity - off) return;
    uint8_t* dst = packed + off;
    switch (b) {
        case 1: encode_tile<NOISE_BITS, VEC, 1>(r, rnd, row_min, row_max, c.n, g0, groups, geo.ng, lane, dst, header, geo.hdr_mode, stage); break;
        case 2: encode_tile<NOISE_BITS, VEC, 2>(r, rnd, row_min, row_max, c.n, g0, groups, geo.ng, lane, dst, header, geo.hdr_mode, stage); break;
        case 3: encode_tile<NOISE_BITS, VEC, 3>(r, rnd, row_min, row_max, c.n, g0, groups, geo.ng, lane, dst, header, geo.hdr_mode, stage); break;
        case 4: encode_tile<NOISE_BITS, VEC, 4>(r, rnd, row_min, row_max, c.n, g0, groups, geo.ng, lane, dst, header, geo.hdr_mode, stage); break;
        case 5: encode_tile<NOISE_BITS, VEC, 5>(r, rnd, row_min, row_max, c.n, g0, groups, geo.ng, lane, dst, header, geo.hdr_mode, stage); break;
        case 6: encode_tile<NOISE_BITS, VEC, 6>(r, rnd, row_min, row_max, c.n, g0, groups, geo.ng, lane, dst, header, geo.hdr_mode, stage); break;
        case 7: encode_tile<NOISE_BITS, VEC, 7>(r, rnd, row_min, row_max, c.n, g0, groups, geo.ng, lane, dst, header, geo.hdr_mode, stage); break;
        case 8: encode_tile<NOISE_BITS, VEC, 8>(r, rnd, row_min, row_max, c.n, g0, groups, geo.ng, lane, dst, header, geo.hdr_mode, stage); break;
        default: break;
    }
}

// ------------------------------------------------------------------------------------
// binary16 input with 16-bit noise and the binary32 header: a lane-to-element map of its own.
//
// With two bytes per element the quantizer is bound by the vector ALU (every SIMD issues all
// the time), so this path exists to issue fewer instructions for the same arithmetic:
//   * a lane works on 32 consecutive elements, so a group is eight lanes and a wavefront
//     takes a run of EIGHT groups: what is paid once per group and lane (the reduction across
//     lanes, the two IEEE divisions, addresses, the header) is spread over twice the elements
//     of the general path's tile.  32 elements are exactly what four Philox calls serve with
//     16-bit noise: a lane uses all words of its own calls and nothing is traded between
//     lanes.  The run's four kilobytes are loaded in address order and dealt to the lanes
//     through the LDS (LDS instructions do not take vector-ALU issue slots);
//   * a lane's 32 codes are 4 B consecutive bytes of the bit stream for every width B, stored
//     by the lane itself: the codes do not pass through the LDS;
//   * minimum and maximum are taken on the packed binary16 pairs as they arrive (min and max
//     of binary16 values are exact in binary16) with the three-operand packed instructions,
//     folded into one packed pair (min, -max) per lane, so the reduction over the eight
//     lanes works on one register with three lane permutations;
//   * the subtraction x - Z reads the binary16 half of the loaded word directly (a
//     mixed-precision fma with the factor 1: fl32(x * 1 - Z) is the separately rounded
//     subtraction), which removes the conversions to binary32 and the half extractions;
//   * the clamp of the scaled value to B = 2^b - 1 is skipped for b <= 7, where it cannot
//     change a code: with r the range and q = fl(B / r) (normal for any binary16 range),
//     fl((x - Z) q) <= fl(r q) <= fl(B (1 + 2^-24)) <= B + ulp(B), and with ulp(B) <= 2^-17
//     the sum B + ulp(B) + (1 - 2^-16) is a binary32 number below B + 1, so the floor is B
//     with or without the clamp.  (For b = 8 one ulp is 2^-16 and the sum reaches 256: the
//     clamp is kept.)
// The arithmetic per element is that of encode_tile, bit for bit.  The last run of a sample
// may hold fewer than eight groups: its spare lanes re-read the sample's last group and store
// nothing.

constexpr int kQpGroupsF16 = 8;   // groups per wavefront
constexpr int kQpStageSlots = 272;   // 16-byte LDS slots per wavefront: the run's 256 pieces and one spare per sixteen

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x3 __attribute__((ext_vector_type(3)));

__device__ __forceinline__ f16x2 as_f16x2(uint32_t u)
{
    f16x2 v;
    __builtin_memcpy(&v, &u, 4);
    return v;
}

__device__ __forceinline__ uint32_t as_u32(f16x2 v)
{
    uint32_t u;
    __builtin_memcpy(&u, &v, 4);
    return u;
}

template <int CTRL>
__device__ __forceinline__ f16x2 dpp_f16x2(f16x2 v)
{
    return as_f16x2(dpp_u32<CTRL>(as_u32(v)));
}

// Minimum over each eight consecutive lanes, per packed half, in every one of the eight.
__device__ __forceinline__ f16x2 eight_lane_min(f16x2 p)
{
    p = __builtin_elementwise_minimum(p, dpp_f16x2<kDppXor1>(p));
    p = __builtin_elementwise_minimum(p, dpp_f16x2<kDppXor2>(p));
    p = __builtin_elementwise_minimum(p, dpp_f16x2<kDppHalfMirror>(p));
    return p;
}

// fl32(half - z) for the low (HIGH = false) or high half of `word`: one instruction, the half is
// widened by the operand selector.  `one` is 1.0f in a register.
template <bool HIGH>
__device__ __forceinline__ float half_minus(uint32_t word, float one, float neg_z)
{
    float r;
    if (HIGH) asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(word), "v"(one), "v"(neg_z));
    else asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel_hi:[1,0,0]" : "=v"(r) : "v"(word), "v"(one), "v"(neg_z));
    return r;
}

// Code of the lane's element j (half j & 1 of loaded word j >> 1, the noise in the same half of
// noise word j >> 1).
template <int B>
__device__ __forceinline__ uint32_t code_f16(const uint32_t (&xw)[16], const uint32_t (&rnd)[16], int j, float one,
                                             float neg_mn, float inv)
{
    constexpr float kB = static_cast<float>((1 << B) - 1);
    const float centred = (j & 1) ? half_minus<true>(xw[j >> 1], one, neg_mn) : half_minus<false>(xw[j >> 1], one, neg_mn);
    float scaled = centred * inv;
    if (B == 8) scaled = fminf(scaled, kB);
    const uint32_t noise = (j & 1) ? rnd[j >> 1] >> 16 : rnd[j >> 1] & 0xffffu;
    return static_cast<uint32_t>(__builtin_fmaf(static_cast<float>(noise), 1.52587890625e-05f, scaled));
}

// The lane's 32 codes, packed LSB first into the B words of `out`.
template <int B>
__device__ __forceinline__ void encode_lane_f16(const uint32_t (&xw)[16], const uint32_t (&rnd)[16], float neg_mn, float inv,
                                                uint32_t (&out)[8])
{
    const float one = 1.0f;
    if constexpr ((B & (B - 1)) == 0) {
        // whole codes per word: word by word, last code first
        constexpr int kPerWord = 32 / B;
#pragma unroll
        for (int w = 0; w < B; ++w) {
            uint32_t acc = 0;
#pragma unroll
            for (int k = kPerWord - 1; k >= 0; --k) {
                const uint32_t q = code_f16<B>(xw, rnd, w * kPerWord + k, one, neg_mn, inv);
                if (k == kPerWord - 1) acc = q;
                else asm("v_lshl_or_b32 %0, %1, %2, %3" : "=v"(acc) : "v"(acc), "n"(B), "v"(q));   // (acc << B) | q, kept one instruction per code
            }
            out[w] = acc;
        }
    } else {
        // codes straddle words
#pragma unroll
        for (int w = 0; w < 8; ++w) out[w] = 0;
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            const uint32_t q = code_f16<B>(xw, rnd, j, one, neg_mn, inv);
            const int w = (j * B) >> 5, sh = (j * B) & 31;
            out[w] |= q << sh;
            if (sh + B > 32) out[w + 1] |= q >> (32 - sh);
            if ((j & 7) == 7) __builtin_amdgcn_sched_barrier(0);   // eight codes at a time keep the temporaries in registers
        }
    }
}

// 4 B bytes of a lane (words w[0 .. B-1]) to a 4-byte aligned address.
template <int B>
__device__ __forceinline__ void store_lane_words(uint8_t* dst, const uint32_t (&w)[8])
{
    typedef u32x4 __attribute__((aligned(4))) u32x4_a4;
    typedef u32x2 __attribute__((aligned(4))) u32x2_a4;
    constexpr int kQuads = B / 4, kRest = B % 4;
#pragma unroll
    for (int h = 0; h < kQuads; ++h) {
        u32x4 v;
        v.x = w[4 * h + 0];
        v.y = w[4 * h + 1];
        v.z = w[4 * h + 2];
        v.w = w[4 * h + 3];
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4_a4*>(dst + 16 * h));
    }
    uint8_t* rest = dst + 16 * kQuads;
    if (kRest == 1) __builtin_nontemporal_store(w[4 * kQuads], reinterpret_cast<uint32_t*>(rest));
    if (kRest == 2) {
        u32x2 v;
        v.x = w[4 * kQuads];
        v.y = w[4 * kQuads + 1];
        __builtin_nontemporal_store(v, reinterpret_cast<u32x2_a4*>(rest));
    }
    if (kRest == 3) {
        u32x2 v;
        v.x = w[4 * kQuads];
        v.y = w[4 * kQuads + 1];
        __builtin_nontemporal_store(v, reinterpret_cast<u32x2_a4*>(rest));
        __builtin_nontemporal_store(w[4 * kQuads + 2], reinterpret_cast<uint32_t*>(rest + 8));
    }
}

template <int B>
__device__ __forceinline__ void encode_store_f16(const uint32_t (&xw)[16], const uint32_t (&rnd)[16], float neg_mn, float inv,
                                                 bool valid, uint8_t* dst)
{
    uint32_t w[8];
    encode_lane_f16<B>(xw, rnd, neg_mn, inv, w);
    // the words are final here, for every lane: left alone, the compiler moves the encoding under the
    // store's condition but keeps the 32 subtractions in front of it, and their results do not fit the registers
#pragma unroll
    for (int k = 0; k < B; ++k) asm volatile("" : "+v"(w[k]));
    if (valid) store_lane_words<B>(dst, w);
}

// A run of up to eight full groups starting at g0 of sample n.  A sample whose width or byte
// range is invalid is skipped, nothing is written.
__device__ __forceinline__ void quantize_run_f16(const _Float16* __restrict__ xs, uint32_t n, uint32_t g0, uint32_t ng,
                                                 int lane, uint32_t k0, uint32_t k1, uint32_t tag0, uint32_t tag1,
                                                 const uint8_t* __restrict__ bits, const uint64_t* __restrict__ offsets,
                                                 uint8_t* __restrict__ packed, uint64_t capacity,
                                                 float* __restrict__ header, u32x4* stage)
{
    // lane l works on elements 32 (l & 7) .. + 31 of group g0 + (l >> 3): bytes 64 l .. 64 l + 63 of the run
    uint32_t g = g0 + (static_cast<uint32_t>(lane) >> 3);
    const bool valid = g < ng;
    g = valid ? g : ng - 1;
    const uint32_t chunk = (g << 3) + (static_cast<uint32_t>(lane) & 7u);   // 64-byte piece of the sample, four noise counters
    // A full run arrives in the order of the addresses (load p takes kilobyte p, lane l its bytes
    // 16 l .. 16 l + 15) and is dealt to the lanes through the LDS further down; loading a lane's own
    // 64 bytes directly costs a third of the kernel's time (121 against 78 us on the ResNet-50 stem
    // tensor: four loads whose lanes are 64 bytes apart touch 32 cache lines each).  Only a sample's
    // last, shorter run is loaded that way.
    const bool full = g0 + kQpGroupsF16 <= ng;   // the same for the whole wavefront
    const uint32_t first = full ? (g0 << 5) + static_cast<uint32_t>(lane) : 4u * chunk;   // in 16-byte pieces of the sample
    const uint32_t step = full ? 64u : 1u;
    const u32x4* src = reinterpret_cast<const u32x4*>(xs);
    u32x4 x[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) x[p] = __builtin_nontemporal_load(src + (static_cast<int64_t>(first) + p * step));
    uint32_t width_word = load_readonly(reinterpret_cast<const uint32_t*>(bits) + (n >> 2));
    uint64_t off = load_readonly(offsets + n);
    // noise: counter = feature index / 8 = 4 chunk and the three after it
    uint32_t rnd[16];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        uint32_t r[4];
        philox4x32_10(4 * chunk + p, n, tag0, tag1, k0, k1, r);
#pragma unroll
        for (int k = 0; k < 4; ++k) rnd[4 * p + k] = r[k];
        // one call after the other (interleaved, the four calls' temporaries cost the eighth wavefront per
        // SIMD), and here, in the shadow of the loads, not behind the look at the sample's width
        asm volatile("" : "+v"(rnd[4 * p]), "+v"(rnd[4 * p + 1]), "+v"(rnd[4 * p + 2]), "+v"(rnd[4 * p + 3]));
        __builtin_amdgcn_sched_barrier(0);
    }
    if (full) {
        // 16-byte piece i of the run sits at slot i + i / 16: one spare slot per 256 bytes, so that the
        // sixteen lanes the LDS serves at a time hit every bank once on the way in and on the way out
#pragma unroll
        for (int p = 0; p < 4; ++p) stage[68 * p + lane + (lane >> 4)] = x[p];
        wave_lds_handover();
#pragma unroll
        for (int p = 0; p < 4; ++p) x[p] = stage[4 * lane + p + (lane >> 2)];
    }
    uint32_t xw[16];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        xw[4 * p + 0] = x[p].x;
        xw[4 * p + 1] = x[p].y;
        xw[4 * p + 2] = x[p].z;
        xw[4 * p + 3] = x[p].w;
    }
    // lane-local minimum and maximum per packed half, then (min, -max) as one pair over the eight lanes
    f16x2 lo2 = as_f16x2(xw[0]), hi2 = as_f16x2(xw[0]);
#pragma unroll
    for (int k = 1; k < 16; ++k) {
        lo2 = __builtin_elementwise_minimum(lo2, as_f16x2(xw[k]));
        hi2 = __builtin_elementwise_maximum(hi2, as_f16x2(xw[k]));
    }
    f16x2 a, b2;
    a[0] = lo2[0]; a[1] = -hi2[0];
    b2[0] = lo2[1]; b2[1] = -hi2[1];
    const f16x2 fold = eight_lane_min(__builtin_elementwise_minimum(a, b2));
    const float mn = static_cast<float>(fold[0]) + 0.0f;   // -0.0 -> +0.0
    const float mx = -static_cast<float>(fold[1]);
    asm volatile("" : "+s"(width_word), "+s"(off));   // the scalar loads are waited for here, behind the noise
    const uint32_t b = (width_word >> ((n & 3u) * 8u)) & 0xffu;
    if (b < 1 || b > 8 || !range_ok(off, static_cast<uint64_t>(ng) * 32u * b, capacity)) return;
    const float kB = static_cast<float>((1u << b) - 1u);
    const float range = mx - mn;
    // one IEEE division for both quotients: lanes 0..3 of a group take B / R, lanes 4..7 R / B, and trade
    const bool inv_side = (lane & 4) == 0;
    const float quotient = (inv_side ? kB : range) / (inv_side ? range : kB);
    const float traded = dpp_f32<kDppHalfMirror>(quotient);
    float inv = inv_side ? quotient : traded;
    float scale = inv_side ? traded : quotient;
    if (!(range != 0.0f) || !__builtin_isfinite(inv)) {   // constant group, or B / R overflows
        inv = 0.0f;
        scale = 0.0f;
    }
    uint8_t* dst = packed + off + static_cast<uint64_t>(chunk) * (4u * b);
    switch (b) {
        case 1: encode_store_f16<1>(xw, rnd, -mn, inv, valid, dst); break;
        case 2: encode_store_f16<2>(xw, rnd, -mn, inv, valid, dst); break;
        case 3: encode_store_f16<3>(xw, rnd, -mn, inv, valid, dst); break;
        case 4: encode_store_f16<4>(xw, rnd, -mn, inv, valid, dst); break;
        case 5: encode_store_f16<5>(xw, rnd, -mn, inv, valid, dst); break;
        case 6: encode_store_f16<6>(xw, rnd, -mn, inv, valid, dst); break;
        case 7: encode_store_f16<7>(xw, rnd, -mn, inv, valid, dst); break;
        default: encode_store_f16<8>(xw, rnd, -mn, inv, valid, dst); break;
    }
    if (valid && (lane & 7) == 0) {
        f32x2 h;
        h.x = mn;
        h.y = scale;
        reinterpret_cast<f32x2*>(header)[static_cast<int64_t>(n) * ng + g] = h;
    }
}

// ------------------------------------------------------------------------------------
// binary32 input with the binary32 header: the same lane-to-element map for four-byte elements.
//
// A lane works on SIXTEEN consecutive elements, a group is one row of sixteen lanes and a
// wavefront takes the tile's four groups: the four kilobytes are loaded in address order and
// dealt to the lanes through the LDS exactly as above.  Sixteen elements are what two Philox
// calls serve with 16-bit noise and four with 24-bit noise, so again nothing is traded between
// lanes; the reduction is four row-local lane permutations on the lane's own minimum and
// maximum; the division pair is per row.  A lane's sixteen codes are 2 B consecutive bytes of
// the bit stream: two neighbouring lanes join theirs (for odd B the odd lane's bits are moved
// up by sixteen) and the even lane stores the 4 B bytes.
// The clamp stays for every width: B / R can be subnormal for a binary32 range, and then the
// bound used above for binary16 input does not hold.

// Minimum over the sixteen lanes of each row, in every lane of the row.
__device__ __forceinline__ float row_min_f32(float v)
{
    v = fminf(v, dpp_f32<kDppXor1>(v));
    v = fminf(v, dpp_f32<kDppXor2>(v));
    v = fminf(v, dpp_f32<kDppHalfMirror>(v));
    v = fminf(v, dpp_f32<kDppXor8>(v));
    return v;
}

// Code of element j of the lane.  16-bit noise: half j & 1 of noise word j >> 1; 24-bit noise: the
// upper 24 bits of noise word j.
template <int NOISE_BITS, int B>
__device__ __forceinline__ uint32_t code_f32(float x, const uint32_t* rnd, int j, float mn, float inv)
{
    constexpr float kB = static_cast<float>((1 << B) - 1);
    const float centred = x - mn;
    float scaled = centred * inv;
    scaled = fminf(scaled, kB);  // the two roundings can overshoot B by an ulp
    if (NOISE_BITS == 16) {
        const uint32_t noise = (j & 1) ? rnd[j >> 1] >> 16 : rnd[j >> 1] & 0xffffu;
        return static_cast<uint32_t>(__builtin_fmaf(static_cast<float>(noise), 1.52587890625e-05f, scaled));
    }
    const float frac = __builtin_amdgcn_fractf(scaled);  // exact for scaled >= 0
    const uint32_t q = static_cast<uint32_t>(scaled);    // truncation = floor
    return q + ((static_cast<float>(rnd[j] >> 8) < frac * 16777216.0f) ? 1u : 0u);
}

// The lane's sixteen codes, packed LSB first: 16 B bits in out[0 .. (B + 1) / 2 - 1], upper bits zero.
template <int NOISE_BITS, int B>
__device__ __forceinline__ void encode_lane_f32(const float (&v)[16], const uint32_t* rnd, float mn, float inv, uint32_t (&out)[4])
{
#pragma unroll
    for (int w = 0; w < 4; ++w) out[w] = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const uint32_t q = code_f32<NOISE_BITS, B>(v[j], rnd, j, mn, inv);
        const int w = (j * B) >> 5, sh = (j * B) & 31;
        out[w] |= q << sh;
        if (sh + B > 32) out[w + 1] |= q >> (32 - sh);
    }
}

template <int NOISE_BITS, int B>
__device__ __forceinline__ void encode_store_f32(const float (&v)[16], const uint32_t* rnd, float mn, float inv,
                                                 bool valid, int lane, uint8_t* dst_pair)
{
    uint32_t own[4];
    encode_lane_f32<NOISE_BITS, B>(v, rnd, mn, inv, own);
    constexpr int kOwn = (B + 1) / 2;   // words that hold the lane's 16 B bits
    uint32_t nb[4] = {0, 0, 0, 0};
#pragma unroll
    for (int k = 0; k < kOwn; ++k) nb[k] = dpp_u32<kDppXor1>(own[k]);   // the neighbour's words (used by the even lane)
    uint32_t w[8];
    if (B % 2 == 0) {
#pragma unroll
        for (int k = 0; k < kOwn; ++k) {
            w[k] = own[k];
            w[kOwn + k] = nb[k];
        }
    } else {
        // own bits end in the middle of word kOwn - 1: the neighbour's follow from bit 16 of it
#pragma unroll
        for (int k = 0; k < kOwn - 1; ++k) w[k] = own[k];
        w[kOwn - 1] = own[kOwn - 1] | (nb[0] << 16);
#pragma unroll
        for (int k = 0; k + 1 < kOwn; ++k) w[kOwn + k] = __builtin_amdgcn_alignbit(nb[k + 1], nb[k], 16);
    }
    // the words are final here, for every lane (see encode_store_f16)
#pragma unroll
    for (int k = 0; k < B; ++k) asm volatile("" : "+v"(w[k]));
    if (valid && (lane & 1) == 0) store_lane_words<B>(dst_pair, w);
}

// The tile of up to four full groups starting at g0 of sample n.  A sample whose width or byte
// range is invalid is skipped, nothing is written.
template <int NOISE_BITS>
__device__ __forceinline__ void quantize_tile_f32(const float* __restrict__ xs, uint32_t n, uint32_t g0, uint32_t ng,
                                                  int lane, uint32_t k0, uint32_t k1, uint32_t tag0, uint32_t tag1,
                                                  const uint8_t* __restrict__ bits, const uint64_t* __restrict__ offsets,
                                                  uint8_t* __restrict__ packed, uint64_t capacity,
                                                  float* __restrict__ header, u32x4* stage)
{
    // lane l works on elements 16 (l & 15) .. + 15 of group g0 + (l >> 4): bytes 64 l .. 64 l + 63 of the tile
    uint32_t g = g0 + (static_cast<uint32_t>(lane) >> 4);
    const bool valid = g < ng;
    g = valid ? g : ng - 1;
    const uint32_t chunk = (g << 4) + (static_cast<uint32_t>(lane) & 15u);   // 64-byte piece of the sample
    const bool full = g0 + kTileGroups <= ng;   // the same for the whole wavefront
    const uint32_t first = full ? (g0 << 6) + static_cast<uint32_t>(lane) : 4u * chunk;   // in 16-byte pieces of the sample
    const uint32_t step = full ? 64u : 1u;
    const u32x4* src = reinterpret_cast<const u32x4*>(xs);
    u32x4 x[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) x[p] = __builtin_nontemporal_load(src + (static_cast<int64_t>(first) + p * step));
    uint32_t width_word = load_readonly(reinterpret_cast<const uint32_t*>(bits) + (n >> 2));
    uint64_t off = load_readonly(offsets + n);
    // noise: counter = feature index / 8 (16-bit noise: two calls) or / 4 (24-bit noise: four calls)
    constexpr int kCalls = NOISE_BITS == 16 ? 2 : 4;
    uint32_t rnd[4 * kCalls];
#pragma unroll
    for (int p = 0; p < kCalls; ++p) {
        uint32_t r[4];
        philox4x32_10(kCalls * chunk + p, n, tag0, tag1, k0, k1, r);
#pragma unroll
        for (int k = 0; k < 4; ++k) rnd[4 * p + k] = r[k];
        // one call after the other, in the shadow of the loads (see quantize_run_f16)
        asm volatile("" : "+v"(rnd[4 * p]), "+v"(rnd[4 * p + 1]), "+v"(rnd[4 * p + 2]), "+v"(rnd[4 * p + 3]));
        __builtin_amdgcn_sched_barrier(0);
    }
    if (full) {
#pragma unroll
        for (int p = 0; p < 4; ++p) stage[68 * p + lane + (lane >> 4)] = x[p];
        wave_lds_handover();
#pragma unroll
        for (int p = 0; p < 4; ++p) x[p] = stage[4 * lane + p + (lane >> 2)];
    }
    float v[16];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        v[4 * p + 0] = __uint_as_float(x[p].x);
        v[4 * p + 1] = __uint_as_float(x[p].y);
        v[4 * p + 2] = __uint_as_float(x[p].z);
        v[4 * p + 3] = __uint_as_float(x[p].w);
    }
    float lo = v[0], hi = v[0];
#pragma unroll
    for (int k = 1; k < 16; ++k) {
        lo = fminf(lo, v[k]);
        hi = fmaxf(hi, v[k]);
    }
    const float mn = row_min_f32(lo) + 0.0f;   // -0.0 -> +0.0
    const float mx = -row_min_f32(-hi);
    asm volatile("" : "+s"(width_word), "+s"(off));   // the scalar loads are waited for here, behind the noise
    const uint32_t b = (width_word >> ((n & 3u) * 8u)) & 0xffu;
    if (b < 1 || b > 8 || !range_ok(off, static_cast<uint64_t>(ng) * 32u * b, capacity)) return;
    const float kB = static_cast<float>((1u << b) - 1u);
    const float range = mx - mn;
    // one IEEE division for both quotients: lanes 0..7 of a row take B / R, lanes 8..15 R / B, and trade
    const bool inv_side = (lane & 8) == 0;
    const float quotient = (inv_side ? kB : range) / (inv_side ? range : kB);
    const float traded = dpp_f32<kDppXor8>(quotient);
    float inv = inv_side ? quotient : traded;
    float scale = inv_side ? traded : quotient;
    if (!(range != 0.0f) || !__builtin_isfinite(inv)) {   // constant group, or B / R overflows
        inv = 0.0f;
        scale = 0.0f;
    }
    // the even lane of a pair stores both lanes' bytes: 4 b bytes from byte 2 b chunk of the sample's stream
    uint8_t* dst = packed + off + static_cast<uint64_t>(chunk) * (2u * b);
    switch (b) {
        case 1: encode_store_f32<NOISE_BITS, 1>(v, rnd, mn, inv, valid, lane, dst); break;
        case 2: encode_store_f32<NOISE_BITS, 2>(v, rnd, mn, inv, valid, lane, dst); break;
        case 3: encode_store_f32<NOISE_BITS, 3>(v, rnd, mn, inv, valid, lane, dst); break;
        case 4: encode_store_f32<NOISE_BITS, 4>(v, rnd, mn, inv, valid, lane, dst); break;
        case 5: encode_store_f32<NOISE_BITS, 5>(v, rnd, mn, inv, valid, lane, dst); break;
        case 6: encode_store_f32<NOISE_BITS, 6>(v, rnd, mn, inv, valid, lane, dst); break;
        case 7: encode_store_f32<NOISE_BITS, 7>(v, rnd, mn, inv, valid, lane, dst); break;
        default: encode_store_f32<NOISE_BITS, 8>(v, rnd, mn, inv, valid, lane, dst); break;
    }
    if (valid && (lane & 15) == 0) {
        f32x2 h;
        h.x = mn;
        h.y = scale;
        reinterpret_cast<f32x2*>(header)[static_cast<int64_t>(n) * ng + g] = h;
    }
}

// One tile per wavefront (grid.x = tiles of a sample, grid.y * grid.z = samples).  Short-lived
// wavefronts lose the least HBM bandwidth to the small writes of codes and headers, and the
// other resident wavefronts' loads hide a tile's ALU work.  (A persistent software pipeline
// -- as many wavefronts as the chip holds, each striding over the tiles with the next tile's
// loads in flight while the current one is encoded -- measured slower in every mode: 80
// against 70 us with 16-bit noise, 96 against 83 us with 24-bit noise on the stage-1 tensor.)
template <typename T, int NOISE_BITS, bool VEC>
__global__ __launch_bounds__(kBlock) void quantize_pack_tile_kernel(
    const T* __restrict__ x, StreamGeometry geo, uint32_t grid_y, const uint8_t* __restrict__ bits,
    const uint64_t* __restrict__ offsets, uint32_t k0, uint32_t k1, uint32_t tag0, uint32_t tag1,
    uint8_t* __restrict__ packed, uint64_t capacity, void* __restrict__ header)
{
    __shared__ uint32_t stage_all[kWavesPerBlock][256];
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t wave_in_block = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6)));
    Cursor c;
    c.n = blockIdx.z * grid_y + blockIdx.y;
    c.t = blockIdx.x * kWavesPerBlock + wave_in_block;
    if (c.n >= geo.N || c.t >= geo.tiles_per_sample) return;
    TileRegs r;
    fetch<T, VEC>(x, geo, bits, offsets, lane, c, r);
    quantize_one<NOISE_BITS, VEC>(r, c, geo, lane, k0, k1, tag0, tag1, packed, capacity, header, stage_all[wave_in_block]);
}

// ------------------------------------------------------------------------------------
// Sec. 4.1: h^ = code * scale + Z.

// NG consecutive groups of one sample, all of them present: straight-line code, every load is
// issued before the first store and nothing branches in between.  (A branch around a load or a
// store makes the compiler wait for *all* outstanding vector memory operations where the paths
// join -- and on this target a store counts until it is acknowledged, so the stores of a
// wavefront would go out one at a time.)
template <typename T, bool VEC, int B, int HDR, int NG, bool VHDR>
__device__ __forceinline__ void dequantize_groups(const uint8_t* __restrict__ src_sample,
                                                  const void* __restrict__ header, T* __restrict__ os,
                                                  int64_t D, uint32_t n, uint32_t g0, uint32_t ng,
                                                  int lane, uint32_t* stage)
{
    // a lane's four codes are the 4*B bits that start at bit 4*B*lane of the group: inside one
    // 32-bit word when B divides 8, possibly across two words otherwise
    constexpr bool kAligned = (8 % B) == 0;
    constexpr uint32_t code_mask = (1u << B) - 1u;
    const uint32_t first_word = static_cast<uint32_t>(lane) * (4u * B) >> 5;
    const uint32_t shift = static_cast<uint32_t>(lane) * (4u * B) & 31u;
    uint32_t word[NG], next[NG];
    f32x2 hd[NG];
    uint32_t vzero = 0;
    if (VHDR) vzero = vector_zero();
    const int64_t hdr0 = static_cast<int64_t>(n) * ng + g0;
    const uint32_t* tile_src = reinterpret_cast<const uint32_t*>(src_sample + static_cast<uint64_t>(g0) * (32 * B));
    if (!kAligned) {
        // The bit stream of the NG groups (NG * 32 * B contiguous bytes) comes in with coalesced
        // word loads and is handed over through the wavefront's LDS slice; every lane then picks
        // the two words that hold its bits.
        constexpr int kWords = NG * 8 * B;
        constexpr int kLoads = (kWords + 63) / 64;
        uint32_t in[kLoads];
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            const int idx = min(j * 64 + lane, kWords - 1);  // clamped: lanes past the end re-read the last word
            in[j] = __builtin_nontemporal_load(tile_src + idx);
        }
#pragma unroll
        for (int u = 0; u < NG; ++u)
            hd[u] = VHDR ? load_header_vector<HDR>(header, hdr0 + u, static_cast<float>(code_mask), vzero)
                         : load_header<HDR>(header, hdr0 + u, static_cast<float>(code_mask));
#pragma unroll
        for (int j = 0; j < kLoads; ++j) stage[j * 64 + lane] = in[j];  // at most 256 words
        wave_lds_handover();
#pragma unroll
        for (int u = 0; u < NG; ++u) {
            // past the last word the neighbour is never used: those lanes' bits end with the word
            word[u] = stage[u * 8 * B + first_word];
            next[u] = stage[u * 8 * B + first_word + 1];
        }
        wave_lds_handover();  // the slice is reused by the next call of this wavefront
    } else {
#pragma unroll
        for (int u = 0; u < NG; ++u) {
            word[u] = __builtin_nontemporal_load(tile_src + u * 8 * B + first_word);
            hd[u] = VHDR ? load_header_vector<HDR>(header, hdr0 + u, static_cast<float>(code_mask), vzero)
                         : load_header<HDR>(header, hdr0 + u, static_cast<float>(code_mask));
        }
    }
#pragma unroll
    for (int u = 0; u < NG; ++u) {
        const uint32_t piece = kAligned ? word[u] >> shift : __builtin_amdgcn_alignbit(next[u], word[u], shift);
        float o[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t q = (piece >> (k * B)) & code_mask;
            o[k] = __builtin_fmaf(static_cast<float>(q), hd[u].y, hd[u].x);
        }
        const int64_t d0 = (static_cast<int64_t>(g0 + u) << 8) + lane * 4;
        if (VEC) {
            Io<T>::store4(os + d0, o);
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (d0 + k < D) Io<T>::store1(os + d0 + k, o[k]);
        }
    }
}

// binary16 output: a lane that owned four elements would store only 8 bytes, so here a lane
// takes eight consecutive elements (16 bytes) and the wavefront covers two groups per step
// (lanes 0..31 the even group, lanes 32..63 the odd one).  Unpacking is free to choose its
// lane-to-element map: nothing is reduced across lanes.
template <bool VEC, int B, int HDR, int NP = 2, bool ALL = false>
__device__ __forceinline__ void dequantize_tile_f16(const uint8_t* __restrict__ src_sample,
                                                    const void* __restrict__ header,
                                                    _Float16* __restrict__ os, int64_t D, uint32_t n, uint32_t g0,
                                                    int groups, uint32_t ng, int lane)
{
    typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
    constexpr uint32_t code_mask = (1u << B) - 1u;
    const int half = lane >> 5;   // which group of the pair
    const int li = lane & 31;     // position inside the group: elements 8*li .. 8*li+7
    uint32_t code_lo[NP], code_hi[NP];  // 8*B bits per lane; the high word only for B = 8
    f32x2 hd[NP];
    bool live[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        code_lo[p] = code_hi[p] = 0;
        const int u = 2 * p + half;
        live[p] = ALL || u < groups;                // ALL: every group of the run is present, nothing branches
        const uint32_t g = g0 + (live[p] ? u : 0);  // a dead lane re-reads the tile's first group
        const uint8_t* src = src_sample + static_cast<uint64_t>(g) * (32 * B) + li * B;  // 8*B bits per lane
        if (B < 4) {
            // the aligned word around the lane's 8*B bits (a group's stream starts 32-byte aligned)
            const uint32_t word = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(src - ((li * B) & 3)));
            code_lo[p] = word >> (((li * B) & 3) * 8);
        }
        if (B == 4) code_lo[p] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(src));
        if (B == 8) {
            const u32x2 w = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(src));
            code_lo[p] = w.x;
            code_hi[p] = w.y;
        }
        // both groups' headers through the scalar data path (their indices are uniform), then the
        // lane's half picks one: a per-lane load would be a second vector load in front of each store
        const int u_even = (ALL || 2 * p < groups) ? 2 * p : 0, u_odd = (ALL || 2 * p + 1 < groups) ? 2 * p + 1 : 0;
        const f32x2 hd_even = load_header<HDR>(header, static_cast<int64_t>(n) * ng + g0 + u_even, static_cast<float>(code_mask));
        const f32x2 hd_odd = load_header<HDR>(header, static_cast<int64_t>(n) * ng + g0 + u_odd, static_cast<float>(code_mask));
        hd[p].x = half ? hd_odd.x : hd_even.x;
        hd[p].y = half ? hd_odd.y : hd_even.y;
    }
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const uint32_t g = g0 + 2 * p + half;
        f16x8 o;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const uint32_t word = (k * B < 32) ? code_lo[p] : code_hi[p];
            const uint32_t q = (word >> ((k * B) & 31)) & code_mask;
            o[k] = Io<_Float16>::narrow(__builtin_fmaf(static_cast<float>(q), hd[p].y, hd[p].x));
        }
        const int64_t d0 = (static_cast<int64_t>(g) << 8) + li * 8;
        if (!live[p]) continue;
        if (VEC) {
            __builtin_nontemporal_store(o, reinterpret_cast<f16x8*>(os + d0));
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (d0 + k < D) os[d0 + k] = o[k];
        }
    }
}

// `groups` (1..NG) groups starting at g0.  All NG present: the straight-line code; the last,
// shorter run of a sample goes group by group.
template <typename T, bool VEC, int B, int HDR, int NG = kTileGroups, bool VHDR = false>
__device__ __forceinline__ void dequantize_any(const uint8_t* __restrict__ src_sample,
                                               const void* __restrict__ header, T* __restrict__ os,
                                               int64_t D, uint32_t n, uint32_t g0, int groups, uint32_t ng, int lane,
                                               uint32_t* stage)
{
    if constexpr (sizeof(T) == 2 && (8 % B) == 0 && NG % 2 == 0) {
        if (groups == NG) dequantize_tile_f16<VEC, B, HDR, NG / 2, true>(src_sample, header, os, D, n, g0, groups, ng, lane);
        else dequantize_tile_f16<VEC, B, HDR, NG / 2, false>(src_sample, header, os, D, n, g0, groups, ng, lane);
    } else {
        // at most four groups at a time: the LDS slice of a wavefront holds 256 words
        constexpr int kStep = NG < kTileGroups ? NG : kTileGroups;
        static_assert(NG % kStep == 0, "whole steps");
        if (groups == NG) {
#pragma unroll
            for (int t = 0; t < NG / kStep; ++t)
                dequantize_groups<T, VEC, B, HDR, kStep, VHDR>(src_sample, header, os, D, n, g0 + t * kStep, ng, lane, stage);
        } else {
            for (int u = 0; u < groups; ++u)
                dequantize_groups<T, VEC, B, HDR, 1, VHDR>(src_sample, header, os, D, n, g0 + u, ng, lane, stage);
        }
    }
}

template <typename T, bool VEC, int HDR>
__global__ __launch_bounds__(kBlock) void unpack_dequantize_kernel(
    const uint8_t* __restrict__ packed, uint64_t capacity, const void* __restrict__ header,
    const uint8_t* __restrict__ bits, const uint64_t* __restrict__ offsets, Geometry geo,
    T* __restrict__ out)
{
    __shared__ uint32_t stage_all[kWavesPerBlock][256];  // 1 KiB per wavefront, private to it (odd widths)
    const int lane = threadIdx.x & (kWave - 1);
    uint32_t* stage = stage_all[threadIdx.x >> 6];
    uint32_t n, tile;
    if (!wave_work(geo, n, tile)) return;
    T* os = out + static_cast<int64_t>(n) * geo.D;
    const uint32_t b = load_width(bits, n);
    const uint64_t off = load_readonly(offsets + n);
    const uint64_t bytes = static_cast<uint64_t>(geo.ng) * 32u * b;
    if ((off & 31u) != 0 || off > capacity || bytes > capacity - off) return;
    const uint8_t* src = packed + off;
    const uint32_t g0 = tile * kTileGroups;
    const int groups = static_cast<int>(min(static_cast<uint32_t>(kTileGroups), geo.ng - g0));
    switch (b) {
        case 1: dequantize_any<T, VEC, 1, HDR>(src, header, os, geo.D, n, g0, groups, geo.ng, lane, stage); break;
        case 2: dequantize_any<T, VEC, 2, HDR>(src, header, os, geo.D, n, g0, groups, geo.ng, lane, stage); break;
        case 3: dequantize_any<T, VEC, 3, HDR>(src, header, os, geo.D, n, g0, groups, geo.ng, lane, stage); break;
        case 4: dequantize_any<T, VEC, 4, HDR>(src, header, os, geo.D, n, g0, groups, geo.ng, lane, stage); break;
        case 5: dequantize_any<T, VEC, 5, HDR>(src, header, os, geo.D, n, g0, groups, geo.ng, lane, stage); break;
        case 6: dequantize_any<T, VEC, 6, HDR>(src, header, os, geo.D, n, g0, groups, geo.ng, lane, stage); break;
        case 7: dequantize_any<T, VEC, 7, HDR>(src, header, os, geo.D, n, g0, groups, geo.ng, lane, stage); break;
        case 8: dequantize_any<T, VEC, 8, HDR>(src, header, os, geo.D, n, g0, groups, geo.ng, lane, stage); break;
        default: return;
    }
}

// ------------------------------------------------------------------------------------
// Several tensors in one launch.  A network saves dozens of activations of very different
// sizes (a ResNet-50 step: 53, from 26 MB to 822 MB at batch 256); one launch per tensor leaves
// the chip draining and refilling 53 times per pass, and the small tensors cannot fill it at
// all.  Here blockIdx.y is the tensor and blockIdx.x runs over its tiles, sample after sample
// (in an order that depends on the kernel, see wave_unit), so the launch walks HBM like
// back-to-back single-tensor launches, without the gaps.  grid.x is sized for the largest
// tensor of the call and the surplus blocks of smaller ones exit at once, so a call should
// group tensors of similar size.  The start of a wavefront is short: one batch of scalar loads
// for the tensor's item from the kernel arguments, one for the sample's width and offset, then
// the data; a multiply-high division splits the linear tile index into sample and tile.
// (Measured alternatives on the 53-tensor sweep: samples in grid.y with all tensors' tiles side
// by side in grid.x -- 53 concurrent streams -- made every kernel 5-20 % slower than single
// launches; one linear grid over all tensors with a ballot over prefix sums to find the tensor
// costs a vector load at the start of every wavefront, which the write-bound dequantizer does
// not hide: 83 against 73 us on the stage-1 tensor.)
// Every tensor has full groups (D a multiple of 256) and the same N, dtype and header format.

struct MultiItem {
    const void* x;            // input of group_stats / quantize_pack
    void* out;                // output of unpack_dequantize
    float* gmin;              // outputs of group_stats
    float* grange;
    void* header;
    const uint8_t* bits;
    const uint64_t* offsets;
    int64_t D;
    FastDiv by_tiles;         // division by the tiles of one sample
    uint32_t tiles;           // tiles of one sample
    uint32_t total_tiles;     // N * tiles
};

struct MultiTable {
    uint32_t count, N, hdr_mode, pad;
    MultiItem item[kMaxMulti];
};

// Linear work index of wavefront `wave` of block `bx`.  Blocks are handed to the eight XCDs in
// turn, so block bx runs on XCD bx % 8 (grid.x is a multiple of 8 * RUN).
// XCD_MAP 0: RUN consecutive blocks' worth of units (RUN * WAVES units) stay on one XCD -- RUN = 1
//   is the plain order, block bx takes units bx * WAVES ...  A longer run keeps whole cache lines
//   of the small per-group outputs inside one XCD's L2, so that they reach HBM as fewer, fuller writes.
// XCD_MAP 1: every run of 8 blocks shares 8 * WAVES consecutive units and block bx takes the
//   units congruent to bx modulo 8: each XCD then writes every eighth unit of the stream.
template <int WAVES, int XCD_MAP, int RUN = 1>
__device__ __forceinline__ uint32_t wave_unit(uint32_t bx, uint32_t wave)
{
    if (XCD_MAP == 1) return (bx >> 3) * (8 * WAVES) + (bx & 7u) + 8 * wave;
    if (RUN > 1) {
        const uint32_t k = bx >> 3;   // position among the blocks of this XCD
        return (((k / RUN) * 8 + (bx & 7u)) * RUN + (k % RUN)) * WAVES + wave;
    }
    return bx * WAVES + wave;
}

// Makes the listed scalar values live at this point of the program: every scalar load that
// produces them has been issued, and is waited for, here -- as one batch.  Left to itself the
// compiler fetches each field of a table item, and each of widths and offsets, right where it
// is first used, which strings four to six dependent scalar memory round trips in front of the
// first vector load of a wavefront.
#define ACTQ_SCALAR_BATCH2(a, b) asm volatile("" : "+s"(a), "+s"(b))
#define ACTQ_SCALAR_BATCH10(a, b, c, d, e, f, g, h, i, j) \
    asm volatile("" : "+s"(a), "+s"(b), "+s"(c), "+s"(d), "+s"(e), "+s"(f), "+s"(g), "+s"(h), "+s"(i), "+s"(j))

// What a wavefront of a multi-tensor launch knows after one batch of scalar loads from the
// table: its sample and its run of groups inside the sample, and the tensor's pointers.
struct MultiCursor {
    uint32_t n, tile;        // sample, run of groups inside the sample
    uint64_t D;
    uintptr_t x, out, header, gmin, grange, bits, offsets;
};

// A pointer that went through an integer register has lost its address space, and the compiler
// would emit flat memory instructions for it (which also tick the LDS counter).  Everything the
// table points to is device memory: the pointer is rebuilt as a global one, and the conversion
// to a generic pointer lets the compiler carry that knowledge to every use.
template <typename P>
__device__ __forceinline__ P* device_pointer(uintptr_t a)
{
    typedef P __attribute__((address_space(1))) * global_pointer;
    return (P*)((global_pointer)a);
}

// False: the wavefront has no work.  XCD_MAP: the order of wave_unit.
template <int WAVES_PER_BLOCK, int XCD_MAP, int RUN = 1>
__device__ __forceinline__ bool multi_cursor(const MultiTable& t, uint32_t wave, MultiCursor& c)
{
    const MultiItem& it = t.item[blockIdx.y];
    const uint32_t lin = wave_unit<WAVES_PER_BLOCK, XCD_MAP, RUN>(blockIdx.x, wave);
    // tiles: low word the runs per sample, high word all runs of the tensor
    uint64_t tiles = (static_cast<uint64_t>(it.total_tiles) << 32) | it.tiles;
    uint64_t div = (static_cast<uint64_t>(it.by_tiles.s) << 32) | it.by_tiles.m;
    c.D = static_cast<uint64_t>(it.D);
    c.x = reinterpret_cast<uintptr_t>(it.x);
    c.out = reinterpret_cast<uintptr_t>(it.out);
    c.header = reinterpret_cast<uintptr_t>(it.header);
    c.gmin = reinterpret_cast<uintptr_t>(it.gmin);
    c.grange = reinterpret_cast<uintptr_t>(it.grange);
    c.bits = reinterpret_cast<uintptr_t>(it.bits);
    c.offsets = reinterpret_cast<uintptr_t>(it.offsets);
    ACTQ_SCALAR_BATCH10(tiles, div, c.D, c.x, c.out, c.header, c.gmin, c.grange, c.bits, c.offsets);
    if (lin >= static_cast<uint32_t>(tiles >> 32)) return false;
    c.n = (__umulhi(lin, static_cast<uint32_t>(div)) + lin) >> static_cast<uint32_t>(div >> 32);
    c.tile = lin - c.n * static_cast<uint32_t>(tiles);
    return true;
}

// Width and byte offset of the cursor's sample, as one batch of scalar loads.
__device__ __forceinline__ void sample_width_offset(const MultiCursor& c, uint32_t& b, uint64_t& off)
{
    uint32_t width_word = load_readonly(reinterpret_cast<const uint32_t*>(c.bits) + (c.n >> 2));
    off = load_readonly(reinterpret_cast<const uint64_t*>(c.offsets) + c.n);
    ACTQ_SCALAR_BATCH2(width_word, off);
    b = (width_word >> ((c.n & 3u) * 8u)) & 0xffu;
}


template <typename T>
__global__ __launch_bounds__(kGsBlock) void group_stats_multi_kernel(MultiTable t)
{
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6)));
    MultiCursor c;
    if (!multi_cursor<kGsBlock / kWave, kGsXcdMap, kGsRun>(t, wave, c)) return;
    const uint32_t n = c.n;
    const int64_t D = static_cast<int64_t>(c.D);
    const uint32_t ng = static_cast<uint32_t>(c.D >> 8);
    const T* xs = device_pointer<const T>(c.x) + static_cast<int64_t>(n) * D;
    float v[kGsTiles][kTileGroups][4];
    bool ok[kTileGroups][4];
    int groups[kGsTiles];
#pragma unroll
    for (int k = 0; k < kGsTiles; ++k) {
        const uint32_t g0 = (c.tile * kGsTiles + k) * kTileGroups;
        groups[k] = g0 < ng ? static_cast<int>(min(static_cast<uint32_t>(kTileGroups), ng - g0)) : 0;
        // a tile past the end of the sample re-reads the sample's first tile (its results are not stored)
        load_tile<T, true>(xs, groups[k] ? g0 : 0u, groups[k] ? groups[k] : 1, lane, D, v[k], ok);
    }
#pragma unroll
    for (int k = 0; k < kGsTiles; ++k) {
        const uint32_t g0 = (c.tile * kGsTiles + k) * kTileGroups;
        float lo[kTileGroups], hi[kTileGroups];
        lane_min_max<true>(v[k], ok, lo, hi);
        float mn, mx;
        tile_min_max(lo, hi, lane, mn, mx);
        mn += 0.0f;  // -0.0 -> +0.0
        const int row = lane >> 4;
        if ((lane & 15) == 0 && row < groups[k]) {
            const int64_t gi = static_cast<int64_t>(n) * ng + g0 + row;
            device_pointer<float>(c.gmin)[gi] = mn;
            device_pointer<float>(c.grange)[gi] = (mx - mn) + 0.0f;
        }
    }
}

template <typename T, int NOISE_BITS>
__global__ __launch_bounds__(kBlock) void quantize_pack_multi_kernel(MultiTable t, uint32_t k0, uint32_t k1, uint64_t tag,
                                                                     uint8_t* __restrict__ packed, uint64_t capacity)
{
    __shared__ uint32_t stage_all[kWavesPerBlock][256];
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6)));
    MultiCursor mc;
    if (!multi_cursor<kWavesPerBlock, kQpXcdMap, kQpRun>(t, wave, mc)) return;
    Cursor c;
    c.n = mc.n;
    c.t = mc.tile;
    StreamGeometry geo;
    geo.D = static_cast<int64_t>(mc.D);
    geo.N = t.N;
    geo.ng = static_cast<uint32_t>(mc.D >> 8);
    geo.tiles_per_sample = (geo.ng + kTileGroups - 1) / kTileGroups;
    geo.hdr_mode = t.hdr_mode;
    const uint64_t tensor_tag = tag + blockIdx.y;  // every tensor of the launch draws its own noise
    TileRegs r;
    fetch<T, true>(device_pointer<const T>(mc.x), geo, device_pointer<const uint8_t>(mc.bits),
                   device_pointer<const uint64_t>(mc.offsets), lane, c, r);
    quantize_one<NOISE_BITS, true>(r, c, geo, lane, k0, k1, static_cast<uint32_t>(tensor_tag),
                                   static_cast<uint32_t>(tensor_tag >> 32), packed, capacity,
                                   device_pointer<void>(mc.header), stage_all[wave]);
}

// binary16 input, 16-bit noise, binary32 header: runs of kQpGroupsF16 groups (the table is built for
// runs of that length).  Eight wavefronts per SIMD are asked for: the kernel lives on other
// wavefronts' issue slots while one waits for its loads.
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(8, 8))) void quantize_pack_f16_multi_kernel(
    MultiTable t, uint32_t k0, uint32_t k1, uint64_t tag, uint8_t* __restrict__ packed, uint64_t capacity)
{
    __shared__ u32x4 stage_all[kWavesPerBlock][kQpStageSlots];
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6)));
    MultiCursor mc;
    if (!multi_cursor<kWavesPerBlock, kQpXcdMap, kQpRun>(t, wave, mc)) return;
    const uint64_t tensor_tag = tag + blockIdx.y;  // every tensor of the launch draws its own noise
    quantize_run_f16(device_pointer<const _Float16>(mc.x) + static_cast<int64_t>(mc.n) * static_cast<int64_t>(mc.D), mc.n,
                     mc.tile * kQpGroupsF16, static_cast<uint32_t>(mc.D >> 8), lane, k0, k1, static_cast<uint32_t>(tensor_tag),
                     static_cast<uint32_t>(tensor_tag >> 32), device_pointer<const uint8_t>(mc.bits),
                     device_pointer<const uint64_t>(mc.offsets), packed, capacity, device_pointer<float>(mc.header),
                     stage_all[wave]);
}

// binary32 input, binary32 header: one tile of four groups per wavefront.
template <int NOISE_BITS>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(8, 8))) void quantize_pack_f32_multi_kernel(
    MultiTable t, uint32_t k0, uint32_t k1, uint64_t tag, uint8_t* __restrict__ packed, uint64_t capacity)
{
    __shared__ u32x4 stage_all[kWavesPerBlock][kQpStageSlots];
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6)));
    MultiCursor mc;
    if (!multi_cursor<kWavesPerBlock, kQpXcdMap, kQpRun>(t, wave, mc)) return;
    const uint64_t tensor_tag = tag + blockIdx.y;  // every tensor of the launch draws its own noise
    quantize_tile_f32<NOISE_BITS>(device_pointer<const float>(mc.x) + static_cast<int64_t>(mc.n) * static_cast<int64_t>(mc.D), mc.n,
                                  mc.tile * kTileGroups, static_cast<uint32_t>(mc.D >> 8), lane, k0, k1,
                                  static_cast<uint32_t>(tensor_tag), static_cast<uint32_t>(tensor_tag >> 32),
                                  device_pointer<const uint8_t>(mc.bits), device_pointer<const uint64_t>(mc.offsets), packed,
                                  capacity, device_pointer<float>(mc.header), stage_all[wave]);
}

template <typename T, int HDR, int NG>
__global__ __launch_bounds__(kDqBlock) void unpack_dequantize_multi_kernel(MultiTable t, const uint8_t* __restrict__ packed,
                                                                           uint64_t capacity)
{
    constexpr int kWaves = kDqBlock / kWave;
    __shared__ uint32_t stage_all[kWaves][256];
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t wave = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6)));
    uint32_t* stage = stage_all[wave];
    MultiCursor c;
    if (!multi_cursor<kWaves, kDqXcdMap, kDqRun>(t, wave, c)) return;
    uint32_t b;
    uint64_t off;
    sample_width_offset(c, b, off);
    const uint32_t ng = static_cast<uint32_t>(c.D >> 8);
    const uint32_t n = c.n;
    const int64_t D = static_cast<int64_t>(c.D);
    T* os = device_pointer<T>(c.out) + static_cast<int64_t>(n) * D;
    const void* header = device_pointer<const void>(c.header);
    if (!range_ok(off, static_cast<uint64_t>(ng) * 32u * b, capacity)) return;
    const uint8_t* src = packed + off;
    const uint32_t g0 = c.tile * NG;
    const int groups = static_cast<int>(min(static_cast<uint32_t>(NG), ng - g0));
    constexpr bool V = kDqVectorHeader;
    switch (b) {
        case 1: dequantize_any<T, true, 1, HDR, NG, V>(src, header, os, D, n, g0, groups, ng, lane, stage); break;
        case 2: dequantize_any<T, true, 2, HDR, NG, V>(src, header, os, D, n, g0, groups, ng, lane, stage); break;
        case 3: dequantize_any<T, true, 3, HDR, NG, V>(src, header, os, D, n, g0, groups, ng, lane, stage); break;
        case 4: dequantize_any<T, true, 4, HDR, NG, V>(src, header, os, D, n, g0, groups, ng, lane, stage); break;
        case 5: dequantize_any<T, true, 5, HDR, NG, V>(src, header, os, D, n, g0, groups, ng, lane, stage); break;
        case 6: dequantize_any<T, true, 6, HDR, NG, V>(src, header, os, D, n, g0, groups, ng, lane, stage); break;
        case 7: dequantize_any<T, true, 7, HDR, NG, V>(src, header, os, D, n, g0, groups, ng, lane, stage); break;
        case 8: dequantize_any<T, true, 8, HDR, NG, V>(src, header, os, D, n, g0, groups, ng, lane, stage); break;
        default: return;
    }
}

// ------------------------------------------------------------------------------------
// One range and zero point for the whole tensor (the per-tensor baseline of Sec. 4.1 and
// Sec. 6.1): Z = min, R = max - min over all elements.  Three tiny launches on the caller's
// stream: set the two result words to the identity, reduce (a fixed number of wavefronts
// stride over the tensor; each block folds its minimum and maximum and issues two atomics),
// and convert.  Minimum and maximum do not depend on the order of the operations, so the
// atomics do not make the result vary.  While the reduction runs the two words hold order-
// preserving integer images of the floats (sign bit flipped for non-negative values, all
// bits flipped for negative ones), on which unsigned min / max order like the floats.

__device__ __forceinline__ uint32_t float_to_ordered(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float ordered_to_float(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

__global__ void tensor_stats_init_kernel(uint32_t* zr)
{
    if (threadIdx.x == 0) {
        zr[0] = 0xffffffffu;  // above every value's image
        zr[1] = 0u;           // below every value's image
    }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void tensor_stats_reduce_kernel(const T* __restrict__ x, int64_t n, uint32_t* zr)
{
    __shared__ float part_lo[kWavesPerBlock], part_hi[kWavesPerBlock];
    constexpr int kE = 16 / sizeof(T);  // elements per 128-bit load
    const int64_t chunks = n / kE;      // whole 128-bit chunks; x is 16-byte aligned
    float lo = __builtin_inff(), hi = -__builtin_inff();
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kBlock;
    for (int64_t c = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; c < chunks; c += stride) {
        if constexpr (sizeof(T) == 4) {
            const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(x) + c);
            lo = fminf(fminf(lo, v.x), fminf(fminf(v.y, v.z), v.w));
            hi = fmaxf(fmaxf(hi, v.x), fmaxf(fmaxf(v.y, v.z), v.w));
        } else {
            typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
            const f16x8 v = __builtin_nontemporal_load(reinterpret_cast<const f16x8*>(x) + c);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                lo = fminf(lo, static_cast<float>(v[k]));
                hi = fmaxf(hi, static_cast<float>(v[k]));
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < n - chunks * kE) {  // the last, partial chunk
        const float v = static_cast<float>(x[chunks * kE + threadIdx.x]);
        lo = fminf(lo, v);
        hi = fmaxf(hi, v);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, d));
        hi = fmaxf(hi, __shfl_xor(hi, d));
    }
    if ((threadIdx.x & (kWave - 1)) == 0) {
        part_lo[threadIdx.x >> 6] = lo;
        part_hi[threadIdx.x >> 6] = hi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kWavesPerBlock; ++w) {
            lo = fminf(lo, part_lo[w]);
            hi = fmaxf(hi, part_hi[w]);
        }
        atomicMin(zr, float_to_ordered(lo));
        atomicMax(zr + 1, float_to_ordered(hi));
    }
}

__global__ void tensor_stats_finish_kernel(uint32_t* zr)
{
    if (threadIdx.x == 0) {
        const float mn = ordered_to_float(zr[0]) + 0.0f;  // -0.0 -> +0.0
        const float mx = ordered_to_float(zr[1]);
        zr[0] = __float_as_uint(mn);
        zr[1] = __float_as_uint((mx - mn) + 0.0f);  // a zero range is +0.0
    }
}

// ------------------------------------------------------------------------------------
// Sec. 4.2, Eq. (8): w_n = (G / 6) * ||grad_n||^2 * sum_g R_ng^2.  One block per sample over the
// group ranges (1/256 of the tensor's size).  The block is as wide as the sample needs (up to
// 1024 lanes) and every lane keeps four independent partial sums, so that a sample with many
// groups has enough loads in flight; the partial sums are combined in a fixed order, so the
// result is reproducible.
constexpr int kSensMaxBlock = 1024;

__global__ __launch_bounds__(kSensMaxBlock) void sample_sensitivity_kernel(const float* __restrict__ grange,
                                                                           uint32_t N, uint32_t ng, uint32_t grid_x,
                                                                           float coeff, const float* __restrict__ grad2,
                                                                           float* __restrict__ w)
{
    __shared__ float partial[kSensMaxBlock / kWave];
    const uint32_t n = blockIdx.y * grid_x + blockIdx.x;
    if (n >= N) return;
    const float* r = grange + static_cast<int64_t>(n) * ng;
    const uint32_t threads = blockDim.x;
    float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
    uint32_t g = threadIdx.x;
    for (; g + 3 * threads < ng; g += 4 * threads) {
        const float r0 = r[g], r1 = r[g + threads], r2 = r[g + 2 * threads], r3 = r[g + 3 * threads];
        a0 = __builtin_fmaf(r0, r0, a0);
        a1 = __builtin_fmaf(r1, r1, a1);
        a2 = __builtin_fmaf(r2, r2, a2);
        a3 = __builtin_fmaf(r3, r3, a3);
    }
    for (; g < ng; g += threads) a0 = __builtin_fmaf(r[g], r[g], a0);
    float acc = (a0 + a1) + (a2 + a3);
    // lanes, then wavefronts, in a fixed order
    acc += dpp_f32<kDppXor1>(acc);
    acc += dpp_f32<kDppXor2>(acc);
    acc += dpp_f32<kDppHalfMirror>(acc);
    acc += dpp_f32<kDppXor8>(acc);
    acc += __shfl_xor(acc, 16);
    acc += __shfl_xor(acc, 32);
    if ((threadIdx.x & (kWave - 1)) == 0) partial[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float total = 0.0f;
        for (uint32_t k = 0; k < threads / kWave; ++k) total += partial[k];
        w[n] = coeff * total * (grad2 ? grad2[n] : 1.0f);
    }
}

// ------------------------------------------------------------------------------------
// Sec. 4.3 on the device: the greedy allocation without the host in the loop.
//
// The greedy applies moves (item i, step r of the width ladder) in ascending order of
// (price, i, r) until enough bits are freed, and an item's prices never decrease along the
// ladder.  Its result is therefore fixed by the price of the last applied move: every move
// strictly cheaper is applied, and the moves of exactly that price are applied in (i, r)
// order until the budget holds.  That price is found by a radix selection over the 64-bit
// patterns of the prices (non-negative doubles order like their bit patterns), eight passes
// of eight bits, each a 256-bin histogram of freed bits; ties are then resolved with a
// prefix sum in item order, and a second prefix sum turns the widths into byte offsets.
// One workgroup does all of it out of LDS.  The prices of a thread's first item stay in
// registers (all of them when M <= the workgroup size); those of further items are
// recomputed in every pass.  Three histograms rotate so that a pass needs one barrier:
// while pass p accumulates into one, every wavefront has already scanned the previous one
// for itself and the third one is being cleared for the pass after.

constexpr int kAllocBlock = 1024;
constexpr int kAllocWavesMax = kAllocBlock / kWave;
constexpr int kMaxSteps = 7;
constexpr int kAllocCached = 11;  // items per thread whose (w, D) the allocator keeps in registers

struct AllocArgs {
    int64_t M;
    int64_t D;               // element count of every item when D_items is null
    const int64_t* D_items;  // per-item element counts, or null
    int64_t budget_bits;
    Ladder lad;
};

// DPP row_shr:K with zero fill: lane i of a row of 16 receives lane i - K, or 0 when there is none.
template <int K>
__device__ __forceinline__ uint64_t row_shift_right(uint64_t v)
{
    const uint32_t lo = dpp_u32<0x110 + K>(static_cast<uint32_t>(v));
    const uint32_t hi = dpp_u32<0x110 + K>(static_cast<uint32_t>(v >> 32));
    return (static_cast<uint64_t>(hi) << 32) | lo;
}

__device__ __forceinline__ uint64_t read_lane(uint64_t v, int src)
{
    const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(static_cast<uint32_t>(v)), src));
    const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(static_cast<uint32_t>(v >> 32)), src));
    return (static_cast<uint64_t>(hi) << 32) | lo;
}

// Inclusive prefix sum over the 64 lanes: four shift-and-add steps inside each row of 16,
// then the totals of the preceding rows, read from the rows' last lanes.
__device__ __forceinline__ uint64_t wave_inclusive_scan(uint64_t v, int lane)
{
    v += row_shift_right<1>(v);
    v += row_shift_right<2>(v);
    v += row_shift_right<4>(v);
    v += row_shift_right<8>(v);
    const uint64_t t0 = read_lane(v, 15), t1 = read_lane(v, 31), t2 = read_lane(v, 47);
    const int row = lane >> 4;
    uint64_t before = 0;
    before += row > 0 ? t0 : 0;
    before += row > 1 ? t1 : 0;
    before += row > 2 ? t2 : 0;
    return v + before;
}

// Exclusive prefix sum over the workgroup in thread order; `total` receives the sum.
__device__ __forceinline__ uint64_t block_exclusive_scan(uint64_t v, uint64_t* wave_totals, uint64_t& total)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int waves = blockDim.x >> 6;
    const uint64_t incl = wave_inclusive_scan(v, lane);
    if (lane == kWave - 1) wave_totals[wave] = incl;
    __syncthreads();
    uint64_t before = 0, all = 0;
    for (int k = 0; k < waves; ++k) {
        const uint64_t t = wave_totals[k];
        before += k < wave ? t : 0;
        all += t;
    }
    __syncthreads();
    total = all;
    return before + incl - v;
}

// price of one step of item (w, D): two separately rounded double operations; -0.0 becomes +0.0
__device__ __forceinline__ uint64_t price_bits(double w, double D, double step_price)
{
    const double key = (w * step_price) / D + 0.0;
    return static_cast<uint64_t>(__double_as_longlong(key));
}

__device__ __forceinline__ uint64_t price_bits(float w, int64_t D, double step_price)
{
    return price_bits(static_cast<double>(w), static_cast<double>(D), step_price);
}

template <int CACHED>
__global__ __launch_bounds__(kAllocBlock) void allocate_bits_kernel(const float* __restrict__ w, AllocArgs a,
                                                                    uint8_t* __restrict__ bits,
                                                                    uint64_t* __restrict__ offsets,
                                                                    int64_t* __restrict__ result)
{
    __shared__ uint64_t hist[3][256];
    __shared__ uint64_t wave_totals[kAllocWavesMax];
    __shared__ int width[8];      // the ladder, in LDS because lanes index it independently
    __shared__ double price[8];
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int threads = blockDim.x;
    const int steps = a.lad.count - 1;
    if (tid < 8) {
        width[tid] = a.lad.width[tid];
        price[tid] = tid < 7 ? a.lad.price[tid] : 0.0;
    }
    for (int k = tid; k < 3 * 256; k += threads) (&hist[0][0])[k] = 0;
    __syncthreads();
    const int widest = width[0], narrowest = width[steps];

    // Totals and validation.  The first CACHED items of every thread stay in registers, as the
    // two doubles their prices are computed from (an empty or invalid slot has D = 0), so that the
    // eight passes below run from registers: a pass that reloads its items pays one memory round
    // trip per item and thread.  The first item also keeps its prices.  (CACHED is 1 when every
    // thread has at most one item, which keeps the kernel of the small problem small.)
    uint64_t my_elems = 0;
    bool bad = false;
    double cached_w[CACHED], cached_D[CACHED];   // D < 2^34 is exact in a double
#pragma unroll
    for (int j = 0; j < CACHED; ++j) {
        const int64_t i = tid + static_cast<int64_t>(j) * threads;
        const bool live = i < a.M;
        const float wi = live ? w[i] : 0.0f;
        const int64_t Di = live ? (a.D_items ? a.D_items[i] : a.D) : 0;
        const bool ok = live && valid_sensitivity_bits(__float_as_uint(wi)) && Di > 0 && Di < (int64_t(1) << 34);
        bad = bad || (live && !ok);
        cached_w[j] = static_cast<double>(wi);
        cached_D[j] = ok ? static_cast<double>(Di) : 0.0;
        my_elems += ok ? static_cast<uint64_t>(Di) : 0;
    }
    uint64_t first_key[kMaxSteps];
#pragma unroll
    for (int r = 0; r < kMaxSteps; ++r)
        first_key[r] = (r < steps && cached_D[0] != 0.0) ? price_bits(cached_w[0], cached_D[0], price[r])
                                                  : ~uint64_t(0);
    for (int64_t i = tid + static_cast<int64_t>(CACHED) * threads; i < a.M; i += threads) {
        const float wi = w[i];
        const int64_t Di = a.D_items ? a.D_items[i] : a.D;
        if (!valid_sensitivity_bits(__float_as_uint(wi)) || Di <= 0 || Di >= (int64_t(1) << 34)) bad = true;
        else my_elems += static_cast<uint64_t>(Di);
    }
    const bool invalid = __syncthreads_or(bad ? 1 : 0) != 0;
    uint64_t elems;
    block_exclusive_scan(my_elems, wave_totals, elems);
    const uint64_t budget = static_cast<uint64_t>(a.budget_bits);
    const bool loose = !invalid && elems * widest <= budget;
    const bool infeasible = !invalid && elems * narrowest > budget;
    const int64_t status = invalid ? ACTQ_EINVAL : (infeasible ? ACTQ_EINFEASIBLE : ACTQ_OK);

    uint64_t threshold = 0, below = 0, need = 0;
    const bool search = !invalid && !loose && !infeasible;
    if (search) {
        need = elems * widest - budget;  // bits that must be freed, > 0
        uint64_t prefix = 0;
        uint32_t alive[(CACHED + 3) / 4];   // one byte per cached item: which of its moves are still in play
#pragma unroll
        for (int k = 0; k < (CACHED + 3) / 4; ++k) alive[k] = ~0u;
        for (int pass = 7; pass >= 0; --pass) {
            uint64_t* h = hist[pass % 3];
            const int shift = 8 * pass;
            // A lane adds up the moves it sends to one bin in a row and issues one atomic per run:
            // in the first passes (sign and exponent bits) nearly every price falls into the same
            // one or two bins, and 64 lanes adding to one LDS address are served one after another.
            uint32_t run_bin = 0;
            uint64_t run_sum = 0;
            const auto add = [&](uint32_t bin, uint64_t freed) {
                if (bin != run_bin && run_sum) {
                    __hip_atomic_fetch_add(&h[run_bin], run_sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    run_sum = 0;
                }
                run_bin = bin;
                run_sum += freed;
            };
            // first item: cached prices
            if (cached_D[0] != 0.0) {
#pragma unroll
                for (int r = 0; r < kMaxSteps; ++r) {
                    if (r >= steps) continue;
                    const uint64_t key = first_key[r];
                    if (pass == 7 || (key >> (shift + 8)) == prefix)
                        add(static_cast<uint32_t>(key >> shift) & 255u, static_cast<uint64_t>(cached_D[0]) * (width[r] - width[r + 1]));
                }
            }
            // further cached items: prices recomputed from registers, but only for the moves whose
            // price still matches the digits found so far -- a move that fell out of the prefix in
            // one pass stays out, and after two passes few are left
#pragma unroll
            for (int j = 1; j < CACHED; ++j) {
                if (static_cast<int64_t>(j) * threads >= a.M) break;   // uniform
                constexpr uint32_t kAll = (1u << kMaxSteps) - 1u;
                const int field = 8 * (j % 4);
                uint32_t in_play = (alive[j / 4] >> field) & kAll;
                if (cached_D[j] == 0.0 || in_play == 0) continue;
                const uint64_t Dj = static_cast<uint64_t>(cached_D[j]);
                for (int r = 0; r < steps; ++r) {
                    if (!((in_play >> r) & 1u)) continue;
                    const uint64_t key = price_bits(cached_w[j], cached_D[j], price[r]);
                    if (pass == 7 || (key >> (shift + 8)) == prefix)
                        add(static_cast<uint32_t>(key >> shift) & 255u, Dj * (width[r] - width[r + 1]));
                    else
                        in_play &= ~(1u << r);
                }
                alive[j / 4] = (alive[j / 4] & ~(kAll << field)) | (in_play << field);
            }
            for (int64_t i = tid + static_cast<int64_t>(CACHED) * threads; i < a.M; i += threads) {
                const float wi = w[i];
                const int64_t Di = a.D_items ? a.D_items[i] : a.D;
                for (int r = 0; r < steps; ++r) {
                    const uint64_t key = price_bits(wi, Di, price[r]);
                    if (pass == 7 || (key >> (shift + 8)) == prefix)
                        add(static_cast<uint32_t>(key >> shift) & 255u, static_cast<uint64_t>(Di) * (width[r] - width[r + 1]));
                }
            }
            if (run_sum)
                __hip_atomic_fetch_add(&h[run_bin], run_sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            __syncthreads();
            // Every wavefront finds, for itself, the bin in which the running sum of freed bits
            // first reaches `need`.  Exactly one lane holds it.
            uint64_t hb[4], mine = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) { hb[k] = h[4 * lane + k]; mine += hb[k]; }
            const uint64_t incl = wave_inclusive_scan(mine, lane);
            uint64_t run = below + incl - mine;
            const bool winner = run < need && run + mine >= need;
            int digit = 4 * lane;
#pragma unroll
            for (int k = 0; k < 3; ++k)
                if (winner && run + hb[k] < need) { run += hb[k]; ++digit; }
                else break;
            const uint64_t vote = __ballot(winner);
            const int src = vote ? __builtin_ctzll(vote) : 0;
            digit = __builtin_amdgcn_readlane(digit, src);
            below = read_lane(run, src);
            prefix = (prefix << 8) | static_cast<uint64_t>(digit);
            // the histogram of the pass before this one is free again: clear it for the pass after the next
            uint64_t* stale = hist[(pass + 1) % 3];
            for (int k = tid; k < 256; k += threads) stale[k] = 0;
        }
        threshold = prefix;
    }

    // Widths, then offsets, in item order.  A round gives every thread Q consecutive items, so the
    // two workgroup prefix sums (ties at the threshold, then bytes) run over thread totals: once
    // per Q * threads items.  The barriers of those sums, not the arithmetic, are what a round costs.
    uint64_t tie_carry = 0, byte_carry = 0;
    const uint64_t rest = need - below;  // bits still to free among the moves priced exactly at the threshold
    const auto assign = [&](auto items_per_thread) {
        constexpr int Q = decltype(items_per_thread)::value;
        for (int64_t base = 0; base < a.M; base += static_cast<int64_t>(threads) * Q) {
            const int64_t i0 = base + static_cast<int64_t>(tid) * Q;
            int64_t Dq[Q];
            int rung[Q], ties[Q];
            bool live[Q];
            uint64_t tie_bits[Q], tie_sum = 0;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const int64_t i = i0 + q;
                live[q] = i < a.M;
                const float wi = live[q] ? w[i] : 0.0f;
                int64_t Di = live[q] ? (a.D_items ? a.D_items[i] : a.D) : 0;
                if (Di <= 0 || Di >= (int64_t(1) << 34)) Di = live[q] ? 1 : 0;  // invalid input: stay memory-safe
                Dq[q] = Di;
                rung[q] = loose ? 0 : steps;
                ties[q] = 0;
                if (search && live[q]) {
                    rung[q] = 0;
                    for (int r = 0; r < steps; ++r) {
                        const uint64_t key = price_bits(wi, Di, price[r]);
                        rung[q] += key < threshold ? 1 : 0;
                        ties[q] += key == threshold ? 1 : 0;
                    }
                }
                tie_bits[q] = static_cast<uint64_t>(Di) * (width[rung[q]] - width[rung[q] + ties[q]]);
                tie_sum += tie_bits[q];
            }
            uint64_t tie_total;
            uint64_t before = tie_carry + block_exclusive_scan(tie_sum, wave_totals, tie_total);
            tie_carry += tie_total;
            uint64_t my_bytes[Q], byte_sum = 0;
            int b[Q];
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                uint64_t freed = before;      // by the tie moves of all items before this one
                before += tie_bits[q];
                for (; ties[q] > 0 && freed < rest; --ties[q], ++rung[q])
                    freed += static_cast<uint64_t>(Dq[q]) * (width[rung[q]] - width[rung[q] + 1]);
                b[q] = width[rung[q]];
                const uint64_t groups = (static_cast<uint64_t>(Dq[q]) + kGroup - 1) / kGroup;
                my_bytes[q] = live[q] ? groups * 32u * b[q] : 0;
                byte_sum += my_bytes[q];
            }
            uint64_t byte_total;
            uint64_t off = byte_carry + block_exclusive_scan(byte_sum, wave_totals, byte_total);
            byte_carry += byte_total;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                if (live[q]) {
                    bits[i0 + q] = static_cast<uint8_t>(b[q]);
                    offsets[i0 + q] = off;
                }
                off += my_bytes[q];
            }
        }
    };
    if (a.M <= threads) assign(std::integral_constant<int, 1>());
    else assign(std::integral_constant<int, 4>());
    if (tid == 0) {
        result[0] = static_cast<int64_t>(byte_carry);
        result[1] = status;
    }
}

// ------------------------------------------------------------------------------------
// Host-side launch geometry.

int make_geometry(const char* who, int64_t N, int64_t D, Geometry* geo, dim3* grid)
{
    const int64_t ng = (D + kGroup - 1) / kGroup;
    const int64_t tps = (ng + kTileGroups - 1) / kTileGroups;
    geo->D = D;
    geo->N = static_cast<uint32_t>(N);
    geo->ng = static_cast<uint32_t>(ng);
    geo->tiles_per_sample = static_cast<uint32_t>(tps);
    geo->hdr_mode = 0;
    const int64_t gx = (tps + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t gy = N < 65535 ? N : 65535;
    const int64_t gz = (N + gy - 1) / gy;
    if (gx >= (int64_t(1) << 31) || gz > 65535)
        return fail(ACTQ_EINVAL, "%s: tensor too large for one launch (grid %lld x %lld x %lld)", who,
                    (long long)gx, (long long)gy, (long long)gz);
    geo->grid_y = static_cast<uint32_t>(gy);
    *grid = dim3(static_cast<unsigned>(gx), static_cast<unsigned>(gy), static_cast<unsigned>(gz));
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

// A binary32 tensor of full groups goes through the multi-tensor kernels as a table of one: their
// linear grid over (sample, tile) and its XCD-aware order measured faster than samples in grid.y
// (group_stats 65 -> 63 us on the stage-1 tensor; binary16 input gained nothing there).
static bool fits_table_of_one(int64_t N, int64_t D, int64_t groups_per_wave)
{
    return vector_ok(D) && N * ((D / kGroup + groups_per_wave - 1) / groups_per_wave) < (int64_t(1) << 31);
}

static bool as_table_of_one(int dtype, int64_t N, int64_t D, int64_t groups_per_wave)
{
    return dtype == ACTQ_F32 && fits_table_of_one(N, D, groups_per_wave);
}

// Groups a wavefront of the multi-tensor quantizer takes: binary16 input with 16-bit noise and the
// binary32 header has a kernel of its own that works on runs of eight.
static bool quantize_by_runs(int dtype, int noise_bits, int hdr) { return dtype == ACTQ_F16 && noise_bits == 16 && hdr == 0; }

static int quantize_groups_per_wave(int dtype, int noise_bits, int hdr)
{
    return quantize_by_runs(dtype, noise_bits, hdr) ? kQpGroupsF16 : kTileGroups;
}


int launch_group_stats(const void* x, int dtype, int64_t N, int64_t D, float* gmin, float* grange,
                       void* stream)
{
    if (as_table_of_one(dtype, N, D, kGsTiles * kTileGroups)) {
        actq_tensor one = {};
        one.x = x;
        one.gmin = gmin;
        one.grange = grange;
        one.D = D;
        return launch_group_stats_multi(&one, 1, dtype, N, stream);
    }
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

template <typename T, int NOISE_BITS, bool VEC>
static int launch_quantize_variant(const T* x, StreamGeometry geo, hipStream_t s, const uint8_t* bits,
                                   const uint64_t* offsets, uint64_t seed, uint64_t tag, uint8_t* packed,
                                   uint64_t capacity, void* header)
{
    const uint32_t k0 = static_cast<uint32_t>(seed), k1 = static_cast<uint32_t>(seed >> 32);
    const uint32_t t0 = static_cast<uint32_t>(tag), t1 = static_cast<uint32_t>(tag >> 32);
    const uint32_t gx = (geo.tiles_per_sample + kWavesPerBlock - 1) / kWavesPerBlock;
    const uint32_t gy = geo.N < 65535u ? geo.N : 65535u;
    const uint32_t gz = (geo.N + gy - 1) / gy;
    if (gz > 65535u) return fail(ACTQ_EINVAL, "actq_quantize_pack: too many samples for one launch");
    quantize_pack_tile_kernel<T, NOISE_BITS, VEC><<<dim3(gx, gy, gz), kBlock, 0, s>>>(x, geo, gy, bits, offsets, k0, k1, t0, t1, packed, capacity, header);
    return ACTQ_OK;
}

template <typename T>
static int launch_quantize_typed(const T* x, const StreamGeometry& geo, hipStream_t s, bool vec,
                                 int noise_bits, const uint8_t* bits, const uint64_t* offsets,
                                 uint64_t seed, uint64_t tag, uint8_t* packed, uint64_t capacity,
                                 void* header)
{
    if (noise_bits == 24) {
        if (vec) return launch_quantize_variant<T, 24, true>(x, geo, s, bits, offsets, seed, tag, packed, capacity, header);
        return launch_quantize_variant<T, 24, false>(x, geo, s, bits, offsets, seed, tag, packed, capacity, header);
    }
    if (vec) return launch_quantize_variant<T, 16, true>(x, geo, s, bits, offsets, seed, tag, packed, capacity, header);
    return launch_quantize_variant<T, 16, false>(x, geo, s, bits, offsets, seed, tag, packed, capacity, header);
}

int launch_quantize_pack(const void* x, int dtype, int64_t N, int64_t D, const uint8_t* bits,
                         const uint64_t* offsets, uint64_t seed, uint64_t tag, int noise_bits,
                         void* packed, uint64_t capacity, void* header, int hdr, void* stream)
{
    // binary16 input with 16-bit noise and the binary32 header as well: its kernel is a multi-tensor one only
    if ((dtype == ACTQ_F32 || quantize_by_runs(dtype, noise_bits, hdr)) &&
        fits_table_of_one(N, D, quantize_groups_per_wave(dtype, noise_bits, hdr))) {
        actq_tensor one = {};
        one.x = x;
        one.header = header;
        one.bits = bits;
        one.offsets = offsets;
        one.D = D;
        return launch_quantize_pack_multi(&one, 1, dtype, N, seed, tag, noise_bits, packed, capacity, hdr, stream);
    }
    const int64_t ng = (D + kGroup - 1) / kGroup;
    const int64_t tps = (ng + kTileGroups - 1) / kTileGroups;
    if (N * tps >= (int64_t(1) << 32))
        return fail(ACTQ_EINVAL, "actq_quantize_pack: tensor too large for one launch (%lld tiles)", (long long)(N * tps));
    StreamGeometry geo;
    geo.D = D;
    geo.N = static_cast<uint32_t>(N);
    geo.ng = static_cast<uint32_t>(ng);
    geo.tiles_per_sample = static_cast<uint32_t>(tps);
    geo.hdr_mode = static_cast<uint32_t>(hdr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool vec = vector_ok(D);
    int rc;
    if (dtype == ACTQ_F32)
        rc = launch_quantize_typed(static_cast<const float*>(x), geo, s, vec, noise_bits, bits, offsets, seed, tag, static_cast<uint8_t*>(packed), capacity, header);
    else
        rc = launch_quantize_typed(static_cast<const _Float16*>(x), geo, s, vec, noise_bits, bits, offsets, seed, tag, static_cast<uint8_t*>(packed), capacity, header);
    if (rc) return rc;
    return check_launch("actq_quantize_pack");
}

int launch_unpack_dequantize(const void* packed, uint64_t capacity, const void* header, int hdr,
                             const uint8_t* bits, const uint64_t* offsets, int64_t N, int64_t D,
                             void* out, int out_dtype, void* stream)
{
    const bool vec = vector_ok(D);
    // A tensor with full groups goes through the multi-tensor kernel as a table of one: its linear
    // grid over (sample, tile) measured 7 % faster on the stage-1 tensor than samples in grid.y
    // (72.9 against 79.3 us in the same run).
    const int64_t per_wave = out_dtype == ACTQ_F16 ? kDqGroupsF16 : kDqGroupsF32;
    if (vec && N * ((D / kGroup + per_wave - 1) / per_wave) < (int64_t(1) << 31)) {
        actq_tensor one = {};
        one.out = out;
        one.header = const_cast<void*>(header);
        one.bits = bits;
        one.offsets = offsets;
        one.D = D;
        return launch_unpack_dequantize_multi(&one, 1, packed, capacity, hdr, N, out_dtype, stream);
    }
    Geometry geo;
    dim3 grid;
    if (int rc = make_geometry("actq_unpack_dequantize", N, D, &geo, &grid)) return rc;
    geo.hdr_mode = static_cast<uint32_t>(hdr);
    hipStream_t s = static_cast<hipStream_t>(stream);
    auto* pk = static_cast<const uint8_t*>(packed);
#define ACTQ_DEQ(T, V, H) unpack_dequantize_kernel<T, V, H><<<grid, kBlock, 0, s>>>(pk, capacity, header, bits, offsets, geo, static_cast<T*>(out))
#define ACTQ_DEQ_H(T, V)                                   \
    do {                                                   \
        if (hdr == ACTQ_HDR_F32) ACTQ_DEQ(T, V, 0);        \
        else if (hdr == ACTQ_HDR_BF16) ACTQ_DEQ(T, V, 1);  \
        else ACTQ_DEQ(T, V, 2);                            \
    } while (0)
    if (out_dtype == ACTQ_F32) {
        if (vec) ACTQ_DEQ_H(float, true); else ACTQ_DEQ_H(float, false);
    } else {
        if (vec) ACTQ_DEQ_H(_Float16, true); else ACTQ_DEQ_H(_Float16, false);
    }
#undef ACTQ_DEQ_H
#undef ACTQ_DEQ
    return check_launch("actq_unpack_dequantize");
}

int launch_allocate_bits(const float* w, const int64_t* D_items, int64_t D, int64_t M, int64_t budget_bits,
                         const Ladder& lad, uint8_t* bits, uint64_t* offsets, int64_t* result, void* stream)
{
    AllocArgs a;
    a.M = M;
    a.D = D;
    a.D_items = D_items;
    a.budget_bits = budget_bits;
    a.lad = lad;
    // a workgroup no larger than the problem: barriers and scans get cheaper with fewer wavefronts
    const int64_t lanes = (M + kWave - 1) / kWave * kWave;
    const int block = static_cast<int>(lanes < kAllocBlock ? lanes : kAllocBlock);
    if (M <= block) allocate_bits_kernel<1><<<1, block, 0, static_cast<hipStream_t>(stream)>>>(w, a, bits, offsets, result);
    else allocate_bits_kernel<kAllocCached><<<1, block, 0, static_cast<hipStream_t>(stream)>>>(w, a, bits, offsets, result);
    return check_launch("actq_allocate_bits_device");
}

static int make_multi_table(const char* who, const actq_tensor* tensors, int32_t count, int64_t N, int hdr,
                            MultiTable* t, dim3* grid, int groups_per_wave = kTileGroups,
                            int waves_per_block = kWavesPerBlock, int run = 1)
{
    t->count = static_cast<uint32_t>(count);
    t->N = static_cast<uint32_t>(N);
    t->hdr_mode = static_cast<uint32_t>(hdr);
    t->pad = 0;
    uint64_t most = 0;
    for (int32_t i = 0; i < count; ++i) {
        const int64_t ng = tensors[i].D / kGroup;
        const uint64_t per_sample = static_cast<uint64_t>((ng + groups_per_wave - 1) / groups_per_wave);
        const uint64_t tiles = per_sample * static_cast<uint64_t>(N);
        if (tiles >= (uint64_t(1) << 31)) return fail(ACTQ_EINVAL, "%s: tensor %d has too many tiles for one launch", who, i);
        if (tiles > most) most = tiles;
        MultiItem& it = t->item[i];
        it.x = tensors[i].x;
        it.out = tensors[i].out;
        it.gmin = tensors[i].gmin;
        it.grange = tensors[i].grange;
        it.header = tensors[i].header;
        it.bits = tensors[i].bits;
        it.offsets = tensors[i].offsets;
        it.D = tensors[i].D;
        it.by_tiles = make_fastdiv(static_cast<uint32_t>(per_sample));
        it.tiles = static_cast<uint32_t>(per_sample);
        it.total_tiles = static_cast<uint32_t>(tiles);
    }
    // whole runs of 8 * run blocks (`run` blocks per XCD): every order of wave_unit covers a run exactly
    const uint64_t blocks_per_run = 8u * static_cast<uint64_t>(run);
    const uint64_t per_run = blocks_per_run * static_cast<uint64_t>(waves_per_block);
    *grid = dim3(static_cast<unsigned>((most + per_run - 1) / per_run * blocks_per_run), static_cast<unsigned>(count));
    return ACTQ_OK;
}

int launch_group_stats_multi(const actq_tensor* tensors, int32_t count, int dtype, int64_t N, void* stream)
{
    MultiTable t;
    dim3 grid;
    if (int rc = make_multi_table("actq_group_stats_multi", tensors, count, N, 0, &t, &grid, kGsTiles * kTileGroups, kGsBlock / kWave, kGsRun)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == ACTQ_F32) group_stats_multi_kernel<float><<<grid, kGsBlock, 0, s>>>(t);
    else group_stats_multi_kernel<_Float16><<<grid, kGsBlock, 0, s>>>(t);
    return check_launch("actq_group_stats_multi");
}

int launch_quantize_pack_multi(const actq_tensor* tensors, int32_t count, int dtype, int64_t N, uint64_t seed,
                               uint64_t tag, int noise_bits, void* packed, uint64_t capacity, int hdr, void* stream)
{
    MultiTable t;
    dim3 grid;
    const int per_wave = quantize_groups_per_wave(dtype, noise_bits, hdr);
    if (int rc = make_multi_table("actq_quantize_pack_multi", tensors, count, N, hdr, &t, &grid, per_wave, kWavesPerBlock, kQpRun)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t k0 = static_cast<uint32_t>(seed), k1 = static_cast<uint32_t>(seed >> 32);
    uint8_t* pk = static_cast<uint8_t*>(packed);
    if (dtype == ACTQ_F32 && hdr == 0) {
        if (noise_bits == 16) quantize_pack_f32_multi_kernel<16><<<grid, kBlock, 0, s>>>(t, k0, k1, tag, pk, capacity);
        else quantize_pack_f32_multi_kernel<24><<<grid, kBlock, 0, s>>>(t, k0, k1, tag, pk, capacity);
    } else if (dtype == ACTQ_F32) {
        if (noise_bits == 16) quantize_pack_multi_kernel<float, 16><<<grid, kBlock, 0, s>>>(t, k0, k1, tag, pk, capacity);
        else quantize_pack_multi_kernel<float, 24><<<grid, kBlock, 0, s>>>(t, k0, k1, tag, pk, capacity);
    } else {
        if (quantize_by_runs(dtype, noise_bits, hdr)) quantize_pack_f16_multi_kernel<<<grid, kBlock, 0, s>>>(t, k0, k1, tag, pk, capacity);
        else if (noise_bits == 16) quantize_pack_multi_kernel<_Float16, 16><<<grid, kBlock, 0, s>>>(t, k0, k1, tag, pk, capacity);
        else quantize_pack_multi_kernel<_Float16, 24><<<grid, kBlock, 0, s>>>(t, k0, k1, tag, pk, capacity);
    }
    return check_launch("actq_quantize_pack_multi");
}

int launch_unpack_dequantize_multi(const actq_tensor* tensors, int32_t count, const void* packed, uint64_t capacity,
                                   int hdr, int64_t N, int out_dtype, void* stream)
{
    MultiTable t;
    dim3 grid;
    const int per_wave = out_dtype == ACTQ_F16 ? kDqGroupsF16 : kDqGroupsF32;
    if (int rc = make_multi_table("actq_unpack_dequantize_multi", tensors, count, N, hdr, &t, &grid, per_wave, kDqBlock / kWave, kDqRun)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint8_t* pk = static_cast<const uint8_t*>(packed);
#define ACTQ_DEQM(T, NG)                                                                                    \
    do {                                                                                                 \
        if (hdr == ACTQ_HDR_F32) unpack_dequantize_multi_kernel<T, 0, NG><<<grid, kDqBlock, 0, s>>>(t, pk, capacity);       \
        else if (hdr == ACTQ_HDR_BF16) unpack_dequantize_multi_kernel<T, 1, NG><<<grid, kDqBlock, 0, s>>>(t, pk, capacity); \
        else unpack_dequantize_multi_kernel<T, 2, NG><<<grid, kDqBlock, 0, s>>>(t, pk, capacity);                           \
    } while (0)
    if (out_dtype == ACTQ_F32) ACTQ_DEQM(float, kDqGroupsF32); else ACTQ_DEQM(_Float16, kDqGroupsF16);
#undef ACTQ_DEQM
    return check_launch("actq_unpack_dequantize_multi");
}

int launch_tensor_stats(const void* x, int dtype, int64_t n, float* zr, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t* words = reinterpret_cast<uint32_t*>(zr);
    const int64_t chunks = n / (dtype == ACTQ_F32 ? 4 : 8);
    int64_t blocks = (chunks + kBlock - 1) / kBlock;
    if (blocks < 1) blocks = 1;
    if (blocks > 2048) blocks = 2048;  // eight resident blocks per compute unit: 4096 atomics in all
    tensor_stats_init_kernel<<<1, kWave, 0, s>>>(words);
    if (dtype == ACTQ_F32)
        tensor_stats_reduce_kernel<float><<<static_cast<unsigned>(blocks), kBlock, 0, s>>>(static_cast<const float*>(x), n, words);
    else
        tensor_stats_reduce_kernel<_Float16><<<static_cast<unsigned>(blocks), kBlock, 0, s>>>(static_cast<const _Float16*>(x), n, words);
    tensor_stats_finish_kernel<<<1, kWave, 0, s>>>(words);
    return check_launch("actq_tensor_stats");
}

int launch_sample_sensitivity(const float* grange, int64_t N, int64_t ng, int32_t G, const float* grad2,
                              float* w, void* stream)
{
    const uint32_t gx = N < 65535 ? static_cast<uint32_t>(N) : 65535u;
    const uint32_t gy = static_cast<uint32_t>((N + gx - 1) / gx);
    if (gy > 65535u) return fail(ACTQ_EINVAL, "actq_sample_sensitivity: too many samples for one launch");
    // one lane per group up to 1024 lanes, whole wavefronts
    const int64_t lanes = (ng + kWave - 1) / kWave * kWave;
    const unsigned block = static_cast<unsigned>(lanes < kSensMaxBlock ? lanes : kSensMaxBlock);
    sample_sensitivity_kernel<<<dim3(gx, gy), block, 0, static_cast<hipStream_t>(stream)>>>(
        grange, static_cast<uint32_t>(N), static_cast<uint32_t>(ng), gx, static_cast<float>(G) / 6.0f, grad2, w);
    return check_launch("actq_sample_sensitivity");
}

}  // namespace actq
