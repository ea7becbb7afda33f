// HIP kernels of libactq for gfx950 (MI355X): the exact layer contexts of ActNN's appendix.
//
//   * ReLU ("Activation Layers"): the context is one bit per element, f'(x) = [x > 0].
//     Forward writes y = max(x, 0) and the bit stream; backward multiplies the incoming
//     gradient by the stored bit (as a selection, so a cleared bit always gives +0).
//   * Max pooling ("Pooling Layers"): the context is, per output location, the 8-bit
//     position of the maximum inside its window.  Backward gathers, for every input
//     location, the output gradients whose stored position points at it.
//
// Both are pure streaming kernels bound by HBM.  ReLU uses the same decomposition as the
// quantizer: one wavefront per tile of four 128-bit loads per lane; the comparison masks
// come out of v_cmp as 64-bit wavefront masks, and a few lanes interleave them into the
// LSB-first stream, so the bits leave as one coalesced store per tile without LDS.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "actq_internal.h"

namespace actq {
namespace {

constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;
constexpr int kBlock = kWave * kWavesPerBlock;
constexpr int kLoadsPerTile = 4;

int launched(const char* who)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ACTQ_EHIP, "%s: launch failed: %s", who, hipGetErrorString(e));
    return ACTQ_OK;
}

// ------------------------------------------------------------------------------------
// ReLU.  A lane owns E consecutive elements per load (E = 4 binary32 or 8 binary16 values:
// 128 bits); a load of the wavefront covers 64*E elements = 2*E words of the bit stream.

template <typename T>
struct Lanes;

template <>
struct Lanes<float> {
    static constexpr int E = 4;
    typedef float vec __attribute__((ext_vector_type(4)));
};

template <>
struct Lanes<_Float16> {
    static constexpr int E = 8;
    typedef _Float16 vec __attribute__((ext_vector_type(8)));
};

// Moves bit t of `piece` (32 / E bits wide) to bit E * t.
template <int E>
__device__ __forceinline__ uint32_t spread(uint32_t piece)
{
    if (E == 4) {  // 8 bits -> every 4th bit
        uint32_t x = piece & 0xffu;
        x = (x | (x << 12)) & 0x000f000fu;
        x = (x | (x << 6)) & 0x03030303u;
        x = (x | (x << 3)) & 0x11111111u;
        return x;
    } else {  // 4 bits -> every 8th bit
        uint32_t x = piece & 0xfu;
        x = (x | (x << 14)) & 0x00030003u;
        x = (x | (x << 7)) & 0x01010101u;
        return x;
    }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void relu_forward_kernel(const T* x, int64_t n, int64_t mask_words,
                                                              T* y, uint32_t* __restrict__ mask)
{
    constexpr int E = Lanes<T>::E;
    typedef typename Lanes<T>::vec vec;
    constexpr int kWordsPerLoad = 2 * E;           // 64 * E bits
    constexpr int kLanesPerWord = 32 / E;          // lanes whose bits share one word
    constexpr int64_t kTileElems = int64_t(kLoadsPerTile) * kWave * E;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t tile = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t first = tile * kTileElems;
    if (first >= n) return;
    const bool full = first + kTileElems <= n;

    vec v[kLoadsPerTile];
    if (full) {
#pragma unroll
        for (int u = 0; u < kLoadsPerTile; ++u)
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const vec*>(x + first + (u * kWave + lane) * E));
    } else {
#pragma unroll
        for (int u = 0; u < kLoadsPerTile; ++u)
#pragma unroll
            for (int k = 0; k < E; ++k) {
                const int64_t i = first + (u * kWave + lane) * E + k;
                v[u][k] = i < n ? x[i] : static_cast<T>(0.0f);  // past the end: bit 0, nothing stored
            }
    }

    // m[u][k]: lane l's bit says whether element k of lane l in load u is positive
    uint64_t m[kLoadsPerTile][E];
#pragma unroll
    for (int u = 0; u < kLoadsPerTile; ++u) {
        vec out;
#pragma unroll
        for (int k = 0; k < E; ++k) {
            const bool positive = static_cast<float>(v[u][k]) > 0.0f;
            m[u][k] = __ballot(positive);
            out[k] = positive ? v[u][k] : static_cast<T>(0.0f);
        }
        if (full) {
            __builtin_nontemporal_store(out, reinterpret_cast<vec*>(y + first + (u * kWave + lane) * E));
        } else {
#pragma unroll
            for (int k = 0; k < E; ++k) {
                const int64_t i = first + (u * kWave + lane) * E + k;
                if (i < n) y[i] = out[k];
            }
        }
    }

    // Word j of the tile's stream (j = lane) holds the bits of kLanesPerWord lanes of load
    // u = j / kWordsPerLoad: stream bit E*l + k is bit l of m[u][k].
    const int u_sel = lane / kWordsPerLoad;
    const int first_lane = (lane % kWordsPerLoad) * kLanesPerWord;
    uint32_t word = 0;
#pragma unroll
    for (int k = 0; k < E; ++k) {
        uint64_t mk = m[0][k];
#pragma unroll
        for (int u = 1; u < kLoadsPerTile; ++u) mk = u_sel == u ? m[u][k] : mk;
        word |= spread<E>(static_cast<uint32_t>(mk >> first_lane)) << k;
    }
    const int64_t w = tile * (kLoadsPerTile * kWordsPerLoad) + lane;
    if (lane < kLoadsPerTile * kWordsPerLoad && w < mask_words) __builtin_nontemporal_store(word, mask + w);
}

template <typename T>
__global__ __launch_bounds__(kBlock) void relu_backward_kernel(const uint32_t* __restrict__ mask, int64_t mask_words,
                                                               const T* grad_y, int64_t n, T* grad_x)
{
    constexpr int E = Lanes<T>::E;
    typedef typename Lanes<T>::vec vec;
    constexpr int kWordsPerLoad = 2 * E;
    constexpr int64_t kTileElems = int64_t(kLoadsPerTile) * kWave * E;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t tile = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t first = tile * kTileElems;
    if (first >= n) return;
    const bool full = first + kTileElems <= n;

    vec g[kLoadsPerTile];
    uint32_t word[kLoadsPerTile];
#pragma unroll
    for (int u = 0; u < kLoadsPerTile; ++u) {
        // the lane's E bits start at bit E*lane of the load's 64*E-bit stretch
        int64_t w = tile * (kLoadsPerTile * kWordsPerLoad) + u * kWordsPerLoad + (lane * E >> 5);
        w = w < mask_words ? w : mask_words - 1;  // past the end: any word, its elements are not stored
        word[u] = __builtin_nontemporal_load(mask + w);
        if (full) {
            g[u] = __builtin_nontemporal_load(reinterpret_cast<const vec*>(grad_y + first + (u * kWave + lane) * E));
        } else {
#pragma unroll
            for (int k = 0; k < E; ++k) {
                const int64_t i = first + (u * kWave + lane) * E + k;
                g[u][k] = i < n ? grad_y[i] : static_cast<T>(0.0f);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kLoadsPerTile; ++u) {
        const uint32_t mine = word[u] >> ((lane * E) & 31);
        vec out;
#pragma unroll
        for (int k = 0; k < E; ++k) out[k] = (mine >> k) & 1u ? g[u][k] : static_cast<T>(0.0f);
        if (full) {
            __builtin_nontemporal_store(out, reinterpret_cast<vec*>(grad_x + first + (u * kWave + lane) * E));
        } else {
#pragma unroll
            for (int k = 0; k < E; ++k) {
                const int64_t i = first + (u * kWave + lane) * E + k;
                if (i < n) grad_x[i] = out[k];
            }
        }
    }
}

// ------------------------------------------------------------------------------------
// Max pooling.

// n / d with the host-computed constants of FastDiv (see actq_internal.h)
__device__ __forceinline__ uint32_t fastdiv(uint32_t n, FastDiv f) { return (__umulhi(n, f.m) + n) >> f.s; }

struct Pool {
    int32_t H, W, OH, OW;
    int32_t kh, kw, sh, sw, ph, pw, dh, dw;
    FastDiv by_OW, by_W, by_sh, by_sw, by_dh, by_dw;
    uint32_t grid_y;  // planes are spread over blockIdx.y and blockIdx.z
};

// One thread per output location; blockIdx.x runs over the locations of one plane, so
// consecutive lanes walk along the rows of the output.  The window is scanned row by row and
// only a strictly larger value replaces the running maximum, so among equal values the first
// position wins; padded positions are skipped.  KH = KW = 0 takes the window size at run time.
template <typename T, int KH, int KW>
__global__ __launch_bounds__(kBlock) void maxpool2d_forward_kernel(const T* __restrict__ x, int64_t planes, Pool g,
                                                                   T* __restrict__ y, uint8_t* __restrict__ argmax)
{
    const int64_t plane = static_cast<int64_t>(blockIdx.z) * g.grid_y + blockIdx.y;
    const uint32_t idx = blockIdx.x * kBlock + threadIdx.x;
    if (plane >= planes || idx >= static_cast<uint32_t>(g.OH * g.OW)) return;
    const int32_t i = static_cast<int32_t>(fastdiv(idx, g.by_OW));
    const int32_t j = static_cast<int32_t>(idx) - i * g.OW;
    const T* xp = x + plane * g.H * g.W;
    const int32_t r0 = g.sh * i - g.ph, c0 = g.sw * j - g.pw;
    const int32_t kh = KH ? KH : g.kh, kw = KW ? KW : g.kw;
    bool have = false;
    float best = 0.0f;
    int32_t best_k = 0;
    if (KH) {
        // fixed window: every load is issued up front from a clamped address, then the scan
        float v[KH ? KH : 1][KW ? KW : 1];
        bool ok[KH ? KH : 1][KW ? KW : 1];
#pragma unroll
        for (int32_t a = 0; a < KH; ++a)
#pragma unroll
            for (int32_t b = 0; b < KW; ++b) {
                const int32_t r = r0 + g.dh * a, c = c0 + g.dw * b;
                ok[a][b] = r >= 0 && r < g.H && c >= 0 && c < g.W;
                const int32_t rc = min(max(r, 0), g.H - 1), cc = min(max(c, 0), g.W - 1);
                v[a][b] = static_cast<float>(xp[rc * g.W + cc]);
            }
#pragma unroll
        for (int32_t a = 0; a < KH; ++a)
#pragma unroll
            for (int32_t b = 0; b < KW; ++b) {
                const bool take = ok[a][b] && (!have || v[a][b] > best);
                best = take ? v[a][b] : best;
                best_k = take ? a * KW + b : best_k;
                have = have || ok[a][b];
            }
    } else {
        for (int32_t a = 0; a < kh; ++a) {
            const int32_t r = r0 + g.dh * a;
            if (r < 0 || r >= g.H) continue;
            for (int32_t b = 0; b < kw; ++b) {
                const int32_t c = c0 + g.dw * b;
                if (c < 0 || c >= g.W) continue;
                const float v = static_cast<float>(xp[r * g.W + c]);
                if (!have || v > best) {
                    have = true;
                    best = v;
                    best_k = a * kw + b;
                }
            }
        }
    }
    const int64_t o = plane * g.OH * g.OW + idx;
    y[o] = static_cast<T>(best);  // exact: `best` is one of the inputs
    argmax[o] = static_cast<uint8_t>(best_k);
}

// One thread per input location.  The outputs whose window contains it are visited row by row
// (ascending output row, then column) and those whose stored position points here are added
// in binary32, the order in which a scatter over the outputs would have added them.
// MC > 0: at most MC output rows (and MC output columns) have a window that contains a given
// input location, i.e. ceil((d*(k-1)+1) / s) <= MC in both directions; the candidates are then
// enumerated directly and all their loads are issued up front from clamped addresses.
// MC = 0: any geometry, window positions scanned one by one.
template <typename T, int MC>
__global__ __launch_bounds__(kBlock) void maxpool2d_backward_kernel(const uint8_t* __restrict__ argmax,
                                                                    const T* __restrict__ grad_y, int64_t planes,
                                                                    Pool g, T* __restrict__ grad_x)
{
    const int64_t plane = static_cast<int64_t>(blockIdx.z) * g.grid_y + blockIdx.y;
    const uint32_t idx = blockIdx.x * kBlock + threadIdx.x;
    if (plane >= planes || idx >= static_cast<uint32_t>(g.H * g.W)) return;
    const int32_t r = static_cast<int32_t>(fastdiv(idx, g.by_W));
    const int32_t c = static_cast<int32_t>(idx) - r * g.W;
    const uint8_t* ap = argmax + plane * g.OH * g.OW;
    const T* gp = grad_y + plane * g.OH * g.OW;
    float acc = 0.0f;
    if (MC) {
        // output rows i with 0 <= r + ph - sh*i <= dh*(kh-1), the offset a multiple of dh
        const int32_t i_hi = static_cast<int32_t>(fastdiv(static_cast<uint32_t>(r + g.ph), g.by_sh));
        const int32_t j_hi = static_cast<int32_t>(fastdiv(static_cast<uint32_t>(c + g.pw), g.by_sw));
        uint32_t code[MC ? MC : 1][MC ? MC : 1];
        float gy[MC ? MC : 1][MC ? MC : 1];
        int32_t want[MC ? MC : 1][MC ? MC : 1];
#pragma unroll
        for (int32_t u = MC - 1; u >= 0; --u)
#pragma unroll
            for (int32_t v = MC - 1; v >= 0; --v) {
                const int32_t i = i_hi - u, j = j_hi - v;
                const int32_t off_r = r + g.ph - g.sh * i, off_c = c + g.pw - g.sw * j;  // >= 0
                const int32_t a = static_cast<int32_t>(fastdiv(static_cast<uint32_t>(off_r), g.by_dh));
                const int32_t b = static_cast<int32_t>(fastdiv(static_cast<uint32_t>(off_c), g.by_dw));
                const bool ok = i >= 0 && j >= 0 && i < g.OH && j < g.OW && a < g.kh && b < g.kw &&
                                a * g.dh == off_r && b * g.dw == off_c;
                const int32_t ic = min(max(i, 0), g.OH - 1), jc = min(max(j, 0), g.OW - 1);
                code[u][v] = ap[ic * g.OW + jc];
                gy[u][v] = static_cast<float>(gp[ic * g.OW + jc]);
                want[u][v] = ok ? a * g.kw + b : -1;
            }
        // ascending output row, then column
#pragma unroll
        for (int32_t u = MC - 1; u >= 0; --u)
#pragma unroll
            for (int32_t v = MC - 1; v >= 0; --v)
                acc += static_cast<int32_t>(code[u][v]) == want[u][v] ? gy[u][v] : 0.0f;  // + 0 changes nothing
    } else {
        for (int32_t a = g.kh - 1; a >= 0; --a) {  // descending window row = ascending output row
            const int32_t tr = r + g.ph - g.dh * a;
            if (tr < 0) continue;
            const int32_t i = static_cast<int32_t>(fastdiv(static_cast<uint32_t>(tr), g.by_sh));
            if (i * g.sh != tr || i >= g.OH) continue;
            for (int32_t b = g.kw - 1; b >= 0; --b) {
                const int32_t tc = c + g.pw - g.dw * b;
                if (tc < 0) continue;
                const int32_t j = static_cast<int32_t>(fastdiv(static_cast<uint32_t>(tc), g.by_sw));
                if (j * g.sw != tc || j >= g.OW) continue;
                if (ap[i * g.OW + j] == static_cast<uint8_t>(a * g.kw + b)) acc += static_cast<float>(gp[i * g.OW + j]);
            }
        }
    }
    grad_x[plane * g.H * g.W + idx] = static_cast<T>(acc);
}

// ------------------------------------------------------------------------------------
// Backward fast path for the common geometries: square window K in {2, 3}, stride S in {1, 2},
// dilation 1, any legal padding.  With one element per lane the backward kernel is bound by
// instruction issue, not by HBM (a wavefront that produces 256 bytes can afford only about two
// dozen vector instructions), so here a lane produces four consecutive elements of a row: the
// index arithmetic, the row checks and the loads of the neighbouring outputs are shared, and
// the result leaves as one 128-bit (binary16: 64-bit) store.  The arithmetic and its order are
// those of the kernel above.  (The same regrouping of the forward kernel was measured slower:
// four windows per lane spread every load of the wavefront over four times as many cache lines.)

template <typename T>
struct Quad;
template <>
struct Quad<float> {
    typedef float vec __attribute__((ext_vector_type(4)));
};
template <>
struct Quad<_Float16> {
    typedef _Float16 vec __attribute__((ext_vector_type(4)));
};

struct QuadGeometry {
    int32_t quads_per_row;  // ceil(row length / 4) of the tensor the kernel produces
    FastDiv by_quads;
    uint32_t vector_ok;     // rows are a multiple of 4 long and the outputs are aligned for vector stores
};

template <typename T, int K, int S>
__global__ __launch_bounds__(kBlock) void maxpool2d_backward_quad_kernel(const uint8_t* __restrict__ argmax,
                                                                         const T* __restrict__ grad_y, int64_t planes,
                                                                         Pool g, QuadGeometry q, T* __restrict__ grad_x)
{
    constexpr int LOG_S = S == 2 ? 1 : 0;
    constexpr int MR = (K - 1) / S + 1;      // output rows whose window can contain one input row
    constexpr int NJ = (S + K + 1) / S + 1;  // output columns whose window can contain one of four input columns
    const int64_t plane = static_cast<int64_t>(blockIdx.z) * g.grid_y + blockIdx.y;
    const uint32_t idx = blockIdx.x * kBlock + threadIdx.x;
    if (plane >= planes || idx >= static_cast<uint32_t>(g.H * q.quads_per_row)) return;
    const int32_t r = static_cast<int32_t>(fastdiv(idx, q.by_quads));
    const int32_t c0 = (static_cast<int32_t>(idx) - r * q.quads_per_row) * 4;
    const uint8_t* ap = argmax + plane * g.OH * g.OW;
    const T* gp = grad_y + plane * g.OH * g.OW;
    // c0 is a multiple of 4 and S divides 4, so the position of column c0 + e inside the window
    // of output column j_lo + t is the same for every lane: b = spare + (K - 1) + e - S*t
    const int32_t spare = S == 2 ? ((g.pw - (K - 1)) & 1) : 0;  // (c0 + pw - (K-1)) mod S
    const int32_t j_lo = (c0 + g.pw - (K - 1) - spare) >> LOG_S;  // exact; arithmetic shift for negative values
    const int32_t i_hi = (r + g.ph) >> LOG_S;
    uint32_t code[MR][NJ];
    float gy[MR][NJ];
    int32_t row_code[MR];                    // a * K for the row, or a value no stored position can match
#pragma unroll
    for (int u = 0; u < MR; ++u) {
        const int32_t i = i_hi - u;
        const int32_t a = r + g.ph - S * i;  // >= 0
        const bool row_ok = i >= 0 && i < g.OH && a < K;
        row_code[u] = row_ok ? a * K : -1000;
        const int32_t ic = min(max(i, 0), g.OH - 1);
#pragma unroll
        for (int t = 0; t < NJ; ++t) {
            const int32_t j = j_lo + t;
            const int32_t jc = min(max(j, 0), g.OW - 1);
            const bool ok = j >= 0 && j < g.OW;
            code[u][t] = ok ? static_cast<uint32_t>(ap[ic * g.OW + jc]) : 0xffffu;
            gy[u][t] = static_cast<float>(gp[ic * g.OW + jc]);
        }
    }
    typename Quad<T>::vec out;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float acc = 0.0f;
#pragma unroll
        for (int u = MR - 1; u >= 0; --u)    // ascending output row
#pragma unroll
            for (int t = 0; t < NJ; ++t) {   // ascending output column
                const int32_t b = spare + (K - 1) + e - S * t;  // the same in every lane
                if (b < 0 || b >= K) continue;
                acc += static_cast<int32_t>(code[u][t]) == row_code[u] + b ? gy[u][t] : 0.0f;  // + 0 changes nothing
            }
        out[e] = static_cast<T>(acc);
    }
    const int64_t o = plane * g.H * g.W + r * g.W + c0;
    if (q.vector_ok) {
        __builtin_nontemporal_store(out, reinterpret_cast<typename Quad<T>::vec*>(grad_x + o));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (c0 + e < g.W) grad_x[o + e] = out[e];
    }
}

}  // namespace

int launch_relu_forward(const void* x, int dtype, int64_t n, void* y, uint8_t* mask, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t mask_words = (n + 255) / 256 * 8;
    if (dtype == ACTQ_F32) {
        const int64_t tiles = (n + 1023) / 1024;
        relu_forward_kernel<float><<<static_cast<unsigned>((tiles + kWavesPerBlock - 1) / kWavesPerBlock), kBlock, 0, s>>>(
            static_cast<const float*>(x), n, mask_words, static_cast<float*>(y), reinterpret_cast<uint32_t*>(mask));
    } else {
        const int64_t tiles = (n + 2047) / 2048;
        relu_forward_kernel<_Float16><<<static_cast<unsigned>((tiles + kWavesPerBlock - 1) / kWavesPerBlock), kBlock, 0, s>>>(
            static_cast<const _Float16*>(x), n, mask_words, static_cast<_Float16*>(y), reinterpret_cast<uint32_t*>(mask));
    }
    return launched("actq_relu_forward");
}

int launch_relu_backward(const uint8_t* mask, const void* grad_y, int dtype, int64_t n, void* grad_x, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t mask_words = (n + 255) / 256 * 8;
    if (dtype == ACTQ_F32) {
        const int64_t tiles = (n + 1023) / 1024;
        relu_backward_kernel<float><<<static_cast<unsigned>((tiles + kWavesPerBlock - 1) / kWavesPerBlock), kBlock, 0, s>>>(
            reinterpret_cast<const uint32_t*>(mask), mask_words, static_cast<const float*>(grad_y), n, static_cast<float*>(grad_x));
    } else {
        const int64_t tiles = (n + 2047) / 2048;
        relu_backward_kernel<_Float16><<<static_cast<unsigned>((tiles + kWavesPerBlock - 1) / kWavesPerBlock), kBlock, 0, s>>>(
            reinterpret_cast<const uint32_t*>(mask), mask_words, static_cast<const _Float16*>(grad_y), n, static_cast<_Float16*>(grad_x));
    }
    return launched("actq_relu_backward");
}

static Pool make_pool(const PoolShape& p, int64_t planes, int64_t per_plane, dim3* grid)
{
    Pool g;
    g.H = p.H; g.W = p.W; g.OH = p.OH; g.OW = p.OW;
    g.kh = p.kh; g.kw = p.kw; g.sh = p.sh; g.sw = p.sw;
    g.ph = p.ph; g.pw = p.pw; g.dh = p.dh; g.dw = p.dw;
    g.by_OW = make_fastdiv(static_cast<uint32_t>(p.OW));
    g.by_W = make_fastdiv(static_cast<uint32_t>(p.W));
    g.by_sh = make_fastdiv(static_cast<uint32_t>(p.sh));
    g.by_sw = make_fastdiv(static_cast<uint32_t>(p.sw));
    g.by_dh = make_fastdiv(static_cast<uint32_t>(p.dh));
    g.by_dw = make_fastdiv(static_cast<uint32_t>(p.dw));
    const int64_t gy = planes < 65535 ? planes : 65535;
    g.grid_y = static_cast<uint32_t>(gy);
    *grid = dim3(static_cast<unsigned>((per_plane + kBlock - 1) / kBlock), static_cast<unsigned>(gy),
                 static_cast<unsigned>((planes + gy - 1) / gy));
    return g;
}

// Forward fast path for stride 2, square windows K in {2, 3}, padding <= 1, dilation 1, rows a
// multiple of four long.  The vector memory pipeline moves 64 bytes per clock and compute unit
// whatever the width of the load, so nine 32-bit loads per output (16 clocks each for a
// wavefront) keep it busier than HBM.  Here a lane produces two neighbouring outputs from one
// aligned 128-bit load per window row plus at most one 32-bit load on either side: three times
// fewer load cycles per output.  Window positions and their order are those of the kernel above.
template <typename T, int K>
__global__ __launch_bounds__(kBlock) void maxpool2d_forward_pair_kernel(const T* __restrict__ x, int64_t planes, Pool g,
                                                                        QuadGeometry q, T* __restrict__ y,
                                                                        uint8_t* __restrict__ argmax)
{
    typedef typename Quad<T>::vec vec4;
    const int64_t plane = static_cast<int64_t>(blockIdx.z) * g.grid_y + blockIdx.y;
    const uint32_t idx = blockIdx.x * kBlock + threadIdx.x;
    if (plane >= planes || idx >= static_cast<uint32_t>(g.OH * q.quads_per_row)) return;  // pairs per row here
    const int32_t i = static_cast<int32_t>(fastdiv(idx, q.by_quads));
    const int32_t m = static_cast<int32_t>(idx) - i * q.quads_per_row;   // outputs 2m and 2m + 1
    const T* xp = x + plane * g.H * g.W;
    const int32_t r0 = 2 * i - g.ph;
    const int32_t c4 = 4 * m;                  // first column of the aligned quad
    // slot t holds input column c4 - 1 + t: slot 0 the left neighbour, 1..4 the quad, 5 the right neighbour
    float v[K][6];
    bool col_ok[6], row_ok[K];
#pragma unroll
    for (int t = 0; t < 6; ++t) col_ok[t] = c4 - 1 + t >= 0 && c4 - 1 + t < g.W;
    const bool quad_ok = c4 + 3 < g.W;
#pragma unroll
    for (int a = 0; a < K; ++a) {
        const int32_t r = r0 + a;
        row_ok[a] = r >= 0 && r < g.H;
        const T* row = xp + min(max(r, 0), g.H - 1) * g.W;
        if (quad_ok) {
            const vec4 w = *reinterpret_cast<const vec4*>(row + c4);
            v[a][1] = static_cast<float>(w[0]); v[a][2] = static_cast<float>(w[1]);
            v[a][3] = static_cast<float>(w[2]); v[a][4] = static_cast<float>(w[3]);
        } else {
#pragma unroll
            for (int t = 1; t < 5; ++t) v[a][t] = static_cast<float>(row[min(c4 - 1 + t, g.W - 1)]);
        }
        v[a][0] = static_cast<float>(row[max(c4 - 1, 0)]);
        v[a][5] = static_cast<float>(row[min(c4 + 4, g.W - 1)]);
    }
    float best[2];
    uint32_t best_k[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        bool have = false;
        best[e] = 0.0f;
        best_k[e] = 0;
#pragma unroll
        for (int a = 0; a < K; ++a)
#pragma unroll
            for (int b = 0; b < K; ++b) {
                // column 2 * (2m + e) - pw + b = c4 + 2e - pw + b: slot 2e + b + 1 - pw, pw in {0, 1}
                const float val = g.pw ? v[a][2 * e + b] : v[a][2 * e + b + 1];
                const bool ok = row_ok[a] && (g.pw ? col_ok[2 * e + b] : col_ok[2 * e + b + 1]);
                const bool take = ok && (!have || val > best[e]);
                best[e] = take ? val : best[e];
                best_k[e] = take ? static_cast<uint32_t>(a * K + b) : best_k[e];
                have = have || ok;
            }
    }
    const int64_t o = plane * g.OH * g.OW + i * g.OW + 2 * m;
    if (2 * m + 1 < g.OW) {   // OW is even on this path, so this always holds; kept as the guard of the pair store
        typedef T pair __attribute__((ext_vector_type(2)));
        pair out;
        out[0] = static_cast<T>(best[0]);
        out[1] = static_cast<T>(best[1]);
        __builtin_nontemporal_store(out, reinterpret_cast<pair*>(y + o));
        __builtin_nontemporal_store(static_cast<uint16_t>(best_k[0] | (best_k[1] << 8)), reinterpret_cast<uint16_t*>(argmax + o));
    }
}

// The same with four outputs per lane when the rows allow it (input rows a multiple of eight and
// output rows a multiple of four long): two aligned 128-bit loads and at most one 32-bit load per
// window row serve four windows.
template <typename T, int K, int P>
__global__ __launch_bounds__(kBlock) void maxpool2d_forward_four_kernel(const T* __restrict__ x, int64_t planes, Pool g,
                                                                        QuadGeometry q, T* __restrict__ y,
                                                                        uint8_t* __restrict__ argmax)
{
    typedef typename Quad<T>::vec vec4;
    const int64_t plane = static_cast<int64_t>(blockIdx.z) * g.grid_y + blockIdx.y;
    const uint32_t idx = blockIdx.x * kBlock + threadIdx.x;
    if (plane >= planes || idx >= static_cast<uint32_t>(g.OH * q.quads_per_row)) return;
    const int32_t i = static_cast<int32_t>(fastdiv(idx, q.by_quads));
    const int32_t m = static_cast<int32_t>(idx) - i * q.quads_per_row;   // outputs 4m .. 4m+3
    const T* xp = x + plane * g.H * g.W;
    const int32_t r0 = 2 * i - P;
    const int32_t c8 = 8 * m;                  // slot t holds input column c8 - 1 + t
    float v[K][9];
    bool row_ok[K];
    const bool left_ok = c8 >= 1;
#pragma unroll
    for (int a = 0; a < K; ++a) {
        const int32_t r = r0 + a;
        row_ok[a] = r >= 0 && r < g.H;
        const T* row = xp + min(max(r, 0), g.H - 1) * g.W;
        const vec4 w0 = *reinterpret_cast<const vec4*>(row + c8);
        const vec4 w1 = *reinterpret_cast<const vec4*>(row + c8 + 4);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            v[a][1 + t] = static_cast<float>(w0[t]);
            v[a][5 + t] = static_cast<float>(w1[t]);
        }
        v[a][0] = P ? static_cast<float>(row[max(c8 - 1, 0)]) : 0.0f;
    }
    vec4 out;
    uint32_t codes = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        bool have = false;
        float best = 0.0f;
        uint32_t best_k = 0;
#pragma unroll
        for (int a = 0; a < K; ++a)
#pragma unroll
            for (int b = 0; b < K; ++b) {
                constexpr int kShift = 1 - P;
                const int t = 2 * e + b + kShift;  // column 2 * (4m + e) - P + b = c8 - 1 + t
                const bool ok = row_ok[a] && (t > 0 || left_ok);
                const bool take = ok && (!have || v[a][t] > best);
                best = take ? v[a][t] : best;
                best_k = take ? static_cast<uint32_t>(a * K + b) : best_k;
                have = have || ok;
            }
        out[e] = static_cast<T>(best);
        codes |= best_k << (8 * e);
    }
    const int64_t o = plane * g.OH * g.OW + i * g.OW + 4 * m;
    __builtin_nontemporal_store(out, reinterpret_cast<vec4*>(y + o));
    __builtin_nontemporal_store(codes, reinterpret_cast<uint32_t*>(argmax + o));
}

// Forward path for the common down-sampling pools (3x3 / stride 2 / padding 1 and 2x2 / stride 2 /
// padding 0 on even extents, H = 2 OH and W = 2 OW, rows a multiple of 16 bytes long).  Because
// H = 2 OH, output row q = plane * OH + i of the whole tensor reads the rows 2q - P .. 2q - P + K - 1
// of the whole input, so planes and rows flatten into one index.  A lane owns 16 bytes of an input
// row (E = 4 or 8 columns) and R consecutive output rows; every load instruction of a wavefront then
// covers whole cache lines (the window-per-lane kernels above touch each line from several
// instructions, which makes the first-level cache, not HBM, the limit).  The one column to the left
// of a lane's 16 bytes (P = 1) comes from the neighbouring lane by a wavefront shift; lane 0 takes
// it through the scalar data path.
struct StreamPool {
    uint32_t chunks_per_row;   // W / E
    FastDiv by_chunks, by_rows;  // by_rows: division by OH / R
    uint32_t rows_per_plane;   // OH / R
    uint32_t total;            // planes * (OH / R) * chunks_per_row
};

template <typename V>
__device__ __forceinline__ V load_uniform(const V* p)
{
    typedef const V __attribute__((address_space(4))) * constant_ptr;
    return *(constant_ptr)(reinterpret_cast<uintptr_t>(p));
}

__device__ __forceinline__ float from_left_lane(float v)
{
    constexpr int kWaveShiftRight1 = 0x138;
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), kWaveShiftRight1, 0xf, 0xf, false));
}

#ifndef ACTQ_POOL_FWD_BLOCK
#define ACTQ_POOL_FWD_BLOCK 256
#endif
#ifndef ACTQ_POOL_BWD_BLOCK
#define ACTQ_POOL_BWD_BLOCK 256
#endif
constexpr int kPoolFwdBlock = ACTQ_POOL_FWD_BLOCK;   // threads per block of the streaming pooling kernels
constexpr int kPoolBwdBlock = ACTQ_POOL_BWD_BLOCK;

template <typename T, int K, int P, int R>
__global__ __launch_bounds__(kPoolFwdBlock) void maxpool2d_forward_stream_kernel(const T* __restrict__ x, Pool g, StreamPool q,
                                                                          T* __restrict__ y,
                                                                          uint8_t* __restrict__ argmax)
{
    constexpr int E = 16 / sizeof(T);    // input columns per lane
    constexpr int NO = E / 2;            // outputs per lane and output row
    constexpr int NR = 2 * R + K - 2;    // input rows per lane
    typedef T vec_in __attribute__((ext_vector_type(E)));
    typedef T vec_out __attribute__((ext_vector_type(NO)));
    const uint32_t idx = blockIdx.x * kPoolFwdBlock + threadIdx.x;
    const bool live = idx < q.total;
    // lanes past the end repeat the last lane's loads (every lane takes part in the shift) and store nothing
    const uint32_t id = live ? idx : q.total - 1;
    const uint32_t strip = fastdiv(id, q.by_chunks);            // plane * (OH / R) + i / R
    const uint32_t c = id - strip * q.chunks_per_row;
    const uint32_t plane = fastdiv(strip, q.by_rows);
    const bool top = strip - plane * q.rows_per_plane == 0;     // the strip starts at output row 0 of its plane
    const int64_t q0 = static_cast<int64_t>(strip) * R;         // first output row, counted over all planes
    const bool left_ok = c > 0;
    const int lane = threadIdx.x & (kWave - 1);
    float v[NR][E + 1];   // slot 0: the column left of the lane's own, slots 1..E its own
    bool row_ok[NR];
#pragma unroll
    for (int a = 0; a < NR; ++a) {
        row_ok[a] = !(P == 1 && a == 0 && top);
        // the row above the plane is padding: read the plane's first row instead and ignore it
        const int64_t r = 2 * q0 - P + a + (row_ok[a] ? 0 : 1);
        const T* row = x + r * g.W + static_cast<int64_t>(E) * c;
        const vec_in w = *reinterpret_cast<const vec_in*>(row);
#pragma unroll
        for (int t = 0; t < E; ++t) v[a][1 + t] = static_cast<float>(w[t]);
        v[a][0] = 0.0f;
        if (P == 1) {
            v[a][0] = from_left_lane(v[a][E]);
            // lane 0 has no neighbour: its left column comes through the scalar data path, as the
            // aligned 32-bit word that ends where the lane's own 16 bytes start
            const uint32_t c_first = __builtin_amdgcn_readfirstlane(c);
            const uint32_t r_lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(r));
            const uint32_t r_hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(static_cast<uint64_t>(r) >> 32));
            const int64_t r_first = static_cast<int64_t>((static_cast<uint64_t>(r_hi) << 32) | r_lo);
            const T* first = x + r_first * g.W + static_cast<int64_t>(E) * c_first;
            float edge = 0.0f;
            if (c_first > 0) {
                const uint32_t word = load_uniform(reinterpret_cast<const uint32_t*>(first) - 1);
                if (sizeof(T) == 4) edge = __uint_as_float(word);
                else {
                    const uint16_t hi = static_cast<uint16_t>(word >> 16);
                    _Float16 h;
                    __builtin_memcpy(&h, &hi, 2);
                    edge = static_cast<float>(h);
                }
            }
            v[a][0] = lane == 0 ? edge : v[a][0];
        }
    }
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        vec_out out;
        uint32_t codes = 0;
#pragma unroll
        for (int e = 0; e < NO; ++e) {
            bool have = false;
            float best = 0.0f;
            uint32_t best_k = 0;
#pragma unroll
            for (int a = 0; a < K; ++a)
#pragma unroll
                for (int b = 0; b < K; ++b) {
                    const int t = 2 * e + b + 1 - P;   // column 2 * (NO c + e) - P + b = E c - 1 + t
                    const bool ok = row_ok[2 * rr + a] && (t > 0 || left_ok);
                    const bool take = ok && (!have || v[2 * rr + a][t] > best);
                    best = take ? v[2 * rr + a][t] : best;
                    best_k = take ? static_cast<uint32_t>(a * K + b) : best_k;
                    have = have || ok;
                }
            out[e] = static_cast<T>(best);
            codes |= best_k << (8 * e);
        }
        if (!live) continue;
        const int64_t o = (q0 + rr) * g.OW + static_cast<int64_t>(NO) * c;
        __builtin_nontemporal_store(out, reinterpret_cast<vec_out*>(y + o));
        if (NO == 2) __builtin_nontemporal_store(static_cast<uint16_t>(codes), reinterpret_cast<uint16_t*>(argmax + o));
        else __builtin_nontemporal_store(codes, reinterpret_cast<uint32_t*>(argmax + o));
    }
}

// Backward fast path for stride 2, square windows K in {2, 3}, padding P <= 1, dilation 1, input
// rows a multiple of eight and output rows a multiple of four long.  A lane produces eight
// consecutive inputs of a row.  The outputs whose window can contain one of them are the six
// columns 4m-1 .. 4m+4 of one or two output rows: their gradients come in as one aligned 128-bit
// load plus a 32-bit load on either side, their positions as one 32-bit load plus two bytes --
// twelve loads for eight inputs instead of four loads per input.  Which window position an
// output column would need for an input column is fixed at compile time; the order of the
// additions is that of the kernels above (ascending output row, then column).
template <typename T, int K, int P>
__global__ __launch_bounds__(kBlock) void maxpool2d_backward_oct_kernel(const uint8_t* __restrict__ argmax,
                                                                        const T* __restrict__ grad_y, int64_t planes,
                                                                        Pool g, QuadGeometry q, T* __restrict__ grad_x)
{
    typedef typename Quad<T>::vec vec4;
    constexpr int MR = (K - 1) / 2 + 1;   // output rows whose window can contain one input row
    const int64_t plane = static_cast<int64_t>(blockIdx.z) * g.grid_y + blockIdx.y;
    const uint32_t idx = blockIdx.x * kBlock + threadIdx.x;
    if (plane >= planes || idx >= static_cast<uint32_t>(g.H * q.quads_per_row)) return;  // octets per row here
    const int32_t r = static_cast<int32_t>(fastdiv(idx, q.by_quads));
    const int32_t m = static_cast<int32_t>(idx) - r * q.quads_per_row;   // inputs 8m .. 8m+7
    const uint8_t* ap = argmax + plane * g.OH * g.OW;
    const T* gp = grad_y + plane * g.OH * g.OW;
    const int32_t j4 = 4 * m;                 // slot t is output column j4 - 1 + t
    const int32_t i_hi = (r + P) >> 1;
    float gy[MR][6];
    uint32_t code[MR][6];
    int32_t row_code[MR];                     // a * K for the row, or a value no stored position can match
    const bool quad_ok = j4 + 3 < g.OW;
#pragma unroll
    for (int u = 0; u < MR; ++u) {
        const int32_t i = i_hi - u;
        const int32_t a = r + P - 2 * i;      // >= 0
        row_code[u] = (i >= 0 && i < g.OH && a < K) ? a * K : -1000;
        const int32_t base = min(max(i, 0), g.OH - 1) * g.OW;
        if (quad_ok) {
            const vec4 w = *reinterpret_cast<const vec4*>(gp + base + j4);
            const uint32_t c = *reinterpret_cast<const uint32_t*>(ap + base + j4);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                gy[u][1 + t] = static_cast<float>(w[t]);
                code[u][1 + t] = (c >> (8 * t)) & 0xffu;
            }
        } else {
#pragma unroll
            for (int t = 1; t < 5; ++t) {
                const int32_t j = j4 - 1 + t;
                gy[u][t] = static_cast<float>(gp[base + min(j, g.OW - 1)]);
                code[u][t] = j < g.OW ? static_cast<uint32_t>(ap[base + min(j, g.OW - 1)]) : 0xffffu;
            }
        }
        gy[u][0] = static_cast<float>(gp[base + max(j4 - 1, 0)]);
        code[u][0] = j4 >= 1 ? static_cast<uint32_t>(ap[base + max(j4 - 1, 0)]) : 0xffffu;
        gy[u][5] = static_cast<float>(gp[base + min(j4 + 4, g.OW - 1)]);
        code[u][5] = j4 + 4 < g.OW ? static_cast<uint32_t>(ap[base + min(j4 + 4, g.OW - 1)]) : 0xffffu;
    }
    T out[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float acc = 0.0f;
#pragma unroll
        for (int u = MR - 1; u >= 0; --u)     // ascending output row
#pragma unroll
            for (int t = 0; t < 6; ++t) {     // ascending output column
                constexpr int kOffset = P + 2;
                const int b = e + kOffset - 2 * t;   // position of input column 8m+e in the window of column j4-1+t
                if (b < 0 || b >= K) continue;
                acc += static_cast<int32_t>(code[u][t]) == row_code[u] + b ? gy[u][t] : 0.0f;  // + 0 changes nothing
            }
        out[e] = static_cast<T>(acc);
    }
    T* dst = grad_x + plane * g.H * g.W + r * g.W + 8 * m;
    vec4 lo, hi;
#pragma unroll
    for (int e = 0; e < 4; ++e) { lo[e] = out[e]; hi[e] = out[4 + e]; }
    __builtin_nontemporal_store(lo, reinterpret_cast<vec4*>(dst));
    __builtin_nontemporal_store(hi, reinterpret_cast<vec4*>(dst) + 1);
}

// Backward counterpart of the streaming forward kernel, for the same geometries.  A lane owns the
// NO = E / 2 output columns of one output row q (counted over all planes) that lie over its 16
// bytes of input columns, and produces the two input rows 2q and 2q + 1 there: every gradient and
// position is loaded once per output row that needs it, in whole cache lines, and the results
// leave as two 128-bit stores.  With a 3x3 window input row 2q + 1 also lies in the window of
// output row q + 1, and the lane's last column in that of the first output column of the lane to
// its right, which arrives by a wavefront shift (lane 63 takes it through the scalar data path).
// The additions run over ascending output row, then column, as in the kernels above.
__device__ __forceinline__ uint32_t from_right_lane(uint32_t v)
{
    constexpr int kWaveShiftLeft1 = 0x130;
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), kWaveShiftLeft1, 0xf, 0xf, false));
}

template <typename T, int K, int P>
__global__ __launch_bounds__(kPoolBwdBlock) void maxpool2d_backward_stream_kernel(const uint8_t* __restrict__ argmax,
                                                                           const T* __restrict__ grad_y, Pool g,
                                                                           StreamPool q, T* __restrict__ grad_x)
{
    constexpr int E = 16 / sizeof(T);    // input columns per lane
    constexpr int NO = E / 2;            // output columns per lane
    constexpr int MR = K == 3 ? 2 : 1;   // output rows whose windows reach the lane's two input rows
    typedef T vec_in __attribute__((ext_vector_type(E)));
    typedef T vec_out __attribute__((ext_vector_type(NO)));
    typedef typename std::conditional<NO == 2, uint16_t, uint32_t>::type code_word;
    const uint32_t idx = blockIdx.x * kPoolBwdBlock + threadIdx.x;
    const bool live = idx < q.total;
    const uint32_t id = live ? idx : q.total - 1;   // every lane takes part in the shift
    const uint32_t strip = fastdiv(id, q.by_chunks);             // output row over all planes
    const uint32_t ch = id - strip * q.chunks_per_row;
    const uint32_t plane = fastdiv(strip, q.by_rows);
    const bool bottom = strip - plane * q.rows_per_plane == q.rows_per_plane - 1;
    const bool right_ok = ch + 1 < q.chunks_per_row;
    const int lane = threadIdx.x & (kWave - 1);
    float gy[MR][NO + 1];
    uint32_t code[MR][NO + 1];
    bool valid[MR];
#pragma unroll
    for (int u = 0; u < MR; ++u) {
        valid[u] = !(u == 1 && bottom);   // below the plane's last output row there is nothing
        const int64_t at = (static_cast<int64_t>(strip) + (valid[u] ? u : 0)) * g.OW + static_cast<int64_t>(NO) * ch;
        const vec_out w = *reinterpret_cast<const vec_out*>(grad_y + at);
        const uint32_t cw = *reinterpret_cast<const code_word*>(argmax + at);
#pragma unroll
        for (int t = 0; t < NO; ++t) {
            gy[u][t] = static_cast<float>(w[t]);
            code[u][t] = (cw >> (8 * t)) & 0xffu;
        }
        gy[u][NO] = 0.0f;
        code[u][NO] = 0;
        if (K == 3) {
            gy[u][NO] = __uint_as_float(from_right_lane(__float_as_uint(gy[u][0])));
            code[u][NO] = from_right_lane(code[u][0]);
            // lane 63: the element after its own, as aligned 32-bit words through the scalar data path
            const uint32_t at_lo = __builtin_amdgcn_readlane(static_cast<uint32_t>(at), kWave - 1);
            const uint32_t at_hi = __builtin_amdgcn_readlane(static_cast<uint32_t>(static_cast<uint64_t>(at) >> 32), kWave - 1);
            const bool last_right_ok = __builtin_amdgcn_readlane(static_cast<uint32_t>(right_ok), kWave - 1) != 0;
            const int64_t next = static_cast<int64_t>((static_cast<uint64_t>(at_hi) << 32) | at_lo) + NO;
            float edge_g = 0.0f;
            uint32_t edge_c = 0;
            if (last_right_ok) {
                if (sizeof(T) == 4) {
                    edge_g = __uint_as_float(load_uniform(reinterpret_cast<const uint32_t*>(grad_y) + next));
                } else {
                    // NO = 4: the element is 8-byte aligned, so it is the low half of its word
                    const uint32_t word = load_uniform(reinterpret_cast<const uint32_t*>(grad_y) + (next >> 1));
                    const uint16_t lo = static_cast<uint16_t>(word);
                    _Float16 h;
                    __builtin_memcpy(&h, &lo, 2);
                    edge_g = static_cast<float>(h);
                }
                const uint32_t word = load_uniform(reinterpret_cast<const uint32_t*>(argmax) + (next >> 2));
                edge_c = (word >> (8 * (static_cast<uint32_t>(next) & 3u))) & 0xffu;
            }
            gy[u][NO] = lane == kWave - 1 ? edge_g : gy[u][NO];
            code[u][NO] = lane == kWave - 1 ? edge_c : code[u][NO];
        }
    }
#pragma unroll
    for (int rr = 0; rr < 2; ++rr) {
        vec_in out;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            float acc = 0.0f;
#pragma unroll
            for (int u = 0; u < MR; ++u) {            // ascending output row
                const int a = rr + P - 2 * u;         // row of input row 2q + rr in the window of output row q + u
                if (a < 0 || a >= K) continue;
#pragma unroll
                for (int t = 0; t <= NO; ++t) {       // ascending output column
                    const int b = e + P - 2 * t;      // column E ch + e in the window of output column NO ch + t
                    if (b < 0 || b >= K) continue;
                    const bool ok = valid[u] && (t < NO || right_ok);
                    acc += ok && code[u][t] == static_cast<uint32_t>(a * K + b) ? gy[u][t] : 0.0f;  // + 0 changes nothing
                }
            }
            out[e] = static_cast<T>(acc);
        }
        if (!live) continue;
        T* dst = grad_x + (2 * static_cast<int64_t>(strip) + rr) * g.W + static_cast<int64_t>(E) * ch;
        __builtin_nontemporal_store(out, reinterpret_cast<vec_in*>(dst));
    }
}

static bool aligned_to(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

static bool quad_geometry(const PoolShape& p) {
    return p.kh == p.kw && (p.kh == 2 || p.kh == 3) && p.sh == p.sw && (p.sh == 1 || p.sh == 2) && p.dh == 1 && p.dw == 1;
}

template <typename T>
static void maxpool_forward_typed(const T* x, int64_t planes, const PoolShape& p, T* y, uint8_t* argmax, hipStream_t s)
{
    dim3 grid;
    const bool pair_geometry = p.kh == p.kw && (p.kh == 2 || p.kh == 3) && p.sh == 2 && p.sw == 2 && p.dh == 1 &&
                               p.dw == 1 && p.pw <= 1 && p.W % 4 == 0 && p.OW % 2 == 0 && aligned_to(x, 4 * sizeof(T)) &&
                               aligned_to(y, 2 * sizeof(T)) && aligned_to(argmax, 2);
    // all window columns of four outputs lie inside [8m - 1, 8m + 7]: K = 3 with P = 1, or K = 2 with P = 0
    const bool four_geometry = pair_geometry && p.ph == p.pw && p.W % 8 == 0 && p.OW % 4 == 0 && 2 * p.OW == p.W &&
                               ((p.kh == 3 && p.pw == 1) || (p.kh == 2 && p.pw == 0)) &&
                               aligned_to(y, 4 * sizeof(T)) && aligned_to(argmax, 4);
    // the flattened streaming path: even extents, whole 16-byte chunks per row, fewer than 2^31 lanes
    constexpr int kE = 16 / static_cast<int>(sizeof(T));
    constexpr int kStreamRows = 1;
    const bool stream_geometry = four_geometry && 2 * p.OH == p.H && p.W % kE == 0 && p.OH % kStreamRows == 0 &&
                                 aligned_to(x, 16) &&
                                 planes * (p.OH / kStreamRows) * (p.W / kE) < (int64_t(1) << 31);
    if (stream_geometry) {
        StreamPool q;
        q.chunks_per_row = static_cast<uint32_t>(p.W / kE);
        q.by_chunks = make_fastdiv(q.chunks_per_row);
        q.rows_per_plane = static_cast<uint32_t>(p.OH / kStreamRows);
        q.by_rows = make_fastdiv(q.rows_per_plane);
        q.total = static_cast<uint32_t>(planes * q.rows_per_plane * q.chunks_per_row);
        dim3 unused;
        const Pool g = make_pool(p, planes, 1, &unused);
        const unsigned blocks = (q.total + kPoolFwdBlock - 1) / kPoolFwdBlock;
        if (p.kh == 3) maxpool2d_forward_stream_kernel<T, 3, 1, kStreamRows><<<blocks, kPoolFwdBlock, 0, s>>>(x, g, q, y, argmax);
        else maxpool2d_forward_stream_kernel<T, 2, 0, kStreamRows><<<blocks, kPoolFwdBlock, 0, s>>>(x, g, q, y, argmax);
        return;
    }
    if (four_geometry) {
        QuadGeometry q;
        q.quads_per_row = p.OW / 4;
        q.by_quads = make_fastdiv(static_cast<uint32_t>(q.quads_per_row));
        q.vector_ok = 1;
        const Pool g = make_pool(p, planes, static_cast<int64_t>(p.OH) * q.quads_per_row, &grid);
        if (p.kh == 3) maxpool2d_forward_four_kernel<T, 3, 1><<<grid, kBlock, 0, s>>>(x, planes, g, q, y, argmax);
        else maxpool2d_forward_four_kernel<T, 2, 0><<<grid, kBlock, 0, s>>>(x, planes, g, q, y, argmax);
        return;
    }
    if (pair_geometry) {
        QuadGeometry q;
        q.quads_per_row = p.OW / 2;   // pairs of outputs per row
        q.by_quads = make_fastdiv(static_cast<uint32_t>(q.quads_per_row));
        q.vector_ok = 1;
        const Pool g = make_pool(p, planes, static_cast<int64_t>(p.OH) * q.quads_per_row, &grid);
        if (p.kh == 3) maxpool2d_forward_pair_kernel<T, 3><<<grid, kBlock, 0, s>>>(x, planes, g, q, y, argmax);
        else maxpool2d_forward_pair_kernel<T, 2><<<grid, kBlock, 0, s>>>(x, planes, g, q, y, argmax);
        return;
    }
    const Pool g = make_pool(p, planes, static_cast<int64_t>(p.OH) * p.OW, &grid);
    if (p.kh == 3 && p.kw == 3) maxpool2d_forward_kernel<T, 3, 3><<<grid, kBlock, 0, s>>>(x, planes, g, y, argmax);
    else if (p.kh == 2 && p.kw == 2) maxpool2d_forward_kernel<T, 2, 2><<<grid, kBlock, 0, s>>>(x, planes, g, y, argmax);
    else maxpool2d_forward_kernel<T, 0, 0><<<grid, kBlock, 0, s>>>(x, planes, g, y, argmax);
}

template <typename T>
static void maxpool_backward_typed(const uint8_t* argmax, const T* grad_y, int64_t planes, const PoolShape& p,
                                   T* grad_x, hipStream_t s)
{
    dim3 grid;
    const bool oct_geometry = p.kh == p.kw && (p.kh == 2 || p.kh == 3) && p.sh == 2 && p.sw == 2 && p.dh == 1 &&
                              p.dw == 1 && p.ph <= 1 && p.pw <= 1 && p.ph == p.pw && p.W % 8 == 0 && p.OW % 4 == 0 &&
                              aligned_to(grad_x, 4 * sizeof(T)) && aligned_to(grad_y, 4 * sizeof(T)) &&
                              aligned_to(argmax, 4);
    constexpr int kE = 16 / static_cast<int>(sizeof(T));
    const bool stream_geometry = oct_geometry && 2 * p.OH == p.H && 2 * p.OW == p.W && p.W % kE == 0 &&
                                 ((p.kh == 3 && p.pw == 1) || (p.kh == 2 && p.pw == 0)) && aligned_to(grad_x, 16) &&
                                 aligned_to(grad_y, 8) && planes * p.OH * (p.W / kE) < (int64_t(1) << 31);
    if (stream_geometry) {
        StreamPool q;
        q.chunks_per_row = static_cast<uint32_t>(p.W / kE);
        q.by_chunks = make_fastdiv(q.chunks_per_row);
        q.rows_per_plane = static_cast<uint32_t>(p.OH);
        q.by_rows = make_fastdiv(q.rows_per_plane);
        q.total = static_cast<uint32_t>(planes * q.rows_per_plane * q.chunks_per_row);
        dim3 unused;
        const Pool g = make_pool(p, planes, 1, &unused);
        const unsigned blocks = (q.total + kPoolBwdBlock - 1) / kPoolBwdBlock;
        if (p.kh == 3) maxpool2d_backward_stream_kernel<T, 3, 1><<<blocks, kPoolBwdBlock, 0, s>>>(argmax, grad_y, g, q, grad_x);
        else maxpool2d_backward_stream_kernel<T, 2, 0><<<blocks, kPoolBwdBlock, 0, s>>>(argmax, grad_y, g, q, grad_x);
        return;
    }
    if (oct_geometry) {
        QuadGeometry q;
        q.quads_per_row = p.W / 8;   // octets of inputs per row
        q.by_quads = make_fastdiv(static_cast<uint32_t>(q.quads_per_row));
        q.vector_ok = 1;
        const Pool g = make_pool(p, planes, static_cast<int64_t>(p.H) * q.quads_per_row, &grid);
#define ACTQ_POOL_OCT(K, P) maxpool2d_backward_oct_kernel<T, K, P><<<grid, kBlock, 0, s>>>(argmax, grad_y, planes, g, q, grad_x)
        if (p.kh == 3 && p.pw == 1) ACTQ_POOL_OCT(3, 1);
        else if (p.kh == 3) ACTQ_POOL_OCT(3, 0);
        else if (p.pw == 1) ACTQ_POOL_OCT(2, 1);
        else ACTQ_POOL_OCT(2, 0);
#undef ACTQ_POOL_OCT
        return;
    }
    if (quad_geometry(p)) {
        QuadGeometry q;
        q.quads_per_row = (p.W + 3) / 4;
        q.by_quads = make_fastdiv(static_cast<uint32_t>(q.quads_per_row));
        q.vector_ok = p.W % 4 == 0 && aligned_to(grad_x, 4 * sizeof(T));
        const Pool g = make_pool(p, planes, static_cast<int64_t>(p.H) * q.quads_per_row, &grid);
#define ACTQ_POOL_BWD(K, S) maxpool2d_backward_quad_kernel<T, K, S><<<grid, kBlock, 0, s>>>(argmax, grad_y, planes, g, q, grad_x)
        if (p.kh == 3 && p.sh == 2) ACTQ_POOL_BWD(3, 2);
        else if (p.kh == 3) ACTQ_POOL_BWD(3, 1);
        else if (p.sh == 2) ACTQ_POOL_BWD(2, 2);
        else ACTQ_POOL_BWD(2, 1);
#undef ACTQ_POOL_BWD
        return;
    }
    const Pool g = make_pool(p, planes, static_cast<int64_t>(p.H) * p.W, &grid);
    // how many output rows / columns can contain one input location
    const int64_t reach_h = (static_cast<int64_t>(p.dh) * (p.kh - 1) + p.sh) / p.sh;
    const int64_t reach_w = (static_cast<int64_t>(p.dw) * (p.kw - 1) + p.sw) / p.sw;
    const int64_t reach = reach_h > reach_w ? reach_h : reach_w;
    if (reach <= 1) maxpool2d_backward_kernel<T, 1><<<grid, kBlock, 0, s>>>(argmax, grad_y, planes, g, grad_x);
    else if (reach == 2) maxpool2d_backward_kernel<T, 2><<<grid, kBlock, 0, s>>>(argmax, grad_y, planes, g, grad_x);
    else if (reach == 3) maxpool2d_backward_kernel<T, 3><<<grid, kBlock, 0, s>>>(argmax, grad_y, planes, g, grad_x);
    else maxpool2d_backward_kernel<T, 0><<<grid, kBlock, 0, s>>>(argmax, grad_y, planes, g, grad_x);
}

int launch_maxpool2d_forward(const void* x, int dtype, int64_t planes, const PoolShape& p, void* y,
                             uint8_t* argmax, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == ACTQ_F32) maxpool_forward_typed(static_cast<const float*>(x), planes, p, static_cast<float*>(y), argmax, s);
    else maxpool_forward_typed(static_cast<const _Float16*>(x), planes, p, static_cast<_Float16*>(y), argmax, s);
    return launched("actq_maxpool2d_forward");
}

int launch_maxpool2d_backward(const uint8_t* argmax, const void* grad_y, int dtype, int64_t planes,
                              const PoolShape& p, void* grad_x, void* stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == ACTQ_F32)
        maxpool_backward_typed(argmax, static_cast<const float*>(grad_y), planes, p, static_cast<float*>(grad_x), s);
    else
        maxpool_backward_typed(argmax, static_cast<const _Float16*>(grad_y), planes, p, static_cast<_Float16*>(grad_x), s);
    return launched("actq_maxpool2d_backward");
}

}  // namespace actq
