// Internal helpers shared by the kernels of libvgg_mi355x.so (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/vgg_mi355x.h"

namespace vgg {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short bf16_t;  // storage type of a bf16 value

constexpr int kWave = 64;  // CDNA wavefront width

__host__ __device__ constexpr inline int round_up16(int v) { return (v + 15) & ~15; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int dtype_size(int dtype) { return dtype == VGG_BF16 ? 2 : 4; }
inline bool dtype_ok(int dtype) { return dtype == VGG_F32 || dtype == VGG_BF16; }

// A kernel that uses more than 64 KB of dynamic LDS has to be told so once per process
// (hipFuncSetAttribute, not a stream operation).  Idempotent, so concurrent first calls are harmless;
// the flag only saves the repeated call.  Defined in api.hip.
bool raise_lds_limit(const void *kernel);

// Maps the HIP error state after enqueueing to a status code.
inline int launch_status() { return hipGetLastError() == hipSuccess ? VGG_OK : VGG_ERR_LAUNCH; }

// fp32 -> bf16, round to nearest even: the hardware conversion (v_cvt_pk_bf16_f32), one
// instruction instead of a dozen.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// The gradient step on one value, rounded once; every kernel that takes the step uses this form, so a
// step fused into a gradient kernel and a separate update leave identical parameters.
__device__ __forceinline__ float sgd_step(float theta, float grad, float lr) { return __builtin_fmaf(-lr, grad, theta); }
__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((unsigned int)h) << 16); }

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
    static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t *p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t *p, float v) { *p = f32_to_bf16(v); }
};

// Four values -> 16 bytes of fp32 or 8 bytes of bf16 (packed hardware conversion; the converted
// vector is only ever reinterpreted whole).
__device__ __forceinline__ void store4(float *dst, float v0, float v1, float v2, float v3)
{
    const f32x4 v = {v0, v1, v2, v3};
    *reinterpret_cast<f32x4 *>(dst) = v;
}
__device__ __forceinline__ void store4(bf16_t *dst, float v0, float v1, float v2, float v3)
{
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t lo = {v0, v1}, hi = {v2, v3};
    const u32x2_t w = {__builtin_bit_cast(unsigned int, __builtin_convertvector(lo, bf16x2_t)),
                       __builtin_bit_cast(unsigned int, __builtin_convertvector(hi, bf16x2_t))};
    *reinterpret_cast<u32x2_t *>(dst) = w;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

// Channel padding granularity: one 64-byte LDS row of the convolution kernels.
inline int padded_channels(int dtype, int C)
{
    const int g = dtype == VGG_BF16 ? 32 : 16;
    return (C + g - 1) / g * g;
}

// ---------------------------------------------------------------------------
// Packed convolution operand: nine taps of a [rows][colsP] matrix whose columns are the contraction
// index (input channels; colsP a multiple of the padding granularity).
//   fp32: element (t, row, col) at (t*rows + row)*colsP + col.
//   bf16: the columns are blocked by 16: element (t, row, col) at
//         ((t*(colsP/16) + col/16)*rows + row)*16 + col%16,
//         so that the 32 rows x 16 columns of one v_mfma_f32_32x32x16_bf16 operand are 1 KB of
//         contiguous memory and a wave can load its fragment straight from global memory.
// Both have 9*rows*colsP elements.
// ---------------------------------------------------------------------------
template <typename T>
__host__ __device__ __forceinline__ size_t packed_w_index(int t, int row, int col, int rows, int colsP)
{
    if (sizeof(T) == 2) return (((size_t)t * (colsP >> 4) + (col >> 4)) * rows + row) * 16 + (col & 15);
    return ((size_t)t * rows + row) * colsP + col;
}
// Byte offset of the 16-byte segment `seg` (0..3) of the 64 bytes of row `row` that start at column c0
// (a multiple of 16 fp32 / 32 bf16 columns): what one LDS row of the convolution kernels holds.
template <typename T>
__host__ __device__ __forceinline__ size_t packed_w_segment(int t, int row, int c0, int seg, int rows, int colsP)
{
    return packed_w_index<T>(t, row, c0 + seg * (16 / (int)sizeof(T)), rows, colsP) * sizeof(T);
}

// ---------------------------------------------------------------------------
// Tile geometry of the convolution kernels.
//
// A tile is a set of up to `rows` output pixels of the NHWC tensor together
// with its halo (every input pixel any of the nine taps touches).  The halo is
// staged in LDS as `S` rows; halo row i holds input pixel halo_pixel(i) or
// zeros when that returns -1.  Tile row j is output pixel m (or -1 when the
// tile sticks out of the tensor) and its tap (kh,kw) input lives in halo row
//     hrow + kh*pitch + kw.
//
// LINEAR mode: the tile is `rows` consecutive pixels m0.. of the flattened
// (n,h,w) index.  Halo rows follow the padded coordinate
//     q(n,h,w) = (n*(H+1) + h)*(W+1) + w,
// where every image row is followed by one pad pixel and every image by one
// pad row; a neighbour (h+dh, w+dw) is at q + dh*(W+1) + dw and lands on a pad
// position exactly when it is outside the image.  pitch = W+1.
//
// TILE2D mode: the tile is a TH x TW patch of one image (rows = TH*TW) with a
// (TH+2) x (TW+2) halo; pitch = TW+2.  Patches may stick out of the image at
// the right and bottom edges.
// ---------------------------------------------------------------------------
// Division of a non-negative 31-bit integer by a run-time constant d >= 1 as a multiply and a
// shift: with L = ceil(log2 d) and mul = ceil(2^(31+L) / d) (which fits 32 bits),
// floor(n / d) == (n * mul) >> (31 + L) for every 0 <= n < 2^31.
struct FastDiv {
    unsigned int mul;
    int shift;
};
inline FastDiv make_fast_div(int d)
{
    FastDiv f;
    int L = 0;
    while ((1ll << L) < d) ++L;
    f.shift = 31 + L;
    f.mul = (unsigned int)(((1ull << f.shift) + (unsigned long long)d - 1) / (unsigned long long)d);
    return f;
}
__host__ __device__ __forceinline__ int fast_div(int n, const FastDiv &f)
{
    return (int)(((unsigned long long)(unsigned int)n * f.mul) >> f.shift);
}

struct TileGeom {
    int N, H, W, M;      // M = N*H*W
    int mode;            // 0 LINEAR, 1 TILE2D
    int rows;            // tile rows (pixels)
    int TH, TW;          // TILE2D patch size (TW == kTileW)
    int tiles_w, tiles_hw;  // TILE2D: patches per image row / per image
    int ntiles;
    int pitch;
    int S;               // halo rows (upper bound over all tiles)
    FastDiv dW, dHW, dWp, dHp, dTilesW, dTilesHW;  // by W, H*W, W+1, H+1, tiles_w, tiles_hw
};

constexpr int kTileW = 16;  // width of a TILE2D patch (compile-time so that row/column splits are shifts)

struct TileOrigin {
    int n, h0, w0;  // TILE2D
    int m0, q0;     // LINEAR
};

__host__ __device__ __forceinline__ TileOrigin tile_origin(const TileGeom &g, int tile)
{
    TileOrigin o;
    if (g.mode) {
        o.n = fast_div(tile, g.dTilesHW);
        const int rem = tile - o.n * g.tiles_hw;
        const int ty = fast_div(rem, g.dTilesW);
        o.h0 = ty * g.TH;
        o.w0 = (rem - ty * g.tiles_w) * kTileW;
        o.m0 = 0; o.q0 = 0;
    } else {
        o.m0 = tile * g.rows;
        const int HW = g.H * g.W;
        const int n = fast_div(o.m0, g.dHW), rem = o.m0 - n * HW, h = fast_div(rem, g.dW), w = rem - h * g.W;
        o.q0 = (n * (g.H + 1) + h) * (g.W + 1) + w;
        o.n = 0; o.h0 = 0; o.w0 = 0;
    }
    return o;
}

__host__ __device__ __forceinline__ int halo_pixel(const TileGeom &g, const TileOrigin &o, int i)
{
    if (g.mode) {
        const int hy = i / (kTileW + 2), hx = i - hy * (kTileW + 2);
        const int h = o.h0 - 1 + hy, w = o.w0 - 1 + hx;
        if (h < 0 || h >= g.H || w < 0 || w >= g.W) return -1;
        return (o.n * g.H + h) * g.W + w;
    }
    const int q = o.q0 - (g.W + 2) + i;
    if (q < 0) return -1;
    const int Wp = g.W + 1, Hp = g.H + 1;
    const int rr = fast_div(q, g.dWp), w = q - rr * Wp, n = fast_div(rr, g.dHp), h = rr - n * Hp;
    if (w >= g.W || h >= g.H || n >= g.N) return -1;
    return (n * g.H + h) * g.W + w;
}

__host__ __device__ __forceinline__ void tile_row(const TileGeom &g, const TileOrigin &o, int j, int &m, int &hrow)
{
    if (g.mode) {
        const int dy = j / kTileW, dx = j - dy * kTileW;
        const int h = o.h0 + dy, w = o.w0 + dx;
        m = (h < g.H && w < g.W) ? (o.n * g.H + h) * g.W + w : -1;
        hrow = dy * (kTileW + 2) + dx;
        return;
    }
    m = o.m0 + j;
    if (m >= g.M) { m = -1; hrow = 0; return; }
    const int HW = g.H * g.W;
    const int n = fast_div(m, g.dHW), rem = m - n * HW, h = fast_div(rem, g.dW), w = rem - h * g.W;
    hrow = (n * (g.H + 1) + h) * (g.W + 1) + w - o.q0;
}

// Output pixel of tile row j only (no halo row: no divisions).
__host__ __device__ __forceinline__ int tile_pixel(const TileGeom &g, const TileOrigin &o, int j)
{
    if (g.mode) {
        const int h = o.h0 + j / kTileW, w = o.w0 + j % kTileW;
        return (h < g.H && w < g.W) ? (o.n * g.H + h) * g.W + w : -1;
    }
    const int m = o.m0 + j;
    return m < g.M ? m : -1;
}

// Host side: chooses the mode and fills the derived fields for tiles of
// `rows` pixels (rows = 256 -> 16x16 patches, 128 -> 8x16).
inline TileGeom make_tile_geom(int N, int H, int W, int rows)
{
    TileGeom g;
    g.N = N; g.H = H; g.W = W; g.M = N * H * W; g.rows = rows;
    g.TW = kTileW; g.TH = rows / kTileW;
    g.dW = make_fast_div(W); g.dHW = make_fast_div(H * W);
    g.dWp = make_fast_div(W + 1); g.dHp = make_fast_div(H + 1);
    g.dTilesW = g.dTilesHW = make_fast_div(1);
    if (H % g.TH == 0 && W % g.TW == 0) {
        g.mode = 1;
        g.tiles_w = W / g.TW;
        g.tiles_hw = g.tiles_w * (H / g.TH);
        g.dTilesW = make_fast_div(g.tiles_w); g.dTilesHW = make_fast_div(g.tiles_hw);
        g.ntiles = N * g.tiles_hw;
        g.pitch = g.TW + 2;
        g.S = (g.TH + 2) * (g.TW + 2);
        return g;
    }
    g.mode = 0;
    g.tiles_w = g.tiles_hw = 0;
    g.ntiles = (g.M + rows - 1) / rows;
    g.pitch = W + 1;
    const long HW = (long)H * W;
    long best = 0;
    for (long m0 = 0; m0 < g.M; m0 += rows) {
        long m1 = m0 + rows - 1;
        if (m1 >= g.M) m1 = g.M - 1;
        auto q = [&](long m) {
            const long n = m / HW, rem = m % HW, h = rem / W, w = rem % W;
            return (n * (H + 1) + h) * (W + 1) + w;
        };
        const long span = q(m1) - q(m0);
        if (span > best) best = span;
    }
    g.S = (int)(best + 2 * (W + 2) + 1);
    return g;
}

}  // namespace vgg
