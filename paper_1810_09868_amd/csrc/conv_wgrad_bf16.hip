// Weight gradient of the 3x3 convolution with bf16 operands and fp32 sums (the matrix unit's
// bf16 x bf16 -> fp32 numerics of the paper's accelerator, applied to the backward pass), gfx950, NHWC.
//
//   dw[t][co][ci] = sum_m g[m][co] * x[m + tap t][ci],   db[co] = sum_m g[m][co]
//
// (backward column of the appendix table: one more "convolution" per layer, plus a "reduce" for
// the bias).  GEMM view per tap: rows = co, columns = ci, contraction over the pixels m.
//
// v_mfma_f32_16x16x32_bf16 wants, per lane, eight consecutive contraction indices of one row: eight
// pixels of one channel.  Memory and LDS hold the opposite (a pixel's channels are contiguous), so
// the fragments are fetched with the LDS transpose read ds_read_b64_tr_b16: within 16 lanes, lane i
// receives element i%4 of the four 8-byte chunks that lanes i/4, i/4+4, i/4+8, i/4+12 point at.
// Lane s of a group points at pixel s/4, channels 4(s%4).. of a 16-channel run: lane i then holds four
// consecutive pixels of channel i.  Two such reads make a lane's eight pixels; the four 16-lane groups
// of a wave take the four runs of eight pixels of two patch rows, so a fragment is 16 channels x the
// 32 pixels of two patch rows.  A tap only shifts the pixel rows that the lanes point at, so all nine
// taps are served from one staged halo.  (The 16x16x32 shape instead of 32x32x16: half the accumulator
// traffic per multiply-add, which under the power this workload's operands draw is worth a few per
// cent; same LDS reads, same registers.)
//
// A tile is a 4 x 16 patch of one image (patches may stick out at the right and bottom edge; what
// is outside reads as zero) and its 6 x 18 halo: MFMA step s of a tile contracts the 32 pixels of
// patch rows 2s and 2s + 1.  LDS rows are 160 bytes (64 channels + 32 bytes of padding); since the
// patch geometry is fixed, every fragment address is one per-lane base plus an immediate.
//
// A workgroup (4 waves) owns a 64(co) x 64(ci) block of all nine taps and a range of tiles.  Wave
// = (ci half) x (taps 0-4 | taps 5-8); it multiplies the four 16-row co fragments with the two 16-column
// x fragments of each of its five or four taps per step.  Staging: global_load_lds_dwordx4 straight
// into one of two LDS buffers, one barrier per tile.  The block writes partial sums; a second kernel
// adds the partials of all splits in a fixed order, so the result does not depend on scheduling.  The
// bias gradient comes from four extra MFMAs per step against a fragment of ones, in the blocks of the
// first ci tile.
//
// At most 32 input channels (the first layer): the second ci half would be padding.  The two waves of
// a tap group then both take the first half and one step each, and write their sums as two separate
// partials; with at most 16 input channels they also skip the second x fragment.
#include "common.h"

namespace vgg {

void wgrad_launch_reduce(const float *part, float *out, size_t n, const float *part2, float *out2, size_t n2, int splits,
                         hipStream_t stream);

namespace {

constexpr int kTH = 4, kTW = 16;                 // patch
constexpr int kP = kTH * kTW;                    // pixels per tile
constexpr int kHW = kTW + 2;                     // halo width
constexpr int kHaloRows = (kTH + 2) * kHW;       // 108
constexpr int kRow = 160;                        // LDS bytes per pixel row
constexpr int kGBytes = kP * kRow;               // 10240
constexpr int kXBytes = kHaloRows * kRow;        // 17280
constexpr int kNW = 4;                           // waves
constexpr int kOps = (kGBytes + kXBytes + kNW * 1024 - 1) / (kNW * 1024);  // copies per lane and tile: 7
constexpr int kBuf = kOps * kNW * 1024;          // 28672 bytes per buffer (tail never read)
constexpr int kCO = 64, kCI = 64;

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
__device__ const u32x4_t kZero16[1] = {};        // what a segment outside the tensors reads

struct WgradBf16Args {
    const bf16_t *x;  // [M][XC]: the first XC <= CinP channels; the others are taken as zero
    const bf16_t *g;  // [M][Cout]
    float *part;      // [splits][9][Cout][CinP]
    float *dbpart;    // [splits][Cout] or null
    int N, H, W, CinP, Cout, XC;
    int tiles_co, tiles_ci, splits, tiles_per_split, ntiles;
    int tiles_w, tiles_hw;
    int narrow;       // CinP <= 32: the waves of a tap group split the patch rows, not the channels
    FastDiv dTilesW, dTilesHW;
};

__device__ __forceinline__ bf16x8 tr_fragment(const char *lds_lo, const char *lds_hi)
{
    typedef __attribute__((address_space(3))) s16x4 *lp;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)lds_lo);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)lds_hi);
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

typedef float f32x4v __attribute__((ext_vector_type(4)));

// Taps [T0, T0 + NT) of one wave.  DB: this wave also sums g over the pixels.  NARROW: see above; NCI: x
// fragments (16 input channels each) per tap.
template <int T0, int NT, bool DB, bool NARROW, int NCI>
__device__ __forceinline__ void wgrad_bf16_body(const WgradBf16Args &p, char *smem, int tco, int tci, int split)
{
    constexpr int NS = NARROW ? 1 : kTH / 2;                 // MFMA steps (pairs of patch rows) of this wave per tile
    constexpr int NCO = kCO / 16;                            // co fragments
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wi = wv & 1;                                   // ci half of this wave (NARROW: its step)
    const int co0 = tco * kCO, ci0 = tci * kCI;

    f32x4v acc[NCO][NCI][NT];
#pragma unroll
    for (int c = 0; c < NCO; ++c)
#pragma unroll
        for (int d = 0; d < NCI; ++d)
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[c][d][t] = f32x4v{0.f, 0.f, 0.f, 0.f};
    f32x4v accb[NCO];
#pragma unroll
    for (int c = 0; c < NCO; ++c) accb[c] = f32x4v{0.f, 0.f, 0.f, 0.f};

    // Copies: lane covers bytes [16 L, 16 L + 16) of a buffer, L = 256 k + tid, k < kOps.  Which
    // tensor, pixel (relative to the patch origin) and channel segment that is never changes.
    int cp_dy[kOps], cp_dx[kOps], cp_col[kOps];  // col < 0: zeros
    bool cp_g[kOps];
#pragma unroll
    for (int k = 0; k < kOps; ++k) {
        const int off = (k * kNW * 64 + tid) * 16;
        const bool isg = off < kGBytes;
        const int o = isg ? off : off - kGBytes;
        const int row = o / kRow, seg = (o - row * kRow) >> 4;
        cp_g[k] = isg;
        if (isg) { cp_dy[k] = row / kTW; cp_dx[k] = row % kTW; }
        else { cp_dy[k] = row / kHW - 1; cp_dx[k] = row % kHW - 1; }
        const int col = (isg ? co0 : ci0) + seg * 8;
        const bool ok = seg < 8 && (isg || row < kHaloRows) && col < (isg ? p.Cout : p.XC);
        cp_col[k] = ok ? col : -1;
    }
    auto issue = [&](int tile, char *base) __attribute__((always_inline)) {
        const int n = fast_div(tile, p.dTilesHW);
        const int rem = tile - n * p.tiles_hw;
        const int ty = fast_div(rem, p.dTilesW);
        const int h0 = ty * kTH, w0 = (rem - ty * p.tiles_w) * kTW;
#pragma unroll
        for (int k = 0; k < kOps; ++k) {
            const int h = h0 + cp_dy[k], w = w0 + cp_dx[k];
            const bool ok = cp_col[k] >= 0 && (unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W;
            const size_t pix = (size_t)((n * p.H + h) * p.W + w);
            const bf16_t *src = cp_g[k] ? p.g + pix * p.Cout + cp_col[k] : p.x + pix * p.XC + cp_col[k];
            if (!ok) src = reinterpret_cast<const bf16_t *>(kZero16);
            const unsigned d = __builtin_amdgcn_readfirstlane(
                (unsigned)(uintptr_t)(__attribute__((address_space(3))) char *)(base + (k * kNW + wv) * 1024));
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(d), "v"(src) : "m0", "memory");
        }
    };

    // Fragment addresses.  Lane 16 G + i points at pixel dx = 8 (G & 1) + (i >> 2) (+4 for the second read) of
    // patch row G >> 1 of the step's two, and at the 8-byte chunk i & 3 of a 32-byte run of 16 channels.
    const int G = lane >> 4, i = lane & 15;
    const int g_off = ((G >> 1) * kTW + 8 * (G & 1) + (i >> 2)) * kRow + (i & 3) * 8 +
                      (NARROW ? wi * 2 * kTW * kRow : 0);           // + co fragment * 32 + 32 s * kRow (+ 4 * kRow)
    const int x_off = kGBytes + ((G >> 1) * kHW + 8 * (G & 1) + (i >> 2)) * kRow + (i & 3) * 8 +
                      (NARROW ? wi * 2 * kHW * kRow : wi * 64);     // + x fragment * 32 + ((2 s + kh) * 18 + kw) * kRow (+ 4 * kRow)

    const int t_begin = split * p.tiles_per_split;
    const int t_end = min(t_begin + p.tiles_per_split, p.ntiles);
    if (t_begin < t_end) issue(t_begin, smem);

    const s16x8 ones_v = {0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x3F80};
    const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_v);

    for (int tile = t_begin; tile < t_end; ++tile) {
        const int buf = (tile - t_begin) & 1;
        // This tile's copies have landed (each wave waits for its own, the barrier publishes all),
        // and every wave is done with the other buffer, which the next copies overwrite.
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        __syncthreads();
        if (tile + 1 < t_end) issue(tile + 1, smem + (buf ^ 1) * kBuf);
        const char *B = smem + buf * kBuf;
        // Fragments are requested one MFMA group ahead of their use (the LDS latency of a transpose read
        // is longer than the MFMAs a fragment feeds, and only two waves share a SIMD).
        auto g_frag = [&](int s, int c) __attribute__((always_inline)) {
            const char *a = B + g_off + c * 32 + (2 * kTW * s) * kRow;
            return tr_fragment(a, a + 4 * kRow);
        };
        auto x_frag = [&](int s, int t, int d) __attribute__((always_inline)) {
            const int kh = (T0 + t) / 3, kw = (T0 + t) % 3;
            const char *a = B + x_off + d * 32 + ((2 * s + kh) * kHW + kw) * kRow;
            return tr_fragment(a, a + 4 * kRow);
        };
        bf16x8 gf[NCO], gf_next[NCO], xf[NCI], xf_next[NCI];
#pragma unroll
        for (int c = 0; c < NCO; ++c) gf_next[c] = g_frag(0, c);
#pragma unroll
        for (int d = 0; d < NCI; ++d) xf_next[d] = x_frag(0, 0, d);
#pragma unroll
        for (int s = 0; s < NS; ++s) {
#pragma unroll
            for (int c = 0; c < NCO; ++c) gf[c] = gf_next[c];
            if (DB) {
#pragma unroll
                for (int c = 0; c < NCO; ++c) accb[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gf[c], ones, accb[c], 0, 0, 0);
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
#pragma unroll
                for (int d = 0; d < NCI; ++d) xf[d] = xf_next[d];
                if (t + 1 < NT) {
#pragma unroll
                    for (int d = 0; d < NCI; ++d) xf_next[d] = x_frag(s, t + 1, d);
                } else if (s + 1 < NS) {
#pragma unroll
                    for (int c = 0; c < NCO; ++c) gf_next[c] = g_frag(s + 1, c);
#pragma unroll
                    for (int d = 0; d < NCI; ++d) xf_next[d] = x_frag(s + 1, 0, d);
                }
                __builtin_amdgcn_sched_barrier(0);   // keep the requests ahead of the MFMAs they overlap with
#pragma unroll
                for (int d = 0; d < NCI; ++d)
#pragma unroll
                    for (int c = 0; c < NCO; ++c)
                        acc[c][d][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gf[c], xf[d], acc[c][d][t], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // accumulator layout: register e of lane l = row 4*(l/16) + e (co), column l%16 (ci)
    const int ci = ci0 + (NARROW ? 0 : wi * 32) + i;
    if (NARROW) split = 2 * split + wi;                      // this wave's own partial
#pragma unroll
    for (int c = 0; c < NCO; ++c)
#pragma unroll
        for (int d = 0; d < NCI; ++d)
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int co = co0 + c * 16 + G * 4 + e;
                    if (co < p.Cout && ci + d * 16 < p.CinP)
                        p.part[(((size_t)split * 9 + T0 + t) * p.Cout + co) * p.CinP + ci + d * 16] = acc[c][d][t][e];
                }
    if (NCI == 1 && NARROW && i + 16 < p.CinP) {             // (columns this variant does not compute: zero)
#pragma unroll
        for (int c = 0; c < NCO; ++c)
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int co = co0 + c * 16 + G * 4 + e;
                    if (co < p.Cout) p.part[(((size_t)split * 9 + T0 + t) * p.Cout + co) * p.CinP + ci + 16] = 0.f;
                }
    }
    if (DB && i == 0) {
#pragma unroll
        for (int c = 0; c < NCO; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int co = co0 + c * 16 + G * 4 + e;
                if (co < p.Cout) p.dbpart[(size_t)split * p.Cout + co] = accb[c][e];
            }
    }
}

__global__ __launch_bounds__(kNW * 64, 2) void conv3x3_wgrad_bf16_kernel(WgradBf16Args p)
{
    extern __shared__ __align__(16) char smem[];
    // Workgroup b runs on XCD b % 8 and every XCD has its own L2: renumber so that an XCD works
    // through whole splits, whose blocks all read the same tiles.
    const int nblk = gridDim.x, xcd = blockIdx.x & 7;
    int b = xcd * (nblk >> 3) + min(xcd, nblk & 7) + (blockIdx.x >> 3);
    const int tco = b % p.tiles_co; b /= p.tiles_co;
    const int tci = b % p.tiles_ci; b /= p.tiles_ci;
    const int split = b;
    // (wave-uniform branches: all bodies execute the same sequence of barriers)
    const int group = __builtin_amdgcn_readfirstlane(threadIdx.x >> 7);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (p.narrow) {
        if (p.XC <= 16) {   // (x holds at most 16 channels: one x fragment per tap)
            if (group == 0) wgrad_bf16_body<0, 5, false, true, 1>(p, smem, tco, tci, split);
            else if (p.dbpart) wgrad_bf16_body<5, 4, true, true, 1>(p, smem, tco, tci, split);   // each wave sums g over its own rows
            else wgrad_bf16_body<5, 4, false, true, 1>(p, smem, tco, tci, split);
            return;
        }
        if (group == 0) wgrad_bf16_body<0, 5, false, true, 2>(p, smem, tco, tci, split);
        else if (p.dbpart) wgrad_bf16_body<5, 4, true, true, 2>(p, smem, tco, tci, split);
        else wgrad_bf16_body<5, 4, false, true, 2>(p, smem, tco, tci, split);
        return;
    }
    if (group == 0) wgrad_bf16_body<0, 5, false, false, 2>(p, smem, tco, tci, split);
    else if (p.dbpart && tci == 0 && wave == 2) wgrad_bf16_body<5, 4, true, false, 2>(p, smem, tco, tci, split);
    else wgrad_bf16_body<5, 4, false, false, 2>(p, smem, tco, tci, split);
}

// ---------------------------------------------------------------------------
// At most three input channels (the first layer; backward column of the appendix table, first "convolution"):
// the contraction over the pixels has only 27 (tap, channel) columns, and the layer is bound by reading g
// once.  No LDS staging and no transpose reads: both MFMA operands are gathered straight from global memory,
// 16-bit element by element, in the layout v_mfma_f32_32x32x16_bf16 wants -- lane (r, half) fetches eight
// consecutive pixels of row r = (tap, channel) of the shifted input (zeros outside the image; row 27 is all
// ones, which makes the bias sum; rows 28..31 are zero) and of output channels r and 32 + r of g -- one unit (16
// pixels of an image row; W must be a multiple of 16) ahead of the two MFMAs that use them.  (A version
// without the matrix unit -- the input pixels moved to scalar registers and fed to v_dot2c_f32_bf16 -- took
// 0.32 ms where this one takes 0.23; fetching those pixels with scalar loads 0.47: the scalar data cache is
// no place to stream an image through.)  The four waves of a workgroup add their sums through LDS and write one
// partial per workgroup, [28][64 channels]; the partials are added by wgrad_launch_reduce and spread into the
// [9][Cout][CinP] layout (zeros in the padding columns) by a small kernel.
// ---------------------------------------------------------------------------
constexpr int kThinK = 28;   // 27 (tap, channel) sums + the bias sum
constexpr int kThinPx = 16;  // pixels per unit

struct WgradThinArgs {
    const bf16_t *x;   // [M][XC], channels 0..2 of a pixel in its first 8 bytes
    const bf16_t *g;   // [M][Cout]
    float *part;       // [gridDim.x][gridDim.y][28][64]
    int H, W, XC, Cout, units, units_per_row;
    FastDiv dUnitsPerRow, dH;
};

typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void conv3x3_wgrad_bf16_thin_kernel(WgradThinArgs p)
{
    __shared__ float red[4][32][64];
    const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, kh8 = (lane >> 5) * 8;
    // MFMA rows: r < 27 is (tap r / 3, channel r % 3), r == 27 a row of ones (the bias sum), the rest zero.
    const int tap = r / 3, ci = r - tap * 3;
    const int dy = tap / 3 - 1, dx = tap - (tap / 3) * 3 - 1;
    const int co_a = min((int)blockIdx.y * 64 + r, p.Cout - 1), co_b = min((int)blockIdx.y * 64 + 32 + r, p.Cout - 1);
    f32x16 acc[2];
#pragma unroll
    for (int e = 0; e < 16; ++e) { acc[0][e] = 0.f; acc[1][e] = 0.f; }
    // A unit's operands as loaded (16-bit values, one per register until the unit's turn comes): the lane's
    // eight pixels (8 kh8.. of the unit's 16) of its (tap, channel) of x, and of its two output channels of g.
    auto load_unit = [&](int u, unsigned(&xr)[8], unsigned(&ga)[8], unsigned(&gb)[8]) __attribute__((always_inline)) {
        const int row = fast_div(u, p.dUnitsPerRow);           // = n * H + h
        const int w0 = (u - row * p.units_per_row) * kThinPx + kh8;
        const int n = fast_div(row, p.dH), h = row - n * p.H;
        const unsigned short *gr = reinterpret_cast<const unsigned short *>(p.g) + ((size_t)row * p.W + w0) * p.Cout;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            ga[e] = gr[(size_t)e * p.Cout + co_a];
            gb[e] = gr[(size_t)e * p.Cout + co_b];
        }
        const int hh = h + dy;
        const bool rowok = r < 27 && (unsigned)hh < (unsigned)p.H;
        const unsigned short *xrow = reinterpret_cast<const unsigned short *>(p.x) + ((size_t)(n * p.H + (rowok ? hh : h)) * p.W) * p.XC + ci;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int ww = w0 + e + dx;
            const bool in = rowok && (unsigned)ww < (unsigned)p.W;
            const unsigned v = xrow[(size_t)(in ? ww : w0) * p.XC];   // (clamped address, loaded unconditionally)
            xr[e] = in ? v : (r == 27 ? 0x3F80u : 0u);
        }
    };
    auto frag = [](const unsigned(&v)[8]) __attribute__((always_inline)) {
        const u32x4_t w = {v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16)};
        return __builtin_bit_cast(bf16x8, w);
    };
    const int first = blockIdx.x * 4 + wv, stride = gridDim.x * 4;
    unsigned xr[8], ga[8], gb[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { xr[e] = 0u; ga[e] = 0u; gb[e] = 0u; }
    if (first < p.units) load_unit(first, xr, ga, gb);
    for (int u = first; u < p.units; u += stride) {
        const bf16x8 xf = frag(xr), gfa = frag(ga), gfb = frag(gb);
        if (u + stride < p.units) load_unit(u + stride, xr, ga, gb);   // (one unit ahead)
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, gfa, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, gfb, acc[1], 0, 0, 0);
    }
    // accumulator layout: register e of lane l = row 8*(e/4) + 4*(l/32) + e%4 (tap, channel), column l%32 (output channel)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) red[wv][(e >> 2) * 8 + (lane >> 5) * 4 + (e & 3)][j * 32 + r] = acc[j][e];
    __syncthreads();
    float *out = p.part + ((size_t)blockIdx.x * gridDim.y + blockIdx.y) * kThinK * 64;
    for (int e = threadIdx.x; e < kThinK * 64; e += 256) {
        const int k = e >> 6, l = e & 63;
        out[e] = (red[0][k][l] + red[1][k][l]) + (red[2][k][l] + red[3][k][l]);
    }
}

// sums [co tiles][28][64] -> dw [9][Cout][CinP] (columns >= 3: zero), db [Cout]
__global__ __launch_bounds__(256) void wgrad_bf16_thin_spread_kernel(const float *sums, float *dw, float *db, int Cout, int CinP)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int n = 9 * Cout * CinP;
    if (i < n) {
        const int ci = i % CinP, co = (i / CinP) % Cout, t = i / (CinP * Cout);
        dw[i] = ci < 3 ? sums[((size_t)(co >> 6) * kThinK + t * 3 + ci) * 64 + (co & 63)] : 0.f;
    } else if (i < n + Cout && db) {
        const int co = i - n;
        db[co] = sums[((size_t)(co >> 6) * kThinK + 27) * 64 + (co & 63)];
    }
}

// workgroups along x of the thin kernel's launch: about four per CU in all, at most one per four units
inline int wgrad_thin_blocks(int units, int co_tiles)
{
    int b = (1024 + co_tiles - 1) / co_tiles;
    if (b > (units + 3) / 4) b = (units + 3) / 4;
    return b < 1 ? 1 : b;
}

void wgrad_bf16_plan(int N, int H, int W, int CinP, int Cout, WgradBf16Args &a)
{
    a.N = N; a.H = H; a.W = W; a.CinP = CinP; a.Cout = Cout;
    a.tiles_w = (W + kTW - 1) / kTW;
    a.tiles_hw = a.tiles_w * ((H + kTH - 1) / kTH);
    a.ntiles = N * a.tiles_hw;
    a.dTilesW = make_fast_div(a.tiles_w);
    a.dTilesHW = make_fast_div(a.tiles_hw);
    a.tiles_co = (Cout + kCO - 1) / kCO;
    a.tiles_ci = (CinP + kCI - 1) / kCI;
    const int groups = a.tiles_co * a.tiles_ci;
    // One round of two resident workgroups per CU.  Every workgroup writes 9 x 64 x 64 partial sums that the
    // reduction reads back, 75 MB each way for 512 workgroups whatever the layer: a second round of
    // workgroups (for balance) doubled that and measured 11 % slower over the whole stack.
    int splits = (512 + groups - 1) / groups;
    if (splits > a.ntiles) splits = a.ntiles;
    if (splits < 1) splits = 1;
    a.tiles_per_split = (a.ntiles + splits - 1) / splits;
    a.splits = (a.ntiles + a.tiles_per_split - 1) / a.tiles_per_split;
    a.narrow = CinP <= kCI / 2;
}
// partial results the reduction adds up
inline int wgrad_bf16_partials(const WgradBf16Args &a) { return a.narrow ? 2 * a.splits : a.splits; }

}  // namespace

static size_t wgrad_bf16_ws_bytes(const WgradBf16Args &a)
{
    const size_t np = (size_t)wgrad_bf16_partials(a);
    return round_up(np * 9 * a.Cout * a.CinP * 4, 256) + round_up(np * a.Cout * 4, 256);
}

size_t conv3x3_wgrad_bf16_workspace(int N, int H, int W, int CinP, int Cout)
{
    WgradBf16Args a;
    wgrad_bf16_plan(N, H, W, CinP, Cout, a);
    return wgrad_bf16_ws_bytes(a);
}

// For inspection: {kernel (16: 4 x 16 patches; 17: the same with both waves of a tap group on one channel
// half; 18: the thin kernel, when the caller passes cin -- the other entries then still describe 17's plan,
// which is what the workspace is sized for), pixel tiles, partial results, tiles per split, workgroups}.
void conv3x3_wgrad_bf16_plan_info(int N, int H, int W, int CinP, int Cout, int info[5], int cin)
{
    WgradBf16Args a;
    wgrad_bf16_plan(N, H, W, CinP, Cout, a);
    info[0] = a.narrow ? 17 : 16;
    if (cin >= 1 && cin <= 3 && W % kThinPx == 0) {
        const int co_tiles = (Cout + 63) / 64;
        const int nb = wgrad_thin_blocks(N * H * (W / kThinPx), co_tiles);
        if (wgrad_bf16_ws_bytes(a) >= ((size_t)nb + 1) * co_tiles * kThinK * 64 * sizeof(float)) info[0] = 18;
    }
    info[1] = a.ntiles;
    info[2] = wgrad_bf16_partials(a);
    info[3] = a.tiles_per_split;
    info[4] = a.tiles_co * a.tiles_ci * a.splits;
}

// x [M][CinP] bf16 (channels >= Cin are zero), g [M][Cout] bf16 -> dw [9][Cout][CinP] fp32, db [Cout] fp32 (may be null).
// Cout and CinP must be multiples of 8 (16-byte channel segments).  x_channels (optional): x holds only that many
// channels per pixel (a multiple of 8, at most CinP), the rest count as zero -- the first layer's three channels
// need one 16-byte segment per pixel, not a whole 64-byte row.  cin (optional): the number of real input channels
// when the caller knows it; one to three of them on an image whose width is a multiple of 16 take the thin kernel.
int conv3x3_wgrad_bf16(int N, int H, int W, int CinP, int Cout, const bf16_t *x, const bf16_t *g, float *dw, float *db,
                       void *ws, size_t ws_bytes, hipStream_t stream, int x_channels, int cin)
{
    if (Cout % 8 || CinP % 8) return VGG_ERR_UNSUPPORTED;
    if (x_channels == 0) x_channels = CinP;
    if (x_channels % 8 || x_channels > CinP) return VGG_ERR_UNSUPPORTED;
    if ((long long)N * H * W >= (1ll << 31) / 2) return VGG_ERR_UNSUPPORTED;
    if (cin >= 1 && cin <= 3 && W % kThinPx == 0) {
        // (falls through to the general kernel when the caller's workspace, sized without knowing cin, is too small)
        WgradThinArgs t;
        t.x = x; t.g = g; t.H = H; t.W = W; t.XC = x_channels; t.Cout = Cout;
        t.units_per_row = W / kThinPx;
        t.units = N * H * t.units_per_row;
        t.dUnitsPerRow = make_fast_div(t.units_per_row);
        t.dH = make_fast_div(H);
        const int co_tiles = (Cout + 63) / 64;
        const int nb = wgrad_thin_blocks(t.units, co_tiles);
        const size_t one = (size_t)co_tiles * kThinK * 64;
        if (ws_bytes >= ((size_t)nb + 1) * one * sizeof(float)) {
            t.part = static_cast<float *>(ws);
            float *sums = t.part + (size_t)nb * one;
            hipLaunchKernelGGL(conv3x3_wgrad_bf16_thin_kernel, dim3((unsigned)nb, (unsigned)co_tiles), dim3(256), 0, stream, t);
            if (hipGetLastError() != hipSuccess) return VGG_ERR_LAUNCH;
            wgrad_launch_reduce(t.part, sums, one, nullptr, nullptr, 0, nb, stream);
            const int total = 9 * Cout * CinP + Cout;
            hipLaunchKernelGGL(wgrad_bf16_thin_spread_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, sums, dw, db,
                               Cout, CinP);
            return launch_status();
        }
    }
    WgradBf16Args a;
    wgrad_bf16_plan(N, H, W, CinP, Cout, a);
    if (ws_bytes < wgrad_bf16_ws_bytes(a)) return VGG_ERR_WORKSPACE;
    a.x = x; a.g = g; a.XC = x_channels;
    const size_t nw = (size_t)9 * Cout * CinP;
    a.part = static_cast<float *>(ws);
    const int np = wgrad_bf16_partials(a);
    a.dbpart = db ? reinterpret_cast<float *>(static_cast<char *>(ws) + round_up((size_t)np * nw * 4, 256)) : nullptr;
    const dim3 grid((unsigned)(a.tiles_co * a.tiles_ci * a.splits));
    hipLaunchKernelGGL(conv3x3_wgrad_bf16_kernel, grid, dim3(kNW * 64), 2 * kBuf, stream, a);
    if (hipGetLastError() != hipSuccess) return VGG_ERR_LAUNCH;
    wgrad_launch_reduce(a.part, dw, nw, a.dbpart, db, db ? (size_t)Cout : 0, np, stream);
    return launch_status();
}

}  // namespace vgg
