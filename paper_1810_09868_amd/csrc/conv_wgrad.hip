// Weight gradient of the 3x3 convolution on fp32 MFMA for gfx950, NHWC.
//
//   dw[t][co][ci] = sum_m g[m][co] * x[m + tap t][ci],   db[co] = sum_m g[m][co]
//
// (backward column of the appendix table: one more "convolution" per layer,
// plus a "reduce" for the bias).  GEMM view per tap: rows = co, columns = ci,
// contraction over the pixels m.  A workgroup owns a 64(co) x 32(ci) block of
// all nine taps and a range of pixel tiles (split-K).  Each of its eight waves
// takes one 32-row half of co, one half of a tile's pixels and five or four of
// the taps, and issues one v_mfma_f32_32x32x2_f32 per tap and pair of pixels,
// all fed from the same g fragment.
//
// Staging: the g rows and the x halo (see TileGeom) of a tile are copied
// straight into LDS by global_load_lds_dwordx4 (lane l of a wave writes bytes
// [16 l, 16 l + 16) of a 1 KB block and supplies its own source address, so
// rows outside the tensor simply read a block of zeros).  Two buffers: the
// copies of tile k+1 are issued between, and in flight during, the MFMA steps of
// tile k, one barrier per tile, no staging registers, no index tables (every lane derives the
// pixels it needs from the tile geometry with a few multiplies).  Rows are
// unpadded; the two pixels of an MFMA step sit in adjacent rows, which for
// 128-byte x rows are already 32 banks apart, and for 256-byte g rows are made
// so by swapping the two halves of every odd row.
//
// The two pixel-halves are added through LDS at the end and the block writes
// its partial sums; a second kernel adds the partials of all splits in a fixed
// order, so the result does not depend on scheduling.
#include "common.h"

namespace vgg {

constexpr int kPK = 64;         // pixels per tile
constexpr int kWaves = 8;
constexpr int kBCO = 64, kBCI = 32;
constexpr int kGRow = kBCO * 4;  // bytes per LDS row of g
constexpr int kXRow = kBCI * 4;  // bytes per LDS row of x

typedef unsigned int wg_u32x4 __attribute__((ext_vector_type(4)));
__device__ const wg_u32x4 kZeroSeg[1] = {};  // what a row outside the tensor reads

struct WgradArgs {
    const float *x;   // [M][CinP]
    const float *g;   // [M][Cout]
    float *part;      // [splits][9][Cout][CinP]
    float *dbpart;    // [splits][Cout] or null
    int CinP, Cout;
    int tiles_co, tiles_ci, splits, tiles_per_split;
    int SX;           // halo rows per buffer (geo.S rounded up to 8)
    TileGeom geo;
};

// Taps [T0, T0 + NT) of one wave: the main loop over the workgroup's tiles and the final sums.
// S0: MFMA step before which the wave prepares the next tile's copies.
// Patch tiles of the weight-gradient kernel: 4 rows x TW columns of one image (TW = 16 or 14, so that the
// VGG widths 224, 112 and 56, 28 divide), halo 6 x (TW + 2).  Unlike the linear tiles (TW = 0, TileGeom
// mode 0) their halo rows are an affine function of the tile row, so every x address of the main loop is
// one per-lane base plus an immediate.  p.geo carries N, H, W, tiles_w, tiles_hw and their divisions.
template <int TW>
__device__ __forceinline__ TileOrigin wg_origin(const TileGeom &g, int tile)
{
    if (TW == 0) return tile_origin(g, tile);
    TileOrigin o;
    o.n = fast_div(tile, g.dTilesHW);
    const int rem = tile - o.n * g.tiles_hw;
    const int ty = fast_div(rem, g.dTilesW);
    o.h0 = ty * 4;
    o.w0 = (rem - ty * g.tiles_w) * TW;
    o.m0 = 0; o.q0 = 0;
    return o;
}
// output pixel of tile row j (-1: none) and, for linear tiles, its halo row
template <int TW>
__device__ __forceinline__ void wg_row(const TileGeom &g, const TileOrigin &o, int j, int &m, int &hrow)
{
    if (TW == 0) { tile_row(g, o, j, m, hrow); return; }
    constexpr int D = TW ? TW : 1;
    const int dy = j / D, dx = j - dy * D;
    const int h = o.h0 + dy, w = o.w0 + dx;
    m = (j < 4 * TW && h < g.H && w < g.W) ? (o.n * g.H + h) * g.W + w : -1;
    hrow = 0;
}
template <int TW>
__device__ __forceinline__ int wg_halo_pixel(const TileGeom &g, const TileOrigin &o, int i)
{
    if (TW == 0) return halo_pixel(g, o, i);
    const int hy = i / (TW + 2), hx = i - hy * (TW + 2);
    const int h = o.h0 - 1 + hy, w = o.w0 - 1 + hx;
    if (h < 0 || h >= g.H || w < 0 || w >= g.W) return -1;
    return (o.n * g.H + h) * g.W + w;
}

template <int T0, int NT, int S0, int TW>
__device__ __forceinline__ void wgrad_body(const WgradArgs &p, char *smem)
{
    constexpr bool PATCH = TW != 0;
    constexpr int PK = PATCH ? 4 * TW : kPK;           // pixels of a tile that are multiplied (g is staged as kPK rows)
    const int buf_bytes = kPK * kGRow + p.SX * kXRow;   // [kPK][256] g rows, then [SX][128] x rows

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = lane & 31, kp = lane >> 5;
    const int wc = wv & 1, wp = (wv >> 1) & 1;  // co half, pixel half (wv >> 2: tap group)

    int b = blockIdx.x;
    const int tco = b % p.tiles_co; b /= p.tiles_co;
    const int tci = b % p.tiles_ci; b /= p.tiles_ci;
    const int split = b;
    const int co0 = tco * kBCO, ci0 = tci * kBCI;
    const int pitch = p.geo.pitch;

    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
    float gsum = 0.f;

    const int t_begin = split * p.tiles_per_split;
    const int t_end = min(t_begin + p.tiles_per_split, p.geo.ntiles);

    // Index arithmetic is kept off the lanes' critical path: a wave-wide instruction costs several
    // cycles whatever it computes, so every pixel index is derived once per tile by one lane and
    // handed to the lanes that need it (ds_bpermute / v_readlane) instead of once per user.
    //
    // Direct-to-LDS copies of a wave: 1 KB block wv + 8k of the g rows (4 rows of 16 segments; odd
    // rows hold their two halves swapped), k < kGOps, and block wv + 8k of the x halo (8 rows of
    // 8 segments), k < nxw.
    constexpr int kGOps = kPK / 4 / kWaves;
    const int nxw = ((p.SX >> 3) - wv + kWaves - 1) / kWaves;   // x blocks of this wave (SX >= 8 * kWaves)
    const int gsub = lane >> 4;                                  // row of this lane within a g block
    const int gcol = co0 + (((lane & 15) ^ ((gsub & 1) << 3)) << 2);
    const bool gok = gcol < p.Cout;
    const int xsub = lane >> 3;                                  // row of this lane within an x block
    const int xcol = ci0 + ((lane & 7) << 2);
    const bool xok = xcol < p.CinP;
    const float *zero = reinterpret_cast<const float *>(kZeroSeg);
    auto dma = [&](const float *src, char *dst) __attribute__((always_inline)) {
        const unsigned d = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(__attribute__((address_space(3))) char *)dst);
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(d), "v"(src) : "m0", "memory");
    };
    constexpr int kXBatch = 3;                 // x blocks of a wave whose copies are spread over the steps
    constexpr int kOps = kGOps + kXBatch;      // copies that are spread over the MFMA steps
    static_assert(S0 + kOps <= PK / 4, "one copy per MFMA step");
    // lane l looks up halo row (l & 7) of this wave's x block k0 + (l >> 3) (blocks k0 .. k0 + 7)
    auto x_lookup = [&](const TileOrigin &org, int k0) __attribute__((always_inline)) {
        const int kk = k0 + (lane >> 3);
        const int i = (wv + kWaves * kk) * 8 + (lane & 7);
        return (kk < nxw && i < p.geo.S) ? wg_halo_pixel<TW>(p.geo, org, i) : -1;
    };
    // source addresses of g copy k / of x copy k of a lookup; m_l: output pixel of tile row `lane`
    auto g_src = [&](int m_l, int k) __attribute__((always_inline)) {
        const int m = __builtin_amdgcn_ds_bpermute(((wv + kWaves * k) * 4 + gsub) << 2, m_l);
        return (gok && m >= 0) ? p.g + (size_t)m * p.Cout + gcol : zero;
    };
    auto x_src = [&](int px_l, int k) __attribute__((always_inline)) {
        const int px = __builtin_amdgcn_ds_bpermute(((k << 3) + xsub) << 2, px_l);
        return (xok && px >= 0) ? p.x + (size_t)px * p.CinP + xcol : zero;
    };
    auto g_dst = [&](char *base, int k) __attribute__((always_inline)) { return base + (wv + kWaves * k) * 1024; };
    auto x_dst = [&](char *base, int k) __attribute__((always_inline)) {
        return base + kPK * kGRow + (wv + kWaves * k) * 1024;
    };
    // x blocks beyond the first batch (large halos): issued in one go
    auto issue_rest = [&](const TileOrigin &org, char *base) __attribute__((always_inline)) {
        for (int k0 = kXBatch; k0 < nxw; k0 += 8) {
            const int px_l = x_lookup(org, k0);
            const int kn = min(nxw - k0, 8);
            for (int k = 0; k < kn; ++k) dma(x_src(px_l, k), x_dst(base, k0 + k));
        }
    };

    const int wrow0 = __builtin_amdgcn_readfirstlane(wp * (PK / 2));
    const int nfirst = min(nxw, kXBatch);
    int hrow_l = 0;  // halo row (tap 0,0) of tile row `lane` of the tile being multiplied
    if (t_begin < t_end) {
        const TileOrigin org0 = wg_origin<TW>(p.geo, t_begin);
        int m_l;
        wg_row<TW>(p.geo, org0, lane, m_l, hrow_l);
#pragma unroll
        for (int k = 0; k < kGOps; ++k) dma(g_src(m_l, k), g_dst(smem, k));
        const int px_l = x_lookup(org0, 0);
        for (int k = 0; k < nfirst; ++k) dma(x_src(px_l, k), x_dst(smem, k));
        issue_rest(org0, smem);
    }
    for (int tile = t_begin; tile < t_end; ++tile) {
        const int buf = (tile - t_begin) & 1;
        // This tile's copies have landed (each wave waits for its own, the barrier publishes all),
        // and every wave is done with the other buffer, which the next copies overwrite.
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        __syncthreads();
        // The next tile's copies are issued one per MFMA step rather than in a burst, and their
        // addresses are prepared before step S0: all waves of all workgroups on a CU run in
        // lockstep, so if every wave did this at the same point the MFMA pipes would idle meanwhile.
        const bool more = tile + 1 < t_end;
        char *nbase = smem + (buf ^ 1) * buf_bytes;
        int hrow_next = 0;
        const float *srcs[kOps];
        TileOrigin orgn;
        const int ncopy = more ? kGOps + nfirst : 0;
        auto prepare = [&]() __attribute__((always_inline)) {
            // all cross-lane reads first, then one wait: each of them has LDS latency
            orgn = wg_origin<TW>(p.geo, more ? tile + 1 : tile);
            int m_l;
            wg_row<TW>(p.geo, orgn, lane, m_l, hrow_next);
            const int px_l = x_lookup(orgn, 0);
#pragma unroll
            for (int k = 0; k < kGOps; ++k) srcs[k] = g_src(m_l, k);
#pragma unroll
            for (int k = 0; k < kXBatch; ++k) srcs[kGOps + k] = x_src(px_l, k);
        };

        const char *Gs = smem + buf * buf_bytes;
        const char *Xs = Gs + kPK * kGRow;
        // this wave: pixels [wp*32, wp*32+32) of the tile, two per MFMA step
        const char *ga = Gs + (wrow0 + kp) * kGRow + (((wc * 32 + r) ^ (kp << 5)) << 2);
        // operands of step s+1 are read from LDS before the MFMAs of step s are issued
        float a_next, b_next[NT];
        // (PATCH) tile row j = wrow0 + 2s + kp sits in halo row (j / TW) * (TW + 2) + j % TW; TW is even and
        // wrow0 two whole patch rows, so the pixel pair of a step never straddles a patch row
        const char *xpatch = Xs + (wp * 2 * (TW + 2) + kp) * kXRow + r * 4;
        auto fetch = [&](int s) __attribute__((always_inline)) {
            a_next = *reinterpret_cast<const float *>(ga + s * 2 * kGRow);
            if (PATCH) {
                constexpr int D = PATCH ? TW : 2;
                const int ro = (((2 * s) / D) * (TW + 2) + (2 * s) % D) * kXRow;
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    b_next[t] = *reinterpret_cast<const float *>(xpatch + ro + (((T0 + t) / 3) * (TW + 2) + (T0 + t) % 3) * kXRow);
                return;
            }
            const int h0 = __builtin_amdgcn_readlane(hrow_l, wrow0 + 2 * s);
            const int h1 = __builtin_amdgcn_readlane(hrow_l, wrow0 + 2 * s + 1);
            const char *xb = Xs + (kp ? h1 : h0) * kXRow + r * 4;
#pragma unroll
            for (int t = 0; t < NT; ++t)
                b_next[t] = *reinterpret_cast<const float *>(xb + (((T0 + t) / 3) * pitch + (T0 + t) % 3) * kXRow);
        };
        fetch(0);
#pragma unroll
        for (int s = 0; s < PK / 4; ++s) {
            if (s == S0) prepare();
            if (s >= S0 && s - S0 < kOps && s - S0 < ncopy)
                dma(srcs[s - S0], s - S0 < kGOps ? g_dst(nbase, s - S0) : x_dst(nbase, s - S0 - kGOps));
            const float a = a_next;
            float bv[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) bv[t] = b_next[t];
            if (s + 1 < PK / 4) fetch(s + 1);
            gsum += a;
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bv[t], acc[t], 0, 0, 0);
        }
        if (more) issue_rest(orgn, nbase);
        hrow_l = hrow_next;
    }

    // add the two pixel halves: waves with wp == 1 park their sums in LDS
    __syncthreads();
    float *red = reinterpret_cast<float *>(smem);  // needs 2 * 9*16*64 floats = 73728 bytes
    if (wp == 1) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) red[((wc * 9 + T0 + t) * 16 + e) * 64 + lane] = acc[t][e];
    }
    __syncthreads();
    float gs_other = __shfl_xor(gsum, 32, kWave);  // the other pixel of the pair
    gsum += gs_other;
    float *dbs = reinterpret_cast<float *>(smem) + 2 * 9 * 16 * 64;  // [2][32]
    if (T0 == 0 && wp == 1 && kp == 0) dbs[wc * 32 + r] = gsum;
    if (wp == 0) {
        // accumulator layout: register e of lane l = row 8*(e/4) + 4*(l/32) + e%4 (co), column l%32 (ci)
        const int ci = ci0 + r;
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int co = co0 + wc * 32 + (e >> 2) * 8 + kp * 4 + (e & 3);
                const float v = acc[t][e] + red[((wc * 9 + T0 + t) * 16 + e) * 64 + lane];
                if (co < p.Cout && ci < p.CinP)
                    p.part[(((size_t)split * 9 + T0 + t) * p.Cout + co) * p.CinP + ci] = v;
            }
    }
    __syncthreads();
    if (T0 == 0 && p.dbpart && tci == 0 && wp == 0 && kp == 0) {
        const int co = co0 + wc * 32 + r;
        if (co < p.Cout) p.dbpart[(size_t)split * p.Cout + co] = gsum + dbs[wc * 32 + r];
    }
}

// Eight waves: (co half) x (pixel half) x (taps 0-4 | taps 5-8).  Splitting the taps halves the
// accumulator registers of a wave, so four waves fit on a SIMD; a wave of each tap group lands on
// every SIMD (wave w runs on SIMD w % 4), which balances the 5:4 split; the two groups also prepare
// the next tile at different points of a tile, so a SIMD always has waves that are multiplying.
template <int TW>
__global__ __launch_bounds__(kWaves * 64, 4) void conv3x3_wgrad_kernel(WgradArgs p)
{
    extern __shared__ __align__(16) char smem[];
    // (wave-uniform branch: both bodies execute the same sequence of barriers)
    if (__builtin_amdgcn_readfirstlane(threadIdx.x >> 8) == 0) wgrad_body<0, 5, 0, TW>(p, smem);
    else wgrad_body<5, 4, (TW ? 4 * TW : kPK) / 8, TW>(p, smem);
}

// Layers with at most three input channels (the first one): (tap, ci) pairs are the <= 27 columns
// of a single 32-wide MFMA tile, so a pair of pixels costs one MFMA per 32 output channels instead
// of nine.  Column c = tap*CI + ci of pixel m is x[m + tap][ci]: lane c reads it from the staged halo
// at a lane-constant offset.  Staging as in the general kernel.  Eight waves = (co half) x (pixel
// quarter); the quarters are added through LDS at the end.
__global__ __launch_bounds__(kWaves * 64, 4) void conv3x3_wgrad_thin_kernel(WgradArgs p, int CI)
{
    extern __shared__ __align__(16) char smem[];
    const int buf_bytes = kPK * kGRow + p.SX * kXRow;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = lane & 31, kp = lane >> 5;
    const int wc = wv & 1, wp = wv >> 1;  // co half, pixel quarter

    int b = blockIdx.x;
    const int tco = b % p.tiles_co; b /= p.tiles_co;
    const int split = b;
    const int co0 = tco * kBCO;
    const int pitch = p.geo.pitch;

    // this lane's column: tap and channel, as a byte offset from the halo row of tap (0,0)
    const bool cvalid = r < 9 * CI;
    const int tap = cvalid ? r / CI : 0, ci = cvalid ? r - tap * CI : 0;
    const int coff = ((tap / 3) * pitch + tap % 3) * kXRow + ci * 4;

    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    float gsum = 0.f;

    const int t_begin = split * p.tiles_per_split;
    const int t_end = min(t_begin + p.tiles_per_split, p.geo.ntiles);

    constexpr int kGOps = kPK / 4 / kWaves;
    const int nxw = ((p.SX >> 3) - wv + kWaves - 1) / kWaves;
    const int gsub = lane >> 4;
    const int gcol = co0 + (((lane & 15) ^ ((gsub & 1) << 3)) << 2);
    const bool gok = gcol < p.Cout;
    const int xsub = lane >> 3;
    const int xcol = (lane & 7) << 2;
    const bool xok = xcol < p.CinP;
    const float *zero = reinterpret_cast<const float *>(kZeroSeg);
    auto dma = [&](const float *src, char *dst) __attribute__((always_inline)) {
        const unsigned d = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(__attribute__((address_space(3))) char *)dst);
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(d), "v"(src) : "m0", "memory");
    };
    // all copies of a tile, in one go (there is little arithmetic to hide them behind)
    auto issue_tile = [&](const TileOrigin &org, char *base, int m_l) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < kGOps; ++k) {
            const int q = wv + kWaves * k;
            const int m = __builtin_amdgcn_ds_bpermute((q * 4 + gsub) << 2, m_l);
            dma((gok && m >= 0) ? p.g + (size_t)m * p.Cout + gcol : zero, base + q * 1024);
        }
        for (int k0 = 0; k0 < nxw; k0 += 8) {
            const int kk = k0 + (lane >> 3);
            const int i = (wv + kWaves * kk) * 8 + (lane & 7);
            const int px_l = (kk < nxw && i < p.geo.S) ? halo_pixel(p.geo, org, i) : -1;
            const int kn = min(nxw - k0, 8);
            for (int k = 0; k < kn; ++k) {
                const int px = __builtin_amdgcn_ds_bpermute(((k << 3) + xsub) << 2, px_l);
                dma((xok && px >= 0) ? p.x + (size_t)px * p.CinP + xcol : zero,
                    base + kPK * kGRow + (wv + kWaves * (k0 + k)) * 1024);
            }
        }
    };

    const int wrow0 = __builtin_amdgcn_readfirstlane(wp * (kPK / 4));
    int hrow_l = 0;
    if (t_begin < t_end) {
        const TileOrigin org0 = tile_origin(p.geo, t_begin);
        int m_l;
        tile_row(p.geo, org0, lane, m_l, hrow_l);
        issue_tile(org0, smem, m_l);
    }
    for (int tile = t_begin; tile < t_end; ++tile) {
        const int buf = (tile - t_begin) & 1;
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this tile's copies have landed
        __syncthreads();
        int hrow_next = 0;
        if (tile + 1 < t_end) {
            const TileOrigin orgn = tile_origin(p.geo, tile + 1);
            int m_l;
            tile_row(p.geo, orgn, lane, m_l, hrow_next);
            issue_tile(orgn, smem + (buf ^ 1) * buf_bytes, m_l);
        }
        const char *Gs = smem + buf * buf_bytes;
        const char *Xs = Gs + kPK * kGRow + coff;
        const char *ga = Gs + (wrow0 + kp) * kGRow + (((wc * 32 + r) ^ (kp << 5)) << 2);
        // this wave: pixels [wp*16, wp*16+16) of the tile, two per MFMA
#pragma unroll
        for (int s = 0; s < kPK / 8; ++s) {
            const int h0 = __builtin_amdgcn_readlane(hrow_l, wrow0 + 2 * s);
            const int h1 = __builtin_amdgcn_readlane(hrow_l, wrow0 + 2 * s + 1);
            const float a = *reinterpret_cast<const float *>(ga + s * 2 * kGRow);
            const float bv = *reinterpret_cast<const float *>(Xs + (kp ? h1 : h0) * kXRow);
            gsum += a;
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bv, acc, 0, 0, 0);
        }
        hrow_l = hrow_next;
    }

    // add the four pixel quarters: waves with wp > 0 park their sums in LDS
    __syncthreads();
    float *red = reinterpret_cast<float *>(smem);            // [2][3][16][64]
    float *dbs = red + 2 * 3 * 16 * 64;                      // [2][3][32]
    gsum += __shfl_xor(gsum, 32, kWave);                     // the other pixel of the pair
    if (wp > 0) {
#pragma unroll
        for (int e = 0; e < 16; ++e) red[((wc * 3 + wp - 1) * 16 + e) * 64 + lane] = acc[e];
        if (kp == 0) dbs[(wc * 3 + wp - 1) * 32 + r] = gsum;
    }
    __syncthreads();
    if (wp == 0) {
        // accumulator layout: register e of lane l = row 8*(e/4) + 4*(l/32) + e%4 (co), column l%32 (tap, ci)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int co = co0 + wc * 32 + (e >> 2) * 8 + kp * 4 + (e & 3);
            float v = acc[e];
#pragma unroll
            for (int q = 0; q < 3; ++q) v += red[((wc * 3 + q) * 16 + e) * 64 + lane];
            if (cvalid && co < p.Cout) p.part[(((size_t)split * 9 + tap) * p.Cout + co) * p.CinP + ci] = v;
        }
        if (p.dbpart && kp == 0) {
            const int co = co0 + wc * 32 + r;
            float v = gsum;
#pragma unroll
            for (int q = 0; q < 3; ++q) v += dbs[(wc * 3 + q) * 32 + r];
            if (co < p.Cout) p.dbpart[(size_t)split * p.Cout + co] = v;
        }
    }
    // padding channels of this block's partial sums: exact zeros
    for (int i = tid; i < 9 * kBCO * (p.CinP - CI); i += kWaves * 64) {
        const int cpad = p.CinP - CI;
        const int t = i / (kBCO * cpad), rem = i - t * (kBCO * cpad), col = rem / cpad, c = CI + rem - col * cpad;
        if (co0 + col < p.Cout) p.part[(((size_t)split * 9 + t) * p.Cout + co0 + col) * p.CinP + c] = 0.f;
    }
}

// out[i] = sum over the splits of part[k][i], in a fixed order.  A workgroup owns 256/RY outputs;
// thread row y adds the splits k = y, y + RY, ... and the RY rows are then added through LDS, so
// that launches with few outputs and many splits (bias gradients, thin layers) still fill the chip.
// Two sets of partials with the same number of splits (the weights' and the bias') share a launch:
// outputs [0, n) come from part, outputs [n, n + n2) from part2.
template <int RY>
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float *part, float *out, size_t n, const float *part2,
                                                           float *out2, size_t n2, int splits)
{
    constexpr int RX = 256 / RY;
    __shared__ float red[256];
    const int x = threadIdx.x % RX, y = threadIdx.x / RX;
    size_t i = (size_t)blockIdx.x * RX + x;
    const bool live = i < n + n2;
    if (i >= n) { i -= n; part = part2; out = out2; n = n2; }
    float s = 0.f;
    if (live)
        for (int k = y; k < splits; k += RY) s += part[(size_t)k * n + i];
    if (RY == 1) {
        if (live) out[i] = s;
        return;
    }
    red[threadIdx.x] = s;
    __syncthreads();
    if (y == 0 && live) {
        float t = 0.f;
#pragma unroll
        for (int r = 0; r < RY; ++r) t += red[r * RX + x];
        out[i] = t;
    }
}

static void launch_reduce(const float *part, float *out, size_t n, const float *part2, float *out2, size_t n2, int splits,
                          hipStream_t stream)
{
    const size_t total = n + n2;
    if (splits >= 128)
        hipLaunchKernelGGL(wgrad_reduce_kernel<16>, dim3((unsigned)((total + 15) / 16)), dim3(256), 0, stream, part, out, n, part2,
                           out2, n2, splits);
    else if (splits >= 16)
        hipLaunchKernelGGL(wgrad_reduce_kernel<4>, dim3((unsigned)((total + 63) / 64)), dim3(256), 0, stream, part, out, n, part2,
                           out2, n2, splits);
    else
        hipLaunchKernelGGL(wgrad_reduce_kernel<1>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, part, out, n, part2,
                           out2, n2, splits);
}

// (also used by the bf16 weight-gradient kernel; part2/out2 may be null with n2 = 0)
void wgrad_launch_reduce(const float *part, float *out, size_t n, const float *part2, float *out2, size_t n2, int splits,
                         hipStream_t stream)
{
    launch_reduce(part, out, n, part2, out2, n2, splits, stream);
}

// Patch width of the general kernel for an image size: 16 or 14 where the image width divides into
// patches (the last patch row of an image may stick out at the bottom: at most three rows of zeros),
// else 0 (linear tiles).
static int wgrad_patch_width(int H, int W) { return H < 4 ? 0 : (W % 16 == 0 ? 16 : (W % 14 == 0 ? 14 : 0)); }

static void wgrad_plan(int N, int H, int W, int CinP, int Cout, WgradArgs &a, bool thin = false)
{
    a.geo = make_tile_geom(N, H, W, kPK);
    const int TW = thin ? 0 : wgrad_patch_width(H, W);
    if (TW != 0) {
        a.geo.mode = 1; a.geo.TH = 4; a.geo.TW = TW;
        a.geo.tiles_w = W / TW;
        a.geo.tiles_hw = a.geo.tiles_w * ((H + 3) / 4);
        a.geo.dTilesW = make_fast_div(a.geo.tiles_w);
        a.geo.dTilesHW = make_fast_div(a.geo.tiles_hw);
        a.geo.ntiles = N * a.geo.tiles_hw;
        a.geo.pitch = TW + 2;
        a.geo.S = 6 * (TW + 2);
    }
    a.SX = (a.geo.S + 7) & ~7;
    if (a.SX < 8 * kWaves) a.SX = 8 * kWaves;  // every wave copies at least one halo block
    a.CinP = CinP; a.Cout = Cout;
    a.tiles_co = (Cout + kBCO - 1) / kBCO;
    a.tiles_ci = thin ? 1 : (CinP + kBCI - 1) / kBCI;
    const int groups = a.tiles_co * a.tiles_ci;
    // One resident round of workgroups (two per CU).  Every workgroup writes its whole block of partial
    // sums, which the reduction reads back -- 38 MB each way for 512 workgroups whatever the layer; four
    // rounds (for balance) quadrupled that and measured 2.7 % slower over the whole stack.
    int splits = (512 + groups - 1) / groups;
    if (splits > a.geo.ntiles) splits = a.geo.ntiles;
    if (splits < 1) splits = 1;
    a.tiles_per_split = (a.geo.ntiles + splits - 1) / splits;
    a.splits = (a.geo.ntiles + a.tiles_per_split - 1) / a.tiles_per_split;
}

// The thin kernel serves layers with at most three input channels; it tiles the pixels linearly, so its
// split count differs from the general kernel's.  Query and launch must agree on which one runs.
static bool wgrad_is_thin(int Cin, int CinP) { return Cin <= 3 && CinP <= kBCI; }

static size_t wgrad_ws_bytes(const WgradArgs &a)
{
    return round_up((size_t)a.splits * 9 * a.Cout * a.CinP * 4, 256) + round_up((size_t)a.splits * a.Cout * 4, 256);
}

size_t conv3x3_wgrad_workspace(int N, int H, int W, int Cin, int CinP, int Cout)
{
    WgradArgs a;
    wgrad_plan(N, H, W, CinP, Cout, a, wgrad_is_thin(Cin, CinP));
    return wgrad_ws_bytes(a);
}

// For inspection: {kernel (0 linear tiles, 14 / 16 patch width, 3 thin), pixel tiles, splits, tiles per split,
// workgroups}.
void conv3x3_wgrad_plan_info(int N, int H, int W, int Cin, int CinP, int Cout, int info[5])
{
    WgradArgs a;
    const bool thin = wgrad_is_thin(Cin, CinP);
    wgrad_plan(N, H, W, CinP, Cout, a, thin);
    info[0] = thin ? 3 : (a.geo.mode == 1 ? a.geo.TW : 0);
    info[1] = a.geo.ntiles;
    info[2] = a.splits;
    info[3] = a.tiles_per_split;
    info[4] = a.tiles_co * a.tiles_ci * a.splits;
}

// x [M][CinP] fp32 (channels >= Cin are zero), g [M][Cout] fp32 -> dw [9][Cout][CinP], db [Cout] (may be null).
// ws_bytes: size of ws; the launch is refused when the partial sums of its own plan would not fit.
int conv3x3_wgrad(int N, int H, int W, int Cin, int CinP, int Cout, const float *x, const float *g, float *dw,
                  float *db, void *ws, size_t ws_bytes, hipStream_t stream)
{
    const bool thin = wgrad_is_thin(Cin, CinP);
    WgradArgs a;
    wgrad_plan(N, H, W, CinP, Cout, a, thin);
    if (ws_bytes < wgrad_ws_bytes(a)) return VGG_ERR_WORKSPACE;
    a.x = x; a.g = g;
    const size_t nw = (size_t)9 * Cout * CinP;
    a.part = static_cast<float *>(ws);
    a.dbpart = db ? reinterpret_cast<float *>(static_cast<char *>(ws) + round_up((size_t)a.splits * nw * 4, 256))
                  : nullptr;
    size_t lds = (size_t)2 * (kPK * kGRow + a.SX * kXRow);
    const size_t red = (size_t)2 * 9 * 16 * 64 * 4 + 64 * 4;
    if (lds < red) lds = red;
    if (lds > 160 * 1024) return VGG_ERR_UNSUPPORTED;
    if (lds > 64 * 1024 &&
        !(raise_lds_limit(reinterpret_cast<const void *>(conv3x3_wgrad_kernel<0>)) &&
          raise_lds_limit(reinterpret_cast<const void *>(conv3x3_wgrad_kernel<16>)) &&
          raise_lds_limit(reinterpret_cast<const void *>(conv3x3_wgrad_kernel<14>)) &&
          raise_lds_limit(reinterpret_cast<const void *>(conv3x3_wgrad_thin_kernel))))
        return VGG_ERR_LAUNCH;
    const dim3 grid((unsigned)(a.tiles_co * a.tiles_ci * a.splits));
    if (thin)
        hipLaunchKernelGGL(conv3x3_wgrad_thin_kernel, grid, dim3(kWaves * 64), lds, stream, a, Cin);
    else if (a.geo.mode == 1 && a.geo.TW == 16)
        hipLaunchKernelGGL(conv3x3_wgrad_kernel<16>, grid, dim3(kWaves * 64), lds, stream, a);
    else if (a.geo.mode == 1)
        hipLaunchKernelGGL(conv3x3_wgrad_kernel<14>, grid, dim3(kWaves * 64), lds, stream, a);
    else
        hipLaunchKernelGGL(conv3x3_wgrad_kernel<0>, grid, dim3(kWaves * 64), lds, stream, a);
    if (hipGetLastError() != hipSuccess) return VGG_ERR_LAUNCH;
    launch_reduce(a.part, dw, nw, a.dbpart, db, db ? (size_t)Cout : 0, a.splits, stream);
    return launch_status();
}

}  // namespace vgg
