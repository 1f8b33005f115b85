// Weight gradient of the 3x3 convolution on fp32 MFMA for gfx950, NHWC.
//
//   dw[t][co][ci] = sum_m g[m][co] * x[m + tap t][ci],   db[co] = sum_m g[m][co]
//
// (backward column of the appendix table: one more "convolution" per layer,
// plus a "reduce" for the bias).  GEMM view per tap: rows = co, columns = ci,
// contraction over the pixels m.  A workgroup owns a 64(co) x 32(ci) block of
// all nine taps and a range of pixel tiles (split-K).  Per tile it stages the
// g rows and the x halo (see TileGeom) in LDS; each of its four waves takes
// one 32-row half of co and one half of the tile's pixels and issues nine
// v_mfma_f32_32x32x2_f32 per pair of pixels, one per tap, all fed from the same
// g fragment.  The two pixel-halves are added through LDS at the end and the
// block writes its partial sums; a second kernel adds the partials of all
// splits in a fixed order, so the result does not depend on scheduling.
#include "common.h"

namespace vgg {

constexpr int kPK = 128;        // pixels per tile
constexpr int kBCO = 64, kBCI = 32;
constexpr int kGRow = kBCO * 4 + 16;  // bytes per LDS row of g (64 floats + pad)
constexpr int kXRow = kBCI * 4 + 16;  // bytes per LDS row of x (32 floats + pad)

struct WgradArgs {
    const float *x;   // [M][CinP]
    const float *g;   // [M][Cout]
    float *part;      // [splits][9][Cout][CinP]
    float *dbpart;    // [splits][Cout] or null
    int CinP, Cout;
    int tiles_co, tiles_ci, splits, tiles_per_split;
    TileGeom geo;
};

__global__ __launch_bounds__(256, 2) void conv3x3_wgrad_kernel(WgradArgs p)
{
    extern __shared__ __align__(16) char smem[];
    const int S = p.geo.S;
    int *pix = reinterpret_cast<int *>(smem);            // [S]
    int *rowm = pix + S;                                 // [kPK] output pixel of tile row or -1
    int *rowh = rowm + kPK;                              // [kPK] halo row of tap (0,0)
    char *Gs = smem + round_up16((S + 2 * kPK) * 4);     // [kPK][kGRow]
    char *Xs = Gs + kPK * kGRow;                         // [S][kXRow]

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = lane & 31, kp = lane >> 5;
    const int wc = wv & 1, wp = wv >> 1;  // co half, pixel half

    int b = blockIdx.x;
    const int tco = b % p.tiles_co; b /= p.tiles_co;
    const int tci = b % p.tiles_ci; b /= p.tiles_ci;
    const int split = b;
    const int co0 = tco * kBCO, ci0 = tci * kBCI;
    const int pitch = p.geo.pitch;

    f32x16 acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
    float gsum = 0.f;

    const int t_begin = split * p.tiles_per_split;
    const int t_end = min(t_begin + p.tiles_per_split, p.geo.ntiles);
    for (int tile = t_begin; tile < t_end; ++tile) {
        const TileOrigin org = tile_origin(p.geo, tile);
        __syncthreads();  // previous tile's reads done
        for (int i = tid; i < S; i += 256) pix[i] = halo_pixel(p.geo, org, i);
        for (int j = tid; j < kPK; j += 256) {
            int m, hrow;
            tile_row(p.geo, org, j, m, hrow);
            rowm[j] = m;
            rowh[j] = hrow;
        }
        __syncthreads();
        // g rows: 64 floats = 16 segments of 16 bytes
        for (int idx = tid; idx < kPK * 16; idx += 256) {
            const int j = idx >> 4, seg = idx & 15;
            const int m = rowm[j];
            uint4 v = make_uint4(0, 0, 0, 0);
            if (m >= 0 && co0 + seg * 4 < p.Cout)
                v = *reinterpret_cast<const uint4 *>(p.g + (size_t)m * p.Cout + co0 + seg * 4);
            *reinterpret_cast<uint4 *>(Gs + j * kGRow + seg * 16) = v;
        }
        // x halo rows: 32 floats = 8 segments
        for (int idx = tid; idx < S * 8; idx += 256) {
            const int i = idx >> 3, seg = idx & 7;
            const int off = pix[i];
            uint4 v = make_uint4(0, 0, 0, 0);
            if (off >= 0 && ci0 + seg * 4 < p.CinP)
                v = *reinterpret_cast<const uint4 *>(p.x + (size_t)off * p.CinP + ci0 + seg * 4);
            *reinterpret_cast<uint4 *>(Xs + i * kXRow + seg * 16) = v;
        }
        __syncthreads();
        // this wave: pixels [wp*64, wp*64+64) of the tile, two per MFMA step
#pragma unroll 2
        for (int s = 0; s < kPK / 4; ++s) {
            const int j = wp * (kPK / 2) + 2 * s + kp;
            const float a = *reinterpret_cast<const float *>(Gs + j * kGRow + (wc * 32 + r) * 4);
            const char *xb = Xs + rowh[j] * kXRow + r * 4;
            gsum += a;
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    const float bv = *reinterpret_cast<const float *>(xb + (kh * pitch + kw) * kXRow);
                    acc[kh * 3 + kw] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bv, acc[kh * 3 + kw], 0, 0, 0);
                }
        }
    }

    // add the two pixel halves: waves with wp == 1 park their sums in LDS
    __syncthreads();
    float *red = reinterpret_cast<float *>(smem);  // needs 2 * 9*16*64 floats = 73728 bytes
    if (wp == 1) {
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) red[((wc * 9 + t) * 16 + e) * 64 + lane] = acc[t][e];
    }
    __syncthreads();
    float gs_other = __shfl_xor(gsum, 32, kWave);  // the other pixel of the pair
    gsum += gs_other;
    float *dbs = reinterpret_cast<float *>(smem) + 2 * 9 * 16 * 64;  // [2][32]
    if (wp == 1 && kp == 0) dbs[wc * 32 + r] = gsum;
    if (wp == 0) {
        // accumulator layout: register e of lane l = row 8*(e/4) + 4*(l/32) + e%4 (co), column l%32 (ci)
        const int ci = ci0 + r;
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int co = co0 + wc * 32 + (e >> 2) * 8 + kp * 4 + (e & 3);
                const float v = acc[t][e] + red[((wc * 9 + t) * 16 + e) * 64 + lane];
                if (co < p.Cout && ci < p.CinP)
                    p.part[(((size_t)split * 9 + t) * p.Cout + co) * p.CinP + ci] = v;
            }
    }
    __syncthreads();
    if (p.dbpart && tci == 0 && wp == 0 && kp == 0) {
        const int co = co0 + wc * 32 + r;
        if (co < p.Cout) p.dbpart[(size_t)split * p.Cout + co] = gsum + dbs[wc * 32 + r];
    }
}

__global__ void wgrad_reduce_kernel(const float *part, float *out, size_t n, int splits)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float s = 0.f;
    for (int k = 0; k < splits; ++k) s += part[(size_t)k * n + i];
    out[i] = s;
}

static void wgrad_plan(int N, int H, int W, int CinP, int Cout, WgradArgs &a)
{
    a.geo = make_tile_geom(N, H, W, kPK);
    a.CinP = CinP; a.Cout = Cout;
    a.tiles_co = (Cout + kBCO - 1) / kBCO;
    a.tiles_ci = (CinP + kBCI - 1) / kBCI;
    const int groups = a.tiles_co * a.tiles_ci;
    int splits = (2048 + groups - 1) / groups;
    if (splits > a.geo.ntiles) splits = a.geo.ntiles;
    if (splits < 1) splits = 1;
    a.tiles_per_split = (a.geo.ntiles + splits - 1) / splits;
    a.splits = (a.geo.ntiles + a.tiles_per_split - 1) / a.tiles_per_split;
}

size_t conv3x3_wgrad_workspace(int N, int H, int W, int CinP, int Cout)
{
    WgradArgs a;
    wgrad_plan(N, H, W, CinP, Cout, a);
    return round_up((size_t)a.splits * 9 * Cout * CinP * 4, 256) + round_up((size_t)a.splits * Cout * 4, 256);
}

// x [M][CinP] fp32, g [M][Cout] fp32 -> dw [9][Cout][CinP], db [Cout] (may be null).
int conv3x3_wgrad(int N, int H, int W, int CinP, int Cout, const float *x, const float *g, float *dw,
                  float *db, void *ws, hipStream_t stream)
{
    WgradArgs a;
    wgrad_plan(N, H, W, CinP, Cout, a);
    a.x = x; a.g = g;
    const size_t nw = (size_t)9 * Cout * CinP;
    a.part = static_cast<float *>(ws);
    a.dbpart = db ? reinterpret_cast<float *>(static_cast<char *>(ws) + round_up((size_t)a.splits * nw * 4, 256))
                  : nullptr;
    size_t lds = round_up((size_t)(a.geo.S + 2 * kPK) * 4, 16) + (size_t)kPK * kGRow + (size_t)a.geo.S * kXRow;
    const size_t red = (size_t)2 * 9 * 16 * 64 * 4 + 64 * 4;
    if (lds < red) lds = red;
    if (lds > 160 * 1024) return VGG_ERR_UNSUPPORTED;
    static bool configured = false;
    if (lds > 64 * 1024 && !configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(conv3x3_wgrad_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return VGG_ERR_LAUNCH;
        configured = true;
    }
    hipLaunchKernelGGL(conv3x3_wgrad_kernel, dim3((unsigned)(a.tiles_co * a.tiles_ci * a.splits)), dim3(256), lds,
                       stream, a);
    if (hipGetLastError() != hipSuccess) return VGG_ERR_LAUNCH;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, stream, a.part, dw, nw,
                       a.splits);
    if (db)
        hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((Cout + 255) / 256)), dim3(256), 0, stream, a.dbpart,
                           db, (size_t)Cout, a.splits);
    return launch_status();
}

}  // namespace vgg
