// First convolution of the network (3 -> 64 channels) read straight from the
// canonical NCHW fp32 image batch and written as NHWC in the compute dtype.
//
// With only 27 contraction indices the layer is bound by writing its output
// (appendix table row "convolution", first of 16); padding the image to a
// full channel row and running the general kernel would read and write an
// extra padded copy of the batch.  Here a workgroup stages the 3 x 18 x 18
// fp32 halo of a 16 x 16 pixel patch in LDS (the next patch's halo is already
// in registers while the current one is multiplied), every lane gathers its
// pixel operand (pixel row, 8 or 1 contraction indices) from that halo, and
// the whole filter bank lives in registers.  Contraction index k = 3*tap + ci;
// the indices 27 (and 28 for bf16) that pad the contraction to a multiple of
// the MFMA depth carry the bias: the pixel operand is 1 there and the filter
// operand the bias (for bf16 split into a rounded value and its remainder), so
// the matrix pipe adds it.  The MFMAs take the filter fragment first, so a lane
// ends up with runs of four consecutive channels of one pixel; those go through
// a per-wave LDS block so that each lane stores 16 contiguous bytes.
#include "common.h"

namespace vgg {

typedef unsigned int u32x4f __attribute__((ext_vector_type(4)));

constexpr int kFirstCout = 64;
constexpr int kHaloW = 20;                       // 18 columns + 2 pad floats per halo row
constexpr int kHaloFloats = 3 * 18 * kHaloW;
constexpr int kHaloElems = 3 * 18 * 18;
constexpr int kHaloPerThread = (kHaloElems + 255) / 256;
constexpr int kFirstEpiRow = 144, kFirstEpiBytes = 32 * kFirstEpiRow;

// float offset inside the staged halo of contraction index k for the pixel at halo origin
__host__ __device__ constexpr int first_koff(int k)
{
    return k < 27 ? ((k % 3) * 18 + (k / 3) / 3) * kHaloW + (k / 3) % 3 : 0;
}

struct FirstArgs {
    const float *x;     // [N][3][H][W]
    const char *w;      // packed [9][64][CinP] in T
    const float *bias;  // [64]
    char *y;            // [N][H][W][64] in T
    int N, H, W, CinP, relu, tiles_w, tiles_hw, ntiles;
    FastDiv dTilesW, dTilesHW;
};

template <typename T>
__global__ __launch_bounds__(256, 3) void conv_first_kernel(FirstArgs p)
{
    __shared__ float xs[kHaloFloats];
    __shared__ __align__(16) char epi_all[4 * kFirstEpiBytes];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = lane & 31, khalf = lane >> 5;
    const T *wp = reinterpret_cast<const T *>(p.w);
    constexpr bool kBf16 = sizeof(T) == 2;
    // filter operand for contraction index k, output channel co (bias at the padding indices)
    auto wval = [&](int k, int co) -> float {
        if (k < 27) return Elem<T>::load(wp + packed_w_index<T>(k / 3, co, k % 3, kFirstCout, p.CinP));
        const float b = p.bias ? p.bias[co] : 0.f;
        if (k == 27) return kBf16 ? bf16_to_f32(f32_to_bf16(b)) : b;
        if (k == 28 && kBf16) return b - bf16_to_f32(f32_to_bf16(b));
        return 0.f;
    };
    // The whole filter bank, loaded once per workgroup and kept in registers.
    bf16x8 bfrag16[kBf16 ? 2 : 1][2];
    float bfrag32[kBf16 ? 1 : 14][2];
    if constexpr (kBf16) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int j = 0; j < 2; ++j) bfrag16[s][j][t] = (__bf16)wval(s * 16 + khalf * 8 + t, j * 32 + r);
    } else {
#pragma unroll
        for (int s = 0; s < 14; ++s)
#pragma unroll
            for (int j = 0; j < 2; ++j) bfrag32[s][j] = wval(2 * s + khalf, j * 32 + r);
    }

    // halo origin (float offset) of this lane's two pixels: tile rows wv*64 + i*32 + r
    int pbase[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int j = wv * 64 + i * 32 + r;
        pbase[i] = (j >> 4) * kHaloW + (j & 15);
    }
    constexpr int VEC = 16 / (int)sizeof(T), CPT = 128 / (int)sizeof(T), TJ = CPT / 32;
    char *epi = epi_all + wv * kFirstEpiBytes;
    T *y = reinterpret_cast<T *>(p.y);
    const int seg = lane & 7, rowq = lane >> 3;
    const float lo = p.relu ? 0.f : -__builtin_inff();

    // The halo elements this thread stages: the same positions of every patch.
    int hy_[kHaloPerThread], hx_[kHaloPerThread], lds_[kHaloPerThread], rel_[kHaloPerThread];
#pragma unroll
    for (int k = 0; k < kHaloPerThread; ++k) {
        const int idx = min(tid + k * 256, kHaloElems - 1);
        const int c = idx / 324, q = idx - c * 324, hy = q / 18, hx = q - hy * 18;
        hy_[k] = hy - 1; hx_[k] = hx - 1;
        lds_[k] = (c * 18 + hy) * kHaloW + hx;
        rel_[k] = (c * p.H + hy - 1) * p.W + hx - 1;
    }
    auto load_halo = [&](int tile, float (&hv)[kHaloPerThread]) __attribute__((always_inline)) {
        const int n = fast_div(tile, p.dTilesHW);
        const int rem = tile - n * p.tiles_hw;
        const int ty = fast_div(rem, p.dTilesW);
        const int h0 = ty * 16, w0 = (rem - ty * p.tiles_w) * 16;
        const float *base = p.x + (size_t)n * 3 * p.H * p.W + h0 * p.W + w0;
#pragma unroll
        for (int k = 0; k < kHaloPerThread; ++k) {
            const int h = h0 + hy_[k], w = w0 + hx_[k];
            const bool ok = h >= 0 && h < p.H && w >= 0 && w < p.W;
            hv[k] = ok ? base[rel_[k]] : 0.f;
        }
    };
    auto store_halo = [&](const float (&hv)[kHaloPerThread]) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < kHaloPerThread; ++k)
            if ((k + 1) * 256 <= kHaloElems || tid + k * 256 < kHaloElems) xs[lds_[k]] = hv[k];
    };

    // Workgroup b runs on XCD b % 8 and every XCD has its own L2.  Each XCD takes a contiguous eighth of the
    // patches and its workgroups walk through it side by side, so the patches in flight on an XCD are
    // neighbours: the halo rows and the partly used cache lines that neighbours share are then fetched from
    // memory once, not once per XCD (measured: a third of the fetched bytes; the kernel's time is set by its
    // output stores and does not change).
    const int xcd = blockIdx.x & 7;
    const int per_xcd = (p.ntiles + 7) / 8;
    const int last = min((xcd + 1) * per_xcd, p.ntiles);
    const int stride = ((int)gridDim.x + 7 - xcd) / 8;        // workgroups of this XCD
    const int first = xcd * per_xcd + ((int)blockIdx.x >> 3);
    // (Barriers without the memory fence of __syncthreads(): that fence waits for every outstanding
    // vector-memory operation, i.e. for the previous patch's output stores.  Only LDS traffic is ordered here.)
    auto lds_barrier = [] { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    float hv[kHaloPerThread];
    if (first < last) load_halo(first, hv);
    for (int tile = first; tile < last; tile += stride) {
        const int n = fast_div(tile, p.dTilesHW);
        const int rem = tile - n * p.tiles_hw;
        const int ty = fast_div(rem, p.dTilesW);
        const int h0 = ty * 16, w0 = (rem - ty * p.tiles_w) * 16;
        lds_barrier();    // previous tile's halo no longer read
        store_halo(hv);
        lds_barrier();
        if (tile + stride < last) load_halo(tile + stride, hv);  // lands during the arithmetic below

        f32x16 acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

        if constexpr (kBf16) {
            // two steps of v_mfma_f32_32x32x16_bf16: k = 16*s + 8*khalf + t
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                bf16x8 afrag[2];
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const int k0 = s * 16 + t, k1 = s * 16 + 8 + t;       // this lane's k is k0 or k1
                    const int off = khalf ? first_koff(k1) : first_koff(k0);
                    const bool data = khalf ? k1 < 27 : k0 < 27;
                    const float pad = (khalf ? (k1 == 27 || k1 == 28) : (k0 == 27 || k0 == 28)) ? 1.f : 0.f;
#pragma unroll
                    for (int i = 0; i < 2; ++i) afrag[i][t] = (__bf16)(data ? xs[pbase[i] + off] : pad);
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag16[s][j], afrag[i], acc[i][j], 0, 0, 0);
            }
        } else {
            // fourteen steps of v_mfma_f32_32x32x2_f32: k = 2*s + khalf
#pragma unroll
            for (int s = 0; s < 14; ++s) {
                const int k = 2 * s + khalf;
                const int off = khalf ? first_koff(2 * s + 1) : first_koff(2 * s);
                float a[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) a[i] = k < 27 ? xs[pbase[i] + off] : (k == 27 ? 1.f : 0.f);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(bfrag32[s][j], a[i], acc[i][j], 0, 0, 0);
            }
        }

        // epilogue: register e of lane l is channel 8*(e/4) + 4*(l/32) + e%4 of pixel row l%32; ReLU,
        // 32 pixels x 128 bytes through this wave's LDS block, 16-byte stores
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int j0 = 0; j0 < 2; j0 += TJ) {
#pragma unroll
                for (int jj = 0; jj < TJ; ++jj) {
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        const f32x16 &t = acc[i][j0 + jj];
                        store4(reinterpret_cast<T *>(epi + r * kFirstEpiRow) + jj * 32 + a * 8 + khalf * 4,
                               fmaxf(t[a * 4], lo), fmaxf(t[a * 4 + 1], lo), fmaxf(t[a * 4 + 2], lo),
                               fmaxf(t[a * 4 + 3], lo));
                    }
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int row = rowq + 8 * q;
                    const u32x4f v = *reinterpret_cast<const u32x4f *>(epi + row * kFirstEpiRow + seg * 16);
                    const int j = wv * 64 + i * 32 + row;
                    const int h = h0 + (j >> 4), w = w0 + (j & 15);
                    if (h < p.H && w < p.W)
                        *reinterpret_cast<u32x4f *>(y + (((size_t)n * p.H + h) * p.W + w) * kFirstCout + j0 * 32 + seg * VEC) = v;
                }
            }
        }
    }
}

// x NCHW fp32 [N][3][H][W]; w packed [9][64][CinP] (dtype); y NHWC [N][H][W][64] (dtype).
int conv_first(int dtype, int N, int H, int W, int CinP, const float *x, const void *w, const float *bias, void *y,
               int relu, hipStream_t stream)
{
    FirstArgs a;
    a.x = x; a.w = static_cast<const char *>(w); a.bias = bias; a.y = static_cast<char *>(y);
    a.N = N; a.H = H; a.W = W; a.CinP = CinP; a.relu = relu;
    a.tiles_w = (W + 15) / 16;
    a.tiles_hw = a.tiles_w * ((H + 15) / 16);
    a.ntiles = N * a.tiles_hw;
    a.dTilesW = make_fast_div(a.tiles_w); a.dTilesHW = make_fast_div(a.tiles_hw);
    const dim3 grid((unsigned)(a.ntiles < 2048 ? a.ntiles : 2048));
    if (dtype == VGG_BF16)
        hipLaunchKernelGGL(conv_first_kernel<bf16_t>, grid, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL(conv_first_kernel<float>, grid, dim3(256), 0, stream, a);
    return launch_status();
}

}  // namespace vgg
