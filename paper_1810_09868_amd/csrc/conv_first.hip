// First convolution of the network (3 -> 64 channels) read straight from the
// canonical NCHW fp32 image batch and written as NHWC in the compute dtype.
//
// With only 27 contraction indices the layer is bound by writing its output
// (appendix table row "convolution", first of 16); padding the image to a
// full channel row and running the general kernel would read and write an
// extra padded copy of the batch.  Here a workgroup stages the 3 x 18 x 18
// fp32 halo of a 16 x 16 pixel patch in LDS, every lane gathers its A
// operand (pixel row, 8 or 1 contraction indices) from that halo, the B
// operand (the whole 27 x 64 filter bank) lives in registers, and the result
// goes through the same LDS transpose as the general kernel so that each
// lane stores 16 contiguous bytes.  Contraction index k = 3*tap + ci.
#include "common.h"

namespace vgg {

typedef unsigned int u32x4f __attribute__((ext_vector_type(4)));

constexpr int kFirstCout = 64;
constexpr int kHaloW = 20;                       // 18 columns + 2 pad floats per halo row
constexpr int kHaloFloats = 3 * 18 * kHaloW;
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
};

template <typename T>
__global__ __launch_bounds__(256) void conv_first_kernel(FirstArgs p)
{
    __shared__ float xs[kHaloFloats];
    __shared__ __align__(16) char epi_all[4 * kFirstEpiBytes];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = lane & 31, khalf = lane >> 5;
    const T *wp = reinterpret_cast<const T *>(p.w);
    auto wval = [&](int k, int co) -> float {  // filter value for contraction index k, output channel co
        return k < 27 ? Elem<T>::load(wp + ((size_t)(k / 3) * kFirstCout + co) * p.CinP + k % 3) : 0.f;
    };
    // The whole filter bank as B operands, loaded once per workgroup and kept in registers.
    constexpr bool kBf16 = sizeof(T) == 2;
    constexpr int NSTEP = kBf16 ? 2 : 14;
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
    float bv[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) bv[j] = p.bias ? p.bias[j * 32 + r] : 0.f;

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

    for (int tile = blockIdx.x; tile < p.ntiles; tile += gridDim.x) {
        const int n = tile / p.tiles_hw;
        const int rem = tile - n * p.tiles_hw;
        const int h0 = (rem / p.tiles_w) * 16, w0 = (rem % p.tiles_w) * 16;
        __syncthreads();  // previous tile's halo no longer read
        for (int idx = tid; idx < 3 * 18 * 18; idx += 256) {
            const int c = idx / 324, q = idx - c * 324, hy = q / 18, hx = q - hy * 18;
            const int h = h0 - 1 + hy, w = w0 - 1 + hx;
            float v = 0.f;
            if (h >= 0 && h < p.H && w >= 0 && w < p.W) v = p.x[(((size_t)n * 3 + c) * p.H + h) * p.W + w];
            xs[(c * 18 + hy) * kHaloW + hx] = v;
        }
        __syncthreads();

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
                    const int k = s * 16 + khalf * 8 + t;
                    const int off = khalf ? first_koff(s * 16 + 8 + t) : first_koff(s * 16 + t);
#pragma unroll
                    for (int i = 0; i < 2; ++i) afrag[i][t] = (__bf16)(k < 27 ? xs[pbase[i] + off] : 0.f);
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag[i], bfrag16[s][j], acc[i][j], 0, 0, 0);
            }
        } else {
            // fourteen steps of v_mfma_f32_32x32x2_f32: k = 2*s + khalf
#pragma unroll
            for (int s = 0; s < 14; ++s) {
                const int k = 2 * s + khalf;
                const int off = khalf ? first_koff(2 * s + 1) : first_koff(2 * s);
                float a[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) a[i] = k < 27 ? xs[pbase[i] + off] : 0.f;
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], bfrag32[s][j], acc[i][j], 0, 0, 0);
            }
        }

        // epilogue: bias, ReLU, transpose 32 rows x 128 bytes through this wave's LDS block, 16-byte stores
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int j0 = 0; j0 < 2; j0 += TJ) {
#pragma unroll
                for (int jj = 0; jj < TJ; ++jj) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        float v = acc[i][j0 + jj][e] + bv[j0 + jj];
                        if (p.relu) v = fmaxf(v, 0.f);
                        const int row = (e >> 2) * 8 + khalf * 4 + (e & 3);
                        Elem<T>::store(reinterpret_cast<T *>(epi + row * kFirstEpiRow) + jj * 32 + r, v);
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
    const dim3 grid((unsigned)(a.ntiles < 2048 ? a.ntiles : 2048));
    if (dtype == VGG_BF16)
        hipLaunchKernelGGL(conv_first_kernel<bf16_t>, grid, dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL(conv_first_kernel<float>, grid, dim3(256), 0, stream, a);
    return launch_status();
}

}  // namespace vgg
