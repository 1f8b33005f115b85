// Implicit-GEMM 3x3 stride-1 pad-1 convolution on MFMA for gfx950, NHWC.
//
// GEMM view: rows = output pixels m = (n,h,w) flattened, columns = output
// channels, contraction index = (tap, input channel).  The forward
// convolution (appendix table row "convolution") and the data-gradient
// convolution (rows "reverse" + "convolution" of the backward column) both run
// through this kernel; they differ only in how the weights were packed.
//
// Staging.  A workgroup owns one tile of BM output pixels (see TileGeom:
// either BM consecutive pixels or a 16x16 patch) and BN output channels.  The
// tile's input halo is staged in LDS once per channel chunk, with zeros where
// the halo leaves the image, and is then read by all nine taps, so zero
// padding and image boundaries inside a tile need no masks.
//
// Every LDS row holds 64 bytes of one pixel's channels (16 fp32 or 32 bf16)
// plus 16 bytes of padding, which makes the 16-byte fragment reads of 32
// consecutive rows bank-conflict free.  A lane reads 16 bytes of A and of B
// at the same (k-group, k-half) position: for bf16 that is the 8-element
// operand of one v_mfma_f32_32x32x16_bf16; for fp32 the four elements feed
// four v_mfma_f32_32x32x2_f32 (any fixed pairing of k indices between A and B
// is a valid contraction order).
#include "common.h"

namespace vgg {

constexpr int kRowBytes = 80;  // 64 data + 16 pad
constexpr int kDataBytes = 64;
constexpr int kMaxAHaloSegsPerBlock = 1536;  // 16-byte halo segments (384 rows) prefetched through registers

struct ConvArgs {
    const char *x;      // [M][CinP] elements of T
    const char *w;      // [9][Cout][CinP]
    const float *bias;  // [Cout] or null
    const char *mask;   // [M][Cout] of T or null: output multiplied by (mask > 0)
    char *y;            // [M][Cout]
    int CinP, Cout;
    int relu;
    int tiles_n;        // number of column tiles
    int rowsA;          // LDS rows reserved for the halo
    TileGeom g;
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ const u32x4 kZeroRow[4] = {};  // 64 zero bytes: what a halo row outside the image reads

template <typename T> struct Mma;
template <> struct Mma<float> {
    static __device__ __forceinline__ void run(f32x16 &acc, const uint4 &a, const uint4 &b)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
    }
};
template <> struct Mma<bf16_t> {
    static __device__ __forceinline__ void run(f32x16 &acc, const uint4 &a, const uint4 &b)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                      __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
    }
};

template <typename T, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM *WN * 64, WM * WN == 8 ? 2 : 2) void conv3x3_igemm_kernel(ConvArgs p)
{
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32;  // 32x32 MFMA tiles per wave along pixels
    constexpr int TN = BN / WN / 32;  // and along channels
    constexpr int KC = kDataBytes / (int)sizeof(T);

    extern __shared__ __align__(16) char smem[];
    const int S = p.g.S;
    const int SA = p.rowsA;                     // rows reserved for the halo (>= S)
    int *pix = reinterpret_cast<int *>(smem);   // [SA] halo row -> input pixel or -1
    char *As = smem + round_up16(SA * 4);       // [SA][80]
    char *Bs = As + (size_t)SA * kRowBytes;     // [3][BN][80]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int wm = wv % WM, wn = wv / WM;
    const int r = lane & 31, khalf = lane >> 5;

    const int tile_n = blockIdx.x % p.tiles_n;
    const int tile_m = blockIdx.x / p.tiles_n;
    const int n0 = tile_n * BN;
    const TileOrigin org = tile_origin(p.g, tile_m);
    const int pitch = p.g.pitch;

    for (int i = tid; i < SA; i += NT) pix[i] = i < S ? halo_pixel(p.g, org, i) : -1;

    // LDS byte offset (for tap (0,0)) of each of this lane's pixel rows
    int abase[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int m, hrow;
        tile_row(p.g, org, wm * (BM / WM) + i * 32 + r, m, hrow);
        abase[i] = hrow * kRowBytes + khalf * 16;
    }
    int bbase[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) bbase[j] = (wn * (BN / WN) + j * 32 + r) * kRowBytes + khalf * 16;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const size_t xrow = (size_t)p.CinP * sizeof(T);
    const int nA = S * 4;  // 16-byte segments of the halo per chunk
    constexpr int NB = 3 * BN * 4 / NT;  // 16-byte weight segments per thread and stage
    constexpr int MAXA = kMaxAHaloSegsPerBlock / NT;  // halo segments per thread prefetched through registers
    const bool a_regs = nA <= MAXA * NT; // then SA == MAXA*NT/4: every thread copies exactly MAXA segments
    const int nstages = (p.CinP / KC) * 3;

    // Global -> register halves of the staging copies.  A stage is (channel chunk, kernel row): it
    // needs the three taps' weights of that row and, when the chunk changes, a new halo.
    // (branch-free: a pad row reads from a block of zeros instead of the tensor)
    auto load_a = [&](int c0, u32x4(&areg)[MAXA]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < MAXA; ++j) {
            const int idx = tid + j * NT;
            const int off = pix[idx >> 2];
            const char *src = off < 0 ? reinterpret_cast<const char *>(kZeroRow)
                                      : p.x + (size_t)off * xrow + (size_t)c0 * sizeof(T);
            areg[j] = *reinterpret_cast<const u32x4 *>(src + (idx & 3) * 16);
        }
    };
    auto store_a = [&](const u32x4(&areg)[MAXA]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < MAXA; ++j) {
            const int idx = tid + j * NT;
            *reinterpret_cast<u32x4 *>(As + (idx >> 2) * kRowBytes + (idx & 3) * 16) = areg[j];
        }
    };
    auto copy_a_direct = [&](int c0) __attribute__((always_inline)) {  // halo too large for the register path
        for (int idx = tid; idx < nA; idx += NT) {
            const int off = pix[idx >> 2];
            u32x4 v = {0u, 0u, 0u, 0u};
            if (off >= 0)
                v = *reinterpret_cast<const u32x4 *>(p.x + (size_t)off * xrow + (size_t)c0 * sizeof(T) + (idx & 3) * 16);
            *reinterpret_cast<u32x4 *>(As + (idx >> 2) * kRowBytes + (idx & 3) * 16) = v;
        }
    };
    auto load_b = [&](int c0, int kh, u32x4(&breg)[NB]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int idx = tid + j * NT;
            const int row = idx >> 2;  // kw*BN + n
            const int kw = row / BN;
            const int n = min(n0 + row - kw * BN, p.Cout - 1);  // columns past Cout are never stored
            breg[j] = *reinterpret_cast<const u32x4 *>(
                p.w + ((size_t)((kh * 3 + kw) * p.Cout + n) * p.CinP + c0) * sizeof(T) + (idx & 3) * 16);
        }
    };
    auto store_b = [&](const u32x4(&breg)[NB]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int idx = tid + j * NT;
            *reinterpret_cast<u32x4 *>(Bs + (idx >> 2) * kRowBytes + (idx & 3) * 16) = breg[j];
        }
    };

    u32x4 areg[MAXA], breg[NB];
    __syncthreads();  // halo table ready
    if (a_regs) { load_a(0, areg); store_a(areg); } else copy_a_direct(0);
    load_b(0, 0, breg);
    store_b(breg);
    __syncthreads();

    auto compute = [&](int kh) __attribute__((always_inline)) {
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            const int toff = (kh * pitch + kw) * kRowBytes;
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                uint4 af[TM], bf[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    af[i] = *reinterpret_cast<const uint4 *>(As + abase[i] + toff + g * 32);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    bf[j] = *reinterpret_cast<const uint4 *>(Bs + kw * BN * kRowBytes + bbase[j] + g * 32);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) Mma<T>::run(acc[i][j], af[i], bf[j]);
            }
        }
    };

    // Software pipeline: the global loads of stage s+1 are issued before the MFMAs of stage s and
    // land in LDS after them, so their latency is covered by the arithmetic.
    int kh = 0, c0 = 0;
    for (int s = 0; s + 1 < nstages; ++s) {
        int nkh = kh + 1, nc0 = c0;
        if (nkh == 3) { nkh = 0; nc0 += KC; }
        const bool new_chunk = nkh == 0;
        load_b(nc0, nkh, breg);
        if (new_chunk && a_regs) load_a(nc0, areg);
        compute(kh);
        __syncthreads();  // every wave is done reading this stage's LDS data
        store_b(breg);
        if (new_chunk) {
            if (a_regs) store_a(areg); else copy_a_direct(nc0);
        }
        __syncthreads();
        kh = nkh; c0 = nc0;
    }
    compute(kh);

    // epilogue: bias, ReLU, optional (mask > 0) factor, convert, store.
    // 32x32 accumulator layout: register e of lane l holds row 8*(e/4) + 4*(l/32) + e%4, column l%32.
    T *y = reinterpret_cast<T *>(p.y);
    const T *mask = reinterpret_cast<const T *>(p.mask);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            int m, hrow;
            tile_row(p.g, org, wm * (BM / WM) + i * 32 + khalf * 4 + (e >> 2) * 8 + (e & 3), m, hrow);
            if (m < 0) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + wn * (BN / WN) + j * 32 + r;
                if (col < p.Cout) {
                    float v = acc[i][j][e] + (p.bias ? p.bias[col] : 0.f);
                    if (p.relu) v = fmaxf(v, 0.f);
                    const size_t o = (size_t)m * p.Cout + col;
                    if (mask && !(Elem<T>::load(mask + o) > 0.f)) v = 0.f;
                    Elem<T>::store(y + o, v);
                }
            }
        }
    }
}

template <typename T, int BM, int BN, int WM, int WN>
static int launch_conv(const ConvArgs &a0, int N, int H, int W, hipStream_t stream)
{
    ConvArgs a = a0;
    a.g = make_tile_geom(N, H, W, BM);
    a.tiles_n = (a.Cout + BN - 1) / BN;
    constexpr int NT = WM * WN * 64;
    a.rowsA = a.g.S * 4 <= kMaxAHaloSegsPerBlock ? kMaxAHaloSegsPerBlock / 4 : a.g.S;
    const size_t lds = round_up((size_t)a.rowsA * 4, 16) + (size_t)a.rowsA * kRowBytes + (size_t)3 * BN * kRowBytes;
    if (lds > 160 * 1024) return VGG_ERR_UNSUPPORTED;
    auto kern = conv3x3_igemm_kernel<T, BM, BN, WM, WN>;
    static bool configured = false;
    if (lds > 64 * 1024 && !configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                160 * 1024) != hipSuccess)
            return VGG_ERR_LAUNCH;
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(a.g.ntiles * a.tiles_n)), dim3(WM * WN * 64), lds, stream, a);
    return launch_status();
}

// x: [N*H*W][CinP], w: [9][Cout][CinP] (elements of dtype); y: [N*H*W][Cout].
int conv3x3_igemm(int dtype, int N, int H, int W, int CinP, int Cout, const void *x, const void *w,
                  const float *bias, const void *mask, void *y, int relu, hipStream_t stream)
{
    ConvArgs a;
    a.x = static_cast<const char *>(x);
    a.w = static_cast<const char *>(w);
    a.bias = bias;
    a.mask = static_cast<const char *>(mask);
    a.y = static_cast<char *>(y);
    a.CinP = CinP; a.Cout = Cout;
    a.relu = relu; a.tiles_n = 0; a.rowsA = 0;
    const bool narrow = Cout <= 64;
    if (dtype == VGG_F32) {
        return narrow ? launch_conv<float, 256, 64, 4, 1>(a, N, H, W, stream)
                      : launch_conv<float, 256, 128, 4, 2>(a, N, H, W, stream);
    }
    return narrow ? launch_conv<bf16_t, 256, 64, 4, 1>(a, N, H, W, stream)
                  : launch_conv<bf16_t, 256, 128, 4, 2>(a, N, H, W, stream);
}

}  // namespace vgg
