// The first two convolutions of the network in one kernel, bf16, gfx950:
//
//   pooled = maxpool2x2( relu(conv3x3( relu(conv3x3(x, w1) + b1), w2) + b2) ),   3 -> 64 -> 64 channels
//
// (first two "convolution" rows and the first "reduce-window" of the appendix table's forward column; the
// paper's compiler fuses operations so that intermediates stay on chip, section on XLA).  At batch 100 the
// 64-channel 224 x 224 activation between the two layers is 642 MB: written once and read once it costs more
// HBM time than either layer's arithmetic.  Here it never leaves the CU.  A workgroup owns a 16 x 32 pixel
// patch of the second layer's output:
//   1. the 3 x 20 x 36 image halo of the patch goes to LDS, rounded to bf16, one 8-byte record (three
//      channels and a zero) per pixel (the next patch's is already in registers);
//   2. the first layer is evaluated on the 18 x 34 pixel halo the second layer needs: contraction index
//      k = 4 tap + ci, so that a lane's eight indices of an MFMA step are two whole records, and the bias
//      rides on a tenth "tap" whose record is (1, 1, 0, 0) (weights there: the bias rounded to bf16 and
//      the remainder), three steps of v_mfma_f32_32x32x16_bf16.  The result goes to LDS as two
//      32-channel chunks of 80-byte rows, zero where the halo pixel lies outside the image (the second
//      layer's zero padding).  The products are those of the stand-alone first-layer kernel; only the
//      order in which the matrix unit adds the 27 of them differs;
//   3. the second layer runs on that halo like the weights-in-registers implicit GEMM: a wave owns four patch
//      rows (128 pixels) x 64 channels, its weight fragments come straight from global memory (L2) five
//      steps ahead, the sums run over (chunk, tap, k-group) in that kernel's order (same results);
//   4. the 2x2 maximum is taken on the fp32 sums in registers (rows of a window are two accumulator blocks
//      of the same lane, columns are neighbouring lanes), then ReLU and rounding (both monotonic, so the
//      result is the maximum of the rounded values); pooled and/or un-pooled tensor leave through a
//      per-wave LDS block as full 128-byte pixel rows.
// One workgroup per CU (107 KB of LDS), persistent over the patches of its XCD's share.
// Needs H % 16 == 0 and W % 32 == 0; no pooling positions (the training step keeps the separate kernels,
// whose outputs its backward pass reads).
#include "common.h"
#include <utility>

namespace vgg {

namespace {

constexpr int kC = 64;                               // channels of both layers
constexpr int kTH = 16, kTW = 32;                    // output patch
constexpr int kYR = kTH + 2, kYC = kTW + 2;          // first-layer halo: 18 x 34 pixels
constexpr int kYRows = kYR * kYC;                    // 612
constexpr int kYBlocks = (kYRows + 31) / 32;         // 20 blocks of 32 pixels
static_assert(kYBlocks % 4 == 0, "every wave takes the same number of blocks");
constexpr int kXR = kTH + 4, kXC = kTW + 4;          // image halo: 20 x 36
constexpr int kXPix = kXR * kXC;                     // 720 pixel records of 8 bytes
constexpr int kXOnes = kXPix, kXZero = kXPix + 1;    // two constant records: (1, 1, 0, 0) and zeros
constexpr int kXBytes = (kXPix + 2) * 8;
constexpr int kXPerThread = (kXPix + 255) / 256;     // 3
constexpr int kRowB = 80;                            // LDS bytes per halo row of a 32-channel chunk (64 + 16 pad)
constexpr int kYBytes = 2 * kYRows * kRowB;          // 97920
constexpr int kStageRow = 144;                       // epilogue staging: 64 channels + 16 bytes of padding
constexpr int kSteps = 36;                           // (chunk, tap, k-group) steps of the second layer
constexpr int kRing = 12, kAhead = kRing - 1;        // weight fragments in registers, prefetch distance (with one wave
                                                     // per SIMD a step is short: eleven of them cover the L2 latency)
static_assert(kSteps % kRing == 0, "ring positions are static");
static_assert(4 * 64 * kStageRow <= kYBytes, "staging blocks live in the halo buffer");

// byte offset of tap t's record relative to the record of the first-layer pixel's own position in the halo
__host__ __device__ constexpr int pair_tap_off(int t)
{
    return ((t / 3) * kXC + t % 3) * 8;
}

struct PairArgs {
    const float *x;     // [N][3][H][W]
    const char *w1;     // first layer, packed bf16 [9][64][CinP1]
    const float *b1;
    const char *w2;     // second layer, packed bf16 [9][64][64]
    const float *b2;
    char *y;            // [N][H][W][64] bf16 or null
    char *pool;         // [N][H/2][W/2][64] bf16 or null
    int N, H, W, CinP1, tiles_w, tiles_hw, ntiles;
    FastDiv dTilesW, dTilesHW;
};

template <typename F, int... S>
__device__ __forceinline__ void pair_for_each(F &&f, std::integer_sequence<int, S...>)
{
    (f(std::integral_constant<int, S>{}), ...);
}

__global__ __launch_bounds__(256, 1) void conv_pair_kernel(PairArgs p)
{
    typedef bf16_t T;
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    extern __shared__ __align__(16) char smem[];
    char *ys = smem;                                             // [2][kYRows][kRowB]; later the staging blocks
    char *xs = smem + kYBytes;                                   // [kXR][kXC] records (c0, c1, c2, 0) + the two constants
    const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 31, khalf = lane >> 5;
    const T *w1p = reinterpret_cast<const T *>(p.w1);
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

    // ---- first layer's filter bank in registers: contraction index k = 4 tap + ci; tap 9 carries the bias
    auto w1val = [&](int k, int co) -> float {
        const int t = k >> 2, ci = k & 3;
        if (t < 9) return ci < 3 ? Elem<T>::load(w1p + packed_w_index<T>(t, co, ci, kC, p.CinP1)) : 0.f;
        const float b = p.b1 ? p.b1[co] : 0.f;
        if (k == 36) return bf16_to_f32(f32_to_bf16(b));
        if (k == 37) return b - bf16_to_f32(f32_to_bf16(b));
        return 0.f;
    };
    bf16x8 w1f[3][2];
#pragma unroll
    for (int s = 0; s < 3; ++s)
#pragma unroll
        for (int t = 0; t < 8; ++t)
#pragma unroll
            for (int j = 0; j < 2; ++j) w1f[s][j][t] = (__bf16)w1val(s * 16 + khalf * 8 + t, j * 32 + r);
    if (tid == 0) {
        *reinterpret_cast<u32x2 *>(xs + kXOnes * 8) = u32x2{0x3F803F80u, 0u};
        *reinterpret_cast<u32x2 *>(xs + kXZero * 8) = u32x2{0u, 0u};
    }

    // ---- the image halo pixels this thread stages: the same positions of every patch
    int hy_[kXPerThread], hx_[kXPerThread];
#pragma unroll
    for (int k = 0; k < kXPerThread; ++k) {
        const int idx = min(tid + k * 256, kXPix - 1);
        const int hy = idx / kXC, hx = idx - hy * kXC;
        hy_[k] = hy - 2; hx_[k] = hx - 2;
    }
    const int plane = p.H * p.W;
    auto tile_pos = [&](int tile, int &n, int &h0, int &w0) __attribute__((always_inline)) {
        n = fast_div(tile, p.dTilesHW);
        const int rem = tile - n * p.tiles_hw;
        const int ty = fast_div(rem, p.dTilesW);
        h0 = ty * kTH;
        w0 = (rem - ty * p.tiles_w) * kTW;
    };
    auto load_halo = [&](int tile, float (&hv)[kXPerThread][3]) __attribute__((always_inline)) {
        int n, h0, w0;
        tile_pos(tile, n, h0, w0);
#pragma unroll
        for (int k = 0; k < kXPerThread; ++k) {
            // (always a load, from a clamped position, and a select afterwards: a load inside a branch is
            // waited for where the branch ends, one memory latency per halo element)
            const int h = h0 + hy_[k], w = w0 + hx_[k];
            const bool ok = h >= 0 && h < p.H && w >= 0 && w < p.W;
            const int hc = min(max(h, 0), p.H - 1), wc = min(max(w, 0), p.W - 1);
            const float *src = p.x + (size_t)n * 3 * plane + hc * p.W + wc;
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                const float v = src[c * plane];
                hv[k][c] = ok ? v : 0.f;
            }
        }
    };
    auto store_halo = [&](const float (&hv)[kXPerThread][3]) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < kXPerThread; ++k)
            if ((k + 1) * 256 <= kXPix || tid + k * 256 < kXPix) {
                typedef float f32x2_t __attribute__((ext_vector_type(2)));
                typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
                const f32x2_t lo = {hv[k][0], hv[k][1]}, hi = {hv[k][2], 0.f};
                const u32x2 rec = {__builtin_bit_cast(unsigned int, __builtin_convertvector(lo, bf16x2_t)),
                                   __builtin_bit_cast(unsigned int, __builtin_convertvector(hi, bf16x2_t))};
                *reinterpret_cast<u32x2 *>(xs + (tid + k * 256) * 8) = rec;
            }
    };
    // (without the memory fence of __syncthreads(), which would wait for the previous patch's output stores)
    auto lds_barrier = [] { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

    // ---- second layer: this wave's four patch rows, all 64 channels
    // weight fragment (tap t, 16-channel block kb, output channels c..c+31): 1 KB at ((4 t + kb) 64 + c) 32 bytes
    unsigned voff[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) voff[j] = (unsigned)(j * 32 + r) * 32u + khalf * 16;
    int arow[4];   // byte offset (inside a chunk) of tap (0,0) of this lane's pixel in each of the four rows
#pragma unroll
    for (int i = 0; i < 4; ++i) arow[i] = ((wv * 4 + i) * kYC + r) * kRowB + khalf * 16;

    // Workgroup b runs on XCD b % 8: each XCD takes a contiguous eighth of the patches (neighbouring patches
    // share image rows and cache lines, which then come from that XCD's L2).
    const int xcd = blockIdx.x & 7;
    const int per_xcd = (p.ntiles + 7) / 8;
    const int last = min((xcd + 1) * per_xcd, p.ntiles);
    const int stride = ((int)gridDim.x + 7 - xcd) / 8;
    const int first = xcd * per_xcd + ((int)blockIdx.x >> 3);
    float hv[kXPerThread][3];
    if (first < last) load_halo(first, hv);

    for (int tile = first; tile < last; tile += stride) {
        int n, h0, w0;
        tile_pos(tile, n, h0, w0);
        lds_barrier();    // the previous patch's staging blocks and image halo are no longer read
        store_halo(hv);
        lds_barrier();
        if (tile + stride < last) load_halo(tile + stride, hv);   // lands during the arithmetic below

        // ---- first layer on the 18 x 34 halo: wave w takes pixel blocks w, w + 4, ...  (The last block has
        // only four pixels: its other lanes repeat the last pixel and store the same bytes to the same place.)
#pragma unroll
        for (int bi = 0; bi < kYBlocks / 4; ++bi) {
            const int blk = wv + 4 * bi;
            const int q = min(blk * 32 + r, kYRows - 1);
            const int hy = q / kYC, hx = q - hy * kYC;
            const char *rec = xs + (hy * kXC + hx) * 8;
            f32x16 a1[2];
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) a1[j][e] = 0.f;
            // step s, lanes 0-31: taps 4s, 4s + 1; lanes 32-63: taps 4s + 2, 4s + 3 (tap 9: the ones, then zeros)
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                u32x2 lo, hi;
                if (s < 2) {
                    lo = *reinterpret_cast<const u32x2 *>(rec + (khalf ? pair_tap_off(4 * s + 2) : pair_tap_off(4 * s)));
                    hi = *reinterpret_cast<const u32x2 *>(rec + (khalf ? pair_tap_off(4 * s + 3) : pair_tap_off(4 * s + 1)));
                } else {
                    lo = *reinterpret_cast<const u32x2 *>(khalf ? xs + kXZero * 8 : rec + pair_tap_off(8));
                    hi = *reinterpret_cast<const u32x2 *>(xs + (khalf ? kXZero : kXOnes) * 8);
                }
                const u32x4 v = {lo[0], lo[1], hi[0], hi[1]};
                const bf16x8 af = __builtin_bit_cast(bf16x8, v);
#pragma unroll
                for (int j = 0; j < 2; ++j) a1[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1f[s][j], af, a1[j], 0, 0, 0);
            }
            // register e of lane l is channel 8 (e / 4) + 4 (l / 32) + e % 4 of pixel l % 32
            const int h = h0 - 1 + hy, w = w0 - 1 + hx;
            const bool inside = h >= 0 && h < p.H && w >= 0 && w < p.W;
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    typedef float f32x2_t __attribute__((ext_vector_type(2)));
                    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
                    float rl[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) asm("v_max_f32 %0, %1, 0" : "=v"(rl[k]) : "v"(a1[j][a * 4 + k]));   // (fmaxf: one more instruction)
                    const f32x2_t v0 = {rl[0], rl[1]};
                    const f32x2_t v1 = {rl[2], rl[3]};
                    u32x2 w2v = {__builtin_bit_cast(unsigned int, __builtin_convertvector(v0, bf16x2_t)),
                                 __builtin_bit_cast(unsigned int, __builtin_convertvector(v1, bf16x2_t))};
                    if (!inside) w2v = u32x2{0u, 0u};
                    *reinterpret_cast<u32x2 *>(ys + (j * kYRows + q) * kRowB + a * 16 + khalf * 8) = w2v;
                }
        }
        lds_barrier();    // the whole halo of the first layer's output is in LDS

        // ---- second layer
        f32x16 acc[4][2];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                f32x4 b = {0.f, 0.f, 0.f, 0.f};
                if (p.b2) b = *reinterpret_cast<const f32x4 *>(p.b2 + j * 32 + a * 8 + khalf * 4);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int k = 0; k < 4; ++k) acc[i][j][a * 4 + k] = b[k];
            }
        u32x4 bq[kRing][2];
        auto w2_fragment = [&](int P) __attribute__((always_inline)) {   // step P = 18 chunk + 2 tap + k-group
            const int c = P / 18, s = P % 18, t = s / 2, g = s % 2;
            return p.w2 + (size_t)((t * 4 + 2 * c + g) * kC) * 32;
        };
        pair_for_each([&](auto ic) {
            constexpr int P = decltype(ic)::value;
#pragma unroll
            for (int j = 0; j < 2; ++j) bq[P % kRing][j] = *reinterpret_cast<const u32x4 *>(w2_fragment(P) + voff[j]);
        }, std::make_integer_sequence<int, kAhead>{});
        u32x4 af[2][4];
#pragma unroll
        for (int i = 0; i < 4; ++i) af[0][i] = *reinterpret_cast<const u32x4 *>(ys + arow[i]);
        pair_for_each([&](auto ic) {
            constexpr int P = decltype(ic)::value;
            constexpr int PN = P + 1;                    // step whose halo fragments are read during this one
            constexpr int nc = (PN % kSteps) / 18, nt = ((PN % kSteps) % 18) / 2, ng = PN % 2;
            const char *abase = ys + (nc * kYRows + (nt / 3) * kYC + nt % 3) * kRowB + ng * 32;
            const u32x4 b0 = bq[P % kRing][0], b1 = bq[P % kRing][1];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bf16x8 a = __builtin_bit_cast(bf16x8, af[P & 1][i]);
                acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, b0), a, acc[i][0], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (PN < kSteps) af[PN & 1][i] = *reinterpret_cast<const u32x4 *>(abase + arow[i]);
                __builtin_amdgcn_sched_barrier(0);
                acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, b1), a, acc[i][1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (i < 2 && P + kAhead < kSteps)
                    bq[(P + kAhead) % kRing][i] = *reinterpret_cast<const u32x4 *>(w2_fragment(P + kAhead) + voff[i]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }, std::make_integer_sequence<int, kSteps>{});
        lds_barrier();    // every wave is done with the halo: its memory now holds the staging blocks

        // ---- epilogue, two patch rows at a time through this wave's block
        char *stage = ys + wv * (64 * kStageRow);
        T *yout = reinterpret_cast<T *>(p.y);
        T *pout = reinterpret_cast<T *>(p.pool);
        const int seg = lane & 7, rowq = lane >> 3;
#pragma unroll
        for (int pair = 0; pair < 2; ++pair) {
            const int hrow = h0 + wv * 4 + pair * 2;      // first of the two image rows
            if (yout) {
#pragma unroll
                for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int a = 0; a < 4; ++a) {
                            const f32x16 &t = acc[pair * 2 + ii][j];
                            store4(reinterpret_cast<T *>(stage + (ii * 32 + r) * kStageRow) + j * 32 + a * 8 + khalf * 4,
                                   fmaxf(t[a * 4], 0.f), fmaxf(t[a * 4 + 1], 0.f), fmaxf(t[a * 4 + 2], 0.f), fmaxf(t[a * 4 + 3], 0.f));
                        }
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int row = rowq + 8 * q;         // 0..63: patch row row / 32, column row % 32
                    const u32x4 v = *reinterpret_cast<const u32x4 *>(stage + row * kStageRow + seg * 16);
                    const size_t px = ((size_t)n * p.H + hrow + (row >> 5)) * p.W + w0 + (row & 31);
                    *reinterpret_cast<u32x4 *>(yout + px * kC + seg * 8) = v;
                }
            }
            if (pout) {
                // window = rows 2 pair, 2 pair + 1 (two accumulator blocks) x pixels r, r ^ 1 (neighbouring lanes)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        float m[4];
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            // max(row 0, row 1, 0), then the maximum with the neighbouring lane's: two instructions
                            // (fmaxf would first quieten signalling NaNs, one more instruction per operand)
                            float v;
                            asm("v_max3_f32 %0, %1, %2, 0" : "=v"(v) : "v"(acc[pair * 2][j][a * 4 + k]), "v"(acc[pair * 2 + 1][j][a * 4 + k]));
                            asm("v_max_f32_dpp %0, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf" : "=&v"(m[k]) : "v"(v));
                        }
                        // (both lanes of a pair hold the result; the even one stores it: pooled pixel r / 2)
                        if ((r & 1) == 0)
                            store4(reinterpret_cast<T *>(stage + (r >> 1) * kStageRow) + j * 32 + a * 8 + khalf * 4, m[0], m[1], m[2], m[3]);
                    }
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int pw = rowq + 8 * u;          // 16 pooled pixels x 8 segments of 16 bytes
                    const u32x4 v = *reinterpret_cast<const u32x4 *>(stage + pw * kStageRow + seg * 16);
                    const size_t px = ((size_t)n * (p.H >> 1) + (hrow >> 1)) * (p.W >> 1) + (w0 >> 1) + pw;
                    *reinterpret_cast<u32x4 *>(pout + px * kC + seg * 8) = v;
                }
            }
        }
    }
}

}  // namespace

bool conv_first_pair_ok(int dtype, int H, int W)
{
    return dtype == VGG_BF16 && H % kTH == 0 && W % kTW == 0;
}

// x NCHW fp32 [N][3][H][W]; w1 packed [9][64][CinP1], w2 packed [9][64][64] (bf16, the layout the convolutions
// read); y NHWC [N][H][W][64] and/or pool [N][H/2][W/2][64] (bf16, either may be null).
int conv_first_pair(int N, int H, int W, int CinP1, const float *x, const void *w1, const float *b1, const void *w2,
                    const float *b2, void *y, void *pool, hipStream_t stream)
{
    if (!conv_first_pair_ok(VGG_BF16, H, W)) return VGG_ERR_UNSUPPORTED;
    PairArgs a;
    a.x = x; a.w1 = static_cast<const char *>(w1); a.b1 = b1; a.w2 = static_cast<const char *>(w2); a.b2 = b2;
    a.y = static_cast<char *>(y); a.pool = static_cast<char *>(pool);
    a.N = N; a.H = H; a.W = W; a.CinP1 = CinP1;
    a.tiles_w = W / kTW;
    a.tiles_hw = a.tiles_w * (H / kTH);
    a.ntiles = N * a.tiles_hw;
    a.dTilesW = make_fast_div(a.tiles_w); a.dTilesHW = make_fast_div(a.tiles_hw);
    const size_t lds = kYBytes + kXBytes;
    if (!raise_lds_limit(reinterpret_cast<const void *>(conv_pair_kernel))) return VGG_ERR_LAUNCH;
    const dim3 grid((unsigned)(a.ntiles < 256 ? a.ntiles : 256));
    hipLaunchKernelGGL(conv_pair_kernel, grid, dim3(256), lds, stream, a);
    return launch_status();
}

}  // namespace vgg
