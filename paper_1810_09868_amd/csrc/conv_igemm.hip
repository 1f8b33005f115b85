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
// Every LDS row holds 64 bytes of one pixel's channels (16 fp32 or 32 bf16).
// Two row layouts keep the 16-byte fragment reads of consecutive rows on
// distinct banks: rows padded to 80 bytes (the register-staged kernel below,
// and the halo of the 8-wave direct-to-LDS kernel with up to 384 halo rows),
// or unpadded 64-byte rows whose 16-byte segments are XOR-swizzled with the
// row number (all weight rows of the direct-to-LDS kernels, and the halo of
// their other variants).  A lane reads 16 bytes of A and of B at the same
// (k-group, k-half) position: for bf16 that is the 8-element operand of one
// v_mfma_f32_32x32x16_bf16; for fp32 the four elements feed four
// v_mfma_f32_32x32x2_f32 (any fixed pairing of k indices between A and B is a
// valid contraction order).
#include "common.h"

#include <type_traits>
#include <utility>

namespace vgg {

constexpr int kRowBytes = 80;  // 64 data + 16 pad
constexpr int kDataBytes = 64;
constexpr int kEpiRow = 144;              // epilogue transpose: 128 data bytes + 16 pad per row
constexpr int kEpiBytes = 32 * kEpiRow;   // per wave
constexpr int kMaxAHaloSegsPerBlock = 1536;  // 16-byte halo segments (384 rows) prefetched through registers
constexpr int kDmaHaloRows = 384;            // halo rows of the direct-to-LDS kernel: 2 workgroups of 74 KB per CU
constexpr int kDmaHaloRowsBig = 448;         // ... and of its variant for tiles that straddle images (78 KB)
constexpr int kDmaHaloRowsHalf = 192;        // ... and of the 128-pixel tiles (38 KB: four workgroups per CU)

struct ConvArgs {
    const char *x;      // [M][CinP] elements of T
    const char *w;      // [9][Cout][CinP]
    const float *bias;  // [Cout] or null
    const char *mask;   // [M][Cout] of T or null: output multiplied by (mask > 0)
    char *y;            // [M][Cout], or null when only the pooled tensor is wanted
    char *pool;         // [N][H/2][W/2][Cout] or null: 2x2 max of the result (patch tiles only)
    int CinP, Cout;
    int relu;
    int tiles_n;        // number of column tiles
    int rowsA;          // LDS rows reserved for the halo
    unsigned char *argmax;  // with pool, optional: [N][H/2][W/2][Cout], 2*dh+dw of the first maximum of each window
    float *part;        // [ksplit][M][Cout] partial sums when the contraction is split over workgroups, else null
    int ksplit;         // workgroups per tile (>= 1)
    int kchunks;        // channel chunks per workgroup
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

// The MFMAs are issued with the weight fragment as the first operand, so a 32x32 accumulator holds
// the tile transposed: register e of lane l is channel 8*(e/4) + 4*(l/32) + e%4 of pixel row l%32,
// i.e. a lane owns runs of four consecutive channels of one pixel.
//
// Accumulators start at the bias, so the epilogue has no bias to fetch or add.  init_acc only
// requests the values (into the first pixel block's registers).
template <int BN, int WN, int TM, int TN>
__device__ __forceinline__ void init_acc(f32x16 (&acc)[TM][TN], const ConvArgs &p, int n0, int wn, int khalf)
{
    // (channels past Cout are never stored: their loads are clamped into range instead of skipped;
    // one uniform branch around straight-line loads, so that none of them waits for another)
    const int c0 = n0 + wn * (BN / WN) + khalf * 4;
    if (!p.bias || p.part) {   // (split contraction: the finishing kernel adds the bias)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[0][j][e] = 0.f;
    } else if ((p.Cout & 3) == 0) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const f32x4 b = *reinterpret_cast<const f32x4 *>(p.bias + min(c0 + j * 32 + a * 8, p.Cout - 4));
#pragma unroll
                for (int k = 0; k < 4; ++k) acc[0][j][a * 4 + k] = b[k];
            }
    } else {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                acc[0][j][e] = p.bias[min(c0 + j * 32 + (e >> 2) * 8 + (e & 3), p.Cout - 1)];
    }
}
// Second half, called once the loads above have had time to land: the other pixel blocks start
// from the same values.
template <int TM, int TN>
__device__ __forceinline__ void spread_acc(f32x16 (&acc)[TM][TN])
{
#pragma unroll
    for (int i = 1; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = acc[0][j];
}

// Epilogue of a workgroup that holds only part of the contraction: raw fp32 sums to the partial
// buffer of its split (a lane owns runs of four consecutive channels of one pixel: 16-byte stores).
template <int BM, int BN, int WM, int WN>
__device__ __forceinline__ void conv_partial_epilogue(f32x16 (&acc)[BM / WM / 32][BN / WN / 32], const ConvArgs &p,
                                                      const TileOrigin &org, int n0, int split)
{
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int wm = wv % WM, wn = wv / WM;
    const int r = lane & 31, khalf = lane >> 5;
    float *part = p.part + (size_t)split * p.g.M * p.Cout;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = tile_pixel(p.g, org, wm * (BM / WM) + i * 32 + r);
        if (m < 0) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int col = n0 + wn * (BN / WN) + j * 32 + a * 8 + khalf * 4;
                if (col < p.Cout) {   // Cout is a multiple of 4 when the contraction is split
                    const f32x4 v = {acc[i][j][a * 4], acc[i][j][a * 4 + 1], acc[i][j][a * 4 + 2], acc[i][j][a * 4 + 3]};
                    *reinterpret_cast<f32x4 *>(part + (size_t)m * p.Cout + col) = v;
                }
            }
    }
}

// Epilogue shared by the kernels below; called by every thread of the workgroup once all MFMAs are
// issued.  smem is the start of the workgroup's dynamic LDS, which is reused here.  How the accumulators
// are spread over lanes and registers is the caller's business: stage(i, j0, epi, lo) writes pixel block i
// (32 tile rows) x the 128 bytes of columns that start at MFMA column tile j0 of the wave into the wave's
// staging block (row r at epi + r * kEpiRow), each value raised to at least lo; each_element(f) calls
// f(tile row, column within the wave's 64- or 128-column range, value) for everything the lane holds.
template <typename T, int BM, int BN, int WM, int WN, typename Stage, typename EachElement>
__device__ __forceinline__ void conv_epilogue_impl(Stage stage, EachElement each_element, const ConvArgs &p,
                                                   const TileOrigin &org, char *smem, int n0)
{
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int wm = wv % WM, wn = wv / WM;
    // Epilogue: ReLU, optional (mask > 0) factor, convert, store (the bias is already in the sums).
    // A lane owns four-channel runs of one pixel (see init_acc).  Each wave passes 32 pixels x 128
    // bytes at a time through a private LDS block so that every lane then stores 16 contiguous bytes.
    T *y = reinterpret_cast<T *>(p.y);
    const T *mask = reinterpret_cast<const T *>(p.mask);
    constexpr int VEC = 16 / (int)sizeof(T);        // elements per 16-byte store
    constexpr int CPT = 128 / (int)sizeof(T);       // columns per transposed pass (64 bf16 / 32 fp32)
    constexpr int TJ = CPT / 32;                    // MFMA column tiles per pass
    static_assert(TN % TJ == 0, "wave tile must hold whole passes");
    __syncthreads();  // staging data no longer needed: LDS is reused
    if (p.Cout % VEC == 0) {
        char *epi = smem + wv * kEpiBytes;
        const int seg = lane & 7, rowq = lane >> 3;
        const float lo = p.relu ? 0.f : -__builtin_inff();
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j0 = 0; j0 < TN; j0 += TJ) {
                stage(i, j0, epi, lo);   // (no ReLU: maximum with -inf, one instruction either way)
                const int colbase = n0 + wn * (BN / WN) + j0 * 32 + seg * VEC;
                if (p.pool) {
                    // Patch tiles: these 32 rows are two patch rows of 16 pixels, i.e. eight whole 2x2
                    // windows; lane = (window, 16-byte segment).  Window (dx) = rows 2dx, 2dx+1, 16+2dx, 17+2dx.
                    const int win = lane >> 3;
                    T best[VEC];
                    unsigned char which[VEC];   // k = 2*dh + dw of the first maximum (replaced only by a strictly greater value)
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const int row = (k >> 1) * kTileW + 2 * win + (k & 1);
                        const u32x4 v = *reinterpret_cast<const u32x4 *>(epi + row * kEpiRow + seg * 16);
                        T ve[VEC];
                        __builtin_memcpy(ve, &v, 16);
#pragma unroll
                        for (int c = 0; c < VEC; ++c)
                            if (k == 0 || Elem<T>::load(ve + c) > Elem<T>::load(best + c)) { best[c] = ve[c]; which[c] = (unsigned char)k; }
                    }
                    const int j = wm * (BM / WM) + i * 32;  // first tile row of this block (even patch row)
                    const int ph = (org.h0 + j / kTileW) >> 1, pw = (org.w0 >> 1) + win;
                    if (2 * ph < p.g.H && 2 * pw < p.g.W && colbase < p.Cout) {
                        u32x4 v;
                        __builtin_memcpy(&v, best, 16);
                        T *po = reinterpret_cast<T *>(p.pool);
                        const size_t at = (((size_t)org.n * (p.g.H >> 1) + ph) * (p.g.W >> 1) + pw) * p.Cout + colbase;
                        *reinterpret_cast<u32x4 *>(po + at) = v;
                        if (p.argmax) __builtin_memcpy(p.argmax + at, which, VEC);
                    }
                }
                if (y == nullptr) continue;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int row = rowq + 8 * q;
                    u32x4 v = *reinterpret_cast<const u32x4 *>(epi + row * kEpiRow + seg * 16);
                    const int m = tile_pixel(p.g, org, wm * (BM / WM) + i * 32 + row);
                    if (m >= 0 && colbase < p.Cout) {
                        const size_t o = (size_t)m * p.Cout + colbase;
                        if (mask) {
                            const u32x4 mk = *reinterpret_cast<const u32x4 *>(mask + o);
                            T ve[VEC], me[VEC];
                            __builtin_memcpy(ve, &v, 16);
                            __builtin_memcpy(me, &mk, 16);
#pragma unroll
                            for (int k = 0; k < VEC; ++k)
                                if (!(Elem<T>::load(me + k) > 0.f)) ve[k] = (T)0;
                            __builtin_memcpy(&v, ve, 16);
                        }
                        *reinterpret_cast<u32x4 *>(y + o) = v;
                    }
                }
            }
        }
        return;
    }
    // channel counts that do not allow 16-byte stores: element-wise
    each_element([&](int row, int c, float v) __attribute__((always_inline)) {
        const int m = tile_pixel(p.g, org, row);
        const int col = n0 + wn * (BN / WN) + c;
        if (m >= 0 && col < p.Cout) {
            if (p.relu) v = fmaxf(v, 0.f);
            const size_t o = (size_t)m * p.Cout + col;
            if (mask && !(Elem<T>::load(mask + o) > 0.f)) v = 0.f;
            Elem<T>::store(y + o, v);
        }
    });
}

// ... for 32x32 accumulators (see init_acc for their layout)
template <typename T, int BM, int BN, int WM, int WN>
__device__ __forceinline__ void conv_epilogue(f32x16 (&acc)[BM / WM / 32][BN / WN / 32], const ConvArgs &p,
                                              const TileOrigin &org, char *smem, int n0)
{
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int TJ = 128 / (int)sizeof(T) / 32;   // MFMA column tiles per staged pass
    const int lane = threadIdx.x & 63, wm = (threadIdx.x >> 6) % WM;
    const int r = lane & 31, khalf = lane >> 5;
    conv_epilogue_impl<T, BM, BN, WM, WN>(
        [&](int i, int j0, char *epi, float lo) __attribute__((always_inline)) {
#pragma unroll
            for (int jj = 0; jj < TJ; ++jj)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const f32x16 &t = acc[i][j0 + jj];
                    store4(reinterpret_cast<T *>(epi + r * kEpiRow) + jj * 32 + a * 8 + khalf * 4, fmaxf(t[a * 4], lo),
                           fmaxf(t[a * 4 + 1], lo), fmaxf(t[a * 4 + 2], lo), fmaxf(t[a * 4 + 3], lo));
                }
        },
        [&](auto f) __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        f(wm * (BM / WM) + i * 32 + r, j * 32 + (e >> 2) * 8 + khalf * 4 + (e & 3), acc[i][j][e]);
        },
        p, org, smem, n0);
}

template <typename T, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM *WN * 64, WM *WN == 8 ? 4 : 2) void conv3x3_igemm_kernel(ConvArgs p)
{
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32;  // 32x32 MFMA tiles per wave along pixels
    constexpr int TN = BN / WN / 32;  // and along channels
    constexpr int KC = kDataBytes / (int)sizeof(T);

    extern __shared__ __align__(16) char smem[];
    const int S = p.g.S;
    const int SA = p.rowsA;                     // rows reserved for the halo (>= S)
    int *pix = reinterpret_cast<int *>(smem);   // [SA] halo row -> input pixel or -1
    char *As = smem + round_up16(SA * 4);              // [SA][80]
    char *Bs = As + (size_t)SA * kRowBytes;            // [3][BN][80]

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
    init_acc<BN, WN>(acc, p, n0, wn, khalf);

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
    auto store_a = [&](const u32x4(&areg)[MAXA], char *As) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < MAXA; ++j) {
            const int idx = tid + j * NT;
            *reinterpret_cast<u32x4 *>(As + (idx >> 2) * kRowBytes + (idx & 3) * 16) = areg[j];
        }
    };
    auto copy_a_direct = [&](int c0, char *As) __attribute__((always_inline)) {  // halo too large for the register path
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
            breg[j] = *reinterpret_cast<const u32x4 *>(p.w + packed_w_segment<T>(kh * 3 + kw, n, c0, idx & 3, p.Cout, p.CinP));
        }
    };
    auto store_b = [&](const u32x4(&breg)[NB], char *Bs) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int idx = tid + j * NT;
            *reinterpret_cast<u32x4 *>(Bs + (idx >> 2) * kRowBytes + (idx & 3) * 16) = breg[j];
        }
    };

    u32x4 areg[MAXA], breg[NB];
    __syncthreads();  // halo table ready
    if (a_regs) { load_a(0, areg); store_a(areg, As); } else copy_a_direct(0, As);
    load_b(0, 0, breg);
    store_b(breg, Bs);
    __syncthreads();
    spread_acc(acc);

    auto compute = [&](int kh, const char *As, const char *Bs) __attribute__((always_inline)) {
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
                    for (int j = 0; j < TN; ++j) Mma<T>::run(acc[i][j], bf[j], af[i]);
            }
        }
    };

    // Software pipeline: the global loads of stage s+1 are issued before the MFMAs of stage s and
    // land in LDS after them (two barriers per stage), so their latency is covered by the arithmetic.
    int kh = 0, c0 = 0;
    for (int s = 0; s + 1 < nstages; ++s) {
        int nkh = kh + 1, nc0 = c0;
        if (nkh == 3) { nkh = 0; nc0 += KC; }
        const bool new_chunk = nkh == 0;
        load_b(nc0, nkh, breg);
        if (new_chunk && a_regs) load_a(nc0, areg);
        compute(kh, As, Bs);
        __syncthreads();  // every wave is done reading this stage's LDS data
        store_b(breg, Bs);
        if (new_chunk) {
            if (a_regs) store_a(areg, As); else copy_a_direct(nc0, As);
        }
        __syncthreads();
        kh = nkh; c0 = nc0;
    }
    compute(kh, As, Bs);

    conv_epilogue<T, BM, BN, WM, WN>(acc, p, org, smem, n0);
}

// ---------------------------------------------------------------------------
// Variant with direct-to-LDS weight loads.  Weight rows in LDS are 64 bytes
// without padding; the 16-byte segment s of row q lives at segment
// s ^ ((q >> 2) & 3), which keeps the fragment reads of 16 consecutive rows on
// distinct banks (halo rows likewise, or padded to 80 bytes where LDS allows).
// The weights of a stage are copied by global_load_lds_dwordx4 (lane l of a
// wave writes bytes [16 l, 16 l + 16) of a 1 KB block, so each lane fetches the
// segment that belongs at its position) into one of two buffers while the
// MFMAs of the previous stage run: no registers, no ds_write, one barrier per
// stage.  The kernel waits for these loads itself (s_waitcnt vmcnt(0) before
// the barrier that publishes a buffer).  The halo still goes through registers once per channel chunk.
// ---------------------------------------------------------------------------
__device__ __forceinline__ int swz(int row) { return (row >> 2) & 3; }

template <typename T, int BM, int BN, int WM, int WN, int SA>
// (the second launch bound is the minimum number of waves per SIMD: two 8-wave or three 4-wave workgroups per CU)
__global__ __launch_bounds__(WM *WN * 64, WM *WN == 8 ? 4 : 3) void conv3x3_igemm_dma_kernel(ConvArgs p)
{
    constexpr int NT = WM * WN * 64, NW = WM * WN;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int KC = kDataBytes / (int)sizeof(T);
    // SA: halo rows reserved in LDS (host guarantees S <= SA)
    constexpr int SEGS = SA * 4;                    // 16-byte halo segments per chunk
    constexpr int MAXA = (SEGS + NT - 1) / NT;      // of which each thread copies at most MAXA
    constexpr int b_bytes = 3 * BN * kDataBytes;
    // Halo rows of the 8-wave kernel with the smaller halo are padded to 80 bytes instead of swizzled:
    // conflict-free as well, and linear, so every tap of a fragment read is the same per-lane
    // address plus an immediate offset (the other variants have no LDS left for the padding).
    constexpr bool APAD = SA == kDmaHaloRows && NW == 8;
    constexpr int AROW = APAD ? kRowBytes : kDataBytes;
    constexpr int NB = 3 * BN / 16 / NW;            // 1 KB blocks of a weight stage per wave
    static_assert(3 * BN % (16 * NW) == 0 && BN % 16 == 0, "weight stage must split into whole 1 KB blocks");

    extern __shared__ __align__(16) char smem[];
    const int S = p.g.S;
    int *pix = reinterpret_cast<int *>(smem);       // [SA]
    char *As = smem + SA * 4;                        // [SA][64]
    char *Bs = As + SA * AROW;                       // [2][3*BN][64]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = tid >> 6;
    const int wm = wv % WM, wn = wv / WM;
    const int r = lane & 31, khalf = lane >> 5;
    // Workgroup b runs on XCD b % 8 and every XCD has its own L2.  Renumber so that each XCD works
    // through one contiguous range of (pixel tile, column tile) pairs: the column tiles of a pixel
    // tile then share the halo, and neighbouring pixel tiles their overlap, in one L2.
    const int nblk = gridDim.x, xcd = blockIdx.x & 7;
    const int bid = xcd * (nblk >> 3) + min(xcd, nblk & 7) + (blockIdx.x >> 3);
    // (split contraction: the ksplit workgroups of a tile are neighbours)
    const int split = bid % p.ksplit, tile = bid / p.ksplit;
    const int tile_n = tile % p.tiles_n;
    const int tile_m = tile / p.tiles_n;
    const int c_first = split * p.kchunks * KC;                    // this workgroup's channel range
    const int c_end = min(c_first + p.kchunks * KC, p.CinP);
    const int n0 = tile_n * BN;
    const TileOrigin org = tile_origin(p.g, tile_m);
    const int pitch = p.g.pitch;

    // This lane's part of the weight stage (c0, kh): NB blocks of 16 rows x 64 bytes.  The per-lane
    // byte offsets inside a kernel row's weights never change; the stage only moves a scalar base.
    unsigned woff[NB];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
        const int row = (wv * NB + q) * 16 + (lane >> 2);   // kw*BN + n
        const int kw = row / BN;
        const int n = min(n0 + row - kw * BN, p.Cout - 1);  // columns past Cout are never stored
        // (offset of this lane's source segment from that of tap (kh, 0), row 0, column c0, segment 0)
        woff[q] = (unsigned)(packed_w_segment<T>(kw, n, 0, (lane & 3) ^ swz(row), p.Cout, p.CinP));
    }
    const unsigned bs_lds = __builtin_amdgcn_readfirstlane(
        (unsigned)(uintptr_t)(__attribute__((address_space(3))) char *)(Bs + wv * NB * 1024));
    auto dma_b = [&](int c0, int kh, int buf) __attribute__((always_inline)) {
        const char *base = p.w + packed_w_segment<T>(kh * 3, 0, c0, 0, p.Cout, p.CinP);
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            // Issued as inline assembly on purpose: the compiler cannot tell that this write and the
            // fragment reads of the other buffer never overlap and would wait for it before every read.
            const unsigned dst = bs_lds + buf * b_bytes + q * 1024;
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(dst), "v"(woff[q]), "s"(base) : "m0", "memory");
        }
    };
    dma_b(c_first, 0, 0);  // first: its latency covers the index arithmetic below

    for (int i = tid; i < SA; i += NT) pix[i] = i < S ? halo_pixel(p.g, org, i) : -1;

    int arow[TM];   // halo row of tap (0,0) of this lane's pixels; padded layout: its byte address
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int m;
        tile_row(p.g, org, wm * (BM / WM) + i * 32 + r, m, arow[i]);
        if (APAD) arow[i] = arow[i] * AROW + khalf * 16;
    }
    int baddr[2][TN];  // per k-group; tap kw adds kw*BN*64
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int row = wn * (BN / WN) + j * 32 + r;
        baddr[0][j] = row * kDataBytes + ((khalf ^ swz(row)) << 4);
        baddr[1][j] = baddr[0][j] ^ 32;
    }

    f32x16 acc[TM][TN];
    init_acc<BN, WN>(acc, p, n0, wn, khalf);

    const size_t xrow = (size_t)p.CinP * sizeof(T);
    // Input pixel (or -1 for a pad row) behind each of this thread's halo segments; global, not
    // generic, loads so that they neither touch the LDS counters nor look like LDS accesses.
    typedef const __attribute__((address_space(1))) u32x4 *gvec_t;
    __syncthreads();  // halo table ready
    auto load_a = [&](int c0, u32x4(&areg)[MAXA]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < MAXA; ++j) {
            const int idx = min(tid + j * NT, SEGS - 1);
            const int px = pix[idx >> 2];  // read again for every chunk: cheaper than MAXA registers held across the loop
            const gvec_t src = px < 0 ? (gvec_t)kZeroRow : (gvec_t)(p.x + (size_t)px * xrow + (size_t)c0 * sizeof(T));
            areg[j] = src[idx & 3];
        }
    };
    auto store_a = [&](const u32x4(&areg)[MAXA]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < MAXA; ++j) {
            const int idx = tid + j * NT;
            const int row = idx >> 2;
            if ((j + 1) * NT <= SEGS || idx < SEGS)
                *reinterpret_cast<u32x4 *>(As + row * AROW + (APAD ? (idx & 3) << 4 : ((idx & 3) ^ swz(row)) << 4)) = areg[j];
        }
    };
    auto compute = [&](int kh, const char *Bt) __attribute__((always_inline)) {
        const char *arow_kh[TM];  // padded layout: this stage's kernel row, once per stage
        if (APAD) {
#pragma unroll
            for (int i = 0; i < TM; ++i) arow_kh[i] = As + arow[i] + kh * pitch * AROW;
        }
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
            int aaddr[TM];
            if (!APAD) {
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const int row = arow[i] + kh * pitch + kw;
                    aaddr[i] = row * kDataBytes + ((khalf ^ swz(row)) << 4);
                }
            }
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                uint4 af[TM], bf[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    af[i] = APAD ? *reinterpret_cast<const uint4 *>(arow_kh[i] + kw * AROW + g * 32)
                                 : *reinterpret_cast<const uint4 *>(As + (aaddr[i] ^ (g * 32)));
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    bf[j] = *reinterpret_cast<const uint4 *>(Bt + kw * BN * kDataBytes + baddr[g][j]);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) Mma<T>::run(acc[i][j], bf[j], af[i]);
            }
        }
    };

    u32x4 areg[MAXA];
    load_a(c_first, areg);
    store_a(areg);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the direct-to-LDS loads have landed
    __syncthreads();
    spread_acc(acc);

    // Software pipeline over the stages.  Weight copies for the next stage go to the buffer that was
    // last read two stages ago; the next chunk's halo is requested at the first stage of a chunk and
    // stored to LDS after its last.
    const int nstages = ((c_end - c_first) / KC) * 3;
    int kh = 0, c0 = c_first, bb = 0;
    for (int s = 0; s + 1 < nstages; ++s) {
        int nkh = kh + 1, nc0 = c0;
        if (nkh == 3) { nkh = 0; nc0 += KC; }
        dma_b(nc0, nkh, bb ^ 1);
        if (kh == 0 && c0 + KC < c_end) load_a(c0 + KC, areg);
        compute(kh, Bs + bb * b_bytes);
        if (nkh == 0) {
            __syncthreads();  // every wave is done reading the halo of this chunk
            store_a(areg);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the weight copies have landed
        __syncthreads();
        kh = nkh; c0 = nc0; bb ^= 1;
    }
    compute(kh, Bs + bb * b_bytes);

    if (p.part) conv_partial_epilogue<BM, BN, WM, WN>(acc, p, org, n0, split);
    else conv_epilogue<T, BM, BN, WM, WN>(acc, p, org, smem, n0);
}

// ---------------------------------------------------------------------------
// bf16 variant with the weight fragments in registers.  The blocked weight layout (packed_w_index)
// keeps the 16 contraction indices of a block contiguous per output channel (32 bytes), so a wave loads
// its weight fragments straight from global memory (L2), two taps ahead, into a small ring of
// registers; LDS holds only the input halo.  Compared with the kernel above this removes the weights
// from LDS traffic (half the fragment reads), the per-stage weight copies and their barrier: one
// barrier per 32-channel chunk, i.e. per 288 MFMAs of a wave.
//
// MFMA shape: v_mfma_f32_16x16x32_bf16, each contracting all 32 channels of a chunk.  It does half the
// accumulator traffic per multiply-add of the 32x32x16 shape, and under the power that the operand values
// of this workload draw the chip sustains it at a higher rate (bare loops on random operands: 2.0 against
// 1.87 PFLOP/s; this kernel: +4.5 % over the same schedule on 32x32x16).
// Lane 16 g + q of a wave holds, of a pixel-block fragment, channels 8 g .. 8 g + 7 of pixel q (16 bytes of
// the pixel's 64-byte LDS row); of a weight fragment, the same contraction indices of output channel q (16
// bytes of the blocked layout: block 2 chunk + g / 2, half g % 2); of a 16x16 accumulator, channels
// 4 g .. 4 g + 3 of pixel q.
//
// Workgroup: WM x WN waves, each a (32 TM)-pixel x 64-channel sub-tile, i.e. 2 TM pixel blocks x 4 channel
// blocks of 16: TM = 4 (128 accumulator registers) with two workgroups per CU, or TM = 5 with one
// workgroup per CU and twice the registers per wave, for launches whose 256-pixel tiles would number
// between one and two per CU (then the CUs with two need twice as long as those with one: 320-pixel
// tiles give every CU at most one).
// A chunk is nine steps, one per tap; a step is 2 TM halo-fragment reads and 8 TM MFMAs.  The four weight
// fragments of a tap are requested two taps ahead into a ring of three taps; halo fragments one per pixel
// block, LA blocks ahead into a ring of LA + 1.  The halo of a chunk is copied by global_load_lds_dwordx4
// into one of two buffers a whole chunk ahead; rows are 80 bytes (64 data + 16 pad, conflict-free fragment
// reads at addresses that are a per-lane base plus an offset per tap); the copy treats a buffer as
// consecutive 16-byte slots, slot s = row s / 5, segment s % 5, every lane supplying the source address of
// its slot (pad slots and rows outside the image read a block of zeros).  Once the last halo fragment of a
// chunk has been requested (LA blocks before the chunk ends) the workgroup synchronises, reads on from the
// other buffer and copies the halo of the chunk after next into the one it has left.
// Every other instruction of a step is issued right after an MFMA, in its shadow: a wave issues in order,
// and issued as a block before the MFMAs they would leave the matrix pipe idle whenever the SIMD's other
// wave is not multiplying.
// All vector-memory waits are written by hand (the loads are inline assembly), counting the loads and
// copies issued since the one waited for; the schedule is static, so the counts are constants.
// ---------------------------------------------------------------------------
constexpr int kWregHaloRows = 384;      // halo rows of the weights-in-registers kernel (64 KB of LDS) ...
constexpr int kWregHaloRowsBig = 448;   // ... and of its variant for tiles that straddle images (72 KB)
__device__ const u32x4 kZeroBlock[128] = {};   // 2 KB of zeros: a halo slot outside the image walks through it chunk by chunk

template <typename F, int... S>
__device__ __forceinline__ void for_each_step(F &&f, std::integer_sequence<int, S...>)
{
    (f(std::integral_constant<int, S>{}), ...);
}

typedef float f32x4v __attribute__((ext_vector_type(4)));

template <int WM, int WN, int SA, int TM, int OCC>
__global__ __launch_bounds__(WM *WN * 64, OCC) void conv3x3_igemm_wreg_kernel(ConvArgs p)
{
    typedef bf16_t T;
    constexpr int NW = WM * WN, NT = NW * 64, BM = WM * TM * 32, BN = WN * 64;
    constexpr int NI = 2 * TM, NJ = 4;           // 16-pixel and 16-channel blocks per wave
    constexpr int KC = 32;                       // channels per chunk (one 64-byte LDS row)
    constexpr int NQ = (SA * 5 + NT - 1) / NT;   // halo copies per thread and chunk
    constexpr int ABUF = NQ * NT * 16;           // bytes per halo buffer (>= SA * 80)
    constexpr int TAPS = 9, RB = 3;              // taps of weight fragments in registers
    constexpr int LA = NI % 4 == 0 ? 3 : 4, RA = LA + 1;
    static_assert(TAPS % RB == 0 && (TAPS * NI) % RA == 0, "ring positions must repeat every chunk");
    static_assert(NJ <= NI - LA && NQ <= 3 * LA, "weight loads and halo copies share the slots after the MFMAs");

    extern __shared__ __align__(16) char smem[];   // [2][ABUF]
    const int tid = threadIdx.x;
    const int lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wv % WM, wn = wv / WM;
    const int q = lane & 15, g = lane >> 4;
    // (XCD-aware numbering as in the kernels above)
    const int nblk = gridDim.x, xcd = blockIdx.x & 7;
    const int bid = xcd * (nblk >> 3) + min(xcd, nblk & 7) + (blockIdx.x >> 3);
    const int tile_n = bid % p.tiles_n, tile_m = bid / p.tiles_n;
    const int n0 = tile_n * BN;
    const TileOrigin org = tile_origin(p.g, tile_m);
    const int pitch = p.g.pitch;
    const int nchunks = p.CinP / KC;
    const size_t xrow = (size_t)p.CinP * sizeof(T);

    // source of each of this lane's halo slots (chunk 0)
    const char *asrc[NQ];
#pragma unroll
    for (int k = 0; k < NQ; ++k) {
        const int slot = (k * NW + wv) * 64 + lane;
        const int row = slot / 5, seg = slot - row * 5;
        const int px = (row < p.g.S && seg < 4) ? halo_pixel(p.g, org, row) : -1;
        asrc[k] = px < 0 ? reinterpret_cast<const char *>(kZeroBlock) : p.x + (size_t)px * xrow + seg * 16;
    }
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char *)smem;
    auto copy_slot = [&](int buf, int k) __attribute__((always_inline)) {
        const unsigned dst = __builtin_amdgcn_readfirstlane(lds0 + buf * ABUF + (k * NW + wv) * 1024);
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(dst), "v"(asrc[k]) : "m0", "memory");
    };
    auto next_chunk = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < NQ; ++k) asrc[k] += KC * sizeof(T);
    };

    // byte address (inside a buffer) of tap (0,0) of this lane's pixels, its 16 bytes of the row included
    int arow[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        int m, hrow;
        tile_row(p.g, org, wm * (TM * 32) + i * 16 + q, m, hrow);
        arow[i] = hrow * kRowBytes + g * 16;
    }

    // weight fragment (tap t, chunk c, channels ch .. ch + 15): lane's 16 bytes at
    // ((t * KB + 2 c + g / 2) * Cout + ch + q) * 32 + (g % 2) * 16
    const int KB = p.CinP / 16;
    unsigned voff[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j)   // channels past Cout are never stored
        voff[j] = (unsigned)min(n0 + wn * 64 + j * 16 + q, p.Cout - 1) * 32u + (g & 1) * 16 + (unsigned)(g >> 1) * p.Cout * 32u;
    u32x4 bq[RB][NJ];
    auto load_w = [&](const char *sb, u32x4(&dst)[NJ]) __attribute__((always_inline)) {
        const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)sb);
        const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)((uintptr_t)sb >> 32));
        const unsigned long long sbase = ((unsigned long long)hi << 32) | lo;
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst[j]) : "v"(voff[j]), "s"(sbase) : "memory");
    };

    // Accumulators start at the bias (requested here into the first pixel block, copied to the others once
    // the loads have had time to land).
    f32x4v acc[NI][NJ];
    {
        const int c0 = n0 + wn * 64 + g * 4;
        if (!p.bias || p.part) {
#pragma unroll
            for (int j = 0; j < NJ; ++j) acc[0][j] = f32x4v{0.f, 0.f, 0.f, 0.f};
        } else if ((p.Cout & 3) == 0) {
#pragma unroll
            for (int j = 0; j < NJ; ++j) acc[0][j] = *reinterpret_cast<const f32x4v *>(p.bias + min(c0 + j * 16, p.Cout - 4));
        } else {
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[0][j][e] = p.bias[min(c0 + j * 16 + e, p.Cout - 1)];
        }
    }

    // prologue: the first two halo chunks and the weights of the first two taps
#pragma unroll
    for (int k = 0; k < NQ; ++k) copy_slot(0, k);
    if (nchunks > 1) {
        next_chunk();
#pragma unroll
        for (int k = 0; k < NQ; ++k) copy_slot(1, k);
    }
    const long long w_tap = (long long)KB * p.Cout * 32;            // next tap of the same chunk
    const long long w_c = 2ll * p.Cout * 32 - 8 * w_tap;            // last tap -> first tap of the next chunk
    const long long w_same = -8 * w_tap;                            // ... of the same chunk again (past the end)
    load_w(p.w, bq[0]);
    load_w(p.w + w_tap, bq[1]);
    const char *wnext = p.w + 2 * w_tap;                            // the fragments requested next: tap 2 of chunk 0
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int i = 1; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = acc[0][j];

    u32x4 af[RA];
#pragma unroll
    for (int f = 0; f < LA; ++f) af[f] = *reinterpret_cast<const u32x4 *>(smem + arow[f]);   // tap 0, pixel blocks 0 .. LA - 1

    for (int c = 0; c < nchunks; ++c) {
        const int ab = c & 1;
        const long long w_wrap = c + 1 < nchunks ? w_c : w_same;
        for_each_step([&](auto ic) {
            constexpr int t = decltype(ic)::value;
            // This tap's four weight fragments were requested during tap t - 2; since then came the four of tap
            // t + 1 and, when the end of a chunk lies in between, its NQ halo copies.
            constexpr int younger = NJ + (t < 2 ? NQ : 0);
            u32x4 b0 = bq[t % RB][0], b1 = bq[t % RB][1], b2 = bq[t % RB][2], b3 = bq[t % RB][3];
            asm volatile("s_waitcnt vmcnt(%4)" : "+v"(b0), "+v"(b1), "+v"(b2), "+v"(b3) : "n"(younger));
            const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)wnext);
            const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)((uintptr_t)wnext >> 32));
            const unsigned long long sbase = ((unsigned long long)hi << 32) | lo;
            wnext += (t + 2) % TAPS == TAPS - 1 ? w_wrap : w_tap;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                constexpr int first_next = NI - LA;   // the pixel block during which the first fragment of the next chunk is requested
                if (t == TAPS - 1 && i == first_next) {
                    // Every halo read of this chunk has been issued; the waits at the taps so far have covered
                    // the next chunk's copies, issued a whole chunk ago.  After the barrier the other buffer is
                    // published and this one is free for the chunk after next.
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    __builtin_amdgcn_s_barrier();
                    if (c + 2 < nchunks) next_chunk();   // (past the end: the last chunk again, never read; keeps the wait counts static)
                }
                const int f = t * NI + i;             // position in the chunk's sequence of halo fragments
                const int fr = (f + LA) % (TAPS * NI), nt = fr / NI, ni = fr % NI;
                const int nbuf = f + LA < TAPS * NI ? ab : ab ^ 1;
                const char *abase = smem + nbuf * ABUF + ((nt / 3) * pitch + nt % 3) * kRowBytes;
                const bf16x8 a = __builtin_bit_cast(bf16x8, af[f % RA]);
                const bool copying = t == TAPS - 1 && i >= first_next;
                acc[i][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, b0), a, acc[i][0], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                af[(f + LA) % RA] = *reinterpret_cast<const u32x4 *>(abase + arow[ni]);
                __builtin_amdgcn_sched_barrier(0);
                acc[i][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, b1), a, acc[i][1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (i < NJ)
                    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(bq[(t + 2) % RB][i]) : "v"(voff[i]), "s"(sbase) : "memory");
                if (copying && (i - first_next) * 3 < NQ) copy_slot(ab, (i - first_next) * 3);
                __builtin_amdgcn_sched_barrier(0);
                acc[i][2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, b2), a, acc[i][2], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (copying && (i - first_next) * 3 + 1 < NQ) copy_slot(ab, (i - first_next) * 3 + 1);
                __builtin_amdgcn_sched_barrier(0);
                acc[i][3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, b3), a, acc[i][3], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (copying && (i - first_next) * 3 + 2 < NQ) copy_slot(ab, (i - first_next) * 3 + 2);
                __builtin_amdgcn_sched_barrier(0);
            }
        }, std::make_integer_sequence<int, TAPS>{});
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the weight loads and halo copies issued past the end

    const int wrow0 = wm * (TM * 32);
    if (p.pool || p.mask || !p.y || (p.Cout & 7)) {
        conv_epilogue_impl<T, BM, BN, WM, WN>(
            [&](int i, int j0, char *epi, float lo) __attribute__((always_inline)) {
                // (bf16: a pass is all 64 columns of the wave; pixel block i of 32 rows = 16-pixel blocks 2 i, 2 i + 1)
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        const f32x4v &t = acc[2 * i + h][j];
                        store4(reinterpret_cast<T *>(epi + (h * 16 + q) * kEpiRow) + j * 16 + g * 4, fmaxf(t[0], lo), fmaxf(t[1], lo),
                               fmaxf(t[2], lo), fmaxf(t[3], lo));
                    }
            },
            [&](auto fn) __attribute__((always_inline)) {
#pragma unroll
                for (int i = 0; i < NI; ++i)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
#pragma unroll
                        for (int e = 0; e < 4; ++e) fn(wrow0 + i * 16 + q, j * 16 + g * 4 + e, acc[i][j][e]);
            },
            p, org, smem, n0);
        return;
    }
    // Plain store epilogue (no pool, no mask): straight from registers.  A lane holds four consecutive channels
    // of a pixel per accumulator; lanes 16 apart (the next four channels of the same pixel) swap the values of
    // one of two pixel blocks (v_permlane16_swap: the even row of 16 lanes ends up with eight channels of the
    // first block, the odd row with eight channels of the second) and store 16 bytes each.
    {
        const float lo = p.relu ? 0.f : -__builtin_inff();
        T *y = reinterpret_cast<T *>(p.y);
#pragma unroll
        for (int ip = 0; ip < NI / 2; ++ip) {
            const int m = tile_pixel(p.g, org, wrow0 + (2 * ip + (g & 1)) * 16 + q);
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                typedef float f32x2_t __attribute__((ext_vector_type(2)));
                typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
                unsigned x[2][2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const f32x4v &t = acc[2 * ip + h][j];
                    const f32x2_t v0 = {fmaxf(t[0], lo), fmaxf(t[1], lo)};
                    const f32x2_t v1 = {fmaxf(t[2], lo), fmaxf(t[3], lo)};
                    x[h][0] = __builtin_bit_cast(unsigned, __builtin_convertvector(v0, bf16x2_t));
                    x[h][1] = __builtin_bit_cast(unsigned, __builtin_convertvector(v1, bf16x2_t));
                }
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const auto sw = __builtin_amdgcn_permlane16_swap(x[0][k], x[1][k], false, false);
                    x[0][k] = sw[0];
                    x[1][k] = sw[1];
                }
                const u32x4 v = {x[0][0], x[0][1], x[1][0], x[1][1]};
                const int col = n0 + wn * 64 + j * 16 + (g >> 1) * 8;
                if (m >= 0 && col < p.Cout) *reinterpret_cast<u32x4 *>(y + (size_t)m * p.Cout + col) = v;
            }
        }
    }
}

template <int WM, int WN, int SA, int TM = 4, int OCC = 2>
static int launch_conv_wreg(const ConvArgs &a0, const TileGeom &g, hipStream_t stream)
{
    ConvArgs a = a0;
    constexpr int NT = WM * WN * 64, BN = WN * 64;
    constexpr int NQ = (SA * 5 + NT - 1) / NT;
    a.g = g;
    a.tiles_n = (a.Cout + BN - 1) / BN;
    a.rowsA = SA;
    const size_t lds = (size_t)2 * NQ * NT * 16;   // (more than the epilogue's staging blocks)
    auto kern = conv3x3_igemm_wreg_kernel<WM, WN, SA, TM, OCC>;
    if (!raise_lds_limit(reinterpret_cast<const void *>(kern))) return VGG_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)(a.g.ntiles * a.tiles_n)), dim3(NT), lds, stream, a);
    return launch_status();
}

template <typename T, int BM, int BN, int WM, int WN, int SA>
static int launch_conv_dma(const ConvArgs &a0, const TileGeom &g, hipStream_t stream)
{
    ConvArgs a = a0;
    a.g = g;
    a.tiles_n = (a.Cout + BN - 1) / BN;
    a.rowsA = SA;
    const size_t arow_bytes = (SA == kDmaHaloRows && WM * WN == 8) ? kRowBytes : kDataBytes;   // as in the kernel
    size_t lds = (size_t)a.rowsA * 4 + (size_t)a.rowsA * arow_bytes + (size_t)2 * 3 * BN * kDataBytes;
    if (lds < (size_t)WM * WN * kEpiBytes) lds = (size_t)WM * WN * kEpiBytes;
    auto kern = conv3x3_igemm_dma_kernel<T, BM, BN, WM, WN, SA>;
    if (lds > 64 * 1024 && !raise_lds_limit(reinterpret_cast<const void *>(kern))) return VGG_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)(a.g.ntiles * a.tiles_n * a.ksplit)), dim3(WM * WN * 64), lds, stream, a);
    return launch_status();
}

template <typename T, int BM, int BN, int WM, int WN>
static int launch_conv(const ConvArgs &a0, int N, int H, int W, hipStream_t stream)
{
    ConvArgs a = a0;
    a.g = make_tile_geom(N, H, W, BM);
    a.tiles_n = (a.Cout + BN - 1) / BN;
    constexpr int NT = WM * WN * 64;
    a.rowsA = a.g.S * 4 <= kMaxAHaloSegsPerBlock ? kMaxAHaloSegsPerBlock / 4 : a.g.S;
    size_t lds = round_up((size_t)a.rowsA * 4, 16) + (size_t)a.rowsA * kRowBytes + (size_t)3 * BN * kRowBytes;
    if (lds < (size_t)WM * WN * kEpiBytes) lds = (size_t)WM * WN * kEpiBytes;
    if (lds > 160 * 1024) return VGG_ERR_UNSUPPORTED;
    auto kern = conv3x3_igemm_kernel<T, BM, BN, WM, WN>;
    if (lds > 64 * 1024 && !raise_lds_limit(reinterpret_cast<const void *>(kern))) return VGG_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)(a.g.ntiles * a.tiles_n)), dim3(WM * WN * 64), lds, stream, a);
    return launch_status();
}

// Sums the partial results of a split contraction: y = f(bias + sum over splits), f = ReLU and/or the
// (mask > 0) factor, converted to T.  One thread per four channels.
template <typename T>
__global__ __launch_bounds__(256) void conv_split_finish_kernel(const float *__restrict__ part, const float *__restrict__ bias,
                                                                const T *__restrict__ mask, T *__restrict__ y, size_t quads,
                                                                int Cout, int ksplit, int relu)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= quads) return;
    const int col = (int)((i * 4) % (size_t)Cout);
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (bias) s = *reinterpret_cast<const f32x4 *>(bias + col);
    for (int k = 0; k < ksplit; ++k) s += *reinterpret_cast<const f32x4 *>(part + ((size_t)k * quads + i) * 4);
    const float lo = relu ? 0.f : -__builtin_inff();
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        s[e] = fmaxf(s[e], lo);
        if (mask && !(Elem<T>::load(mask + i * 4 + e) > 0.f)) s[e] = 0.f;
    }
    store4(y + i * 4, s[0], s[1], s[2], s[3]);
}

// Which kernel a shape gets, and whether its contraction is split over several workgroups per tile.
struct ConvPlan {
    TileGeom g;
    bool narrow, dma, dma_big, half, wreg, tall;
    int ksplit, kchunks;
};

static ConvPlan conv_plan(int dtype, int N, int H, int W, int CinP, int Cout, bool pool)
{
    ConvPlan c;
    c.narrow = Cout <= 64;
    c.g = make_tile_geom(N, H, W, 256);
    c.dma = c.g.S <= kDmaHaloRows;
    c.dma_big = !c.dma && c.g.S <= kDmaHaloRowsBig;
    // Too few 256x128 tiles to give every CU two workgroups (the 14x14 layers): 64-wide column tiles
    // double the workgroup count and three of them fit on a CU.
    if (c.g.ntiles * ((Cout + 127) / 128) < 512) c.narrow = true;
    // Small batches: fewer tiles than CUs, each walking the whole contraction alone.  Then several
    // workgroups share a tile, each taking a range of channel chunks (at least two), and a second
    // kernel adds their partial sums.
    const int chunks = CinP * dtype_size(dtype) / kDataBytes;
    const int total = c.g.ntiles * ((Cout + (c.narrow ? 63 : 127)) / (c.narrow ? 64 : 128));
    c.ksplit = 1; c.kchunks = chunks;
    // Measured: pays when at most half the CUs would have a workgroup and a tile's contraction is
    // long enough (a bf16 chunk takes a quarter of the time of an fp32 one).
    if ((c.dma || c.dma_big) && !pool && Cout % 4 == 0 && total <= 128 &&
        chunks >= (dtype == VGG_BF16 ? 8 : 4)) {
        int want = (512 + total - 1) / total;   // two workgroups per CU
        if (want > chunks / 2) want = chunks / 2;
        c.kchunks = (chunks + want - 1) / want;
        c.ksplit = (chunks + c.kchunks - 1) / c.kchunks;
    }
    // fp32, 64-wide tiles, a launch of only a few workgroups per CU (the 14x14 layers at batch 100: 616
    // on 768 slots): 128-pixel tiles double the count and even out the load, +15 % there.  (bf16 loses
    // 5 % the same way: its workgroups are short enough that the smaller tile's overhead weighs more.)
    c.half = false;
    if (dtype == VGG_F32 && c.narrow && (c.dma || c.dma_big) && !pool && c.ksplit == 1 && total >= 256 && total < 2048) {
        const TileGeom h = make_tile_geom(N, H, W, 128);
        if (h.S <= kDmaHaloRowsHalf) { c.g = h; c.half = true; }
    }
    // bf16, 128-wide column tiles, whole contraction in one workgroup: the kernel that keeps the weights in
    // registers (its 256-pixel tile and halo are those of the direct-to-LDS kernels, so dma / dma_big decide
    // the halo size here as well)
    c.wreg = dtype == VGG_BF16 && !c.narrow && (c.dma || c.dma_big) && c.ksplit == 1;
    // bf16, a launch that 256-pixel tiles cannot spread evenly (the 14x14 layers at batch 100: 308 tiles of 128
    // channels, so some CUs would get two workgroups and the rest one): 320-pixel tiles, five pixel blocks per
    // wave and one workgroup per CU with all its registers, when that gives every CU at most one tile.
    c.tall = false;
    if (dtype == VGG_BF16 && Cout > 64 && !pool && c.ksplit == 1 && c.g.ntiles * ((Cout + 127) / 128) < 512) {
        const TileGeom t = make_tile_geom(N, H, W, 320);
        const int tiles = t.ntiles * ((Cout + 127) / 128);
        if (t.S <= kWregHaloRowsBig && tiles > 128 && tiles <= 256) {
            c.g = t;
            c.tall = c.wreg = true;
            c.narrow = c.half = false;
            c.dma = t.S <= kWregHaloRows;
            c.dma_big = !c.dma;
        }
    }
    return c;
}

// Bytes of partial sums conv3x3_igemm needs for this shape (0: the contraction is not split).
size_t conv3x3_igemm_workspace(int dtype, int N, int H, int W, int CinP, int Cout)
{
    const ConvPlan c = conv_plan(dtype, N, H, W, CinP, Cout, false);
    return c.ksplit > 1 ? round_up((size_t)c.ksplit * N * H * W * Cout * 4, 256) : 0;
}

// For inspection: {kernel (0 register-staged, 1 / 2 / 3 direct-to-LDS with 384 / 448 / 192 halo rows), pixels per
// tile, channels per tile, tile mode (0 consecutive pixels, 1 patches), pixel tiles, workgroups per tile (split
// contraction), workgroups}.
void conv3x3_igemm_plan_info(int dtype, int N, int H, int W, int CinP, int Cout, bool pool, int info[7])
{
    const ConvPlan c = conv_plan(dtype, N, H, W, CinP, Cout, pool);
    const int bn = c.narrow ? 64 : 128;
    info[0] = c.wreg ? (c.dma ? 4 : 5) + (c.tall ? 2 : 0) : (c.half ? 3 : (c.dma ? 1 : (c.dma_big ? 2 : 0)));
    info[1] = c.g.rows;
    info[2] = bn;
    info[3] = c.g.mode;
    info[4] = c.g.ntiles;
    info[5] = c.ksplit;
    info[6] = c.g.ntiles * ((Cout + bn - 1) / bn) * c.ksplit;
}

bool conv3x3_pool_fusable(int dtype, int H, int W, int Cout)
{
    return H % 16 == 0 && W % kTileW == 0 && Cout % (16 / dtype_size(dtype)) == 0;
}

// x: [N*H*W][CinP], w: [9][Cout][CinP] (elements of dtype); y: [N*H*W][Cout].
// pool (optional): 2x2 max of y, only when conv3x3_pool_fusable(); y may then be null; argmax (optional, with pool).
// part_ws: conv3x3_igemm_workspace() bytes, or null (then the contraction is never split).
int conv3x3_igemm(int dtype, int N, int H, int W, int CinP, int Cout, const void *x, const void *w,
                  const float *bias, const void *mask, void *y, void *pool, unsigned char *argmax, int relu, void *part_ws,
                  hipStream_t stream)
{
    if (pool && !conv3x3_pool_fusable(dtype, H, W, Cout)) return VGG_ERR_UNSUPPORTED;
    ConvPlan c = conv_plan(dtype, N, H, W, CinP, Cout, pool != nullptr);
    if (!part_ws || !y) { c.ksplit = 1; c.kchunks = CinP * dtype_size(dtype) / kDataBytes; }
    ConvArgs a;
    a.x = static_cast<const char *>(x);
    a.w = static_cast<const char *>(w);
    a.bias = bias;
    a.mask = static_cast<const char *>(mask);
    a.y = static_cast<char *>(y);
    a.pool = static_cast<char *>(pool);
    a.argmax = pool ? argmax : nullptr;
    a.CinP = CinP; a.Cout = Cout;
    a.relu = relu; a.tiles_n = 0; a.rowsA = 0;
    a.part = c.ksplit > 1 ? static_cast<float *>(part_ws) : nullptr;
    a.ksplit = c.ksplit; a.kchunks = c.kchunks;
    const bool narrow = c.narrow, dma = c.dma, dma_big = c.dma_big;
    const TileGeom &g = c.g;
    int rc;
    if (dtype == VGG_F32) {
        if (c.half)
            rc = launch_conv_dma<float, 128, 64, 4, 1, kDmaHaloRowsHalf>(a, g, stream);
        else if (dma)
            rc = narrow ? launch_conv_dma<float, 256, 64, 4, 1, kDmaHaloRows>(a, g, stream)
                        : launch_conv_dma<float, 256, 128, 4, 2, kDmaHaloRows>(a, g, stream);
        else if (dma_big)
            rc = narrow ? launch_conv_dma<float, 256, 64, 4, 1, kDmaHaloRowsBig>(a, g, stream)
                        : launch_conv_dma<float, 256, 128, 4, 2, kDmaHaloRowsBig>(a, g, stream);
        else
            rc = narrow ? launch_conv<float, 256, 64, 4, 1>(a, N, H, W, stream)
                        : launch_conv<float, 256, 128, 4, 2>(a, N, H, W, stream);
    } else {
        // (weights in registers)
        if (c.tall)
            rc = dma ? launch_conv_wreg<2, 2, kWregHaloRows, 5, 1>(a, g, stream) : launch_conv_wreg<2, 2, kWregHaloRowsBig, 5, 1>(a, g, stream);
        else if (c.wreg && c.ksplit == 1)
            rc = dma ? launch_conv_wreg<2, 2, kWregHaloRows>(a, g, stream) : launch_conv_wreg<2, 2, kWregHaloRowsBig>(a, g, stream);
        else if (dma)
            rc = narrow ? launch_conv_dma<bf16_t, 256, 64, 4, 1, kDmaHaloRows>(a, g, stream)
                        : launch_conv_dma<bf16_t, 256, 128, 4, 2, kDmaHaloRows>(a, g, stream);
        else if (dma_big)
            rc = narrow ? launch_conv_dma<bf16_t, 256, 64, 4, 1, kDmaHaloRowsBig>(a, g, stream)
                        : launch_conv_dma<bf16_t, 256, 128, 4, 2, kDmaHaloRowsBig>(a, g, stream);
        else
            rc = narrow ? launch_conv<bf16_t, 256, 64, 4, 1>(a, N, H, W, stream)
                        : launch_conv<bf16_t, 256, 128, 4, 2>(a, N, H, W, stream);
    }
    if (rc != VGG_OK || c.ksplit == 1) return rc;
    const size_t quads = (size_t)N * H * W * Cout / 4;
    const dim3 grid((unsigned)((quads + 255) / 256));
    if (dtype == VGG_F32)
        hipLaunchKernelGGL(conv_split_finish_kernel<float>, grid, dim3(256), 0, stream, a.part, bias,
                           static_cast<const float *>(mask), static_cast<float *>(y), quads, Cout, c.ksplit, relu);
    else
        hipLaunchKernelGGL(conv_split_finish_kernel<bf16_t>, grid, dim3(256), 0, stream, a.part, bias,
                           static_cast<const bf16_t *>(mask), static_cast<bf16_t *>(y), quads, Cout, c.ksplit, relu);
    return launch_status();
}

}  // namespace vgg
