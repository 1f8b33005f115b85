// Dense layers on MFMA for gfx950: z = a * W^T + b (the paper's
// dense(W, x, b) = W*x + b, listing "dense", HLO "dot") and its two backward
// products.  At batch ~100 these are weight-streaming problems: every weight
// is read from HBM exactly once and the batch rows are the MFMA's M side.
#include "common.h"

namespace vgg {

constexpr int kFcRow = 80;  // LDS row: 64 data bytes + 16 pad (same fragment format as the convolution)

template <typename T> struct FcMma;
template <> struct FcMma<float> {
    static __device__ __forceinline__ void run(f32x16 &acc, const uint4 &a, const uint4 &b)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
    }
};
template <> struct FcMma<bf16_t> {
    static __device__ __forceinline__ void run(f32x16 &acc, const uint4 &a, const uint4 &b)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                      __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
    }
};

// Four consecutive floats row[c..c+3] with zeros at and beyond column C.  The
// vector path needs the row to be 16-byte aligned (C a multiple of 4).
__device__ __forceinline__ uint4 load_row4(const float *row, int c, int C, bool vec)
{
    if (vec && c + 3 < C) return *reinterpret_cast<const uint4 *>(row + c);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (c < C) v.x = __float_as_uint(row[c]);
    if (c + 1 < C) v.y = __float_as_uint(row[c + 1]);
    if (c + 2 < C) v.z = __float_as_uint(row[c + 2]);
    if (c + 3 < C) v.w = __float_as_uint(row[c + 3]);
    return v;
}

// ------------------------------------------------------------------ forward
// Workgroup: 128 batch rows x 128 outputs x a range of 64-byte K units.
// Wave w owns outputs [32w, 32w+32) and all four 32-row blocks.  The
// activations of a step (4 units = 256 bytes per row) go through LDS; each
// weight fragment is read straight from global memory by the one lane that
// needs it (a weight is used by exactly one wave).
struct FcArgs {
    const char *a;   // [N][In]
    const char *w;   // [Out][In]
    float *part;     // [splits][N][Out]
    int N, In, Out;
    int units;            // 64-byte K units per row: In * sizeof(T) / 64, rounded up
    int units_per_split;
    int tiles_n;          // column tiles
    int tiles_m;          // row tiles
};

// 16 bytes at byte offset `off` of a row of `rowbytes` bytes, zeros at and beyond the row's end.
// vec: rows are 16-byte aligned and a whole number of 16-byte segments (one load); otherwise the
// segment is gathered element by element, so that any row length works.
template <typename T>
__device__ __forceinline__ uint4 load_seg(const char *row, size_t off, size_t rowbytes, bool vec)
{
    uint4 v = make_uint4(0, 0, 0, 0);
    if (vec) {
        if (off < rowbytes) v = *reinterpret_cast<const uint4 *>(row + off);
        return v;
    }
    T e[16 / sizeof(T)];
#pragma unroll
    for (int k = 0; k < (int)(16 / sizeof(T)); ++k)
        e[k] = off + k * sizeof(T) < rowbytes ? reinterpret_cast<const T *>(row + off)[k] : (T)0;
    __builtin_memcpy(&v, e, 16);
    return v;
}

// EXACT: every row is a whole number of 64-byte units (In a multiple of 16 fp32 / 32 bf16), the case
// of the network's own layers.  Otherwise the last unit of a row is completed with zeros in registers.
template <typename T, bool EXACT>
__global__ __launch_bounds__(256) void fc_fwd_kernel(FcArgs p)
{
    __shared__ __align__(16) char As[4 * 128 * kFcRow];  // [unit][row][80]
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = lane & 31, khalf = lane >> 5;
    int b = blockIdx.x;
    const int tn = b % p.tiles_n; b /= p.tiles_n;
    const int tm = b % p.tiles_m; b /= p.tiles_m;
    const int split = b;
    const int row0 = tm * 128, o0 = tn * 128;
    const int u_begin = split * p.units_per_split;
    const int u_end = min(u_begin + p.units_per_split, p.units);
    const size_t rowbytes = (size_t)p.In * sizeof(T);
    const bool vec = EXACT || rowbytes % 16 == 0;

    const int ocol = o0 + wv * 32 + r;
    const bool ook = ocol < p.Out;
    const char *wrow = p.w + (size_t)(ook ? ocol : 0) * rowbytes + khalf * 16;

    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

    // Both operands of a step are requested one step ahead and held in registers, so the weight
    // stream from HBM never pauses for the staging and the MFMAs.  The barriers are issued without
    // the fence of __syncthreads(), which would wait for those loads.
    auto barrier = [] { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    constexpr int NA = 4 * 128 * 4 / 256;   // activation segments per thread and step
    auto load_w = [&](int u0, uint4 (&bf)[4][2]) __attribute__((always_inline)) {
        const int nu = min(4, u_end - u0);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                bf[u][g] = make_uint4(0, 0, 0, 0);
                if (u < nu && ook) {
                    if (EXACT) bf[u][g] = *reinterpret_cast<const uint4 *>(wrow + (size_t)(u0 + u) * 64 + g * 32);
                    else bf[u][g] = load_seg<T>(wrow - khalf * 16, (size_t)(u0 + u) * 64 + g * 32 + khalf * 16, rowbytes, vec);
                }
            }
    };
    auto load_a = [&](int u0, uint4 (&av)[NA]) __attribute__((always_inline)) {
        const int nu = min(4, u_end - u0);
#pragma unroll
        for (int k = 0; k < NA; ++k) {
            const int idx = tid + k * 256;
            const int seg = idx & 3, row = (idx >> 2) & 127, u = idx >> 9;
            av[k] = make_uint4(0, 0, 0, 0);
            if (u < nu && row0 + row < p.N) {
                if (EXACT) av[k] = *reinterpret_cast<const uint4 *>(p.a + (size_t)(row0 + row) * rowbytes + (size_t)(u0 + u) * 64 + seg * 16);
                else av[k] = load_seg<T>(p.a + (size_t)(row0 + row) * rowbytes, (size_t)(u0 + u) * 64 + seg * 16, rowbytes, vec);
            }
        }
    };
    uint4 bf_next[4][2], a_next[NA];
    if (u_begin < u_end) { load_a(u_begin, a_next); load_w(u_begin, bf_next); }
    for (int u0 = u_begin; u0 < u_end; u0 += 4) {
        barrier();  // the previous step's fragment reads are done
#pragma unroll
        for (int k = 0; k < NA; ++k) {
            const int idx = tid + k * 256;
            *reinterpret_cast<uint4 *>(As + ((idx >> 9) * 128 + ((idx >> 2) & 127)) * kFcRow + (idx & 3) * 16) = a_next[k];
        }
        uint4 bf[4][2];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int g = 0; g < 2; ++g) bf[u][g] = bf_next[u][g];
        if (u0 + 4 < u_end) { load_a(u0 + 4, a_next); load_w(u0 + 4, bf_next); }
        barrier();  // the staged activations are visible
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint4 af = *reinterpret_cast<const uint4 *>(As + (u * 128 + i * 32 + r) * kFcRow + g * 32 + khalf * 16);
                    FcMma<T>::run(acc[i], af, bf[u][g]);
                }
    }
    if (ook) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = row0 + i * 32 + (e >> 2) * 8 + khalf * 4 + (e & 3);
                if (row < p.N) p.part[((size_t)split * p.N + row) * p.Out + ocol] = acc[i][e];
            }
    }
}

// z = f(bias + sum over splits), converted to TZ.
template <typename TZ>
__global__ void fc_finish_kernel(const float *__restrict__ part, const float *__restrict__ bias, TZ *__restrict__ z, int N,
                                 int Out, int splits, int relu)
{
    const size_t n = (size_t)N * Out;
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float s = bias ? bias[i % Out] : 0.f;
    for (int k = 0; k < splits; ++k) s += part[(size_t)k * n + i];
    if (relu) s = fmaxf(s, 0.f);
    Elem<TZ>::store(z + i, s);
}

static void fc_plan(int dtype, int N, int In, int Out, FcArgs &a)
{
    a.N = N; a.In = In; a.Out = Out;
    a.units = (In * dtype_size(dtype) + 63) / 64;
    a.tiles_n = (Out + 127) / 128;
    a.tiles_m = (N + 127) / 128;
    const int tiles = a.tiles_n * a.tiles_m;
    int splits = (512 + tiles - 1) / tiles;
    const int max_splits = (a.units + 7) / 8;  // at least two steps per split
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    a.units_per_split = ((a.units + splits - 1) / splits + 3) / 4 * 4;
}

static int fc_splits(const FcArgs &a) { return (a.units + a.units_per_split - 1) / a.units_per_split; }

size_t fc_workspace(int dtype, int N, int In, int Out)
{
    FcArgs a;
    fc_plan(dtype, N, In, Out, a);
    return round_up((size_t)fc_splits(a) * N * Out * 4, 256);
}

int fc_forward(int dtype, int N, int In, int Out, const void *a_, const void *w, const float *bias, void *z, int z_dtype,
               int relu, void *ws, hipStream_t s)
{
    FcArgs a;
    fc_plan(dtype, N, In, Out, a);
    const int splits = fc_splits(a);
    a.a = static_cast<const char *>(a_);
    a.w = static_cast<const char *>(w);
    a.part = static_cast<float *>(ws);
    const dim3 grid((unsigned)(a.tiles_n * a.tiles_m * splits));
    const bool exact = (size_t)In * dtype_size(dtype) % 64 == 0;
    if (dtype == VGG_BF16) {
        if (exact) hipLaunchKernelGGL((fc_fwd_kernel<bf16_t, true>), grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL((fc_fwd_kernel<bf16_t, false>), grid, dim3(256), 0, s, a);
    } else {
        if (exact) hipLaunchKernelGGL((fc_fwd_kernel<float, true>), grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL((fc_fwd_kernel<float, false>), grid, dim3(256), 0, s, a);
    }
    if (hipGetLastError() != hipSuccess) return VGG_ERR_LAUNCH;
    const size_t n = (size_t)N * Out;
    const dim3 g2((unsigned)((n + 255) / 256));
    if (z_dtype == VGG_BF16)
        hipLaunchKernelGGL(fc_finish_kernel<bf16_t>, g2, dim3(256), 0, s, a.part, bias, (bf16_t *)z, N, Out, splits, relu);
    else
        hipLaunchKernelGGL(fc_finish_kernel<float>, g2, dim3(256), 0, s, a.part, bias, (float *)z, N, Out, splits, relu);
    return launch_status();
}

// ------------------------------------------------- backward: dW = dz^T * a
// fp32.  Workgroup: 128 (o) x 128 (i) block of dW; the batch is the
// contraction index, staged through LDS 32 rows at a time.  Wave (wo, wi)
// owns a 64x64 sub-block = 2x2 MFMA tiles.
__global__ __launch_bounds__(256) void fc_dw_kernel(const float *__restrict__ a, const float *__restrict__ dz,
                                                    float *__restrict__ dw, int N, int In, int Out)
{
    constexpr int ROW = 128 * 4 + 16;
    __shared__ __align__(16) char Ds[32 * ROW];
    __shared__ __align__(16) char As[32 * ROW];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = lane & 31, kp = lane >> 5;
    const int wo = wv & 1, wi = wv >> 1;
    const int tiles_i = (In + 127) / 128;
    const int i0 = (blockIdx.x % tiles_i) * 128, o0 = (blockIdx.x / tiles_i) * 128;

    f32x16 acc[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[x][y][e] = 0.f;

    // The 32 batch rows of a step are requested one step ahead; barriers without the fence of
    // __syncthreads(), which would wait for those loads.
    auto barrier = [] { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    uint4 vd[4], va[4];
    auto request = [&](int n0) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int idx = tid + q * 256;
            const int seg = idx & 31, row = idx >> 5;
            vd[q] = make_uint4(0, 0, 0, 0);
            va[q] = make_uint4(0, 0, 0, 0);
            if (n0 + row < N) {
                vd[q] = load_row4(dz + (size_t)(n0 + row) * Out, o0 + seg * 4, Out, (Out & 3) == 0);
                va[q] = load_row4(a + (size_t)(n0 + row) * In, i0 + seg * 4, In, (In & 3) == 0);
            }
        }
    };
    request(0);
    for (int n0 = 0; n0 < N; n0 += 32) {
        barrier();  // the previous step's fragment reads are done
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int idx = tid + q * 256;
            const int seg = idx & 31, row = idx >> 5;
            *reinterpret_cast<uint4 *>(Ds + row * ROW + seg * 16) = vd[q];
            *reinterpret_cast<uint4 *>(As + row * ROW + seg * 16) = va[q];
        }
        barrier();  // the staged rows are visible
        if (n0 + 32 < N) request(n0 + 32);
#pragma unroll 4
        for (int s = 0; s < 16; ++s) {
            const int n = 2 * s + kp;
            float af[2], bf[2];
#pragma unroll
            for (int x = 0; x < 2; ++x) af[x] = *reinterpret_cast<const float *>(Ds + n * ROW + (wo * 64 + x * 32 + r) * 4);
#pragma unroll
            for (int y = 0; y < 2; ++y) bf[y] = *reinterpret_cast<const float *>(As + n * ROW + (wi * 64 + y * 32 + r) * 4);
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y)
                    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[x], bf[y], acc[x][y], 0, 0, 0);
        }
    }
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) {
            const int i = i0 + wi * 64 + y * 32 + r;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int o = o0 + wo * 64 + x * 32 + (e >> 2) * 8 + kp * 4 + (e & 3);
                // (streamed out: 411 MB for the first dense layer, re-read only by the update, long after it has left every cache)
                if (o < Out && i < In) __builtin_nontemporal_store(acc[x][y][e], &dw[(size_t)o * In + i]);
            }
        }
}

// db[o] = sum_n dz[n][o].  A workgroup owns 64 outputs; each of its four waves sums every fourth row and
// the four partial sums are added in a fixed order (one thread per output walking all rows alone was a
// chain of N dependent loads on sixteen CUs: 29 us for 4096 outputs).
__global__ __launch_bounds__(256) void fc_db_kernel(const float *__restrict__ dz, float *__restrict__ db, int N, int Out)
{
    __shared__ float part[4][64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int o = blockIdx.x * 64 + lane;
    float s = 0.f;
    if (o < Out) {
#pragma unroll 4
        for (int n = wv; n < N; n += 4) s += dz[(size_t)n * Out + o];
    }
    part[wv][lane] = s;
    __syncthreads();
    if (wv == 0 && o < Out) db[o] = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
}

// --------------------------------------------------- backward: da = dz * W
// fp32.  Workgroup: 128 batch rows x 256 inputs x a range of outputs (the
// contraction index).  Wave (wr, wc) owns rows [64wr, 64wr+64) and the 128
// inputs [128wc, 128wc+128).  A lane loads four consecutive inputs of one
// weight row with one 16-byte load and feeds them to four different MFMA
// column tiles, so accumulator tile j of lane r holds input 4r+j of the
// wave's 128: the stores are 16-byte vectors as well.
struct FcDaArgs {
    const float *dz;  // [N][Out]
    const float *w;   // [Out][In]
    float *part;      // [splits][N][In]
    int N, In, Out;
    int tiles_i, tiles_m, o_per_split;
};

// VEC: In is a multiple of 4, so a lane's four inputs are one aligned 16-byte load and store; otherwise
// they are read and written one by one, with zeros beyond the row's end.
template <bool VEC>
__global__ __launch_bounds__(256) void fc_da_kernel(FcDaArgs p)
{
    __shared__ __align__(16) char Ds[128 * kFcRow];  // dz rows, 16 outputs per chunk
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = lane & 31, khalf = lane >> 5;
    const int wr = wv & 1, wc = wv >> 1;
    int b = blockIdx.x;
    const int ti = b % p.tiles_i; b /= p.tiles_i;
    const int tm = b % p.tiles_m; b /= p.tiles_m;
    const int split = b;
    const int row0 = tm * 128;
    const int icol = ti * 256 + wc * 128 + 4 * r;  // first of this lane's 4 inputs
    const bool iok = icol < p.In;
    const int o_begin = split * p.o_per_split, o_end = min(o_begin + p.o_per_split, p.Out);

    f32x16 acc[2][4];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[x][j][e] = 0.f;

    // Operands of a chunk of 16 outputs are requested one chunk ahead: the weight stream from HBM never
    // pauses for the staging and the MFMAs.  The barriers are issued without the fence that
    // __syncthreads() carries (it would wait for the loads in flight); they only order LDS accesses.
    auto barrier = [] { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    f32x4 w_next[2][4];
    uint4 dz_next[2];
    auto request = [&](int oc) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int idx = tid + q * 256;
            const int seg = idx & 3, row = idx >> 2;
            dz_next[q] = make_uint4(0, 0, 0, 0);
            if (row0 + row < p.N)
                dz_next[q] = load_row4(p.dz + (size_t)(row0 + row) * p.Out, oc + seg * 4, o_end, (p.Out & 3) == 0);
        }
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                // this lane's four contraction indices of half g: oc + 8g + 4*khalf + e
                const int o = oc + g * 8 + khalf * 4 + e;
                w_next[g][e] = (f32x4){0.f, 0.f, 0.f, 0.f};
                if (iok && o < o_end) {
                    const float *wp = p.w + (size_t)o * p.In + icol;
                    if (VEC) w_next[g][e] = *reinterpret_cast<const f32x4 *>(wp);
                    else
#pragma unroll
                        for (int j = 0; j < 4; ++j) w_next[g][e][j] = icol + j < p.In ? wp[j] : 0.f;
                }
            }
    };
    if (o_begin < o_end) request(o_begin);
    for (int oc = o_begin; oc < o_end; oc += 16) {
        barrier();  // the previous chunk's fragment reads are done
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int idx = tid + q * 256;
            *reinterpret_cast<uint4 *>(Ds + (idx >> 2) * kFcRow + (idx & 3) * 16) = dz_next[q];
        }
        f32x4 wv4[2][4];
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) wv4[g][e] = w_next[g][e];
        barrier();  // the staged rows are visible
        if (oc + 16 < o_end) request(oc + 16);
#pragma unroll
        for (int g = 0; g < 2; ++g) {
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const f32x4 af = *reinterpret_cast<const f32x4 *>(Ds + (wr * 64 + x * 32 + r) * kFcRow + g * 32 + khalf * 16);
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[x][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[e], wv4[g][e][j], acc[x][j], 0, 0, 0);
            }
        }
    }
    if (iok) {
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = row0 + wr * 64 + x * 32 + (e >> 2) * 8 + khalf * 4 + (e & 3);
                if (row < p.N) {
                    const f32x4 v = {acc[x][0][e], acc[x][1][e], acc[x][2][e], acc[x][3][e]};
                    float *dst = p.part + ((size_t)split * p.N + row) * p.In + icol;
                    if (VEC) *reinterpret_cast<f32x4 *>(dst) = v;
                    else
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (icol + j < p.In) dst[j] = v[j];
                }
            }
    }
}

// da = (sum over splits) [* (a > 0)]
template <typename T>
__global__ void fc_da_finish_kernel(const float *__restrict__ part, const T *__restrict__ a, T *__restrict__ da, size_t n,
                                    int splits, int relu_mask)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float s = 0.f;
    for (int k = 0; k < splits; ++k) s += part[(size_t)k * n + i];
    if (relu_mask && !(Elem<T>::load(a + i) > 0.f)) s = 0.f;
    Elem<T>::store(da + i, s);
}

static void fc_da_plan(int N, int In, int Out, FcDaArgs &a)
{
    a.N = N; a.In = In; a.Out = Out;
    a.tiles_i = (In + 255) / 256;
    a.tiles_m = (N + 127) / 128;
    const int tiles = a.tiles_i * a.tiles_m;
    int splits = (512 + tiles - 1) / tiles;
    const int max_splits = (Out + 63) / 64;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    a.o_per_split = ((Out + splits - 1) / splits + 15) / 16 * 16;
}
static int fc_da_splits(const FcDaArgs &a) { return (a.Out + a.o_per_split - 1) / a.o_per_split; }

size_t fc_bwd_workspace(int N, int In, int Out)
{
    FcDaArgs a;
    fc_da_plan(N, In, Out, a);
    return round_up((size_t)fc_da_splits(a) * N * In * 4, 256);
}

int fc_backward(int N, int In, int Out, const float *a, const float *w, const float *dz, float *dw, float *db, float *da,
                int relu_mask, void *ws, hipStream_t s)
{
    const int tiles_i = (In + 127) / 128, tiles_o = (Out + 127) / 128;
    hipLaunchKernelGGL(fc_dw_kernel, dim3((unsigned)(tiles_i * tiles_o)), dim3(256), 0, s, a, dz, dw, N, In, Out);
    if (db) hipLaunchKernelGGL(fc_db_kernel, dim3((Out + 63) / 64), dim3(256), 0, s, dz, db, N, Out);
    if (da) {
        FcDaArgs p;
        fc_da_plan(N, In, Out, p);
        const int splits = fc_da_splits(p);
        p.dz = dz; p.w = w; p.part = static_cast<float *>(ws);
        if (In % 4 == 0) hipLaunchKernelGGL(fc_da_kernel<true>, dim3((unsigned)(p.tiles_i * p.tiles_m * splits)), dim3(256), 0, s, p);
        else hipLaunchKernelGGL(fc_da_kernel<false>, dim3((unsigned)(p.tiles_i * p.tiles_m * splits)), dim3(256), 0, s, p);
        const size_t n = (size_t)N * In;
        hipLaunchKernelGGL(fc_da_finish_kernel<float>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p.part, a, da, n,
                           splits, relu_mask);
    }
    return launch_status();
}

// =========================================================================
// bf16 operands (activations and weights bf16, dz rounded to bf16, fp32 sums and fp32 results): the
// matrix-unit numerics of the paper's accelerator applied to the dense layers' backward products.
//
// Both products contract over an index that is NOT the contiguous one of its operands in memory
// (dW: the batch index of dz[n][o] and a[n][i]; dA: the output index of W[o][i]), while
// v_mfma_f32_32x32x16_bf16 wants eight consecutive contraction indices per lane.  The tiles are staged
// in LDS as they lie in memory and the fragments are fetched with the LDS transpose read
// ds_read_b64_tr_b16 (within 16 lanes, lane i receives element i%4 of the 8-byte chunks that lanes
// i/4, i/4+4, i/4+8, i/4+12 point at: lane s points at contraction index s/4 and channel chunk s%4, so
// lane i ends up with four consecutive contraction indices of channel i).  LDS rows are 288 bytes
// (128 channels + 32 bytes of padding): four consecutive rows start 32 bytes apart in the banks.
// =========================================================================
namespace {

constexpr int kTrRow = 288;

__device__ __forceinline__ bf16x8 fc_tr_fragment(const char *lds_lo, const char *lds_hi)
{
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    typedef __attribute__((address_space(3))) s16x4 *lp;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)lds_lo);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lp)lds_hi);
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// byte offset of this lane's chunk inside a 16-row x 32-channel block of a staged tile
__device__ __forceinline__ int fc_tr_lane_offset()
{
    const int lane = threadIdx.x & 63, G = lane >> 4, i = lane & 15;
    return (8 * (G >> 1) + (i >> 2)) * kTrRow + (G & 1) * 32 + (i & 3) * 8;
}

constexpr int kDwRows = 64;   // batch rows per pass of the dW kernel: four MFMA steps, 2 x 64 x 288 bytes of LDS (four workgroups per CU)

// dW = dz^T * a.  Workgroup: 128 (o) x 128 (i) block of dW; wave (wo, wi) owns a 64 x 64 sub-block = 2 x 2 MFMA
// tiles.  dzb: dz rounded to bf16, rows of OutP >= Out + 7 elements (a multiple of 8), zeros beyond Out.
__global__ __launch_bounds__(256) void fc_dw_bf16_kernel(const bf16_t *__restrict__ a, const bf16_t *__restrict__ dzb,
                                                            float *__restrict__ dw, int N, int In, int Out, int OutP)
{
    __shared__ __align__(16) char Ds[kDwRows * kTrRow];
    __shared__ __align__(16) char As[kDwRows * kTrRow];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = lane & 31, kp = lane >> 5;
    const int wo = wv & 1, wi = wv >> 1;
    const int tiles_i = (In + 127) / 128;
    const int i0 = (blockIdx.x % tiles_i) * 128, o0 = (blockIdx.x / tiles_i) * 128;
    const int loff = fc_tr_lane_offset();

    f32x16 acc[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[x][y][e] = 0.f;

    for (int n0 = 0; n0 < N; n0 += kDwRows) {
        __syncthreads();
        for (int idx = tid; idx < kDwRows * 16; idx += 256) {       // dz: 16 segments of 8 outputs per row
            const int seg = idx & 15, row = idx >> 4;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (n0 + row < N && o0 + seg * 8 < Out)
                v = *reinterpret_cast<const uint4 *>(dzb + (size_t)(n0 + row) * OutP + o0 + seg * 8);
            *reinterpret_cast<uint4 *>(Ds + row * kTrRow + seg * 16) = v;
        }
        for (int idx = tid; idx < kDwRows * 16; idx += 256) {       // a: 16 segments of 8 inputs per row
            const int seg = idx & 15, row = idx >> 4;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (n0 + row < N && i0 + seg * 8 < In)                  // In is a multiple of 8
                v = *reinterpret_cast<const uint4 *>(a + (size_t)(n0 + row) * In + i0 + seg * 8);
            *reinterpret_cast<uint4 *>(As + row * kTrRow + seg * 16) = v;
        }
        __syncthreads();
        const int steps = min(kDwRows, N - n0 + 15) / 16;
        for (int s = 0; s < steps; ++s) {
            bf16x8 df[2], af[2];
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const char *q = Ds + loff + (2 * wo + x) * 64 + 16 * s * kTrRow;
                df[x] = fc_tr_fragment(q, q + 4 * kTrRow);
            }
#pragma unroll
            for (int y = 0; y < 2; ++y) {
                const char *q = As + loff + (2 * wi + y) * 64 + 16 * s * kTrRow;
                af[y] = fc_tr_fragment(q, q + 4 * kTrRow);
            }
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int y = 0; y < 2; ++y) acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(df[x], af[y], acc[x][y], 0, 0, 0);
        }
    }
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) {
            const int i = i0 + wi * 64 + y * 32 + r;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int o = o0 + wo * 64 + x * 32 + (e >> 2) * 8 + kp * 4 + (e & 3);
                if (o < Out && i < In) __builtin_nontemporal_store(acc[x][y][e], &dw[(size_t)o * In + i]);
            }
        }
}

// dz fp32 [N][Out] -> bf16 [N][OutP] with zeros in the padding columns
__global__ void fc_dz_to_bf16_kernel(const float *__restrict__ dz, bf16_t *__restrict__ out, int N, int Out, int OutP)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)N * OutP) return;
    const int n = (int)(idx / OutP), o = (int)(idx % OutP);
    out[idx] = o < Out ? f32_to_bf16(dz[(size_t)n * Out + o]) : (bf16_t)0;
}

struct FcDaBf16Args {
    const bf16_t *dzb;  // [N][OutP], zeros beyond Out
    const bf16_t *w;    // [Out][In]
    float *part;        // [splits][N][In]
    int N, In, Out, OutP;
    int tiles_i, tiles_m, o_per_split;
};

// dA = dz * W.  Workgroup: 128 batch rows x 128 inputs x a range of outputs (the contraction index), 32 at a
// time.  Wave w owns inputs [32w, 32w+32) and all four 32-row blocks.  The weight rows of the next chunk are
// and the dz fragments (straight from the L2-resident bf16 copy) are requested while the current one is multiplied.
__global__ __launch_bounds__(256) void fc_da_bf16_kernel(FcDaBf16Args p)
{
    __shared__ __align__(16) char Ws[32 * kTrRow];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = lane & 31, kp = lane >> 5;
    int b = blockIdx.x;
    const int ti = b % p.tiles_i; b /= p.tiles_i;
    const int tm = b % p.tiles_m; b /= p.tiles_m;
    const int split = b;
    const int row0 = tm * 128, i0 = ti * 128;
    const int o_begin = split * p.o_per_split, o_end = min(o_begin + p.o_per_split, p.Out);
    const int loff = fc_tr_lane_offset() + wv * 64;

    f32x16 acc[4];
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[x][e] = 0.f;

    auto barrier = [] { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    uint4 w_next[2], d_next[2][4];
    auto request = [&](int oc) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int idx = tid + q * 256;
            const int seg = idx & 15, row = idx >> 4;
            w_next[q] = make_uint4(0, 0, 0, 0);
            if (oc + row < o_end && i0 + seg * 8 < p.In)
                w_next[q] = *reinterpret_cast<const uint4 *>(p.w + (size_t)(oc + row) * p.In + i0 + seg * 8);
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int n = row0 + x * 32 + r;
                d_next[ks][x] = make_uint4(0, 0, 0, 0);
                if (n < p.N) d_next[ks][x] = *reinterpret_cast<const uint4 *>(p.dzb + (size_t)n * p.OutP + oc + 16 * ks + 8 * kp);
            }
    };
    if (o_begin < o_end) request(o_begin);
    for (int oc = o_begin; oc < o_end; oc += 32) {
        barrier();  // the previous chunk's fragment reads are done
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int idx = tid + q * 256;
            *reinterpret_cast<uint4 *>(Ws + (idx >> 4) * kTrRow + (idx & 15) * 16) = w_next[q];
        }
        uint4 d_cur[2][4];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int x = 0; x < 4; ++x) d_cur[ks][x] = d_next[ks][x];
        barrier();  // the staged rows are visible
        if (oc + 32 < o_end) request(oc + 32);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const char *q = Ws + loff + 16 * ks * kTrRow;
            const bf16x8 wf = fc_tr_fragment(q, q + 4 * kTrRow);
#pragma unroll
            for (int x = 0; x < 4; ++x)
                acc[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, d_cur[ks][x]), wf, acc[x], 0, 0, 0);
        }
    }
    const int i = i0 + wv * 32 + r;
    if (i < p.In) {
#pragma unroll
        for (int x = 0; x < 4; ++x)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int n = row0 + x * 32 + (e >> 2) * 8 + kp * 4 + (e & 3);
                if (n < p.N) p.part[((size_t)split * p.N + n) * p.In + i] = acc[x][e];
            }
    }
}

// da = (sum over splits) [* (a > 0)], a in bf16
__global__ void fc_da_bf16_finish_kernel(const float *__restrict__ part, const bf16_t *__restrict__ a, float *__restrict__ da,
                                         size_t n, int splits, int relu_mask)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float s = 0.f;
    for (int k = 0; k < splits; ++k) s += part[(size_t)k * n + i];
    if (relu_mask && !(bf16_to_f32(a[i]) > 0.f)) s = 0.f;
    da[i] = s;
}

void fc_da_bf16_plan(int N, int In, int Out, FcDaBf16Args &a)
{
    a.N = N; a.In = In; a.Out = Out;
    a.OutP = (Out + 31) / 32 * 32 + 32;   // a fragment load may start up to 24 columns before the end of the last chunk
    a.tiles_i = (In + 127) / 128;
    a.tiles_m = (N + 127) / 128;
    const int tiles = a.tiles_i * a.tiles_m;
    int splits = (768 + tiles - 1) / tiles;
    const int max_splits = (Out + 63) / 64;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    a.o_per_split = ((Out + splits - 1) / splits + 31) / 32 * 32;
}
int fc_da_bf16_splits(const FcDaBf16Args &a) { return (a.Out + a.o_per_split - 1) / a.o_per_split; }

}  // namespace

size_t fc_bwd_bf16_workspace(int N, int In, int Out)
{
    FcDaBf16Args a;
    fc_da_bf16_plan(N, In, Out, a);
    return round_up((size_t)N * a.OutP * 2, 256) + round_up((size_t)fc_da_bf16_splits(a) * N * In * 4, 256);
}

// a [N][In] bf16, w [Out][In] bf16, dz [N][Out] fp32 -> dw [Out][In] fp32, db [Out] fp32 (may be null),
// da [N][In] fp32 (may be null; optionally masked by a > 0).  In must be a multiple of 8.
int fc_backward_bf16(int N, int In, int Out, const bf16_t *a, const bf16_t *w, const float *dz, float *dw, float *db, float *da,
                     int relu_mask, void *ws, hipStream_t s)
{
    FcDaBf16Args p;
    fc_da_bf16_plan(N, In, Out, p);
    bf16_t *dzb = static_cast<bf16_t *>(ws);
    const size_t nd = (size_t)N * p.OutP;
    hipLaunchKernelGGL(fc_dz_to_bf16_kernel, dim3((unsigned)((nd + 255) / 256)), dim3(256), 0, s, dz, dzb, N, Out, p.OutP);
    const int tiles_i = (In + 127) / 128, tiles_o = (Out + 127) / 128;
    hipLaunchKernelGGL(fc_dw_bf16_kernel, dim3((unsigned)(tiles_i * tiles_o)), dim3(256), 0, s, a, dzb, dw, N, In, Out, p.OutP);
    if (db) hipLaunchKernelGGL(fc_db_kernel, dim3((Out + 63) / 64), dim3(256), 0, s, dz, db, N, Out);
    if (da) {
        const int splits = fc_da_bf16_splits(p);
        p.dzb = dzb; p.w = w;
        p.part = reinterpret_cast<float *>(static_cast<char *>(ws) + round_up(nd * 2, 256));
        hipLaunchKernelGGL(fc_da_bf16_kernel, dim3((unsigned)(p.tiles_i * p.tiles_m * splits)), dim3(256), 0, s, p);
        const size_t n = (size_t)N * In;
        hipLaunchKernelGGL(fc_da_bf16_finish_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p.part, a, da, n,
                           splits, relu_mask);
    }
    return launch_status();
}

}  // namespace vgg
