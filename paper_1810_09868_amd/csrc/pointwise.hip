// Bandwidth-bound kernels: 2x2 max-pool (forward with argmax, scatter
// backward), softmax, cross-entropy, SGD, layout transforms, weight packing.
// All are plain coalesced streaming kernels; NHWC tensors are handled as
// vectors of 4 (fp32) or 8 (bf16) channels, i.e. 16 bytes per lane.
#include "common.h"
#include "flip_jobs.h"

namespace vgg {

// ---------------------------------------------------------------- max-pool
// One thread per (output pixel, 16-byte channel vector).  Window scan order
// (0,0),(0,1),(1,0),(1,1); a later element wins only when strictly greater,
// so ties resolve to the first (appendix table row "reduce-window").
template <typename T, int V>
__global__ void maxpool2x2_kernel(const T *__restrict__ x, T *__restrict__ y, uint8_t *__restrict__ arg, int N, int H,
                                  int W, int C)
{
    const int Ho = H / 2, Wo = W / 2, CV = C / V;
    const size_t total = (size_t)N * Ho * Wo * CV;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int cv = (int)(idx % CV);
    size_t pix = idx / CV;
    const int j = (int)(pix % Wo); pix /= Wo;
    const int i = (int)(pix % Ho);
    const int n = (int)(pix / Ho);
    const T *base = x + (((size_t)n * H + 2 * i) * W + 2 * j) * C + cv * V;
    float best[V];
    int a[V];
#pragma unroll
    for (int v = 0; v < V; ++v) { best[v] = Elem<T>::load(base + v); a[v] = 0; }
#pragma unroll
    for (int k = 1; k < 4; ++k) {
        const T *q = base + ((size_t)(k >> 1) * W + (k & 1)) * C;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const float f = Elem<T>::load(q + v);
            if (f > best[v]) { best[v] = f; a[v] = k; }
        }
    }
    const size_t o = idx * V;
#pragma unroll
    for (int v = 0; v < V; ++v) Elem<T>::store(y + o + v, best[v]);
    if (arg) {
#pragma unroll
        for (int v = 0; v < V; ++v) arg[o + v] = (uint8_t)a[v];
    }
}

// One thread per (pooled pixel, channel vector): writes the four positions
// of its window (appendix table row "select-and-scatter").
template <typename T, int V>
__global__ void maxpool2x2_bwd_kernel(const T *__restrict__ dy, const uint8_t *__restrict__ arg, T *__restrict__ dx,
                                      int N, int H, int W, int C)
{
    const int Ho = H / 2, Wo = W / 2, CV = C / V;
    const size_t total = (size_t)N * Ho * Wo * CV;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int cv = (int)(idx % CV);
    size_t pix = idx / CV;
    const int j = (int)(pix % Wo); pix /= Wo;
    const int i = (int)(pix % Ho);
    const int n = (int)(pix / Ho);
    T *base = dx + (((size_t)n * H + 2 * i) * W + 2 * j) * C + cv * V;
    const size_t o = idx * V;
    float d[V];
    int a[V];
#pragma unroll
    for (int v = 0; v < V; ++v) { d[v] = Elem<T>::load(dy + o + v); a[v] = arg[o + v]; }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        T *q = base + ((size_t)(k >> 1) * W + (k & 1)) * C;
#pragma unroll
        for (int v = 0; v < V; ++v) Elem<T>::store(q + v, a[v] == k ? d[v] : 0.f);
    }
}

int maxpool2x2(int dtype, int N, int H, int W, int C, const void *x, void *y, uint8_t *arg, hipStream_t s)
{
    const int V = dtype == VGG_BF16 ? 8 : 4;
    const size_t total = (size_t)N * (H / 2) * (W / 2) * (C / V);
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (dtype == VGG_BF16)
        hipLaunchKernelGGL((maxpool2x2_kernel<bf16_t, 8>), grid, block, 0, s, (const bf16_t *)x, (bf16_t *)y, arg, N, H, W, C);
    else
        hipLaunchKernelGGL((maxpool2x2_kernel<float, 4>), grid, block, 0, s, (const float *)x, (float *)y, arg, N, H, W, C);
    return launch_status();
}

int maxpool2x2_bwd(int dtype, int N, int H, int W, int C, const void *dy, const uint8_t *arg, void *dx, hipStream_t s)
{
    const int V = dtype == VGG_BF16 ? 8 : 4;
    const size_t total = (size_t)N * (H / 2) * (W / 2) * (C / V);
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (dtype == VGG_BF16)
        hipLaunchKernelGGL((maxpool2x2_bwd_kernel<bf16_t, 8>), grid, block, 0, s, (const bf16_t *)dy, arg, (bf16_t *)dx, N, H, W, C);
    else
        hipLaunchKernelGGL((maxpool2x2_bwd_kernel<float, 4>), grid, block, 0, s, (const float *)dy, arg, (float *)dx, N, H, W, C);
    return launch_status();
}

// ----------------------------------------------------------------- softmax
// One wavefront per row: max, sum of exponentials and normalisation through
// wavefront reductions (listing "softmax").
__global__ __launch_bounds__(256) void softmax_kernel(const float *__restrict__ z, float *__restrict__ p, int N, int K)
{
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= N) return;
    const float *zr = z + (size_t)row * K;
    float *pr = p + (size_t)row * K;
    float m = -INFINITY;
    for (int k = lane; k < K; k += 64) m = fmaxf(m, zr[k]);
    m = wave_max(m);
    float s = 0.f;
    for (int k = lane; k < K; k += 64) s += expf(zr[k] - m);
    s = wave_sum(s);
    const float inv = 1.f / s;
    for (int k = lane; k < K; k += 64) pr[k] = expf(zr[k] - m) * inv;
}

// dz = (p - onehot)/N and the per-row loss terms; one wavefront per row.
__global__ __launch_bounds__(256) void xent_bwd_kernel(const float *__restrict__ p, const int32_t *__restrict__ labels,
                                                       float *__restrict__ rowloss, float *__restrict__ dz, int N, int K)
{
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= N) return;
    const int y = labels[row];
    const float invN = 1.f / (float)N;
    if (dz)
        for (int k = lane; k < K; k += 64) dz[(size_t)row * K + k] = (p[(size_t)row * K + k] - (k == y ? 1.f : 0.f)) * invN;
    if (rowloss && lane == 0) rowloss[row] = (y >= 0 && y < K) ? -logf(p[(size_t)row * K + y]) : 0.f;
}

// Sums the N per-row terms in a fixed order (one wavefront), divides by N.
__global__ __launch_bounds__(64) void loss_reduce_kernel(const float *__restrict__ rowloss, float *__restrict__ loss, int N)
{
    float s = 0.f;
    for (int i = threadIdx.x; i < N; i += 64) s += rowloss[i];
    s = wave_sum(s);
    if (threadIdx.x == 0) loss[0] = s / (float)N;
}

int softmax_rows(int N, int K, const float *z, float *p, hipStream_t s)
{
    hipLaunchKernelGGL(softmax_kernel, dim3((N + 3) / 4), dim3(256), 0, s, z, p, N, K);
    return launch_status();
}

// rowloss: N floats of scratch (only needed when loss != null).
int softmax_xent_bwd(int N, int K, const float *p, const int32_t *labels, float *loss, float *dz, float *rowloss,
                     hipStream_t s)
{
    hipLaunchKernelGGL(xent_bwd_kernel, dim3((N + 3) / 4), dim3(256), 0, s, p, labels, loss ? rowloss : nullptr, dz, N, K);
    if (loss) hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(64), 0, s, rowloss, loss, N);
    return launch_status();
}

// --------------------------------------------------------------------- SGD
__global__ void sgd_kernel(float *__restrict__ theta, const float *__restrict__ grad, float lr, size_t n4, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n4) {
        f32x4 t = reinterpret_cast<f32x4 *>(theta)[i];
        const f32x4 g = reinterpret_cast<const f32x4 *>(grad)[i];
        t.x = sgd_step(t.x, g.x, lr); t.y = sgd_step(t.y, g.y, lr); t.z = sgd_step(t.z, g.z, lr); t.w = sgd_step(t.w, g.w, lr);
        reinterpret_cast<f32x4 *>(theta)[i] = t;
    } else if (i == n4) {
        for (size_t k = n4 * 4; k < n; ++k) theta[k] = sgd_step(theta[k], grad[k], lr);
    }
}

int sgd_update(size_t n, float *theta, const float *grad, float lr, hipStream_t s)
{
    const size_t n4 = n / 4;
    hipLaunchKernelGGL(sgd_kernel, dim3((unsigned)((n4 + 1 + 255) / 256)), dim3(256), 0, s, theta, grad, lr, n4, n);
    return launch_status();
}

// Mixed precision: the fp32 master value takes the step and the working copy (bf16 weights, fp32
// biases) is refreshed from it in the same pass.  n must be a multiple of 4.
template <typename TC>
__global__ void sgd_master_kernel(float *__restrict__ theta, const float *__restrict__ grad, float lr, TC *__restrict__ copy,
                                  size_t n4)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n4) return;
    f32x4 t = reinterpret_cast<f32x4 *>(theta)[i];
    const f32x4 g = reinterpret_cast<const f32x4 *>(grad)[i];
    t.x = sgd_step(t.x, g.x, lr); t.y = sgd_step(t.y, g.y, lr); t.z = sgd_step(t.z, g.z, lr); t.w = sgd_step(t.w, g.w, lr);
    reinterpret_cast<f32x4 *>(theta)[i] = t;
    store4(copy + i * 4, t.x, t.y, t.z, t.w);
}

int sgd_update_master(size_t n, float *theta, const float *grad, float lr, void *copy, int copy_dtype, hipStream_t s)
{
    if (n % 4) return VGG_ERR_UNSUPPORTED;
    const size_t n4 = n / 4;
    const dim3 grid((unsigned)((n4 + 255) / 256));
    if (copy_dtype == VGG_BF16)
        hipLaunchKernelGGL(sgd_master_kernel<bf16_t>, grid, dim3(256), 0, s, theta, grad, lr, (bf16_t *)copy, n4);
    else
        hipLaunchKernelGGL(sgd_master_kernel<float>, grid, dim3(256), 0, s, theta, grad, lr, (float *)copy, n4);
    return launch_status();
}

// The same for the convolution weights of a whole network in one launch: the fp32 master tensors are
// [9][Cout][CinP] row-major (as are the gradients), the bf16 working copies have their columns blocked by
// 16 (packed_w_index).  Workgroups [first[j], first[j+1]) serve tensor j, one thread per four columns.
__global__ __launch_bounds__(256) void sgd_master_conv_kernel(SgdConvJobs J, float lr)
{
    int j = 0;
    while (j + 1 < J.n && (int)blockIdx.x >= J.first[j + 1]) ++j;
    const int Cout = J.Cout[j], CinP = J.CinP[j];
    const size_t i = (size_t)((int)blockIdx.x - J.first[j]) * 256 + threadIdx.x;   // quad index
    const size_t n4 = (size_t)9 * Cout * CinP / 4;
    if (i >= n4) return;
    f32x4 t = reinterpret_cast<f32x4 *>(J.theta[j])[i];
    const f32x4 g = reinterpret_cast<const f32x4 *>(J.grad[j])[i];
    t.x = sgd_step(t.x, g.x, lr); t.y = sgd_step(t.y, g.y, lr); t.z = sgd_step(t.z, g.z, lr); t.w = sgd_step(t.w, g.w, lr);
    reinterpret_cast<f32x4 *>(J.theta[j])[i] = t;
    const size_t e = i * 4;
    const int col = (int)(e % CinP);
    const size_t tr = e / CinP;
    const int row = (int)(tr % Cout), tap = (int)(tr / Cout);
    store4(J.copy[j] + packed_w_index<bf16_t>(tap, row, col, Cout, CinP), t.x, t.y, t.z, t.w);
}

int sgd_update_master_conv(SgdConvJobs &jobs, float lr, hipStream_t s)
{
    if (jobs.n < 1 || jobs.n > kMaxFlipJobs) return VGG_ERR_UNSUPPORTED;
    int total = 0;
    for (int j = 0; j < jobs.n; ++j) {
        if (jobs.CinP[j] % 4) return VGG_ERR_UNSUPPORTED;
        jobs.first[j] = total;
        total += (int)(((size_t)9 * jobs.Cout[j] * jobs.CinP[j] / 4 + 255) / 256);
    }
    jobs.first[jobs.n] = total;
    hipLaunchKernelGGL(sgd_master_conv_kernel, dim3((unsigned)total), dim3(256), 0, s, jobs, lr);
    return launch_status();
}

// ------------------------------------------------------- layout transforms
// NCHW fp32 -> NHWC T with zero padding of the channels up to Cpad.  One
// thread per output pixel; reads are coalesced along w for each channel.
template <typename T>
__global__ void nchw_to_nhwc_kernel(const float *__restrict__ x, T *__restrict__ y, int N, int C, int H, int W, int Cpad)
{
    const size_t HW = (size_t)H * W;
    const size_t pix = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (pix >= (size_t)N * HW) return;
    const size_t n = pix / HW, hw = pix % HW;
    T *o = y + pix * Cpad;
    constexpr int V = 16 / (int)sizeof(T);
    if (Cpad % V == 0) {
        // 16-byte stores: V channels at a time
        for (int c0 = 0; c0 < Cpad; c0 += V) {
            T tmp[V];
#pragma unroll
            for (int k = 0; k < V; ++k) Elem<T>::store(tmp + k, c0 + k < C ? x[(n * C + c0 + k) * HW + hw] : 0.f);
            f32x4 v;
            __builtin_memcpy(&v, tmp, 16);
            *reinterpret_cast<f32x4 *>(o + c0) = v;
        }
        return;
    }
    for (int c = 0; c < Cpad; ++c) Elem<T>::store(o + c, c < C ? x[(n * C + c) * HW + hw] : 0.f);
}

template <typename T>
__global__ void nhwc_to_nchw_kernel(const T *__restrict__ x, float *__restrict__ y, int N, int C, int H, int W, int Cpad)
{
    const size_t HW = (size_t)H * W;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // over N*C*HW, hw fastest
    if (idx >= (size_t)N * C * HW) return;
    const size_t hw = idx % HW, c = (idx / HW) % C, n = idx / (HW * C);
    y[idx] = Elem<T>::load(x + (n * HW + hw) * Cpad + c);
}

int nchw_to_nhwc(int dtype, int N, int C, int H, int W, int Cpad, const float *x, void *y, hipStream_t s)
{
    const size_t total = (size_t)N * H * W;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (dtype == VGG_BF16)
        hipLaunchKernelGGL(nchw_to_nhwc_kernel<bf16_t>, grid, block, 0, s, x, (bf16_t *)y, N, C, H, W, Cpad);
    else
        hipLaunchKernelGGL(nchw_to_nhwc_kernel<float>, grid, block, 0, s, x, (float *)y, N, C, H, W, Cpad);
    return launch_status();
}

int nhwc_to_nchw(int dtype, int N, int C, int H, int W, int Cpad, const void *x, float *y, hipStream_t s)
{
    const size_t total = (size_t)N * C * H * W;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (dtype == VGG_BF16)
        hipLaunchKernelGGL(nhwc_to_nchw_kernel<bf16_t>, grid, block, 0, s, (const bf16_t *)x, y, N, C, H, W, Cpad);
    else
        hipLaunchKernelGGL(nhwc_to_nchw_kernel<float>, grid, block, 0, s, (const float *)x, y, N, C, H, W, Cpad);
    return launch_status();
}

// Pads the channel dimension of an NHWC tensor with zeros (C -> Cpad).
template <typename T>
__global__ void pad_channels_kernel(const T *__restrict__ x, T *__restrict__ y, size_t pixels, int C, int Cpad)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= pixels * Cpad) return;
    const size_t pix = idx / Cpad;
    const int c = (int)(idx % Cpad);
    y[idx] = c < C ? x[pix * C + c] : (T)0;
}

int pad_channels(int dtype, size_t pixels, int C, int Cpad, const void *x, void *y, hipStream_t s)
{
    const size_t total = pixels * Cpad;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (dtype == VGG_BF16)
        hipLaunchKernelGGL(pad_channels_kernel<bf16_t>, grid, block, 0, s, (const bf16_t *)x, (bf16_t *)y, pixels, C, Cpad);
    else
        hipLaunchKernelGGL(pad_channels_kernel<float>, grid, block, 0, s, (const float *)x, (float *)y, pixels, C, Cpad);
    return launch_status();
}

template <typename TS, typename TD>
__global__ void convert_kernel(const TS *__restrict__ a, TD *__restrict__ b, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) Elem<TD>::store(b + i, Elem<TS>::load(a + i));
}

int convert(int sd, int dd, size_t n, const void *src, void *dst, hipStream_t s)
{
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    if (sd == VGG_F32 && dd == VGG_F32)
        hipLaunchKernelGGL((convert_kernel<float, float>), grid, block, 0, s, (const float *)src, (float *)dst, n);
    else if (sd == VGG_F32)
        hipLaunchKernelGGL((convert_kernel<float, bf16_t>), grid, block, 0, s, (const float *)src, (bf16_t *)dst, n);
    else if (dd == VGG_F32)
        hipLaunchKernelGGL((convert_kernel<bf16_t, float>), grid, block, 0, s, (const bf16_t *)src, (float *)dst, n);
    else
        hipLaunchKernelGGL((convert_kernel<bf16_t, bf16_t>), grid, block, 0, s, (const bf16_t *)src, (bf16_t *)dst, n);
    return launch_status();
}

// ---------------------------------------------------------- weight packing
// forward:  element (t, co, ci) of a [Cout][CinP] operand  = w[co][ci][t]          (zeros for ci >= Cin)
// flipped:  element (t, ci, co) of a [Cin][CoutP] operand  = w[co][ci][8 - t]      (zeros for co >= Cout)
// at the position packed_w_index<T> gives (fp32: row-major; bf16: columns blocked by 16).
template <typename T>
__global__ void pack_conv_w_kernel(const float *__restrict__ w, T *__restrict__ dst, int Cin, int Cout, int rows,
                                   int colsP, int flip)
{
    const size_t total = (size_t)9 * rows * colsP;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int c = (int)(idx % colsP);
    const int rr = (int)((idx / colsP) % rows);
    const int t = (int)(idx / ((size_t)colsP * rows));
    float v = 0.f;
    if (!flip) {
        if (c < Cin) v = w[((size_t)rr * Cin + c) * 9 + t];
    } else {
        if (c < Cout) v = w[((size_t)c * Cin + rr) * 9 + (8 - t)];
    }
    Elem<T>::store(dst + packed_w_index<T>(t, rr, c, rows, colsP), v);
}

// colsP: padded length of the contiguous dimension (0: the granularity of dtype)
int pack_conv_w(int dtype, int Cin, int Cout, const float *w, void *dst, int flip, hipStream_t s, int colsP = 0)
{
    const int rows = flip ? Cin : Cout;
    if (colsP == 0) colsP = padded_channels(dtype, flip ? Cout : Cin);
    const size_t total = (size_t)9 * rows * colsP;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (dtype == VGG_BF16)
        hipLaunchKernelGGL(pack_conv_w_kernel<bf16_t>, grid, block, 0, s, w, (bf16_t *)dst, Cin, Cout, rows, colsP, flip);
    else
        hipLaunchKernelGGL(pack_conv_w_kernel<float>, grid, block, 0, s, w, (float *)dst, Cin, Cout, rows, colsP, flip);
    return launch_status();
}

// Packed-forward fp32 [9][Cout][CinP] -> the flipped operand [9][Cin'][CoutP] where
// Cin' = CinP rows are kept (padding rows are zero anyway).
// One 32 x 32 (ci, co) block of one tap per workgroup, transposed through LDS so that both the reads
// (ci contiguous) and the writes (co contiguous) are coalesced.
template <typename TD>
__global__ __launch_bounds__(256) void flip_packed_w_kernel(const float *__restrict__ src, TD *__restrict__ dst, int CinP, int Cout,
                                                            int CoutP)
{
    __shared__ float tile[32][33];
    const int t = blockIdx.z, ci0 = blockIdx.x * 32, co0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
    for (int r = ty; r < 32; r += 8) {
        const int co = co0 + r, ci = ci0 + tx;
        tile[r][tx] = (co < Cout && ci < CinP) ? src[((size_t)(8 - t) * Cout + co) * CinP + ci] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int r = ty; r < 32; r += 8) {
        const int ci = ci0 + r, co = co0 + tx;
        if (ci < CinP && co < CoutP) Elem<TD>::store(dst + packed_w_index<TD>(t, ci, co, CinP, CoutP), tile[tx][r]);
    }
}

int flip_packed_w(int dst_dtype, int CinP, int Cout, int CoutP, const float *src, void *dst, hipStream_t s)
{
    const dim3 grid((unsigned)((CinP + 31) / 32), (unsigned)((CoutP + 31) / 32), 9);
    if (dst_dtype == VGG_BF16)
        hipLaunchKernelGGL(flip_packed_w_kernel<bf16_t>, grid, dim3(256), 0, s, src, (bf16_t *)dst, CinP, Cout, CoutP);
    else
        hipLaunchKernelGGL(flip_packed_w_kernel<float>, grid, dim3(256), 0, s, src, (float *)dst, CinP, Cout, CoutP);
    return launch_status();
}

// The same for several tensors in one launch (a training step flips fifteen of them, each a few
// microseconds of work): workgroups [first[j], first[j+1]) serve tensor j.
template <typename TD>
__global__ __launch_bounds__(256) void flip_packed_w_all_kernel(FlipJobs J)
{
    __shared__ float tile[32][33];
    int j = 0;
    while (j + 1 < J.n && (int)blockIdx.x >= J.first[j + 1]) ++j;
    const float *__restrict__ src = J.src[j];
    TD *__restrict__ dst = static_cast<TD *>(J.dst[j]);
    const int CinP = J.CinP[j], Cout = J.Cout[j], CoutP = J.CoutP[j];
    const int nbx = (CinP + 31) / 32, nby = (CoutP + 31) / 32;
    const int local = (int)blockIdx.x - J.first[j];
    const int bx = local % nbx, by = (local / nbx) % nby, t = local / (nbx * nby);
    const int ci0 = bx * 32, co0 = by * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
    for (int r = ty; r < 32; r += 8) {
        const int co = co0 + r, ci = ci0 + tx;
        tile[r][tx] = (co < Cout && ci < CinP) ? src[((size_t)(8 - t) * Cout + co) * CinP + ci] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int r = ty; r < 32; r += 8) {
        const int ci = ci0 + r, co = co0 + tx;
        if (ci < CinP && co < CoutP) Elem<TD>::store(dst + packed_w_index<TD>(t, ci, co, CinP, CoutP), tile[tx][r]);
    }
}

// jobs.first is filled here
int flip_packed_w_all(int dst_dtype, FlipJobs &jobs, hipStream_t s)
{
    if (jobs.n < 1 || jobs.n > kMaxFlipJobs) return VGG_ERR_UNSUPPORTED;
    int total = 0;
    for (int j = 0; j < jobs.n; ++j) {
        jobs.first[j] = total;
        total += ((jobs.CinP[j] + 31) / 32) * ((jobs.CoutP[j] + 31) / 32) * 9;
    }
    jobs.first[jobs.n] = total;
    if (dst_dtype == VGG_BF16)
        hipLaunchKernelGGL(flip_packed_w_all_kernel<bf16_t>, dim3((unsigned)total), dim3(256), 0, s, jobs);
    else
        hipLaunchKernelGGL(flip_packed_w_all_kernel<float>, dim3((unsigned)total), dim3(256), 0, s, jobs);
    return launch_status();
}

__global__ void unpack_conv_w_kernel(const float *__restrict__ src, float *__restrict__ w, int Cin, int Cout, int CinP)
{
    const size_t total = (size_t)Cout * Cin * 9;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int t = (int)(idx % 9);
    const int ci = (int)((idx / 9) % Cin);
    const int co = (int)(idx / ((size_t)9 * Cin));
    w[idx] = src[((size_t)t * Cout + co) * CinP + ci];
}

// CinP: channel stride of src (0: the fp32 granularity)
int unpack_conv_w(int Cin, int Cout, const float *src, float *w, hipStream_t s, int CinP = 0)
{
    const size_t total = (size_t)Cout * Cin * 9;
    hipLaunchKernelGGL(unpack_conv_w_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, src, w, Cin, Cout,
                       CinP ? CinP : padded_channels(VGG_F32, Cin));
    return launch_status();
}

// Dense weights [Out][C*HW] with columns in (c,hw) order <-> columns in (hw,c)
// order (the order in which the NHWC pooled tensor is flattened).  to_hwc != 0:
// dst[o][hw*C + c] = src[o][c*HW + hw]; otherwise the inverse.
template <typename TS, typename TD>
__global__ void permute_fc_cols_kernel(const TS *__restrict__ src, TD *__restrict__ dst, int Out, int C, int HW, int to_hwc)
{
    const size_t In = (size_t)C * HW;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // index into dst
    if (idx >= (size_t)Out * In) return;
    const size_t o = idx / In, col = idx % In;
    size_t scol;
    if (to_hwc) { const size_t hw = col / C, c = col % C; scol = c * HW + hw; }
    else        { const size_t c = col / HW, hw = col % HW; scol = hw * C + c; }
    Elem<TD>::store(dst + idx, Elem<TS>::load(src + o * In + scol));
}

int permute_fc_cols(int dst_dtype, int Out, int C, int HW, int to_hwc, const float *src, void *dst, hipStream_t s)
{
    const size_t total = (size_t)Out * C * HW;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (dst_dtype == VGG_BF16)
        hipLaunchKernelGGL((permute_fc_cols_kernel<float, bf16_t>), grid, block, 0, s, src, (bf16_t *)dst, Out, C, HW, to_hwc);
    else
        hipLaunchKernelGGL((permute_fc_cols_kernel<float, float>), grid, block, 0, s, src, (float *)dst, Out, C, HW, to_hwc);
    return launch_status();
}

}  // namespace vgg
