/*
 * Plain fp64 CPU oracle for the VGG19 forward pass and training step.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call into this
 * file; it exists so that tests, the smoke check and the benchmark's CPU
 * baseline leg have an independent, obviously-correct result to compare with.
 * It shares no code, header, table or helper with the GPU library.
 *
 * Every function is the textbook definition written out as direct loops in
 * double precision.  Layouts are the canonical ones: activations
 * [N][C][H][W], convolution weights [Cout][Cin][3][3], dense weights
 * [Out][In], all row-major.  The only parallelism is an OpenMP loop over
 * independent output slices (image and channel, or output rows).
 *
 * What the paper fixes (section "VGG19 forward pass", section "VGG19
 * backward pass", the listing defining dense and softmax, and the appendix
 * table of HLO instruction counts):
 *   - the forward pass is 16 convolutions, 5 window-max reductions, 3 dot
 *     products, bias adds, and element-wise maxima (ReLU), then softmax;
 *   - dense(W, x, b) = W*x + b with W stored [out][in];
 *   - softmax(xs) = exp(xs) / sum(exp(xs));
 *   - the backward pass has one kernel reversal per data-gradient
 *     convolution and none in the forward pass, i.e. the forward op is a
 *     cross-correlation (no kernel flip).
 *
 * Return value of every function: 0 on success, -1 on a null pointer,
 * -2 on a bad shape.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REF_OK 0
#define REF_ERR_NULL (-1)
#define REF_ERR_SHAPE (-2)

int ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * 3x3, stride 1, zero padding 1 cross-correlation with bias and optional
 * ReLU (appendix table rows "convolution", "add", "maximum"):
 *   y[n,co,h,w] = f( b[co] + sum_{ci,kh,kw} x[n,ci,h+kh-1,w+kw-1] * wt[co,ci,kh,kw] )
 * where x is taken as zero outside [0,H)x[0,W) and f is max(0,.) when relu
 * is non-zero, identity otherwise.  bias may be NULL (treated as zeros).
 */
int ref_conv3x3_fwd(int N, int Cin, int Cout, int H, int W,
                    const double *x, const double *wt, const double *bias,
                    int relu, double *y)
{
    if (!x || !wt || !y) return REF_ERR_NULL;
    if (N <= 0 || Cin <= 0 || Cout <= 0 || H <= 0 || W <= 0) return REF_ERR_SHAPE;
    const size_t HW = (size_t)H * W;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int n = 0; n < N; ++n) {
        for (int co = 0; co < Cout; ++co) {
            double *yp = y + ((size_t)n * Cout + co) * HW;
            const double b = bias ? bias[co] : 0.0;
            for (size_t i = 0; i < HW; ++i) yp[i] = b;
            for (int ci = 0; ci < Cin; ++ci) {
                const double *xp = x + ((size_t)n * Cin + ci) * HW;
                for (int kh = 0; kh < 3; ++kh) {
                    for (int kw = 0; kw < 3; ++kw) {
                        const double wv = wt[(((size_t)co * Cin + ci) * 3 + kh) * 3 + kw];
                        for (int h = 0; h < H; ++h) {
                            const int hi = h + kh - 1;
                            if (hi < 0 || hi >= H) continue;
                            for (int w = 0; w < W; ++w) {
                                const int wi = w + kw - 1;
                                if (wi < 0 || wi >= W) continue;
                                yp[(size_t)h * W + w] += xp[(size_t)hi * W + wi] * wv;
                            }
                        }
                    }
                }
            }
            if (relu)
                for (size_t i = 0; i < HW; ++i) yp[i] = yp[i] > 0.0 ? yp[i] : 0.0;
        }
    }
    return REF_OK;
}

/*
 * Gradient of the bias-free convolution with respect to its input (the
 * "reverse" + "convolution" pairs of the backward column of the appendix
 * table).  g is the gradient with respect to the pre-activation output:
 *   dx[n,ci,h,w] = sum_{co,kh,kw} g[n,co,h-kh+1,w-kw+1] * wt[co,ci,kh,kw]
 * with g taken as zero outside the image.
 */
int ref_conv3x3_bwd_data(int N, int Cin, int Cout, int H, int W,
                         const double *g, const double *wt, double *dx)
{
    if (!g || !wt || !dx) return REF_ERR_NULL;
    if (N <= 0 || Cin <= 0 || Cout <= 0 || H <= 0 || W <= 0) return REF_ERR_SHAPE;
    const size_t HW = (size_t)H * W;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int n = 0; n < N; ++n) {
        for (int ci = 0; ci < Cin; ++ci) {
            double *dp = dx + ((size_t)n * Cin + ci) * HW;
            for (size_t i = 0; i < HW; ++i) dp[i] = 0.0;
            for (int co = 0; co < Cout; ++co) {
                const double *gp = g + ((size_t)n * Cout + co) * HW;
                for (int kh = 0; kh < 3; ++kh) {
                    for (int kw = 0; kw < 3; ++kw) {
                        const double wv = wt[(((size_t)co * Cin + ci) * 3 + kh) * 3 + kw];
                        for (int h = 0; h < H; ++h) {
                            const int ho = h - kh + 1;
                            if (ho < 0 || ho >= H) continue;
                            for (int w = 0; w < W; ++w) {
                                const int wo = w - kw + 1;
                                if (wo < 0 || wo >= W) continue;
                                dp[(size_t)h * W + w] += gp[(size_t)ho * W + wo] * wv;
                            }
                        }
                    }
                }
            }
        }
    }
    return REF_OK;
}

/*
 * Gradient with respect to the weights and the bias:
 *   dw[co,ci,kh,kw] = sum_{n,h,w} g[n,co,h,w] * x[n,ci,h+kh-1,w+kw-1]
 *   db[co]          = sum_{n,h,w} g[n,co,h,w]
 * db may be NULL.
 */
int ref_conv3x3_bwd_weight(int N, int Cin, int Cout, int H, int W,
                           const double *x, const double *g, double *dw, double *db)
{
    if (!x || !g || !dw) return REF_ERR_NULL;
    if (N <= 0 || Cin <= 0 || Cout <= 0 || H <= 0 || W <= 0) return REF_ERR_SHAPE;
    const size_t HW = (size_t)H * W;
#pragma omp parallel for schedule(dynamic)
    for (int co = 0; co < Cout; ++co) {
        if (db) {
            double s = 0.0;
            for (int n = 0; n < N; ++n) {
                const double *gp = g + ((size_t)n * Cout + co) * HW;
                for (size_t i = 0; i < HW; ++i) s += gp[i];
            }
            db[co] = s;
        }
        for (int ci = 0; ci < Cin; ++ci) {
            for (int kh = 0; kh < 3; ++kh) {
                for (int kw = 0; kw < 3; ++kw) {
                    double s = 0.0;
                    for (int n = 0; n < N; ++n) {
                        const double *gp = g + ((size_t)n * Cout + co) * HW;
                        const double *xp = x + ((size_t)n * Cin + ci) * HW;
                        for (int h = 0; h < H; ++h) {
                            const int hi = h + kh - 1;
                            if (hi < 0 || hi >= H) continue;
                            for (int w = 0; w < W; ++w) {
                                const int wi = w + kw - 1;
                                if (wi < 0 || wi >= W) continue;
                                s += gp[(size_t)h * W + w] * xp[(size_t)hi * W + wi];
                            }
                        }
                    }
                    dw[(((size_t)co * Cin + ci) * 3 + kh) * 3 + kw] = s;
                }
            }
        }
    }
    return REF_OK;
}

/*
 * 2x2 window, stride 2 maximum (appendix table row "reduce-window").
 *   p[n,c,i,j] = max over dh,dw in {0,1} of x[n,c,2i+dh,2j+dw]
 * arg (may be NULL) receives 2*dh+dw of the first maximum met when the
 * window is scanned (0,0),(0,1),(1,0),(1,1); a later element replaces the
 * current one only when strictly greater.
 */
int ref_maxpool2x2(int N, int C, int H, int W, const double *x, double *p, uint8_t *arg)
{
    if (!x || !p) return REF_ERR_NULL;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || (H & 1) || (W & 1)) return REF_ERR_SHAPE;
    const int Ho = H / 2, Wo = W / 2;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            const double *xp = x + ((size_t)n * C + c) * H * W;
            const size_t ob = ((size_t)n * C + c) * Ho * Wo;
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) {
                    double best = xp[(size_t)(2 * i) * W + 2 * j];
                    int a = 0;
                    for (int dh = 0; dh < 2; ++dh)
                        for (int dw = 0; dw < 2; ++dw) {
                            const double v = xp[(size_t)(2 * i + dh) * W + 2 * j + dw];
                            if (v > best) { best = v; a = 2 * dh + dw; }
                        }
                    p[ob + (size_t)i * Wo + j] = best;
                    if (arg) arg[ob + (size_t)i * Wo + j] = (uint8_t)a;
                }
        }
    return REF_OK;
}

/*
 * Backward of the 2x2 maximum (appendix table row "select-and-scatter"):
 * the pooled gradient goes to the recorded arg position of each window and
 * the other three positions receive zero.  H, W are the un-pooled sizes.
 */
int ref_maxpool2x2_bwd(int N, int C, int H, int W, const double *dp, const uint8_t *arg, double *dx)
{
    if (!dp || !arg || !dx) return REF_ERR_NULL;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || (H & 1) || (W & 1)) return REF_ERR_SHAPE;
    const int Ho = H / 2, Wo = W / 2;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double *xp = dx + ((size_t)n * C + c) * H * W;
            const size_t ob = ((size_t)n * C + c) * Ho * Wo;
            for (size_t i = 0; i < (size_t)H * W; ++i) xp[i] = 0.0;
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) {
                    const int a = arg[ob + (size_t)i * Wo + j];
                    if (a < 0 || a > 3) continue;
                    xp[(size_t)(2 * i + (a >> 1)) * W + 2 * j + (a & 1)] = dp[ob + (size_t)i * Wo + j];
                }
        }
    return REF_OK;
}

/*
 * Dense layer, the paper's dense(W, x, b) = W*x + b applied to each of the
 * N columns x = a[n,:] (listing "dense"; the HLO "dot" contracts the second
 * index of W with the first of x):
 *   z[n,o] = f( b[o] + sum_i w[o,i] * a[n,i] )
 */
int ref_fc(int N, int In, int Out, const double *a, const double *w, const double *bias,
           int relu, double *z)
{
    if (!a || !w || !z) return REF_ERR_NULL;
    if (N <= 0 || In <= 0 || Out <= 0) return REF_ERR_SHAPE;
#pragma omp parallel for schedule(static)
    for (int o = 0; o < Out; ++o) {
        const double *wr = w + (size_t)o * In;
        for (int n = 0; n < N; ++n) {
            const double *ar = a + (size_t)n * In;
            double s = bias ? bias[o] : 0.0;
            for (int i = 0; i < In; ++i) s += wr[i] * ar[i];
            if (relu && !(s > 0.0)) s = 0.0;
            z[(size_t)n * Out + o] = s;
        }
    }
    return REF_OK;
}

/*
 * Backward of the dense layer; dz is the gradient with respect to the
 * pre-activation z:
 *   dw[o,i] = sum_n dz[n,o] a[n,i],  db[o] = sum_n dz[n,o],
 *   da[n,i] = sum_o dz[n,o] w[o,i].
 * db and da may be NULL.
 */
int ref_fc_bwd(int N, int In, int Out, const double *a, const double *w, const double *dz,
               double *dw, double *db, double *da)
{
    if (!a || !w || !dz || !dw) return REF_ERR_NULL;
    if (N <= 0 || In <= 0 || Out <= 0) return REF_ERR_SHAPE;
#pragma omp parallel for schedule(static)
    for (int o = 0; o < Out; ++o) {
        double sb = 0.0;
        for (int n = 0; n < N; ++n) sb += dz[(size_t)n * Out + o];
        if (db) db[o] = sb;
        for (int i = 0; i < In; ++i) {
            double s = 0.0;
            for (int n = 0; n < N; ++n) s += dz[(size_t)n * Out + o] * a[(size_t)n * In + i];
            dw[(size_t)o * In + i] = s;
        }
    }
    if (da) {
#pragma omp parallel for schedule(static)
        for (int n = 0; n < N; ++n) {
            double *dr = da + (size_t)n * In;
            for (int i = 0; i < In; ++i) dr[i] = 0.0;
            for (int o = 0; o < Out; ++o) {
                const double d = dz[(size_t)n * Out + o];
                const double *wr = w + (size_t)o * In;
                for (int i = 0; i < In; ++i) dr[i] += d * wr[i];
            }
        }
    }
    return REF_OK;
}

/*
 * softmax(xs) = exp(xs) / sum(exp(xs)) over the K classes of each of the N
 * rows (listing "softmax").  Evaluated with the row maximum subtracted from
 * the exponent, which leaves the value unchanged in exact arithmetic.
 */
int ref_softmax(int N, int K, const double *z, double *p)
{
    if (!z || !p) return REF_ERR_NULL;
    if (N <= 0 || K <= 0) return REF_ERR_SHAPE;
    for (int n = 0; n < N; ++n) {
        const double *zr = z + (size_t)n * K;
        double *pr = p + (size_t)n * K;
        double m = zr[0];
        for (int k = 1; k < K; ++k) if (zr[k] > m) m = zr[k];
        double s = 0.0;
        for (int k = 0; k < K; ++k) { pr[k] = exp(zr[k] - m); s += pr[k]; }
        for (int k = 0; k < K; ++k) pr[k] /= s;
    }
    return REF_OK;
}

/*
 * Vector-Jacobian product of softmax: given u = dL/dp returns dL/dz,
 *   dz[n,j] = p[n,j] * ( u[n,j] - sum_k u[n,k] p[n,k] ).
 * With u = all ones (the paper's stand-in loss sum(m(x)), section "VGG19
 * backward pass") the result is identically zero.
 */
int ref_softmax_vjp(int N, int K, const double *p, const double *u, double *dz)
{
    if (!p || !u || !dz) return REF_ERR_NULL;
    if (N <= 0 || K <= 0) return REF_ERR_SHAPE;
    for (int n = 0; n < N; ++n) {
        double dot = 0.0;
        for (int k = 0; k < K; ++k) dot += u[(size_t)n * K + k] * p[(size_t)n * K + k];
        for (int k = 0; k < K; ++k)
            dz[(size_t)n * K + k] = p[(size_t)n * K + k] * (u[(size_t)n * K + k] - dot);
    }
    return REF_OK;
}

/*
 * Mean cross-entropy of softmax probabilities against integer labels and
 * its gradient with respect to the logits:
 *   L = -(1/N) sum_n log p[n,label[n]],   dz = (p - onehot(label)) / N.
 * loss and dz may each be NULL.
 */
int ref_softmax_xent(int N, int K, const double *p, const int32_t *labels, double *loss, double *dz)
{
    if (!p || !labels) return REF_ERR_NULL;
    if (N <= 0 || K <= 0) return REF_ERR_SHAPE;
    double L = 0.0;
    for (int n = 0; n < N; ++n) {
        const int y = labels[n];
        if (y < 0 || y >= K) return REF_ERR_SHAPE;
        L -= log(p[(size_t)n * K + y]);
        if (dz)
            for (int k = 0; k < K; ++k)
                dz[(size_t)n * K + k] = (p[(size_t)n * K + k] - (k == y ? 1.0 : 0.0)) / (double)N;
    }
    if (loss) *loss = L / (double)N;
    return REF_OK;
}

/* ReLU backward: g = dy where the forward output y is strictly positive, else 0. */
int ref_relu_bwd(size_t n, const double *y, const double *dy, double *g)
{
    if (!y || !dy || !g) return REF_ERR_NULL;
    for (size_t i = 0; i < n; ++i) g[i] = y[i] > 0.0 ? dy[i] : 0.0;
    return REF_OK;
}

/* Plain stochastic gradient descent: theta <- theta - lr * grad. */
int ref_sgd(size_t n, double *theta, const double *grad, double lr)
{
    if (!theta || !grad) return REF_ERR_NULL;
    for (size_t i = 0; i < n; ++i) theta[i] -= lr * grad[i];
    return REF_OK;
}
