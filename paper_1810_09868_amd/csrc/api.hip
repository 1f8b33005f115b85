// C ABI of libvgg_mi355x.so: argument validation on the host, then kernel
// launches; plus the two model-level launch sequences (section "VGG19 forward
// pass" / "VGG19 backward pass").
#include "common.h"
#include "flip_jobs.h"

#include <mutex>

#include <map>

namespace vgg {

bool raise_lds_limit(const void *kernel)
{
    // kernels whose limit has been raised in this process; guarded: entry points may be called from several threads
    static std::mutex mu;
    static std::map<const void *, bool> done;
    std::lock_guard<std::mutex> lock(mu);
    if (done.count(kernel)) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return false;
    done[kernel] = true;
    return true;
}

// kernels' host launchers (defined in the other translation units)
int conv3x3_igemm(int dtype, int N, int H, int W, int CinP, int Cout, const void *x, const void *w, const float *bias,
                  const void *mask, void *y, void *pool, unsigned char *argmax, int relu, void *part_ws, hipStream_t stream);
size_t conv3x3_igemm_workspace(int dtype, int N, int H, int W, int CinP, int Cout);
bool conv3x3_pool_fusable(int dtype, int H, int W, int Cout);
bool conv_first_pair_ok(int dtype, int H, int W);
int conv_first_pair(int N, int H, int W, int CinP1, const float *x, const void *w1, const float *b1, const void *w2,
                    const float *b2, void *y, void *pool, hipStream_t stream);
int conv_first(int dtype, int N, int H, int W, int CinP, const float *x, const void *w, const float *bias, void *y,
               int relu, hipStream_t stream);
void conv3x3_igemm_plan_info(int dtype, int N, int H, int W, int CinP, int Cout, bool pool, int info[7]);
size_t conv3x3_wgrad_workspace(int N, int H, int W, int Cin, int CinP, int Cout);
void conv3x3_wgrad_plan_info(int N, int H, int W, int Cin, int CinP, int Cout, int info[5]);
size_t conv3x3_wgrad_bf16_workspace(int N, int H, int W, int CinP, int Cout);
void conv3x3_wgrad_bf16_plan_info(int N, int H, int W, int CinP, int Cout, int info[5], int cin = 0);
int conv3x3_wgrad_bf16(int N, int H, int W, int CinP, int Cout, const bf16_t *x, const bf16_t *g, float *dw, float *db,
                       void *ws, size_t ws_bytes, hipStream_t stream, int x_channels = 0, int cin = 0);
// Channels per pixel of the NHWC copy of the images that the first layer's weight gradient reads: with bf16
// operands one 16-byte segment (the three channels and five zeros) instead of a whole 64-byte row.
inline int x0_channels(int dtype, int cinp0) { return dtype == VGG_BF16 ? 8 : cinp0; }
int conv3x3_wgrad(int N, int H, int W, int Cin, int CinP, int Cout, const float *x, const float *g, float *dw, float *db, void *ws,
                  size_t ws_bytes, hipStream_t stream);
size_t mfma_probe_sink_bytes();
int mfma_probe(int dtype, int random, int iters, float *sink, double *flops, hipStream_t stream);
int maxpool2x2(int dtype, int N, int H, int W, int C, const void *x, void *y, uint8_t *arg, hipStream_t s);
int maxpool2x2_bwd(int dtype, int N, int H, int W, int C, const void *dy, const uint8_t *arg, void *dx, hipStream_t s);
int softmax_rows(int N, int K, const float *z, float *p, hipStream_t s);
int softmax_xent_bwd(int N, int K, const float *p, const int32_t *labels, float *loss, float *dz, float *rowloss,
                     hipStream_t s);
int sgd_update(size_t n, float *theta, const float *grad, float lr, hipStream_t s);
int sgd_update_master(size_t n, float *theta, const float *grad, float lr, void *copy, int copy_dtype, hipStream_t s);
int sgd_update_master_conv(SgdConvJobs &jobs, float lr, hipStream_t s);
int nchw_to_nhwc(int dtype, int N, int C, int H, int W, int Cpad, const float *x, void *y, hipStream_t s);
int nhwc_to_nchw(int dtype, int N, int C, int H, int W, int Cpad, const void *x, float *y, hipStream_t s);
int pad_channels(int dtype, size_t pixels, int C, int Cpad, const void *x, void *y, hipStream_t s);
int convert(int sd, int dd, size_t n, const void *src, void *dst, hipStream_t s);
int pack_conv_w(int dtype, int Cin, int Cout, const float *w, void *dst, int flip, hipStream_t s, int colsP = 0);
int flip_packed_w(int dst_dtype, int CinP, int Cout, int CoutP, const float *src, void *dst, hipStream_t s);
int flip_packed_w_all(int dst_dtype, FlipJobs &jobs, hipStream_t s);
int unpack_conv_w(int Cin, int Cout, const float *src, float *w, hipStream_t s, int CinP = 0);
int permute_fc_cols(int dst_dtype, int Out, int C, int HW, int to_hwc, const float *src, void *dst, hipStream_t s);
size_t fc_workspace(int dtype, int N, int In, int Out);
int fc_forward(int dtype, int N, int In, int Out, const void *a, const void *w, const float *bias, void *z, int z_dtype,
               int relu, void *ws, hipStream_t s);
size_t fc_bwd_workspace(int N, int In, int Out);
int fc_backward(int N, int In, int Out, const float *a, const float *w, const float *dz, float *dw, float *db, float *da,
                int relu_mask, void *ws, hipStream_t s);
size_t fc_bwd_bf16_workspace(int N, int In, int Out);
int fc_backward_bf16(int N, int In, int Out, const bf16_t *a, const bf16_t *w, const float *dz, float *dw, float *db, float *da,
                     int relu_mask, void *ws, hipStream_t s);

namespace {

const int kConvCh[VGG19_NUM_CONV][2] = {{3, 64},    {64, 64},   {64, 128},  {128, 128}, {128, 256}, {256, 256},
                                        {256, 256}, {256, 256}, {256, 512}, {512, 512}, {512, 512}, {512, 512},
                                        {512, 512}, {512, 512}, {512, 512}, {512, 512}};
inline bool pool_after(int l) { return l == 1 || l == 3 || l == 7 || l == 11 || l == 15; }

bool cfg_ok(const vgg_config *c)
{
    return c && dtype_ok(c->dtype) && c->N > 0 && c->H > 0 && c->W > 0 && c->H % 32 == 0 && c->W % 32 == 0 &&
           c->fc_hidden > 0 && c->fc_hidden % 32 == 0 && c->classes > 0 &&
           (c->flags == 0 || (c->flags == VGG_FLAG_FP32_MASTER && c->dtype == VGG_BF16)) &&
           (long)c->N * c->H * c->W <= (1L << 27);
}

struct Bump {
    size_t off = 0;
    size_t take(size_t bytes) { const size_t o = off; off += round_up(bytes, 256); return o; }
};

// Offsets inside the packed parameter block.
struct PackedLayout {
    size_t conv_w[VGG19_NUM_CONV], conv_b[VGG19_NUM_CONV], fc_w[VGG19_NUM_FC], fc_b[VGG19_NUM_FC];
    int cinp[VGG19_NUM_CONV];
    int fc_in[VGG19_NUM_FC], fc_out[VGG19_NUM_FC];
    size_t total;
};

// master: the fp32 copy that a bf16 block with VGG_FLAG_FP32_MASTER carries behind it (same element
// order inside every tensor, i.e. the bf16 channel padding).
PackedLayout packed_layout(const vgg_config *c, bool master = false)
{
    PackedLayout L;
    Bump b;
    const int es = master ? 4 : dtype_size(c->dtype);
    for (int l = 0; l < VGG19_NUM_CONV; ++l) {
        L.cinp[l] = padded_channels(c->dtype, kConvCh[l][0]);
        L.conv_w[l] = b.take((size_t)9 * kConvCh[l][1] * L.cinp[l] * es);
    }
    for (int l = 0; l < VGG19_NUM_CONV; ++l) L.conv_b[l] = b.take((size_t)kConvCh[l][1] * 4);
    const int flat = 512 * (c->H / 32) * (c->W / 32);
    const int dims[4] = {flat, c->fc_hidden, c->fc_hidden, c->classes};
    for (int l = 0; l < VGG19_NUM_FC; ++l) {
        L.fc_in[l] = dims[l];
        L.fc_out[l] = dims[l + 1];
        L.fc_w[l] = b.take((size_t)dims[l] * dims[l + 1] * es);
    }
    for (int l = 0; l < VGG19_NUM_FC; ++l) L.fc_b[l] = b.take((size_t)dims[l + 1] * 4);
    L.total = b.off;
    return L;
}
inline bool has_master(const vgg_config *c) { return c->dtype == VGG_BF16 && c->flags == VGG_FLAG_FP32_MASTER; }
inline size_t packed_total(const vgg_config *c)
{
    return packed_layout(c).total + (has_master(c) ? packed_layout(c, true).total : 0);
}

// Workspace layout of the model-level calls.
struct WsLayout {
    size_t x0;                         // padded NHWC input
    size_t act[VGG19_NUM_CONV];        // conv outputs (training: all kept; inference: ping-pong)
    size_t pooled[VGG19_NUM_CONV];     // pool outputs (index = conv layer the pool follows)
    size_t argmax[VGG19_NUM_CONV];
    size_t z1, z2, logits, probs, fcws;
    size_t convpart;                   // partial sums of convolutions whose contraction is split
    // training only
    size_t dlogits, dz2, dz1, gA, gB, grads, wgws, fcbws, rowloss;
    size_t wflip[VGG19_NUM_CONV];      // data-gradient operands (flipped, transposed weights) of layers 1..15
    size_t dflat32;                    // bf16 training: fp32 gradient with respect to the flattened pool output
    size_t wgws_bytes;                 // size of the weight gradients' partial-sum buffer at wgws
    size_t total;
    int H[VGG19_NUM_CONV], W[VGG19_NUM_CONV];  // spatial size of each conv layer
};

WsLayout ws_layout(const vgg_config *c, const PackedLayout &P, bool training)
{
    WsLayout L;
    Bump b;
    const size_t es = dtype_size(c->dtype);
    const size_t N = c->N;
    int h = c->H, w = c->W;
    L.x0 = b.take(N * h * w * x0_channels(c->dtype, P.cinp[0]) * es);
    size_t max_act = 0;
    for (int l = 0; l < VGG19_NUM_CONV; ++l) {
        L.H[l] = h; L.W[l] = w;
        const size_t a = N * h * w * kConvCh[l][1] * es;
        if (a > max_act) max_act = a;
        if (pool_after(l)) { h /= 2; w /= 2; }
    }
    if (training) {
        for (int l = 0; l < VGG19_NUM_CONV; ++l) {
            const size_t elems = N * L.H[l] * L.W[l] * kConvCh[l][1];
            L.act[l] = b.take(elems * es);
            L.pooled[l] = L.argmax[l] = 0;
            if (pool_after(l)) {
                L.pooled[l] = b.take(elems / 4 * es);
                L.argmax[l] = b.take(elems / 4);
            }
        }
    } else {
        const size_t pA = b.take(max_act), pB = b.take(max_act);
        // forward ping-pong: every launch reads one buffer and writes the other.  A convolution with
        // the pool fused into its epilogue (see run_forward) writes only the pooled tensor, so that one
        // takes the place of the convolution's output; it must never share the buffer of the input,
        // which other workgroups of the same launch are still reading.
        int cur = 0;
        for (int l = 0; l < VGG19_NUM_CONV; ++l) {
            const bool fuse = l > 0 && pool_after(l) && conv3x3_pool_fusable(c->dtype, L.H[l], L.W[l], kConvCh[l][1]);
            L.act[l] = cur ? pB : pA; cur ^= 1;
            L.pooled[l] = L.argmax[l] = 0;
            if (fuse) L.pooled[l] = L.act[l];
            else if (pool_after(l)) { L.pooled[l] = cur ? pB : pA; cur ^= 1; }
        }
    }
    L.z1 = b.take(N * c->fc_hidden * es);
    L.z2 = b.take(N * c->fc_hidden * es);
    L.logits = b.take(N * c->classes * 4);
    L.probs = b.take(N * c->classes * 4);
    size_t fw = 0;
    for (int l = 0; l < VGG19_NUM_FC; ++l) {
        const size_t s = fc_workspace(c->dtype, c->N, P.fc_in[l], P.fc_out[l]);
        if (s > fw) fw = s;
    }
    L.fcws = b.take(fw);
    size_t cpart = 0;
    for (int l = 1; l < VGG19_NUM_CONV; ++l) {
        size_t s = conv3x3_igemm_workspace(c->dtype, c->N, L.H[l], L.W[l], P.cinp[l], kConvCh[l][1]);
        if (s > cpart) cpart = s;
        if (training) s = conv3x3_igemm_workspace(c->dtype, c->N, L.H[l], L.W[l], kConvCh[l][1], kConvCh[l][0]);
        if (s > cpart) cpart = s;
    }
    L.convpart = b.take(cpart);
    for (int l = 0; l < VGG19_NUM_CONV; ++l) L.wflip[l] = 0;
    L.dlogits = L.dz2 = L.dz1 = L.gA = L.gB = L.grads = L.wgws = L.fcbws = L.rowloss = L.dflat32 = L.wgws_bytes = 0;
    if (training) {
        L.dlogits = b.take(N * c->classes * 4);
        L.dz2 = b.take(N * c->fc_hidden * 4);
        L.dz1 = b.take(N * c->fc_hidden * 4);
        L.gA = b.take(max_act);
        L.gB = b.take(max_act);
        L.wflip[0] = 0;
        for (int l = 1; l < VGG19_NUM_CONV; ++l) L.wflip[l] = b.take((size_t)9 * P.cinp[l] * kConvCh[l][1] * es);
        const bool mixed = c->dtype == VGG_BF16;
        L.grads = b.take(mixed ? packed_layout(c, true).total : P.total);
        if (mixed) L.dflat32 = b.take(N * P.fc_in[0] * 4);
        size_t wg = 0, fb = 0;
        for (int l = 0; l < VGG19_NUM_CONV; ++l) {
            const size_t s = mixed ? conv3x3_wgrad_bf16_workspace(c->N, L.H[l], L.W[l], P.cinp[l], kConvCh[l][1])
                                   : conv3x3_wgrad_workspace(c->N, L.H[l], L.W[l], kConvCh[l][0], P.cinp[l], kConvCh[l][1]);
            if (s > wg) wg = s;
        }
        for (int l = 0; l < VGG19_NUM_FC; ++l) {
            const size_t s = mixed ? fc_bwd_bf16_workspace(c->N, P.fc_in[l], P.fc_out[l]) : fc_bwd_workspace(c->N, P.fc_in[l], P.fc_out[l]);
            if (s > fb) fb = s;
        }
        L.wgws = b.take(wg);
        L.wgws_bytes = wg;
        L.fcbws = b.take(fb);
        L.rowloss = b.take(N * 4);
    }
    L.total = b.off;
    return L;
}

// Records the launch plan and, unless dry, stops at the first failing launch.
struct Recorder {
    int *kinds; int cap; int n; bool dry; int rc;
    hipEvent_t *events = nullptr;  // when set (cap+1 events): one is recorded before every step
    hipStream_t stream = nullptr;
    bool skip(int kind)
    {
        if (rc != VGG_OK) return true;
        if (kinds && n < cap) kinds[n] = kind;
        if (events && !dry && n < cap && hipEventRecord(events[n], stream) != hipSuccess) rc = VGG_ERR_LAUNCH;
        ++n;
        return dry;
    }
};
#define VGG_STEP(rec, kind, call) do { if (!(rec).skip(kind)) (rec).rc = (call); } while (0)

enum { K_CONV = 1, K_DGRAD = 2, K_WGRAD = 3, K_POOL = 4, K_POOLB = 5, K_FC = 6, K_FCDW = 7, K_FCDA = 8, K_OTHER = 9 };

void run_forward(const vgg_config *c, const PackedLayout &P, const WsLayout &L, const float *x, const char *pk, float *logits,
                 float *probs, bool want_probs, char *ws, bool training, hipStream_t s, Recorder &rec)
{
    const int dt = c->dtype, N = c->N;
    // The first convolution reads the NCHW batch itself; training also keeps a channel-padded NHWC copy
    // of the images, which the first layer's weight gradient reads.
    if (training) VGG_STEP(rec, K_OTHER, nchw_to_nhwc(dt, N, 3, c->H, c->W, x0_channels(dt, P.cinp[0]), x, ws + L.x0, s));
    const char *cur = ws + L.x0;
    // Forward only, bf16, patch-tiled image sizes: the first two convolutions and the first pool run as one
    // kernel and the 64-channel full-resolution activations between and after them are never written (the
    // backward pass would need them, so the training step keeps the separate launches).
    const bool pair = !training && conv_first_pair_ok(dt, c->H, c->W);
    if (pair) {
        VGG_STEP(rec, K_CONV, conv_first_pair(N, c->H, c->W, P.cinp[0], x, pk + P.conv_w[0],
                                             reinterpret_cast<const float *>(pk + P.conv_b[0]), pk + P.conv_w[1],
                                             reinterpret_cast<const float *>(pk + P.conv_b[1]), nullptr, ws + L.pooled[1], s));
        rec.skip(K_CONV);  // the second convolution and the pool: in the launch above; listed so that the plan
        rec.skip(K_POOL);  // still shows sixteen convolutions and five pools
        cur = ws + L.pooled[1];
    }
    for (int l = pair ? 2 : 0; l < VGG19_NUM_CONV; ++l) {
        char *out = ws + L.act[l];
        // On patch-tiled layers the 2x2 maximum (and, for training, its position) is taken in the
        // convolution's epilogue and the un-pooled tensor is never written: the backward pass needs
        // only the pooled tensor (next layer's input and ReLU mask) and the positions.
        const bool fuse = l > 0 && pool_after(l) && conv3x3_pool_fusable(dt, L.H[l], L.W[l], kConvCh[l][1]);
        if (l == 0)   // (reads the NCHW batch itself; the padded NHWC copy above is only the weight gradient's operand)
            VGG_STEP(rec, K_CONV, conv_first(dt, N, c->H, c->W, P.cinp[0], x, pk + P.conv_w[0],
                                            reinterpret_cast<const float *>(pk + P.conv_b[0]), out, 1, s));
        else
            VGG_STEP(rec, K_CONV, conv3x3_igemm(dt, N, L.H[l], L.W[l], P.cinp[l], kConvCh[l][1], cur, pk + P.conv_w[l],
                                               reinterpret_cast<const float *>(pk + P.conv_b[l]), nullptr,
                                               fuse ? nullptr : out, fuse ? ws + L.pooled[l] : nullptr,
                                               fuse && training ? reinterpret_cast<uint8_t *>(ws + L.argmax[l]) : nullptr, 1,
                                               ws + L.convpart, s));
        cur = out;
        if (fuse) {
            rec.skip(K_POOL);  // fused into the launch above; listed so that the plan still shows five pools
            cur = ws + L.pooled[l];
        } else if (pool_after(l)) {
            char *po = ws + L.pooled[l];
            uint8_t *arg = training ? reinterpret_cast<uint8_t *>(ws + L.argmax[l]) : nullptr;
            VGG_STEP(rec, K_POOL, maxpool2x2(dt, N, L.H[l], L.W[l], kConvCh[l][1], cur, po, arg, s));
            cur = po;
        }
    }
    float *lg = logits ? logits : reinterpret_cast<float *>(ws + L.logits);
    VGG_STEP(rec, K_FC, fc_forward(dt, N, P.fc_in[0], P.fc_out[0], cur, pk + P.fc_w[0],
                                   reinterpret_cast<const float *>(pk + P.fc_b[0]), ws + L.z1, dt, 1, ws + L.fcws, s));
    VGG_STEP(rec, K_FC, fc_forward(dt, N, P.fc_in[1], P.fc_out[1], ws + L.z1, pk + P.fc_w[1],
                                   reinterpret_cast<const float *>(pk + P.fc_b[1]), ws + L.z2, dt, 1, ws + L.fcws, s));
    VGG_STEP(rec, K_FC, fc_forward(dt, N, P.fc_in[2], P.fc_out[2], ws + L.z2, pk + P.fc_w[2],
                                   reinterpret_cast<const float *>(pk + P.fc_b[2]), lg, VGG_F32, 0, ws + L.fcws, s));
    if (want_probs) {
        float *pr = probs ? probs : reinterpret_cast<float *>(ws + L.probs);
        VGG_STEP(rec, K_OTHER, softmax_rows(N, c->classes, lg, pr, s));
    }
}

void run_train(const vgg_config *c, const PackedLayout &P, const WsLayout &L, const float *x, const int32_t *labels, char *pk,
               const vgg19_params *grads_out, float *loss, float *logits, char *ws, hipStream_t s, Recorder &rec)
{
    const int N = c->N, dt = c->dtype;
    // bf16: operands (activations, gradients with respect to activations, working weights) are bf16,
    // sums fp32; the fp32 master parameters behind the bf16 block take the update.  The gradients with
    // respect to the dense layers' pre-activations stay fp32 between the dense layers and are rounded
    // to bf16 as they enter a product.
    const bool mixed = dt == VGG_BF16;
    const PackedLayout Pm = mixed ? packed_layout(c, true) : P;
    char *pm = mixed ? pk + P.total : pk;
    float *lg = logits ? logits : reinterpret_cast<float *>(ws + L.logits);
    float *pr = reinterpret_cast<float *>(ws + L.probs);
    run_forward(c, P, L, x, pk, lg, pr, true, ws, true, s, rec);
    char *gr = ws + L.grads;  // gradient block, same layout as the (master) parameters
    auto F = [](char *p) { return reinterpret_cast<float *>(p); };
    VGG_STEP(rec, K_OTHER, softmax_xent_bwd(N, c->classes, pr, labels, loss, F(ws + L.dlogits), F(ws + L.rowloss), s));
    // dense layers, last to first; each data gradient is masked by (input > 0)
    const char *fc_in[3] = {ws + L.pooled[15], ws + L.z1, ws + L.z2};
    float *fc_dz[3] = {F(ws + L.dz1), F(ws + L.dz2), F(ws + L.dlogits)};
    float *dflat = F(mixed ? ws + L.dflat32 : ws + L.gA);
    for (int l = 2; l >= 0; --l) {
        float *da = l == 0 ? dflat : fc_dz[l - 1];
        if (!rec.skip(K_FCDW)) {
            if (mixed)
                rec.rc = fc_backward_bf16(N, P.fc_in[l], P.fc_out[l], reinterpret_cast<const bf16_t *>(fc_in[l]),
                                          reinterpret_cast<const bf16_t *>(pk + P.fc_w[l]), fc_dz[l], F(gr + Pm.fc_w[l]),
                                          F(gr + Pm.fc_b[l]), da, 1, ws + L.fcbws, s);
            else
                rec.rc = fc_backward(N, P.fc_in[l], P.fc_out[l], reinterpret_cast<const float *>(fc_in[l]), F(pk + P.fc_w[l]),
                                     fc_dz[l], F(gr + P.fc_w[l]), F(gr + P.fc_b[l]), da, 1, ws + L.fcbws, s);
        }
        rec.skip(K_FCDA);  // issued by the same call; listed for the plan
    }
    if (mixed) VGG_STEP(rec, K_OTHER, convert(VGG_F32, VGG_BF16, (size_t)N * P.fc_in[0], dflat, ws + L.gA, s));
    // convolution stack, last to first.  The data gradients' operands first, all in one launch: the same
    // implicit GEMM runs on flipped, transposed weights.
    {
        FlipJobs jobs;
        jobs.n = 0;
        for (int l = 1; l < VGG19_NUM_CONV; ++l) {
            const int j = jobs.n++;
            jobs.src[j] = F(pm + Pm.conv_w[l]);
            jobs.dst[j] = ws + L.wflip[l];
            jobs.CinP[j] = P.cinp[l]; jobs.Cout[j] = kConvCh[l][1]; jobs.CoutP[j] = kConvCh[l][1];
        }
        VGG_STEP(rec, K_OTHER, flip_packed_w_all(dt, jobs, s));
    }
    char *gbuf[2] = {ws + L.gA, ws + L.gB};
    int cur = 0;  // gbuf[cur] holds the gradient w.r.t. the output of layer l (after its pool, if any)
    for (int l = VGG19_NUM_CONV - 1; l >= 0; --l) {
        const int H = L.H[l], W = L.W[l], Cin = kConvCh[l][0], Cout = kConvCh[l][1];
        if (pool_after(l)) {
            VGG_STEP(rec, K_POOLB, maxpool2x2_bwd(dt, N, H, W, Cout, gbuf[cur],
                                                  reinterpret_cast<const uint8_t *>(ws + L.argmax[l]), gbuf[cur ^ 1], s));
            cur ^= 1;
        }
        const char *xin = l == 0 ? ws + L.x0 : (pool_after(l - 1) ? ws + L.pooled[l - 1] : ws + L.act[l - 1]);
        if (mixed)
            VGG_STEP(rec, K_WGRAD, conv3x3_wgrad_bf16(N, H, W, P.cinp[l], Cout, reinterpret_cast<const bf16_t *>(xin),
                                                     reinterpret_cast<const bf16_t *>(gbuf[cur]), F(gr + Pm.conv_w[l]),
                                                     F(gr + Pm.conv_b[l]), ws + L.wgws, L.wgws_bytes, s,
                                                     l == 0 ? x0_channels(dt, P.cinp[0]) : 0, Cin));
        else
            VGG_STEP(rec, K_WGRAD, conv3x3_wgrad(N, H, W, kConvCh[l][0], P.cinp[l], Cout, reinterpret_cast<const float *>(xin),
                                                F(gbuf[cur]), F(gr + P.conv_w[l]), F(gr + P.conv_b[l]), ws + L.wgws,
                                                L.wgws_bytes, s));
        if (l > 0) {
            // data gradient = the same implicit GEMM with flipped, transposed weights; fused ReLU mask (x > 0)
            VGG_STEP(rec, K_DGRAD, conv3x3_igemm(dt, N, H, W, Cout, Cin, gbuf[cur], ws + L.wflip[l], nullptr, xin,
                                                gbuf[cur ^ 1], nullptr, nullptr, 0, ws + L.convpart, s));
            cur ^= 1;
        }
    }
    if (grads_out) {
        for (int l = 0; l < VGG19_NUM_CONV; ++l) {
            VGG_STEP(rec, K_OTHER, unpack_conv_w(kConvCh[l][0], kConvCh[l][1], F(gr + Pm.conv_w[l]), grads_out->conv_w[l], s,
                                                 Pm.cinp[l]));
            VGG_STEP(rec, K_OTHER, convert(VGG_F32, VGG_F32, kConvCh[l][1], gr + Pm.conv_b[l], grads_out->conv_b[l], s));
        }
        VGG_STEP(rec, K_OTHER, permute_fc_cols(VGG_F32, P.fc_out[0], 512, P.fc_in[0] / 512, 0, F(gr + Pm.fc_w[0]),
                                               grads_out->fc_w[0], s));
        for (int l = 1; l < VGG19_NUM_FC; ++l)
            VGG_STEP(rec, K_OTHER, convert(VGG_F32, VGG_F32, (size_t)P.fc_in[l] * P.fc_out[l], gr + Pm.fc_w[l], grads_out->fc_w[l], s));
        for (int l = 0; l < VGG19_NUM_FC; ++l)
            VGG_STEP(rec, K_OTHER, convert(VGG_F32, VGG_F32, P.fc_out[l], gr + Pm.fc_b[l], grads_out->fc_b[l], s));
    }
    if (!mixed) {
        VGG_STEP(rec, K_OTHER, sgd_update(P.total / 4, F(pk), F(gr), c->lr, s));
        return;
    }
    // master <- master - lr * gradient, working copy <- master (bf16 weights, fp32 biases).  Inside the two
    // blocks the tensors follow each other in the same order; where a group of tensors is laid out
    // proportionally (bf16 offsets exactly half the fp32 ones, which the 256-byte alignment gives whenever
    // every bf16 tensor size is a multiple of 256 bytes) the whole group, gaps included, takes one launch.
    auto group = [&](size_t m_first, size_t m_end, size_t w_first, size_t w_end, int copy_dtype) {
        const size_t n = (m_end - m_first) / 4;
        if ((w_end - w_first) * (copy_dtype == VGG_BF16 ? 2 : 1) != m_end - m_first || n % 4) return false;
        VGG_STEP(rec, K_OTHER, sgd_update_master(n, F(pm + m_first), F(gr + m_first), c->lr, pk + w_first, copy_dtype, s));
        return true;
    };
    bool fc_prop = true;
    for (int l = 0; l < VGG19_NUM_FC; ++l) fc_prop = fc_prop && Pm.fc_w[l] - Pm.fc_w[0] == 2 * (P.fc_w[l] - P.fc_w[0]);
    {
        // convolution weights: the bf16 copies are in the blocked layout, the masters row-major
        SgdConvJobs jobs;
        jobs.n = VGG19_NUM_CONV;
        for (int l = 0; l < VGG19_NUM_CONV; ++l) {
            jobs.theta[l] = F(pm + Pm.conv_w[l]);
            jobs.grad[l] = F(gr + Pm.conv_w[l]);
            jobs.copy[l] = reinterpret_cast<unsigned short *>(pk + P.conv_w[l]);
            jobs.Cout[l] = kConvCh[l][1]; jobs.CinP[l] = P.cinp[l];
        }
        VGG_STEP(rec, K_OTHER, sgd_update_master_conv(jobs, c->lr, s));
    }
    if (!group(Pm.conv_b[0], Pm.fc_w[0], P.conv_b[0], P.fc_w[0], VGG_F32))
        for (int l = 0; l < VGG19_NUM_CONV; ++l)
            VGG_STEP(rec, K_OTHER, sgd_update_master(kConvCh[l][1], F(pm + Pm.conv_b[l]), F(gr + Pm.conv_b[l]), c->lr,
                                                     pk + P.conv_b[l], VGG_F32, s));
    if (!(fc_prop && group(Pm.fc_w[0], Pm.fc_b[0], P.fc_w[0], P.fc_b[0], VGG_BF16)))
        for (int l = 0; l < VGG19_NUM_FC; ++l)
            VGG_STEP(rec, K_OTHER, sgd_update_master((size_t)P.fc_in[l] * P.fc_out[l], F(pm + Pm.fc_w[l]), F(gr + Pm.fc_w[l]),
                                                     c->lr, pk + P.fc_w[l], VGG_BF16, s));
    if (!group(Pm.fc_b[0], Pm.total, P.fc_b[0], P.total, VGG_F32))
        for (int l = 0; l < VGG19_NUM_FC; ++l) {
            // (bias counts need not be multiples of four: the plain kernels)
            VGG_STEP(rec, K_OTHER, sgd_update(P.fc_out[l], F(pm + Pm.fc_b[l]), F(gr + Pm.fc_b[l]), c->lr, s));
            VGG_STEP(rec, K_OTHER, convert(VGG_F32, VGG_F32, P.fc_out[l], pm + Pm.fc_b[l], pk + P.fc_b[l], s));
        }
}

bool params_ok(const vgg19_params *p)
{
    if (!p) return false;
    for (int l = 0; l < VGG19_NUM_CONV; ++l)
        if (!p->conv_w[l] || !p->conv_b[l]) return false;
    for (int l = 0; l < VGG19_NUM_FC; ++l)
        if (!p->fc_w[l] || !p->fc_b[l]) return false;
    return true;
}
bool params_aligned(const vgg19_params *p)
{
    for (int l = 0; l < VGG19_NUM_CONV; ++l)
        if (!aligned16(p->conv_w[l]) || !aligned16(p->conv_b[l])) return false;
    for (int l = 0; l < VGG19_NUM_FC; ++l)
        if (!aligned16(p->fc_w[l]) || !aligned16(p->fc_b[l])) return false;
    return true;
}

bool conv_shape_ok(int N, int H, int W, int Cin, int Cout)
{
    return N > 0 && H > 0 && W > 0 && Cin > 0 && Cout > 0 && (long)N * H * W <= (1L << 27) &&
           (long)N * H * W * (long)(Cin > Cout ? Cin : Cout) <= (1L << 33);
}

}  // namespace
}  // namespace vgg

using namespace vgg;

extern "C" {

const char *vgg_strerror(int status)
{
    switch (status) {
    case VGG_OK: return "ok";
    case VGG_ERR_NULL: return "null pointer";
    case VGG_ERR_SHAPE: return "bad shape";
    case VGG_ERR_DTYPE: return "bad dtype";
    case VGG_ERR_ALIGN: return "pointer not 16-byte aligned";
    case VGG_ERR_WORKSPACE: return "workspace missing or too small";
    case VGG_ERR_LAUNCH: return "kernel launch failed";
    case VGG_ERR_UNSUPPORTED: return "unsupported request";
    case VGG_ERR_TOO_LARGE: return "problem needs more scratch memory than the library's built-in buffer holds";
    default: return "unknown status";
    }
}

int vgg_padded_channels(int dtype, int C) { return (C > 0 && dtype_ok(dtype)) ? padded_channels(dtype, C) : 0; }

int vgg_conv_pack_weights(int dtype, int Cin, int Cout, const float *w_oihw, void *w_packed, int transpose_flip, void *stream)
{
    if (!w_oihw || !w_packed) return VGG_ERR_NULL;
    if (!dtype_ok(dtype)) return VGG_ERR_DTYPE;
    if (Cin <= 0 || Cout <= 0) return VGG_ERR_SHAPE;
    if (!aligned16(w_oihw) || !aligned16(w_packed)) return VGG_ERR_ALIGN;
    return pack_conv_w(dtype, Cin, Cout, w_oihw, w_packed, transpose_flip ? 1 : 0, (hipStream_t)stream);
}

int vgg_conv_unpack_weights(int Cin, int Cout, const float *w_packed, float *w_oihw, void *stream)
{
    if (!w_oihw || !w_packed) return VGG_ERR_NULL;
    if (Cin <= 0 || Cout <= 0) return VGG_ERR_SHAPE;
    if (!aligned16(w_oihw) || !aligned16(w_packed)) return VGG_ERR_ALIGN;
    return unpack_conv_w(Cin, Cout, w_packed, w_oihw, (hipStream_t)stream);
}

int vgg_nchw_to_nhwc(int dtype, int N, int C, int H, int W, int Cpad, const float *x, void *y, void *stream)
{
    if (!x || !y) return VGG_ERR_NULL;
    if (!dtype_ok(dtype)) return VGG_ERR_DTYPE;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || Cpad < C) return VGG_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(y)) return VGG_ERR_ALIGN;
    return nchw_to_nhwc(dtype, N, C, H, W, Cpad, x, y, (hipStream_t)stream);
}

int vgg_nhwc_to_nchw(int dtype, int N, int C, int H, int W, int Cpad, const void *x, float *y, void *stream)
{
    if (!x || !y) return VGG_ERR_NULL;
    if (!dtype_ok(dtype)) return VGG_ERR_DTYPE;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || Cpad < C) return VGG_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(y)) return VGG_ERR_ALIGN;
    return nhwc_to_nchw(dtype, N, C, H, W, Cpad, x, y, (hipStream_t)stream);
}

int vgg_convert(int sd, int dd, size_t n, const void *src, void *dst, void *stream)
{
    if (!src || !dst) return VGG_ERR_NULL;
    if (!dtype_ok(sd) || !dtype_ok(dd)) return VGG_ERR_DTYPE;
    if (n == 0) return VGG_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(dst)) return VGG_ERR_ALIGN;
    return convert(sd, dd, n, src, dst, (hipStream_t)stream);
}

size_t vgg_conv3x3_fwd_workspace_bytes(int dtype, int N, int H, int W, int Cin, int Cout)
{
    if (!dtype_ok(dtype) || !conv_shape_ok(N, H, W, Cin, Cout)) return 0;
    const int cp = padded_channels(dtype, Cin);
    const size_t pad = cp == Cin ? 0 : round_up((size_t)N * H * W * cp * dtype_size(dtype), 256);
    return pad + conv3x3_igemm_workspace(dtype, N, H, W, cp, Cout);
}

static int conv_fwd_common(int dtype, int N, int H, int W, int Cin, int Cout, const void *x, const void *w, const float *bias,
                           void *y, void *pooled, uint8_t *argmax, int relu, void *ws, size_t ws_bytes, void *stream)
{
    if (!x || !w || (!y && !pooled)) return VGG_ERR_NULL;
    if (!dtype_ok(dtype)) return VGG_ERR_DTYPE;
    if (!conv_shape_ok(N, H, W, Cin, Cout)) return VGG_ERR_SHAPE;
    if (pooled && !conv3x3_pool_fusable(dtype, H, W, Cout)) return VGG_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(w) || (y && !aligned16(y)) || (pooled && !aligned16(pooled)) || (ws && !aligned16(ws)))
        return VGG_ERR_ALIGN;
    const int cp = padded_channels(dtype, Cin);
    // (with the pool fused the contraction is never split: only the padded copy is needed then)
    const size_t part_bytes = pooled ? 0 : conv3x3_igemm_workspace(dtype, N, H, W, cp, Cout);
    const size_t need = vgg_conv3x3_fwd_workspace_bytes(dtype, N, H, W, Cin, Cout) - (pooled ? conv3x3_igemm_workspace(dtype, N, H, W, cp, Cout) : 0);
    if (need && (!ws || ws_bytes < need)) return VGG_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    char *part = static_cast<char *>(ws);  // [padded copy of x][partial sums], either may be empty
    if (cp != Cin) {
        const int rc = pad_channels(dtype, (size_t)N * H * W, Cin, cp, x, ws, s);
        if (rc) return rc;
        x = ws;
        part += round_up((size_t)N * H * W * cp * dtype_size(dtype), 256);
    }
    if (!part_bytes) part = nullptr;
    return conv3x3_igemm(dtype, N, H, W, cp, Cout, x, w, bias, nullptr, y, pooled, argmax, relu ? 1 : 0, part, s);
}

int vgg_conv3x3_fwd(int dtype, int N, int H, int W, int Cin, int Cout, const void *x, const void *w, const float *bias,
                    void *y, int relu, void *ws, size_t ws_bytes, void *stream)
{
    if (!y) return VGG_ERR_NULL;
    return conv_fwd_common(dtype, N, H, W, Cin, Cout, x, w, bias, y, nullptr, nullptr, relu, ws, ws_bytes, stream);
}

int vgg_conv3x3_fwd_pool(int dtype, int N, int H, int W, int Cin, int Cout, const void *x, const void *w, const float *bias,
                         void *y_or_null, void *pooled, uint8_t *argmax_or_null, int relu, void *ws, size_t ws_bytes,
                         void *stream)
{
    if (!pooled) return VGG_ERR_NULL;
    return conv_fwd_common(dtype, N, H, W, Cin, Cout, x, w, bias, y_or_null, pooled, argmax_or_null, relu, ws, ws_bytes, stream);
}

int vgg_conv3x3_fwd_first(int dtype, int N, int H, int W, const float *x_nchw, const void *w, const float *bias, void *y,
                          int relu, void *stream)
{
    if (!x_nchw || !w || !y) return VGG_ERR_NULL;
    if (!dtype_ok(dtype)) return VGG_ERR_DTYPE;
    if (!conv_shape_ok(N, H, W, 3, 64)) return VGG_ERR_SHAPE;
    if (!aligned16(x_nchw) || !aligned16(w) || !aligned16(y)) return VGG_ERR_ALIGN;
    return conv_first(dtype, N, H, W, padded_channels(dtype, 3), x_nchw, w, bias, y, relu ? 1 : 0, (hipStream_t)stream);
}

int vgg_conv3x3_fwd_first_pair(int dtype, int N, int H, int W, const float *x_nchw, const void *w1, const float *bias1,
                               const void *w2, const float *bias2, void *y2_or_null, void *pooled_or_null, void *stream)
{
    if (!x_nchw || !w1 || !w2 || (!y2_or_null && !pooled_or_null)) return VGG_ERR_NULL;
    if (!dtype_ok(dtype)) return VGG_ERR_DTYPE;
    if (!conv_shape_ok(N, H, W, 3, 64)) return VGG_ERR_SHAPE;
    if (!conv_first_pair_ok(dtype, H, W)) return VGG_ERR_UNSUPPORTED;
    if (!aligned16(x_nchw) || !aligned16(w1) || !aligned16(w2) || !aligned16(y2_or_null) || !aligned16(pooled_or_null) ||
        !aligned16(bias2))
        return VGG_ERR_ALIGN;
    return conv_first_pair(N, H, W, padded_channels(dtype, 3), x_nchw, w1, bias1, w2, bias2, y2_or_null, pooled_or_null,
                           (hipStream_t)stream);
}

size_t vgg_conv3x3_bwd_data_workspace_bytes(int dtype, int N, int H, int W, int Cin, int Cout)
{
    if (!dtype_ok(dtype) || !conv_shape_ok(N, H, W, Cin, Cout)) return 0;
    const int cp = padded_channels(dtype, Cout);
    const size_t pad = cp == Cout ? 0 : round_up((size_t)N * H * W * cp * dtype_size(dtype), 256);
    return pad + conv3x3_igemm_workspace(dtype, N, H, W, cp, Cin);
}

int vgg_conv3x3_bwd_data(int dtype, int N, int H, int W, int Cin, int Cout, const void *g, const void *w_tf,
                         const void *relu_src, void *dx, void *ws, size_t ws_bytes, void *stream)
{
    if (!g || !w_tf || !dx) return VGG_ERR_NULL;
    if (!dtype_ok(dtype)) return VGG_ERR_DTYPE;
    if (!conv_shape_ok(N, H, W, Cin, Cout)) return VGG_ERR_SHAPE;
    if (!aligned16(g) || !aligned16(w_tf) || !aligned16(dx) || (relu_src && !aligned16(relu_src)) || (ws && !aligned16(ws)))
        return VGG_ERR_ALIGN;
    const size_t need = vgg_conv3x3_bwd_data_workspace_bytes(dtype, N, H, W, Cin, Cout);
    if (need && (!ws || ws_bytes < need)) return VGG_ERR_WORKSPACE;
    const int cp = padded_channels(dtype, Cout);
    hipStream_t s = (hipStream_t)stream;
    char *part = static_cast<char *>(ws);  // [padded copy of g][partial sums], either may be empty
    if (cp != Cout) {
        const int rc = pad_channels(dtype, (size_t)N * H * W, Cout, cp, g, ws, s);
        if (rc) return rc;
        g = ws;
        part += round_up((size_t)N * H * W * cp * dtype_size(dtype), 256);
    }
    if (!conv3x3_igemm_workspace(dtype, N, H, W, cp, Cin)) part = nullptr;
    return conv3x3_igemm(dtype, N, H, W, cp, Cin, g, w_tf, nullptr, relu_src, dx, nullptr, nullptr, 0, part, s);
}

size_t vgg_conv3x3_bwd_weight_workspace_bytes(int dtype, int N, int H, int W, int Cin, int Cout)
{
    if (!dtype_ok(dtype) || !conv_shape_ok(N, H, W, Cin, Cout)) return 0;
    const int cp = padded_channels(dtype, Cin);
    size_t pad = cp == Cin ? 0 : round_up((size_t)N * H * W * cp * dtype_size(dtype), 256);
    return pad + (dtype == VGG_F32 ? conv3x3_wgrad_workspace(N, H, W, Cin, cp, Cout) : conv3x3_wgrad_bf16_workspace(N, H, W, cp, Cout));
}

int vgg_conv3x3_bwd_weight(int dtype, int N, int H, int W, int Cin, int Cout, const void *x, const void *g, float *dw,
                           float *db, void *ws, size_t ws_bytes, void *stream)
{
    if (!x || !g || !dw) return VGG_ERR_NULL;
    if (!dtype_ok(dtype)) return VGG_ERR_DTYPE;
    if (!conv_shape_ok(N, H, W, Cin, Cout)) return VGG_ERR_SHAPE;
    if (Cout % (dtype == VGG_F32 ? 4 : 8)) return VGG_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(g) || !aligned16(dw) || (db && !aligned16(db)) || (ws && !aligned16(ws))) return VGG_ERR_ALIGN;
    const size_t need = vgg_conv3x3_bwd_weight_workspace_bytes(dtype, N, H, W, Cin, Cout);
    if (!ws || ws_bytes < need) return VGG_ERR_WORKSPACE;
    const int cp = padded_channels(dtype, Cin);
    hipStream_t s = (hipStream_t)stream;
    char *wsp = static_cast<char *>(ws);
    int xc = 0;   // channels per pixel of the padded copy when fewer than cp (bf16, at most three channels: one 16-byte segment)
    if (cp != Cin) {
        const int to = dtype == VGG_BF16 && Cin <= 3 ? x0_channels(dtype, cp) : cp;
        const int rc = pad_channels(dtype, (size_t)N * H * W, Cin, to, x, wsp, s);
        if (rc) return rc;
        x = wsp;
        if (to != cp) xc = to;
        const size_t pad = round_up((size_t)N * H * W * cp * dtype_size(dtype), 256);   // (as the workspace query reserves it)
        wsp += pad;
        ws_bytes -= pad;
    }
    // (the launchers compare what is left of the workspace with the partial sums of the plan they run)
    if (dtype == VGG_BF16)
        return conv3x3_wgrad_bf16(N, H, W, cp, Cout, static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(g), dw, db, wsp,
                                  ws_bytes, s, xc, Cin);
    return conv3x3_wgrad(N, H, W, Cin, cp, Cout, static_cast<const float *>(x), static_cast<const float *>(g), dw, db, wsp,
                         ws_bytes, s);
}

int vgg_maxpool2x2(int dtype, int N, int H, int W, int C, const void *x, void *y, uint8_t *argmax, void *stream)
{
    if (!x || !y) return VGG_ERR_NULL;
    if (!dtype_ok(dtype)) return VGG_ERR_DTYPE;
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || (H & 1) || (W & 1) || C % 8) return VGG_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(y)) return VGG_ERR_ALIGN;
    return maxpool2x2(dtype, N, H, W, C, x, y, argmax, (hipStream_t)stream);
}

int vgg_maxpool2x2_bwd(int dtype, int N, int H, int W, int C, const void *dy, const uint8_t *argmax, void *dx, void *stream)
{
    if (!dy || !argmax || !dx) return VGG_ERR_NULL;
    if (!dtype_ok(dtype)) return VGG_ERR_DTYPE;
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0 || (H & 1) || (W & 1) || C % 8) return VGG_ERR_SHAPE;
    if (!aligned16(dy) || !aligned16(dx)) return VGG_ERR_ALIGN;
    return maxpool2x2_bwd(dtype, N, H, W, C, dy, argmax, dx, (hipStream_t)stream);
}

size_t vgg_fc_workspace_bytes(int dtype, int N, int In, int Out)
{
    if (!dtype_ok(dtype) || N <= 0 || In <= 0 || Out <= 0) return 0;
    return fc_workspace(dtype, N, In, Out);
}

int vgg_fc(int dtype, int N, int In, int Out, const void *a, const void *w, const float *bias, void *z, int z_dtype, int relu,
           void *ws, size_t ws_bytes, void *stream)
{
    if (!a || !w || !z) return VGG_ERR_NULL;
    if (!dtype_ok(dtype) || !dtype_ok(z_dtype)) return VGG_ERR_DTYPE;
    if (N <= 0 || In <= 0 || Out <= 0) return VGG_ERR_SHAPE;
    if (!aligned16(a) || !aligned16(w) || !aligned16(z) || (ws && !aligned16(ws))) return VGG_ERR_ALIGN;
    if (!ws || ws_bytes < fc_workspace(dtype, N, In, Out)) return VGG_ERR_WORKSPACE;
    return fc_forward(dtype, N, In, Out, a, w, bias, z, z_dtype, relu ? 1 : 0, ws, (hipStream_t)stream);
}

// ---- vgg_fc for callers that cannot allocate: the partial sums of the split contraction go to a buffer
// that is part of the library's device image instead of a caller's workspace.
static __device__ __align__(256) unsigned char scratch[VGG_FC_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];   // per device: address of that device's copy of `scratch`
std::mutex g_scratch_mutex;

// Device address of the current device's copy of the buffer, looked up once per device.  (In host code the
// array's name is only a handle for this lookup, never an address a kernel could use.)
int scratch_of_current_device(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return VGG_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return VGG_ERR_LAUNCH;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return VGG_OK;
}
}  // namespace

int vgg_fc_static(int dtype, int N, int In, int Out, const void *a, const void *w, const float *bias, void *z, int z_dtype,
                  int relu, void *stream)
{
    if (!a || !w || !z) return VGG_ERR_NULL;
    if (!dtype_ok(dtype) || !dtype_ok(z_dtype)) return VGG_ERR_DTYPE;
    if (N <= 0 || In <= 0 || Out <= 0) return VGG_ERR_SHAPE;
    if (!aligned16(a) || !aligned16(w) || !aligned16(z)) return VGG_ERR_ALIGN;
    if (fc_workspace(dtype, N, In, Out) > (size_t)VGG_FC_STATIC_SCRATCH_BYTES) return VGG_ERR_TOO_LARGE;
    void *ptr = nullptr;
    const int rc = scratch_of_current_device(&ptr);
    if (rc != VGG_OK) return rc;
    // (every partial sum the second kernel reads is written by the first: nothing to clear between calls)
    return fc_forward(dtype, N, In, Out, a, w, bias, z, z_dtype, relu ? 1 : 0, ptr, (hipStream_t)stream);
}

size_t vgg_fc_bwd_workspace_bytes(int dtype, int N, int In, int Out)
{
    if (!dtype_ok(dtype) || N <= 0 || In <= 0 || Out <= 0 || (dtype == VGG_BF16 && In % 8)) return 0;
    return dtype == VGG_F32 ? fc_bwd_workspace(N, In, Out) : fc_bwd_bf16_workspace(N, In, Out);
}

int vgg_fc_bwd(int dtype, int N, int In, int Out, const void *a, const void *w, const void *dz, float *dw, float *db, void *da,
               int relu_mask, void *ws, size_t ws_bytes, void *stream)
{
    if (!a || !w || !dz || !dw) return VGG_ERR_NULL;
    if (!dtype_ok(dtype)) return VGG_ERR_DTYPE;
    if (N <= 0 || In <= 0 || Out <= 0) return VGG_ERR_SHAPE;
    if (dtype == VGG_BF16 && In % 8) return VGG_ERR_UNSUPPORTED;   // 16-byte segments of bf16 rows
    if (!aligned16(a) || !aligned16(w) || !aligned16(dz) || !aligned16(dw) || (da && !aligned16(da)) || (ws && !aligned16(ws)))
        return VGG_ERR_ALIGN;
    // (bf16: the rounded copy of dz lives in the workspace, so it is needed even without da)
    if ((da || dtype == VGG_BF16) && (!ws || ws_bytes < vgg_fc_bwd_workspace_bytes(dtype, N, In, Out))) return VGG_ERR_WORKSPACE;
    if (dtype == VGG_BF16)
        return fc_backward_bf16(N, In, Out, static_cast<const bf16_t *>(a), static_cast<const bf16_t *>(w),
                                static_cast<const float *>(dz), dw, db, static_cast<float *>(da), relu_mask ? 1 : 0, ws,
                                (hipStream_t)stream);
    return fc_backward(N, In, Out, static_cast<const float *>(a), static_cast<const float *>(w), static_cast<const float *>(dz),
                       dw, db, static_cast<float *>(da), relu_mask ? 1 : 0, ws, (hipStream_t)stream);
}

int vgg_softmax(int N, int K, const float *z, float *p, void *stream)
{
    if (!z || !p) return VGG_ERR_NULL;
    if (N <= 0 || K <= 0) return VGG_ERR_SHAPE;
    return softmax_rows(N, K, z, p, (hipStream_t)stream);
}

int vgg_softmax_xent_bwd(int N, int K, const float *p, const int32_t *labels, float *loss, float *dz, void *ws, size_t ws_bytes,
                         void *stream)
{
    if (!p || !labels) return VGG_ERR_NULL;
    if (N <= 0 || K <= 0) return VGG_ERR_SHAPE;
    if (loss && (!ws || ws_bytes < (size_t)N * 4)) return VGG_ERR_WORKSPACE;
    return softmax_xent_bwd(N, K, p, labels, loss, dz, static_cast<float *>(ws), (hipStream_t)stream);
}

int vgg_sgd_update(size_t n, float *theta, const float *grad, float lr, void *stream)
{
    if (!theta || !grad) return VGG_ERR_NULL;
    if (n == 0) return VGG_ERR_SHAPE;
    if (!aligned16(theta) || !aligned16(grad)) return VGG_ERR_ALIGN;
    return sgd_update(n, theta, grad, lr, (hipStream_t)stream);
}

size_t vgg19_packed_bytes(const vgg_config *cfg) { return cfg_ok(cfg) ? packed_total(cfg) : 0; }

size_t vgg19_forward_workspace_bytes(const vgg_config *cfg)
{
    if (!cfg_ok(cfg)) return 0;
    return ws_layout(cfg, packed_layout(cfg), false).total;
}

size_t vgg19_train_workspace_bytes(const vgg_config *cfg)
{
    if (!cfg_ok(cfg) || (cfg->dtype != VGG_F32 && !has_master(cfg))) return 0;
    return ws_layout(cfg, packed_layout(cfg), true).total;
}

int vgg19_pack_params(const vgg_config *cfg, const vgg19_params *canon, void *packed, size_t packed_bytes, void *stream)
{
    if (!cfg || !canon || !packed) return VGG_ERR_NULL;
    if (!dtype_ok(cfg->dtype)) return VGG_ERR_DTYPE;
    if (!cfg_ok(cfg)) return VGG_ERR_SHAPE;
    if (!params_ok(canon)) return VGG_ERR_NULL;
    if (!aligned16(packed) || !params_aligned(canon)) return VGG_ERR_ALIGN;
    if (packed_bytes < packed_total(cfg)) return VGG_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    int rc = VGG_OK;
    // the block in cfg->dtype, then (bf16 with fp32 master) the same tensors in fp32 behind it
    for (int pass = 0; pass < (has_master(cfg) ? 2 : 1) && !rc; ++pass) {
        const PackedLayout P = packed_layout(cfg, pass == 1);
        const int dt = pass == 1 ? VGG_F32 : cfg->dtype;
        char *pk = static_cast<char *>(packed) + (pass == 1 ? packed_layout(cfg).total : 0);
        for (int l = 0; l < VGG19_NUM_CONV && !rc; ++l) {
            rc = pack_conv_w(dt, kConvCh[l][0], kConvCh[l][1], canon->conv_w[l], pk + P.conv_w[l], 0, s, P.cinp[l]);
            if (!rc) rc = convert(VGG_F32, VGG_F32, kConvCh[l][1], canon->conv_b[l], pk + P.conv_b[l], s);
        }
        if (!rc) rc = permute_fc_cols(dt, P.fc_out[0], 512, P.fc_in[0] / 512, 1, canon->fc_w[0], pk + P.fc_w[0], s);
        for (int l = 1; l < VGG19_NUM_FC && !rc; ++l)
            rc = convert(VGG_F32, dt, (size_t)P.fc_in[l] * P.fc_out[l], canon->fc_w[l], pk + P.fc_w[l], s);
        for (int l = 0; l < VGG19_NUM_FC && !rc; ++l) rc = convert(VGG_F32, VGG_F32, P.fc_out[l], canon->fc_b[l], pk + P.fc_b[l], s);
    }
    return rc;
}

int vgg19_unpack_params(const vgg_config *cfg, const void *packed, size_t packed_bytes, const vgg19_params *out, void *stream)
{
    if (!cfg || !out || !packed) return VGG_ERR_NULL;
    if (!dtype_ok(cfg->dtype)) return VGG_ERR_DTYPE;
    if (!cfg_ok(cfg)) return VGG_ERR_SHAPE;
    if (cfg->dtype != VGG_F32 && !has_master(cfg)) return VGG_ERR_UNSUPPORTED;
    if (!params_ok(out)) return VGG_ERR_NULL;
    if (!aligned16(packed) || !params_aligned(out)) return VGG_ERR_ALIGN;
    if (packed_bytes < packed_total(cfg)) return VGG_ERR_WORKSPACE;
    // (bf16 with fp32 master: the master copy is what is read back)
    const PackedLayout P = packed_layout(cfg, has_master(cfg));
    hipStream_t s = (hipStream_t)stream;
    const char *pk = static_cast<const char *>(packed) + (has_master(cfg) ? packed_layout(cfg).total : 0);
    int rc = VGG_OK;
    for (int l = 0; l < VGG19_NUM_CONV && !rc; ++l) {
        rc = unpack_conv_w(kConvCh[l][0], kConvCh[l][1], reinterpret_cast<const float *>(pk + P.conv_w[l]), out->conv_w[l], s,
                           P.cinp[l]);
        if (!rc) rc = convert(VGG_F32, VGG_F32, kConvCh[l][1], pk + P.conv_b[l], out->conv_b[l], s);
    }
    if (!rc)
        rc = permute_fc_cols(VGG_F32, P.fc_out[0], 512, P.fc_in[0] / 512, 0, reinterpret_cast<const float *>(pk + P.fc_w[0]),
                             out->fc_w[0], s);
    for (int l = 1; l < VGG19_NUM_FC && !rc; ++l)
        rc = convert(VGG_F32, VGG_F32, (size_t)P.fc_in[l] * P.fc_out[l], pk + P.fc_w[l], out->fc_w[l], s);
    for (int l = 0; l < VGG19_NUM_FC && !rc; ++l) rc = convert(VGG_F32, VGG_F32, P.fc_out[l], pk + P.fc_b[l], out->fc_b[l], s);
    return rc;
}

int vgg19_forward(const vgg_config *cfg, const float *x, const void *packed, float *logits, float *probs, void *ws,
                  size_t ws_bytes, void *stream)
{
    if (!cfg || !x || !packed) return VGG_ERR_NULL;
    if (!dtype_ok(cfg->dtype)) return VGG_ERR_DTYPE;
    if (!cfg_ok(cfg)) return VGG_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(packed) || (logits && !aligned16(logits)) || (probs && !aligned16(probs)) ||
        (ws && !aligned16(ws)))
        return VGG_ERR_ALIGN;
    const PackedLayout P = packed_layout(cfg);
    const WsLayout L = ws_layout(cfg, P, false);
    if (!ws || ws_bytes < L.total) return VGG_ERR_WORKSPACE;
    Recorder rec{nullptr, 0, 0, false, VGG_OK};
    run_forward(cfg, P, L, x, static_cast<const char *>(packed), logits, probs, probs != nullptr, static_cast<char *>(ws),
                false, (hipStream_t)stream, rec);
    return rec.rc;
}

int vgg19_train_step(const vgg_config *cfg, const float *x, const int32_t *labels, void *packed, size_t packed_bytes,
                     const vgg19_params *grads, float *loss, float *logits, void *ws, size_t ws_bytes, void *stream)
{
    if (!cfg || !x || !labels || !packed) return VGG_ERR_NULL;
    if (!dtype_ok(cfg->dtype)) return VGG_ERR_DTYPE;
    if (!cfg_ok(cfg)) return VGG_ERR_SHAPE;
    if (cfg->dtype != VGG_F32 && !has_master(cfg)) return VGG_ERR_UNSUPPORTED;
    if (grads && !params_ok(grads)) return VGG_ERR_NULL;
    if (!aligned16(x) || !aligned16(packed) || (logits && !aligned16(logits)) || (ws && !aligned16(ws)) ||
        (grads && !params_aligned(grads)))
        return VGG_ERR_ALIGN;
    const PackedLayout P = packed_layout(cfg);
    if (packed_bytes < packed_total(cfg)) return VGG_ERR_WORKSPACE;
    const WsLayout L = ws_layout(cfg, P, true);
    if (!ws || ws_bytes < L.total) return VGG_ERR_WORKSPACE;
    Recorder rec{nullptr, 0, 0, false, VGG_OK};
    run_train(cfg, P, L, x, labels, static_cast<char *>(packed), grads, loss, logits, static_cast<char *>(ws),
              (hipStream_t)stream, rec);
    return rec.rc;
}

int vgg19_timed(const vgg_config *cfg, int training, const float *x, const int32_t *labels, void *packed,
                size_t packed_bytes, float *logits, void *ws, size_t ws_bytes, int *kinds_host, float *ms_host, int cap,
                void *stream)
{
    if (!cfg || !x || !packed || !kinds_host || !ms_host || (training && !labels)) return VGG_ERR_NULL;
    if (!dtype_ok(cfg->dtype)) return VGG_ERR_DTYPE;
    if (!cfg_ok(cfg) || cap <= 0) return VGG_ERR_SHAPE;
    if (training && cfg->dtype != VGG_F32 && !has_master(cfg)) return VGG_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(packed) || (logits && !aligned16(logits)) || (ws && !aligned16(ws))) return VGG_ERR_ALIGN;
    const PackedLayout P = packed_layout(cfg);
    if (packed_bytes < (training ? packed_total(cfg) : P.total)) return VGG_ERR_WORKSPACE;
    const WsLayout L = ws_layout(cfg, P, training != 0);
    if (!ws || ws_bytes < L.total) return VGG_ERR_WORKSPACE;
    const int need = vgg19_plan(cfg, training, nullptr, 0);
    if (need < 0) return need;
    if (cap < need) return VGG_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t *ev = new hipEvent_t[need + 1];
    int made = 0;
    int rc = VGG_OK;
    for (; made <= need; ++made)
        if (hipEventCreate(&ev[made]) != hipSuccess) { rc = VGG_ERR_LAUNCH; break; }
    if (rc == VGG_OK) {
        Recorder rec{kinds_host, need, 0, false, VGG_OK};
        rec.events = ev;
        rec.stream = s;
        if (training)
            run_train(cfg, P, L, x, labels, static_cast<char *>(packed), nullptr, nullptr, logits, static_cast<char *>(ws), s, rec);
        else
            run_forward(cfg, P, L, x, static_cast<const char *>(packed), logits, nullptr, true, static_cast<char *>(ws), false, s, rec);
        rc = rec.rc;
        if (rc == VGG_OK && (hipEventRecord(ev[need], s) != hipSuccess || hipEventSynchronize(ev[need]) != hipSuccess))
            rc = VGG_ERR_LAUNCH;
        for (int i = 0; i < need && rc == VGG_OK; ++i)
            if (hipEventElapsedTime(&ms_host[i], ev[i], ev[i + 1]) != hipSuccess) rc = VGG_ERR_LAUNCH;
        if (rc == VGG_OK) rc = need;
    }
    for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
    delete[] ev;
    return rc;
}

int vgg19_plan(const vgg_config *cfg, int training, int *kinds_host, int cap)
{
    if (!cfg) return VGG_ERR_NULL;
    if (!dtype_ok(cfg->dtype)) return VGG_ERR_DTYPE;
    if (!cfg_ok(cfg)) return VGG_ERR_SHAPE;
    if (training && cfg->dtype != VGG_F32 && !has_master(cfg)) return VGG_ERR_UNSUPPORTED;
    const PackedLayout P = packed_layout(cfg);
    const WsLayout L = ws_layout(cfg, P, training != 0);
    Recorder rec{kinds_host, kinds_host ? cap : 0, 0, true, VGG_OK};
    if (training)
        run_train(cfg, P, L, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, rec);
    else
        run_forward(cfg, P, L, nullptr, nullptr, nullptr, nullptr, true, nullptr, false, nullptr, rec);
    return rec.n;
}

int vgg_conv3x3_plan(int op, int dtype, int N, int H, int W, int Cin, int Cout, int *info_host, int cap)
{
    if (!info_host) return VGG_ERR_NULL;
    if (!dtype_ok(dtype)) return VGG_ERR_DTYPE;
    if (!conv_shape_ok(N, H, W, Cin, Cout) || op < VGG_PLAN_FWD || op > VGG_PLAN_BWD_WEIGHT || cap < VGG_PLAN_INFO_LEN)
        return VGG_ERR_SHAPE;
    int info[VGG_PLAN_INFO_LEN] = {0, 0, 0, 0, 0, 1, 0};
    if (op == VGG_PLAN_BWD_WEIGHT) {
        int w[5];
        const int cp = padded_channels(dtype, Cin);
        if (dtype == VGG_F32) conv3x3_wgrad_plan_info(N, H, W, Cin, cp, Cout, w);
        else conv3x3_wgrad_bf16_plan_info(N, H, W, cp, Cout, w, Cin);
        info[0] = 100 + w[0];
        info[1] = w[0] == 14 ? 56 : 64;
        info[2] = 64;
        info[3] = (w[0] == 0 || w[0] == 3) ? 0 : 1;
        info[4] = w[1];
        info[5] = w[2];
        info[6] = w[4];
    } else if (op == VGG_PLAN_FWD_POOL && !conv3x3_pool_fusable(dtype, H, W, Cout)) {
        return VGG_ERR_UNSUPPORTED;
    } else if (op == VGG_PLAN_BWD_DATA) {
        conv3x3_igemm_plan_info(dtype, N, H, W, padded_channels(dtype, Cout), Cin, false, info);
    } else {
        conv3x3_igemm_plan_info(dtype, N, H, W, padded_channels(dtype, Cin), Cout, op == VGG_PLAN_FWD_POOL, info);
    }
    for (int i = 0; i < VGG_PLAN_INFO_LEN; ++i) info_host[i] = info[i];
    return VGG_OK;
}

size_t vgg_mfma_probe_sink_bytes(void) { return mfma_probe_sink_bytes(); }

int vgg_mfma_probe(int dtype, int random_operands, int iters, float *sink, size_t sink_bytes, double *flops_host,
                   void *stream)
{
    if (!sink) return VGG_ERR_NULL;
    if (!dtype_ok(dtype)) return VGG_ERR_DTYPE;
    if (iters <= 0 || random_operands < 0 || random_operands > 3) return VGG_ERR_SHAPE;
    if ((random_operands & 2) && dtype != VGG_BF16) return VGG_ERR_UNSUPPORTED;
    if (!aligned16(sink)) return VGG_ERR_ALIGN;
    if (sink_bytes < mfma_probe_sink_bytes()) return VGG_ERR_WORKSPACE;
    return mfma_probe(dtype, random_operands, iters, sink, flops_host, (hipStream_t)stream);
}

}  // extern "C"
