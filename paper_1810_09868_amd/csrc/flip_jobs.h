// Arguments of the batched weight flip (flip_packed_w_all in pointwise.hip): tensor j is [9][Cout][CinP]
// fp32 at src[j] and becomes [9][CinP][CoutP], taps rotated by 180 degrees, at dst[j] -- the operand of the
// data gradient (appendix table, backward column: one "reverse" per convolution).
#pragma once

namespace vgg {

constexpr int kMaxFlipJobs = 16;
struct FlipJobs {
    const float *src[kMaxFlipJobs];
    void *dst[kMaxFlipJobs];
    int CinP[kMaxFlipJobs], Cout[kMaxFlipJobs], CoutP[kMaxFlipJobs];
    int first[kMaxFlipJobs + 1];   // first workgroup of each tensor (filled by the launcher)
    int n;
};

// Arguments of the batched update of packed convolution weights with a bf16 working copy
// (sgd_update_master_conv in pointwise.hip): tensor j is [9][Cout][CinP] fp32 at theta[j] (master) and
// grad[j]; copy[j] is its bf16 copy in the layout the convolution kernels read.
struct SgdConvJobs {
    float *theta[kMaxFlipJobs];
    const float *grad[kMaxFlipJobs];
    unsigned short *copy[kMaxFlipJobs];
    int Cout[kMaxFlipJobs], CinP[kMaxFlipJobs];
    int first[kMaxFlipJobs + 1];   // first workgroup of each tensor (filled by the launcher)
    int n;
};

}  // namespace vgg
