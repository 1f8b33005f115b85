// Measurement aid: what a loop of nothing but MFMA instructions sustains on this chip.
//
// The roofline of the convolution kernels is priced against the data-sheet rate (issue rate x
// nominal clock).  Under matrix load the chip runs below its nominal clock, by an amount that
// depends on how much the operand bits toggle, so the rate a kernel can reach at all is lower.
// This kernel keeps its operands and 2x2 accumulator blocks in registers, touches no memory in
// the loop, and runs four waves per SIMD on every CU: timing it gives that ceiling.
#include "common.h"

namespace vgg {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeBlocksPerCU = 4;   // of 4 waves each: four waves per SIMD
constexpr int kProbeMfmaPerIter = 8;   // per wave

// M16 (bf16 only): v_mfma_f32_16x16x32_bf16, twice as many instructions of half the size on the same operands
// and as many accumulator registers (each 32x32 block as four 16x16 ones), instead of v_mfma_f32_32x32x16_bf16.
template <typename T, bool M16>
__global__ __launch_bounds__(256, kProbeBlocksPerCU) void mfma_probe_kernel(float *sink, int iters, int random)
{
    typedef float f32x4p __attribute__((ext_vector_type(4)));
    const int tid = threadIdx.x;
    f32x16 acc[2][2];
    f32x4p acc4[2][2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
#pragma unroll
            for (int q = 0; q < 4; ++q) acc4[i][j][q] = f32x4p{0.f, 0.f, 0.f, 0.f};
        }
    // operands: 1.0 everywhere, or values in +-[0.5, 1) with random mantissas and signs
    unsigned h = tid * 2654435761u + blockIdx.x * 40503u;
    unsigned a[2][4], b[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            h = h * 1664525u + 1013904223u;
            const unsigned ra = sizeof(T) == 2 ? (((h >> 3) & 0x807f807fu) | 0x3f003f00u) : (((h >> 3) & 0x807fffffu) | 0x3f000000u);
            h = h * 1664525u + 1013904223u;
            const unsigned rb = sizeof(T) == 2 ? (((h >> 3) & 0x807f807fu) | 0x3f003f00u) : (((h >> 3) & 0x807fffffu) | 0x3f000000u);
            const unsigned one = sizeof(T) == 2 ? 0x3f803f80u : 0x3f800000u;
            a[i][q] = random ? ra : one;
            b[i][q] = random ? rb : one;
        }
    if constexpr (M16) {
        const u32x4 a0 = {a[0][0], a[0][1], a[0][2], a[0][3]}, a1 = {a[1][0], a[1][1], a[1][2], a[1][3]};
        const u32x4 b0 = {b[0][0], b[0][1], b[0][2], b[0][3]}, b1 = {b[1][0], b[1][1], b[1][2], b[1][3]};
        for (int it = 0; it < iters; ++it) {   // every 16x16 accumulator once: 16 instructions per iteration
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        acc4[i][j][q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, i ? a1 : a0),
                                                                                __builtin_bit_cast(bf16x8, j ? b1 : b0), acc4[i][j][q], 0, 0, 0);
        }
    } else {
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < kProbeMfmaPerIter / 4; ++u)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        if constexpr (sizeof(T) == 2) {
                            const u32x4 av = {a[i][0], a[i][1], a[i][2], a[i][3]}, bv = {b[j][0], b[j][1], b[j][2], b[j][3]};
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av),
                                                                               __builtin_bit_cast(bf16x8, bv), acc[i][j], 0, 0, 0);
                        } else {
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[i][u & 3]), __uint_as_float(b[j][u & 3]),
                                                                            acc[i][j], 0, 0, 0);
                        }
                    }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int e = 0; e < 16; ++e) s += acc[i][j][e];
#pragma unroll
            for (int q = 0; q < 4; ++q) s += acc4[i][j][q][0] + acc4[i][j][q][1] + acc4[i][j][q][2] + acc4[i][j][q][3];
        }
    sink[(size_t)blockIdx.x * 256 + tid] = s;
}

static int probe_blocks()
{
    static int blocks = 0;
    if (!blocks) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        blocks = cus * kProbeBlocksPerCU;
    }
    return blocks;
}

size_t mfma_probe_sink_bytes() { return (size_t)probe_blocks() * 256 * sizeof(float); }

// Launches the loop; *flops (host) receives the number of floating-point operations it performs.
// random: bit 0 random operands, bit 1 (bf16) the 16x16x32 instruction shape.
int mfma_probe(int dtype, int random, int iters, float *sink, double *flops, hipStream_t stream)
{
    const int blocks = probe_blocks();
    const double per_mfma = dtype == VGG_BF16 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
    if (flops) *flops = (double)blocks * 4 * iters * kProbeMfmaPerIter * per_mfma;
    if (dtype == VGG_BF16 && (random & 2))
        hipLaunchKernelGGL((mfma_probe_kernel<bf16_t, true>), dim3(blocks), dim3(256), 0, stream, sink, iters, random & 1);
    else if (dtype == VGG_BF16)
        hipLaunchKernelGGL((mfma_probe_kernel<bf16_t, false>), dim3(blocks), dim3(256), 0, stream, sink, iters, random & 1);
    else
        hipLaunchKernelGGL((mfma_probe_kernel<float, false>), dim3(blocks), dim3(256), 0, stream, sink, iters, random & 1);
    return launch_status();
}

}  // namespace vgg
