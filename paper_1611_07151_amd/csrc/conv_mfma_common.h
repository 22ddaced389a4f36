// Shared pieces of the matrix-core convolution kernels (internal).
#pragma once

#include "sq_internal.h"

namespace sq {
namespace mfma {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kLdsBytes = 160 * 1024;

struct KParams {
    const float *in;
    const float *w;
    const float *b;
    float *out;
    int N, Cin, H, W, Cout, P, relu;
    int Ho, Wo, HoWo, HW, ldc, coff;
    int PT;      // N*Ho*Wo
    int VH;      // virtual rows per image
    int LW;      // patch columns staged
    int LWs;     // LDS row stride of the patch
    int PRcap;   // patch rows the LDS plane can hold
    int plane;   // LDS floats per input layer
    int mtiles;  // tiles along output layers
    int ntiles;  // tiles along pixels
    int nchunks;
};

template <int MT> struct Mfma;
template <> struct Mfma<32> {
    using Acc = f32x16;
    static constexpr int KQ = 2, NR = 16;
    static __device__ __forceinline__ Acc run(float a, float b, Acc c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
    // output-layer row held by accumulator register r of this lane
    static __device__ __forceinline__ int row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }
};
template <> struct Mfma<16> {
    using Acc = f32x4;
    static constexpr int KQ = 4, NR = 4;
    static __device__ __forceinline__ Acc run(float a, float b, Acc c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row(int r, int lane) { return 4 * (lane >> 4) + r; }
};

// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Renumber so
// that every XCD works on one contiguous range of tiles (neighbouring tiles share
// halo rows and the same kernels).
__device__ __forceinline__ int xcd_remap(int b, int total)
{
    const int q = total >> 3, r = total & 7;
    const int xcd = b & 7, idx = b >> 3;
    const int start = xcd < r ? xcd * (q + 1) : r * (q + 1) + (xcd - r) * q;
    return start + idx;
}


// conv1-type layers (7x7, stride 2, three input layers, at most 96 output layers) have
// their own persistent kernel; BN (pixels per tile) is 256 or 128.
typedef void (*KernelFn)(const KParams);
KernelFn conv7s2c3_kernel_for(int BN);

}  // namespace mfma
}  // namespace sq
