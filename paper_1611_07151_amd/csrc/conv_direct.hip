// Direct convolution: one thread per output element.
//
// This is the mapping of section "Parallel Computation of Output Elements": the
// output holds numOutputLayers x outputHeight x outputWidth independent elements
// and thread x owns element (m, h, w) = (x / (Wo*Ho), (x / Wo) % Ho, x % Wo); each
// thread walks its Cin x K x K window.  It accepts any K, S, P and serves as the
// always-available fallback behind the matrix-core kernels.
#include "sq_internal.h"

namespace sq {
namespace {

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

template <typename T>
__global__ __launch_bounds__(256) void conv_direct_kernel(
    const T *__restrict__ in, const T *__restrict__ w, const float *__restrict__ b,
    float *__restrict__ out, int N, int Cin, int H, int W, int Cout, int K, int S, int P,
    int relu, int Ho, int Wo, int ldc, int coff)
{
    const size_t total = (size_t)N * Cout * Ho * Wo;
    for (size_t x = (size_t)blockIdx.x * blockDim.x + threadIdx.x; x < total;
         x += (size_t)gridDim.x * blockDim.x) {
        const int ow = (int)(x % Wo);
        const int oh = (int)((x / Wo) % Ho);
        const int m = (int)((x / ((size_t)Wo * Ho)) % Cout);
        const int n = (int)(x / ((size_t)Wo * Ho * Cout));
        float acc = b ? b[m] : 0.f;
        const T *wm = w + (size_t)m * Cin * K * K;
        for (int c = 0; c < Cin; ++c) {
            const T *plane = in + ((size_t)n * Cin + c) * H * W;
            for (int i = 0; i < K; ++i) {
                const int ih = oh * S + i - P;
                if (ih < 0 || ih >= H) continue;
                for (int j = 0; j < K; ++j) {
                    const int iw = ow * S + j - P;
                    if (iw < 0 || iw >= W) continue;
                    acc = fmaf(to_f32(plane[(size_t)ih * W + iw]), to_f32(wm[(c * K + i) * K + j]), acc);
                }
            }
        }
        if (relu) acc = fmaxf(acc, 0.f);
        out[(((size_t)n * ldc + coff + m) * Ho + oh) * Wo + ow] = acc;
    }
}

}  // namespace

int conv_direct(const ConvArgs &a)
{
    const size_t total = (size_t)a.N * a.Cout * a.Ho * a.Wo;
    size_t blocks = (total + 255) / 256;
    if (blocks > (1u << 20)) blocks = 1u << 20;
    dim3 grid((unsigned)blocks), block(256);
    LaunchScope scope("conv_direct", conv_flops(a), conv_bytes(a), 0.0);   // vector-ALU arithmetic, no MFMA
    if (a.dtype == SQ_F32) {
        hipLaunchKernelGGL(conv_direct_kernel<float>, grid, block, 0, current_stream(),
                           (const float *)a.in, (const float *)a.w, a.b, a.out, a.N, a.Cin, a.H,
                           a.W, a.Cout, a.K, a.S, a.P, a.relu, a.Ho, a.Wo, a.out_channels, a.c_offset);
    } else {
        hipLaunchKernelGGL(conv_direct_kernel<uint16_t>, grid, block, 0, current_stream(),
                           (const uint16_t *)a.in, (const uint16_t *)a.w, a.b, a.out, a.N, a.Cin,
                           a.H, a.W, a.Cout, a.K, a.S, a.P, a.relu, a.Ho, a.Wo, a.out_channels,
                           a.c_offset);
    }
    return check_launch();
}

}  // namespace sq
