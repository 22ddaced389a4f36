// A convolution with stride S >= 2 as a stride-1 convolution of a space-to-depth copy of its input.
//
// With i = i'*S + dy and j = j'*S + dx (dy, dx < S) the convolution layer's sum (section "Convolutional Neural
// Networks") over input layer c and kernel offsets (i, j) at stride S,
//     out[n][m][oh][ow] = b[m] + sum_{c,i,j} in[n][c][oh*S + i - P][ow*S + j - P] * w[m][c][i][j],
// is the stride-1, unpadded sum over layer c' = (c*S + dy)*S + dx and offsets (i', j') < K' = ceil(K / S) of
//     in2[n][c'][y][x]   = in[n][c][y*S + dy - P][x*S + dx - P]     (zero outside the image),  y < Ho + K' - 1,
//     w2[m][c'][i'][j']  = w[m][c][i'*S + dy][j'*S + dx]            (zero where that passes K).
// The large strided layers of other networks (11x11 stride 4: K' = 3 on 16 times the input layers) thereby run on
// the 3x3 tilings of the matrix-core family instead of a tiling of their own that keeps a 15-row patch per pixel
// row in LDS and registers.  Costs: one pass over the input (copied once, S*S*K'*K'/(K*K) more multiplications).
#include "sq_internal.h"

namespace sq {
namespace {

struct S2dShape {
    int K2, C2, H2, W2;
    size_t map_elems, w_elems;
};

bool s2d_shape(int N, int Cin, int Cout, int K, int S, int Ho, int Wo, S2dShape &s)
{
    if (S < 2) return false;
    s.K2 = (K + S - 1) / S;
    const long long C2 = (long long)Cin * S * S;
    if (C2 >= (1 << 20)) return false;
    s.C2 = (int)C2;
    s.H2 = Ho + s.K2 - 1;
    s.W2 = Wo + s.K2 - 1;
    s.map_elems = (size_t)N * s.C2 * s.H2 * s.W2;
    s.w_elems = (size_t)Cout * s.C2 * s.K2 * s.K2;
    return true;
}

// One thread per element of the space-to-depth map; T carries the bits of an fp32 or bfloat16 element.
template <typename T>
__global__ __launch_bounds__(256) void s2d_map_kernel(const T *__restrict__ in, T *__restrict__ out, int C, int H, int W,
                                                      int S, int P, int H2, int W2, size_t total)
{
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
        const int x = (int)(e % W2);
        size_t r = e / W2;
        const int y = (int)(r % H2);
        r /= H2;
        const int c2 = (int)(r % ((size_t)C * S * S));
        const size_t n = r / ((size_t)C * S * S);
        const int dx = c2 % S, dy = (c2 / S) % S, c = c2 / (S * S);
        const int ih = y * S + dy - P, iw = x * S + dx - P;
        T v = 0;
        if (ih >= 0 && ih < H && iw >= 0 && iw < W) v = in[((n * C + c) * H + ih) * (size_t)W + iw];
        out[e] = v;
    }
}

// The same for a stride known at compile time: one thread per S horizontally adjacent input elements, which it
// reads as one run (a wavefront reads 64*S consecutive elements of an input row) and writes to the S phase images
// dx = 0..S-1 (each store of a wavefront covers 64 consecutive elements).
template <typename T, int S>
__global__ __launch_bounds__(256) void s2d_map_rows_kernel(const T *__restrict__ in, T *__restrict__ out, int C, int H, int W,
                                                           int P, int H2, int W2, size_t total)
{
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
        const int x = (int)(e % W2);
        size_t r = e / W2;
        const int y = (int)(r % H2);
        r /= H2;
        const int dy = (int)(r % S);
        const size_t nc = r / S;                   // n * C + c
        const int ih = y * S + dy - P, iw0 = x * S - P;
        const bool row = ih >= 0 && ih < H;
        const T *src = in + (nc * H + (row ? ih : 0)) * (size_t)W;
        T v[S];
#pragma unroll
        for (int dx = 0; dx < S; ++dx) {
            const int iw = iw0 + dx;
            v[dx] = (row && iw >= 0 && iw < W) ? src[iw] : (T)0;
        }
        T *dst = out + ((nc * S + dy) * S) * ((size_t)H2 * W2) + (size_t)y * W2 + x;
#pragma unroll
        for (int dx = 0; dx < S; ++dx) dst[(size_t)dx * H2 * W2] = v[dx];
    }
}

// One thread per element of the regrouped kernels.
template <typename T>
__global__ __launch_bounds__(256) void s2d_kernels_kernel(const T *__restrict__ w, T *__restrict__ w2, int Cin, int K, int S,
                                                          int K2, size_t total)
{
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (size_t)gridDim.x * 256) {
        const int j2 = (int)(e % K2);
        size_t r = e / K2;
        const int i2 = (int)(r % K2);
        r /= K2;
        const int c2 = (int)(r % ((size_t)Cin * S * S));
        const size_t m = r / ((size_t)Cin * S * S);
        const int dx = c2 % S, dy = (c2 / S) % S, c = c2 / (S * S);
        const int i = i2 * S + dy, j = j2 * S + dx;
        T v = 0;
        if (i < K && j < K) v = w[((m * Cin + c) * K + i) * (size_t)K + j];
        w2[e] = v;
    }
}

unsigned grid_for(size_t total)
{
    const size_t blocks = (total + 255) / 256;
    return (unsigned)(blocks < (1u << 20) ? (blocks ? blocks : 1) : (1u << 20));
}

}  // namespace

size_t conv_s2d_workspace_bytes(int N, int Cin, int H, int W, int Cout, int K, int S, int P)
{
    S2dShape s;
    const int Ho = (H + 2 * P - K) / S + 1, Wo = (W + 2 * P - K) / S + 1;
    if (Ho <= 0 || Wo <= 0 || !s2d_shape(N, Cin, Cout, K, S, Ho, Wo, s)) return 0;
    return align_up(s.map_elems * 4, 256) + align_up(s.w_elems * 4, 256);
}

int conv_s2d(const ConvArgs &a)
{
    S2dShape s;
    if (a.pool_H || !a.ws || !s2d_shape(a.N, a.Cin, a.Cout, a.K, a.S, a.Ho, a.Wo, s)) return SQ_ERR_UNSUPPORTED;
    const size_t esz = a.dtype == SQ_BF16 ? 2 : 4;
    const size_t map_bytes = align_up(s.map_elems * esz, 256), w_bytes = align_up(s.w_elems * esz, 256);
    if (a.ws_bytes < map_bytes + w_bytes) return SQ_ERR_UNSUPPORTED;
    ConvArgs a2 = a;
    a2.in = a.ws;
    a2.w = (const char *)a.ws + map_bytes;
    a2.Cin = s.C2; a2.H = s.H2; a2.W = s.W2; a2.K = s.K2; a2.S = 1; a2.P = 0;
    a2.ws = nullptr; a2.ws_bytes = 0; a2.ws_ready = false;
    // only where a matrix-core tiling serves the stride-1 form (its Ho, Wo are those of the call)
    if (conv_mfma_choice(a2) < 0) return SQ_ERR_UNSUPPORTED;
    int rc;
    {
        LaunchScope scope("s2d_map", 0.0, (double)esz * ((double)a.N * a.Cin * a.H * a.W + (double)s.map_elems));
        const size_t runs = s.map_elems / a.S;   // threads of the form that takes S elements each
        if (a.S == 4 && esz == 4)
            hipLaunchKernelGGL((s2d_map_rows_kernel<uint32_t, 4>), dim3(grid_for(runs)), dim3(256), 0, current_stream(),
                               (const uint32_t *)a.in, (uint32_t *)a.ws, a.Cin, a.H, a.W, a.P, s.H2, s.W2, runs);
        else if (a.S == 2 && esz == 4)
            hipLaunchKernelGGL((s2d_map_rows_kernel<uint32_t, 2>), dim3(grid_for(runs)), dim3(256), 0, current_stream(),
                               (const uint32_t *)a.in, (uint32_t *)a.ws, a.Cin, a.H, a.W, a.P, s.H2, s.W2, runs);
        else if (a.S == 4)
            hipLaunchKernelGGL((s2d_map_rows_kernel<uint16_t, 4>), dim3(grid_for(runs)), dim3(256), 0, current_stream(),
                               (const uint16_t *)a.in, (uint16_t *)a.ws, a.Cin, a.H, a.W, a.P, s.H2, s.W2, runs);
        else if (a.S == 2)
            hipLaunchKernelGGL((s2d_map_rows_kernel<uint16_t, 2>), dim3(grid_for(runs)), dim3(256), 0, current_stream(),
                               (const uint16_t *)a.in, (uint16_t *)a.ws, a.Cin, a.H, a.W, a.P, s.H2, s.W2, runs);
        else if (esz == 4)
            hipLaunchKernelGGL(s2d_map_kernel<uint32_t>, dim3(grid_for(s.map_elems)), dim3(256), 0, current_stream(),
                               (const uint32_t *)a.in, (uint32_t *)a.ws, a.Cin, a.H, a.W, a.S, a.P, s.H2, s.W2, s.map_elems);
        else
            hipLaunchKernelGGL(s2d_map_kernel<uint16_t>, dim3(grid_for(s.map_elems)), dim3(256), 0, current_stream(),
                               (const uint16_t *)a.in, (uint16_t *)a.ws, a.Cin, a.H, a.W, a.S, a.P, s.H2, s.W2, s.map_elems);
        if ((rc = check_launch())) return rc;
    }
    {
        LaunchScope scope("s2d_kernels", 0.0, (double)esz * ((double)a.Cout * a.Cin * a.K * a.K + (double)s.w_elems));
        if (esz == 4)
            hipLaunchKernelGGL(s2d_kernels_kernel<uint32_t>, dim3(grid_for(s.w_elems)), dim3(256), 0, current_stream(),
                               (const uint32_t *)a.w, (uint32_t *)const_cast<void *>(a2.w), a.Cin, a.K, a.S, s.K2, s.w_elems);
        else
            hipLaunchKernelGGL(s2d_kernels_kernel<uint16_t>, dim3(grid_for(s.w_elems)), dim3(256), 0, current_stream(),
                               (const uint16_t *)a.w, (uint16_t *)const_cast<void *>(a2.w), a.Cin, a.K, a.S, s.K2, s.w_elems);
        if ((rc = check_launch())) return rc;
    }
    return conv_mfma(a2, -1);
}

}  // namespace sq
