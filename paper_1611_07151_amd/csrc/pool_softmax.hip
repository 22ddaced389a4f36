// The cheap layers around the convolutions (section "Pooling and Softmax"): max
// pooling, whole-plane average pooling and softmax.  All three are bound by HBM
// traffic; each reads its input once (pool windows overlap in cache) and writes
// its output once.
#include "sq_internal.h"

namespace sq {
namespace {

// One thread per output element, ow fastest so a wavefront reads neighbouring
// windows of one input row.
__global__ __launch_bounds__(256) void maxpool_kernel(const float *__restrict__ in,
                                                      float *__restrict__ out, size_t planes,
                                                      int H, int W, int K, int S, int Ho, int Wo)
{
    const size_t total = planes * Ho * Wo;
    for (size_t x = (size_t)blockIdx.x * blockDim.x + threadIdx.x; x < total;
         x += (size_t)gridDim.x * blockDim.x) {
        const int ow = (int)(x % Wo);
        const int oh = (int)((x / Wo) % Ho);
        const size_t pl = x / ((size_t)Wo * Ho);
        const float *src = in + pl * H * W + (size_t)(oh * S) * W + ow * S;
        float best = src[0];
        for (int i = 0; i < K; ++i)
            for (int j = 0; j < K; ++j) best = fmaxf(best, src[(size_t)i * W + j]);
        out[x] = best;
    }
}

// Workgroup per group of G consecutive planes: the planes (contiguous in memory) are
// copied once, coalesced, into LDS and every output reads its window from there, so HBM
// sees each input element exactly once and each output once.
__global__ __launch_bounds__(256) void maxpool_lds_kernel(const float *__restrict__ in,
                                                          float *__restrict__ out, size_t planes, int G,
                                                          int H, int W, int K, int S, int Ho, int Wo)
{
    extern __shared__ float tile[];
    const size_t first = (size_t)blockIdx.x * G;
    const int g = (int)min((size_t)G, planes - first);
    const int HW = H * W, HoWo = Ho * Wo;
    const float *src = in + first * HW;
    const int n_in = g * HW;
    for (int i = threadIdx.x; i < n_in; i += 256) tile[i] = src[i];
    __syncthreads();
    float *dst = out + first * HoWo;
    const int n_out = g * HoWo;
    for (int x = threadIdx.x; x < n_out; x += 256) {
        const int pl = x / HoWo, r = x - pl * HoWo;
        const int oh = r / Wo, ow = r - oh * Wo;
        const float *win = tile + pl * HW + (oh * S) * W + ow * S;
        float best = win[0];
        for (int i = 0; i < K; ++i)
            for (int j = 0; j < K; ++j) best = fmaxf(best, win[i * W + j]);
        dst[x] = best;
    }
}

__device__ __forceinline__ float wave_sum(float v)
{
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// One wavefront per (image, layer) plane.
__global__ __launch_bounds__(256) void avgpool_kernel(const float *__restrict__ in,
                                                      float *__restrict__ out, size_t planes, int HW)
{
    const int lane = threadIdx.x & 63;
    const size_t pl = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (pl >= planes) return;
    const float *src = in + pl * HW;
    float s = 0.f;
    for (int i = lane; i < HW; i += 64) s += src[i];
    s = wave_sum(s);
    if (lane == 0) out[pl] = s / (float)HW;
}

// One 256-thread workgroup per image.
__global__ __launch_bounds__(256) void softmax_kernel(const float *__restrict__ in,
                                                      float *__restrict__ out, int C)
{
    __shared__ float red[4];
    __shared__ float bcast;
    const float *x = in + (size_t)blockIdx.x * C;
    float *y = out + (size_t)blockIdx.x * C;
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;

    float mx = -INFINITY;
    for (int c = t; c < C; c += 256) mx = fmaxf(mx, x[c]);
    mx = wave_max(mx);
    if (lane == 0) red[wv] = mx;
    __syncthreads();
    if (t == 0) bcast = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    mx = bcast;

    float s = 0.f;
    for (int c = t; c < C; c += 256) s += expf(x[c] - mx);
    s = wave_sum(s);
    __syncthreads();
    if (lane == 0) red[wv] = s;
    __syncthreads();
    if (t == 0) bcast = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
    const float inv = 1.f / bcast;
    for (int c = t; c < C; c += 256) y[c] = expf(x[c] - mx) * inv;
}

}  // namespace

int maxpool(const float *in, float *out, int N, int C, int H, int W, int K, int S)
{
    const int Ho = (H - K) / S + 1, Wo = (W - K) / S + 1;
    const size_t planes = (size_t)N * C;
    size_t blocks = (planes * Ho * Wo + 255) / 256;
    if (blocks > (1u << 20)) blocks = 1u << 20;
    LaunchScope scope("maxpool", 0.0, 4.0 * planes * ((double)H * W + (double)Ho * Wo));
    const size_t plane_bytes = (size_t)H * W * sizeof(float);
    if (plane_bytes <= 50 * 1024) {  // up to three workgroups per CU
        int G = (int)(50 * 1024 / plane_bytes);
        // keep at least ~4 workgroups per CU in flight when there are few planes
        while (G > 1 && (planes + G - 1) / G < 1024) --G;
        const size_t groups = (planes + G - 1) / G;
        if (groups < (1u << 31)) {
            hipLaunchKernelGGL(maxpool_lds_kernel, dim3((unsigned)groups), dim3(256), (size_t)G * plane_bytes,
                               current_stream(), in, out, planes, G, H, W, K, S, Ho, Wo);
            return check_launch();
        }
    }
    hipLaunchKernelGGL(maxpool_kernel, dim3((unsigned)blocks), dim3(256), 0, current_stream(), in,
                       out, planes, H, W, K, S, Ho, Wo);
    return check_launch();
}

int avgpool_global(const float *in, float *out, int N, int C, int H, int W)
{
    const size_t planes = (size_t)N * C;
    LaunchScope scope("avgpool", 0.0, 4.0 * planes * ((double)H * W + 1.0));
    hipLaunchKernelGGL(avgpool_kernel, dim3((unsigned)((planes + 3) / 4)), dim3(256), 0,
                       current_stream(), in, out, planes, H * W);
    return check_launch();
}

int softmax(const float *in, float *out, int N, int C)
{
    LaunchScope scope("softmax", 0.0, 8.0 * N * C);
    hipLaunchKernelGGL(softmax_kernel, dim3((unsigned)N), dim3(256), 0, current_stream(), in, out, C);
    return check_launch();
}

}  // namespace sq
