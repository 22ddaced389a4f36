// The cheap layers around the convolutions (section "Pooling and Softmax"): max
// pooling, whole-plane average pooling and softmax.  All three are bound by HBM
// traffic; each reads its input once (pool windows overlap in cache) and writes
// its output once.
#include "sq_internal.h"

#include <algorithm>

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

// 3x3 / stride 2 pooling, the only kind the network uses.  A group of LP lanes (64, 32 or
// 16, the smallest with 2*LP >= W) owns one plane and walks down its rows: lane l holds
// columns 2l and 2l+1 of the current input rows, keeps the last row of one window as the
// first row of the next (every input element is loaded exactly once, coalesced), and gets
// column 2l+2 from its neighbour lane.  Output row oh is written by lanes l < Wo.
template <int LP>
__global__ __launch_bounds__(256) void maxpool3s2_kernel(const float *__restrict__ in, float *__restrict__ out,
                                                         size_t planes, int H, int W, int Ho, int Wo, int RB)
{
    // blockIdx.y selects a band of RB output rows (a multiple of four): small batches have too
    // few planes to fill the chip with one wavefront group per plane
    const int oh_begin = blockIdx.y * RB, oh_end = min(oh_begin + RB, Ho);
    const int lane = threadIdx.x & 63, sub = lane / LP, l = lane % LP;
    const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const size_t pl = wave * (64 / LP) + sub;
    const bool live = pl < planes;
    const float *src = in + (live ? pl : 0) * (size_t)H * W;
    float *dst = out + (live ? pl : 0) * (size_t)Ho * Wo;
    const bool has0 = live && 2 * l < W, has1 = live && 2 * l + 1 < W;
    // Each lane reads two adjacent floats per row (one 8-byte load).  The lane holding the
    // last column of an odd-width row reads the pair one to the left and keeps its right half.
    const int cb = has1 ? 2 * l : (has0 ? 2 * l - 1 : 0);
    auto load2 = [&](int ih, float &a, float &b) {
        const float *q = src + (size_t)ih * W + cb;
        const float v0 = q[0], v1 = q[1];
        a = has1 ? v0 : v1;
        b = v1;
    };
    float a0, b0;
    load2(2 * oh_begin, a0, b0);
    // four output rows per trip: the eight row loads of a trip are independent and issued
    // together (rows past the end are clamped for the load and never stored)
    constexpr int U = 4;
    for (int oh0 = oh_begin; oh0 < oh_end; oh0 += U) {
        float a[2 * U], b[2 * U];
#pragma unroll
        for (int u = 0; u < 2 * U; ++u) load2(min(2 * oh0 + 1 + u, H - 1), a[u], b[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float ma = has0 ? fmaxf(fmaxf(a0, a[2 * u]), a[2 * u + 1]) : -INFINITY;
            const float mb = has1 ? fmaxf(fmaxf(b0, b[2 * u]), b[2 * u + 1]) : -INFINITY;
            const float mc = __shfl_down(ma, 1, LP);     // column 2l+2
            if (live && l < Wo && oh0 + u < oh_end) dst[(size_t)(oh0 + u) * Wo + l] = fmaxf(fmaxf(ma, mb), mc);
            a0 = a[2 * u + 1];
            b0 = b[2 * u + 1];
        }
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

// One wavefront per (image, layer) plane: any plane size.
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

// Planes of at most 64*IT pixels, PL consecutive planes per wavefront: all PL*IT loads of a lane are issued
// before the first sum, where the loop above waits for memory once per 64 pixels.  The order of the sums is
// that of the loop above, so both give the same bits.
template <int PL, int IT>
__global__ __launch_bounds__(256) void avgpool_small_kernel(const float *__restrict__ in,
                                                            float *__restrict__ out, size_t planes, int HW)
{
    const int lane = threadIdx.x & 63;
    const size_t pl0 = ((size_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * PL;
    if (pl0 >= planes) return;
    float v[PL][IT];
#pragma unroll
    for (int q = 0; q < PL; ++q)
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int i = lane + 64 * j;
            v[q][j] = (i < HW && pl0 + q < planes) ? in[(pl0 + q) * HW + i] : 0.f;
        }
    float mine = 0.f;
#pragma unroll
    for (int q = 0; q < PL; ++q) {
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < IT; ++j) s += v[q][j];
        s = wave_sum(s);
        if (lane == q) mine = s;
    }
    if (lane < PL && pl0 + lane < planes) out[pl0 + lane] = mine / (float)HW;
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

// Second half of "1x1 convolution -> global average pooling -> softmax" (section "Pooling and Softmax") when the
// convolution has written per-image plane sums per pixel tile (conv_mfma_kernel.h, averaging form): one workgroup per
// image adds the slots that belong to its image, divides by the plane size, optionally writes the means, and applies
// the max-shifted softmax.  sums: [pixel tile][WN][slots][C]; pixel tile pt covers pixels [pt * BN, (pt + 1) * BN) of the
// batch-flattened pixel index n * HW + pixel, and its slot s belongs to image (pt * BN) / HW + s.  C <= 256 * kAvgPer.
constexpr int kAvgPer = 8, kAvgTerms = 16;
__global__ __launch_bounds__(256) void avg_softmax_kernel(const float *__restrict__ sums, float *__restrict__ means,
                                                          float *__restrict__ probs, int C, int HW, int BN, int WN, int slots)
{
    __shared__ float red[4];
    __shared__ float bcast;
    const int n = blockIdx.x, t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int t0 = (n * HW) / BN, t1 = (n * HW + HW - 1) / BN;
    const float inv_hw = 1.f / (float)HW;
    // The (pixel tile, wavefront column) terms of this image, in the order they are added.  Up to kAvgTerms of them
    // have their table offsets worked out once (they are the same for every thread) and their loads issued together;
    // an image spread over more terms takes the plain loop.
    const int nterms = (t1 - t0 + 1) * WN;
    uint32_t off[kAvgTerms];
#pragma unroll
    for (int k = 0; k < kAvgTerms; ++k) {
        const int pt = t0 + k / WN, wn = k - (k / WN) * WN;
        const int slot = n - (pt * BN) / HW;
        off[k] = k < nterms ? (uint32_t)__builtin_amdgcn_readfirstlane(((pt * WN + wn) * slots + slot) * C) : 0u;
    }
    float v[kAvgPer];
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < kAvgPer; ++j) {
        const int c = t + 256 * j;
        float s = 0.f;
        if (c < C) {
            if (nterms <= kAvgTerms) {
                float term[kAvgTerms];
#pragma unroll
                for (int k = 0; k < kAvgTerms; ++k) term[k] = k < nterms ? sums[off[k] + c] : 0.f;
#pragma unroll
                for (int k = 0; k < kAvgTerms; ++k) s += term[k];
            } else {
                for (int pt = t0; pt <= t1; ++pt) {
                    const int slot = n - (pt * BN) / HW;
                    for (int wn = 0; wn < WN; ++wn) s += sums[((size_t)(pt * WN + wn) * slots + slot) * C + c];
                }
            }
            s *= inv_hw;
            if (means) means[(size_t)n * C + c] = s;
            mx = fmaxf(mx, s);
        }
        v[j] = s;
    }
    mx = wave_max(mx);
    if (lane == 0) red[wv] = mx;
    __syncthreads();
    if (t == 0) bcast = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    mx = bcast;
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < kAvgPer; ++j) {
        v[j] = t + 256 * j < C ? expf(v[j] - mx) : 0.f;
        s += v[j];
    }
    s = wave_sum(s);
    __syncthreads();
    if (lane == 0) red[wv] = s;
    __syncthreads();
    if (t == 0) bcast = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
    const float inv = 1.f / bcast;
#pragma unroll
    for (int j = 0; j < kAvgPer; ++j)
        if (t + 256 * j < C) probs[(size_t)n * C + t + 256 * j] = v[j] * inv;
}

}  // namespace

int avg_softmax(const float *sums, const AvgLayout &lay, float *means, float *probs, int N, int C, int HW)
{
    if (C > 256 * kAvgPer || (long long)N * HW >= (1ll << 31) || (long long)lay.ntiles * lay.WN * lay.slots * C >= (1ll << 31))
        return SQ_ERR_UNSUPPORTED;
    LaunchScope scope("planesums+softmax", 0.0, 4.0 * ((double)lay.ntiles * lay.WN * lay.slots * C + 2.0 * N * C));
    hipLaunchKernelGGL(avg_softmax_kernel, dim3((unsigned)N), dim3(256), 0, current_stream(), sums, means, probs, C, HW, lay.BN,
                       lay.WN, lay.slots);
    return check_launch();
}

int maxpool(const float *in, float *out, int N, int C, int H, int W, int K, int S)
{
    const int Ho = (H - K) / S + 1, Wo = (W - K) / S + 1;
    const size_t planes = (size_t)N * C;
    size_t blocks = (planes * Ho * Wo + 255) / 256;
    if (blocks > (1u << 20)) blocks = 1u << 20;
    LaunchScope scope("maxpool", 0.0, 4.0 * planes * ((double)H * W + (double)Ho * Wo));
    if (K == 3 && S == 2 && W <= 128) {
        const int LP = W <= 32 ? 16 : W <= 64 ? 32 : 64;
        const size_t waves = (planes + (64 / LP) - 1) / (64 / LP);
        const size_t groups = (waves + 3) / 4;
        if (groups < (1u << 31)) {
            auto fn = LP == 16 ? maxpool3s2_kernel<16> : LP == 32 ? maxpool3s2_kernel<32> : maxpool3s2_kernel<64>;
            // with few planes, split the rows of a plane into bands so that about 2048 wavefronts exist
            const int max_bands = (Ho + 3) / 4;
            int bands = (int)std::min<size_t>((size_t)max_bands, (2048 + waves - 1) / waves);
            if (bands < 1) bands = 1;
            const int RB = ((Ho + bands - 1) / bands + 3) / 4 * 4;
            bands = (Ho + RB - 1) / RB;
            hipLaunchKernelGGL(fn, dim3((unsigned)groups, (unsigned)bands), dim3(256), 0, current_stream(), in, out, planes,
                               H, W, Ho, Wo, RB);
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
    const int HW = H * W, IT = (HW + 63) / 64;
    // four planes per wavefront once that still leaves every compute unit a dozen wavefronts
    const int PL = planes >= 16384 ? 4 : 1;
    const dim3 grid((unsigned)((planes + 4 * PL - 1) / (4 * PL)));
    void (*kernel)(const float *, float *, size_t, int) = avgpool_kernel;
    switch (IT * 8 + PL) {
        case 1 * 8 + 1: kernel = avgpool_small_kernel<1, 1>; break;
        case 2 * 8 + 1: kernel = avgpool_small_kernel<1, 2>; break;
        case 3 * 8 + 1: kernel = avgpool_small_kernel<1, 3>; break;
        case 4 * 8 + 1: kernel = avgpool_small_kernel<1, 4>; break;
        case 1 * 8 + 4: kernel = avgpool_small_kernel<4, 1>; break;
        case 2 * 8 + 4: kernel = avgpool_small_kernel<4, 2>; break;
        case 3 * 8 + 4: kernel = avgpool_small_kernel<4, 3>; break;
        case 4 * 8 + 4: kernel = avgpool_small_kernel<4, 4>; break;
        default: break;   // larger planes: the loop, one plane per wavefront
    }
    const dim3 grid_used = kernel == avgpool_kernel ? dim3((unsigned)((planes + 3) / 4)) : grid;
    hipLaunchKernelGGL(kernel, grid_used, dim3(256), 0, current_stream(), in, out, planes, HW);
    return check_launch();
}

int softmax(const float *in, float *out, int N, int C)
{
    LaunchScope scope("softmax", 0.0, 8.0 * N * C);
    hipLaunchKernelGGL(softmax_kernel, dim3((unsigned)N), dim3(256), 0, current_stream(), in, out, C);
    return check_launch();
}

}  // namespace sq
