// C boundary: argument validation, per-thread stream, algorithm choice, and the
// fire-layer and whole-network drivers that sequence the kernels.
#include "sq_internal.h"

namespace sq {
namespace {
thread_local hipStream_t g_stream = nullptr;
thread_local int g_last_hip = 0;
}  // namespace

hipStream_t current_stream() { return g_stream; }

int check_launch()
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        return SQ_ERR_HIP;
    }
    return SQ_OK;
}

namespace {

int out_extent(int in, int k, int s, int p) { return (in + 2 * p - k) / s + 1; }

int validate_conv(const void *in, const void *w, const float *out, int N, int Cin, int H, int W,
                  int Cout, int K, int S, int P)
{
    if (!in || !w || !out) return SQ_ERR_NULL;
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0 || K <= 0 || S < 1 || P < 0)
        return SQ_ERR_SHAPE;
    if (H + 2 * P < K || W + 2 * P < K) return SQ_ERR_SHAPE;
    return SQ_OK;
}

int run_conv(const ConvArgs &a, int algo)
{
    if (algo == SQ_ALGO_DIRECT) return conv_direct(a);
    if (algo == SQ_ALGO_AUTO) {
        const int rc = conv_mfma(a, -1);
        if (rc != SQ_ERR_UNSUPPORTED) return rc;
        return conv_direct(a);
    }
    const int v = algo - SQ_ALGO_VARIANT0;
    if (v < 0 || v >= conv_mfma_variant_count()) return SQ_ERR_UNSUPPORTED;
    return conv_mfma(a, v);
}

ConvArgs make_args(const void *in, const void *w, const float *b, float *out, int N, int Cin, int H,
                   int W, int Cout, int K, int S, int P, int relu, int out_channels, int c_offset,
                   int dtype)
{
    ConvArgs a;
    a.in = in; a.w = w; a.b = b; a.out = out;
    a.N = N; a.Cin = Cin; a.H = H; a.W = W; a.Cout = Cout; a.K = K; a.S = S; a.P = P;
    a.relu = relu ? 1 : 0;
    a.Ho = out_extent(H, K, S, P);
    a.Wo = out_extent(W, K, S, P);
    a.out_channels = out_channels;
    a.c_offset = c_offset;
    a.dtype = dtype;
    return a;
}

// Unchecked fire layer: squeeze into `sq_map`, then both expands into `out`.
int fire_impl(const void *in, const void *w_sq, const float *b_sq, const void *w_e1,
              const float *b_e1, const void *w_e3, const float *b_e3, float *out, int N, int Cin,
              int H, int W, int Csq, int Ce1, int Ce3, float *sq_map)
{
    int rc = run_conv(make_args(in, w_sq, b_sq, sq_map, N, Cin, H, W, Csq, 1, 1, 0, 1, Csq, 0, SQ_F32),
                      SQ_ALGO_AUTO);
    if (rc) return rc;
    rc = run_conv(make_args(sq_map, w_e1, b_e1, out, N, Csq, H, W, Ce1, 1, 1, 0, 1, Ce1 + Ce3, 0, SQ_F32),
                  SQ_ALGO_AUTO);
    if (rc) return rc;
    return run_conv(make_args(sq_map, w_e3, b_e3, out, N, Csq, H, W, Ce3, 3, 1, 1, 1, Ce1 + Ce3, Ce1, SQ_F32),
                    SQ_ALGO_AUTO);
}

struct FireCfg { int cin, sq, e; };
const FireCfg kFires[8] = {{96, 16, 64},   {128, 16, 64},  {128, 32, 128}, {256, 32, 128},
                           {256, 48, 192}, {384, 48, 192}, {384, 64, 256}, {512, 64, 256}};

// Workspace carve-up of the network call: two activation buffers used in turn and
// the squeeze map.  Buffer A must hold conv1's output, buffer B the largest of the
// others (fire4's output), both per image.
constexpr size_t kBufA = (size_t)96 * 111 * 111;
constexpr size_t kBufB = (size_t)256 * 55 * 55;
constexpr size_t kBufS = (size_t)32 * 55 * 55;

int copy_tap(float *const *taps, int idx, const float *src, size_t count)
{
    if (!taps || !taps[idx]) return SQ_OK;
    const hipError_t e = hipMemcpyAsync(taps[idx], src, count * sizeof(float),
                                        hipMemcpyDeviceToDevice, current_stream());
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        return SQ_ERR_HIP;
    }
    return SQ_OK;
}

}  // namespace
}  // namespace sq

using namespace sq;

extern "C" {

const char *sq_strerror(int status)
{
    switch (status) {
        case SQ_OK: return "ok";
        case SQ_ERR_NULL: return "a required pointer is NULL";
        case SQ_ERR_SHAPE: return "invalid shape, stride, padding or channel range";
        case SQ_ERR_UNSUPPORTED: return "no kernel for this dtype/algorithm/shape";
        case SQ_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case SQ_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

int sq_last_hip_error(void) { return g_last_hip; }

int sq_set_stream(void *hip_stream)
{
    g_stream = (hipStream_t)hip_stream;
    return SQ_OK;
}

int sq_conv_variant_count(void) { return conv_mfma_variant_count(); }

const char *sq_conv_variant_name(int index)
{
    if (index < 0 || index >= conv_mfma_variant_count()) return "";
    return conv_mfma_variant_name(index);
}

int sq_conv2d_forward_ex(const void *in, const void *w, const float *b, float *out, int N, int Cin,
                         int H, int W, int Cout, int K, int S, int P, int relu, int out_channels,
                         int c_offset, int in_dtype, int algo)
{
    const int rc = validate_conv(in, w, out, N, Cin, H, W, Cout, K, S, P);
    if (rc) return rc;
    if (c_offset < 0 || out_channels <= 0 || (long long)c_offset + Cout > out_channels)
        return SQ_ERR_SHAPE;
    if (in_dtype != SQ_F32 && in_dtype != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if (algo < 0) return SQ_ERR_UNSUPPORTED;
    return run_conv(make_args(in, w, b, out, N, Cin, H, W, Cout, K, S, P, relu, out_channels,
                              c_offset, in_dtype), algo);
}

int sq_conv2d_forward(const void *in, const void *w, const float *b, float *out, int N, int Cin,
                      int H, int W, int Cout, int K, int S, int P, int relu)
{
    return sq_conv2d_forward_ex(in, w, b, out, N, Cin, H, W, Cout, K, S, P, relu, Cout, 0, SQ_F32,
                                SQ_ALGO_AUTO);
}

int sq_maxpool(const float *in, float *out, int N, int C, int H, int W, int K, int S)
{
    if (!in || !out) return SQ_ERR_NULL;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || S < 1 || K > H || K > W) return SQ_ERR_SHAPE;
    return maxpool(in, out, N, C, H, W, K, S);
}

int sq_avgpool_global(const float *in, float *out, int N, int C, int H, int W)
{
    if (!in || !out) return SQ_ERR_NULL;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return SQ_ERR_SHAPE;
    return avgpool_global(in, out, N, C, H, W);
}

int sq_softmax(const float *in, float *out, int N, int C)
{
    if (!in || !out) return SQ_ERR_NULL;
    if (N <= 0 || C <= 0) return SQ_ERR_SHAPE;
    return softmax(in, out, N, C);
}

size_t sq_fire_workspace_bytes(int N, int H, int W, int Csq)
{
    if (N <= 0 || H <= 0 || W <= 0 || Csq <= 0) return 0;
    return align_up((size_t)N * Csq * H * W * sizeof(float), 256);
}

int sq_fire_forward(const void *in, const void *w_sq, const float *b_sq, const void *w_e1,
                    const float *b_e1, const void *w_e3, const float *b_e3, float *out, int N,
                    int Cin, int H, int W, int Csq, int Ce1, int Ce3, void *workspace,
                    size_t workspace_bytes)
{
    if (!in || !w_sq || !w_e1 || !w_e3 || !out) return SQ_ERR_NULL;
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Csq <= 0 || Ce1 <= 0 || Ce3 <= 0) return SQ_ERR_SHAPE;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < sq_fire_workspace_bytes(N, H, W, Csq))
        return SQ_ERR_WORKSPACE;
    return fire_impl(in, w_sq, b_sq, w_e1, b_e1, w_e3, b_e3, out, N, Cin, H, W, Csq, Ce1, Ce3,
                     (float *)workspace);
}

size_t sq_squeezenet_workspace_bytes(int N)
{
    if (N <= 0) return 0;
    const size_t n = (size_t)N;
    return align_up(n * kBufA * 4, 256) + align_up(n * kBufB * 4, 256) + align_up(n * kBufS * 4, 256) +
           align_up(n * 1000 * 4, 256);
}

int sq_squeezenet_forward(const void *in, const void *const *params, float *probs, int N,
                          void *workspace, size_t workspace_bytes, float *const *taps)
{
    if (!in || !params || !probs) return SQ_ERR_NULL;
    if (N <= 0) return SQ_ERR_SHAPE;
    for (int i = 0; i < 52; ++i)
        if (!params[i]) return SQ_ERR_NULL;
    if (taps && taps[15]) return SQ_ERR_UNSUPPORTED;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < sq_squeezenet_workspace_bytes(N))
        return SQ_ERR_WORKSPACE;

    const size_t n = (size_t)N;
    char *base = (char *)workspace;
    float *bufA = (float *)base;
    float *bufB = (float *)(base + align_up(n * kBufA * 4, 256));
    float *bufS = (float *)((char *)bufB + align_up(n * kBufB * 4, 256));
    float *means = (float *)((char *)bufS + align_up(n * kBufS * 4, 256));
    auto P = [&](int i) { return (const float *)params[i]; };

    int rc = run_conv(make_args(in, params[0], P(1), bufA, N, 3, 224, 224, 96, 7, 2, 2, 1, 96, 0, SQ_F32),
                      SQ_ALGO_AUTO);
    if (rc) return rc;
    if ((rc = copy_tap(taps, 0, bufA, n * 96 * 111 * 111))) return rc;
    if ((rc = maxpool(bufA, bufB, N, 96, 111, 111, 3, 2))) return rc;
    if ((rc = copy_tap(taps, 1, bufB, n * 96 * 55 * 55))) return rc;

    float *cur = bufB, *nxt = bufA;
    int C = 96, H = 55, tap = 2, p = 2;
    for (int f = 0; f < 8; ++f) {
        const FireCfg &fc = kFires[f];
        rc = fire_impl(cur, params[p], P(p + 1), params[p + 2], P(p + 3), params[p + 4], P(p + 5), nxt,
                       N, C, H, H, fc.sq, fc.e, fc.e, bufS);
        if (rc) return rc;
        p += 6;
        C = 2 * fc.e;
        if ((rc = copy_tap(taps, tap++, nxt, n * C * H * H))) return rc;
        { float *t = cur; cur = nxt; nxt = t; }
        if (f == 2 || f == 6) {  // pooling follows fire4 and fire8
            if ((rc = maxpool(cur, nxt, N, C, H, H, 3, 2))) return rc;
            H = (H - 3) / 2 + 1;
            if ((rc = copy_tap(taps, tap++, nxt, n * C * H * H))) return rc;
            { float *t = cur; cur = nxt; nxt = t; }
        }
    }
    rc = run_conv(make_args(cur, params[50], P(51), nxt, N, 512, H, H, 1000, 1, 1, 0, 1, 1000, 0, SQ_F32),
                  SQ_ALGO_AUTO);
    if (rc) return rc;
    if ((rc = copy_tap(taps, 12, nxt, n * 1000 * H * H))) return rc;
    if ((rc = avgpool_global(nxt, means, N, 1000, H, H))) return rc;
    if ((rc = copy_tap(taps, 13, means, n * 1000))) return rc;
    if ((rc = softmax(means, probs, N, 1000))) return rc;
    return copy_tap(taps, 14, probs, n * 1000);
}

}  // extern "C"
