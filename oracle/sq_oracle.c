/*
 * CPU oracle for the SqueezeNet forward path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain, obviously-correct statement of what the GPU
 * library must compute.  It is used by the tests, by the smoke check and by the
 * benchmark's CPU-baseline leg, and by nothing else; the product path never
 * calls it.  It shares no code, headers, tables or helpers with the HIP path.
 *
 * Every layer is the textbook definition written as nested loops, with the
 * accumulation carried in double and the result rounded to float once at the
 * end.  There is no blocking, no fusion and no reordering: the loop nest of
 * oracle_conv2d is the paper's sequential convolution (section "Parallel
 * Algorithm Design": one loop over output layers around a five-deep 3-D
 * convolution, kernel bank slid by stride S).  OpenMP is applied only across
 * independent (image, output-layer) planes, which the paper notes are
 * perfectly parallel (section "Parallel Computation of Output Elements").
 *
 * Readings taken where the paper is silent (all are the usual CNN ones):
 *   - cross-correlation, i.e. the kernel is not flipped;
 *   - symmetric zero padding of P pixels, padded taps contribute nothing;
 *   - output size floor((H + 2P - K) / S) + 1;
 *   - bias is added once per output element, ReLU (if asked) follows the bias;
 *   - max pooling uses floor mode and no padding;
 *   - a fire layer is squeeze 1x1 -> {expand 1x1, expand 3x3 pad 1}, all with
 *     bias and ReLU, the two expand results concatenated along the layer axis
 *     with the 1x1 part first (section "Convolutional Neural Networks": one
 *     squeeze layer and two expand layers);
 *   - SqueezeNet is two plain convolutions and eight fire layers (same
 *     section), 224x224 RGB in, 1000 classes out, v1.0 wiring.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py
 * (hand-computed cases, closed forms, invariants, an independent library
 * routine, and a brute-force scatter formulation).  The one thing that cannot
 * be pinned is agreement with the paper's trained-network predictions: the
 * dataset and weights are not available ("parity unpinned" for that claim
 * only; the arithmetic itself is defined for arbitrary weights).
 *
 * Tensors are dense row-major: activations [N][C][H][W], kernels
 * [Cout][Cin][K][K], bias [Cout].
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

static int out_extent(int in, int k, int s, int p)
{
    return (in + 2 * p - k) / s + 1;
}

/* Convolution layer: numInputLayers = Cin, numOutputLayers = Cout, K x K
 * kernels, stride S (section "Convolutional Neural Networks"), plus the
 * zero padding P, the bias b (may be NULL = zero) and the optional ReLU. */
int oracle_conv2d(const float *in, const float *w, const float *b, float *out,
                  int N, int Cin, int H, int W, int Cout, int K, int S, int P,
                  int relu)
{
    if (!in || !w || !out) return -1;
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0 || K <= 0 ||
        S <= 0 || P < 0 || H + 2 * P < K || W + 2 * P < K)
        return -2;
    const int Ho = out_extent(H, K, S, P);
    const int Wo = out_extent(W, K, S, P);
    int n, m;
#pragma omp parallel for collapse(2) schedule(static)
    for (n = 0; n < N; ++n) {
        for (m = 0; m < Cout; ++m) {                      /* output layers */
            for (int oh = 0; oh < Ho; ++oh) {
                for (int ow = 0; ow < Wo; ++ow) {
                    double acc = b ? (double)b[m] : 0.0;
                    for (int c = 0; c < Cin; ++c) {       /* input layers  */
                        for (int i = 0; i < K; ++i) {
                            const int ih = oh * S + i - P;
                            if (ih < 0 || ih >= H) continue;
                            for (int j = 0; j < K; ++j) {
                                const int iw = ow * S + j - P;
                                if (iw < 0 || iw >= W) continue;
                                const double x =
                                    in[(((size_t)n * Cin + c) * H + ih) * W + iw];
                                const double k =
                                    w[(((size_t)m * Cin + c) * K + i) * K + j];
                                acc += x * k;
                            }
                        }
                    }
                    if (relu && acc < 0.0) acc = 0.0;
                    out[(((size_t)n * Cout + m) * Ho + oh) * Wo + ow] = (float)acc;
                }
            }
        }
    }
    return 0;
}

/* Max pooling (section "Pooling and Softmax"): the largest value in each
 * K x K window, windows S apart, floor mode, no padding. */
int oracle_maxpool(const float *in, float *out, int N, int C, int H, int W,
                   int K, int S)
{
    if (!in || !out) return -1;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || S <= 0 || H < K || W < K)
        return -2;
    const int Ho = out_extent(H, K, S, 0);
    const int Wo = out_extent(W, K, S, 0);
    int n, c;
#pragma omp parallel for collapse(2) schedule(static)
    for (n = 0; n < N; ++n) {
        for (c = 0; c < C; ++c) {
            const float *src = in + ((size_t)n * C + c) * H * W;
            float *dst = out + ((size_t)n * C + c) * Ho * Wo;
            for (int oh = 0; oh < Ho; ++oh) {
                for (int ow = 0; ow < Wo; ++ow) {
                    float best = src[(size_t)(oh * S) * W + ow * S];
                    for (int i = 0; i < K; ++i)
                        for (int j = 0; j < K; ++j) {
                            const float v = src[(size_t)(oh * S + i) * W + ow * S + j];
                            if (v > best) best = v;
                        }
                    dst[(size_t)oh * Wo + ow] = best;
                }
            }
        }
    }
    return 0;
}

/* Average pooling over the whole H x W plane (section "Pooling and
 * Softmax"); the network uses it once, on the 13 x 13 classifier maps. */
int oracle_avgpool_global(const float *in, float *out, int N, int C, int H, int W)
{
    if (!in || !out) return -1;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return -2;
    int n, c;
#pragma omp parallel for collapse(2) schedule(static)
    for (n = 0; n < N; ++n) {
        for (c = 0; c < C; ++c) {
            const float *src = in + ((size_t)n * C + c) * H * W;
            double s = 0.0;
            for (int i = 0; i < H * W; ++i) s += (double)src[i];
            out[(size_t)n * C + c] = (float)(s / (double)(H * W));
        }
    }
    return 0;
}

/* Softmax over the C class scores of each image (section "Pooling and
 * Softmax"), in the max-shifted form so large scores cannot overflow. */
int oracle_softmax(const float *in, float *out, int N, int C)
{
    if (!in || !out) return -1;
    if (N <= 0 || C <= 0) return -2;
    for (int n = 0; n < N; ++n) {
        const float *x = in + (size_t)n * C;
        float *y = out + (size_t)n * C;
        double mx = (double)x[0];
        for (int c = 1; c < C; ++c)
            if ((double)x[c] > mx) mx = (double)x[c];
        double sum = 0.0;
        for (int c = 0; c < C; ++c) sum += exp((double)x[c] - mx);
        for (int c = 0; c < C; ++c) y[c] = (float)(exp((double)x[c] - mx) / sum);
    }
    return 0;
}

/* Fire layer (section "Convolutional Neural Networks"): squeeze 1x1 to Csq
 * layers, then expand 1x1 to Ce1 and expand 3x3 (pad 1) to Ce3 layers, both
 * reading the squeeze result; output layers [0,Ce1) are the 1x1 part and
 * [Ce1,Ce1+Ce3) the 3x3 part.  The squeeze map is rounded to float, as it
 * would be when stored between two layers. */
int oracle_fire(const float *in, const float *w_sq, const float *b_sq,
                const float *w_e1, const float *b_e1, const float *w_e3,
                const float *b_e3, float *out, int N, int Cin, int H, int W,
                int Csq, int Ce1, int Ce3)
{
    if (!in || !w_sq || !w_e1 || !w_e3 || !out) return -1;
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Csq <= 0 || Ce1 <= 0 || Ce3 <= 0)
        return -2;
    const size_t plane = (size_t)H * W;
    float *sq = (float *)malloc(sizeof(float) * N * Csq * plane);
    float *e1 = (float *)malloc(sizeof(float) * N * Ce1 * plane);
    float *e3 = (float *)malloc(sizeof(float) * N * Ce3 * plane);
    int rc = -3;
    if (sq && e1 && e3) {
        rc = oracle_conv2d(in, w_sq, b_sq, sq, N, Cin, H, W, Csq, 1, 1, 0, 1);
        if (!rc) rc = oracle_conv2d(sq, w_e1, b_e1, e1, N, Csq, H, W, Ce1, 1, 1, 0, 1);
        if (!rc) rc = oracle_conv2d(sq, w_e3, b_e3, e3, N, Csq, H, W, Ce3, 3, 1, 1, 1);
        if (!rc) {
            for (int n = 0; n < N; ++n) {
                float *dst = out + (size_t)n * (Ce1 + Ce3) * plane;
                memcpy(dst, e1 + (size_t)n * Ce1 * plane, sizeof(float) * Ce1 * plane);
                memcpy(dst + (size_t)Ce1 * plane, e3 + (size_t)n * Ce3 * plane,
                       sizeof(float) * Ce3 * plane);
            }
        }
    }
    free(sq); free(e1); free(e3);
    return rc;
}

/* ------------------------------------------------------------------------
 * SqueezeNet v1.0 forward (section "Convolutional Neural Networks": two
 * convolution layers, eight fire layers, pooling, softmax; 224 x 224 RGB
 * input, 1000 output nodes).
 *
 * params: 52 pointers, weight then bias for each of the 26 convolutions in
 *   network order: conv1, then (squeeze, expand1x1, expand3x3) of fire2 ..
 *   fire9, then conv10.
 * taps: NULL, or 16 pointers that receive each stage's result (any may be
 *   NULL): 0 conv1, 1 pool1, 2..4 fire2..fire4, 5 pool4, 6..9 fire5..fire8,
 *   10 pool8, 11 fire9, 12 conv10, 13 class means, 14 probabilities,
 *   15 unused.
 * conv1 takes P = 2 so that 224 -> 111 -> 55 -> 27 -> 13 as the workload
 * configurations state.
 * ---------------------------------------------------------------------- */
struct fire_cfg { int cin, sq, e; };

int oracle_squeezenet(const float *in, const float *const *params, float *probs,
                      int N, float *const *taps)
{
    static const struct fire_cfg fires[8] = {
        {96, 16, 64},  {128, 16, 64}, {128, 32, 128}, {256, 32, 128},
        {256, 48, 192}, {384, 48, 192}, {384, 64, 256}, {512, 64, 256}};
    if (!in || !params || !probs) return -1;
    if (N <= 0) return -2;

    int C = 96, H = 111;
    size_t cap = (size_t)N * 96 * 111 * 111;       /* largest activation */
    float *a = (float *)malloc(sizeof(float) * cap);
    float *b = (float *)malloc(sizeof(float) * cap);
    float *means = (float *)malloc(sizeof(float) * (size_t)N * 1000);
    int rc = -3;
    if (!a || !b || !means) goto done;

#define TAP(idx, ptr, count)                                                   \
    do { if (taps && taps[idx]) memcpy(taps[idx], ptr, sizeof(float) * (count)); } while (0)

    rc = oracle_conv2d(in, params[0], params[1], a, N, 3, 224, 224, 96, 7, 2, 2, 1);
    if (rc) goto done;
    TAP(0, a, (size_t)N * C * H * H);
    rc = oracle_maxpool(a, b, N, C, H, H, 3, 2);
    if (rc) goto done;
    H = 55;
    TAP(1, b, (size_t)N * C * H * H);
    { float *t = a; a = b; b = t; }                 /* a = current activation */

    int tap = 2, p = 2;
    for (int f = 0; f < 8; ++f) {
        const struct fire_cfg *fc = &fires[f];
        if (fc->cin != C) { rc = -4; goto done; }
        rc = oracle_fire(a, params[p], params[p + 1], params[p + 2], params[p + 3],
                         params[p + 4], params[p + 5], b, N, C, H, H, fc->sq, fc->e, fc->e);
        if (rc) goto done;
        p += 6;
        C = 2 * fc->e;
        TAP(tap, b, (size_t)N * C * H * H);
        ++tap;
        { float *t = a; a = b; b = t; }
        if (f == 2 || f == 6) {                     /* after fire4 and fire8 */
            rc = oracle_maxpool(a, b, N, C, H, H, 3, 2);
            if (rc) goto done;
            H = (H - 3) / 2 + 1;
            TAP(tap, b, (size_t)N * C * H * H);
            ++tap;
            { float *t = a; a = b; b = t; }
        }
    }
    rc = oracle_conv2d(a, params[50], params[51], b, N, 512, H, H, 1000, 1, 1, 0, 1);
    if (rc) goto done;
    TAP(12, b, (size_t)N * 1000 * H * H);
    rc = oracle_avgpool_global(b, means, N, 1000, H, H);
    if (rc) goto done;
    TAP(13, means, (size_t)N * 1000);
    rc = oracle_softmax(means, probs, N, 1000);
    if (rc) goto done;
    TAP(14, probs, (size_t)N * 1000);
#undef TAP
done:
    free(a); free(b); free(means);
    return rc;
}
