/*
 * sq.h -- C boundary of the SqueezeNet forward library for AMD MI355X (gfx950).
 *
 * The library computes the forward path of the network the paper accelerates
 * (section "Convolutional Neural Networks"): convolution layers with
 * numInputLayers -> numOutputLayers feature maps, K x K kernels slid by stride
 * S, the fire layer (one squeeze and two expand convolutions), max and average
 * pooling and softmax (section "Pooling and Softmax"), and the whole SqueezeNet
 * chain.  Bias and ReLU are fused into every convolution.
 *
 * Conventions that hold for every entry point
 *   - Every data pointer is a DEVICE pointer to memory of the current HIP
 *     device, owned by the caller.  The forward calls never allocate, free,
 *     copy to the host or synchronise: work is enqueued on the stream given
 *     to sq_set_stream() (default: the null stream) and the call returns.
 *     Scratch, where an operation needs it, is the caller's (the workspace
 *     arguments).  The one host-side array is the parameter table of
 *     sq_squeezenet_forward, which is read before the call returns.  Only the
 *     opt-in profiler (sq_profile_begin / sq_profile_end) creates and
 *     destroys HIP events and waits for them.
 *   - Tensors are dense and row-major.  Activations are [N][C][H][W] ("row
 *     major" order D of section "Data Reordering", one image after another),
 *     kernels are [Cout][Cin][K][K], biases [Cout].  fp32 unless stated.
 *   - Inputs and outputs must not overlap.
 *   - Convolution is a cross-correlation (no kernel flip) with P pixels of
 *     zero padding on every side; output extent is floor((H + 2P - K)/S) + 1.
 *   - Every function returns SQ_OK (0) or a negative sq_status.  Arguments are
 *     validated on the host before any GPU work is issued; on an argument
 *     error nothing has been enqueued and no output is touched.  SQ_ERR_HIP
 *     reports a failed launch; sq_last_hip_error() then gives the HIP code.
 *   - Host threads.  The stream (sq_set_stream), the arithmetic mode
 *     (sq_set_dtype), the last HIP error and the profiler are settings of the
 *     calling host thread; every other piece of library state is read-only
 *     after it has been filled under a lock, so two host threads may call any
 *     entry points at the same time (on different streams, with different
 *     workspaces).
 *   - First use.  Kernels that need more than the default 64 KB of LDS have
 *     that limit raised (hipFuncSetAttribute) the first time each is launched;
 *     sq_init() does it for all of them at once.  Call sq_init() -- or run the
 *     same call once as a warm-up -- before capturing library calls in a HIP
 *     graph, so that the captured region holds kernel launches only.
 *   - Sizes.  The matrix-core kernels address a tensor through 32-bit byte
 *     offsets, so they serve a convolution only while its input, its whole
 *     output tensor ([N][out_channels][Ho][Wo]) and its kernels each have fewer
 *     than 2^29 elements.  Beyond that SQ_ALGO_AUTO runs the direct algorithm
 *     (64-bit indices, correct, far slower) and an explicitly chosen tiling
 *     returns SQ_ERR_UNSUPPORTED.  The two network calls reject a batch beyond
 *     SQ_SQUEEZENET_MAX_BATCH / SQ_SQUEEZENET_BF16_MAX_BATCH with
 *     SQ_ERR_UNSUPPORTED before anything is enqueued: split such a batch.
 */
#ifndef SQ_H
#define SQ_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sq_status {
    SQ_OK = 0,
    SQ_ERR_NULL = -1,        /* a required pointer is NULL                         */
    SQ_ERR_SHAPE = -2,       /* a dimension is <= 0, S < 1, P < 0, or K > H + 2P   */
    SQ_ERR_UNSUPPORTED = -3, /* dtype / algorithm / shape no kernel here covers    */
    SQ_ERR_WORKSPACE = -4,   /* workspace missing, misaligned or too small         */
    SQ_ERR_HIP = -5          /* a HIP launch failed; see sq_last_hip_error()       */
} sq_status;

/* Largest batch of sq_squeezenet_forward (conv1's output, 96 x 111 x 111 per image,
 * stays below 2^29 elements) and of sq_squeezenet_forward_bf16 (the same map in
 * bfloat16 stays below 2^31 bytes). */
#define SQ_SQUEEZENET_MAX_BATCH 453
#define SQ_SQUEEZENET_BF16_MAX_BATCH 907

typedef enum sq_dtype {
    SQ_F32 = 0,  /* IEEE binary32 inputs and kernels                               */
    SQ_BF16 = 1  /* bfloat16 inputs and kernels, fp32 accumulate, fp32 bias/output */
} sq_dtype;

/* Algorithm selector of sq_conv2d_forward_ex.  Values >= SQ_ALGO_VARIANT0 pick
 * one tiling of the matrix-core kernel family (how much output one workgroup
 * and one wavefront produce -- the counterpart of the thread granularity g of
 * section "Optimizing Thread Granularity"); sq_conv_variant_count() says how
 * many exist.  Every algorithm must give the same result up to rounding. */
enum {
    SQ_ALGO_AUTO = 0,     /* library's per-shape choice                            */
    SQ_ALGO_DIRECT = 1,   /* one thread per output element, any K, S, P            */
    SQ_ALGO_VARIANT0 = 2  /* first matrix-core tiling; VARIANT0 + i is the i-th    */
};

/* Human-readable text for a status code (static storage, never NULL). */
const char *sq_strerror(int status);

/* hipError_t (as int) of the last failed launch on this host thread, 0 if none. */
int sq_last_hip_error(void);

/* Stream (a hipStream_t passed as void*, NULL = null stream) on which every
 * later call from this host thread enqueues its kernels. */
int sq_set_stream(void *hip_stream);

/* Arithmetic mode of the entry points that carry no dtype argument, for this host thread
 * (default SQ_F32).  SQ_BF16 is the reduced-precision mode standing in for the paper's relaxed
 * arithmetic (section "Imprecise Computing"): bfloat16 operands, fp32 sums, fp32 bias.
 *   sq_conv2d_forward:            `in` and `w` are read as that type (out and b stay fp32).
 *   sq_squeezenet_forward_packed: the network runs in that mode on kernels packed for it.
 *   sq_fire_forward, sq_fire_forward_packed, sq_squeezenet_forward: SQ_F32 only, otherwise
 *     SQ_ERR_UNSUPPORTED (reduced precision works on packed kernels and blocked maps:
 *     sq_blocked_fire_forward, sq_squeezenet_forward_packed).
 * Errors: SQ_ERR_UNSUPPORTED for a value that is not an sq_dtype. */
int sq_set_dtype(int dtype);

/* Optional one-time set-up for the current device: raises the LDS limit of every kernel of the
 * library (see "First use" above).  May be called more than once and from any thread.
 * Errors: SQ_ERR_HIP. */
int sq_init(void);

/* Number of matrix-core tilings and a short name for each ("" if out of range). */
int sq_conv_variant_count(void);
const char *sq_conv_variant_name(int index);

/*
 * Convolution layer (section "Convolutional Neural Networks"; sequential form in
 * section "Parallel Algorithm Design"), with bias and optional ReLU:
 *   out[n][m][oh][ow] = act( b[m] + sum_{c,i,j} in[n][c][oh*S+i-P][ow*S+j-P] * w[m][c][i][j] )
 * taps outside the image contribute zero; act = max(.,0) if relu != 0.
 *   in  [N][Cin][H][W], w [Cout][Cin][K][K], b [Cout] or NULL (= zero),
 *   out [N][Cout][Ho][Wo], Ho = floor((H+2P-K)/S)+1, Wo likewise.  All fp32.
 * Errors: SQ_ERR_NULL (in, w or out NULL), SQ_ERR_SHAPE, SQ_ERR_HIP.
 */
int sq_conv2d_forward(const void *in, const void *w, const float *b, float *out,
                      int N, int Cin, int H, int W, int Cout, int K, int S, int P,
                      int relu);

/*
 * Same operation with three extras.
 *   out_channels, c_offset: the result is written into layers
 *     [c_offset, c_offset + Cout) of an output tensor [N][out_channels][Ho][Wo];
 *     other layers are left untouched.  This is how the two expand convolutions
 *     of a fire layer produce one concatenated tensor with no copy (the paper
 *     likewise stores results directly in the layout the next layer reads,
 *     section "Zero-overhead Vectorization").  Need 0 <= c_offset and
 *     c_offset + Cout <= out_channels, else SQ_ERR_SHAPE.
 *   in_dtype: SQ_F32, or SQ_BF16 = `in` and `w` hold bfloat16 (2 bytes each,
 *     the upper half of the binary32 pattern); products are accumulated in fp32,
 *     b and out stay fp32.  This is the reduced-precision mode standing in for
 *     the paper's relaxed arithmetic (section "Imprecise Computing").
 *   algo: SQ_ALGO_AUTO, SQ_ALGO_DIRECT or SQ_ALGO_VARIANT0 + i.  A variant
 *     that cannot run the given shape returns SQ_ERR_UNSUPPORTED.
 */
int sq_conv2d_forward_ex(const void *in, const void *w, const float *b, float *out,
                         int N, int Cin, int H, int W, int Cout, int K, int S, int P,
                         int relu, int out_channels, int c_offset, int in_dtype,
                         int algo);

/*
 * sq_conv2d_forward_ex with caller scratch.  Some algorithms first rewrite the
 * kernels into another form (the 3x3 stride-1 pad-1 layers can run as a
 * minimal-filtering convolution: 16 instead of 36 multiplications per input layer
 * and 2x2 output pixels, on once-transformed kernels); they need device scratch
 * for that and are only chosen, or selectable through `algo`, when it is given.
 *   workspace: device scratch, 256-byte aligned (else SQ_ERR_WORKSPACE), of
 *     workspace_bytes bytes; NULL = none.  With at least
 *     sq_conv2d_workspace_bytes(Cin, Cout, K, S, P) bytes every algorithm that
 *     fits the shape can run; a smaller one only rules those algorithms out.
 *     Contents on return are unspecified; the same scratch must not be used by
 *     two calls in flight at once.
 *   A layer with stride S >= 2 can also run as a stride-1 convolution of a
 *     space-to-depth copy of its input (S*S times the input layers, kernels of
 *     ceil(K/S) x ceil(K/S)), which the library makes in the workspace; under
 *     SQ_ALGO_AUTO it does so when workspace_bytes is at least
 *     sq_conv2d_strided_workspace_bytes(N, Cin, H, W, Cout, K, S, P) (0 = the
 *     form does not apply) and a matrix-core tiling serves the stride-1 form
 *     (regrouped kernels of 1x1, 3x3 or 5x5: e.g. 11x11 stride 4, 5x5 stride 2).
 *   With bfloat16 operands (in_dtype = SQ_BF16) and workspace_bytes of at least
 *     sq_conv2d_bf16_workspace_bytes(N, Cin, H, W, Cout, K, S, P) (0 = the form
 *     does not apply) SQ_ALGO_AUTO runs the layer on the bfloat16 matrix
 *     instructions: input and kernels are re-ordered inside the workspace, sums
 *     are fp32 and the fp32 results are not rounded.  It applies where that is
 *     faster than widening the operands into the fp32 kernels: 3x3 and 5x5
 *     layers of stride 1 with pad (K-1)/2, 1x1 layers with at least 128 input
 *     layers and more output than input layers, the conv1 type (7x7, stride 2, three input layers, at most
 *     96 output layers); Cin a multiple of 16 (except the conv1 type), Cout a
 *     multiple of 8.  (Sized for out_channels = Cout; a larger output tensor
 *     only matters for the 2^31-byte limit.)
 * Everything else as for sq_conv2d_forward_ex; the result is the same up to
 * rounding whichever algorithm runs.
 */
int sq_conv2d_forward_ws(const void *in, const void *w, const float *b, float *out,
                         int N, int Cin, int H, int W, int Cout, int K, int S, int P,
                         int relu, int out_channels, int c_offset, int in_dtype,
                         int algo, void *workspace, size_t workspace_bytes);

size_t sq_conv2d_workspace_bytes(int Cin, int Cout, int K, int S, int P);
size_t sq_conv2d_strided_workspace_bytes(int N, int Cin, int H, int W, int Cout, int K, int S, int P);
size_t sq_conv2d_bf16_workspace_bytes(int N, int Cin, int H, int W, int Cout, int K, int S, int P);

/*
 * Max pooling (section "Pooling and Softmax"): out[n][c][oh][ow] = largest of the
 * K x K window whose corner is (oh*S, ow*S).  No padding, floor mode:
 * Ho = floor((H-K)/S)+1.  in [N][C][H][W], out [N][C][Ho][Wo], fp32.
 * Errors: SQ_ERR_NULL, SQ_ERR_SHAPE (incl. K > H or K > W), SQ_ERR_HIP.
 */
int sq_maxpool(const float *in, float *out, int N, int C, int H, int W, int K, int S);

/*
 * The network's max pooling (3 x 3 window, stride 2; section "Pooling and
 * Softmax") and the 1 x 1 convolution that reads its result (the squeeze of a
 * fire layer, section "Convolutional Neural Networks"), as one operation: the
 * pooled map is formed while the convolution stages its input and is never
 * written to memory.  The result equals sq_maxpool(in, K=3, S=2) followed by
 * sq_conv2d_forward_ex(K=1, S=1, P=0) with the same algorithm, bit for bit
 * (the maximum is exact and the contraction runs in the same order).
 *   in:  [N][Cin][H][W] fp32, H >= 3 and W >= 3 (else SQ_ERR_SHAPE)
 *   w:   [Cout][Cin] fp32;  b: [Cout] fp32 or NULL
 *   out: [N][out_channels][Hp][Wp] fp32 with Hp = floor((H-3)/2)+1, likewise Wp;
 *        layers [c_offset, c_offset+Cout) are written
 *   algo: SQ_ALGO_AUTO or SQ_ALGO_VARIANT0 + i for a 1 x 1 tiling of the fp32
 *        matrix-core kernel whose input-layer chunk divides Cin; anything else
 *        returns SQ_ERR_UNSUPPORTED (there is no other implementation).
 * All pointers are device pointers owned by the caller.
 */
int sq_maxpool_conv2d_forward(const float *in, const float *w, const float *b, float *out,
                              int N, int Cin, int H, int W, int Cout, int relu,
                              int out_channels, int c_offset, int algo);

/*
 * Average pooling over the whole plane (section "Pooling and Softmax"; the
 * network applies it to the 13 x 13 classifier maps):
 * out[n][c] = mean over h,w of in[n][c][h][w].  in [N][C][H][W], out [N][C].
 */
int sq_avgpool_global(const float *in, float *out, int N, int C, int H, int W);

/*
 * Softmax over the C scores of each image (section "Pooling and Softmax"; the
 * paper leaves it on the CPU, here it runs on the GPU so the network call has no
 * host round trip): out[n][c] = exp(in[n][c] - max_n) / sum_c exp(in[n][c] - max_n).
 * in, out [N][C].
 */
int sq_softmax(const float *in, float *out, int N, int C);

/*
 * The classifier end of the network as one operation (sections "Convolutional Neural Networks"
 * and "Pooling and Softmax"): 1 x 1 convolution with bias and ReLU, average pooling over the
 * whole plane, softmax over the layers:
 *   means[n][m] = mean over h,w of relu(b[m] + sum_c in[n][c][h][w] * w[m][c]),
 *   probs[n][m] = exp(means[n][m] - max_n) / sum_m exp(means[n][m] - max_n).
 * The convolution's map [N][Cout][H][W] is not formed in memory where the library has a kernel
 * for that (the convolution then writes per-image sums of its results, and a second launch
 * finishes means and softmax); otherwise the three layers run one after the other.  The result
 * is the same up to rounding.
 *   in [N][Cin][H][W], w [Cout][Cin], b [Cout] or NULL, all fp32 (device).
 *   means [N][Cout] or NULL (not wanted); probs [N][Cout].
 *   workspace: device scratch of at least sq_classifier_workspace_bytes(N, Cin, H, W, Cout)
 *   bytes, 256-byte aligned; contents on return are unspecified.
 * Errors: SQ_ERR_NULL, SQ_ERR_SHAPE, SQ_ERR_WORKSPACE, SQ_ERR_UNSUPPORTED (under
 * sq_set_dtype(SQ_BF16)), SQ_ERR_HIP.
 */
size_t sq_classifier_workspace_bytes(int N, int Cin, int H, int W, int Cout);
int sq_classifier_forward(const float *in, const float *w, const float *b, float *means,
                          float *probs, int N, int Cin, int H, int W, int Cout,
                          void *workspace, size_t workspace_bytes);

/*
 * Fire layer (section "Convolutional Neural Networks": one squeeze layer and two
 * expand layers).  s = relu(conv1x1(in; w_sq, b_sq)) with Csq layers;
 * out layers [0, Ce1)        = relu(conv1x1(s; w_e1, b_e1)),
 * out layers [Ce1, Ce1+Ce3)  = relu(conv3x3 pad 1 (s; w_e3, b_e3)); the padding
 * of the 3x3 is zero in the squeeze map s.
 *   in [N][Cin][H][W]; w_sq [Csq][Cin][1][1]; w_e1 [Ce1][Csq][1][1];
 *   w_e3 [Ce3][Csq][3][3]; biases [Csq], [Ce1], [Ce3] (each may be NULL);
 *   out [N][Ce1+Ce3][H][W].  All fp32.
 *   workspace: device scratch of at least sq_fire_workspace_bytes(N, H, W, Csq, Ce3)
 *   bytes, 256-byte aligned, holding the squeeze map and the transformed 3x3
 *   kernels during the call; contents on return are unspecified.
 * Errors: SQ_ERR_NULL, SQ_ERR_SHAPE, SQ_ERR_WORKSPACE, SQ_ERR_HIP.
 */
int sq_fire_forward(const void *in, const void *w_sq, const float *b_sq,
                    const void *w_e1, const float *b_e1, const void *w_e3,
                    const float *b_e3, float *out, int N, int Cin, int H, int W,
                    int Csq, int Ce1, int Ce3, void *workspace, size_t workspace_bytes);

size_t sq_fire_workspace_bytes(int N, int H, int W, int Csq, int Ce3);

/*
 * sq_fire_forward for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * operation, same kernels and same results as sq_fire_forward, bit for bit; the squeeze map and
 * the transformed 3x3 kernels live in an array of SQ_FIRE_STATIC_SCRATCH_BYTES bytes that is
 * part of the library's device code (each GPU the library runs on holds its own copy until the
 * process ends).  The call allocates and frees nothing.
 *   Limit: sq_fire_workspace_bytes(N, H, W, Csq, Ce3) <= SQ_FIRE_STATIC_SCRATCH_BYTES, otherwise
 *   SQ_ERR_WORKSPACE and nothing is enqueued (fire2 of the network fits up to 172 images, fire9
 *   up to 751).
 *   All calls on one GPU share that GPU's array: two such calls in flight at once on one GPU --
 *   from two streams or two threads -- race.  Calls on one stream are ordered and safe.  Nothing
 *   in the array needs clearing between calls: every byte a call reads it has written first.
 *   The first call on a device (or sq_init()) looks the array's device address up once
 *   (hipGetSymbolAddress); call sq_init() before capturing this entry point in a graph.
 * Errors: as sq_fire_forward.
 */
#define SQ_FIRE_STATIC_SCRATCH_BYTES (32u << 20)
int sq_fire_forward_static(const void *in, const void *w_sq, const float *b_sq,
                           const void *w_e1, const float *b_e1, const void *w_e3,
                           const float *b_e3, float *out, int N, int Cin, int H, int W,
                           int Csq, int Ce1, int Ce3);

/*
 * The fire layer on kernels re-ordered ahead of time (section "Zero-overhead Vectorization":
 * the paper re-orders the kernels once, offline, into the order its threads read them).
 * Here the re-ordered form of the expand3x3 kernels is their minimal-filtering transform
 * G g G^T, laid out in the order the matrix-core lanes load it.
 *   sq_fire_packed_bytes(Csq, Ce3): size of that form; 0 = the shape has none (Csq not a
 *     multiple of 8 or Ce3 not a multiple of 32): use sq_fire_forward.
 *   sq_fire_pack_weights(): writes it from w_e3 [Ce3][Csq][3][3] (fp32) into `packed` (device,
 *     256-byte aligned, at least sq_fire_packed_bytes bytes).  One launch on the thread's stream.
 *   sq_fire_forward_packed(): sq_fire_forward without the per-call transform; `packed_e3` is
 *     only read.  workspace: at least N*Csq*H*W*4 bytes rounded up to 256 (the squeeze map).
 * Errors: as sq_fire_forward; SQ_ERR_UNSUPPORTED where sq_fire_packed_bytes is 0.
 */
size_t sq_fire_packed_bytes(int Csq, int Ce3);
int sq_fire_pack_weights(const void *w_e3, void *packed, size_t packed_bytes, int Csq, int Ce3);
int sq_fire_forward_packed(const void *in, const void *w_sq, const float *b_sq,
                           const void *w_e1, const float *b_e1, const void *w_e3,
                           const float *b_e3, const void *packed_e3, float *out, int N,
                           int Cin, int H, int W, int Csq, int Ce1, int Ce3,
                           void *workspace, size_t workspace_bytes);

/*
 * SqueezeNet v1.0 forward (section "Convolutional Neural Networks": two
 * convolution layers and eight fire layers; 224 x 224 RGB input, 1000 classes):
 *   conv1 96@7x7 stride 2 pad 2 +ReLU -> maxpool 3/2 -> fire2 (16, 64+64) ->
 *   fire3 (16, 64+64) -> fire4 (32, 128+128) -> maxpool 3/2 -> fire5 (32, 128+128)
 *   -> fire6 (48, 192+192) -> fire7 (48, 192+192) -> fire8 (64, 256+256) ->
 *   maxpool 3/2 -> fire9 (64, 256+256) -> conv10 1x1 to 1000 +ReLU ->
 *   global average pool 13x13 -> softmax.
 * (conv1 takes pad 2 so that 224 -> 111 -> 55 -> 27 -> 13.)
 *   in     [N][3][224][224] fp32 (device).
 *   params HOST array of 52 DEVICE pointers: kernel then bias of each of the 26
 *          convolutions in network order (conv1; squeeze, expand1x1, expand3x3 of
 *          fire2..fire9; conv10), shapes as above, fp32.  No bias may be NULL.
 *   probs  [N][1000] fp32 (device), rows sum to 1.
 *   workspace: device scratch of at least sq_squeezenet_workspace_bytes(N) bytes,
 *          256-byte aligned; holds every intermediate activation.
 *   taps   NULL, or a HOST array of 16 DEVICE pointers; each non-NULL entry
 *          receives a copy of one stage's result: 0 conv1 [N][96][111][111],
 *          1 pool1 [N][96][55][55], 2 fire2, 3 fire3 [N][128][55][55], 4 fire4
 *          [N][256][55][55], 5 pool4 [N][256][27][27], 6 fire5, 7 fire6, 8 fire7
 *          [N][384][27][27], 9 fire8 [N][512][27][27], 10 pool8, 11 fire9
 *          [N][512][13][13], 12 conv10 [N][1000][13][13], 13 class means
 *          [N][1000], 14 probabilities [N][1000], 15 reserved (must be NULL).
 * Errors: SQ_ERR_NULL, SQ_ERR_SHAPE (N <= 0), SQ_ERR_WORKSPACE, SQ_ERR_HIP.
 */
int sq_squeezenet_forward(const void *in, const void *const *params, float *probs,
                          int N, void *workspace, size_t workspace_bytes,
                          float *const *taps);

size_t sq_squeezenet_workspace_bytes(int N);

/*
 * The network on kernels re-ordered once, ahead of time (section "Zero-overhead
 * Vectorization"), in the arithmetic mode of sq_set_dtype():
 *   sq_packed_weights_bytes(dtype): size of the packed kernels for that mode.
 *   sq_pack_weights(params, dtype, packed, packed_bytes): writes them (device memory, 256-byte
 *     aligned) from the parameter table of sq_squeezenet_forward.  SQ_F32: the minimal-filtering
 *     transforms of the eight expand3x3 kernels (every other fp32 kernel is read as it lies);
 *     SQ_BF16: all 26 kernels as bfloat16 in matrix-core operand order (the same bytes as
 *     sq_squeezenet_bf16_pack_params).  Not part of a timed forward pass.
 *   sq_squeezenet_forward_packed(): sq_squeezenet_forward without the per-call kernel
 *     transform (SQ_F32), or sq_squeezenet_forward_bf16 on an fp32 image (SQ_BF16); `packed`
 *     must have been written for the mode in force and is only read.  Workspace and taps as
 *     for sq_squeezenet_forward.
 * Errors: SQ_ERR_NULL, SQ_ERR_SHAPE, SQ_ERR_WORKSPACE (packed misaligned or too small),
 * SQ_ERR_UNSUPPORTED (unknown dtype, batch too large), SQ_ERR_HIP.
 */
size_t sq_packed_weights_bytes(int dtype);
int sq_pack_weights(const void *const *params, int dtype, void *packed, size_t packed_bytes);
int sq_squeezenet_forward_packed(const void *in, const void *const *params, const void *packed,
                                 float *probs, int N, void *workspace, size_t workspace_bytes,
                                 float *const *taps);

/*
 * Reduced-precision path (the counterpart of the paper's relaxed-precision mode,
 * section "Imprecise computing", on the layer-private vector layout of sections
 * "Data Reordering" and "Zero-overhead vectorization"): feature maps and kernels are
 * bfloat16, every sum is accumulated in fp32, biases stay fp32, and every layer
 * writes its result directly in the layout the next one reads.
 *
 * Blocked map: [N][ceil(C/8)][H][W][8] bfloat16 (device) -- the eight layers
 * 8k..8k+7 of one pixel are adjacent; layers past C in the last block hold zero.
 * sq_blocked_map_bytes() is its size.  sq_blocked_pack() converts an NCHW tensor
 * (in_dtype SQ_F32 or SQ_BF16; fp32 values are rounded to nearest even) into it,
 * sq_blocked_unpack() converts a blocked map back to fp32 NCHW (exact).
 *
 * Packed kernels: sq_blocked_pack_kernels() re-orders the kernels [Cout][Cin][K][K]
 * (w_dtype SQ_F32 or SQ_BF16) of one convolution once, ahead of time, into the order
 * the matrix cores read them (sq_blocked_kernel_bytes() bytes, 16-byte aligned).
 *
 * sq_blocked_conv2d_forward(): K x K convolution, stride 1, zero padding P = (K-1)/2
 * (K = 1, 3 or 5), +bias, optional ReLU, on a blocked map; the Cout results, rounded
 * to bfloat16, go to layers [c_offset, c_offset+Cout) of a blocked map with
 * ldc_channels layers (the concatenation hook of the fire layer).  Cin must be a
 * multiple of 16; Cout, ldc_channels and c_offset multiples of 8; the kernels of 32
 * output layers (K*K*Cin*64 bytes) must fit half the LDS -- otherwise
 * SQ_ERR_UNSUPPORTED.  in and out must not overlap.
 * sq_blocked_conv7s2_forward(): the conv1-type layer -- 7 x 7 kernels, stride 2, zero
 * padding P, exactly three input layers -- reading an NCHW image (in_dtype SQ_F32 or
 * SQ_BF16; fp32 pixels are rounded to bfloat16 as they are staged) and writing layers
 * [c_offset, c_offset+Cout) of a blocked map [N][ldc_channels/8][Ho][Wo][8],
 * Ho = (H + 2P - 7)/2 + 1.  Cout <= 96 and a multiple of 8.  Its kernels
 * [Cout][3][7][7] are packed by sq_blocked_pack_kernels7() into a buffer of
 * sq_blocked_kernel7_bytes() bytes.
 * sq_blocked_fire_forward(): the fire layer of sq_fire_forward on blocked maps, with
 * packed kernels (squeeze [Csq][Cin][1][1], expand [Ce1][Csq][1][1] and [Ce3][Csq][3][3]);
 * the squeeze map is rounded to bfloat16, both expands run in one launch and write
 * layers [0, Ce1) and [Ce1, Ce1+Ce3) of out.  workspace:
 * device scratch of at least sq_blocked_map_bytes(N, Csq, H, W) bytes, 256-byte aligned
 * (room for the squeeze map; contents on return are unspecified).
 * Cin and Csq multiples of 16, Ce1 and Ce3 multiples of 8.
 * sq_blocked_pool_conv2d_forward(): max pooling (3 x 3 window, stride 2, floor mode) of a
 * blocked map [N][Cin/8][Hin][Win][8] followed by a 1 x 1 convolution (+bias, optional
 * ReLU) to Cout layers, in one launch; the pooled map is not written.  The result has
 * extents H = (Hin-3)/2 + 1, W = (Win-3)/2 + 1 and equals sq_blocked_maxpool followed by
 * sq_blocked_conv2d_forward bit for bit.  Same divisibility rules as the convolution.
 * sq_blocked_maxpool(): K x K window, stride S, floor mode, no padding.
 * sq_blocked_avgpool_global(): mean over H x W of each layer, fp32 [N][C] out.
 * Errors: SQ_ERR_NULL, SQ_ERR_SHAPE, SQ_ERR_UNSUPPORTED, SQ_ERR_HIP.
 */
size_t sq_blocked_map_bytes(int N, int C, int H, int W);
int sq_blocked_pack(const void *in, sq_dtype in_dtype, void *out, int N, int C, int H, int W);
int sq_blocked_unpack(const void *in, float *out, int N, int C, int H, int W);
size_t sq_blocked_kernel_bytes(int Cout, int Cin, int K);
int sq_blocked_pack_kernels(const void *w, sq_dtype w_dtype, void *packed, int Cout, int Cin, int K);
int sq_blocked_conv2d_forward(const void *in, const void *packed_w, const float *b, void *out,
                              int N, int Cin, int H, int W, int Cout, int K, int P, int relu,
                              int ldc_channels, int c_offset);
size_t sq_blocked_kernel7_bytes(void);
int sq_blocked_pack_kernels7(const void *w, sq_dtype w_dtype, void *packed, int Cout);
int sq_blocked_conv7s2_forward(const void *in, sq_dtype in_dtype, const void *packed_w, const float *b,
                               void *out, int N, int H, int W, int Cout, int P, int relu,
                               int ldc_channels, int c_offset);
int sq_blocked_pool_conv2d_forward(const void *in, const void *packed_w, const float *b, void *out,
                                   int N, int Cin, int Hin, int Win, int Cout, int relu,
                                   int ldc_channels, int c_offset);
int sq_blocked_fire_forward(const void *in, const void *packed_sq, const float *b_sq,
                            const void *packed_e1, const float *b_e1, const void *packed_e3,
                            const float *b_e3, void *out, int N, int Cin, int H, int W,
                            int Csq, int Ce1, int Ce3, void *workspace, size_t workspace_bytes);
int sq_blocked_maxpool(const void *in, void *out, int N, int C, int H, int W, int K, int S);
int sq_blocked_avgpool_global(const void *in, float *out, int N, int C, int H, int W);

/*
 * SqueezeNet v1.0 forward in reduced precision: the network of sq_squeezenet_forward
 * with bfloat16 feature maps and kernels (fp32 sums, fp32 biases, fp32 class means
 * and probabilities).  conv1 reads the NCHW image (in_dtype SQ_F32, or SQ_BF16 for a
 * bfloat16 image; fp32 pixels are rounded to bfloat16 as they are staged) and writes a
 * blocked map; everything after it stays blocked.
 *   params  as for sq_squeezenet_forward (fp32; only the biases are read here).
 *   packed  device buffer of sq_squeezenet_bf16_packed_bytes() bytes, 256-byte
 *           aligned, filled once by sq_squeezenet_bf16_pack_params(params, packed,
 *           bytes) -- the ahead-of-time kernel re-ordering.
 *   workspace: at least sq_squeezenet_bf16_workspace_bytes(N) bytes, 256-byte aligned.
 *   taps    as for sq_squeezenet_forward: fp32 NCHW copies of the stage results
 *           (converted back from the blocked maps); NULL in timed runs.
 * Errors: SQ_ERR_NULL, SQ_ERR_SHAPE, SQ_ERR_WORKSPACE, SQ_ERR_UNSUPPORTED, SQ_ERR_HIP.
 */
size_t sq_squeezenet_bf16_packed_bytes(void);
int sq_squeezenet_bf16_pack_params(const void *const *params, void *packed, size_t packed_bytes);
size_t sq_squeezenet_bf16_workspace_bytes(int N);
int sq_squeezenet_forward_bf16(const void *in, sq_dtype in_dtype, const void *const *params,
                               const void *packed, float *probs, int N, void *workspace,
                               size_t workspace_bytes, float *const *taps);

/*
 * Per-launch timing, off by default.  Between sq_profile_begin() and sq_profile_end()
 * every kernel the library launches from this host thread is bracketed by a pair of
 * HIP events on the library's stream.  These two calls are the only ones in the
 * library that create and destroy HIP objects; sq_profile_end() also waits for the
 * recorded work.  Launches beyond max_launches are not recorded.
 * After sq_profile_end(), sq_profile_count() entries can be read with
 * sq_profile_get(): one entry per distinct "stage|kernel" name (stage is the network
 * stage, e.g. "fire4/e3", empty outside sq_squeezenet_forward and sq_fire_forward),
 * with its launch count, summed duration in milliseconds and summed algorithmic FLOPs
 * (2 x multiply-accumulates of the layer definition, nothing for padding or tile
 * waste) and algorithmic bytes (each input, kernel and output element once).
 * Errors: SQ_ERR_SHAPE (bad count/index), SQ_ERR_UNSUPPORTED (begin twice / end
 * without begin), SQ_ERR_NULL, SQ_ERR_HIP.
 */
int sq_profile_begin(int max_launches);
int sq_profile_end(void);
int sq_profile_count(void);
int sq_profile_get(int index, char *name, int name_cap, long long *launches,
                   double *total_ms, double *flops, double *bytes);
/* For the same entry: the floating-point operations its launches issued on the matrix cores (2 x the
 * multiply-accumulates of the MFMA instructions executed: padding of tiles, contraction and layers
 * included; for the minimal-filtering kernels the products they really form, 16 instead of 36 per input
 * layer and 2 x 2 pixels).  Divided by the time this is matrix-core utilisation, where flops / time is
 * the algorithmic rate.  0 for kernels without MFMA instructions. */
int sq_profile_get_mfma_flops(int index, double *mfma_flops);

#ifdef __cplusplus
}
#endif
#endif /* SQ_H */
