// Internal declarations shared by the library's translation units (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "sq.h"
#include "sq_tuning.h"

namespace sq {

// Stream of the calling host thread (set by sq_set_stream).
hipStream_t current_stream();

// Compute units of the current device (256 if the query fails); cached after the first call.
int num_cus();

// Folds the sticky launch error into a status code and records it.
int check_launch();

// Arithmetic mode of the calling host thread (set by sq_set_dtype).
int current_dtype();

// Raises the dynamic-LDS limit of a kernel function to the hardware's 160 KB the first time it is asked for
// that function; safe to call from several host threads.  sq_init() asks for every kernel of the library, so
// that no later call issues anything but launches.
bool allow_big_lds(const void *fn);
bool conv_mfma_register_kernels();
bool blocked_register_kernels();
bool fire_bf16_register_kernels();

// One convolution call after validation.  Ho/Wo are precomputed; the result goes
// to layers [c_offset, c_offset+Cout) of an [N][out_channels][Ho][Wo] tensor.
// Max pooling (3x3 window, stride 2, floor mode; section "Pooling and Softmax") split between the layer before it and
// the 1x1 layer behind it, so that about half of the producer's map goes through memory and the pooled map never
// exists.  The producer (a layer with ReLU) writes a column-pooled map [N][layers][Ho][row_stride]: for pooled column x
// (x < Wp = (Wo - 3) / 2 + 1) of its row r the maximum of its columns 2x, 2x+1, 2x+2.  Its work items cover 2 rows x
// 2^shift pooled columns ("groups"; pooled column x of producer tile row ty of image n is slot q = n * slots_image +
// ty * slots_row + x, group = q >> shift).  In the last slot of a group the third column lies in the next group:
// the value there is the maximum of two columns only, and the next group's item writes its first column, unpooled,
// into a seam slot right behind it.  So column x of tile row ty sits at position x + (number of group ends before
// it in this row) = x + ((q0 + x) >> shift) - (q0 >> shift), q0 = the row's first slot, and a seam slot follows
// wherever (q0 + x) % 2^shift is the last of its group.  The consumer takes the maximum over rows 2y..2y+2 and, at
// those columns, the seam slots (one 8-byte load per row), and a zero: the producer's ReLU, which it leaves to the
// consumer (the map holds values before ReLU; relu(max(a, b)) = max(relu(a), relu(b))).  Exact: a maximum picks one
// of the producer's values whatever the order.
struct ColPool {
    int shift = 0, slots_row = 0, slots_image = 0;
    int row_stride = 0;   // floats per row of the map: Wp + (Wp >> shift) + 2 holds every seam slot
};
inline int colpool_row_stride(int Wo, int shift) { const int Wp = (Wo - 3) / 2 + 1; return Wp + (Wp >> shift) + 2; }

struct ConvArgs {
    const void *in;
    const void *w;
    const float *b;
    float *out;
    int N, Cin, H, W, Cout, K, S, P, relu;
    int Ho, Wo, out_channels, c_offset;
    int dtype;  // sq_dtype of in and w
    void *ws;         // caller scratch some algorithms need (16-byte aligned), or nullptr
    size_t ws_bytes;
    bool ws_ready;    // ws already holds this layer's transformed kernels (conv_prepare_kernels)
    // 1x1 convolution of a map that is max-pooled (3x3 window, stride 2, no padding) on the way in: extents of
    // the map in memory; H and W are then the pooled extents.  0 = the input is read as it is.
    int pool_H, pool_W;
    // split pooling: cp_in = `in` is a column-pooled map of pool_H rows (pool_W = the producer's row length before
    // pooling, W = the number of pooled columns) and this 1x1 layer pools the rows; cp_out = this layer writes such a
    // map instead of its plain map (conv1-type and expand-pair kernels; Ho, Wo stay the unpooled extents)
    bool cp_in = false, cp_out = false;
    ColPool cp;
};

inline double conv_flops(const ConvArgs &a)
{
    return 2.0 * a.N * a.Cout * a.Ho * a.Wo * (double)a.Cin * a.K * a.K;
}
inline double conv_bytes(const ConvArgs &a)
{
    const double esz = a.dtype == SQ_BF16 ? 2.0 : 4.0;
    const double in_plane = a.cp_in ? (double)a.pool_H * a.cp.row_stride : a.pool_H ? (double)a.pool_H * a.pool_W : (double)a.H * a.W;
    return esz * ((double)a.N * a.Cin * in_plane + (double)a.Cout * a.Cin * a.K * a.K) +
           4.0 * ((double)a.N * a.Cout * a.Ho * (a.cp_out ? a.cp.row_stride : a.Wo) + a.Cout);
}

int conv_direct(const ConvArgs &a);

// Matrix-core family.  variant < 0 = pick by shape; returns SQ_ERR_UNSUPPORTED when
// the (variant, shape, dtype) combination has no kernel.
int conv_mfma(const ConvArgs &a, int variant);
// Both expands of a fire layer (a3: 3x3 pad 1, a1: 1x1, same input map and output tensor) in one launch, where the
// measured choice for a3 is the minimal-filtering kernel and a compiled expand1x1 tiling fits; SQ_ERR_UNSUPPORTED
// otherwise.
int conv_expand_pair(const ConvArgs &a3, const ConvArgs &a1);
// whether conv_expand_pair has a kernel for (a3, a1) -- nothing is launched
bool conv_expand_pair_supported(const ConvArgs &a3, const ConvArgs &a1);
// 1x1 convolution (+bias, ReLU) followed directly by a global average pooling: the convolution kernel writes per-image
// plane sums of its results (a table of conv_mfma_avg_bytes() bytes, laid out as AvgLayout says) instead of the results;
// avg_softmax() adds them up, divides by the plane size and applies softmax.  variant < 0 = the tiling of the
// automatic choice.  SQ_ERR_UNSUPPORTED / 0 bytes where that tiling has no averaging form.
struct AvgLayout {
    int ntiles, WN, slots, BN;
};
size_t conv_mfma_avg_bytes(const ConvArgs &a, int variant);
int conv_mfma_avg(const ConvArgs &a, int variant, float *sums, size_t sums_bytes, AvgLayout *lay);
int avg_softmax(const float *sums, const AvgLayout &lay, float *means, float *probs, int N, int C, int HW);
// The tiling conv_mfma(a, -1) runs, or -1.
int conv_mfma_choice(const ConvArgs &a);
// Fused expand of a fire layer: the 3x3 convolution a3 and a 1x1 convolution of the same
// input in one launch; SQ_ERR_UNSUPPORTED if no compiled tiling fits.
int conv_expand_fused(const ConvArgs &a3, const void *w1, const float *b1, int Cout1, int coff1);
// Scratch bytes with which every algorithm can run this layer shape (0 if none needs any).
size_t conv_workspace_bytes(int Cin, int Cout, int K, int S, int P);
// Transforms the 3x3 kernels of n <= 8 layers (fp32) into their scratch areas in one launch;
// a layer whose ConvArgs then carries that area with ws_ready set skips its own transform.
struct KernelPrepJob {
    const void *w;
    void *ws;
    int Cin, Cout;
};
int conv_prepare_kernels(const KernelPrepJob *jobs, int n, int dtype);
// Whether this call will run an algorithm that works on transformed kernels; fire_expand says that it is the
// expand3x3 of a fire layer, which may share a launch with the expand1x1 (conv_expand_pair).
bool conv_wants_prepared_kernels(const ConvArgs &a, bool fire_expand);
// A convolution of stride >= 2 as a stride-1 convolution of a space-to-depth copy of its input (conv_s2d.hip): needs
// a.ws of conv_s2d_workspace_bytes() bytes; SQ_ERR_UNSUPPORTED where that form has no matrix-core tiling.
size_t conv_s2d_workspace_bytes(int N, int Cin, int H, int W, int Cout, int K, int S, int P);
int conv_s2d(const ConvArgs &a);
int conv_mfma_variant_count();
const char *conv_mfma_variant_name(int i);

// Reduced-precision path on blocked bfloat16 maps [N][ceil(C/8)][H][W][8] (blocked_bf16.hip).
size_t blocked_map_bytes(int N, int C, int H, int W);
size_t blocked_packed_kernel_bytes(int Cout, int Cin, int K);
bool blocked_conv_supported(int Cin, int Cout, int K, int P);
int blocked_pack_map(const void *in, int dtype, void *out, int N, int C, int H, int W);
int blocked_unpack_map(const void *in, float *out, int N, int C, int H, int W);
int blocked_pack_kernels(const void *w, int dtype, void *packed, int Cout, int Cin, int K);
// f32_out: `out` is an fp32 NCHW map of ldc_channels layers and takes the unrounded results
int blocked_conv(const void *in, const void *wp, const float *b, void *out, int N, int Cin, int H, int W, int Cout, int K, int P,
                 int relu, int ldc_channels, int c_offset, bool f32_out = false);
size_t blocked_packed_kernel7_bytes();
int blocked_pack_kernels7(const void *w, int dtype, void *packed, int Cout);
int blocked_conv7s2(const void *in, int dtype, const void *wp, const float *b, void *out, int N, int H, int W, int Cout, int P,
                    int relu, int ldc_channels, int c_offset, bool f32_out = false);
// A convolution with bfloat16 NCHW inputs and kernels on the bf16 matrix instructions: the input is re-ordered into a
// blocked map and the kernels into operand order in the caller's scratch, and the blocked kernel writes fp32 NCHW
// results (fp32 accumulate, nothing rounded after the inputs).  For the layers where that beats widening the inputs
// into the fp32 kernels: 3x3 and 5x5 stride 1, wide 1x1 with more output than input layers, the conv1 type.  Bytes of
// scratch (0 = the form does not apply to the shape) and the call (SQ_ERR_UNSUPPORTED / SQ_ERR_WORKSPACE: take the
// other path).
size_t conv_bf16_mfma_workspace_bytes(int N, int Cin, int H, int W, int Cout, int K, int S, int P, int out_channels);
int conv_bf16_mfma(const ConvArgs &a);
int blocked_conv_pair(const void *in, const void *wp1, const float *b1, int Cout1, int c_offset1, const void *wpk,
                      const float *bk, int Coutk, int c_offsetk, int K, void *out, int N, int Cin, int H, int W, int relu,
                      int ldc_channels);
bool blocked_fire_fused_supported(int Cin, int Csq, int Ce1, int Ce3, int W);
int blocked_fire_fused(const void *in, const void *wp_sq, const float *b_sq, const void *wp_e1, const float *b_e1,
                       const void *wp_e3, const float *b_e3, void *out, int N, int Cin, int H, int W, int Csq, int Ce1,
                       int Ce3);
int blocked_pool_conv(const void *in, const void *wp, const float *b, void *out, int N, int Cin, int Hin, int Win, int Cout,
                      int relu, int ldc_channels, int c_offset);
int blocked_maxpool(const void *in, void *out, int N, int C, int H, int W, int K, int S);
int blocked_avgpool_global(const void *in, float *out, int N, int C, int H, int W);

int maxpool(const float *in, float *out, int N, int C, int H, int W, int K, int S);
int avgpool_global(const float *in, float *out, int N, int C, int H, int W);
int softmax(const float *in, float *out, int N, int C);

// Optional per-launch timing (sq_profile_begin/end).  A LaunchScope brackets one kernel
// launch with a pair of HIP events on the library's stream when profiling is on and
// costs one thread-local load when it is off.  flops and bytes are the algorithmic
// figures of the launch (2 * MACs; compulsory input + kernel + output bytes).
// mfma_flops: the floating-point operations the launch issues on the matrix cores (2 x the multiply-accumulates of
// its MFMA instructions: tile, contraction and layer padding included, and for the minimal-filtering kernels the
// products they really form); negative = the same as flops, 0 = none (a kernel without MFMA instructions).
struct LaunchScope {
    LaunchScope(const char *kernel, double flops, double bytes, double mfma_flops = -1.0);
    ~LaunchScope();
    int slot;
};
// Name of the network stage the next launches belong to ("" outside the network call).
void set_stage(const char *stage);

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace sq
