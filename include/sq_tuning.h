/*
 * sq_tuning.h -- measurement and test hooks of libsq.so.  Not part of the interface a user of
 * the library needs: they override, for the calling host thread only, choices the library
 * otherwise makes from measured tables, so that the tuner can time every form and the tests
 * can run every form against the reference results.  Each setter returns nothing and takes
 * effect for later calls of the same thread; passing the default restores the library's own
 * choice.
 */
#ifndef SQ_TUNING_H
#define SQ_TUNING_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* fp32 network: which 3x3 stride-2 max poolings run inside the squeeze layer that reads them
 * (bit 0 pool1, bit 1 pool4, bit 2 pool8), and which are split between the layer before them, which
 * pools the columns as it writes, and that squeeze layer, which pools the rows as it reads (bits 3, 4, 5;
 * a split without a kernel for its shape runs like bits 0..2); -1 = by batch size (default). */
void sq_tune_fuse_pools_f32(int mask);

/* The kernels behind bits 3..5 of sq_tune_fuse_pools_f32, one at a time, for the tests and the tuner (fp32, device
 * pointers, the conventions of sq.h).  A "column-pooled map" of a layer with Ho x Wo results per output layer is
 * [N][layers][Ho][geometry[3]] floats: row r holds, for pooled column x < (Wo - 3) / 2 + 1, the maximum of columns
 * 2x, 2x+1, 2x+2 of the layer's row r BEFORE its ReLU (the reader applies it).  The writer's work items cover two
 * rows and 2^geometry[0] pooled columns; pooled column x of its tile row ty (rows 2ty, 2ty+1) of image n is slot
 * q = n * geometry[2] + ty * geometry[1] + x.  Where q + 1 is a multiple of 2^geometry[0] the third column is
 * missing from the maximum and sits on its own in a seam slot right behind; so column x is found at position
 * x + ((q0 + x) >> geometry[0]) - (q0 >> geometry[0]) of its row, q0 = the slot of x = 0.  Other positions are
 * not written.
 *   sq_tune_conv2d_forward_poolcols: a conv1-type layer (Cin = 3, K = 7, S = 2, Cout = 96, bias, ReLU) writing the
 *     column-pooled map of its result into out (room for N * Cout * Ho * Wo floats is enough); fills geometry[4].
 *   sq_tune_fire_forward_poolcols: sq_fire_forward with the same kind of output.  SQ_ERR_UNSUPPORTED where no
 *     kernel does it for the shape (nothing is launched then).
 *   sq_tune_poolrows_conv2d_forward: sq_maxpool_conv2d_forward reading a column-pooled map of H x W results per
 *     layer (H, W: the extents before any pooling) with the given geometry: pools the rows, applies the writer's ReLU. */
int sq_tune_conv2d_forward_poolcols(const float *in, const float *w, const float *b, float *out, int N, int Cin, int H, int W,
                                    int Cout, int K, int S, int P, int *geometry);
int sq_tune_fire_forward_poolcols(const float *in, const float *w_sq, const float *b_sq, const float *w_e1, const float *b_e1,
                                  const float *w_e3, const float *b_e3, float *out, int N, int Cin, int H, int W, int Csq,
                                  int Ce1, int Ce3, void *workspace, size_t workspace_bytes, int *geometry);
int sq_tune_poolrows_conv2d_forward(const float *in, const float *w, const float *b, float *out, int N, int Cin, int H, int W,
                                    int Cout, int relu, int out_channels, int c_offset, int algo, const int *geometry);

/* fp32 network and sq_classifier_forward: the last convolution writes plane sums for the average pooling
 * instead of its map (1), convolution, pooling and softmax run one after the other (0), or the batch size decides
 * (-1, default: plane sums from eight images on). */
void sq_tune_fuse_classifier(int on);

/* fp32 fire layer, both expands in one launch behind the minimal-filtering expand3x3:
 * -1 = from three images on, in the form measured faster for the layer (default), 0 = never,
 * 1 + i = in the i-th compiled form (0, 1: four-wavefront expand3x3 with expand1x1 tiles of 64x128 / 64x256 behind it;
 * 2: autonomous-wavefront expand3x3 with the expand1x1 inside its items). */
void sq_tune_expand_pair(int v);

/* fp32 fire layer, both expands inside the tiles of one direct 3x3 kernel: -3 = never, -2 = up to
 * 16 images (default), -1 = always, i >= 0 = always with tiling i of sq_conv_variant_name. */
void sq_tune_force_expand(int v);

/* Reduced-precision network: poolings inside the following squeeze (bits as above); -1 = default. */
void sq_tune_fuse_pools(int mask);

/* Reduced-precision fire layer as a single launch: 1 = where the shape allows, 0 = never,
 * -1 = by batch size (default: never, it measured slower). */
void sq_tune_fire_one_launch(int mode);

/* Reduced-precision convolution: operand ring depth (0 = automatic), and blocks of 32 output layers
 * per workgroup / of 32 pixels per wavefront tile (0 = automatic). */
void sq_tune_blocked_force_depth(int depth);
void sq_tune_blocked_force_tile(int layer_blocks, int pixel_blocks);

/* bfloat16 conv1-type convolution with fp32 results (sq_conv2d_forward_ws with scratch): the tiles that span the
 * image width, which write a map larger than the memory-side cache in whole cache lines; 1 = always, 0 = never,
 * -1 = for maps of 200 MiB and more (default).  Per host thread. */
void sq_tune_conv7_f32out_rows(int mode);

/* Host-side self check of the division-by-multiplication the kernels use: number of x in
 * [0, x_max] for which it disagrees with x / d. */
long long sq_tune_fastdiv_mismatches(unsigned d, unsigned x_max);

#ifdef __cplusplus
}
#endif
#endif /* SQ_TUNING_H */
