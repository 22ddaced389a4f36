// Host side of the implicit-GEMM convolution family on the fp32 matrix cores (MFMA) of
// gfx950: planning, tiling choice and launch.  The kernel itself is in conv_mfma_kernel.h.
//
// The convolution layer of section "Convolutional Neural Networks" is the
// contraction  out[m][p] = sum_k w[m][k] * patch[k][p]  with m an output layer,
// p an output pixel (all images of the batch flattened: p = (n*Ho + oh)*Wo + ow)
// and k = (c, i, j) an input layer and kernel tap.  The paper assigns g output
// elements to a thread (section "Optimizing Thread Granularity"); here a
// workgroup owns a BM x BN tile of (layers x pixels), each of its wavefronts a
// (BM/WM) x (BN/WN) sub-tile held in MFMA accumulators, and the tile shape is the
// tunable granularity.
//
// Data movement per K-chunk of CC input layers:
//   * kernels  [BM][CC*K*K] are copied as they lie in memory (k contiguous) into
//     LDS rows of odd stride, so both the copy and the per-lane MFMA reads are
//     free of bank conflicts;
//   * the input patch that the BN pixels need -- CC planes of (rows x columns)
//     with halo, zero where padding or another image would be -- is staged once
//     and every tap (i, j) reads it at a shifted LDS address.  Rows are addressed
//     in a "virtual row" space in which the images of the batch are stacked with
//     K-S dead rows between them, so a pixel tile may straddle two images.
//   * chunks are double-buffered in LDS: the global loads of chunk t+1 are issued
//     before the MFMAs of chunk t and written to the other buffer afterwards.
// MFMA operand mapping (v_mfma_f32_32x32x2_f32 / v_mfma_f32_16x16x4_f32): the A
// operand carries output layers, the B operand pixels, so that an accumulator
// register holds consecutive pixels across lanes and the NCHW store is coalesced.
// The KQ (2 or 4) k-values one MFMA consumes are the same tap of KQ consecutive
// input layers, which makes the per-lane LDS offsets loop-invariant.
#include "conv_mfma_common.h"
#include "conv_mfma_variants.h"

#include <math.h>
#include <stdio.h>
#include <algorithm>
#include <string.h>

namespace sq {
size_t wino_transformed_bytes(int Cout, int Cin);
size_t wino_auto_offset(int Cout, int Cin);
size_t wino_auto_bytes(int Cout, int Cin);
namespace {

using namespace mfma;

// ---------------------------------------------------------------------------------------
struct Variant {
    const char *name;
    int KS, S, BM, BN, MT, CC, PE, NBUF, NT, WN;
    bool conv1_type;      // the persistent 7x7/stride-2/three-layer kernel
    bool wino;            // a minimal-filtering F(2x2, 3x3) kernel (BN = tiles of 2x2 pixels)
    bool wino_auto;       // ... the one with autonomous wavefronts (BM x BN per wavefront item)
};

#define SQ_V(KS, S, BM, BN, WM, WN, MT, CC, PE, MINW)                                               \
    {"k" #KS "s" #S "_" #BM "x" #BN "_w" #WM "x" #WN "_m" #MT "_c" #CC "_o" #MINW, KS, S, BM, BN, MT, CC, PE, 2, \
     WM * WN * 64, WN, false, false, false},
#define SQ_C(NW) {"k7s2c3_waves" #NW, 7, 2, 96, 32 * NW, 32, 3, 64, 2, 64 * NW, 1, true, false, false},
#define SQ_C1(NW) {"k7s2c3_waves" #NW "_m32", 7, 2, 32, 32 * NW, 32, 3, 64, 2, 64 * NW, 1, true, false, false},
#define SQ_W(BM, BT, CC) {"k3s1_f2x2_" #BM "x" #BT "_c" #CC, 3, 1, BM, BT, 32, CC, 0, 2, 256, 1, false, true, false},
#define SQ_WA(BM, BT) {"k3s1_f2x2a_" #BM "x" #BT, 3, 1, BM, BT, 16, 8, 0, 1, kWinoAutoWaves * 64, 1, false, true, true},
static_assert(kWinoAutoLayers == 32 && kWinoAutoTiles == 16, "the WA() entry of the variant list names these");
static_assert(kWinoBM == 64 && kWinoBT == 32 && kWinoCC == 8, "the W() entry of the variant list names these");
const Variant kVariants[] = {SQ_VARIANT_LIST(SQ_V, SQ_V, SQ_C, SQ_W, SQ_C1, SQ_WA)};
#undef SQ_V
#undef SQ_C
#undef SQ_C1
#undef SQ_W
#undef SQ_WA
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

struct Plan {
    KParams kp;
    size_t lds_bytes;
    unsigned blocks, blocks_y;
};

// kernels of tiling v for the given input type
const KernelSet &kernel_set(const Variant &v, int dtype)
{
    const int i = (int)(&v - kVariants);
    return dtype == SQ_BF16 ? conv_mfma_kernels_bf16[i] : conv_mfma_kernels_f32[i];
}

struct FusedE1 {
    const void *w1;
    const float *b1;
    int Cout1, coff1;
};

// Fills the launch parameters of variant v for this call; false if v cannot run it.
bool plan(const Variant &v, const ConvArgs &a, Plan &pl, const FusedE1 *e1 = nullptr)
{
    const KernelSet &ks = kernel_set(v, a.dtype);
    if (e1 && (!ks.fused_e1 || a.Cin % v.CC != 0)) return false;
    if (a.pool_H && (!(a.cp_in ? ks.rowpool : ks.pooled) || e1 || a.Cin % v.CC != 0)) return false;
    if (a.cp_in && (a.dtype != SQ_F32 || a.W != (a.pool_W - 3) / 2 + 1 || a.cp.row_stride < colpool_row_stride(a.pool_W, a.cp.shift))) return false;
    // a column-pooled map is written by the conv1-type kernels and by the expand pair of autonomous wavefronts
    const int Wp = a.cp_out ? (a.Wo - 3) / 2 + 1 : 0;
    if (a.cp_out && (!(v.conv1_type || v.wino_auto) || a.dtype != SQ_F32 || !a.relu || a.Wo < 3 || a.cp.row_stride < colpool_row_stride(a.Wo, a.cp.shift))) return false;
    if (a.K != v.KS || a.S != v.S) return false;
    if (!v.conv1_type && !ks.plain) return false;
    if (a.W + 2 * a.P < a.K) return false;
    const long long in_elems = (long long)a.N * a.Cin * (a.cp_in ? (long long)a.pool_H * a.cp.row_stride : a.pool_H ? (long long)a.pool_H * a.pool_W : (long long)a.H * a.W);
    const long long out_elems = (long long)a.N * a.out_channels * a.Ho * (a.cp_out ? a.cp.row_stride : a.Wo);
    const long long pixels = (long long)a.N * a.Ho * a.Wo;
    // per-lane addresses are 32-bit byte offsets from a uniform base
    const long long w_elems = (long long)a.Cout * a.Cin * a.K * a.K;
    if (in_elems >= kMaxBufferElems || out_elems >= kMaxBufferElems || w_elems >= kMaxBufferElems ||
        pixels + v.BN >= kMaxBufferElems)
        return false;
    if (v.conv1_type && (a.Cin != 3 || a.Cout > 96 || a.Cout % 8 != 0)) return false;
    if (v.wino && (a.P != 1 || a.Cin % v.CC != 0 || a.Cout % 32 != 0 || !a.ws || ((uintptr_t)a.ws & 15) ||
                   a.ws_bytes < conv_workspace_bytes(a.Cin, a.Cout, 3, 1, 1)))
        return false;

    pl.blocks_y = 1;
    KParams &k = pl.kp;
    k.in = (const float *)a.in; k.w = (const float *)a.w; k.b = a.b; k.out = a.out;
    k.N = a.N; k.Cin = a.Cin; k.H = a.H; k.W = a.W; k.Cout = a.Cout; k.P = a.P; k.relu = a.relu;
    k.Ho = a.Ho; k.Wo = a.Wo; k.HoWo = a.Ho * a.Wo; k.HW = a.H * a.W;
    k.ldc = a.out_channels; k.coff = a.c_offset;
    k.Win = a.cp_in ? a.cp.row_stride : a.pool_W; k.HWin = a.pool_H * k.Win;
    k.cpShift = a.cp.shift; k.cpSlotsRow = a.cp.slots_row; k.cpSlotsImage = a.cp.slots_image; k.cpWp = Wp; k.cpRS = a.cp.row_stride;
    k.PT = (int)pixels;
    k.mtiles = ((e1 && e1->Cout1 > a.Cout ? e1->Cout1 : a.Cout) + v.BM - 1) / v.BM;
    k.w1 = e1 ? (const float *)e1->w1 : nullptr; k.b1 = e1 ? e1->b1 : nullptr;
    k.Cout1 = e1 ? e1->Cout1 : 0; k.coff1 = e1 ? e1->coff1 : 0;
    k.w1_bytes = e1 ? (uint32_t)((long long)e1->Cout1 * a.Cin * (a.dtype == SQ_BF16 ? 2 : 4)) : 0u;
    k.ntiles = (int)((pixels + v.BN - 1) / v.BN);
    k.nchunks = (a.Cin + v.CC - 1) / v.CC;
    const int KK = v.KS * v.KS, RUN = v.CC * KK, LDK = RUN + ((RUN & 1) ? 0 : 1);

    if (v.wino) {
        k.TX = (a.Wo + 1) / 2;
        k.TXY = k.TX * ((a.Ho + 1) / 2);
        const long long tiles = (long long)a.N * k.TXY;
        if (tiles + v.BN >= kMaxBufferElems) return false;
        k.T = (int)tiles;
        k.dTX = make_fastdiv(k.TX); k.dTXY = make_fastdiv(k.TXY);
        k.ntiles = (int)((tiles + v.BN - 1) / v.BN);
        k.VH = a.Ho; k.LW = a.Wo; k.LWs = a.Wo; k.PRcap = 0; k.plane = 0;
        if (wino_transformed_bytes(a.Cout, a.Cin) >= (size_t)kMaxBufferElems * 4) return false;   // read through a buffer
        k.wu = (const float *)a.ws;
        k.wu_bytes = (uint32_t)wino_transformed_bytes(a.Cout, a.Cin);
        if (v.wino_auto) {
            // steps of four input layers; items = layer blocks x tile groups
            k.nchunks = a.Cin / 4;
            k.mtiles = a.Cout / kWinoAutoLayers;
            k.wu = (const float *)((const char *)a.ws + wino_auto_offset(a.Cout, a.Cin));
            k.wu_bytes = (uint32_t)wino_auto_bytes(a.Cout, a.Cin);
            if ((long long)k.mtiles * k.ntiles >= (1ll << 30)) return false;
        }
    } else if (v.KS == 1 && v.S == 1) {
        if (a.P != 0) return false;  // a padded 1x1 is left to the direct kernel
        k.VH = a.Ho; k.LW = a.Wo; k.LWs = a.Wo; k.PRcap = 0;
        k.plane = v.BN + v.MT;
    } else {
        const int dead = v.KS > v.S ? v.KS - v.S : 0;
        k.VH = a.Ho * v.S + dead;
        k.LW = (a.Wo - 1) * v.S + v.KS;
        k.LWs = k.LW;
        // most output rows BN consecutive pixels can touch, and image boundaries among them
        const int nr = v.BN >= 2 ? (v.BN - 2) / a.Wo + 2 : 1;
        const int cross = nr >= 2 ? (nr - 2) / a.Ho + 1 : 0;
        k.PRcap = (nr - 1) * v.S + v.KS + cross * dead;
        if ((long long)k.PRcap * k.LW > (long long)v.PE * v.NT) return false;
        const int raw = k.PRcap * k.LWs;
        k.plane = raw + (((v.MT - raw) % 64) + 64) % 64;  // plane = MT (mod 64): the KQ lane groups hit different banks
    }
    k.dWo = make_fastdiv(k.Wo); k.dHo = make_fastdiv(k.Ho); k.dLW = make_fastdiv(k.LW);
    k.dVH = make_fastdiv(k.VH); k.dHW = make_fastdiv(k.HW); k.dHoWo = make_fastdiv(k.HoWo);
    k.dMtiles = make_fastdiv(k.mtiles);
    const long long esz = a.dtype == SQ_BF16 ? 2 : 4;
    k.in_bytes = (uint32_t)(in_elems * esz); k.out_bytes = (uint32_t)(out_elems * 4); k.w_bytes = (uint32_t)(w_elems * esz);
    long long blocks = (long long)k.mtiles * k.ntiles;
    if (v.conv1_type) {
        // autonomous wavefronts: tiles of 2 x 16 output pixels, NW = NT/64 wavefronts per
        // workgroup, one workgroup per CU at most
        const int NW = v.NT / 64;
        k.RG = (a.Ho + kConv7TileRows - 1) / kConv7TileRows;
        k.CB = (a.Wo + kConv7TileCols - 1) / kConv7TileCols;
        const long long tiles = (long long)a.N * k.RG * k.CB;
        if (tiles >= (1ll << 30)) return false;
        k.dRG = make_fastdiv(k.RG); k.dCB = make_fastdiv(k.CB);
        k.dMtiles = make_fastdiv(k.RG * k.CB);
        k.ntiles = (int)tiles;
        if (a.cp_out && (a.cp.shift != 3 || a.cp.slots_row != 8 * k.CB || a.cp.slots_image != 8 * k.CB * k.RG)) return false;
        pl.lds_bytes = conv7s2c3_lds_bytes(NW, v.BM / 32);
        blocks = (tiles + NW - 1) / NW;
        if (blocks > num_cus()) blocks = num_cus();
        if (v.BM == 32) pl.blocks_y = (unsigned)k.mtiles;   // one workgroup per block of 32 output layers
    } else if (v.wino_auto) {
        blocks = std::min<long long>((long long)k.mtiles * k.ntiles, num_cus());   // persistent: one workgroup per CU
        if (blocks >= k.mtiles) {
            k.wa_cnt = (int)(blocks / k.mtiles); k.wa_big = (int)(blocks % k.mtiles);
            k.wa_q0 = k.ntiles / k.wa_cnt; k.wa_r0 = k.ntiles % k.wa_cnt;
            k.wa_q1 = k.ntiles / (k.wa_cnt + 1); k.wa_r1 = k.ntiles % (k.wa_cnt + 1);
        }
        if (a.cp_out && (a.cp.shift != 4 || a.cp.slots_row != k.TX || a.cp.slots_image != k.TXY)) return false;
        pl.lds_bytes = (size_t)k.nchunks * kWinoAutoStep * sizeof(float) + 64;   // U of one layer block + the item counter
    } else if (v.wino) {
        blocks = std::min<long long>(blocks, 2ll * num_cus());   // persistent: two workgroups per CU
        pl.lds_bytes = (size_t)(2 * 16 * 2 * kWinoBT * 4) * sizeof(float);   // two V images
    } else {
        pl.lds_bytes = ((size_t)v.NBUF * v.BM * LDK + (size_t)v.NBUF * v.CC * k.plane +
                        (e1 ? (size_t)2 * v.BM * (v.CC + 1) : 0)) * sizeof(float);
    }
    if (pl.lds_bytes > (size_t)kLdsBytes) return false;
    if (blocks >= (1ll << 31)) return false;
    pl.blocks = (unsigned)blocks;
    return true;
}

// a launch that pools on the way in is reported under a name of its own ("pool3s2+<tiling>"); the table is
// filled during static initialisation, so concurrent launches only read it
// (likewise "poolrows+<tiling>" for a 1x1 kernel that pools the rows of a column-pooled map, "<tiling>+poolcols" for
// a kernel that writes such a map)
struct PooledNames {
    char name[kNumVariants][64], rows[kNumVariants][64], cols[kNumVariants][64];
    PooledNames()
    {
        for (int i = 0; i < kNumVariants; ++i) {
            snprintf(name[i], sizeof(name[i]), "pool3s2+%s", kVariants[i].name);
            snprintf(rows[i], sizeof(rows[i]), "poolrows+%s", kVariants[i].name);
            snprintf(cols[i], sizeof(cols[i]), "%s+poolcols", kVariants[i].name);
        }
    }
};
const PooledNames kPooledNames;

// Floating-point operations the MFMA instructions of a launch of tiling v execute (all padding included).
double mfma_flops_of(const Variant &v, const Plan &pl, const ConvArgs &a, bool e1)
{
    const KParams &k = pl.kp;
    if (v.conv1_type) {
        // tiles of 32 pixels, 74 steps of two k-values, all layer blocks of 32 the workgroups compute
        const double layer_rows = v.BM == 32 ? 32.0 * k.mtiles : 96.0;
        return 2.0 * k.ntiles * 32.0 * layer_rows * 148.0;
    }
    if (v.wino_auto) return 2.0 * k.mtiles * k.ntiles * (double)kWinoAutoLayers * kWinoAutoTiles * a.Cin * (e1 ? 20.0 : 16.0);
    if (v.wino) return 2.0 * k.mtiles * k.ntiles * (double)v.BM * v.BN * 16.0 * k.nchunks * v.CC;
    const double kk = v.KS * v.KS;
    return 2.0 * k.mtiles * k.ntiles * (double)v.BM * v.BN * k.nchunks * v.CC * (kk + (e1 ? 1.0 : 0.0));
}

int launch(int vi, const Plan &pl, const ConvArgs &a, const FusedE1 *e1 = nullptr)
{
    const Variant &v = kVariants[vi];
    const KernelSet &ks = kernel_set(v, a.dtype);
    KernelFn fn = e1 ? ks.fused_e1 : ks.plain;
    if (v.conv1_type) fn = conv7s2c3_kernel_for(v.NT / 64, a.Cout == 96, a.dtype == SQ_BF16, v.BM / 32, a.cp_out);
    if (!v.conv1_type && !v.wino && !e1 && a.Cin % v.CC != 0) fn = ks.tail;
    if (a.pool_H) fn = a.cp_in ? ks.rowpool : ks.pooled;
    if (!fn || (a.cp_out && !v.conv1_type)) return SQ_ERR_UNSUPPORTED;   // (on its own the minimal-filtering kernel writes plain maps)
    if (!allow_big_lds((const void *)fn)) {
        const int rc = check_launch();
        return rc ? rc : SQ_ERR_HIP;
    }
    double flops = conv_flops(a), bytes = conv_bytes(a);
    if (e1) {
        flops += 2.0 * a.N * e1->Cout1 * a.Ho * a.Wo * (double)a.Cin;
        bytes += 4.0 * ((double)e1->Cout1 * a.Cin + (double)a.N * e1->Cout1 * a.Ho * a.Wo + e1->Cout1);
    }
    if (v.wino && !a.ws_ready) {
        const KernelPrepJob job{a.w, a.ws, a.Cin, a.Cout};
        const int rc = conv_prepare_kernels(&job, 1, a.dtype);
        if (rc) return rc;
    }
    LaunchScope scope(a.cp_in ? kPooledNames.rows[vi] : a.pool_H ? kPooledNames.name[vi] : a.cp_out ? kPooledNames.cols[vi] : v.name, flops, bytes,
                      mfma_flops_of(v, pl, a, e1 != nullptr));
    hipLaunchKernelGGL(fn, dim3(pl.blocks, pl.blocks_y), dim3(v.NT), pl.lds_bytes, current_stream(), pl.kp);
    return check_launch();
}

// Measured winners (written by tune.py).  An entry applies to its exact layer shape and to
// the batch sizes nearest to the one it was measured at.  P = -1 marks a 1x1 layer that pools
// on the way in (H, W are then the pooled extents).
struct Tuned {
    int K, S, P, Cin, Cout, H, W, N;
    const char *variant;        // fastest of all
    const char *variant_plain;  // fastest of those that need no caller scratch
};
const Tuned kTuned[] = {
#include "tuned_table.inc"
    {0, 0, 0, 0, 0, 0, 0, 0, "", ""}};

int tuned_variant(const ConvArgs &a)
{
    const Tuned *best = nullptr;
    double best_dist = 0;
    for (const Tuned *e = kTuned; e->K; ++e) {
        if (e->K != a.K || e->S != a.S || e->P != (a.pool_H ? -1 : a.P) || e->Cin != a.Cin || e->Cout != a.Cout || e->H != a.H ||
            e->W != a.W)
            continue;
        const double d = fabs(log((double)a.N / e->N));
        if (!best || d < best_dist) {
            best = e; best_dist = d;
        }
    }
    if (!best) return -1;
    for (int pass = 0; pass < 2; ++pass) {
        const char *name = pass ? best->variant_plain : best->variant;
        for (int i = 0; i < kNumVariants; ++i) {
            if (strcmp(kVariants[i].name, name)) continue;
            if (!kVariants[i].wino || a.ws_bytes >= conv_workspace_bytes(a.Cin, a.Cout, a.K, a.S, a.P)) return i;
        }
    }
    return -1;
}

// Estimated cost of a variant for a shape: MFMA work including tile and contraction
// padding, times the number of rounds the tiles need on the CUs.  Lower is better.
double estimate(const Variant &v, const Plan &pl, const ConvArgs &a)
{
    const double tiles = (double)pl.kp.mtiles * pl.kp.ntiles;
    // the minimal-filtering kernel multiplies 16 times per 2x2 pixels and input layer, i.e.
    // 4 per pixel where the direct form needs 9; BN counts tiles of 4 pixels there
    const double kpad = v.conv1_type ? 148.0 : v.wino_auto ? a.Cin * 16.0 : (double)pl.kp.nchunks * v.CC * (v.wino ? 16 : v.KS * v.KS);
    const double work_per_tile = (double)v.BM * v.BN * kpad;
    const double occ = v.conv1_type ? 1.0 : ((size_t)2 * pl.lds_bytes <= (size_t)kLdsBytes ? 2.0 : 1.0);
    const double rounds = ceil(tiles / (num_cus() * occ));
    // small tiles pay more LDS traffic and staging per flop
    const double tile_eff = v.conv1_type ? 1.0 : 1.0 / (1.0 + 24.0 / v.BM + 24.0 / v.BN);
    return rounds * occ * work_per_tile / tile_eff;
}

}  // namespace

// Host-side self check of the division-by-multiplication used in the kernels: number of
// x in [0, x_max] for which it disagrees with x / d (exported for the tests, not part of
// the public interface).
extern "C" long long sq_tune_fastdiv_mismatches(unsigned d, unsigned x_max)
{
    const mfma::FastDiv f = mfma::make_fastdiv(d);
    long long bad = 0;
    for (unsigned long long x = 0; x <= x_max; ++x) bad += mfma::fastdiv_host((unsigned)x, f) != (unsigned)x / (d ? d : 1);
    return bad;
}

size_t conv_workspace_bytes(int Cin, int Cout, int K, int S, int P)
{
    if (K == 3 && S == 1 && P == 1 && Cin % kWinoCC == 0 && Cout % 32 == 0)
        return wino_auto_offset(Cout, Cin) + align_up(wino_auto_bytes(Cout, Cin), 256);   // both layouts of the transformed kernels
    return 0;
}

// Whether the two expands of a fire layer share a launch (expand_pair_kernel): -1 = from kExpandPairMinBatch images
// on (the default), 0 = never, 1 + i = like -1 with the i-th compiled expand1x1 tiling.  A tuning hook, not part of
// the public interface.  Measured on whole fp32 passes: with the pair on every fire layer 4 % / 10 % / 9 % / 11 % /
// 6 % / 3 % faster at batch 4 / 8 / 16 / 32 / 64 / 256 than the best of the other forms (both expands in the tiles
// of one direct 3x3 kernel up to batch 16, separate launches above), slower only at batches 1 and 2.
thread_local int g_expand_pair = -1;
extern "C" void sq_tune_expand_pair(int v) { g_expand_pair = v; }
constexpr int kExpandPairMinBatch = 3;

static bool expand_pair_wanted(const ConvArgs &a3)
{
    return g_expand_pair != 0 && a3.N >= kExpandPairMinBatch && a3.dtype == SQ_F32 && a3.K == 3 && a3.S == 1 && a3.P == 1;
}

// The minimal-filtering tiling if this layer is to run in it -- because it is the measured choice for the layer
// on its own, or (pair = true) as the first part of an expand pair, which takes it wherever it fits; -1 otherwise.
static int wino_choice(const ConvArgs &a, Plan &pl, bool pair)
{
    const int tv = tuned_variant(a);
    if (tv >= 0 && kVariants[tv].wino) return plan(kVariants[tv], a, pl) ? tv : -1;
    if (pair)
        for (int i = 0; i < kNumVariants; ++i)
            if (kVariants[i].wino && plan(kVariants[i], a, pl)) return i;
    return -1;
}

// fire_expand: this is the expand3x3 of a fire layer (it may run as part of an expand pair)
bool conv_wants_prepared_kernels(const ConvArgs &a, bool fire_expand)
{
    Plan pl;
    return wino_choice(a, pl, fire_expand && expand_pair_wanted(a)) >= 0;
}

// Every kernel of this family whose launch may ask for more dynamic LDS than the default limit.
bool conv_mfma_register_kernels()
{
    bool ok = true;
    for (int i = 0; i < kNumVariants; ++i)
        for (const KernelSet *ks : {&conv_mfma_kernels_f32[i], &conv_mfma_kernels_bf16[i]})
            for (KernelFn fn : {ks->plain, ks->tail, ks->fused_e1, ks->pooled, ks->avg, ks->rowpool}) ok &= allow_big_lds((const void *)fn);
    for (int nw : {4, 8})
        for (int full = 0; full < 2; ++full)
            for (int bf = 0; bf < 2; ++bf)
                for (int tm : {1, 3}) ok &= allow_big_lds((const void *)conv7s2c3_kernel_for(nw, full, bf, tm));
    for (int i = 0; i < num_expand_pair_kernels; ++i) {
        ok &= allow_big_lds((const void *)expand_pair_kernels[i].fn);
        ok &= allow_big_lds((const void *)expand_pair_kernels[i].fn_colpool);
    }
    for (int nw : {4, 8})
        for (int tm : {1, 3}) ok &= allow_big_lds((const void *)conv7s2c3_kernel_for(nw, true, false, tm, true));
    return ok;
}

int conv_mfma_variant_count() { return kNumVariants; }
const char *conv_mfma_variant_name(int i) { return kVariants[i].name; }

// Which tiling runs the fused expand: -3 = never fuse, -2 = the default policy (fuse at batches of at
// most 16 images, where a fire layer is bound by its launches: measured 14 % / 10 % / 5 % / 3 % / 4 %
// faster network passes at batch 1 / 2 / 4 / 8 / 16, slower from 32 on, where the fused kernel's lower
// occupancy costs more than the launch it saves), -1 = always, automatic choice of tiling,
// i >= 0 = tiling i.  The setter is a tuning hook, not part of the public interface.
thread_local int g_force_expand = -2;
extern "C" void sq_tune_force_expand(int v) { g_force_expand = v; }

// 3x3 (pad 1, stride 1) convolution a3 plus the 1x1 convolution (w1, b1, Cout1 layers) of the
// same input, results in layers [a3.c_offset, +a3.Cout) and [coff1, +Cout1) of one tensor.
int conv_expand_fused(const ConvArgs &a3, const void *w1, const float *b1, int Cout1, int coff1)
{
    if (a3.K != 3 || a3.S != 1 || a3.P != 1 || a3.dtype != SQ_F32) return SQ_ERR_UNSUPPORTED;
    const FusedE1 e1{w1, b1, Cout1, coff1};
    Plan pl;
    if (g_force_expand == -3 || (g_force_expand == -2 && a3.N > 16)) return SQ_ERR_UNSUPPORTED;
    if (g_force_expand >= 0) {
        if (g_force_expand >= kNumVariants || !plan(kVariants[g_force_expand], a3, pl, &e1)) return SQ_ERR_UNSUPPORTED;
        return launch(g_force_expand, pl, a3, &e1);
    }
    const int tv = tuned_variant(a3);
    if (tv >= 0 && plan(kVariants[tv], a3, pl, &e1)) return launch(tv, pl, a3, &e1);
    int best = -1;
    double best_cost = 0;
    Plan best_plan;
    for (int i = 0; i < kNumVariants; ++i) {
        if (!plan(kVariants[i], a3, pl, &e1)) continue;
        const double c = estimate(kVariants[i], pl, a3);
        if (best < 0 || c < best_cost) {
            best = i; best_cost = c; best_plan = pl;
        }
    }
    if (best < 0) return SQ_ERR_UNSUPPORTED;
    return launch(best, best_plan, a3, &e1);
}

// The tiling the automatic choice runs for this call (the measured winner where the table has the shape,
// else the lowest estimate), its plan in pl; -1 if no tiling can run it.
static int choose_variant(const ConvArgs &a, Plan &pl)
{
    const int tv = tuned_variant(a);
    if (tv >= 0 && plan(kVariants[tv], a, pl)) return tv;
    int best = -1;
    double best_cost = 0;
    Plan cand;
    for (int i = 0; i < kNumVariants; ++i) {
        if (!plan(kVariants[i], a, cand)) continue;
        const double c = estimate(kVariants[i], cand, a);
        if (best < 0 || c < best_cost) {
            best = i; best_cost = c; pl = cand;
        }
    }
    return best;
}

int conv_mfma_choice(const ConvArgs &a)
{
    Plan pl;
    return choose_variant(a, pl);
}

// Which compiled pair runs (a3, a1), with its launch parameters; < 0 if none does.
static int plan_expand_pair(const ConvArgs &a3, const ConvArgs &a1, Plan &p3, Plan &p1, int &v3)
{
    if (!expand_pair_wanted(a3) || a1.dtype != SQ_F32) return -1;
    if (a1.K != 1 || a1.S != 1 || a1.P != 0 || a1.pool_H || a1.in != a3.in || a1.out != a3.out || a1.N != a3.N) return -1;
    if (a1.cp_out != a3.cp_out || (a3.cp_out && a1.cp.row_stride != a3.cp.row_stride)) return -1;
    auto variant_named = [](const char *name) {
        for (int i = 0; i < kNumVariants; ++i)
            if (!strcmp(kVariants[i].name, name)) return i;
        return -1;
    };
    // Which compiled pair.  Pair 2 is the autonomous-wavefront form of the expand3x3 with the expand1x1 inside its
    // items; pairs 0 and 1 the four-wavefront form with expand1x1 tiles of 64x128 / 64x256 behind it (the stand-alone
    // winners 64x64 and 48x64 lose there, 128x128 too).  Measured per fire layer inside whole passes at batch 64
    // (pair 2 against pair 0, us): 16 -> 64 at 55x55 41-46 / 41, 32 -> 128 at 55x55 103 / 112, 32 -> 128 at 27x27
    // 36.9 / 36.1, 48 -> 192 at 27x27 58 / 60, 64 -> 256 at 27x27 92.2 / 92.5, 64 -> 256 at 13x13 32.5 / 32.4: pair 2
    // from 48 input layers on and for 32 input layers on the large maps; pair 1 instead of pair 0 from batch 128 on.
    // Only pair 2 can write a column-pooled map.
    const bool auto_form = a3.cp_out || (a3.H * a3.W >= 27 * 27 && (a3.Cin >= 48 || (a3.Cin >= 32 && a3.H * a3.W >= 55 * 55)));
    const int prefer = g_expand_pair > 0 ? g_expand_pair - 1 : (auto_form ? 2 : a1.N >= 128 ? 1 : 0);
    if (prefer >= num_expand_pair_kernels) return -1;
    int pair = -1;
    for (int k = 0; k < num_expand_pair_kernels && pair < 0; ++k) {
        if (g_expand_pair > 0 && k > 0) break;                    // a forced pair has no substitute
        const int i = (prefer + k) % num_expand_pair_kernels;     // the preferred one first, then the others
        if (a3.cp_out && !expand_pair_kernels[i].fn_colpool) continue;
        v3 = variant_named(expand_pair_kernels[i].e3_variant);
        if (v3 < 0 || !plan(kVariants[v3], a3, p3)) continue;
        if (!expand_pair_kernels[i].e1_variant) {
            // the expand1x1 runs inside the items of the autonomous-wavefront expand3x3: same layers, steps in fours
            if (a1.Cout != a3.Cout || a1.Cin % 16 != 0 || !kVariants[v3].wino_auto) continue;
            KParams &k = p3.kp;
            k.w1 = (const float *)a1.w; k.b1 = a1.b; k.Cout1 = a1.Cout; k.coff1 = a1.c_offset;
            p3.lds_bytes += (size_t)k.nchunks * 128 * sizeof(float);
            if (p3.lds_bytes > (size_t)kLdsBytes) continue;
            p1.blocks = 0; p1.blocks_y = 1; p1.lds_bytes = 0; p1.kp = p3.kp;
            pair = i;
            continue;
        }
        const int v = variant_named(expand_pair_kernels[i].e1_variant);
        if (v >= 0 && a1.Cin % kVariants[v].CC == 0 && plan(kVariants[v], a1, p1) && kVariants[v].NT == kVariants[v3].NT) pair = i;
    }
    if (pair < 0) return -1;
    const long long blocks = (long long)p3.blocks + p1.blocks;
    if (blocks >= (1ll << 31) || p1.blocks_y != 1) return -1;
    return pair;
}

bool conv_expand_pair_supported(const ConvArgs &a3, const ConvArgs &a1)
{
    Plan p3, p1;
    int v3 = -1;
    return plan_expand_pair(a3, a1, p3, p1, v3) >= 0;
}

int conv_expand_pair(const ConvArgs &a3, const ConvArgs &a1)
{
    Plan p3, p1;
    int v3 = -1;
    const int pair = plan_expand_pair(a3, a1, p3, p1, v3);
    if (pair < 0) return SQ_ERR_UNSUPPORTED;
    const long long blocks = (long long)p3.blocks + p1.blocks;
    const PairKernel &pk = expand_pair_kernels[pair];
    const PairFn fn = a3.cp_out ? pk.fn_colpool : pk.fn;
    if (!allow_big_lds((const void *)fn)) {
        const int rc = check_launch();
        return rc ? rc : SQ_ERR_HIP;
    }
    if (!a3.ws_ready) {
        const KernelPrepJob job{a3.w, a3.ws, a3.Cin, a3.Cout};
        const int rc = conv_prepare_kernels(&job, 1, a3.dtype);
        if (rc) return rc;
    }
    const bool folded = !pk.e1_variant;
    double mf = mfma_flops_of(kVariants[v3], p3, a3, folded);
    if (!folded)
        for (int i = 0; i < kNumVariants; ++i)
            if (!strcmp(kVariants[i].name, pk.e1_variant)) mf += mfma_flops_of(kVariants[i], p1, a1, false);
    LaunchScope scope(a3.cp_out ? pk.name_colpool : pk.name, conv_flops(a3) + conv_flops(a1), conv_bytes(a3) + conv_bytes(a1), mf);
    hipLaunchKernelGGL(fn, dim3((unsigned)blocks), dim3(kVariants[v3].NT), std::max(p3.lds_bytes, p1.lds_bytes), current_stream(),
                       p3.kp, p1.kp, (int)p3.blocks);
    return check_launch();
}

// 1x1 convolution (+bias, ReLU) whose result is wanted only as per-image plane sums: the averaging form of the
// tiling the automatic choice would run (variant < 0) or of tiling `variant`.  sums: the table the kernel writes,
// [lay->ntiles][lay->WN][lay->slots][Cout] floats.  SQ_ERR_UNSUPPORTED where that tiling has no such form.
static bool plan_avg(const ConvArgs &a, int variant, Plan &pl, int &vi, AvgLayout &lay)
{
    if (a.K != 1 || a.S != 1 || a.P != 0 || a.dtype != SQ_F32 || a.pool_H) return false;
    if (variant >= 0) {
        if (variant >= kNumVariants || !plan(kVariants[variant], a, pl)) return false;
        vi = variant;
    } else {
        vi = choose_variant(a, pl);
    }
    if (vi < 0) return false;
    const Variant &v = kVariants[vi];
    if (!kernel_set(v, a.dtype).avg || a.Cin % v.CC != 0) return false;
    lay.ntiles = pl.kp.ntiles; lay.WN = v.WN; lay.BN = v.BN;
    lay.slots = (a.Ho * a.Wo + v.BN - 2) / (a.Ho * a.Wo) + 1;
    return true;
}

size_t conv_mfma_avg_bytes(const ConvArgs &a, int variant)
{
    Plan pl; int vi; AvgLayout lay;
    if (!plan_avg(a, variant, pl, vi, lay)) return 0;
    return (size_t)lay.ntiles * lay.WN * lay.slots * a.Cout * sizeof(float);
}

int conv_mfma_avg(const ConvArgs &a, int variant, float *sums, size_t sums_bytes, AvgLayout *lay)
{
    Plan pl; int vi;
    if (!plan_avg(a, variant, pl, vi, *lay)) return SQ_ERR_UNSUPPORTED;
    if (sums_bytes < (size_t)lay->ntiles * lay->WN * lay->slots * a.Cout * sizeof(float)) return SQ_ERR_WORKSPACE;
    const Variant &v = kVariants[vi];
    KernelFn fn = kernel_set(v, a.dtype).avg;
    if (!allow_big_lds((const void *)fn)) {
        const int rc = check_launch();
        return rc ? rc : SQ_ERR_HIP;
    }
    pl.kp.out = sums;
    pl.kp.avg_slots = lay->slots;
    static const struct Names {
        char name[kNumVariants][64];
        Names() { for (int i = 0; i < kNumVariants; ++i) snprintf(name[i], sizeof(name[i]), "%s+planesums", kVariants[i].name); }
    } names;
    LaunchScope scope(names.name[vi], conv_flops(a), conv_bytes(a) - 4.0 * a.N * a.Cout * a.Ho * a.Wo + 4.0 * lay->ntiles * lay->WN * lay->slots * a.Cout,
                      mfma_flops_of(v, pl, a, false));
    hipLaunchKernelGGL(fn, dim3(pl.blocks, pl.blocks_y), dim3(v.NT), pl.lds_bytes, current_stream(), pl.kp);
    return check_launch();
}

int conv_mfma(const ConvArgs &a, int variant)
{
    Plan pl;
    if (variant >= 0) {
        if (variant >= kNumVariants || !plan(kVariants[variant], a, pl)) return SQ_ERR_UNSUPPORTED;
        return launch(variant, pl, a);
    }
    const int best = choose_variant(a, pl);
    if (best < 0) return SQ_ERR_UNSUPPORTED;
    return launch(best, pl, a);
}

}  // namespace sq
