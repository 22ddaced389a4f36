// Implicit-GEMM convolution on the fp32 matrix cores (MFMA) of gfx950.
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

namespace sq {
namespace {

using namespace mfma;

template <int KS, int S, int BM, int BN, int WM, int WN, int MT, int CC, int PE, int NBUF, int MINW>
__global__ __launch_bounds__(WM * WN * 64, MINW) void conv_mfma_f32_kernel(const KParams p)
{
    using M = Mfma<MT>;
    using Acc = typename M::Acc;
    constexpr int KK = KS * KS, KQ = M::KQ, NT = WM * WN * 64;
    constexpr int TM = BM / WM / MT, TN = BN / WN / MT;
    constexpr int RUN = CC * KK;
    constexpr int LDK = RUN + ((RUN & 1) ? 0 : 1);
    constexpr int WREG = (BM * RUN + NT - 1) / NT;
    constexpr bool POINTWISE = (KS == 1 && S == 1);
    constexpr int XREG = POINTWISE ? (CC * BN / NT) : CC * PE;
    static_assert(BM % (WM * MT) == 0 && BN % (WN * MT) == 0, "tile split");
    static_assert(CC % KQ == 0, "chunk must hold whole MFMA k-groups");
    static_assert(!POINTWISE || (NT % BN == 0 && (CC * BN) % NT == 0), "pointwise staging split");

    extern __shared__ float smem[];
    float *const Ws = smem;                       // [NBUF][BM*LDK]
    float *const Xs = smem + NBUF * BM * LDK;     // [NBUF][CC*plane]
    const int plane = p.plane;

    const int tile = xcd_remap(blockIdx.x, p.mtiles * p.ntiles);
    const int mt = tile % p.mtiles, pt = tile / p.mtiles;
    const int P0 = pt * BN, m0 = mt * BM;
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int wm = wv / WN, wn = wv % WN;
    const int li = lane % MT, kk = lane / MT;

    // ---- geometry of the staged patch ------------------------------------------------
    int va = 0, PRt = 0;
    if constexpr (!POINTWISE) {
        const int Ra = P0 / p.Wo;
        const int last = min(P0 + BN, p.PT) - 1;
        const int Rb = last / p.Wo;
        const int na = Ra / p.Ho, nb = Rb / p.Ho;
        va = na * p.VH + (Ra - na * p.Ho) * S;
        PRt = nb * p.VH + (Rb - nb * p.Ho) * S + KS - va;
    }

    // per-lane LDS offsets of the two MFMA operands (loop invariant)
    int aoff[TM], boff[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) aoff[i] = (wm * (BM / WM) + i * MT + li) * LDK + kk * KK;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int pl = wn * (BN / WN) + j * MT + li;
        if constexpr (POINTWISE) {
            boff[j] = pl + kk * plane;
        } else {
            const int pp = min(P0 + pl, p.PT - 1);
            const int R = pp / p.Wo, ow = pp - R * p.Wo;
            const int n = R / p.Ho;
            const int v = n * p.VH + (R - n * p.Ho) * S;
            boff[j] = (v - va) * p.LWs + ow * S + kk * plane;
        }
    }

    // ---- staging maps (what this thread copies for every chunk) ----------------------
    // kernels: element e = t + NT*r of the [BM][RUN] slab
    // patch:   general  -> element e = t + NT*r of one [rows][LW] plane, all CC layers
    //          pointwise-> pixel t % BN, layers t / BN + (NT/BN)*r
    int xsrc[POINTWISE ? 1 : PE], xdst[POINTWISE ? 1 : PE];
    if constexpr (POINTWISE) {
        const int pl = t % BN, pp = P0 + pl;
        if (pp < p.PT) {
            const int n = pp / p.HW;
            xsrc[0] = n * p.Cin * p.HW + (pp - n * p.HW);
        } else {
            xsrc[0] = -1;
        }
        xdst[0] = pl;
    } else {
#pragma unroll
        for (int r = 0; r < PE; ++r) {
            const int e = t + NT * r;
            const int vr = e / p.LW, pc = e - vr * p.LW;
            const int v = va + vr;
            const int n = v / p.VH, ih = v - n * p.VH - p.P, iw = pc - p.P;
            const bool stage = vr < PRt;
            const bool inb = stage && n < p.N && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
            xsrc[r] = inb ? (n * p.Cin * p.H + ih) * p.W + iw : -1;
            xdst[r] = stage ? vr * p.LWs + pc : -1;
        }
    }

    // Register staging (NBUF == 2) keeps one chunk in flight while the previous one is
    // being multiplied; with a single buffer the copy goes straight through.
    float wreg[NBUF == 2 ? WREG : 1], xreg[NBUF == 2 ? XREG : 1];

    auto w_value = [&](int c0, int r) -> float {
        const int e = t + NT * r;
        const int m = e / RUN, q = e - m * RUN;
        const bool ok = (BM * RUN % NT == 0 || e < BM * RUN) && (m0 + m < p.Cout) && (c0 + q / KK < p.Cin);
        return ok ? p.w[(size_t)(m0 + m) * p.Cin * KK + c0 * KK + q] : 0.f;
    };
    auto w_store = [&](float *ws, int r, float v) {
        const int e = t + NT * r;
        const int m = e / RUN, q = e - m * RUN;
        if (BM * RUN % NT == 0 || e < BM * RUN) ws[m * LDK + q] = v;
    };
    // patch value r of this thread: pointwise -> layer t/BN + (NT/BN)*r of pixel xsrc[0];
    // general -> layer r / PE, plane element r % PE
    auto x_value = [&](int c0, int r) -> float {
        const int c = POINTWISE ? t / BN + (NT / BN) * r : r / (POINTWISE ? 1 : PE);
        const int src = xsrc[POINTWISE ? 0 : r % (POINTWISE ? 1 : PE)];
        const bool ok = src >= 0 && c0 + c < p.Cin;
        return ok ? p.in[(size_t)src + (size_t)(c0 + c) * p.HW] : 0.f;
    };
    auto x_store = [&](float *xs, int r, float v) {
        if constexpr (POINTWISE) {
            xs[(t / BN + (NT / BN) * r) * plane + xdst[0]] = v;
        } else {
            const int d = xdst[r % (POINTWISE ? 1 : PE)];
            if (d >= 0) xs[(r / (POINTWISE ? 1 : PE)) * plane + d] = v;
        }
    };

    auto load_chunk = [&](int ch) {
        const int c0 = ch * CC;
#pragma unroll
        for (int r = 0; r < WREG; ++r) wreg[r] = w_value(c0, r);
#pragma unroll
        for (int r = 0; r < XREG; ++r) xreg[r] = x_value(c0, r);
    };
    auto store_chunk = [&](int buf) {
        float *ws = Ws + buf * (BM * LDK);
        float *xs = Xs + buf * (CC * plane);
#pragma unroll
        for (int r = 0; r < WREG; ++r) w_store(ws, r, wreg[r]);
#pragma unroll
        for (int r = 0; r < XREG; ++r) x_store(xs, r, xreg[r]);
    };
    auto copy_chunk = [&](int ch) {  // single-buffer path
        const int c0 = ch * CC;
#pragma unroll 8
        for (int r = 0; r < WREG; ++r) w_store(Ws, r, w_value(c0, r));
#pragma unroll 8
        for (int r = 0; r < XREG; ++r) x_store(Xs, r, x_value(c0, r));
    };

    Acc acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < M::NR; ++r) acc[i][j][r] = 0.f;

    auto compute_chunk = [&](int buf) {
        const float *ws = Ws + buf * (BM * LDK);
        const float *xs = Xs + buf * (CC * plane);
#pragma unroll
        for (int cq = 0; cq < CC / KQ; ++cq) {
#pragma unroll
            for (int i = 0; i < KS; ++i) {
                const int rowoff = cq * KQ * plane + (POINTWISE ? 0 : i * p.LWs);
#pragma unroll
                for (int j = 0; j < KS; ++j) {
                    float a[TM], b[TN];
#pragma unroll
                    for (int x = 0; x < TM; ++x) a[x] = ws[aoff[x] + cq * KQ * KK + i * KS + j];
#pragma unroll
                    for (int y = 0; y < TN; ++y) b[y] = xs[boff[y] + rowoff + j];
#pragma unroll
                    for (int x = 0; x < TM; ++x)
#pragma unroll
                        for (int y = 0; y < TN; ++y) acc[x][y] = M::run(a[x], b[y], acc[x][y]);
                }
            }
        }
    };

    // ---- main loop -------------------------------------------------------------------
    if constexpr (NBUF == 2) {
        load_chunk(0);
        store_chunk(0);
        __syncthreads();
        for (int ch = 0; ch < p.nchunks; ++ch) {
            const bool more = ch + 1 < p.nchunks;
            if (more) load_chunk(ch + 1);
            compute_chunk(ch & 1);
            if (more) store_chunk((ch + 1) & 1);
            __syncthreads();
        }
    } else {
        for (int ch = 0; ch < p.nchunks; ++ch) {
            copy_chunk(ch);
            __syncthreads();
            compute_chunk(0);
            __syncthreads();
        }
    }

    // ---- epilogue: bias, ReLU, store into layers [coff, coff+Cout) ---------------------
#pragma unroll
    for (int y = 0; y < TN; ++y) {
        const int pp = P0 + wn * (BN / WN) + y * MT + li;
        if (pp >= p.PT) continue;
        const int n = pp / p.HoWo, q = pp - n * p.HoWo;
        float *obase = p.out + ((size_t)n * p.ldc + p.coff) * p.HoWo + q;
#pragma unroll
        for (int x = 0; x < TM; ++x) {
#pragma unroll
            for (int r = 0; r < M::NR; ++r) {
                const int m = m0 + wm * (BM / WM) + x * MT + M::row(r, lane);
                if (m < p.Cout) {
                    float v = acc[x][y][r] + (p.b ? p.b[m] : 0.f);
                    if (p.relu) v = fmaxf(v, 0.f);
                    obase[(size_t)m * p.HoWo] = v;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
struct Variant {
    const char *name;
    int KS, S, BM, BN, MT, CC, PE, NBUF, NT;
    KernelFn kernel;
    bool conv1_type;  // the persistent 7x7/stride-2/three-layer kernel
};

#define SQ_VARIANT(KS, S, BM, BN, WM, WN, MT, CC, PE, NBUF, MINW)                                     \
    {"k" #KS "s" #S "_" #BM "x" #BN "_w" #WM "x" #WN "_m" #MT "_c" #CC "_b" #NBUF "_o" #MINW, KS, S, BM, BN, MT, CC, PE, NBUF, \
     WM * WN * 64, conv_mfma_f32_kernel<KS, S, BM, BN, WM, WN, MT, CC, PE, NBUF, MINW>, false}

const Variant kVariants[] = {
    // 3x3 stride 1 (expand3x3)
    SQ_VARIANT(3, 1, 128, 128, 2, 2, 32, 4, 2, 2, 2),
    SQ_VARIANT(3, 1, 64, 128, 2, 2, 32, 4, 2, 2, 2),
    SQ_VARIANT(3, 1, 64, 64, 2, 2, 32, 4, 2, 2, 2),
    SQ_VARIANT(3, 1, 64, 128, 1, 4, 16, 4, 2, 2, 2),
    SQ_VARIANT(3, 1, 32, 64, 2, 2, 16, 4, 8, 2, 2),
    // 1x1 (squeeze, expand1x1, conv10)
    SQ_VARIANT(1, 1, 128, 128, 2, 2, 32, 16, 0, 2, 2),
    SQ_VARIANT(1, 1, 64, 128, 2, 2, 32, 16, 0, 2, 2),
    SQ_VARIANT(1, 1, 64, 64, 2, 2, 32, 16, 0, 2, 2),
    SQ_VARIANT(1, 1, 16, 256, 1, 4, 16, 16, 0, 2, 2),
    SQ_VARIANT(1, 1, 32, 128, 1, 4, 16, 16, 0, 2, 2),
    SQ_VARIANT(1, 1, 48, 128, 1, 4, 16, 16, 0, 2, 2),
    // 7x7 stride 2 with three input layers (conv1): persistent kernel, 148-long contraction
    {"k7s2c3_persist_96x256", 7, 2, 96, 256, 32, 3, 8, 2, 512, conv7s2c3_kernel_for(256), true},
    {"k7s2c3_persist_96x128", 7, 2, 96, 128, 32, 3, 15, 2, 256, conv7s2c3_kernel_for(128), true},
    // 7x7 stride 2, generic: all input layers in one chunk, padded to four
    SQ_VARIANT(7, 2, 96, 128, 1, 4, 32, 4, 15, 1, 1),
    SQ_VARIANT(7, 2, 96, 64, 1, 4, 16, 4, 13, 1, 1),
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

struct Plan {
    KParams kp;
    size_t lds_bytes;
    unsigned blocks;
};

int num_cus()
{
    static int cus = 0;
    if (!cus) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
        (void)hipGetLastError();
    }
    return cus;
}

// Fills the launch parameters of variant v for this call; false if v cannot run it.
bool plan(const Variant &v, const ConvArgs &a, Plan &pl)
{
    if (a.dtype != SQ_F32 || a.K != v.KS || a.S != v.S) return false;
    if (a.W + 2 * a.P < a.K) return false;
    const long long in_elems = (long long)a.N * a.Cin * a.H * a.W;
    const long long out_elems = (long long)a.N * a.out_channels * a.Ho * a.Wo;
    const long long pixels = (long long)a.N * a.Ho * a.Wo;
    if (in_elems >= (1ll << 31) || out_elems >= (1ll << 31) || pixels + v.BN >= (1ll << 31)) return false;
    if (v.NBUF == 1 && a.Cin > v.CC) return false;
    if (v.conv1_type && (a.Cin != 3 || a.Cout > 96)) return false;

    KParams &k = pl.kp;
    k.in = (const float *)a.in; k.w = (const float *)a.w; k.b = a.b; k.out = a.out;
    k.N = a.N; k.Cin = a.Cin; k.H = a.H; k.W = a.W; k.Cout = a.Cout; k.P = a.P; k.relu = a.relu;
    k.Ho = a.Ho; k.Wo = a.Wo; k.HoWo = a.Ho * a.Wo; k.HW = a.H * a.W;
    k.ldc = a.out_channels; k.coff = a.c_offset;
    k.PT = (int)pixels;
    k.mtiles = (a.Cout + v.BM - 1) / v.BM;
    k.ntiles = (int)((pixels + v.BN - 1) / v.BN);
    k.nchunks = (a.Cin + v.CC - 1) / v.CC;
    const int KK = v.KS * v.KS, RUN = v.CC * KK, LDK = RUN + ((RUN & 1) ? 0 : 1);

    if (v.KS == 1 && v.S == 1) {
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
    long long blocks = (long long)k.mtiles * k.ntiles;
    if (v.conv1_type) {
        // kernels [96][149] + bias [96] + two patch buffers of three planes; if the bank
        // padding of the plane does not fit, fall back to the unpadded plane
        const size_t fixed = (size_t)96 * 149 + 96;
        if ((fixed + (size_t)6 * k.plane) * sizeof(float) > (size_t)kLdsBytes) k.plane = k.PRcap * k.LWs;
        pl.lds_bytes = (fixed + (size_t)6 * k.plane) * sizeof(float);
        if (blocks > num_cus()) blocks = num_cus();  // persistent: one workgroup per CU
    } else {
        pl.lds_bytes = ((size_t)v.NBUF * v.BM * LDK + (size_t)v.NBUF * v.CC * k.plane) * sizeof(float);
    }
    if (pl.lds_bytes > (size_t)kLdsBytes) return false;
    if (blocks >= (1ll << 31)) return false;
    pl.blocks = (unsigned)blocks;
    return true;
}

bool g_attr_done[kNumVariants] = {};

int launch(int vi, const Plan &pl, const ConvArgs &a)
{
    const Variant &v = kVariants[vi];
    if (!g_attr_done[vi]) {
        // dynamic LDS above the default limit must be opted into once per kernel
        if (hipFuncSetAttribute((const void *)v.kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess) {
            const int rc = check_launch();
            return rc ? rc : SQ_ERR_HIP;
        }
        g_attr_done[vi] = true;
    }
    LaunchScope scope(v.name, conv_flops(a), conv_bytes(a));
    hipLaunchKernelGGL(v.kernel, dim3(pl.blocks), dim3(v.NT), pl.lds_bytes, current_stream(), pl.kp);
    return check_launch();
}

// Estimated cost of a variant for a shape: MFMA work including tile and contraction
// padding, times the number of rounds the tiles need on the CUs.  Lower is better.
double estimate(const Variant &v, const Plan &pl, const ConvArgs &a)
{
    (void)a;
    const double tiles = (double)pl.kp.mtiles * pl.kp.ntiles;
    const double kpad = v.conv1_type ? 148.0 : (double)pl.kp.nchunks * v.CC * v.KS * v.KS;
    const double work_per_tile = (double)v.BM * v.BN * kpad;
    const double occ = v.conv1_type ? 1.0 : ((size_t)2 * pl.lds_bytes <= (size_t)kLdsBytes ? 2.0 : 1.0);
    const double rounds = ceil(tiles / (num_cus() * occ));
    // small tiles pay more LDS traffic and staging per flop
    const double tile_eff = v.conv1_type ? 1.0 : 1.0 / (1.0 + 24.0 / v.BM + 24.0 / v.BN);
    return rounds * occ * work_per_tile / tile_eff;
}

}  // namespace

int conv_mfma_variant_count() { return kNumVariants; }
const char *conv_mfma_variant_name(int i) { return kVariants[i].name; }

int conv_mfma(const ConvArgs &a, int variant)
{
    Plan pl;
    if (variant >= 0) {
        if (variant >= kNumVariants || !plan(kVariants[variant], a, pl)) return SQ_ERR_UNSUPPORTED;
        return launch(variant, pl, a);
    }
    int best = -1;
    double best_cost = 0;
    Plan best_plan;
    for (int i = 0; i < kNumVariants; ++i) {
        if (!plan(kVariants[i], a, pl)) continue;
        const double c = estimate(kVariants[i], pl, a);
        if (best < 0 || c < best_cost) {
            best = i; best_cost = c; best_plan = pl;
        }
    }
    if (best < 0) return SQ_ERR_UNSUPPORTED;
    return launch(best, best_plan, a);
}

}  // namespace sq
