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

#include <math.h>
#include <string.h>

namespace sq {
namespace {

using namespace mfma;

// TAIL: the number of input layers is not a multiple of CC, so the last chunk is partly
// padding (compiled separately to keep the common loop free of the test).
// E1: fused expand -- next to the KxK convolution the workgroup also computes a 1x1
// convolution of the same input (its kernels p.w1) for the same pixels and its own tile of
// layers, written to layers [coff1, coff1+Cout1): the 1x1 reuses the centre-tap patch
// operands, so the input is staged once for both (fire layer, section "Convolutional
// Neural Networks": the two expand layers read the same squeeze result).
template <int KS, int S, int BM, int BN, int WM, int WN, int MT, int CC, int PE, int MINW, bool TAIL, bool E1 = false>
__global__ __launch_bounds__(WM * WN * 64, MINW) void conv_mfma_f32_kernel(const KParams p)
{
    using M = Mfma<MT>;
    using Acc = typename M::Acc;
    constexpr int KK = KS * KS, KQ = M::KQ, NT = WM * WN * 64;
    constexpr int TM = BM / WM / MT, TN = BN / WN / MT;
    constexpr int RUN = CC * KK;
    constexpr int LDK = RUN + ((RUN & 1) ? 0 : 1);
    constexpr int WBUF = BM * LDK;
    constexpr int WREG = (BM * RUN + NT - 1) / NT;
    constexpr bool WEXACT = (BM * RUN) % NT == 0;
    constexpr bool POINTWISE = (KS == 1 && S == 1);
    constexpr int XMAP = POINTWISE ? 1 : PE;
    constexpr int XREG = POINTWISE ? (CC * BN / NT) : CC * PE;
    static_assert(BM % (WM * MT) == 0 && BN % (WN * MT) == 0, "tile split");
    static_assert(CC % KQ == 0, "chunk must hold whole MFMA k-groups");
    static_assert(!POINTWISE || (NT % BN == 0 && BN % 64 == 0 && (CC * BN) % NT == 0), "pointwise staging split");
    static_assert(!E1 || (KS % 2 == 1 && S == 1 && !TAIL), "fused expand needs a centre tap");
    constexpr int LD1 = CC + 1;                       // LDS row stride of the 1x1 kernels
    constexpr int W1BUF = E1 ? BM * LD1 : 0;
    constexpr int W1REG = E1 ? (BM * CC + NT - 1) / NT : 1;

    extern __shared__ float smem[];
    float *const Ws = smem;               // [2][BM*LDK]
    float *const W1s = smem + 2 * WBUF;   // [2][BM*LD1] (fused expand only)
    float *const Xs = W1s + 2 * W1BUF;    // [2][CC*plane]
    const int plane = p.plane;
    const int XBUF = CC * plane;

    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wv / WN, wn = wv % WN;
    const int li = lane % MT, kk = lane / MT;

    const int tile = xcd_remap(blockIdx.x, p.mtiles * p.ntiles);
    const int pt = fdiv(tile, p.dMtiles), mt = tile - pt * p.mtiles;
    const int P0 = pt * BN, m0 = mt * BM;
    const bool full_m = m0 + BM <= p.Cout && (!E1 || m0 + BM <= p.Cout1);

    // ---- geometry of the staged patch ------------------------------------------------
    int va = 0, PRt = 0;
    if constexpr (!POINTWISE) {
        const int Ra = fdiv(P0, p.dWo);
        const int Rb = fdiv(min(P0 + BN, p.PT) - 1, p.dWo);
        const int na = fdiv(Ra, p.dHo), nb = fdiv(Rb, p.dHo);
        va = na * p.VH + (Ra - na * p.Ho) * S;
        PRt = nb * p.VH + (Rb - nb * p.Ho) * S + KS - va;
    }

    // per-lane LDS offsets of the two MFMA operands (loop invariant)
    int aoff[TM], boff[TN], a1off[E1 ? TM : 1];
#pragma unroll
    for (int i = 0; i < TM; ++i) aoff[i] = (wm * (BM / WM) + i * MT + li) * LDK + kk * KK;
    if constexpr (E1) {
#pragma unroll
        for (int i = 0; i < TM; ++i) a1off[i] = (wm * (BM / WM) + i * MT + li) * LD1 + kk;
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int pl = wn * (BN / WN) + j * MT + li;
        if constexpr (POINTWISE) {
            boff[j] = pl + kk * plane;
        } else {
            const int pp = min(P0 + pl, p.PT - 1);
            const int R = fdiv(pp, p.dWo), ow = pp - R * p.Wo;
            const int n = fdiv(R, p.dHo);
            const int v = n * p.VH + (R - n * p.Ho) * S;
            boff[j] = (v - va) * p.LWs + ow * S + kk * plane;
        }
    }

    // ---- staging maps: what this thread copies for every chunk -------------------------
    // kernels: element e = t + NT*r of the [BM][RUN] slab (k contiguous, as in memory)
    // patch:   general   -> element e = t + NT*r of one [rows][LW] plane, all CC layers
    //          pointwise -> pixel t % BN, layers t / BN + (NT/BN)*r
    // *src are byte offsets (0 where nothing is to be read), *ok says whether the value
    // is real or zero, *dst the LDS float index (-1 = nothing to store).
    uint32_t wsrc[WREG];
    int wdst[WREG];
#pragma unroll
    for (int r = 0; r < WREG; ++r) {
        const int e = t + NT * r;
        const int m = e / RUN, q = e - m * RUN;
        const bool inrange = WEXACT || e < BM * RUN;
        wsrc[r] = (inrange && m0 + m < p.Cout) ? (uint32_t)(((m0 + m) * p.Cin * KK + q) * 4) : kOob;
        wdst[r] = inrange ? m * LDK + q : -1;
    }
    uint32_t w1src[W1REG];
    int w1dst[W1REG];
    if constexpr (E1) {
#pragma unroll
        for (int r = 0; r < W1REG; ++r) {
            const int e = t + NT * r;
            const int m = e / CC, c = e - m * CC;
            const bool inrange = e < BM * CC;
            w1src[r] = (inrange && m0 + m < p.Cout1) ? (uint32_t)(((m0 + m) * p.Cin + c) * 4) : kOob;
            w1dst[r] = inrange ? m * LD1 + c : -1;
        }
    }
    uint32_t xsrc[XMAP];
    int xdst[XMAP];
    if constexpr (POINTWISE) {
        const int pl = t % BN, pp = P0 + pl;
        const int n = fdiv(pp, p.dHW);
        xsrc[0] = pp < p.PT ? (uint32_t)((n * p.Cin * p.HW + (pp - n * p.HW)) * 4) : kOob;
        xdst[0] = pl;
    } else {
#pragma unroll
        for (int r = 0; r < PE; ++r) {
            const int e = t + NT * r;
            const int vr = fdiv(e, p.dLW), pc = e - vr * p.LW;
            const int v = va + vr;
            const int n = fdiv(v, p.dVH), ih = v - n * p.VH - p.P, iw = pc - p.P;
            const bool stage = vr < PRt;
            const bool inb = stage && n < p.N && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
            xsrc[r] = inb ? (uint32_t)(((n * p.Cin * p.H + ih) * p.W + iw) * 4) : kOob;
            xdst[r] = stage ? vr * p.LWs + pc : -1;
        }
    }
    const int cpart = POINTWISE ? __builtin_amdgcn_readfirstlane(t / BN) : 0;

    float wreg[WREG], xreg[XREG], w1reg[W1REG];

    // Global loads of one chunk through buffer addressing: the per-lane offsets were fixed
    // above (kOob where the value is padding, which the hardware turns into zero), the chunk
    // and input-layer offsets are uniform.  Only a last chunk that runs past the input
    // layers (Cin not a multiple of CC) needs extra tests.
    const rsrc_t rw = make_rsrc(p.w, p.w_bytes), rin = make_rsrc(p.in, p.in_bytes);
    const rsrc_t rw1 = make_rsrc(E1 ? p.w1 : p.w, E1 ? p.w1_bytes : 0u);
    auto load_chunk = [&](int ch_) {
        // readfirstlane keeps the chunk offsets in scalar registers (otherwise every buffer
        // load is wrapped in a loop over the distinct values of its "uniform" offset)
        const int c0 = __builtin_amdgcn_readfirstlane(ch_ * CC);
        const uint32_t wchunk = (uint32_t)(c0 * KK * 4);
        if (TAIL && c0 + CC > p.Cin) {
            // last chunk runs past the input layers: those kernel values and patch planes are zero
#pragma unroll
            for (int r = 0; r < WREG; ++r) {
                const int q = (t + NT * r) % RUN;
                wreg[r] = buf_ld(rw, c0 + q / KK < p.Cin ? wsrc[r] : kOob, wchunk);
            }
#pragma unroll
            for (int r = 0; r < XREG; ++r) {
                const int c = POINTWISE ? cpart + (NT / BN) * r : r / XMAP;   // uniform
                const int i = POINTWISE ? 0 : r % XMAP;
                if (c0 + c < p.Cin)
                    xreg[r] = buf_ld(rin, xsrc[i], (uint32_t)__builtin_amdgcn_readfirstlane((c0 + c) * p.HW * 4));
                else
                    xreg[r] = 0.f;
            }
            return;
        }
#pragma unroll
        for (int r = 0; r < WREG; ++r) wreg[r] = buf_ld(rw, wsrc[r], wchunk);
        if constexpr (E1) {
#pragma unroll
            for (int r = 0; r < W1REG; ++r) w1reg[r] = buf_ld(rw1, w1src[r], (uint32_t)(c0 * 4));
        }
#pragma unroll
        for (int r = 0; r < XREG; ++r) {
            const int c = POINTWISE ? cpart + (NT / BN) * r : r / XMAP;       // uniform
            const int i = POINTWISE ? 0 : r % XMAP;
            xreg[r] = buf_ld(rin, xsrc[i], (uint32_t)__builtin_amdgcn_readfirstlane((c0 + c) * p.HW * 4));
        }
    };

    auto store_chunk = [&](int buf) {
        float *ws = Ws + buf * WBUF;
        float *xs = Xs + buf * XBUF;
#pragma unroll
        for (int r = 0; r < WREG; ++r)
            if (WEXACT || r + 1 < WREG || wdst[r] >= 0) ws[wdst[r]] = wreg[r];
        if constexpr (E1) {
            float *w1s = W1s + buf * W1BUF;
#pragma unroll
            for (int r = 0; r < W1REG; ++r)
                if (w1dst[r] >= 0) w1s[w1dst[r]] = w1reg[r];
        }
        if constexpr (POINTWISE) {
#pragma unroll
            for (int r = 0; r < XREG; ++r) xs[(cpart + (NT / BN) * r) * plane + xdst[0]] = xreg[r];
        } else {
#pragma unroll
            for (int i = 0; i < XMAP; ++i)
                if (xdst[i] >= 0) {
#pragma unroll
                    for (int c = 0; c < CC; ++c) xs[c * plane + xdst[i]] = xreg[c * XMAP + i];
                }
        }
    };

    Acc acc[TM][TN], acc1[E1 ? TM : 1][E1 ? TN : 1];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < M::NR; ++r) {
                acc[i][j][r] = 0.f;
                if constexpr (E1) acc1[i][j][r] = 0.f;
            }

    // One MFMA step consumes, for every lane, one kernel value per layer block and one patch
    // value per pixel block.  LDS latency (~120 cycles) is longer than a short group of
    // MFMAs, so the operands are fetched PD steps ahead into a small register ring, and
    // scheduling barriers keep the compiler from sinking the reads back next to their use.
    auto compute_chunk = [&](int buf) {
        const float *ws = Ws + buf * WBUF;
        const float *xs = Xs + buf * XBUF;
        constexpr int STEPS = (CC / KQ) * KK;
        constexpr int STEP_CYCLES = TM * TN * (MT == 32 ? 64 : 32);
        constexpr int PD0 = (240 + STEP_CYCLES - 1) / STEP_CYCLES;      // steps to cover the latency
        constexpr int PD = PD0 < 1 ? 1 : (PD0 > 3 ? 3 : PD0);
        constexpr int RING = PD + 1;
        constexpr int CENTRE = (KS / 2) * KS + KS / 2;
        const float *w1s = W1s + buf * W1BUF;
        float a[RING][TM], b[RING][TN], a1[RING][E1 ? TM : 1];
        auto fetch = [&](int s, float *av, float *bv, float *a1v) {
            const int cq = s / KK, tap = s - cq * KK, i = tap / KS, j = tap - i * KS;
            const int rowoff = cq * KQ * plane + (POINTWISE ? 0 : i * p.LWs) + j;
#pragma unroll
            for (int x = 0; x < TM; ++x) av[x] = ws[aoff[x] + cq * KQ * KK + tap];
#pragma unroll
            for (int y = 0; y < TN; ++y) bv[y] = xs[boff[y] + rowoff];
            if constexpr (E1) {
                if (tap == CENTRE) {
#pragma unroll
                    for (int x = 0; x < TM; ++x) a1v[x] = w1s[a1off[x] + cq * KQ];
                }
            }
        };
#pragma unroll
        for (int s = 0; s < PD && s < STEPS; ++s) fetch(s, a[s % RING], b[s % RING], a1[s % RING]);
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            if (s + PD < STEPS) fetch(s + PD, a[(s + PD) % RING], b[(s + PD) % RING], a1[(s + PD) % RING]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int x = 0; x < TM; ++x)
#pragma unroll
                for (int y = 0; y < TN; ++y) acc[x][y] = M::run(a[s % RING][x], b[s % RING][y], acc[x][y]);
            if constexpr (E1) {
                if (s % KK == CENTRE) {
#pragma unroll
                    for (int x = 0; x < TM; ++x)
#pragma unroll
                        for (int y = 0; y < TN; ++y) acc1[x][y] = M::run(a1[s % RING][x], b[s % RING][y], acc1[x][y]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop, two chunks per trip so the LDS buffer index is a constant -------------
    load_chunk(0);
    store_chunk(0);
    __syncthreads();
    for (int ch = 0; ch < p.nchunks; ch += 2) {
        const bool more1 = ch + 1 < p.nchunks;
        if (more1) load_chunk(ch + 1);
        compute_chunk(0);
        if (more1) store_chunk(1);
        __syncthreads();
        if (!more1) break;
        const bool more2 = ch + 2 < p.nchunks;
        if (more2) load_chunk(ch + 2);
        compute_chunk(1);
        if (more2) store_chunk(0);
        __syncthreads();
    }

    // ---- epilogue: bias, ReLU, store into layers [coff, coff+Cout) ---------------------
    // An accumulator register holds MT consecutive pixels across lanes, so each store
    // instruction writes contiguous runs.  The layer index splits into a uniform part
    // (scalar address arithmetic) and a per-lane part folded into the lane's byte offset.
    const int mw = m0 + wm * (BM / WM);          // uniform: first layer of this wavefront
    const int lrow = M::row_lane(lane);          // per lane
    const rsrc_t rout = make_rsrc(p.out, p.out_bytes);
    const uint32_t hs = (uint32_t)p.HoWo * 4u;
    auto write_out = [&](Acc (&res)[TM][TN], const float *bptr, int cout, int coff) {
        float bias[TM][M::NR];
        if (bptr) {
            const rsrc_t rb = make_rsrc(bptr, (uint32_t)cout * 4u);   // layers beyond cout read zero
#pragma unroll
            for (int x = 0; x < TM; ++x)
#pragma unroll
                for (int r = 0; r < M::NR; ++r) {
                    // with a partial layer tile the whole index goes into the range-checked lane
                    // offset, so nothing is read past the end of the bias array
                    const int mu = mw + x * MT + M::row_reg(r);
                    bias[x][r] = full_m ? buf_ld(rb, (uint32_t)(lrow * 4), (uint32_t)mu * 4u)
                                        : buf_ld(rb, (uint32_t)((mu + lrow) * 4), 0u);
                }
        } else {
#pragma unroll
            for (int x = 0; x < TM; ++x)
#pragma unroll
                for (int r = 0; r < M::NR; ++r) bias[x][r] = 0.f;
        }
#pragma unroll
        for (int y = 0; y < TN; ++y) {
            const int pp = P0 + wn * (BN / WN) + y * MT + li;
            const int ppc = min(pp, p.PT - 1);
            const int n = fdiv(ppc, p.dHoWo), q = ppc - n * p.HoWo;
            // pixels past the end get an offset the range check rejects
            const uint32_t lbase = pp < p.PT ? (uint32_t)(((n * p.ldc + coff + lrow) * p.HoWo + q) * 4) : kOob;
#pragma unroll
            for (int x = 0; x < TM; ++x) {
#pragma unroll
                for (int r = 0; r < M::NR; ++r) {
                    const int mu = mw + x * MT + M::row_reg(r);
                    float v = res[x][y][r] + bias[x][r];
                    if (p.relu) v = fmaxf(v, 0.f);
                    if (full_m)
                        buf_st(rout, lbase, (uint32_t)mu * hs, v);
                    else
                        buf_st(rout, mu + lrow < cout ? lbase : kOob, (uint32_t)mu * hs, v);
                }
            }
        }
    };
    if (m0 < p.Cout) write_out(acc, p.b, p.Cout, p.coff);
    if constexpr (E1) {
        if (m0 < p.Cout1) write_out(acc1, p.b1, p.Cout1, p.coff1);
    }
}

// ---------------------------------------------------------------------------------------
struct Variant {
    const char *name;
    int KS, S, BM, BN, MT, CC, PE, NBUF, NT;
    KernelFn kernel;
    bool conv1_type;      // the persistent 7x7/stride-2/three-layer kernel
    KernelFn kernel_tail; // same tiling for Cin not a multiple of CC (nullptr for conv1_type)
    KernelFn kernel_e1;   // same tiling with the fused 1x1 expand (nullptr if not compiled)
};

#define SQ_VARIANT(KS, S, BM, BN, WM, WN, MT, CC, PE, MINW)                                          \
    {"k" #KS "s" #S "_" #BM "x" #BN "_w" #WM "x" #WN "_m" #MT "_c" #CC "_o" #MINW, KS, S, BM, BN, MT, CC, PE, 2, \
     WM * WN * 64, conv_mfma_f32_kernel<KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, false>, false,        \
     conv_mfma_f32_kernel<KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, true>, nullptr}

// a 3x3 tiling that is also compiled with the fused 1x1 expand
#define SQ_VARIANT_E1(KS, S, BM, BN, WM, WN, MT, CC, PE, MINW)                                       \
    {"k" #KS "s" #S "_" #BM "x" #BN "_w" #WM "x" #WN "_m" #MT "_c" #CC "_o" #MINW, KS, S, BM, BN, MT, CC, PE, 2, \
     WM * WN * 64, conv_mfma_f32_kernel<KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, false>, false,        \
     conv_mfma_f32_kernel<KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, true>,                              \
     conv_mfma_f32_kernel<KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, false, true>}

const Variant kVariants[] = {
    // 3x3 stride 1 (expand3x3)
    SQ_VARIANT(3, 1, 128, 128, 2, 2, 32, 4, 2, 2),
    SQ_VARIANT_E1(3, 1, 64, 128, 2, 2, 32, 4, 2, 2),
    SQ_VARIANT_E1(3, 1, 64, 128, 1, 4, 32, 4, 2, 2),
    SQ_VARIANT_E1(3, 1, 64, 64, 2, 2, 32, 4, 2, 2),
    SQ_VARIANT_E1(3, 1, 64, 128, 1, 4, 16, 4, 2, 2),
    SQ_VARIANT(3, 1, 32, 64, 2, 2, 16, 4, 8, 2),
    SQ_VARIANT(3, 1, 64, 128, 2, 2, 32, 8, 2, 2),
    SQ_VARIANT(3, 1, 64, 256, 1, 4, 32, 4, 3, 2),
    SQ_VARIANT(3, 1, 128, 128, 2, 2, 32, 8, 2, 1),
    SQ_VARIANT(3, 1, 128, 256, 2, 2, 32, 4, 3, 1),
    // 1x1 (squeeze, expand1x1, conv10)
    SQ_VARIANT(1, 1, 128, 128, 2, 2, 32, 16, 0, 2),
    SQ_VARIANT(1, 1, 64, 128, 2, 2, 32, 16, 0, 2),
    SQ_VARIANT(1, 1, 64, 128, 1, 4, 32, 16, 0, 2),
    SQ_VARIANT(1, 1, 64, 64, 2, 2, 32, 16, 0, 2),
    SQ_VARIANT(1, 1, 16, 256, 1, 4, 16, 16, 0, 2),
    SQ_VARIANT(1, 1, 32, 128, 1, 4, 16, 16, 0, 2),
    SQ_VARIANT(1, 1, 32, 128, 1, 4, 32, 16, 0, 2),
    SQ_VARIANT(1, 1, 32, 256, 1, 4, 32, 16, 0, 2),
    SQ_VARIANT(1, 1, 48, 128, 1, 4, 16, 16, 0, 2),
    SQ_VARIANT(1, 1, 64, 256, 1, 4, 32, 16, 0, 2),
    SQ_VARIANT(1, 1, 128, 128, 2, 2, 16, 16, 0, 2),
    SQ_VARIANT(1, 1, 64, 64, 2, 2, 16, 32, 0, 3),
    SQ_VARIANT(1, 1, 128, 128, 2, 2, 32, 32, 0, 2),
    // small tiles for the layers with few pixels (more workgroups than CUs)
    SQ_VARIANT(1, 1, 32, 64, 1, 4, 16, 16, 0, 2),
    SQ_VARIANT(1, 1, 16, 128, 1, 4, 16, 16, 0, 2),
    SQ_VARIANT(1, 1, 16, 64, 1, 4, 16, 32, 0, 2),
    SQ_VARIANT(1, 1, 32, 64, 1, 4, 16, 32, 0, 2),
    SQ_VARIANT(1, 1, 64, 64, 2, 2, 16, 16, 0, 2),
    SQ_VARIANT(1, 1, 48, 64, 1, 4, 16, 16, 0, 2),
    // 7x7 stride 2 with three input layers (conv1): persistent autonomous wavefronts,
    // 148-long contraction (BN and PE are unused for these two)
    {"k7s2c3_waves8", 7, 2, 96, 256, 32, 3, 64, 2, 512, conv7s2c3_kernel_for(8, true), true, nullptr, nullptr},
    {"k7s2c3_waves4", 7, 2, 96, 128, 32, 3, 64, 2, 256, conv7s2c3_kernel_for(4, true), true, nullptr, nullptr},
    // 7x7 stride 2, any number of input layers, two per chunk
    SQ_VARIANT(7, 2, 96, 128, 1, 4, 32, 2, 15, 1),
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
struct FusedE1 {
    const void *w1;
    const float *b1;
    int Cout1, coff1;
};

bool plan(const Variant &v, const ConvArgs &a, Plan &pl, const FusedE1 *e1 = nullptr)
{
    if (e1 && (!v.kernel_e1 || a.Cin % v.CC != 0)) return false;
    if (a.dtype != SQ_F32 || a.K != v.KS || a.S != v.S) return false;
    if (a.W + 2 * a.P < a.K) return false;
    const long long in_elems = (long long)a.N * a.Cin * a.H * a.W;
    const long long out_elems = (long long)a.N * a.out_channels * a.Ho * a.Wo;
    const long long pixels = (long long)a.N * a.Ho * a.Wo;
    // per-lane addresses are 32-bit byte offsets from a uniform base
    const long long w_elems = (long long)a.Cout * a.Cin * a.K * a.K;
    if (in_elems >= kMaxBufferElems || out_elems >= kMaxBufferElems || w_elems >= kMaxBufferElems ||
        pixels + v.BN >= kMaxBufferElems)
        return false;
    if (v.conv1_type && (a.Cin != 3 || a.Cout > 96 || a.Cout % 8 != 0)) return false;

    KParams &k = pl.kp;
    k.in = (const float *)a.in; k.w = (const float *)a.w; k.b = a.b; k.out = a.out;
    k.N = a.N; k.Cin = a.Cin; k.H = a.H; k.W = a.W; k.Cout = a.Cout; k.P = a.P; k.relu = a.relu;
    k.Ho = a.Ho; k.Wo = a.Wo; k.HoWo = a.Ho * a.Wo; k.HW = a.H * a.W;
    k.ldc = a.out_channels; k.coff = a.c_offset;
    k.PT = (int)pixels;
    k.mtiles = ((e1 && e1->Cout1 > a.Cout ? e1->Cout1 : a.Cout) + v.BM - 1) / v.BM;
    k.w1 = e1 ? (const float *)e1->w1 : nullptr; k.b1 = e1 ? e1->b1 : nullptr;
    k.Cout1 = e1 ? e1->Cout1 : 0; k.coff1 = e1 ? e1->coff1 : 0;
    k.w1_bytes = e1 ? (uint32_t)((long long)e1->Cout1 * a.Cin * 4) : 0u;
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
    k.dWo = make_fastdiv(k.Wo); k.dHo = make_fastdiv(k.Ho); k.dLW = make_fastdiv(k.LW);
    k.dVH = make_fastdiv(k.VH); k.dHW = make_fastdiv(k.HW); k.dHoWo = make_fastdiv(k.HoWo);
    k.dMtiles = make_fastdiv(k.mtiles);
    k.in_bytes = (uint32_t)(in_elems * 4); k.out_bytes = (uint32_t)(out_elems * 4); k.w_bytes = (uint32_t)(w_elems * 4);
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
        pl.lds_bytes = conv7s2c3_lds_bytes(NW);
        blocks = (tiles + NW - 1) / NW;
        if (blocks > num_cus()) blocks = num_cus();
    } else {
        pl.lds_bytes = ((size_t)v.NBUF * v.BM * LDK + (size_t)v.NBUF * v.CC * k.plane +
                        (e1 ? (size_t)2 * v.BM * (v.CC + 1) : 0)) * sizeof(float);
    }
    if (pl.lds_bytes > (size_t)kLdsBytes) return false;
    if (blocks >= (1ll << 31)) return false;
    pl.blocks = (unsigned)blocks;
    return true;
}

// Dynamic LDS above the default limit must be opted into once per kernel function.
bool allow_big_lds(KernelFn fn)
{
    static KernelFn done[2 * kNumVariants + 4];
    static int ndone = 0;
    for (int i = 0; i < ndone; ++i)
        if (done[i] == fn) return true;
    if (hipFuncSetAttribute((const void *)fn, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess)
        return false;
    if (ndone < (int)(sizeof(done) / sizeof(done[0]))) done[ndone++] = fn;
    return true;
}

int launch(int vi, const Plan &pl, const ConvArgs &a, const FusedE1 *e1 = nullptr)
{
    const Variant &v = kVariants[vi];
    KernelFn fn = e1 ? v.kernel_e1 : v.kernel;
    if (v.conv1_type && a.Cout != 96) fn = conv7s2c3_kernel_for(v.NT / 64, false);
    if (!v.conv1_type && !e1 && a.Cin % v.CC != 0) fn = v.kernel_tail;
    if (!allow_big_lds(fn)) {
        const int rc = check_launch();
        return rc ? rc : SQ_ERR_HIP;
    }
    double flops = conv_flops(a), bytes = conv_bytes(a);
    if (e1) {
        flops += 2.0 * a.N * e1->Cout1 * a.Ho * a.Wo * (double)a.Cin;
        bytes += 4.0 * ((double)e1->Cout1 * a.Cin + (double)a.N * e1->Cout1 * a.Ho * a.Wo + e1->Cout1);
    }
    LaunchScope scope(v.name, flops, bytes);
    hipLaunchKernelGGL(fn, dim3(pl.blocks), dim3(v.NT), pl.lds_bytes, current_stream(), pl.kp);
    return check_launch();
}

// Measured winners (written by tune.py).  An entry applies to its exact layer shape and to
// the batch sizes nearest to the one it was measured at.
struct Tuned {
    int K, S, P, Cin, Cout, H, W, N;
    const char *variant;
};
const Tuned kTuned[] = {
#include "tuned_table.inc"
    {0, 0, 0, 0, 0, 0, 0, 0, ""}};

int tuned_variant(const ConvArgs &a)
{
    const Tuned *best = nullptr;
    double best_dist = 0;
    for (const Tuned *e = kTuned; e->K; ++e) {
        if (e->K != a.K || e->S != a.S || e->P != a.P || e->Cin != a.Cin || e->Cout != a.Cout || e->H != a.H ||
            e->W != a.W)
            continue;
        const double d = fabs(log((double)a.N / e->N));
        if (!best || d < best_dist) {
            best = e; best_dist = d;
        }
    }
    if (!best) return -1;
    for (int i = 0; i < kNumVariants; ++i)
        if (!strcmp(kVariants[i].name, best->variant)) return i;
    return -1;
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

// Host-side self check of the division-by-multiplication used in the kernels: number of
// x in [0, x_max] for which it disagrees with x / d (exported for the tests, not part of
// the public interface).
extern "C" long long sq_internal_fastdiv_mismatches(unsigned d, unsigned x_max)
{
    const mfma::FastDiv f = mfma::make_fastdiv(d);
    long long bad = 0;
    for (unsigned long long x = 0; x <= x_max; ++x) bad += mfma::fastdiv_host((unsigned)x, f) != (unsigned)x / (d ? d : 1);
    return bad;
}

int conv_mfma_variant_count() { return kNumVariants; }
const char *conv_mfma_variant_name(int i) { return kVariants[i].name; }

// Which tiling runs the fused expand: -2 = never fuse (the default: measured on MI355X the
// fused kernel's lower occupancy cancels what it saves), -1 = automatic
// choice, i >= 0 = tiling i.  The setter is a tuning hook, not part of the public interface.
int g_force_expand = -2;
extern "C" void sq_internal_force_expand(int v) { g_force_expand = v; }

// 3x3 (pad 1, stride 1) convolution a3 plus the 1x1 convolution (w1, b1, Cout1 layers) of the
// same input, results in layers [a3.c_offset, +a3.Cout) and [coff1, +Cout1) of one tensor.
int conv_expand_fused(const ConvArgs &a3, const void *w1, const float *b1, int Cout1, int coff1)
{
    if (a3.K != 3 || a3.S != 1 || a3.P != 1 || a3.dtype != SQ_F32) return SQ_ERR_UNSUPPORTED;
    const FusedE1 e1{w1, b1, Cout1, coff1};
    Plan pl;
    if (g_force_expand == -2) return SQ_ERR_UNSUPPORTED;
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

int conv_mfma(const ConvArgs &a, int variant)
{
    Plan pl;
    if (variant >= 0) {
        if (variant >= kNumVariants || !plan(kVariants[variant], a, pl)) return SQ_ERR_UNSUPPORTED;
        return launch(variant, pl, a);
    }
    const int tv = tuned_variant(a);
    if (tv >= 0 && plan(kVariants[tv], a, pl)) return launch(tv, pl, a);
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
