// Kernel template of the implicit-GEMM convolution on the fp32 matrix cores (MFMA) of gfx950
// (internal; instantiated per input type in conv_mfma_f32.hip and conv_mfma_bf16.hip).
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
#pragma once

#include "conv_mfma_common.h"

namespace sq {
namespace mfma {

// TAIL: the number of input layers is not a multiple of CC, so the last chunk is partly
// padding (compiled separately to keep the common loop free of the test).
// E1: fused expand -- next to the KxK convolution the workgroup also computes a 1x1
// convolution of the same input (its kernels p.w1) for the same pixels and its own tile of
// layers, written to layers [coff1, coff1+Cout1): the 1x1 reuses the centre-tap patch
// operands, so the input is staged once for both (fire layer, section "Convolutional
// Neural Networks": the two expand layers read the same squeeze result).
// TIN: element type of the input and the kernels in memory, float or uint16_t (bfloat16).
// bfloat16 values are widened to fp32 while they are staged (a shift), so LDS and the MFMAs
// are the same as for fp32 inputs; products of two bfloat16 values are exact in fp32.
// POOL (1x1 kernels only): the input is max-pooled (3x3 window, stride 2, floor mode) on the way
// in -- in this network every pooled map is read by exactly one squeeze layer, so it need not
// exist in memory.  p.H, p.W are the pooled extents, p.Win / p.HWin those of the map in memory; a
// staged element is the maximum of nine loads (per window row one 8-byte and one 4-byte load).
// POOL == 2: the layer before has already pooled the columns (column-pooled map, see ColPool): row r of the map
// in memory holds, for pooled column x, the maximum over columns 2x..2x+2 of that layer's row r -- except in the
// last pooled column of a column group of the producer (a conv1 tile, a tile group of the minimal-filtering
// kernel), where the third column belongs to the next group and sits, unpooled, in a seam slot right behind.  This
// kernel takes the maximum over rows 2y..2y+2 and, at those columns, the seam slots: three 8-byte loads per staged
// element instead of nine values, and about half the bytes.  The second value of a load is used only at a seam
// (chosen with a select, so whatever else lies there does no harm).  The producers leave their ReLU to this kernel:
// the maximum it takes always contains a zero (the value selected where there is no seam).
//
// conv_mfma_tile is the work of one workgroup (tile number `block` of the launch), conv_mfma_kernel the
// kernel that consists of nothing else; the expand pair kernel (conv_wino_kernel.h) runs the same tiles
// behind its own.
// AVG (1x1 kernels only): instead of the results themselves the tile writes, per output layer, the sums of its
// ReLU'd results over the pixels of each image it touches -- the first half of a global average pooling (section
// "Pooling and Softmax") that follows the convolution directly, so that the convolution's map is never written.
// p.out is then a table [pixel tile][WN][p.avg_slots][Cout]: slot s of pixel tile pt holds the sum over the pixels of
// image (first image of the tile) + s among the BN / WN pixels of wavefront column wn; whoever adds the slots of an
// image up (avg_softmax_kernel) has the plane sums.  Slots without pixels hold zero.
template <typename TIN, int KS, int S, int BM, int BN, int WM, int WN, int MT, int CC, int PE, bool TAIL, bool E1 = false,
          int POOL = 0, bool AVG = false>
__device__ __forceinline__ void conv_mfma_tile(const KParams &p, const int block)
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
    static_assert(!POOL || (POINTWISE && !TAIL && !E1), "pooling on the way in is for plain 1x1 kernels");
    static_assert(POOL != 2 || sizeof(TIN) == 4, "a column-pooled map is fp32");
    constexpr int NWIN = POOL == 2 ? 6 : 9;
    static_assert(!AVG || (POINTWISE && !E1 && !POOL), "plane sums are for plain 1x1 kernels");
    constexpr int ESZ = (int)sizeof(TIN);
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

    const int tile = xcd_remap(block, p.mtiles * p.ntiles);
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
        wsrc[r] = (inrange && m0 + m < p.Cout) ? (uint32_t)(((m0 + m) * p.Cin * KK + q) * ESZ) : kOob;
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
            w1src[r] = (inrange && m0 + m < p.Cout1) ? (uint32_t)(((m0 + m) * p.Cin + c) * ESZ) : kOob;
            w1dst[r] = inrange ? m * LD1 + c : -1;
        }
    }
    uint32_t xsrc[XMAP];
    uint32_t xsrcB = kOob;   // POOL == 2: the third row
    bool seamA = false, seamB = false;
    int xdst[XMAP];
    if constexpr (POINTWISE) {
        const int pl = t % BN, pp = P0 + pl;
        const int n = fdiv(pp, p.dHW);
        if constexpr (POOL == 2) {
            // this pixel's column in rows 2y, 2y+1 (one producer tile row) and 2y+2 (the next one): the position
            // counts the seam slots before it, which depends on where the row's slots fall in their groups
            const int pix = pp - n * p.HW, y = fdiv(pix, p.dWo), x = pix - y * p.Wo;
            const int gm = (1 << p.cpShift) - 1;
            const int qa = n * p.cpSlotsImage + y * p.cpSlotsRow, qb = qa + p.cpSlotsRow;
            const int posa = x + ((qa + x) >> p.cpShift) - (qa >> p.cpShift), posb = x + ((qb + x) >> p.cpShift) - (qb >> p.cpShift);
            xsrc[0] = pp < p.PT ? (uint32_t)((n * p.Cin * p.HWin + 2 * y * p.Win + posa) * ESZ) : kOob;
            xsrcB = pp < p.PT ? (uint32_t)((n * p.Cin * p.HWin + (2 * y + 2) * p.Win + posb) * ESZ) : kOob;
            seamA = ((qa + x) & gm) == gm;
            seamB = ((qb + x) & gm) == gm;
        } else if constexpr (POOL == 1) {
            // first element of this pixel's window in the map before pooling
            const int pix = pp - n * p.HW, y = fdiv(pix, p.dWo), x = pix - y * p.Wo;
            xsrc[0] = pp < p.PT ? (uint32_t)((n * p.Cin * p.HWin + 2 * y * p.Win + 2 * x) * ESZ) : kOob;
        } else {
            xsrc[0] = pp < p.PT ? (uint32_t)((n * p.Cin * p.HW + (pp - n * p.HW)) * ESZ) : kOob;
        }
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
            xsrc[r] = inb ? (uint32_t)(((n * p.Cin * p.H + ih) * p.W + iw) * ESZ) : kOob;
            xdst[r] = stage ? vr * p.LWs + pc : -1;
        }
    }
    const int cpart = POINTWISE ? __builtin_amdgcn_readfirstlane(t / BN) : 0;

    float wreg[WREG], xreg[XREG], w1reg[W1REG], xwin[POOL ? XREG : 1][NWIN];

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
        const uint32_t wchunk = (uint32_t)(c0 * KK * ESZ);
        if (TAIL && c0 + CC > p.Cin) {
            // last chunk runs past the input layers: those kernel values and patch planes are zero
#pragma unroll
            for (int r = 0; r < WREG; ++r) {
                const int q = (t + NT * r) % RUN;
                wreg[r] = buf_ld_in<TIN>(rw, c0 + q / KK < p.Cin ? wsrc[r] : kOob, wchunk);
            }
#pragma unroll
            for (int r = 0; r < XREG; ++r) {
                const int c = POINTWISE ? cpart + (NT / BN) * r : r / XMAP;   // uniform
                const int i = POINTWISE ? 0 : r % XMAP;
                if (c0 + c < p.Cin)
                    xreg[r] = buf_ld_in<TIN>(rin, xsrc[i], (uint32_t)__builtin_amdgcn_readfirstlane((c0 + c) * p.HW * ESZ));
                else
                    xreg[r] = 0.f;
            }
            return;
        }
#pragma unroll
        for (int r = 0; r < WREG; ++r) wreg[r] = buf_ld_in<TIN>(rw, wsrc[r], wchunk);
        if constexpr (E1) {
#pragma unroll
            for (int r = 0; r < W1REG; ++r) w1reg[r] = buf_ld_in<TIN>(rw1, w1src[r], (uint32_t)(c0 * ESZ));
        }
        if constexpr (POOL == 2) {
#pragma unroll
            for (int r = 0; r < XREG; ++r) {
                const uint32_t so = (uint32_t)__builtin_amdgcn_readfirstlane((c0 + cpart + (NT / BN) * r) * p.HWin * ESZ);
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    uint32_t off = i < 2 ? xsrc[0] + (uint32_t)(i * p.Win * ESZ) : xsrcB;
                    asm volatile("" : "+v"(off));   // the two loads differ by an immediate and merge into one of 8 bytes
                    xwin[r][2 * i] = buf_ld_in<TIN>(rin, off, so);
                    xwin[r][2 * i + 1] = buf_ld_in<TIN>(rin, off + (uint32_t)ESZ, so);
                }
            }
            return;
        }
        if constexpr (POOL == 1) {
            // the nine values of every window stay in registers until store_chunk takes their maximum, so that
            // the loads are in flight during the MFMAs of the chunk before (an out-of-range pixel reads zeros)
#pragma unroll
            for (int r = 0; r < XREG; ++r) {
                const uint32_t so = (uint32_t)__builtin_amdgcn_readfirstlane((c0 + cpart + (NT / BN) * r) * p.HWin * ESZ);
#pragma unroll
                for (int i = 0; i < 3; ++i) {
                    uint32_t off = xsrc[0] + (uint32_t)(i * p.Win * ESZ);   // an offset turned away stays beyond the range
                    asm volatile("" : "+v"(off));   // the loads of a window row differ by immediates: two of them merge
#pragma unroll
                    for (int jx = 0; jx < 3; ++jx) xwin[r][3 * i + jx] = buf_ld_in<TIN>(rin, off + (uint32_t)(jx * ESZ), so);
                }
            }
            return;
        }
#pragma unroll
        for (int r = 0; r < XREG; ++r) {
            const int c = POINTWISE ? cpart + (NT / BN) * r : r / XMAP;       // uniform
            const int i = POINTWISE ? 0 : r % XMAP;
            xreg[r] = buf_ld_in<TIN>(rin, xsrc[i], (uint32_t)__builtin_amdgcn_readfirstlane((c0 + c) * p.HW * ESZ));
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
        if constexpr (POOL == 2) {
#pragma unroll
            for (int r = 0; r < XREG; ++r) {
                const float m = fmaxf(fmaxf(xwin[r][0], xwin[r][2]), xwin[r][4]);
                // a missing seam counts as zero, which is also the producer's ReLU
                const float sa = seamA ? fmaxf(xwin[r][1], xwin[r][3]) : 0.f, sb = seamB ? xwin[r][5] : 0.f;
                xs[(cpart + (NT / BN) * r) * plane + xdst[0]] = fmaxf(m, fmaxf(sa, sb));
            }
        } else if constexpr (POOL == 1) {
#pragma unroll
            for (int r = 0; r < XREG; ++r) {
                float m = xwin[r][0];
#pragma unroll
                for (int e = 1; e < NWIN; ++e) m = fmaxf(m, xwin[r][e]);
                xs[(cpart + (NT / BN) * r) * plane + xdst[0]] = m;
            }
        } else if constexpr (POINTWISE) {
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

    // Accumulators start from the bias (zero without one), so the epilogue has no addition
    // left: every vector-ALU instruction there would add to the run time, since such work
    // does not overlap with the fp32 MFMAs of other wavefronts.  The layer index of a result
    // register splits into a uniform part and a per-lane part; with a partial layer tile the
    // whole index goes into the range-checked lane offset, so nothing is read past the end of
    // the bias array.
    const int mw = m0 + wm * (BM / WM);          // uniform: first layer of this wavefront
    const int lrow = M::row_lane(lane);          // per lane
    Acc acc[TM][TN], acc1[E1 ? TM : 1][E1 ? TN : 1];
    auto start_from_bias = [&](Acc (&a)[TM][TN], const float *bptr, int cout) {
        if (bptr) {
            const rsrc_t rb = make_rsrc(bptr, (uint32_t)cout * 4u);   // layers beyond cout read zero
#pragma unroll
            for (int x = 0; x < TM; ++x)
#pragma unroll
                for (int r = 0; r < M::NR; ++r) {
                    const int mu = mw + x * MT + M::row_reg(r);
                    const float bv = full_m ? buf_ld(rb, (uint32_t)(lrow * 4), (uint32_t)mu * 4u)
                                            : buf_ld(rb, (uint32_t)((mu + lrow) * 4), 0u);
#pragma unroll
                    for (int y = 0; y < TN; ++y) a[x][y][r] = bv;
                }
        } else {
#pragma unroll
            for (int x = 0; x < TM; ++x)
#pragma unroll
                for (int y = 0; y < TN; ++y)
#pragma unroll
                    for (int r = 0; r < M::NR; ++r) a[x][y][r] = 0.f;
        }
    };
    start_from_bias(acc, p.b, p.Cout);
    if constexpr (E1) start_from_bias(acc1, p.b1, p.Cout1);

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

    if constexpr (AVG) {
        // ---- epilogue of the averaging form: per-image sums over this wavefront's pixels ----
        const float lowest = p.relu ? 0.f : -__builtin_inff();
        const int imgA = fdiv(P0, p.dHoWo);
        int slot_of[TN];
#pragma unroll
        for (int y = 0; y < TN; ++y) {
            const int pp = P0 + wn * (BN / WN) + y * MT + li;
            slot_of[y] = pp < p.PT ? fdiv(pp, p.dHoWo) - imgA : -1;
        }
        float *part = p.out + (size_t)(pt * WN + wn) * p.avg_slots * p.Cout;
        for (int s = 0; s < p.avg_slots; ++s) {
#pragma unroll
            for (int x = 0; x < TM; ++x)
#pragma unroll
                for (int r = 0; r < M::NR; ++r) {
                    float v = 0.f;
#pragma unroll
                    for (int y = 0; y < TN; ++y) v += slot_of[y] == s ? fmaxf(acc[x][y][r], lowest) : 0.f;
#pragma unroll
                    for (int off = MT / 2; off >= 1; off >>= 1) v += __shfl_xor(v, off);
                    const int mu = mw + x * MT + M::row_reg(r) + lrow;
                    if (li == 0 && mu < p.Cout) part[s * p.Cout + mu] = v;
                }
        }
        return;
    }

    // ---- epilogue: ReLU, store into layers [coff, coff+Cout) ------------------------------
    // An accumulator register holds MT consecutive pixels across lanes, so each store
    // instruction writes contiguous runs: uniform layer part in the scalar offset, per-lane
    // part in the lane's byte offset, one vector-ALU instruction (the ReLU) per register.
    const rsrc_t rout = make_rsrc(p.out, p.out_bytes);
    const uint32_t hs = (uint32_t)p.HoWo * 4u;
    const float lowest = p.relu ? 0.f : -__builtin_inff();
    auto write_out = [&](Acc (&res)[TM][TN], int cout, int coff, auto full_tile) {
        constexpr bool FULL = decltype(full_tile)::value;
        if constexpr (WN == 1 && TN > 1) {
            // One wavefront holds all BN pixels of its layers: layer by layer, the pixel blocks one after the other,
            // so that consecutive stores of a wavefront fill whole cache lines (a map much larger than the
            // memory-side cache is written at half the rate when its lines reach memory in pieces).
            uint32_t lb[TN];
#pragma unroll
            for (int y = 0; y < TN; ++y) {
                const int pp = P0 + y * MT + li;
                const int ppc = min(pp, p.PT - 1);
                const int n = fdiv(ppc, p.dHoWo), q = ppc - n * p.HoWo;
                lb[y] = pp < p.PT ? (uint32_t)(((n * p.ldc + coff + lrow) * p.HoWo + q) * 4) : kOob;
            }
#pragma unroll
            for (int x = 0; x < TM; ++x)
#pragma unroll
                for (int r = 0; r < M::NR; ++r) {
                    const int mu = mw + x * MT + M::row_reg(r);
                    const bool ok = FULL || mu + lrow < cout;
#pragma unroll
                    for (int y = 0; y < TN; ++y) buf_st(rout, ok ? lb[y] : kOob, (uint32_t)mu * hs, fmaxf(res[x][y][r], lowest));
                }
            return;
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
                    const float v = fmaxf(res[x][y][r], lowest);
                    if constexpr (FULL)
                        buf_st(rout, lbase, (uint32_t)mu * hs, v);
                    else
                        buf_st(rout, mu + lrow < cout ? lbase : kOob, (uint32_t)mu * hs, v);
                }
            }
        }
    };
    if (full_m) {
        write_out(acc, p.Cout, p.coff, std::true_type{});
        if constexpr (E1) write_out(acc1, p.Cout1, p.coff1, std::true_type{});
    } else {
        if (m0 < p.Cout) write_out(acc, p.Cout, p.coff, std::false_type{});
        if constexpr (E1) {
            if (m0 < p.Cout1) write_out(acc1, p.Cout1, p.coff1, std::false_type{});
        }
    }
}

template <typename TIN, int KS, int S, int BM, int BN, int WM, int WN, int MT, int CC, int PE, int MINW, bool TAIL, bool E1 = false,
          int POOL = 0, bool AVG = false>
__global__ __launch_bounds__(WM * WN * 64, MINW) void conv_mfma_kernel(const KParams p)
{
    conv_mfma_tile<TIN, KS, S, BM, BN, WM, WN, MT, CC, PE, TAIL, E1, POOL, AVG>(p, (int)blockIdx.x);
}

}  // namespace mfma
}  // namespace sq
