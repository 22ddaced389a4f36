// 3x3 / stride 1 / pad 1 convolution through the minimal-filtering form F(2x2, 3x3) on the
// fp32 matrix cores of gfx950 (internal).
//
// The layer of section "Convolutional Neural Networks" computes, per 2x2 block of output
// pixels ("tile") and output layer m,  Y = sum_c  g[m][c] (*) d[c]  with d the 4x4 input patch
// under the tile.  With the transforms  U = G g G^T,  V = B^T d B  (both 4x4) the same Y is
// A^T ( sum_c U (.) V ) A:  per position xi of the 4x4 grid one small matrix product
//   M_xi[m][tile] = sum_c U_xi[m][c] * V_xi[c][tile],
// i.e. 16 multiplies per input layer and tile where the direct form needs 36.  The sixteen
// products are independent contractions over the input layers and run on the MFMA units;
// the transforms are a few additions per element on the vector ALU.
//
//   B^T = | 1  0 -1  0 |   G = | 1    0    0  |   A^T = | 1  1  1  0 |
//         | 0  1  1  0 |       | 1/2  1/2  1/2|         | 0  1 -1 -1 |
//         | 0 -1  1  0 |       | 1/2 -1/2  1/2|
//         | 0  1  0 -1 |       | 0    0    1  |
//
// Two kernels.  wino_kernel_transform writes U for all (m, c) once per call (for several
// layers at once when the caller has several), already in the order in which the lanes of
// the main kernel take it as MFMA operands, so the main kernel loads it with 16-byte loads
// and spends no arithmetic on it.  conv_wino_kernel: a workgroup owns 64 output
// layers x 32 tiles and has 4 wavefronts (pr, x): wavefront (pr, x) accumulates the eight
// positions of two grid rows for layers 32x..32x+31 and all 32 tiles in eight
// accumulators of v_mfma_f32_32x32x2_f32 (A operand = output layers, B operand = tiles).
// Input layers are taken eight at a time; U in memory and the V image in LDS hold, per
// position and per lane half kk, the four values c = kk, kk+2, kk+4, kk+6 of a layer (tile)
// side by side, so one 16-byte read feeds four MFMAs.  A wavefront needs exactly a quarter
// of the U of a chunk, and no other wavefront needs that quarter: it goes from memory (L2)
// straight into the wavefront's registers, one chunk ahead of its use.  Every thread
// transforms the patch of one (tile, input layer) per chunk and writes it into one of two V
// images in LDS while the other one is being multiplied: one barrier per chunk.  Two
// persistent workgroups share a CU (256 registers per wavefront) and loop over tiles.  At the
// end a wavefront folds its two grid rows with A and half of A^T, swaps the other half with
// its partner (pr ^ 1) through LDS, and writes output row pr of its tiles.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

#include "conv_mfma_common.h"
#include "conv_mfma_kernel.h"
#include "conv_wino_auto_kernel.h"

namespace sq {
namespace mfma {

// U = G g G^T for every (m, c) of up to kWinoMaxJobs layers in one launch, written per layer as
// [m / 64][c / 8][xi][c & 1][m % 64][(c % 8) / 2]; layers past Cout (up to the next multiple of
// 64) are written as zeros.  Thread i of the grid handles element i - first of the job that
// holds it.
struct WinoJobs {
    const void *w[kWinoMaxJobs];
    float *u[kWinoMaxJobs];
    float *u2[kWinoMaxJobs];       // the same values in the order of conv_wino_auto_kernel.h (layers < Cout only)
    int Cout[kWinoMaxJobs], Cin[kWinoMaxJobs];
    int first[kWinoMaxJobs + 1];   // running totals of Cout (rounded up to 64) * Cin
    int n;
};

template <typename TIN>
__global__ __launch_bounds__(256) void wino_kernel_transform(const WinoJobs jobs)
{
    const int gi = blockIdx.x * 256 + threadIdx.x;
    if (gi >= jobs.first[jobs.n]) return;
    int j = 0;
    while (gi >= jobs.first[j + 1]) ++j;
    const int i = gi - jobs.first[j], Cin = jobs.Cin[j], Cout = jobs.Cout[j];
    const TIN *w = (const TIN *)jobs.w[j];
    const int m = i / Cin, c = i - m * Cin;
    float g[9];
#pragma unroll
    for (int q = 0; q < 9; ++q) {
        if (m >= Cout) g[q] = 0.f;
        else if constexpr (sizeof(TIN) == 2) g[q] = __builtin_bit_cast(float, (uint32_t)w[(size_t)i * 9 + q] << 16);
        else g[q] = w[(size_t)i * 9 + q];
    }
    float tt[4][3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        const float s = g[k] + g[6 + k];
        tt[0][k] = g[k];
        tt[1][k] = 0.5f * (s + g[3 + k]);
        tt[2][k] = 0.5f * (s - g[3 + k]);
        tt[3][k] = g[6 + k];
    }
    const int cl = c % kWinoCC;
    float *dst = jobs.u[j] + ((size_t)(m / kWinoBM) * (Cin / kWinoCC) + c / kWinoCC) * kWinoImage + (cl & 1) * 256 +
                 (m % kWinoBM) * 4 + (cl >> 1);
    // second layout: [m / 32][c / 4][position / 2][lane = (c % 4) * 16 + m % 16][2 * (position % 2) + (m % 32) / 16]
    float *dst2 = jobs.u2[j] + ((size_t)(m / 32) * (Cin / 4) + c / 4) * kWinoAutoStep + ((c & 3) * 16 + (m & 15)) * 4 + ((m & 31) >> 4);
    const bool second = m < Cout;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float s = tt[r][0] + tt[r][2];
        const float u4[4] = {tt[r][0], 0.5f * (s + tt[r][1]), 0.5f * (s - tt[r][1]), tt[r][2]};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int pos = 4 * r + q;
            dst[pos * 512] = u4[q];
            if (second) dst2[(pos >> 1) * 256 + 2 * (pos & 1)] = u4[q];
        }
    }
}

// conv_wino_tiles: what one persistent workgroup does -- tile blocks first, first + stride, ... of the layer.
template <typename TIN>
__device__ __forceinline__ void conv_wino_tiles(const KParams &p, const int first, const int stride)
{
    constexpr int BM = kWinoBM, BT = kWinoBT, CC = kWinoCC;
    static_assert(BM == 64 && BT == 32 && CC == 8, "thread roles below are written for this tile");
    constexpr int US = kWinoImage;             // floats of the U image [16][2][64][4] of one (layer block, chunk) in memory
    constexpr int VS = 16 * 2 * BT * 4;        // floats of the V image [16][2][32][4]; LDS holds two of them
    constexpr uint32_t ESZ = sizeof(TIN);
    using M = Mfma<32>;
    using Acc = M::Acc;
    extern __shared__ __attribute__((aligned(16))) float lds[];

    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int pr = wv & 1, wx = wv >> 1;
    const int li = lane & 31, kk = lane >> 5;

    // Persistent workgroups (two per CU): a workgroup that retires keeps its registers and LDS
    // until its last stores have drained; looping over tiles lets the next tile start behind them.
    const int ntile_blocks = p.mtiles * p.ntiles;
    for (int bid_raw = first; bid_raw < ntile_blocks; bid_raw += stride) {
    if (bid_raw != first) __syncthreads();   // the exchange area of the previous tile has been read out
    const int bid = xcd_remap(bid_raw, ntile_blocks);
    const int tb = fdiv(bid, p.dMtiles);
    const int mt = bid - tb * p.mtiles, m0 = mt * BM, t0 = tb * BT;

    // ---- staging maps ----------------------------------------------------------------------
    // patches: thread -> (tile vt = t % 32, input layer vc = t / 32 of the chunk).
    // Per patch row two lane offsets: the first column on its own (rows outside the image, a
    // tile past the end, or column -1 get the top bit, which the buffer range check turns
    // into zeros) and columns 2, 3, 4 of the patch as one 12-byte run.  Offsets of real
    // elements are never negative.  Columns 3 and 4 may lie right of the image; there the
    // run reads addresses of the next row, or past the last row of the last input layer whatever
    // lies behind the tensor, and the column transform replaces what it read by zero with a
    // select (c2ok, c3ok) -- not with a factor of zero, which would let a NaN or an infinity
    // among those bytes through.
    const int vt = t & 31, vc = t >> 5;
    uint32_t xrow[4], xcol0[4];
    bool c2ok, c3ok;
    {
        const int tg = t0 + vt, tgc = min(tg, p.T - 1);
        const int n = fdiv(tgc, p.dTXY), rem = tgc - n * p.TXY;
        const int ty = fdiv(rem, p.dTX), tx = rem - ty * p.TX;
        const int ih0 = 2 * ty - 1, iw0 = 2 * tx - 1;
        const uint32_t base = (uint32_t)((n * p.Cin + vc) * p.HW + ih0 * p.W + iw0 + 1) * ESZ;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const uint32_t bad = tg < p.T && (unsigned)(ih0 + a) < (unsigned)p.H ? 0u : kOob;
            xrow[a] = (base + (uint32_t)(a * p.W) * ESZ) | bad;
            xcol0[a] = (base + (uint32_t)(a * p.W) * ESZ - ESZ) | bad | (iw0 >= 0 ? 0u : kOob);
        }
        c2ok = iw0 + 2 < p.W;
        c3ok = iw0 + 3 < p.W;
    }
    // V image position of (tile vt, layer vc): lane half vc & 1, slot vc >> 1
    const int vdst = (vc & 1) * (BT * 4) + vt * 4 + (vc >> 1);

    // The wavefront's two grid rows are taken in the order (0, 1) for pr = 0 and (3, 2) for pr = 1, so that the
    // row the partner needs (1 or 2) is the second one in both and the output transform has no per-wavefront
    // choice of registers: accumulator s belongs to grid position gpos(s).
    auto gpos = [&](int s) { return (s < 4 ? 12 * pr : 4 * pr) + s; };   // uniform

    float dpatch[16];
    // A operands.  Of the U image of a (layer block, chunk), wavefront (pr, x) needs exactly the quarter
    // [its 8 positions][kk][32x..32x+31][4]: lane (li, kk) takes its 16 bytes of every position straight from
    // memory (L2) into registers -- the image never passes through LDS.  The uniform offset carries layer block,
    // chunk and position, the lane offset never changes.
    f32x4 A[8];
    const rsrc_t ru = make_rsrc(p.wu, p.wu_bytes);
    uint32_t ulane = (uint32_t)((kk * 64 + 32 * wx + li) * 16);
    auto load_A = [&](int ch, int s_) {
        const uint32_t ub = (uint32_t)__builtin_amdgcn_readfirstlane((mt * p.nchunks + ch) * (US * 4) + gpos(s_) * 2048);
        asm volatile("" : "+v"(ulane));   // four adjacent dword loads from one lane offset merge into one of 16 bytes
        A[s_].x = buf_ld(ru, ulane, ub);
        A[s_].y = buf_ld(ru, ulane + 4, ub);
        A[s_].z = buf_ld(ru, ulane + 8, ub);
        A[s_].w = buf_ld(ru, ulane + 12, ub);
    };
    auto load_patch = [&](int ch) {
        // The chunk's first input layer goes into the base of the resource (scalar arithmetic), not into the
        // uniform offset of the loads: the hardware checks only the lane offset against the size, so a run that
        // ends past the last row of the last input layer of the last image is cut off exactly at the end of `in`.
        const uint32_t so = (uint32_t)__builtin_amdgcn_readfirstlane(ch * CC * p.HW) * ESZ;
        const rsrc_t rxc = make_rsrc((const char *)p.in + so, p.in_bytes - so);
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            asm volatile("" : "+v"(xrow[a]));   // keeps the column steps immediates, so the run is one load
            dpatch[4 * a] = buf_ld_in<TIN>(rxc, xcol0[a], 0u);
#pragma unroll
            for (int b = 1; b < 4; ++b) dpatch[4 * a + b] = buf_ld_in<TIN>(rxc, xrow[a] + (b - 1) * ESZ, 0u);
        }
    };
    auto store_V = [&](float *img) {
        // V = B^T d B
        float rr[4][4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            rr[0][b] = dpatch[0 + b] - dpatch[8 + b];
            rr[1][b] = dpatch[4 + b] + dpatch[8 + b];
            rr[2][b] = dpatch[8 + b] - dpatch[4 + b];
            rr[3][b] = dpatch[4 + b] - dpatch[12 + b];
        }
        float *vs = img + vdst;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const float r2 = c2ok ? rr[a][2] : 0.f;   // columns 0 (zero-filled by the range check) and 1 are always real
            const float r3 = c3ok ? rr[a][3] : 0.f;
            vs[(4 * a + 0) * (2 * BT * 4)] = rr[a][0] - r2;
            vs[(4 * a + 1) * (2 * BT * 4)] = rr[a][1] + r2;
            vs[(4 * a + 2) * (2 * BT * 4)] = r2 - rr[a][1];
            vs[(4 * a + 3) * (2 * BT * 4)] = rr[a][1] - r3;
        }
    };

    // The accumulators start from the first MFMA of the first chunk, which takes a constant
    // zero as its addend, except grid position (1, 1): that one enters all four outputs of a
    // tile with weight +1, so starting it from the bias adds the bias to every pixel.
    const int mw = m0 + wx * 32;                 // uniform: first layer this wavefront handles
    const int lrow = M::row_lane(lane);
    Acc acc[8], start11;
    if (p.b && pr == 0) {
        const rsrc_t rb = make_rsrc(p.b, (uint32_t)p.Cout * 4u);   // layers past Cout read zero
#pragma unroll
        for (int q = 0; q < 16; ++q) start11[q] = buf_ld(rb, (uint32_t)((mw + M::row_reg(q) + lrow) * 4), 0u);
    } else {
#pragma unroll
        for (int q = 0; q < 16; ++q) start11[q] = 0.f;
    }

    // per-lane B operand offsets within a V image: V[xi][kk][li][0..3]; [g]: offset such that accumulator s
    // (row g = s / 4 of the wavefront's order) reads at vbo[g] + s * stride
    int vbo[2];
    vbo[0] = 12 * pr * (2 * BT * 4) + kk * (BT * 4) + li * 4;
    vbo[1] = vbo[0] - 8 * pr * (2 * BT * 4);
    // Multiplies chunk ch out of the V image img; reload: fetch the A operands of chunk ch + 1 into the registers
    // of each pair of positions as soon as its MFMAs have been issued (a whole chunk ahead of their use).
    auto compute_chunk = [&](auto first_chunk, const float *img, const bool reload, const int ch) {
        constexpr bool FIRST = decltype(first_chunk)::value;
        // two grid positions at a time, their MFMAs interleaved: consecutive MFMAs never
        // wait for each other's accumulator
        f32x4 b[4];
#pragma unroll
        for (int e = 0; e < 2; ++e) b[e] = *(const f32x4 *)(img + vbo[0] + e * (2 * BT * 4));
#pragma unroll
        for (int s = 0; s < 8; s += 2) {
            const int cur2 = s & 2, nxt2 = cur2 ^ 2;
            if (s + 2 < 8) {
#pragma unroll
                for (int e = 0; e < 2; ++e) b[nxt2 + e] = *(const f32x4 *)(img + vbo[(s + 2 + e) / 4] + (s + 2 + e) * (2 * BT * 4));
            }
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (FIRST) {
                // grid position (1, 1) is accumulator 5 of the wavefronts with pr = 0; for pr = 1
                // start11 is zero like the others
                Acc zero;
#pragma unroll
                for (int q = 0; q < 16; ++q) zero[q] = 0.f;
                acc[s] = M::run(A[s].x, b[cur2].x, zero);
                acc[s + 1] = M::run(A[s + 1].x, b[cur2 + 1].x, s + 1 == 5 ? start11 : zero);
            } else {
                acc[s] = M::run(A[s].x, b[cur2].x, acc[s]);
                acc[s + 1] = M::run(A[s + 1].x, b[cur2 + 1].x, acc[s + 1]);
            }
            acc[s] = M::run(A[s].y, b[cur2].y, acc[s]);
            acc[s + 1] = M::run(A[s + 1].y, b[cur2 + 1].y, acc[s + 1]);
            acc[s] = M::run(A[s].z, b[cur2].z, acc[s]);
            acc[s + 1] = M::run(A[s + 1].z, b[cur2 + 1].z, acc[s + 1]);
            acc[s] = M::run(A[s].w, b[cur2].w, acc[s]);
            acc[s + 1] = M::run(A[s + 1].w, b[cur2 + 1].w, acc[s + 1]);
            __builtin_amdgcn_sched_barrier(0);
            if (reload) {
                load_A(ch + 1, s);
                load_A(ch + 1, s + 1);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop ---------------------------------------------------------------------------
    // Chunk ch is multiplied out of V image ch & 1 while chunk ch + 1 is written into the other one: one barrier
    // per chunk, and no phase in which a workgroup only stages.  (With one image and the kernels staged through
    // LDS as well, a quarter of the time went into such phases: the two workgroups of a CU fall into step, since
    // the one behind gets the matrix pipe to itself and catches up, and then both stage at once.)
    load_patch(0);
#pragma unroll
    for (int s = 0; s < 8; ++s) load_A(0, s);
    store_V(lds);
    if (p.nchunks > 1) load_patch(1);
    __syncthreads();
    for (int ch = 0; ch < p.nchunks; ++ch) {
        const bool more = ch + 1 < p.nchunks;
        float *cur = lds + (ch & 1) * VS, *oth = lds + ((ch & 1) ^ 1) * VS;
        if (more) {
            store_V(oth);                                    // the patches of chunk ch + 1, loaded a chunk ago
            if (ch + 2 < p.nchunks) load_patch(ch + 2);
        }
        if (ch == 0) compute_chunk(std::true_type{}, cur, more, ch);
        else compute_chunk(std::false_type{}, cur, more, ch);
        __syncthreads();               // image ch & 1 has been read by all, image (ch + 1) & 1 written by all
    }

    // ---- output transform -------------------------------------------------------------------
    // acc[4g + s] is column s of the wavefront's g-th grid row (rows 0, 1 for pr = 0; rows 3, 2 for pr = 1).
    // Folding a row with A gives
    //   z(row)[0] = m0 + m1 + m2,   z(row)[1] = m1 - m2 - m3,
    // and the output rows are  Y[0] = z(0) + z(1) + z(2),  Y[1] = z(1) - z(2) - z(3).
    // pr = 0 keeps z(0) + z(1) for Y[0] and hands z(1), its second row, to its partner;
    // pr = 1 keeps -z(3) - z(2) for Y[1] and hands z(2), its second row, over.
    // Exchange area: [wavefront][zz][register][lane]; the images are free by now.
    constexpr int ZQ = 16 * 64;
    static_assert(4 * 2 * ZQ <= 2 * VS, "exchange area must fit the two V images");
    // keep[zz] = z(first row)[zz] + z(second row)[zz]; its sign (pr = 1: minus) goes into the
    // final multiply-add.  The vector-ALU work here and below is kept minimal: it cannot
    // overlap with the MFMAs of the workgroup sharing the SIMDs.
    Acc keep[2];
    {
        float *z = lds + wv * 2 * ZQ + lane;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const float z0a = acc[0][q] + acc[1][q] + acc[2][q], z1a = acc[1][q] - acc[2][q] - acc[3][q];
            const float z0b = acc[4][q] + acc[5][q] + acc[6][q], z1b = acc[5][q] - acc[6][q] - acc[7][q];
            keep[0][q] = z0a + z0b;
            keep[1][q] = z1a + z1b;
            z[q * 64] = z0b;
            z[ZQ + q * 64] = z1b;
        }
    }
    __syncthreads();
    if (mw >= p.Cout) continue;
    const float sg = pr ? -1.f : 1.f;
    const rsrc_t rout = make_rsrc(p.out, p.out_bytes);
    const uint32_t hs = (uint32_t)p.HoWo * 4u;
    // this wavefront writes output row pr of its tiles: pixels (2ty + pr, 2tx) and (.., 2tx + 1)
    uint32_t o2, o1;   // lane offsets for a tile with both columns inside the image / only the first
    {
        const int tg = t0 + li, tgc = min(tg, p.T - 1);
        const int n = fdiv(tgc, p.dTXY), rem = tgc - n * p.TXY;
        const int ty = fdiv(rem, p.dTX), tx = rem - ty * p.TX;
        const int oh = 2 * ty + pr, ow = 2 * tx;
        const bool ok = tg < p.T && oh < p.Ho;
        const uint32_t o = (uint32_t)(((n * p.ldc + p.coff + lrow) * p.HoWo + oh * p.Wo + ow) * 4);
        o2 = ok && ow + 1 < p.Wo ? o : kOob;
        o1 = ok && ow + 1 >= p.Wo ? o : kOob;
    }
    // all LDS reads first, so that their latency is paid once and not per output register
    const float *zr = lds + (wv ^ 1) * 2 * ZQ + lane;
    Acc zin[2];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        zin[0][q] = zr[q * 64];
        zin[1][q] = zr[ZQ + q * 64];
    }
    __builtin_amdgcn_sched_barrier(0);
    // then all arithmetic, then all stores: a run of pure memory instructions proceeds while
    // the other workgroup's MFMAs occupy the SIMD, a run mixed with vector-ALU work does not
    const float lowest = p.relu ? 0.f : -__builtin_inff();
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        zin[0][q] = fmaxf(__builtin_fmaf(sg, keep[0][q], zin[0][q]), lowest);
        zin[1][q] = fmaxf(__builtin_fmaf(sg, keep[1][q], zin[1][q]), lowest);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const uint32_t so = (uint32_t)__builtin_amdgcn_readfirstlane(mw + M::row_reg(q)) * hs;
        buf_st2(rout, o2, so, zin[0][q], zin[1][q]);
    }
    // tiles cut by the right edge (odd widths) have one column: only their lanes take part, so that the memory
    // pipe is not kept busy by sixteen instructions whose lanes are nearly all turned away
    if (o1 != kOob) {
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const uint32_t so = (uint32_t)__builtin_amdgcn_readfirstlane(mw + M::row_reg(q)) * hs;
            buf_st(rout, o1, so, zin[0][q]);
        }
    }
    }   // tiles of this workgroup
}

template <typename TIN>
__global__ __launch_bounds__(256, 2) void conv_wino_kernel(const KParams p)
{
    conv_wino_tiles<TIN>(p, (int)blockIdx.x, (int)gridDim.x);
}

// Both expands of a fire layer in one launch at large batches: the first wino_blocks workgroups are the
// persistent workgroups of the minimal-filtering expand3x3 (p3), the others one tile each of the expand1x1 (p1)
// in the tiling <BM, BN, WM, WN, MT, CC>.  The two write different layers of one tensor and read the same map.
// expand3x3 is bound by the matrix cores and its persistent workgroups finish at different times (at batch 64
// the layers of this network give a CU 6.1 tile blocks on average, so some CUs take seven and most six);
// expand1x1 is bound by its stores.  Its workgroups come last in the grid, so they are placed as the others
// retire and fill the CUs that would idle until the launch ends -- without the cost of a second stream.
template <int BM, int BN, int WM, int WN, int MT, int CC>
__global__ __launch_bounds__(256, 2) void expand_pair_kernel(const KParams p3, const KParams p1, const int wino_blocks)
{
    static_assert(WM * WN == 4, "both parts run with four wavefronts");
    if ((int)blockIdx.x < wino_blocks) conv_wino_tiles<float>(p3, (int)blockIdx.x, wino_blocks);
    else conv_mfma_tile<float, 1, 1, BM, BN, WM, WN, MT, CC, 0, false>(p1, (int)blockIdx.x - wino_blocks);
}

}  // namespace mfma
}  // namespace sq
