// 3x3 / stride 1 / pad 1 convolution in the minimal-filtering form F(2x2, 3x3) with autonomous
// wavefronts (internal).  Same mathematics as conv_wino_kernel.h (U = G g G^T, V = B^T d B,
// Y = A^T (sum_c U (.) V) A; section "Convolutional Neural Networks" defines the layer); what
// differs is how the work is cut.
//
// There a workgroup of four wavefronts shares one tile block: patches are transformed by all
// threads into an LDS image, every wavefront multiplies half of the grid positions, halves are
// exchanged through LDS for the output transform -- one barrier per chunk of input layers and two
// per tile block, and all work is dealt out in workgroup-sized pieces.  Counters on the network's
// fire layers showed the matrix pipe busy half of the time, a sixth spent in vector-ALU work and a
// third idle: waiting at those barriers, and in the last round of pieces that do not divide by
// the number of CUs.
//
// Here every wavefront works alone, as in the conv1 kernel:
//   * A persistent workgroup of eight wavefronts keeps the transformed kernels U of ONE block of
//     32 output layers (all input layers, all 16 grid positions) in LDS: Cin * 2 KB, staged once.
//   * A wavefront draws an item = 16 consecutive tiles (2x2 output pixels each) from a counter in
//     LDS and computes all 16 grid positions for 32 layers x 16 tiles with
//     v_mfma_f32_16x16x4_f32: 32 accumulators of 4 registers.  The k-dimension of one MFMA is
//     four consecutive input layers.
//   * The B operand never touches LDS: lane (tile j = lane % 16, k = lane / 16) loads the 4x4
//     patch of tile j in input layer 4*step + k, transforms it in registers and holds exactly the
//     sixteen values V[pos] that the sixteen MFMAs of this step want from this lane.
//   * The A operand comes from LDS, one 16-byte read per lane feeding four MFMAs.
//   * All sixteen positions of a (layer, tile) end up in the same lane, so the output transform
//     needs no exchange; bias enters through the start value of position (1,1).
//   * No barrier except when a workgroup moves on to another layer block.
// A workgroup's share of the work is a range of tile groups of one layer block (with fewer workgroups
// than layer blocks: several whole blocks); within it its wavefronts balance themselves.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

#include "conv_mfma_common.h"

namespace sq {
namespace mfma {

// The work of one persistent workgroup on one layer block: tile groups [lo, end) of block lbk.
// E1: the wavefront also computes the 1x1 convolution p.w1 (+ p.b1) of the same input for the same tiles and the
// same block of 32 layers, written to layers [p.coff1, p.coff1 + p.Cout1) -- the other expand of a fire layer
// (section "Convolutional Neural Networks": both expand layers read the squeeze result).  Its B operands are the
// four centre values of the patch, untransformed; its kernels sit in LDS beside U.
// CP: the results go out as a column-pooled map (the max pooling behind this layer split between this kernel and the
// squeeze layer that follows, see ColPool).  The sixteen tiles of an item sit in the sixteen lanes of a DPP row, so
// pooled column tx = max(both columns of tile tx, first column of tile tx + 1) takes one row shift per pixel row;
// lane 15 lacks its neighbour, whose item writes that column, unpooled, into the seam slot behind it.
template <typename TIN, bool E1, bool CP = false>
__device__ __forceinline__ void conv_wino_auto_items(const KParams &p, const int lbk, const int lo, const int end)
{
    static_assert(!CP || sizeof(TIN) == 4, "column-pooled maps come from fp32 layers");
    constexpr uint32_t ESZ = sizeof(TIN);
    using M = Mfma<16>;
    using Acc = M::Acc;
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int KS = p.nchunks;                               // steps of four input layers
    float *const w1s = lds + KS * kWinoAutoStep;            // [KS][64 lanes][2 row blocks] kernels of the 1x1 part
    int *const counter = reinterpret_cast<int *>(w1s + (E1 ? KS * 128 : 0));

    const int t = threadIdx.x, lane = t & 63;
    const int tj = lane & 15, tk = lane >> 4;

    const rsrc_t rout = make_rsrc(p.out, p.out_bytes);
    const uint32_t hs = (uint32_t)(CP ? p.Ho * p.cpRS : p.HoWo) * 4u;   // layer stride of the map written
    // CP: no ReLU here -- the layer that reads the column-pooled map ends its maximum with a zero, and
    // max(relu(a), relu(b)) = relu(max(a, b)); the zeros a row shift brings in at the end of a row vanish the same way
    const float lowest = p.relu && !CP ? 0.f : -__builtin_inff();

    {
        __syncthreads();                                    // everybody has left the previous block
        {
            // U of this layer block: KS * 8 KB, copied as it lies in memory
            const f32x4 *src = reinterpret_cast<const f32x4 *>(p.wu + (size_t)lbk * KS * kWinoAutoStep);
            f32x4 *dst = reinterpret_cast<f32x4 *>(lds);
            // eight loads in flight per thread before the first LDS write (one load at a time would pay the
            // memory latency once per 8 KB)
            constexpr int NT = kWinoAutoWaves * 64, UNR = 8;
            const int total = KS * (kWinoAutoStep / 4);     // a multiple of NT
            for (int base = t; base < total; base += UNR * NT) {
                f32x4 tmp[UNR];
#pragma unroll
                for (int u = 0; u < UNR; ++u)
                    if (base + u * NT < total) tmp[u] = src[base + u * NT];
#pragma unroll
                for (int u = 0; u < UNR; ++u)
                    if (base + u * NT < total) dst[base + u * NT] = tmp[u];
            }
            if constexpr (E1) {
                // thread -> layer t / 16 of the block, input layers t % 16, + 16, ...
                const int m = t >> 4;
                for (int c = t & 15; c < p.Cin; c += 16) {
                    const int mg = lbk * kWinoAutoLayers + m;
                    float wv = 0.f;
                    if (mg < p.Cout1) {
                        if constexpr (sizeof(TIN) == 2) wv = __builtin_bit_cast(float, (uint32_t)((const uint16_t *)p.w1)[mg * p.Cin + c] << 16);
                        else wv = p.w1[mg * p.Cin + c];
                    }
                    w1s[((c >> 2) * 64 + (c & 3) * 16 + (m & 15)) * 2 + (m >> 4)] = wv;
                }
            }
            if (t == 0) *counter = lo;
        }
        __syncthreads();

        // bias of this lane's eight layers: position (1,1) has weight +1 in all four pixels of a tile
        const int m0 = lbk * kWinoAutoLayers;
        Acc start11[2];
#pragma unroll
        for (int lb = 0; lb < 2; ++lb)
#pragma unroll
            for (int r = 0; r < 4; ++r) start11[lb][r] = p.b ? p.b[m0 + lb * 16 + 4 * tk + r] : 0.f;

        auto draw = [&]() -> int {
            int g = 0;
            if (lane == 0) g = atomicAdd(counter, 1);
            return __builtin_amdgcn_readfirstlane(g);
        };

        // Per-item lane state: patch offsets (rows of the 4x4 patch: first column on its own, then a 12-byte run),
        // right-edge flags, and the output offsets.
        struct Item {
            uint32_t xrow[4], xcol0[4];
            bool c2ok, c3ok;
            uint32_t o;                 // byte offset of output pixel (2ty, 2tx) in this lane's first layer
            bool ok0, ok1, two;         // rows 2ty, 2ty + 1 exist; column 2tx + 1 exists
            bool seam;                  // CP: this lane's first column goes into the seam slot before its position
        };
        auto setup = [&](int item, Item &it) {
            const int t0 = item * kWinoAutoTiles;
            const int tg = t0 + tj, tgc = min(tg, p.T - 1);
            const int n = fdiv(tgc, p.dTXY), rem = tgc - n * p.TXY;
            const int ty = fdiv(rem, p.dTX), tx = rem - ty * p.TX;
            const int ih0 = 2 * ty - 1, iw0 = 2 * tx - 1;
            const uint32_t base = (uint32_t)((n * p.Cin + tk) * p.HW + ih0 * p.W + iw0 + 1) * ESZ;
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const uint32_t bad = tg < p.T && (unsigned)(ih0 + a) < (unsigned)p.H ? 0u : kOob;
                it.xrow[a] = (base + (uint32_t)(a * p.W) * ESZ) | bad;
                it.xcol0[a] = (base + (uint32_t)(a * p.W) * ESZ - ESZ) | bad | (iw0 >= 0 ? 0u : kOob);
            }
            it.c2ok = iw0 + 2 < p.W;
            it.c3ok = iw0 + 3 < p.W;
            // output pixels (2ty + pr, 2tx) and (.., 2tx + 1); the lane's first layer goes into the lane offset
            const int oh = 2 * ty, ow = 2 * tx;
            if constexpr (CP) {
                // pooled column tx of rows 2ty, 2ty + 1 in the column-pooled map: its position counts the group ends
                // before it in this tile row (tgc is the slot number); the last tile of a row has no pooled column
                const int pos = tx + (tgc >> 4) - ((tgc - tx) >> 4);
                it.o = (uint32_t)((((n * p.ldc + p.coff + m0 + 4 * tk) * p.Ho + oh) * p.cpRS + pos) * 4);
                it.ok0 = tg < p.T && tx < p.cpWp;
                it.ok1 = it.ok0 && oh + 1 < p.Ho;
                it.two = oh + 1 < p.Ho;       // (here: the second row exists, for the seam store)
                it.seam = tj == 0 && tg < p.T && tx > 0;
            } else {
                it.o = (uint32_t)(((n * p.ldc + p.coff + m0 + 4 * tk) * p.HoWo + oh * p.Wo + ow) * 4);
                it.ok0 = tg < p.T;
                it.ok1 = tg < p.T && oh + 1 < p.Ho;
                it.two = ow + 1 < p.Wo;
            }
        };
        // Patch of this lane's (tile, input layer 4 * ks + k).  The step's first input layer goes into the base of
        // the resource (scalar arithmetic): the hardware checks only the lane offset against the size, so a run that
        // ends past the last row of the last input layer of the last image is cut off exactly at the end of `in`.
        // `real` = false describes zero bytes, so that every load returns zero and fetches nothing: the loads of a
        // step past the last one, or of an item that does not exist, are issued like all others, which keeps the
        // loop free of branches around loads (a value that is either loaded or kept needs copies on every trip).
        auto load_patch = [&](const Item &it, int ks, bool real, float (&d)[16]) {
            const uint32_t so = (uint32_t)__builtin_amdgcn_readfirstlane(real ? ks * 4 * p.HW : 0) * ESZ;
            const rsrc_t rx = make_rsrc((const char *)p.in + so, real ? p.in_bytes - so : 0u);
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                uint32_t row = it.xrow[a];
                asm volatile("" : "+v"(row));   // keeps the column steps immediates, so the run is one load
                d[4 * a] = buf_ld_in<TIN>(rx, it.xcol0[a], 0u);
#pragma unroll
                for (int b = 1; b < 4; ++b) d[4 * a + b] = buf_ld_in<TIN>(rx, row + (b - 1) * ESZ, 0u);
            }
        };
        // V = B^T d B; columns right of the image were read from the next row (or from behind the tensor) and are
        // replaced by zero with a select.
        auto transform = [&](const Item &it, const float (&d)[16], float (&v)[16]) {
            float rr[4][4];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                rr[0][b] = d[0 + b] - d[8 + b];
                rr[1][b] = d[4 + b] + d[8 + b];
                rr[2][b] = d[8 + b] - d[4 + b];
                rr[3][b] = d[4 + b] - d[12 + b];
            }
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const float r2 = it.c2ok ? rr[a][2] : 0.f;
                const float r3 = it.c3ok ? rr[a][3] : 0.f;
                v[4 * a + 0] = rr[a][0] - r2;
                v[4 * a + 1] = rr[a][1] + r2;
                v[4 * a + 2] = r2 - rr[a][1];
                v[4 * a + 3] = rr[a][1] - r3;
            }
        };

        Acc acc[16][2];
        Acc e[E1 ? 4 : 1][2];                                            // the 1x1 part: four pixels of a tile x two row blocks
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        const f32x2 *wa = reinterpret_cast<const f32x2 *>(w1s) + lane;   // A operands of the 1x1 part, step ks: wa[ks * 64]
        const f32x4 *ua = reinterpret_cast<const f32x4 *>(lds) + lane;    // quad q of the stream is ua[q * 64]
        // One step: sixteen positions x two row blocks.  The A quad of a position pair is read while the pair before is multiplied.
        // c4: the four centre values of the untransformed patch (the pixels of the tile), B operands of the 1x1 part;
        // bias1: its start values
        auto mfma_step = [&](auto first_step, int ks, const float (&v)[16], const float (&c4)[4], const Acc (&bias1)[2]) {
            constexpr bool FIRST = decltype(first_step)::value;
            const f32x4 *u = ua + ks * (8 * 64);
            f32x4 a[2];
            f32x2 a1 = {0.f, 0.f};
            if constexpr (E1) a1 = wa[ks * 64];
            a[0] = u[0];
#pragma unroll
            for (int pq = 0; pq < 8; ++pq) {
                if (pq + 1 < 8) a[(pq + 1) & 1] = u[(pq + 1) * 64];
                __builtin_amdgcn_sched_barrier(0);
                const f32x4 aq = a[pq & 1];
                if constexpr (FIRST) {
                    Acc zero = {0.f, 0.f, 0.f, 0.f};
                    acc[2 * pq][0] = M::run(aq.x, v[2 * pq], zero);
                    acc[2 * pq][1] = M::run(aq.y, v[2 * pq], zero);
                    acc[2 * pq + 1][0] = M::run(aq.z, v[2 * pq + 1], 2 * pq + 1 == 5 ? start11[0] : zero);
                    acc[2 * pq + 1][1] = M::run(aq.w, v[2 * pq + 1], 2 * pq + 1 == 5 ? start11[1] : zero);
                } else {
                    acc[2 * pq][0] = M::run(aq.x, v[2 * pq], acc[2 * pq][0]);
                    acc[2 * pq][1] = M::run(aq.y, v[2 * pq], acc[2 * pq][1]);
                    acc[2 * pq + 1][0] = M::run(aq.z, v[2 * pq + 1], acc[2 * pq + 1][0]);
                    acc[2 * pq + 1][1] = M::run(aq.w, v[2 * pq + 1], acc[2 * pq + 1][1]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (E1) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    e[q][0] = M::run(a1.x, c4[q], FIRST ? bias1[0] : e[q][0]);
                    e[q][1] = M::run(a1.y, c4[q], FIRST ? bias1[1] : e[q][1]);
                }
            }
        };

        // ---- item loop ----------------------------------------------------------------------------------
        int item = draw();
        if (item < end) {
            Item cur, nxt;
            float pa[16], pb[E1 ? 1 : 16], v[16], c4[4] = {0.f, 0.f, 0.f, 0.f};
            Acc bias1[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
            setup(item, cur);
            load_patch(cur, 0, true, pa);
            if constexpr (!E1) load_patch(cur, 1, true, pb);        // KS >= 2
            while (true) {
                const int next = draw();
                const bool more = next < end;
                if constexpr (E1) {
                    // One patch buffer: a step's patch is transformed (and its centre copied for the 1x1 part), then the
                    // buffer takes the loads of the next step, which fly during this step's forty MFMAs.
#pragma unroll
                    for (int lb = 0; lb < 2; ++lb)
#pragma unroll
                        for (int r = 0; r < 4; ++r) bias1[lb][r] = p.b1 ? p.b1[m0 + lb * 16 + 4 * tk + r] : 0.f;
                    transform(cur, pa, v);
                    c4[0] = pa[5]; c4[1] = pa[6]; c4[2] = pa[9]; c4[3] = pa[10];
                    load_patch(cur, 1, true, pa);
                    mfma_step(std::true_type{}, 0, v, c4, bias1);
                    for (int ks = 1; ks < KS; ++ks) {
                        transform(cur, pa, v);
                        c4[0] = pa[5]; c4[1] = pa[6]; c4[2] = pa[9]; c4[3] = pa[10];
                        load_patch(cur, ks + 1, ks + 1 < KS, pa);
                        mfma_step(std::false_type{}, ks, v, c4, bias1);
                    }
                    setup(more ? next : 0, nxt);
                    load_patch(nxt, 0, more, pa);
                } else {
                    transform(cur, pa, v);
                    // steps in pairs: patches of step ks + 2 are requested while step ks is multiplied
                    load_patch(cur, 2, 2 < KS, pa);
                    mfma_step(std::true_type{}, 0, v, c4, bias1);
                    transform(cur, pb, v);
                    load_patch(cur, 3, 3 < KS, pb);
                    mfma_step(std::false_type{}, 1, v, c4, bias1);
                    for (int ks = 2; ks < KS; ks += 2) {
                        transform(cur, pa, v);
                        load_patch(cur, ks + 2, ks + 2 < KS, pa);
                        mfma_step(std::false_type{}, ks, v, c4, bias1);
                        transform(cur, pb, v);
                        load_patch(cur, ks + 3, ks + 3 < KS, pb);
                        mfma_step(std::false_type{}, ks + 1, v, c4, bias1);
                    }
                    // the next item's first patches fly during the output transform and the stores (past the last item:
                    // the offsets of the first tile group, through a descriptor of zero bytes)
                    setup(more ? next : 0, nxt);
                    load_patch(nxt, 0, more, pa);
                    load_patch(nxt, 1, more, pb);
                }
                // ---- output transform: Y = A^T M A per (layer, tile), all sixteen positions in this lane -----
                // lane offsets of the two pixel rows: both columns (8-byte store) or, for tiles cut by the right edge
                // (odd widths), the first column only
                uint32_t o2[2], o1[2];
                o2[0] = !CP && cur.ok0 && cur.two ? cur.o : kOob;
                o2[1] = !CP && cur.ok1 && cur.two ? cur.o + (uint32_t)(p.Wo * 4) : kOob;
                o1[0] = cur.ok0 && (CP || !cur.two) ? cur.o : kOob;
                o1[1] = cur.ok1 && (CP || !cur.two) ? cur.o + (uint32_t)((CP ? p.cpRS : p.Wo) * 4) : kOob;
                // CP: the two pooled values of this lane's tile column, and lane 0's unpooled first column
                uint32_t os[2] = {kOob, kOob};
                if constexpr (CP) {
                    os[0] = cur.seam ? cur.o - 4u : kOob;
                    os[1] = cur.seam && cur.two ? cur.o - 4u + (uint32_t)(p.cpRS * 4) : kOob;
                }
                auto put_pooled = [&](uint32_t d, int layer, float y00, float y01, float y10, float y11) {
                    const float h0 = fmaxf(fmaxf(y00, y01), row_shl<1>(y00));
                    const float h1 = fmaxf(fmaxf(y10, y11), row_shl<1>(y10));
                    const uint32_t so = (uint32_t)__builtin_amdgcn_readfirstlane(layer) * hs;
                    buf_st(rout, o1[0] == kOob ? kOob : o1[0] + d, so, h0);
                    buf_st(rout, o1[1] == kOob ? kOob : o1[1] + d, so, h1);
                    buf_st(rout, os[0] == kOob ? kOob : os[0] + d, so, y00);
                    buf_st(rout, os[1] == kOob ? kOob : os[1] + d, so, y10);
                };
#pragma unroll
                for (int lb = 0; lb < 2; ++lb) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float z[4][2];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            z[i][0] = acc[4 * i][lb][r] + acc[4 * i + 1][lb][r] + acc[4 * i + 2][lb][r];
                            z[i][1] = acc[4 * i + 1][lb][r] - acc[4 * i + 2][lb][r] - acc[4 * i + 3][lb][r];
                        }
                        const float y00 = CP ? z[0][0] + z[1][0] + z[2][0] : fmaxf(z[0][0] + z[1][0] + z[2][0], lowest);
                        const float y01 = CP ? z[0][1] + z[1][1] + z[2][1] : fmaxf(z[0][1] + z[1][1] + z[2][1], lowest);
                        const float y10 = CP ? z[1][0] - z[2][0] - z[3][0] : fmaxf(z[1][0] - z[2][0] - z[3][0], lowest);
                        const float y11 = CP ? z[1][1] - z[2][1] - z[3][1] : fmaxf(z[1][1] - z[2][1] - z[3][1], lowest);
                        if constexpr (CP) {
                            put_pooled(0u, lb * 16 + r, y00, y01, y10, y11);
                        } else {
                            const uint32_t so = (uint32_t)__builtin_amdgcn_readfirstlane(lb * 16 + r) * hs;
                            buf_st2(rout, o2[0], so, y00, y01);
                            buf_st2(rout, o2[1], so, y10, y11);
                            buf_st(rout, o1[0], so, y00);
                            buf_st(rout, o1[1], so, y10);
                        }
                    }
                }
                if constexpr (E1) {
                    // ---- the 1x1 part: ReLU and stores, same pixels, layers [coff1 + m0, +32) ----
                    const uint32_t d1 = (uint32_t)(p.coff1 - p.coff) * hs;               // modulo 2^32, like the offsets
#pragma unroll
                    for (int lb = 0; lb < 2; ++lb) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const uint32_t so = (uint32_t)__builtin_amdgcn_readfirstlane(lb * 16 + r) * hs;
                            const float y00 = CP ? e[0][lb][r] : fmaxf(e[0][lb][r], lowest), y01 = CP ? e[1][lb][r] : fmaxf(e[1][lb][r], lowest);
                            const float y10 = CP ? e[2][lb][r] : fmaxf(e[2][lb][r], lowest), y11 = CP ? e[3][lb][r] : fmaxf(e[3][lb][r], lowest);
                            if constexpr (CP) {
                                put_pooled(d1, lb * 16 + r, y00, y01, y10, y11);
                                continue;
                            }
                            buf_st2(rout, o2[0] == kOob ? kOob : o2[0] + d1, so, y00, y01);
                            buf_st2(rout, o2[1] == kOob ? kOob : o2[1] + d1, so, y10, y11);
                            buf_st(rout, o1[0] == kOob ? kOob : o1[0] + d1, so, y00);
                            buf_st(rout, o1[1] == kOob ? kOob : o1[1] + d1, so, y10);
                        }
                    }
                }
                if (!more) break;
                cur = nxt;
                item = next;
            }
        }
    }
}

// The share of workgroup w of W: items are (layer block, tile group) pairs.  With at least as many workgroups as
// layer blocks every workgroup stays with one block (its U is staged once): the first p.wa_big blocks have
// p.wa_cnt + 1 workgroups each, the others p.wa_cnt, and the workgroups of a block split its tile groups evenly
// (quotients and remainders come from the host).  Workgroups are dealt to the eight XCDs in turn, so the k-th
// workgroup of every block is given a place on the same XCD (rank = position in the order XCD by XCD; block =
// rank mod blocks): the blocks that read the same stretch of the input then share one L2 instead of fetching it
// once per XCD.  With fewer workgroups than blocks each takes whole blocks w, w + W, ...
template <typename TIN, bool E1, bool CP = false>
__device__ __forceinline__ void conv_wino_auto_share(const KParams &p, const int w, const int W)
{
    const int nb = p.mtiles, G = p.ntiles;
    if (W >= nb) {
        const int rank = (W & 7) == 0 ? (w & 7) * (W >> 3) + (w >> 3) : w;
        const int even = nb * p.wa_cnt;   // ranks below this go round the blocks; the rest are the big blocks' last
        int blk, idx;
        if (rank < even) {
            idx = fdiv(rank, p.dMtiles); blk = rank - idx * nb;
        } else {
            blk = rank - even; idx = p.wa_cnt;
        }
        const int q = blk < p.wa_big ? p.wa_q1 : p.wa_q0, r = blk < p.wa_big ? p.wa_r1 : p.wa_r0;
        const int lo = idx * q + min(idx, r);
        conv_wino_auto_items<TIN, E1, CP>(p, __builtin_amdgcn_readfirstlane(blk), lo, lo + q + (idx < r ? 1 : 0));
    } else {
        for (int blk = w; blk < nb; blk += W) conv_wino_auto_items<TIN, E1, CP>(p, blk, 0, G);
    }
}

template <typename TIN>
__global__ __launch_bounds__(kWinoAutoWaves * 64, 1) void conv_wino_auto_kernel(const KParams p)
{
    conv_wino_auto_share<TIN, false>(p, (int)blockIdx.x, (int)gridDim.x);
}

// Both expands of a fire layer in one launch: every wavefront item is 32 layers x 16 tiles of the expand3x3 followed
// by the same layers and tiles of the expand1x1 (p.w1, p.b1, p.coff1; the number of layers is the same).
// CP: the pair writes a column-pooled map.
template <typename TIN, bool CP = false>
__global__ __launch_bounds__(kWinoAutoWaves * 64, 1) void expand_pair_auto_kernel(const KParams p, const KParams, const int)
{
    conv_wino_auto_share<TIN, true, CP>(p, (int)blockIdx.x, (int)gridDim.x);
}

}  // namespace mfma
}  // namespace sq
