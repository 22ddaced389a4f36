// conv1-type layer on the fp32 matrix cores: 7x7 kernels, stride 2, three input layers,
// at most 96 output layers (section "Convolutional Neural Networks": the first layer of
// the network reads the 224 x 224 RGB image).
//
// Why it has its own kernel.  The contraction length is 3*49 = 147, which the generic
// kernel can only cover by padding the three input layers to four (196, a third of the
// MFMA work wasted).  Here the two k-values of each v_mfma_f32_32x32x2_f32 are chosen so
// that the LDS offset between the pair is a per-lane constant and the one spare slot
// carries the bias (148 = 74 MFMA steps):
//     steps  0..48   tap (i,j) of input layer 0   with the same tap of input layer 1
//     steps 49..69   tap (i,j), i<3, of layer 2   with tap (i+3, j) of layer 2
//     steps 70..72   tap (6,j), j in {0,1,4}, of layer 2 with tap (6, j+2) of layer 2
//     step  73       tap (6,5) of layer 2         with bias[m] * 1.0
// The kernels are stored in LDS in exactly that order (slot 2*step + pair member).
//
// Execution model.  fp32 MFMA shares the SIMD with ordinary vector instructions (they do
// not overlap), and a workgroup barrier per tile keeps all wavefronts in the same phase,
// so here each wavefront is autonomous after the kernels are staged once per workgroup:
//   * a wavefront owns tiles of 2 x 16 output pixels (one 32-wide MFMA pixel block, all
//     96 layers: 74 x 3 MFMAs) and walks over them with a fixed stride;
//   * it stages the 9 x 37 x 3 input patch of its next tile into its own double-buffered
//     LDS area (global loads before the MFMA loop, LDS writes after it), columns
//     de-interleaved into even | odd so that the stride-2 reads are conflict free;
//     every LDS offset of the MFMA loop is a compile-time constant;
//   * results are kept in a second accumulator set and stored, one store per MFMA step,
//     during the MFMA loop of the following tile;
//   * the bias comes out of the contraction and ReLU is the only vector work per result.
//
// Column-pooled form (CP; the max pooling behind conv1 split between this kernel and the squeeze layer that
// follows, see ColPool).  The 16 pixels of a tile row sit in the 16 lanes of a DPP row, so the maximum over columns
// c, c+1, c+2 is two v_max with a row shift (lanes past the row read zero; the ReLU is left to the reader of the map).
// Even lanes then hold the eight pooled columns of the tile and store them to the column-pooled map (tile cb of a row
// at positions 9 cb .. 9 cb + 7); the eighth lacks the first column of the next tile, which that tile's lane 0
// writes, unpooled, into the seam slot between the two (position 9 cb - 1 of its own row).
#include <type_traits>

#include "conv_mfma_common.h"

namespace sq {
namespace mfma {
namespace {

constexpr int kKS = 7, kS = 2, kKK = 49, kK = 147, kLDK = 149;
constexpr int kTR = kConv7TileRows, kTC = kConv7TileCols;
constexpr int kPR = (kTR - 1) * kS + kKS;      // 9 patch rows
constexpr int kPC = (kTC - 1) * kS + kKS;      // 37 patch columns
constexpr int kHalf = (kPC + 1) / 2;           // even columns first (19), then the odd ones
constexpr int kLWs = 40;                       // LDS row stride: the two pixel rows of a tile on disjoint banks
constexpr int kPlane = 416;                    // >= 9*40, = 32 (mod 64): the two k-halves on disjoint banks
constexpr int kOne = 3 * kPlane;               // word holding 1.0 (multiplier of the bias slot)
constexpr int kXbuf = 3 * kPlane + 32;         // floats per patch buffer
// LDS floats of the kernels of 32*TM output layers (padded: the tile counter lives in the padding)
constexpr int ws_floats(int TM) { return 32 * TM * kLDK + 32 - (32 * TM * kLDK) % 32; }
static_assert(kPR * kLWs <= kPlane && kPC <= kLWs, "patch plane");

// position of patch column c inside a row: even columns, then odd columns
__host__ __device__ constexpr int col_slot(int c) { return (c & 1) * kHalf + (c >> 1); }

// LDS slot of kernel value k = (c, i, j) in the pairing order above.
__device__ __forceinline__ int pair_slot(int k)
{
    const int c = k / kKK, tap = k - c * kKK;
    if (c < 2) return 2 * tap + c;
    const int i = tap / kKS, j = tap - i * kKS;
    if (i < 3) return 2 * (49 + tap);
    if (i < 6) return 2 * (49 + tap - 21) + 1;
    switch (j) {
        case 0: return 140;
        case 2: return 141;
        case 1: return 142;
        case 3: return 143;
        case 4: return 144;
        case 6: return 145;
        default: return 146;  // j == 5, paired with the bias
    }
}

// B-operand LDS offset of MFMA step s relative to the lane's base (compile-time)
__host__ __device__ constexpr int step_offset(int s)
{
    if (s < 49) return (s / 7) * kLWs + col_slot(s % 7);
    if (s < 70) return ((s - 49) / 7) * kLWs + col_slot((s - 49) % 7);
    if (s == 70) return col_slot(0);
    if (s == 71) return col_slot(1);
    return col_slot(4);  // s == 72; step 73 has its own per-lane address
}

// FULL: the layer has exactly 96 output layers, so no store needs a layer test.
// TM: blocks of 32 output layers a workgroup computes (3 = all 96; 1 = blockIdx.y picks one block, which
// triples the number of wavefronts and cuts the MFMA chain of a tile to a third -- for small batches,
// where there are too few tiles to fill the GPU and a pass is bound by the latency of each launch).
// TIN: float, or uint16_t = bfloat16 input and kernels, widened to fp32 while staged.
template <typename TIN, int NW, bool FULL, int MINW, int TM, bool CP = false>
__global__ __launch_bounds__(NW * 64, MINW) void conv7s2c3_kernel(const KParams p)
{
    static_assert(!CP || (FULL && sizeof(TIN) == 4), "the column-pooled form is for fp32 and 96 layers");
    constexpr int kTM = TM, kBM = 32 * TM, kWsFloats = ws_floats(TM);
    const int m0 = (int)blockIdx.y * kBM;          // first output layer of this workgroup
    constexpr int ESZ = (int)sizeof(TIN);
    using M = Mfma<32>;
    using Acc = typename M::Acc;
    constexpr int NT = NW * 64;

    extern __shared__ float smem[];
    float *const Ws = smem;
    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    float *const Xw = smem + kWsFloats + wv * (2 * kXbuf);   // this wavefront's two patch buffers
    const int li = lane & 31, kk = lane >> 5;

    // ---- kernels (pairing order) and bias, once per workgroup ---------------------------
    // all loads are issued before the first use so their latencies overlap
    {
        constexpr int WR = (kBM * kK + NT - 1) / NT;
        const rsrc_t rw = make_rsrc(p.w, p.w_bytes);   // rows beyond Cout read zero
        float wv_[WR];
#pragma unroll
        for (int r = 0; r < WR; ++r) {
            const int e = t + NT * r;
            wv_[r] = buf_ld_in<TIN>(rw, e < kBM * kK ? (uint32_t)((m0 * kK + e) * ESZ) : kOob, 0);
        }
#pragma unroll
        for (int r = 0; r < WR; ++r) {
            const int e = t + NT * r;
            const int m = e / kK, k = e - m * kK;
            if (e < kBM * kK) Ws[m * kLDK + pair_slot(k)] = wv_[r];
        }
    }
    if (t < kBM) {
        Ws[t * kLDK + 147] = (p.b && m0 + t < p.Cout) ? p.b[m0 + t] : 0.f;
        Ws[t * kLDK + 148] = 0.f;
    }
    if (lane < 2) Xw[lane * kXbuf + kOne] = 1.0f;
    int *const next_tile = reinterpret_cast<int *>(smem + kBM * kLDK + 8);   // in the padding after the kernels
    if (t == 0) *next_tile = 0;
    __syncthreads();   // the only workgroup barrier

    // ---- loop-invariant per-lane LDS offsets ---------------------------------------------
    int aoff[kTM];
#pragma unroll
    for (int x = 0; x < kTM; ++x) aoff[x] = (x * 32 + li) * kLDK + kk;
    const int prow = li >> 4, pcol = li & 15;                 // this lane's pixel inside the tile
    const int lbase = prow * kS * kLWs + pcol;                // even/odd split makes the column stride 1
    const int b1 = lbase + kk * kPlane;
    const int b2 = lbase + 2 * kPlane + kk * 3 * kLWs;
    const int b3 = lbase + 2 * kPlane + 6 * kLWs + kk;
    const int b4 = kk ? kOne : lbase + 2 * kPlane + 6 * kLWs + col_slot(5);
    const int xdst = col_slot(lane < kPC ? lane : 0);        // patch column staged by this lane

    const int tiles_per_image = p.RG * p.CB;
    const int ntiles = p.N * tiles_per_image;
    const uint32_t hs1 = (uint32_t)((CP ? p.Ho * p.cpRS : p.HoWo) * 4);   // layer stride of the map written

    // tile -> image n, first output row oh0, first output column ow0 (all uniform)
    // (readfirstlane tells the compiler these are wavefront-uniform, so all row arithmetic
    // below runs on the scalar unit)
    auto decode = [&](int tile_, int &n, int &oh0, int &ow0) {
        const int tile = __builtin_amdgcn_readfirstlane(tile_);
        n = fdiv(tile, p.dMtiles);               // dMtiles divides by tiles_per_image here
        const int rem = tile - n * tiles_per_image;
        const int rg = fdiv(rem, p.dCB);
        n = __builtin_amdgcn_readfirstlane(n);
        oh0 = __builtin_amdgcn_readfirstlane(rg * kTR);
        ow0 = __builtin_amdgcn_readfirstlane((rem - rg * p.CB) * kTC);
    };

    const rsrc_t rin = make_rsrc(p.in, p.in_bytes), rout = make_rsrc(p.out, p.out_bytes);

    float xreg[3 * kPR];
    auto load_patch = [&](int tile) {
        int n, oh0, ow0;
        decode(tile, n, oh0, ow0);
        const int ih0 = oh0 * kS - p.P, iw = ow0 * kS - p.P + lane;
        // columns outside the image (and lanes beyond the patch width) read zero through the
        // buffer range check; rows outside the image are skipped by a uniform branch
        const uint32_t coff = (lane < kPC && iw >= 0 && iw < p.W) ? (uint32_t)(iw * ESZ) : kOob;
#pragma unroll
        for (int r = 0; r < kPR; ++r) {
            const int ih = ih0 + r;                                   // uniform
            if (ih >= 0 && ih < p.H) {
                const uint32_t row = (uint32_t)((n * 3 * p.H + ih) * p.W) * (uint32_t)ESZ;
#pragma unroll
                for (int c = 0; c < 3; ++c) xreg[c * kPR + r] = buf_ld_in<TIN>(rin, coff, row + (uint32_t)c * (uint32_t)p.HW * (uint32_t)ESZ);
            } else {
#pragma unroll
                for (int c = 0; c < 3; ++c) xreg[c * kPR + r] = 0.f;
            }
        }
    };
    auto store_patch = [&](int buf) {
        float *xs = Xw + buf * kXbuf;
        if (lane < kPC) {
#pragma unroll
            for (int r = 0; r < kPR; ++r)
#pragma unroll
                for (int c = 0; c < 3; ++c) xs[c * kPlane + r * kLWs + xdst] = xreg[c * kPR + r];
        }
    };
    // lane byte offset of this lane's output pixel; pixels outside the image get an offset the
    // buffer range check rejects, so their stores vanish.  The layer part is a uniform offset.
    auto out_offset = [&](int tile) -> uint32_t {
        int n, oh0, ow0;
        decode(tile, n, oh0, ow0);
        const int oh = oh0 + prow, ow = ow0 + pcol;
        if constexpr (CP) {
            // even lanes: pooled column j = ow / 2 of row oh, at position j + j / 8 (a seam slot after every eighth)
            const int j = ow >> 1;
            const uint32_t off = (uint32_t)((((n * p.ldc + p.coff + M::row_lane(lane)) * p.Ho + oh) * p.cpRS + j + (j >> 3)) * 4);
            return (oh < p.Ho && !(pcol & 1) && j < p.cpWp) ? off : kOob;
        }
        const uint32_t off = (uint32_t)(((n * p.ldc + p.coff + M::row_lane(lane)) * p.HoWo + oh * p.Wo + ow) * 4);
        return (oh < p.Ho && ow < p.Wo) ? off : kOob;
    };
    // seam slot of this lane: the one before the tile's first pooled column, written by the lanes of the tile's
    // first column (the first tile of a row has none)
    auto seam_offset = [&](int tile) -> uint32_t {
        int n, oh0, ow0;
        decode(tile, n, oh0, ow0);
        const int oh = oh0 + prow, j = ow0 >> 1;
        const uint32_t off = (uint32_t)((((n * p.ldc + p.coff + M::row_lane(lane)) * p.Ho + oh) * p.cpRS + j + (j >> 3) - 1) * 4);
        return (pcol == 0 && ow0 > 0 && oh < p.Ho) ? off : kOob;
    };
    // one result register of a finished tile: the plain value, or its column maximum plus the seam value
    auto put = [&](uint32_t off, uint32_t soff, int mu, float val) {
        if constexpr (CP) {
            const float u = fmaxf(fmaxf(val, row_shl<1>(val)), row_shl<2>(val));
            buf_st(rout, off, (uint32_t)mu * hs1, u);
            buf_st(rout, soff, (uint32_t)mu * hs1, val);
        } else {
            buf_st(rout, off, (uint32_t)mu * hs1, val);
        }
    };

    // What is left to store of a finished tile: lane offsets of its layer blocks (kOob = block not computed, or
    // nothing to store yet) and of their seam slots (CP).  Where block 0 of the accumulators holds another layer block
    // than the first, the difference is part of the lane offset, so that the scalar offset of every store stays a
    // compile-time multiple of the layer stride (computed next to the store it would cost wait states each time).
    struct Pending {
        uint32_t off[kTM], soff[kTM];
    };
    // One tile: 74 MFMA steps into NB of the accumulators (NB = kTM: all layer blocks, A operands at aoff[];
    // NB = 1: the one block whose A operands start abase floats behind aoff[0], into acc[0]), with the previous
    // tile's results (`prev`, already ReLU'd) stored one per MFMA step at the walking byte offsets of `pend`.
    auto tile_mfma = [&](auto nb_tag, int buf, Acc (&acc)[kTM], int abase, const Acc (&prev)[kTM], const Pending &pend, int pend_mbase) {
        constexpr int NB = decltype(nb_tag)::value;
        const float *xs = Xw + buf * kXbuf;
        const float *wsb = Ws + abase;
        auto b_read = [&](int s) -> float {
            if (s == 73) return xs[b4];
            const int base = s < 49 ? b1 : s < 70 ? b2 : b3;
            return xs[base + step_offset(s)];
        };
        float av[2][NB], bv[2];
        auto fetch = [&](int s, float *a, float &b) {
#pragma unroll
            for (int x = 0; x < NB; ++x) a[x] = wsb[aoff[x] + 2 * s];
            b = b_read(s);
        };
        fetch(0, av[0], bv[0]);
#pragma unroll
        for (int s = 0; s < 74; ++s) {
            if (s + 1 < 74) fetch(s + 1, av[(s + 1) & 1], bv[(s + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);  // reads of step s+1 stay ahead of the MFMAs of step s
#pragma unroll
            for (int x = 0; x < NB; ++x) {
                if (s == 0) {
                    Acc z;
#pragma unroll
                    for (int r = 0; r < 16; ++r) z[r] = 0.f;
                    acc[x] = M::run(av[0][x], bv[0], z);
                } else {
                    acc[x] = M::run(av[s & 1][x], bv[s & 1], acc[x]);
                }
            }
            if (s < 16 * kTM) {
                // layers come in groups of 8 (rows mu..mu+3 in the lower half-wave, +4 in the
                // upper), and Cout is a multiple of 8, so the layer test is uniform
                const int x = s / 16, r = s % 16;
                const int mu = m0 + x * 32 + M::row_reg(r);
                if (FULL || mu + pend_mbase < p.Cout) put(pend.off[x], pend.soff[x], mu, prev[x][r]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // (CP: no ReLU here -- the layer that reads the column-pooled map ends its maximum with a zero, and
        // max(relu(a), relu(b)) = relu(max(a, b)); the zeros a row shift brings in past a row's end vanish likewise)
        if (p.relu && !CP) {
#pragma unroll
            for (int x = 0; x < NB; ++x)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[x][r] = fmaxf(acc[x][r], 0.f);
        }
    };

    // The tiles of the workgroups of one XCD are one contiguous eighth of all tiles (neighbouring tiles share five
    // of their nine patch rows and meet in one L2); a workgroup takes every step-th of them.  Its wavefronts draw k
    // from a counter in LDS, so a wavefront that gets less of the SIMD (the hardware favours the
    // older one of two) simply takes fewer tiles and all finish together.  Every wavefront
    // leaves the loop as soon as its draw is past the last tile.  (Fewer than eight workgroups: plain striding.)
    //
    // The last round.  A workgroup's tiles are rarely a multiple of its wavefronts.  With all layer blocks in one
    // workgroup (kTM = 3) the tiles left over after the last full round are therefore dealt out by layer block, a
    // third of a tile per draw, where that shortens the round (up to five tiles left for eight wavefronts).  Measured
    // on the layer alone: 3-11 % faster at batches 2 to 48 (one to nine rounds per wavefront), nothing at batch 64
    // and above (98 tiles per workgroup = 12 1/4 rounds: there the wavefronts of a CU drift apart by more than a
    // tile over the launch, and the CUs among themselves, so the last tiles never were a round of their own).
    const bool by_xcd = gridDim.x >= 8;
    const XcdShare share = xcd_share((int)blockIdx.x, (int)gridDim.x, ntiles);
    int whole = 1 << 30;   // draws below this are whole tiles
    int parts = 0;         // draws from `whole` on: one layer block each, this many
    if (kTM == 3 && by_xcd && share.end > share.first) {
        const int cnt = (share.end - share.first + share.step - 1) / share.step;
        const int rem = cnt % NW;
        if (rem > 0 && (3 * rem + NW - 1) / NW < 3) {
            whole = cnt - rem;
            parts = 3 * rem;
        }
    }
    // -> tile (ntiles = none left) and layer block (-1 = all)
    auto draw = [&](int &part) -> int {
        int k = 0;
        if (lane == 0) k = atomicAdd(next_tile, 1);
        k = __builtin_amdgcn_readfirstlane(k);
        part = -1;
        if (!by_xcd) return (int)blockIdx.x + k * (int)gridDim.x;
        if (k >= whole) {
            const int j = k - whole;
            if (j >= parts) return ntiles;
            const int t3 = (j * 11) >> 5;   // j / 3 for j < 32
            part = j - 3 * t3;
            k = whole + t3;
        }
        const long long tl = (long long)share.first + (long long)k * share.step;
        return tl < share.end ? (int)tl : ntiles;
    };
    int part = -1;
    int tile = draw(part);
    if (tile >= ntiles) return;
    load_patch(tile);
    store_patch(0);

    Acc accA[kTM], accB[kTM];
#pragma unroll
    for (int x = 0; x < kTM; ++x)
#pragma unroll
        for (int r = 0; r < 16; ++r) accA[x][r] = accB[x][r] = 0.f;
    Pending pendA, pendB;   // nothing to store yet
#pragma unroll
    for (int x = 0; x < kTM; ++x) pendA.off[x] = pendA.soff[x] = pendB.off[x] = pendB.soff[x] = kOob;
    int mbaseA = 0, mbaseB = 0;   // first layer of accumulator block 0 (only the partial-layer test needs it)
    bool lastA = true;

    // the tile just computed, as its stores will want it
    auto pending_of = [&](int tile_, int part_, Pending &pd, int &mbase) {
        mbase = part_ < 0 ? 0 : part_ * 32;
        const uint32_t shift = (uint32_t)mbase * hs1;     // kOob + shift stays beyond every range
        const uint32_t o = out_offset(tile_) + shift;
        uint32_t so = kOob;
        if constexpr (CP) so = seam_offset(tile_) + shift;
#pragma unroll
        for (int x = 0; x < kTM; ++x) {
            const bool have = part_ < 0 || x == 0;
            pd.off[x] = have ? o : kOob;
            pd.soff[x] = have ? so : kOob;
        }
    };
    auto compute = [&](int buf, int part_, Acc (&acc)[kTM], const Acc (&prev)[kTM], const Pending &pend, int pend_mbase) {
        if (kTM > 1 && part_ >= 0) tile_mfma(std::integral_constant<int, 1>{}, buf, acc, part_ * 32 * kLDK, prev, pend, pend_mbase);
        else tile_mfma(std::integral_constant<int, kTM>{}, buf, acc, 0, prev, pend, pend_mbase);
    };

    // two tiles per trip: even tiles use patch buffer 0 and accumulators A, odd ones 1 and B
    while (true) {
        {
            int npart;
            const int next = draw(npart);
            const bool more = next < ntiles;
            if (more) load_patch(next);
            compute(0, part, accA, accB, pendB, mbaseB);
            pending_of(tile, part, pendA, mbaseA);
            lastA = true;
            if (!more) break;
            store_patch(1);
            tile = next; part = npart;
        }
        {
            int npart;
            const int next = draw(npart);
            const bool more = next < ntiles;
            if (more) load_patch(next);
            compute(1, part, accB, accA, pendA, mbaseA);
            pending_of(tile, part, pendB, mbaseB);
            lastA = false;
            if (!more) break;
            store_patch(0);
            tile = next; part = npart;
        }
    }
    // results of the last tile
    const Pending &pl = lastA ? pendA : pendB;
    const int mbl = lastA ? mbaseA : mbaseB;
#pragma unroll
    for (int x = 0; x < kTM; ++x)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int mu = m0 + x * 32 + M::row_reg(r);
            if (FULL || mu + mbl < p.Cout) put(pl.off[x], pl.soff[x], mu, lastA ? accA[x][r] : accB[x][r]);
        }
}

}  // namespace

KernelFn conv7s2c3_kernel_for(int NW, bool full, bool bf16, int TM, bool colpool)
{
    if (colpool) {
        if (!full || bf16) return nullptr;
        if (TM == 1) return NW == 4 ? conv7s2c3_kernel<float, 4, true, 2, 1, true> : nullptr;
        if (NW == 8) return conv7s2c3_kernel<float, 8, true, 1, 3, true>;
        if (NW == 4) return conv7s2c3_kernel<float, 4, true, 1, 3, true>;
        return nullptr;
    }
    if (TM == 1) {
        if (NW != 4) return nullptr;
        if (bf16) return full ? conv7s2c3_kernel<uint16_t, 4, true, 2, 1> : conv7s2c3_kernel<uint16_t, 4, false, 2, 1>;
        return full ? conv7s2c3_kernel<float, 4, true, 2, 1> : conv7s2c3_kernel<float, 4, false, 2, 1>;
    }
    if (bf16) {
        if (NW == 8) return full ? conv7s2c3_kernel<uint16_t, 8, true, 1, 3> : conv7s2c3_kernel<uint16_t, 8, false, 1, 3>;
        if (NW == 4) return full ? conv7s2c3_kernel<uint16_t, 4, true, 1, 3> : conv7s2c3_kernel<uint16_t, 4, false, 1, 3>;
        return nullptr;
    }
    if (NW == 8) return full ? conv7s2c3_kernel<float, 8, true, 1, 3> : conv7s2c3_kernel<float, 8, false, 1, 3>;
    if (NW == 4) return full ? conv7s2c3_kernel<float, 4, true, 1, 3> : conv7s2c3_kernel<float, 4, false, 1, 3>;
    return nullptr;
}

size_t conv7s2c3_lds_bytes(int NW, int TM) { return ((size_t)ws_floats(TM) + (size_t)NW * 2 * kXbuf) * sizeof(float); }

}  // namespace mfma
}  // namespace sq
