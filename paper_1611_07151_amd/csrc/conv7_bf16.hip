// conv1-type layer of the reduced-precision path: 7x7 kernels, stride 2, three input
// layers, at most 96 output layers (section "Convolutional Neural Networks": the first
// layer reads the RGB image).  The image arrives as NCHW (fp32 or bfloat16); the result
// leaves as a blocked bfloat16 map [N][layers/8][Ho][Wo][8], the layout every later layer
// of this path reads, so nothing is re-ordered afterwards (sections "Data Reordering" and
// "Zero-overhead vectorization").
//
// Contraction on v_mfma_f32_32x32x16_bf16.  One k-group of eight values = the seven taps
// of one kernel row (input layer c, kernel row i) plus a zero: for output column ow these
// are the eight consecutive input pixels 2*ow - P .. 2*ow - P + 7 of image row 2*oh - P + i,
// i.e. 16 contiguous bytes of a bfloat16 copy of the image.  An MFMA takes two k-groups
// (lane halves), so the 21 (c, i) pairs need 11 MFMA steps (176 of which 147 are real).
//
// A workgroup of four wavefronts works on tiles of 8 output rows x 16 output columns; each
// wavefront owns two rows (one 32-pixel MFMA block) and all 96 layers (3 accumulators).
// The 21 x 37 x 3 input patch of a tile is converted to bfloat16 and staged in LDS by the
// whole workgroup; the patch of the next tile is fetched into registers before the MFMA
// loop and written to the other LDS buffer after it (one barrier per tile).  The packed
// kernels (33 KB) stay in LDS for the lifetime of the persistent workgroup.
#include "conv_mfma_common.h"

namespace sq {
namespace blocked {

using namespace mfma;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kTR = 8, kTC = 16;                 // output rows and columns per workgroup tile
constexpr int kPR = (kTR - 1) * 2 + 7;           // 21 patch rows per input layer
constexpr int kPC = (kTC - 1) * 2 + 7 + 1;       // 38 patch columns (37 used + the zero-weight tap)
constexpr int kPairs = kPC / 2;                  // 19 column pairs = dwords per patch row
constexpr int kRowDw = 20;                       // LDS row stride in dwords
constexpr int kPatchDw = 3 * kPR * kRowDw;       // 1260 dwords per patch buffer
constexpr int kSteps = 11;                       // MFMA steps: (c, i) pairs 2s and 2s + 1
constexpr int kWpElems = 3 * kSteps * 64;        // 16-byte elements of the packed kernels
constexpr int kThreads7 = 256;
constexpr int kLoads = (3 * kPR * kPairs + kThreads7 - 1) / kThreads7;   // column pairs per thread (5)

// [Cout][3][7][7] -> [3 blocks of 32 layers][11 steps][64 lanes][8]: lane l = layer 32*mb + l%32,
// (c, i) pair e = 2*step + l/32 (pair 21 is zero), value k = tap j (k = 7 is zero).
template <typename TIN>
__global__ void pack_kernels7_kernel(const TIN *w, u32x4 *wp, int Cout)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= kWpElems) return;
    const int lane = e & 63, step = (e >> 6) % kSteps, mb = (e >> 6) / kSteps;
    const int m = mb * 32 + (lane & 31), pair = 2 * step + (lane >> 5);
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        float x = 0.f;
        if (m < Cout && pair < 21 && k < 7) {
            const TIN raw = w[(size_t)m * 147 + pair * 7 + k];       // pair = c*7 + i
            if constexpr (sizeof(TIN) == 4) x = raw;
            else x = __builtin_bit_cast(float, (uint32_t)raw << 16);
        }
        v[k] = x;
    }
    u32x4 o = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
    wp[e] = o;
}

struct Conv7Params {
    const void *in;     // [N][3][H][W], TIN
    const void *wp;     // packed kernels
    const float *b;     // [Cout] or nullptr
    void *out;          // blocked [N][ldcb][Ho][Wo][8]; F32OUT: fp32 [N][ldcb][Ho][Wo]
    uint32_t in_bytes, out_bytes;
    int N, H, W, Ho, Wo, HoWo, Cout, P, relu;
    int ldcb, coffb;    // layer blocks of 8 per image in `out` and the first one written (F32OUT: layers, first layer)
    int RG, CG;         // tiles per image: row groups, column groups
    int tiles;
    FastDiv dCG, dTilesPerImage;
};

// F32OUT: the results leave unrounded, as an fp32 NCHW map (a convolution called on its own with bfloat16 inputs; the
// network's layers write the blocked bfloat16 map the next layer reads).
template <typename TIN, bool F32OUT = false>
__global__ __launch_bounds__(kThreads7, 3) void conv7s2c3_blocked_kernel(const Conv7Params p)
{
    constexpr uint32_t ESZ = sizeof(TIN);
    __shared__ __attribute__((aligned(16))) u32x4 wl[kWpElems];          // A operands
    __shared__ __attribute__((aligned(16))) uint32_t patch[2][kPatchDw];   // bfloat16 pairs
    __shared__ __attribute__((aligned(16))) float bl[96];

    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int j = lane & 31, h = lane >> 5;
    const int pr = j >> 4, pc = j & 15;

    {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(p.wp);
        for (int e = t; e < kWpElems; e += kThreads7) wl[e] = src[e];
        if (t < 96) bl[t] = (p.b && t < p.Cout) ? p.b[t] : 0.f;
    }

    const rsrc_t rin = make_rsrc(p.in, p.in_bytes), rout = make_rsrc(p.out, p.out_bytes);
    const int tiles_per_image = p.RG * p.CG;

    // ---- staging: thread t fetches column pairs e = t + 256 k of the patch (row-major: layer, row, pair)
    int st_row[kLoads], st_pair[kLoads];     // patch row (0..62) and pair (0..18); row < 0 = nothing
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
        const int e = t + kThreads7 * k;
        const int row = e / kPairs;
        st_row[k] = e < 3 * kPR * kPairs ? row : -1;
        st_pair[k] = e - row * kPairs;
    }
    float xr[kLoads][2];
    auto fetch = [&](int tile) {
        const int n = fdiv(tile, p.dTilesPerImage), rem = tile - n * tiles_per_image;
        const int rg = fdiv(rem, p.dCG), cg = rem - rg * p.CG;
        const int ih0 = rg * kTR * 2 - p.P, iw0 = cg * kTC * 2 - p.P;
#pragma unroll
        for (int k = 0; k < kLoads; ++k) {
            const int c = st_row[k] / kPR, r = st_row[k] - c * kPR;
            const int ih = ih0 + r, iw = iw0 + 2 * st_pair[k];
            const bool rok = st_row[k] >= 0 && ih >= 0 && ih < p.H;
            const uint32_t base = (uint32_t)(((n * 3 + c) * p.H + ih) * p.W + iw) * ESZ;
            xr[k][0] = buf_ld_in<TIN>(rin, rok && iw >= 0 && iw < p.W ? base : kOob, 0u);
            xr[k][1] = buf_ld_in<TIN>(rin, rok && iw + 1 >= 0 && iw + 1 < p.W ? base + ESZ : kOob, 0u);
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int k = 0; k < kLoads; ++k)
            if (st_row[k] >= 0) patch[buf][st_row[k] * kRowDw + st_pair[k]] = pack_bf16x2(xr[k][0], xr[k][1]);
    };

    // ---- B operand: lane (pixel (pr, pc) of this wavefront's two rows, half h) reads the four dwords
    // pc .. pc + 3 of patch row  c*21 + 2*(2 wv + pr) + i,  (c, i) = pair 2 s + h
    const int lane_dw = (2 * (2 * wv + pr)) * kRowDw + pc;
    int step_dw[kSteps];
#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
        const int e0 = 2 * s, e1 = 2 * s + 1 < 21 ? 2 * s + 1 : 20;    // the zero pair may read any valid row
        const int o0 = ((e0 / 7) * kPR + e0 % 7) * kRowDw, o1 = ((e1 / 7) * kPR + e1 % 7) * kRowDw;
        step_dw[s] = lane_dw + (h ? o1 : o0);
    }

    // tiles in memory order per XCD: neighbouring tiles share patch rows and columns, which then come out of one L2
    const mfma::XcdShare share = mfma::xcd_share((int)blockIdx.x, (int)gridDim.x, p.tiles);
    int tile = share.first;
    if (tile < share.end) {
        fetch(tile);
        stash(0);
    }
    __syncthreads();
    const float lowest = p.relu ? 0.f : -__builtin_inff();
    int buf = 0;
    for (; tile < share.end; tile += share.step) {
        const int next = tile + share.step;
        const bool more = next < share.end;
        if (more) fetch(next);

        f32x16 acc[3];
#pragma unroll
        for (int cb = 0; cb < 3; ++cb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 bv = *reinterpret_cast<const f32x4 *>(bl + cb * 32 + 8 * q + 4 * h);
                acc[cb][4 * q + 0] = bv.x; acc[cb][4 * q + 1] = bv.y; acc[cb][4 * q + 2] = bv.z; acc[cb][4 * q + 3] = bv.w;
            }
        const uint32_t *pb = patch[buf];
#pragma unroll
        for (int s = 0; s < kSteps; ++s) {
            u32x4 braw = {pb[step_dw[s]], pb[step_dw[s] + 1], pb[step_dw[s] + 2], pb[step_dw[s] + 3]};
            const bf16x8 b = __builtin_bit_cast(bf16x8, braw);
#pragma unroll
            for (int cb = 0; cb < 3; ++cb) {
                const bf16x8 a = __builtin_bit_cast(bf16x8, wl[(cb * kSteps + s) * 64 + lane]);
                acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[cb], 0, 0, 0);
            }
        }

        // ---- ReLU, round to bfloat16, 8-byte stores (four consecutive layers of one pixel)
        {
            const int n = fdiv(tile, p.dTilesPerImage), rem = tile - n * tiles_per_image;
            const int rg = fdiv(rem, p.dCG), cg = rem - rg * p.CG;
            const int oh = rg * kTR + 2 * wv + pr, ow = cg * kTC + pc;
            const uint32_t o = !(oh < p.Ho && ow < p.Wo) ? kOob
                               : F32OUT ? (uint32_t)(((n * p.ldcb + p.coffb + 4 * h) * p.HoWo + oh * p.Wo + ow) * 4)
                                        : (uint32_t)(((n * p.ldcb + p.coffb) * p.HoWo + oh * p.Wo + ow) * 16 + 8 * h);
#pragma unroll
            for (int cb = 0; cb < 3; ++cb)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int lb = cb * 4 + q;
                    if constexpr (F32OUT) {
                        // register 4q + i = layer 8 lb + 4h + i: 16 neighbouring pixels per store and half-wavefront
                        if (lb * 8 < p.Cout) {
#pragma unroll
                            for (int i = 0; i < 4; ++i)
                                buf_st(rout, o, (uint32_t)((lb * 8 + i) * p.HoWo) * 4u, fmaxf(acc[cb][4 * q + i], lowest));
                        }
                    } else if (lb * 8 < p.Cout) {
                        const float v0 = fmaxf(acc[cb][4 * q + 0], lowest), v1 = fmaxf(acc[cb][4 * q + 1], lowest);
                        const float v2 = fmaxf(acc[cb][4 * q + 2], lowest), v3 = fmaxf(acc[cb][4 * q + 3], lowest);
                        buf_st2(rout, o, (uint32_t)(lb * p.HoWo) * 16u, __builtin_bit_cast(float, pack_bf16x2(v0, v1)),
                                __builtin_bit_cast(float, pack_bf16x2(v2, v3)));
                    }
                }
        }
        if (more) stash(buf ^ 1);
        __syncthreads();    // the other buffer is complete; everyone is done reading this one
        buf ^= 1;
    }
}


// ---- F32OUT for large batches: tiles of 8 output rows x 112 output columns ----------------------------------------
// An fp32 NCHW map much larger than the memory-side cache is written at a fraction of the memory's rate when its
// cache lines reach memory in pieces: a 1.2 GB map goes out at 2.0 TB/s in the 64-byte runs of the 8 x 16 tiles
// above, at 4.4 TB/s when one wavefront writes the pieces of a row one after the other (measured with a store-only
// kernel).  So here a wavefront owns two whole rows of a tile that spans the image width (up to seven column blocks
// of 16; wider images take several such tiles per row group), computes them one block of 32 layers at a time
// (7 accumulators), and stores layer by layer with the column blocks innermost: seven consecutive stores cover
// the two rows, which lie one behind the other in the plane, of two layers.  The 21 x 230 x 3 patch (29 KB as
// bfloat16 pairs) has one LDS buffer (wavefront w fetches patch rows w, w + 4, ...: the row is uniform, so its
// address is scalar arithmetic); with the packed kernels (33 KB) two workgroups fit a CU.
constexpr int kRBlocks = 7;                          // column blocks of 16 per tile
constexpr int kRCols = kRBlocks * kTC;               // 112 output columns
constexpr int kRPairs = kRCols + 3;                  // dwords of a patch row that are read: pairs 0 .. 114
constexpr int kRRowDw = 116;                         // LDS row stride in dwords
constexpr int kRRows = 3 * kPR;                      // 63 patch rows (layer, row)
constexpr int kRPatchDw = kRRows * kRRowDw;
constexpr int kRPerWave = (kRRows + 3) / 4;          // patch rows a wavefront fetches (16)
static_assert(kRPairs <= 128 && kRPairs <= kRRowDw, "two column pairs per lane cover a patch row");

// PAIRS: image width and padding are even and the image is 4-byte aligned, so the two values of a patch pair lie in
// one aligned dword and are loaded together.
template <bool PAIRS>
__global__ __launch_bounds__(kThreads7, 2) void conv7s2c3_rows_kernel(const Conv7Params p)
{
    constexpr uint32_t ESZ = 2;                                          // the image is bfloat16
    __shared__ __attribute__((aligned(16))) u32x4 wl[kWpElems];          // A operands
    __shared__ __attribute__((aligned(16))) uint32_t patch[kRPatchDw];   // bfloat16 pairs
    __shared__ __attribute__((aligned(16))) float bl[96];

    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int j = lane & 31, h = lane >> 5;
    const int pr = j >> 4, pc = j & 15;

    {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(p.wp);
        for (int e = t; e < kWpElems; e += kThreads7) wl[e] = src[e];
        if (t < 96) bl[t] = (p.b && t < p.Cout) ? p.b[t] : 0.f;
    }

    const rsrc_t rin = make_rsrc(p.in, p.in_bytes), rout = make_rsrc(p.out, p.out_bytes);
    const int tiles_per_image = p.RG * p.CG;

    // tile -> image, first output row, first output column (uniform)
    auto decode = [&](int tile_, int &n, int &oh0, int &ow0) {
        const int tile = __builtin_amdgcn_readfirstlane(tile_);
        n = fdiv(tile, p.dTilesPerImage);
        const int rem = tile - n * tiles_per_image, rg = fdiv(rem, p.dCG);
        n = __builtin_amdgcn_readfirstlane(n);
        oh0 = __builtin_amdgcn_readfirstlane(rg * kTR);
        ow0 = __builtin_amdgcn_readfirstlane((rem - rg * p.CG) * kRCols);
    };

    // ---- staging: this wavefront's patch rows R = wv + 4k (layer R / 21, row R % 21), lanes take column pairs
    // lane and lane + 64.  The patch is a plain copy of the image: the two bfloat16 values of a pair are loaded on
    // their own (the image need not be 4-byte aligned) and put together by `pair_up`.  Every load of a tile is issued
    // before the first one is waited for (a row outside the image gets offsets the range check turns away, not a
    // branch), and the values wait in registers until the next tile starts.
    short xr[kRPerWave][2][2];
    uint32_t xp[kRPerWave][2];
    auto fetch = [&](int tile) {
        int n, oh0, ow0;
        decode(tile, n, oh0, ow0);
        const int ih0 = oh0 * 2 - p.P, iw0 = ow0 * 2 - p.P;
        uint32_t loff[2][2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int pj = lane + 64 * q, iw = iw0 + 2 * pj;
#pragma unroll
            for (int e = 0; e < 2; ++e) loff[q][e] = (pj < kRPairs && iw + e >= 0 && iw + e < p.W) ? (uint32_t)(iw + e) * ESZ : kOob;
        }
#pragma unroll
        for (int k = 0; k < kRPerWave; ++k) {
            const int R = wv + 4 * k, c = R / kPR, r = R - c * kPR;      // uniform
            const int ih = ih0 + r;
            const bool rok = R < kRRows && ih >= 0 && ih < p.H;
            const uint32_t row = rok ? (uint32_t)(((n * 3 + c) * p.H + ih) * p.W) * ESZ : 0u;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                if constexpr (PAIRS) {
                    // (an even first column: a pair is inside the image or outside it as a whole)
                    xp[k][q] = __builtin_bit_cast(uint32_t, buf_ld(rin, rok ? loff[q][0] : kOob, row));
                } else {
#pragma unroll
                    for (int e = 0; e < 2; ++e)
                        xr[k][q][e] = __builtin_amdgcn_raw_buffer_load_b16(rin, (int)(rok ? loff[q][e] : kOob), (int)row, 0);
                }
            }
        }
    };
    // Where this stands in the program is where the loads are waited for (the empty statements keep the compiler
    // from doing the shifts, and with them the wait, right behind the loads).
    auto pair_up = [&]() {
#pragma unroll
        for (int k = 0; k < kRPerWave; ++k)
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                if constexpr (PAIRS) {
                    asm volatile("" : "+v"(xp[k][q]));
                } else {
                    asm volatile("" : "+v"(xr[k][q][0]), "+v"(xr[k][q][1]));
                    xp[k][q] = (uint32_t)(uint16_t)xr[k][q][0] | ((uint32_t)(uint16_t)xr[k][q][1] << 16);
                }
            }
    };
    auto stash = [&]() {
#pragma unroll
        for (int k = 0; k < kRPerWave; ++k) {
            const int R = wv + 4 * k;
            if (R < kRRows) {
#pragma unroll
                for (int q = 0; q < 2; ++q)
                    if (lane + 64 * q < kRPairs) patch[R * kRRowDw + lane + 64 * q] = xp[k][q];
            }
        }
    };

    // ---- B operand of column block 0: lane (pixel (pr, pc) of this wavefront's two rows, half h) reads the four
    // dwords pc .. pc + 3 of patch row  c*21 + 2*(2 wv + pr) + i,  (c, i) = pair 2 s + h; block k lies 16 dwords on
    const int lane_dw = (2 * (2 * wv + pr)) * kRRowDw + pc;
    int step_dw[kSteps];
#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
        const int e0 = 2 * s, e1 = 2 * s + 1 < 21 ? 2 * s + 1 : 20;    // the zero pair may read any valid row
        const int o0 = ((e0 / 7) * kPR + e0 % 7) * kRRowDw, o1 = ((e1 / 7) * kPR + e1 % 7) * kRRowDw;
        step_dw[s] = lane_dw + (h ? o1 : o0);
    }

    const mfma::XcdShare share = mfma::xcd_share((int)blockIdx.x, (int)gridDim.x, p.tiles);
    const float lowest = p.relu ? 0.f : -__builtin_inff();
    // The next tile's patch is asked for at the start of a tile, behind the stores that fill the memory pipeline a
    // load takes most of a tile's time to come back.
    if (share.first < share.end) {
        fetch(share.first);
        pair_up();
    }
    for (int tile = share.first; tile < share.end; tile += share.step) {
        const bool more = tile + share.step < share.end;
        __syncthreads();    // everyone is done with the previous tile's patch
        stash();
        __syncthreads();
        if (more) fetch(tile + share.step);

        // lane byte offsets of this lane's pixel in the seven column blocks (layer 4h of the image's first one)
        uint32_t o[kRBlocks];
        {
            int n, oh0, ow0;
            decode(tile, n, oh0, ow0);
            const int oh = oh0 + 2 * wv + pr;
            const uint32_t base = (uint32_t)(((n * p.ldcb + p.coffb + 4 * h) * p.HoWo + oh * p.Wo + ow0 + pc) * 4);
#pragma unroll
            for (int k = 0; k < kRBlocks; ++k) o[k] = (oh < p.Ho && ow0 + 16 * k + pc < p.Wo) ? base + 64u * k : kOob;
        }
        // (unrolled: in front of a loop that uses loaded values the compiler waits for every load)
#pragma unroll
        for (int cb = 0; cb < 3; ++cb) {
            if (cb * 32 >= p.Cout) break;
            f32x16 acc[kRBlocks];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 bv = *reinterpret_cast<const f32x4 *>(bl + cb * 32 + 8 * q + 4 * h);
#pragma unroll
                for (int k = 0; k < kRBlocks; ++k) {
                    acc[k][4 * q + 0] = bv.x; acc[k][4 * q + 1] = bv.y; acc[k][4 * q + 2] = bv.z; acc[k][4 * q + 3] = bv.w;
                }
            }
#pragma unroll
            for (int s = 0; s < kSteps; ++s) {
                const bf16x8 a = __builtin_bit_cast(bf16x8, wl[(cb * kSteps + s) * 64 + lane]);
#pragma unroll
                for (int k = 0; k < kRBlocks; ++k) {
                    const uint32_t *pb = patch + step_dw[s] + 16 * k;
                    u32x4 braw = {pb[0], pb[1], pb[2], pb[3]};
                    acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, braw), acc[k], 0, 0, 0);
                }
            }
            if (cb == 0 && more) {
                // The next tile's patch is waited for here, before this block's stores, where the only older
                // stores are those of the tile before (measured equal to waiting at the start of the next tile,
                // behind this tile's 336 stores; it halves the registers the patch holds from here on).
                pair_up();
            }
            // register 4q + i = layer 32 cb + 8q + 4h + i; per layer the seven column blocks one after the other
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (cb * 32 + q * 8 < p.Cout) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t layer = (uint32_t)((cb * 32 + q * 8 + i) * p.HoWo) * 4u;
#pragma unroll
                        for (int k = 0; k < kRBlocks; ++k) buf_st(rout, o[k], layer, fmaxf(acc[k][4 * q + i], lowest));
                    }
                }
            }
        }
    }
}

}  // namespace
}  // namespace blocked

using namespace blocked;

// fp32 results through the tiles that span the image width: -1 = by batch size, 0 = never, 1 = always
thread_local int g_f32out_rows = -1;
extern "C" void sq_tune_conv7_f32out_rows(int mode) { g_f32out_rows = mode; }

size_t blocked_packed_kernel7_bytes() { return (size_t)kWpElems * 16; }

int blocked_pack_kernels7(const void *w, int dtype, void *packed, int Cout)
{
    if (Cout > 96) return SQ_ERR_UNSUPPORTED;
    LaunchScope scope("pack_kernels7", 0.0, (dtype == SQ_BF16 ? 2.0 : 4.0) * Cout * 147 + 16.0 * kWpElems);
    const int blocks = (kWpElems + 255) / 256;
    if (dtype == SQ_BF16)
        hipLaunchKernelGGL(pack_kernels7_kernel<uint16_t>, dim3(blocks), dim3(256), 0, current_stream(), (const uint16_t *)w,
                           (u32x4 *)packed, Cout);
    else
        hipLaunchKernelGGL(pack_kernels7_kernel<float>, dim3(blocks), dim3(256), 0, current_stream(), (const float *)w,
                           (u32x4 *)packed, Cout);
    return check_launch();
}

// 7x7, stride 2, pad P, three input layers (NCHW image of type dtype) -> layers [c_offset, +Cout) of a
// blocked bfloat16 map with ldc_channels layers, or (f32_out) of an fp32 NCHW map with ldc_channels layers.
int blocked_conv7s2(const void *in, int dtype, const void *wp, const float *b, void *out, int N, int H, int W, int Cout, int P,
                    int relu, int ldc_channels, int c_offset, bool f32_out)
{
    if (Cout > 96 || Cout % 8 != 0) return SQ_ERR_UNSUPPORTED;
    if (!f32_out && (ldc_channels % 8 != 0 || c_offset % 8 != 0)) return SQ_ERR_UNSUPPORTED;
    if (H + 2 * P < 7 || W + 2 * P < 7) return SQ_ERR_SHAPE;
    const int Ho = (H + 2 * P - 7) / 2 + 1, Wo = (W + 2 * P - 7) / 2 + 1;
    const long long in_bytes = (long long)N * 3 * H * W * (dtype == SQ_BF16 ? 2 : 4);
    const long long out_bytes = f32_out ? (long long)N * ldc_channels * Ho * Wo * 4 : (long long)blocked_map_bytes(N, ldc_channels, Ho, Wo);
    Conv7Params p;
    p.RG = (Ho + kTR - 1) / kTR;
    p.CG = (Wo + kTC - 1) / kTC;
    // fp32 results of a large batch: tiles that span the image width (see conv7s2c3_rows_kernel), once the map
    // outgrows the memory-side cache (measured on 224 x 224 images: slower up to batch 40, faster from 48 on) and
    // there are two such tiles per CU
    const int row_tiles = (Wo + kRCols - 1) / kRCols;
    const bool big = (long long)N * Cout * Ho * Wo * 4 >= (200ll << 20) && (long long)N * p.RG * row_tiles >= 2ll * num_cus();
    const bool rows = f32_out && dtype == SQ_BF16 && (g_f32out_rows < 0 ? big : g_f32out_rows > 0);
    if (rows) p.CG = row_tiles;
    const long long tiles = (long long)N * p.RG * p.CG;
    if (in_bytes >= (1ll << 31) || out_bytes >= (1ll << 31) || tiles >= (1ll << 30)) return SQ_ERR_UNSUPPORTED;
    p.in = in; p.wp = wp; p.b = b; p.out = out;
    p.in_bytes = (uint32_t)in_bytes; p.out_bytes = (uint32_t)out_bytes;
    p.N = N; p.H = H; p.W = W; p.Ho = Ho; p.Wo = Wo; p.HoWo = Ho * Wo; p.Cout = Cout; p.P = P; p.relu = relu;
    p.ldcb = f32_out ? ldc_channels : ldc_channels / 8; p.coffb = f32_out ? c_offset : c_offset / 8;
    p.tiles = (int)tiles;
    p.dCG = make_fastdiv(p.CG); p.dTilesPerImage = make_fastdiv(p.RG * p.CG);
    long long blocks = (rows ? 2ll : 3ll) * num_cus();
    if (blocks > tiles) blocks = tiles;
    LaunchScope scope(rows ? "k7s2c3_bf16_8x112_f32out" : f32_out ? "k7s2c3_bf16_8x16_f32out" : "k7s2c3_bf16_8x16", 2.0 * N * Cout * Ho * Wo * 147.0,
                      (dtype == SQ_BF16 ? 2.0 : 4.0) * N * 3 * H * W + 2.0 * Cout * 147 + (f32_out ? 4.0 : 2.0) * N * Cout * Ho * Wo + 4.0 * Cout);
    if (rows) {
        const bool pairs = W % 2 == 0 && P % 2 == 0 && (reinterpret_cast<uintptr_t>(in) & 3) == 0;
        hipLaunchKernelGGL(pairs ? conv7s2c3_rows_kernel<true> : conv7s2c3_rows_kernel<false>, dim3((unsigned)blocks), dim3(kThreads7), 0,
                           current_stream(), p);
    } else if (f32_out) {
        if (dtype == SQ_BF16)
            hipLaunchKernelGGL((conv7s2c3_blocked_kernel<uint16_t, true>), dim3((unsigned)blocks), dim3(kThreads7), 0, current_stream(), p);
        else
            hipLaunchKernelGGL((conv7s2c3_blocked_kernel<float, true>), dim3((unsigned)blocks), dim3(kThreads7), 0, current_stream(), p);
    } else if (dtype == SQ_BF16) {
        hipLaunchKernelGGL(conv7s2c3_blocked_kernel<uint16_t>, dim3((unsigned)blocks), dim3(kThreads7), 0, current_stream(), p);
    } else {
        hipLaunchKernelGGL(conv7s2c3_blocked_kernel<float>, dim3((unsigned)blocks), dim3(kThreads7), 0, current_stream(), p);
    }
    return check_launch();
}

}  // namespace sq
