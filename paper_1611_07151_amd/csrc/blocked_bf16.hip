// Reduced-precision path: feature maps and kernels in bfloat16, sums in fp32 (the
// counterpart of the paper's relaxed-precision mode, section "Imprecise computing"; its
// layer-private vector layout, sections "Data Reordering" and "Zero-overhead
// vectorization", is used here with vectors of eight layers).
//
// Layout ("blocked"): a feature map of C layers is stored as [N][ceil(C/8)][H][W][8]
// bfloat16 -- the eight layers 8k..8k+7 of one pixel are one 16-byte element, which is
// exactly the operand a lane feeds to v_mfma_f32_32x32x16_bf16 (8 consecutive k values).
// Every layer of the network writes its output directly in this layout, so nothing is
// ever re-ordered between layers.  Layers past C in the last block are zero.
//
// Kernels are packed once (offline in the paper's terms) into MFMA A-operand order:
//   wp[ceil(Cout/32)][K*K][Cin/16][64 lanes][8]:  lane l holds output layer 32*mb + l%32,
//   tap t, input layers 16*g + 8*(l/32) .. +7.
//
// Convolution kernel (K x K, stride 1, pad (K-1)/2).  D(32 layers x 32 pixels) +=
// A(32 x 16) B(16 x 32) per MFMA, with A = packed kernels from LDS (one 16-byte read per
// lane) and B = one 16-byte element per lane loaded straight from global memory into the
// operand registers (pixel l%32 of the tile, shifted by the tap; layer block 2g + l/32).
// A persistent workgroup of 8 wavefronts owns 32*CB output layers, keeps all their
// kernels in LDS and walks over tiles of 32*PB pixels; the wavefronts are autonomous
// after the one barrier.  Loads run D steps ahead of the MFMAs in a register ring.  Zero
// padding comes from the buffer range check (an invalid tap gets an out-of-range
// offset).  Results leave as 8-byte stores (four consecutive layers of one pixel), which
// a wavefront lays down as 512 contiguous bytes per layer block.
#include "conv_mfma_common.h"

namespace sq {
namespace blocked {

using namespace mfma;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512, kWaves = kThreads / 64;

__device__ __forceinline__ uint32_t pack2(float a, float b) { return pack_bf16x2(a, b); }   // round to nearest even
__device__ __forceinline__ float bf_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

// ------------------------------------------------------------------------------- layout
// NCHW (fp32 or bf16) -> blocked bf16.  One thread per 16-byte element.
template <typename TIN>
__global__ void pack_map_kernel(const TIN *in, u32x4 *out, int N, int C, int HW, int CB, FastDiv dHW, FastDiv dCB)
{
    const long long total = (long long)N * CB * HW;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (long long)gridDim.x * blockDim.x) {
        const int ncb = fdiv((int)e, dHW), pix = (int)e - ncb * HW;
        const int n = fdiv(ncb, dCB), cb = ncb - n * CB;
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int c = cb * 8 + k;
            float x = 0.f;
            if (c < C) {
                const TIN raw = in[((size_t)n * C + c) * HW + pix];
                if constexpr (sizeof(TIN) == 4) x = raw;
                else x = __builtin_bit_cast(float, (uint32_t)raw << 16);
            }
            v[k] = x;
        }
        u32x4 o = {pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7])};
        out[e] = o;
    }
}

// The same for a bfloat16 NCHW map whose address is a multiple of 16, by whole 16-byte loads: a workgroup takes 504
// pixels of a block of eight layers; of each layer it loads the (at most 64) aligned 16-byte pieces that hold those
// pixels into LDS, and every thread then gathers the eight layers of a pixel from there.  (One thread per element with
// eight 2-byte loads, as above, moves 2.2 TB/s at batch 256: a wavefront-wide load costs the same whatever its width.)
constexpr int kPackChunk = 504;   // 504 + 7 elements of misalignment fit 64 pieces of 8
__global__ __launch_bounds__(256) void pack_map_bf16_kernel(const uint16_t *in, u32x4 *out, int C, int HW, int CB, int chunks, int items,
                                                            FastDiv dChunks, FastDiv dCB, uint32_t in_bytes)
{
    __shared__ __attribute__((aligned(16))) uint16_t raw[8][512];
    const int t = threadIdx.x, k = t >> 5, v0 = t & 31;
    const rsrc_t rin = make_rsrc(in, in_bytes);
    for (int item = (int)blockIdx.x; item < items; item += (int)gridDim.x) {
        const int g = fdiv(item, dChunks), ch = item - g * chunks;     // g = n * CB + cb
        const int n = fdiv(g, dCB), cb = g - n * CB;
        const int p0 = ch * kPackChunk, cnt = min(kPackChunk, HW - p0);
        const int first = (n * C + cb * 8) * HW + p0;                  // element of layer 8 cb at pixel p0
        {
            const int c = cb * 8 + k;
            const uint32_t a0 = (uint32_t)(first + k * HW) & ~7u;      // first aligned piece of this thread's layer
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int vi = v0 + 32 * j;
                uint32_t off = c < C ? (a0 + 8u * (uint32_t)vi) * 2u : kOob;   // (bytes past the end of the map read zero)
                asm volatile("" : "+v"(off));   // keeps +4, +8, +12 as immediates so that the four loads merge
                float w[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) w[q] = buf_ld(rin, off + 4u * q, 0u);
                *reinterpret_cast<f32x4 *>(&raw[k][vi * 8]) = f32x4{w[0], w[1], w[2], w[3]};
            }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int px = t + 256 * r;
            if (px < cnt) {
                uint32_t e[8];
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) e[kk] = raw[kk][((first + kk * HW) & 7) + px];
                out[(size_t)g * HW + p0 + px] = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
            }
        }
        __syncthreads();
    }
}

// blocked bf16 -> NCHW fp32.  One thread per 16-byte element.
__global__ void unpack_map_kernel(const u32x4 *in, float *out, int N, int C, int HW, int CB, FastDiv dHW, FastDiv dCB)
{
    const long long total = (long long)N * CB * HW;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (long long)gridDim.x * blockDim.x) {
        const int ncb = fdiv((int)e, dHW), pix = (int)e - ncb * HW;
        const int n = fdiv(ncb, dCB), cb = ncb - n * CB;
        const u32x4 v = in[e];
        const float f[8] = {bf_lo(v.x), bf_hi(v.x), bf_lo(v.y), bf_hi(v.y), bf_lo(v.z), bf_hi(v.z), bf_lo(v.w), bf_hi(v.w)};
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int c = cb * 8 + k;
            if (c < C) out[((size_t)n * C + c) * HW + pix] = f[k];
        }
    }
}

// [Cout][Cin][K][K] (fp32 or bf16) -> MFMA A-operand order (see the header of this file).
template <typename TIN>
__global__ void pack_kernels_kernel(const TIN *w, u32x4 *wp, int Cout, int Cin, int KK, int G, int total)
{
    for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < total; e += gridDim.x * blockDim.x) {
        const int lane = e & 63;
        int r = e >> 6;
        const int g = r % G;
        r /= G;
        const int tap = r % KK, mb = r / KK;
        const int m = mb * 32 + (lane & 31), c0 = g * 16 + 8 * (lane >> 5);
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int c = c0 + k;
            float x = 0.f;
            if (m < Cout && c < Cin) {
                const TIN raw = w[((size_t)m * Cin + c) * KK + tap];
                if constexpr (sizeof(TIN) == 4) x = raw;
                else x = __builtin_bit_cast(float, (uint32_t)raw << 16);
            }
            v[k] = x;
        }
        u32x4 o = {pack2(v[0], v[1]), pack2(v[2], v[3]), pack2(v[4], v[5]), pack2(v[6], v[7])};
        wp[e] = o;
    }
}

// --------------------------------------------------------------------------- convolution
struct ConvParams {
    const void *in;      // blocked [N][Cin/8][H][W][8]
    const void *wp;      // packed kernels
    const float *b;      // [Cout] or nullptr
    void *out;           // blocked [N][ldcb][H][W][8]; F32OUT kernels: fp32 [N][ldcb][H][W]
    uint32_t in_bytes, out_bytes, wp_elems;   // wp_elems: 16-byte elements of wp
    int N, Cin, H, W, HW, Cout, K, P, relu;
    int G;               // Cin / 16
    int steps;           // K*K*G, a multiple of the ring depth
    int ldcb, coffb;     // layer blocks (of 8) per image in `out`, first block written (F32OUT: layers, first layer)
    int PT;              // N*H*W
    int tiles;           // pixel tiles of 32*PB
    int ncblk;           // groups of 32*CB output layers = workgroups that share a pixel range
    int Hin, Win;        // pooled-input kernel: extents of the map before the 3x3 stride-2 max pooling (H, W = after)
    FastDiv dHW, dW, dG, dK, dNcblk;
};

// Two convolutions of the same input and the same CB/PB/D may share a launch (the two expands of
// a fire layer): workgroups [0, split) run pa, the rest run pb.  A single convolution passes
// split = gridDim.x.
// F32OUT: the results leave unrounded, as an fp32 NCHW map (a convolution called on its own with bfloat16 inputs:
// fp32 accumulate and output); the network's layers write the blocked bfloat16 map the next layer reads.
template <int CB, int PB, int D, bool F32OUT = false>
__global__ __launch_bounds__(kThreads, 2) void conv_blocked_kernel(const ConvParams pa, const ConvParams pb, const int split)
{
    const bool second = (int)blockIdx.x >= split;
    const ConvParams p = second ? pb : pa;   // by value: every field becomes a scalar select
    const int wg = second ? (int)blockIdx.x - split : (int)blockIdx.x;
    const int nwg = second ? (int)gridDim.x - split : split;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    u32x4 *const wl = reinterpret_cast<u32x4 *>(smem);                 // [CB][steps][64] A operands
    const int per_mb = p.steps * 64;                                      // 16-byte elements per 32 layers
    float *const bl = reinterpret_cast<float *>(smem + (size_t)CB * per_mb * 16);   // [CB*32] bias

    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int j = lane & 31, h = lane >> 5;
    const int slot = fdiv(wg, p.dNcblk), cblk = wg - slot * p.ncblk;
    const int nslots = nwg / p.ncblk;                     // the host launches a multiple of ncblk
    const int mb0 = cblk * CB;                            // first block of 32 output layers

    // ---- this workgroup's kernels and bias into LDS (a straight copy: they are packed) ----
    {
        // (all loads of a batch are issued before the first LDS write, so their latencies overlap: with up to
        // 74 KB per workgroup a load-then-write loop would spend ten memory round trips before the first MFMA)
        const u32x4 *src = reinterpret_cast<const u32x4 *>(p.wp);
        const uint32_t first = (uint32_t)mb0 * (uint32_t)per_mb;
        constexpr int kBatch = 10;
        for (int e0 = t; e0 < CB * per_mb; e0 += kBatch * kThreads) {
            u32x4 v[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                const int e = e0 + k * kThreads;
                v[k] = u32x4{0u, 0u, 0u, 0u};
                if (e < CB * per_mb && first + (uint32_t)e < p.wp_elems) v[k] = src[first + e];
            }
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                const int e = e0 + k * kThreads;
                if (e < CB * per_mb) wl[e] = v[k];
            }
        }
        if (t < CB * 32) {
            const int m = mb0 * 32 + t;
            bl[t] = (p.b && m < p.Cout) ? p.b[m] : 0.f;
        }
    }
    __syncthreads();   // the only barrier

    const rsrc_t rin = make_rsrc(p.in, p.in_bytes);
    const rsrc_t rout = make_rsrc(p.out, p.out_bytes);
    const float lowest = p.relu ? 0.f : -__builtin_inff();
    const uint32_t hw16 = (uint32_t)p.HW * 16u;
    const int KK = p.K * p.K;

    for (int tile = slot * kWaves + wv; tile < p.tiles; tile += nslots * kWaves) {
        // ---- this lane's pixels: input offset (layer block h of a pair), output offset, tap validity
        uint32_t ibase[PB], obase[PB], vmask[PB];
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            const int gp = (tile * PB + pb) * 32 + j;
            const bool ok = gp < p.PT;
            const int gq = ok ? gp : 0;
            const int n = fdiv(gq, p.dHW), pix = gq - n * p.HW;
            const int y = fdiv(pix, p.dW), x = pix - y * p.W;
            ibase[pb] = (uint32_t)((n * (p.Cin >> 3) + h) * p.HW + pix) * 16u;
            obase[pb] = !ok ? kOob
                        : F32OUT ? (uint32_t)((n * p.ldcb + p.coffb + 4 * h) * p.HW + pix) * 4u
                                 : (uint32_t)((n * p.ldcb + p.coffb) * p.HW + pix) * 16u + 8u * (uint32_t)h;
            uint32_t m = 0;
            for (int tap = 0; tap < KK; ++tap) {
                const int ky = fdiv(tap, p.dK), kx = tap - ky * p.K;
                const bool v = ok && (unsigned)(y + ky - p.P) < (unsigned)p.H && (unsigned)(x + kx - p.P) < (unsigned)p.W;
                m |= (v ? 1u : 0u) << tap;
            }
            vmask[pb] = m;
        }

        // input of step s = (tap, pair of layer blocks g): one 16-byte element per lane and pixel block,
        // loaded as four adjacent dwords the compiler merges.  Steps are loaded in order, so the position
        // (tap, g) of the next one is a cursor that is advanced after every load: one scalar add per step
        // and the per-lane offsets of a tap only when the tap changes (the scalar unit of a SIMD is shared
        // by its wavefronts; recomputing the position of every step from its index by divisions kept it
        // busy 74 % of the kernel's time).
        float bx[D][PB][4];
        int g_i = 0, tap_i = 0, ky_i = 0, kx_i = 0;
        uint32_t so_i = 0, off_i[PB];
        auto set_tap = [&]() {
            const int shift = ((ky_i - p.P) * p.W + (kx_i - p.P)) * 16;
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) off_i[pb] = ((vmask[pb] >> tap_i) & 1u) ? ibase[pb] + (uint32_t)shift : kOob;
        };
        set_tap();
        auto issue = [&](int ring) {
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                uint32_t off = off_i[pb];
                asm volatile("" : "+v"(off));   // keeps +4, +8, +12 as immediates so that the four loads merge
#pragma unroll
                for (int q = 0; q < 4; ++q) bx[ring][pb][q] = buf_ld(rin, off + 4u * q, so_i);
            }
            so_i += 2u * hw16;
            if (++g_i == p.G) {      // uniform: next tap
                g_i = 0;
                so_i = 0;
                ++tap_i;
                if (++kx_i == p.K) {
                    kx_i = 0;
                    ++ky_i;
                }
                set_tap();
            }
        };
#pragma unroll
        for (int r = 0; r < D; ++r) issue(r);

        // ---- accumulators start from the bias: registers 4q..4q+3 = layers 8q + 4h .. +3 of the block
        f32x16 acc[CB][PB];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 bv = *reinterpret_cast<const f32x4 *>(bl + cb * 32 + 8 * q + 4 * h);
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) {
                    acc[cb][pb][4 * q + 0] = bv.x; acc[cb][pb][4 * q + 1] = bv.y;
                    acc[cb][pb][4 * q + 2] = bv.z; acc[cb][pb][4 * q + 3] = bv.w;
                }
            }

        // A operands are read from LDS one step ahead of their MFMAs (the read of step s+1 is issued before the
        // MFMAs of step s), so the LDS latency is not on the path from one step to the next
        bf16x8 a_cur[CB], a_nxt[CB];
        auto read_a = [&](bf16x8 (&a)[CB], int s) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) a[cb] = __builtin_bit_cast(bf16x8, wl[(cb * p.steps + s) * 64 + lane]);
        };
        auto compute = [&](int ring, int s) {
            read_a(a_nxt, s + 1 < p.steps ? s + 1 : s);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                f32x4 raw = {bx[ring][pb][0], bx[ring][pb][1], bx[ring][pb][2], bx[ring][pb][3]};
                const bf16x8 b = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
                    acc[cb][pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_cur[cb], b, acc[cb][pb], 0, 0, 0);
            }
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) a_cur[cb] = a_nxt[cb];
        };
        read_a(a_cur, 0);
        int s0 = 0;
        for (; s0 < p.steps - D; s0 += D) {
#pragma unroll
            for (int r = 0; r < D; ++r) {
                compute(r, s0 + r);
                issue(r);
            }
        }
#pragma unroll
        for (int r = 0; r < D; ++r) compute(r, s0 + r);

        // ---- ReLU, round to bfloat16, 8-byte stores
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int lb = (mb0 + cb) * 4 + q;              // layer block (of 8) inside this convolution
                if constexpr (F32OUT) {
                    // register 4q + i = layer 8 lb + 4h + i: 32 neighbouring pixels per store and half-wavefront
                    if (lb * 8 < p.Cout) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const uint32_t so = (uint32_t)((lb * 8 + i) * p.HW) * 4u;
#pragma unroll
                            for (int pb = 0; pb < PB; ++pb) buf_st(rout, obase[pb], so, fmaxf(acc[cb][pb][4 * q + i], lowest));
                        }
                    }
                } else if (lb * 8 < p.Cout) {                            // uniform
                    const uint32_t so = (uint32_t)lb * hw16;
#pragma unroll
                    for (int pb = 0; pb < PB; ++pb) {
                        const float v0 = fmaxf(acc[cb][pb][4 * q + 0], lowest), v1 = fmaxf(acc[cb][pb][4 * q + 1], lowest);
                        const float v2 = fmaxf(acc[cb][pb][4 * q + 2], lowest), v3 = fmaxf(acc[cb][pb][4 * q + 3], lowest);
                        buf_st2(rout, obase[pb], so, __builtin_bit_cast(float, pack2(v0, v1)),
                                __builtin_bit_cast(float, pack2(v2, v3)));
                    }
                }
            }
    }
}

// Max pooling (3x3 window, stride 2, floor mode) fused into the 1x1 convolution that reads its
// result -- in this network every pooled map is read by exactly one squeeze layer, so the pooled
// map never exists in memory.  Same structure as conv_blocked_kernel with one pixel block per
// wavefront tile; the B operand of a step is the maximum over the nine window elements, each a
// 16-byte load of eight layers.  bfloat16 values are compared as 16-bit integers after the usual
// order-preserving map (negative: all bits flipped, else sign bit flipped), two per 32-bit operation.
typedef short i16x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t order_key(uint32_t x)
{
    const i16x2 sign = __builtin_bit_cast(i16x2, x) >> 15;                          // 0xffff where negative
    return x ^ (__builtin_bit_cast(uint32_t, sign) | 0x80008000u);
}
__device__ __forceinline__ uint32_t order_key_inverse(uint32_t k)
{
    const i16x2 top = __builtin_bit_cast(i16x2, k) >> 15;                           // 0xffff where the value was not negative
    return k ^ (~__builtin_bit_cast(uint32_t, top) | 0x80008000u);
}
__device__ __forceinline__ uint32_t max_u16x2(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}

template <int CB, int D>
__global__ __launch_bounds__(kThreads, 2) void pool_conv_blocked_kernel(const ConvParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    u32x4 *const wl = reinterpret_cast<u32x4 *>(smem);
    const int per_mb = p.steps * 64;
    float *const bl = reinterpret_cast<float *>(smem + (size_t)CB * per_mb * 16);

    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int j = lane & 31, h = lane >> 5;
    const int slot = fdiv((int)blockIdx.x, p.dNcblk), cblk = (int)blockIdx.x - slot * p.ncblk;
    const int nslots = (int)gridDim.x / p.ncblk;
    const int mb0 = cblk * CB;
    {
        // (all loads of a batch are issued before the first LDS write, so their latencies overlap: with up to
        // 74 KB per workgroup a load-then-write loop would spend ten memory round trips before the first MFMA)
        const u32x4 *src = reinterpret_cast<const u32x4 *>(p.wp);
        const uint32_t first = (uint32_t)mb0 * (uint32_t)per_mb;
        constexpr int kBatch = 10;
        for (int e0 = t; e0 < CB * per_mb; e0 += kBatch * kThreads) {
            u32x4 v[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                const int e = e0 + k * kThreads;
                v[k] = u32x4{0u, 0u, 0u, 0u};
                if (e < CB * per_mb && first + (uint32_t)e < p.wp_elems) v[k] = src[first + e];
            }
#pragma unroll
            for (int k = 0; k < kBatch; ++k) {
                const int e = e0 + k * kThreads;
                if (e < CB * per_mb) wl[e] = v[k];
            }
        }
        if (t < CB * 32) {
            const int m = mb0 * 32 + t;
            bl[t] = (p.b && m < p.Cout) ? p.b[m] : 0.f;
        }
    }
    __syncthreads();

    const rsrc_t rin = make_rsrc(p.in, p.in_bytes);
    const rsrc_t rout = make_rsrc(p.out, p.out_bytes);
    const float lowest = p.relu ? 0.f : -__builtin_inff();
    const uint32_t hw16 = (uint32_t)p.HW * 16u, hwin16 = (uint32_t)(p.Hin * p.Win) * 16u, row16 = (uint32_t)p.Win * 16u;

    for (int tile = slot * kWaves + wv; tile < p.tiles; tile += nslots * kWaves) {
        const int gp = tile * 32 + j;
        const bool ok = gp < p.PT;
        const int gq = ok ? gp : 0;
        const int n = fdiv(gq, p.dHW), pix = gq - n * p.HW;
        const int y = fdiv(pix, p.dW), x = pix - y * p.W;
        // first element of this pixel's window in layer block h of a pair; every window lies inside the map
        const uint32_t ibase = ok ? (uint32_t)(((n * (p.Cin >> 3) + h) * p.Hin + 2 * y) * p.Win + 2 * x) * 16u : kOob;
        const uint32_t obase = ok ? (uint32_t)((n * p.ldcb + p.coffb) * p.HW + pix) * 16u + 8u * (uint32_t)h : kOob;

        float bx[D][9][4];
        auto issue = [&](int ring, int s_) {
            const int s = __builtin_amdgcn_readfirstlane(s_);
            const uint32_t so = (uint32_t)s * 2u * hwin16;
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                uint32_t off = ok ? ibase + (uint32_t)i * row16 : kOob;
                asm volatile("" : "+v"(off));   // the twelve loads of a window row differ by immediates only
#pragma unroll
                for (int jx = 0; jx < 3; ++jx)
#pragma unroll
                    for (int q = 0; q < 4; ++q) bx[ring][3 * i + jx][q] = buf_ld(rin, off + 16u * jx + 4u * q, so);
            }
        };
#pragma unroll
        for (int r = 0; r < D; ++r) issue(r, r);

        f32x16 acc[CB];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 bv = *reinterpret_cast<const f32x4 *>(bl + cb * 32 + 8 * q + 4 * h);
                acc[cb][4 * q + 0] = bv.x; acc[cb][4 * q + 1] = bv.y; acc[cb][4 * q + 2] = bv.z; acc[cb][4 * q + 3] = bv.w;
            }
        auto compute = [&](int ring, int s) {
            u32x4 m;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t k = order_key(__builtin_bit_cast(uint32_t, bx[ring][0][q]));
#pragma unroll
                for (int e = 1; e < 9; ++e) k = max_u16x2(k, order_key(__builtin_bit_cast(uint32_t, bx[ring][e][q])));
                m[q] = order_key_inverse(k);
            }
            const bf16x8 b = __builtin_bit_cast(bf16x8, m);
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const bf16x8 a = __builtin_bit_cast(bf16x8, wl[(cb * p.steps + s) * 64 + lane]);
                acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[cb], 0, 0, 0);
            }
        };
        int s0 = 0;
        for (; s0 < p.steps - D; s0 += D) {
#pragma unroll
            for (int r = 0; r < D; ++r) {
                compute(r, s0 + r);
                issue(r, s0 + r + D);
            }
        }
#pragma unroll
        for (int r = 0; r < D; ++r) compute(r, s0 + r);

#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int lb = (mb0 + cb) * 4 + q;
                if (lb * 8 < p.Cout) {
                    const float v0 = fmaxf(acc[cb][4 * q + 0], lowest), v1 = fmaxf(acc[cb][4 * q + 1], lowest);
                    const float v2 = fmaxf(acc[cb][4 * q + 2], lowest), v3 = fmaxf(acc[cb][4 * q + 3], lowest);
                    buf_st2(rout, obase, (uint32_t)lb * hw16, __builtin_bit_cast(float, pack2(v0, v1)),
                            __builtin_bit_cast(float, pack2(v2, v3)));
                }
            }
    }
}

// ------------------------------------------------------------------------------- pooling
// Max pooling K x K stride S (floor mode, no padding) on blocked maps: one thread per
// 16-byte output element (eight layers of one pixel).
// KT, ST: window and stride known at compile time (the network's 3x3 stride 2: all nine loads of a window are
// issued before the first maximum), or 0 = taken from the arguments.
template <int KT, int ST>
__global__ void maxpool_blocked_kernel(const u32x4 *in, u32x4 *out, int planes, int H, int W, int Ho, int Wo, int K_, int S_,
                                       FastDiv dWo, FastDiv dHoWo)
{
    const int K = KT ? KT : K_, S = ST ? ST : S_;
    const long long total = (long long)planes * Ho * Wo;
    for (long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (long long)gridDim.x * blockDim.x) {
        const int pl = fdiv((int)e, dHoWo), rem = (int)e - pl * Ho * Wo;
        const int oh = fdiv(rem, dWo), ow = rem - oh * Wo;
        const u32x4 *src = in + ((size_t)pl * H + oh * S) * W + ow * S;
        float m[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) m[k] = -__builtin_inff();
        auto take = [&](const u32x4 v) {
            m[0] = fmaxf(m[0], bf_lo(v.x)); m[1] = fmaxf(m[1], bf_hi(v.x));
            m[2] = fmaxf(m[2], bf_lo(v.y)); m[3] = fmaxf(m[3], bf_hi(v.y));
            m[4] = fmaxf(m[4], bf_lo(v.z)); m[5] = fmaxf(m[5], bf_hi(v.z));
            m[6] = fmaxf(m[6], bf_lo(v.w)); m[7] = fmaxf(m[7], bf_hi(v.w));
        };
        if constexpr (KT > 0) {
            u32x4 v[KT * KT];
#pragma unroll
            for (int i = 0; i < KT; ++i)
#pragma unroll
                for (int jx = 0; jx < KT; ++jx) v[i * KT + jx] = src[i * W + jx];
#pragma unroll
            for (int q = 0; q < KT * KT; ++q) take(v[q]);
        } else {
            for (int i = 0; i < K; ++i)
                for (int jx = 0; jx < K; ++jx) take(src[i * W + jx]);
        }
        // the maxima are bfloat16 values already: keeping the upper halves is exact
        u32x4 o;
        o.x = (__builtin_bit_cast(uint32_t, m[0]) >> 16) | (__builtin_bit_cast(uint32_t, m[1]) & 0xffff0000u);
        o.y = (__builtin_bit_cast(uint32_t, m[2]) >> 16) | (__builtin_bit_cast(uint32_t, m[3]) & 0xffff0000u);
        o.z = (__builtin_bit_cast(uint32_t, m[4]) >> 16) | (__builtin_bit_cast(uint32_t, m[5]) & 0xffff0000u);
        o.w = (__builtin_bit_cast(uint32_t, m[6]) >> 16) | (__builtin_bit_cast(uint32_t, m[7]) & 0xffff0000u);
        out[e] = o;
    }
}

// Global average pooling of a blocked map into fp32 [N][C]: one wavefront per (image, layer block).
// IT: the plane has at most 64*IT pixels and a lane issues its IT loads before the first sum (a zero element adds
// nothing, so the sums are those of the loop); 0 = any size, a loop.
template <int IT>
__global__ __launch_bounds__(256) void avgpool_blocked_kernel(const u32x4 *in, float *out, int planes, int C, int CB, int HW,
                                                              FastDiv dCB)
{
    const int lane = threadIdx.x & 63;
    const int pl = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (pl >= planes) return;
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    auto add = [&](const u32x4 v) {
        s[0] += bf_lo(v.x); s[1] += bf_hi(v.x); s[2] += bf_lo(v.y); s[3] += bf_hi(v.y);
        s[4] += bf_lo(v.z); s[5] += bf_hi(v.z); s[6] += bf_lo(v.w); s[7] += bf_hi(v.w);
    };
    if constexpr (IT > 0) {
        u32x4 v[IT];
#pragma unroll
        for (int j = 0; j < IT; ++j) {
            const int pix = lane + 64 * j;
            v[j] = pix < HW ? in[(size_t)pl * HW + pix] : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int j = 0; j < IT; ++j) add(v[j]);
    } else {
        for (int pix = lane; pix < HW; pix += 64) add(in[(size_t)pl * HW + pix]);
    }
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) s[k] += __shfl_xor(s[k], d, 64);
    if (lane < 8) {
        const int n = fdiv(pl, dCB), cb = pl - n * CB, c = cb * 8 + lane;
        float v = s[0];
#pragma unroll
        for (int k = 1; k < 8; ++k) v = lane == k ? s[k] : v;
        if (c < C) out[(size_t)n * C + c] = v / (float)HW;
    }
}

}  // namespace blocked

// ------------------------------------------------------------------------------ host side
using namespace blocked;

namespace {

int grid_for(long long total, int threads)
{
    long long b = (total + threads - 1) / threads;
    const long long cap = 256ll * 32;
    if (b > cap) b = cap;
    if (b < 1) b = 1;
    return (int)b;
}

typedef void (*BlockedConvFn)(const ConvParams, const ConvParams, int);
template <int CB, int PB, bool F32OUT = false> BlockedConvFn conv_fn(int D)
{
    switch (D) {
        case 4: return conv_blocked_kernel<CB, PB, 4, F32OUT>;
        case 3: return conv_blocked_kernel<CB, PB, 3, F32OUT>;
        case 2: return conv_blocked_kernel<CB, PB, 2, F32OUT>;
        default: return conv_blocked_kernel<CB, PB, 1, F32OUT>;
    }
}

bool allow_lds(BlockedConvFn fn) { return allow_big_lds((const void *)fn); }

}  // namespace

// Tuning hooks (not part of the public interface): ring depth to use where it divides the step count;
// blocks of 32 output layers per workgroup and of 32 pixels per wavefront tile (0 = automatic).
thread_local int g_force_depth = 0, g_force_cb = 0, g_force_pb = 0;
extern "C" void sq_tune_blocked_force_depth(int d) { g_force_depth = d; }
extern "C" void sq_tune_blocked_force_tile(int cb, int pb) { g_force_cb = cb; g_force_pb = pb; }

size_t blocked_map_bytes(int N, int C, int H, int W) { return (size_t)N * ((C + 7) / 8) * H * W * 16; }

size_t blocked_packed_kernel_bytes(int Cout, int Cin, int K)
{
    return (size_t)((Cout + 31) / 32) * K * K * ((Cin + 15) / 16) * 64 * 16;
}

int blocked_pack_map(const void *in, int dtype, void *out, int N, int C, int H, int W)
{
    const int CB = (C + 7) / 8, HW = H * W;
    const long long total = (long long)N * CB * HW;
    if (total >= (1ll << 31)) return SQ_ERR_UNSUPPORTED;
    LaunchScope scope("pack_map", 0.0, (dtype == SQ_BF16 ? 2.0 : 4.0) * N * C * HW + 16.0 * total);
    const long long chunks = (HW + kPackChunk - 1) / kPackChunk, items = (long long)N * CB * chunks;
    if (dtype == SQ_BF16 && (reinterpret_cast<uintptr_t>(in) & 15) == 0 && items < (1ll << 31) && (long long)N * CB * 8 * HW < (1ll << 30)) {
        hipLaunchKernelGGL(pack_map_bf16_kernel, dim3((unsigned)std::min<long long>(items, 256ll * 16)), dim3(256), 0, current_stream(),
                           (const uint16_t *)in, (u32x4 *)out, C, HW, CB, (int)chunks, (int)items, make_fastdiv((int)chunks), make_fastdiv(CB),
                           (uint32_t)((long long)N * C * HW * 2));
        return check_launch();
    }
    if (dtype == SQ_BF16)
        hipLaunchKernelGGL(pack_map_kernel<uint16_t>, dim3(grid_for(total, 256)), dim3(256), 0, current_stream(),
                           (const uint16_t *)in, (u32x4 *)out, N, C, HW, CB, make_fastdiv(HW), make_fastdiv(CB));
    else
        hipLaunchKernelGGL(pack_map_kernel<float>, dim3(grid_for(total, 256)), dim3(256), 0, current_stream(),
                           (const float *)in, (u32x4 *)out, N, C, HW, CB, make_fastdiv(HW), make_fastdiv(CB));
    return check_launch();
}

int blocked_unpack_map(const void *in, float *out, int N, int C, int H, int W)
{
    const int CB = (C + 7) / 8, HW = H * W;
    const long long total = (long long)N * CB * HW;
    if (total >= (1ll << 31)) return SQ_ERR_UNSUPPORTED;
    LaunchScope scope("unpack_map", 0.0, 4.0 * N * C * HW + 16.0 * total);
    hipLaunchKernelGGL(unpack_map_kernel, dim3(grid_for(total, 256)), dim3(256), 0, current_stream(), (const u32x4 *)in, out, N,
                       C, HW, CB, make_fastdiv(HW), make_fastdiv(CB));
    return check_launch();
}

int blocked_pack_kernels(const void *w, int dtype, void *packed, int Cout, int Cin, int K)
{
    const int G = (Cin + 15) / 16, KK = K * K;
    const long long total = (long long)((Cout + 31) / 32) * KK * G * 64;
    if (total >= (1ll << 31)) return SQ_ERR_UNSUPPORTED;
    LaunchScope scope("pack_kernels", 0.0, (dtype == SQ_BF16 ? 2.0 : 4.0) * Cout * Cin * KK + 16.0 * total);
    if (dtype == SQ_BF16)
        hipLaunchKernelGGL(pack_kernels_kernel<uint16_t>, dim3(grid_for(total, 256)), dim3(256), 0, current_stream(),
                           (const uint16_t *)w, (u32x4 *)packed, Cout, Cin, KK, G, (int)total);
    else
        hipLaunchKernelGGL(pack_kernels_kernel<float>, dim3(grid_for(total, 256)), dim3(256), 0, current_stream(),
                           (const float *)w, (u32x4 *)packed, Cout, Cin, KK, G, (int)total);
    return check_launch();
}

// Whether the blocked convolution kernel covers this shape (the checks need no GPU).
bool blocked_conv_supported(int Cin, int Cout, int K, int P)
{
    if (K < 1 || K > 5 || (K & 1) == 0 || P != (K - 1) / 2) return false;
    if (Cin % 16 != 0 || Cout % 8 != 0) return false;
    // kernels of 32 output layers must fit LDS with room for a second workgroup
    const size_t per_mb = (size_t)K * K * (Cin / 16) * 64 * 16;
    return per_mb + 256 <= (size_t)mfma::kLdsBytes / 2;
}

namespace {

struct ConvPlan {
    ConvParams p;
    int CB, PB, D;
    size_t per_mb;     // bytes of packed kernels per 32 output layers
    double flops, bytes;
};

// Fills the launch parameters of one convolution; CB/PB/D = 0 lets this function choose.
int plan_conv(ConvPlan &pl, const void *in, const void *wp, const float *b, void *out, int N, int Cin, int H, int W, int Cout,
              int K, int P, int relu, int ldc_channels, int c_offset, int CB, int PB, int D, bool f32_out = false)
{
    if (!blocked_conv_supported(Cin, Cout, K, P)) return SQ_ERR_UNSUPPORTED;
    if (!f32_out && (ldc_channels % 8 != 0 || c_offset % 8 != 0)) return SQ_ERR_UNSUPPORTED;
    const long long in_bytes = (long long)blocked_map_bytes(N, Cin, H, W);
    const long long out_bytes = f32_out ? (long long)N * ldc_channels * H * W * 4 : (long long)blocked_map_bytes(N, ldc_channels, H, W);
    const long long PT = (long long)N * H * W;
    if (in_bytes >= (1ll << 31) || out_bytes >= (1ll << 31) || PT >= (1ll << 30)) return SQ_ERR_UNSUPPORTED;

    ConvParams &p = pl.p;
    p.in = in; p.wp = wp; p.b = b; p.out = out;
    p.in_bytes = (uint32_t)in_bytes; p.out_bytes = (uint32_t)out_bytes;
    p.wp_elems = (uint32_t)(blocked_packed_kernel_bytes(Cout, Cin, K) / 16);
    p.N = N; p.Cin = Cin; p.H = H; p.W = W; p.HW = H * W; p.Cout = Cout; p.K = K; p.P = P; p.relu = relu;
    p.Hin = H; p.Win = W;
    p.G = Cin / 16;
    p.steps = K * K * p.G;
    p.ldcb = f32_out ? ldc_channels : ldc_channels / 8; p.coffb = f32_out ? c_offset : c_offset / 8;
    p.PT = (int)PT;
    p.dHW = make_fastdiv(p.HW); p.dW = make_fastdiv(W); p.dG = make_fastdiv(p.G); p.dK = make_fastdiv(K);

    // 64 output layers per workgroup when their kernels fit half the LDS, else 32
    pl.per_mb = (size_t)p.steps * 64 * 16;
    const bool two_fit = 2 * pl.per_mb + 512 <= (size_t)mfma::kLdsBytes / 2;
    if (CB == 0) CB = (Cout > 32 && two_fit) ? 2 : 1;
    if (CB == 2 && !two_fit) return SQ_ERR_UNSUPPORTED;
    // wavefront tiles of 32 pixels: measured equal to or faster than 64 on every layer of the network; with fp32 NCHW
    // results 64 pixels (256-byte runs per layer and store) are 3-20 % faster at batch 256
    if (PB == 0) PB = f32_out ? 2 : 1;
    if (g_force_cb == 1 || (g_force_cb == 2 && two_fit)) CB = g_force_cb;
    if (g_force_pb == 1 || g_force_pb == 2) PB = g_force_pb;
    if (D == 0) {
        D = p.steps % 4 == 0 ? 4 : p.steps % 3 == 0 ? 3 : p.steps % 2 == 0 ? 2 : 1;
        if (g_force_depth > 0 && p.steps % g_force_depth == 0) D = g_force_depth;
    }
    if (p.steps % D != 0) return SQ_ERR_UNSUPPORTED;
    pl.CB = CB; pl.PB = PB; pl.D = D;
    p.tiles = (int)((PT + 32 * PB - 1) / (32 * PB));
    p.ncblk = (Cout + 32 * CB - 1) / (32 * CB);
    p.dNcblk = make_fastdiv(p.ncblk);
    pl.flops = 2.0 * N * Cout * H * W * (double)Cin * K * K;
    pl.bytes = 2.0 * ((double)N * Cin * H * W + (double)Cout * Cin * K * K) + (f32_out ? 4.0 : 2.0) * N * Cout * H * W + 4.0 * Cout;
    return SQ_OK;
}

BlockedConvFn kernel_for(int CB, int PB, int D, bool f32_out = false)
{
    if (f32_out) return CB == 2 ? (PB == 2 ? conv_fn<2, 2, true>(D) : conv_fn<2, 1, true>(D)) : (PB == 2 ? conv_fn<1, 2, true>(D) : conv_fn<1, 1, true>(D));
    return CB == 2 ? (PB == 2 ? conv_fn<2, 2>(D) : conv_fn<2, 1>(D)) : (PB == 2 ? conv_fn<1, 2>(D) : conv_fn<1, 1>(D));
}

// workgroups a convolution can use: a multiple of its layer groups, at most `cap`, no more than its tiles need
long long slots_for(const ConvPlan &pl, long long cap)
{
    long long slots = cap / pl.p.ncblk;
    const long long need = (pl.p.tiles + kWaves - 1) / kWaves;
    if (slots > need) slots = need;
    return slots < 1 ? 1 : slots;
}

// the profiler keeps the pointer: one permanent string per shape of launch
const char *launch_name(int K, int CB, int PB, int D, int kind)   // kind: 0 one convolution, 1 expand pair, 2 fp32 NCHW out
{
    // filled once (function-local statics are initialised under a lock), read-only afterwards
    struct Names {
        char n[3][6][3][3][5][28];
        Names()
        {
            static const char *const fmt[3] = {"k%db_%dx%d_d%d", "k1b+k%db_%dx%d_d%d", "k%db_%dx%d_d%d_f32out"};
            for (int pr = 0; pr < 3; ++pr)
                for (int k = 0; k < 6; ++k)
                    for (int cb = 0; cb < 3; ++cb)
                        for (int pb = 0; pb < 3; ++pb)
                            for (int d = 0; d < 5; ++d)
                                snprintf(n[pr][k][cb][pb][d], sizeof n[0][0][0][0][0], fmt[pr], k, 32 * cb, 32 * pb, d);
        }
    };
    static const Names names;
    return names.n[kind][K][CB][PB][D];
}

}  // namespace

// f32_out: `out` is an fp32 NCHW map of ldc_channels layers (results unrounded) instead of a blocked bfloat16 one
int blocked_conv(const void *in, const void *wp, const float *b, void *out, int N, int Cin, int H, int W, int Cout, int K, int P,
                 int relu, int ldc_channels, int c_offset, bool f32_out)
{
    ConvPlan pl;
    const int rc = plan_conv(pl, in, wp, b, out, N, Cin, H, W, Cout, K, P, relu, ldc_channels, c_offset, 0, 0, 0, f32_out);
    if (rc) return rc;
    BlockedConvFn fn = kernel_for(pl.CB, pl.PB, pl.D, f32_out);
    if (!allow_lds(fn)) {
        const int e = check_launch();
        return e ? e : SQ_ERR_HIP;
    }
    // persistent: at most two workgroups per CU
    const long long wgs = slots_for(pl, 2ll * num_cus()) * pl.p.ncblk;
    const size_t lds = (size_t)pl.CB * pl.per_mb + (size_t)pl.CB * 32 * sizeof(float);
    LaunchScope scope(launch_name(K, pl.CB, pl.PB, pl.D, f32_out ? 2 : 0), pl.flops, pl.bytes);
    hipLaunchKernelGGL(fn, dim3((unsigned)wgs), dim3(kThreads), lds, current_stream(), pl.p, pl.p, (int)wgs);
    return check_launch();
}

// The two expands of a fire layer in one launch: a 1x1 convolution (w1, b1 -> layers [c_offset1, +Cout1)) and a K x K
// convolution (wk, bk -> layers [c_offsetk, +Coutk)) of the same input into the same output map.
int blocked_conv_pair(const void *in, const void *wp1, const float *b1, int Cout1, int c_offset1, const void *wpk,
                      const float *bk, int Coutk, int c_offsetk, int K, void *out, int N, int Cin, int H, int W, int relu,
                      int ldc_channels)
{
    ConvPlan p1, pk;
    int rc = plan_conv(pk, in, wpk, bk, out, N, Cin, H, W, Coutk, K, (K - 1) / 2, relu, ldc_channels, c_offsetk, 0, 0, 0);
    if (rc) return rc;
    // the ring depth must divide both step counts; the 1x1 has the fewer steps
    const int G = Cin / 16;
    const int D = G % 4 == 0 ? 4 : G % 3 == 0 ? 3 : G % 2 == 0 ? 2 : 1;
    if ((rc = plan_conv(pk, in, wpk, bk, out, N, Cin, H, W, Coutk, K, (K - 1) / 2, relu, ldc_channels, c_offsetk, pk.CB, pk.PB, D)))
        return rc;
    if ((rc = plan_conv(p1, in, wp1, b1, out, N, Cin, H, W, Cout1, 1, 0, relu, ldc_channels, c_offset1, pk.CB, pk.PB, D))) return rc;
    BlockedConvFn fn = kernel_for(pk.CB, pk.PB, D);
    if (!allow_lds(fn)) {
        const int e = check_launch();
        return e ? e : SQ_ERR_HIP;
    }
    // Workgroups are shared out between the two parts so that both finish together.  The K x K part has K*K times
    // the MFMA steps, but both write the same number of bytes and a tile's time is mostly its stores and its
    // fixed part: measured on whole passes at batches 1 to 256, a fifth of the workgroups for the 1x1 part is
    // best (8 % faster at batches 64 and 256 than the share by steps, a tenth; no slower at any batch).
    const long long cap = 2ll * num_cus();
    long long cap1 = K == 1 ? cap / 2 : cap * Cout1 / (Cout1 + 4ll * Coutk);
    if (cap1 < p1.p.ncblk) cap1 = p1.p.ncblk;
    const long long wg1 = slots_for(p1, cap1) * p1.p.ncblk;
    const long long wgk = slots_for(pk, cap - wg1 > pk.p.ncblk ? cap - wg1 : pk.p.ncblk) * pk.p.ncblk;
    const size_t ldsk = (size_t)pk.CB * pk.per_mb, lds1 = (size_t)p1.CB * p1.per_mb;
    const size_t lds = (ldsk > lds1 ? ldsk : lds1) + (size_t)pk.CB * 32 * sizeof(float);
    LaunchScope scope(launch_name(K, pk.CB, pk.PB, D, 1), p1.flops + pk.flops, p1.bytes + pk.bytes - 2.0 * N * Cin * H * W);
    hipLaunchKernelGGL(fn, dim3((unsigned)(wg1 + wgk)), dim3(kThreads), lds, current_stream(), p1.p, pk.p, (int)wg1);
    return check_launch();
}

// 3x3 stride-2 max pooling of a blocked map of Cin layers (Hin x Win) followed by a 1x1 convolution to Cout layers,
// in one launch; the pooled map is never written.
int blocked_pool_conv(const void *in, const void *wp, const float *b, void *out, int N, int Cin, int Hin, int Win, int Cout,
                      int relu, int ldc_channels, int c_offset)
{
    if (Hin < 3 || Win < 3) return SQ_ERR_SHAPE;
    const int H = (Hin - 3) / 2 + 1, W = (Win - 3) / 2 + 1;
    ConvPlan pl;
    // planned on the pooled extents (they are the output's); the input side is patched afterwards
    int rc = plan_conv(pl, in, wp, b, out, N, Cin, H, W, Cout, 1, 0, relu, ldc_channels, c_offset, 0, 1, 0);
    if (rc) return rc;
    const long long in_bytes = (long long)blocked_map_bytes(N, Cin, Hin, Win);
    if (in_bytes >= (1ll << 31)) return SQ_ERR_UNSUPPORTED;
    pl.p.in_bytes = (uint32_t)in_bytes;
    pl.p.Hin = Hin; pl.p.Win = Win;
    // nine 16-byte loads per lane and step: two steps in flight is what the registers hold
    const int D = pl.p.steps % 2 == 0 ? 2 : 1;
    typedef void (*PoolConvFn)(const ConvParams);
    PoolConvFn fn = pl.CB == 2 ? (D == 2 ? pool_conv_blocked_kernel<2, 2> : pool_conv_blocked_kernel<2, 1>)
                               : (D == 2 ? pool_conv_blocked_kernel<1, 2> : pool_conv_blocked_kernel<1, 1>);
    if (!allow_big_lds((const void *)fn)) {
        const int e = check_launch();
        return e ? e : SQ_ERR_HIP;
    }
    const long long wgs = slots_for(pl, 2ll * num_cus()) * pl.p.ncblk;
    const size_t lds = (size_t)pl.CB * pl.per_mb + (size_t)pl.CB * 32 * sizeof(float);
    static const char *const names[3][3] = {{"", "", ""},
                                            {"", "pool3s2+k1b_32x32_d1", "pool3s2+k1b_32x32_d2"},
                                            {"", "pool3s2+k1b_64x32_d1", "pool3s2+k1b_64x32_d2"}};
    LaunchScope scope(names[pl.CB][D], pl.flops, 2.0 * ((double)N * Cin * Hin * Win + (double)Cout * Cin + (double)N * Cout * H * W) + 4.0 * Cout);
    hipLaunchKernelGGL(fn, dim3((unsigned)wgs), dim3(kThreads), lds, current_stream(), pl.p);
    return check_launch();
}

// Every kernel of this file whose launch may ask for more dynamic LDS than the default limit.
bool blocked_register_kernels()
{
    bool ok = true;
    for (int cb = 1; cb <= 2; ++cb)
        for (int pb = 1; pb <= 2; ++pb)
            for (int d = 1; d <= 4; ++d) ok &= allow_big_lds((const void *)kernel_for(cb, pb, d)) && allow_big_lds((const void *)kernel_for(cb, pb, d, true));
    ok &= allow_big_lds((const void *)pool_conv_blocked_kernel<1, 1>) && allow_big_lds((const void *)pool_conv_blocked_kernel<1, 2>) &&
          allow_big_lds((const void *)pool_conv_blocked_kernel<2, 1>) && allow_big_lds((const void *)pool_conv_blocked_kernel<2, 2>);
    return ok;
}

// ---- a convolution with bfloat16 NCHW operands on these kernels (see sq_internal.h) ---------------------------
namespace {
bool bf16_mfma_conv1_type(int Cin, int Cout, int K, int S) { return Cin == 3 && K == 7 && S == 2 && Cout <= 96 && Cout % 8 == 0; }
}

size_t conv_bf16_mfma_workspace_bytes(int N, int Cin, int H, int W, int Cout, int K, int S, int P, int out_channels)
{
    if (N <= 0 || Cin <= 0 || Cout <= 0 || H <= 0 || W <= 0 || P < 0 || H + 2 * P < K || W + 2 * P < K) return 0;
    const long long Ho = (H + 2 * P - K) / S + 1, Wo = (W + 2 * P - K) / S + 1;
    if ((long long)N * out_channels * Ho * Wo * 4 >= (1ll << 31) || (long long)N * Ho * Wo >= (1ll << 30)) return 0;
    if (bf16_mfma_conv1_type(Cin, Cout, K, S)) {
        if ((long long)N * 3 * H * W * 2 >= (1ll << 31)) return 0;
        return align_up(blocked_packed_kernel7_bytes(), 256);
    }
    if (S != 1 || !blocked_conv_supported(Cin, Cout, K, P)) return 0;
    // 1x1 layers: re-ordering the input and writing fp32 costs more than the matrix cores save unless the contraction is
    // long and the layer widens (measured at batch 256: 512 -> 1000 at 13x13 369 -> 137 us, 64 -> 256 at 27x27 70 -> 77 us)
    if (K == 1 && (Cout <= Cin || Cin < 128)) return 0;
    if ((long long)blocked_map_bytes(N, Cin, H, W) >= (1ll << 31)) return 0;
    return align_up(blocked_map_bytes(N, Cin, H, W), 256) + align_up(blocked_packed_kernel_bytes(Cout, Cin, K), 256);
}

int conv_bf16_mfma(const ConvArgs &a)
{
    if (a.dtype != SQ_BF16 || a.pool_H || a.cp_in || a.cp_out) return SQ_ERR_UNSUPPORTED;
    const size_t need = conv_bf16_mfma_workspace_bytes(a.N, a.Cin, a.H, a.W, a.Cout, a.K, a.S, a.P, a.out_channels);
    if (!need) return SQ_ERR_UNSUPPORTED;
    if (!a.ws || ((uintptr_t)a.ws & 255) || a.ws_bytes < need) return SQ_ERR_WORKSPACE;
    int rc;
    if (bf16_mfma_conv1_type(a.Cin, a.Cout, a.K, a.S)) {
        if ((rc = blocked_pack_kernels7(a.w, SQ_BF16, a.ws, a.Cout))) return rc;
        return blocked_conv7s2(a.in, SQ_BF16, a.ws, a.b, a.out, a.N, a.H, a.W, a.Cout, a.P, a.relu, a.out_channels, a.c_offset, true);
    }
    char *map = (char *)a.ws, *wp = map + align_up(blocked_map_bytes(a.N, a.Cin, a.H, a.W), 256);
    if ((rc = blocked_pack_map(a.in, SQ_BF16, map, a.N, a.Cin, a.H, a.W))) return rc;
    if ((rc = blocked_pack_kernels(a.w, SQ_BF16, wp, a.Cout, a.Cin, a.K))) return rc;
    return blocked_conv(map, wp, a.b, a.out, a.N, a.Cin, a.H, a.W, a.Cout, a.K, a.P, a.relu, a.out_channels, a.c_offset, true);
}

int blocked_maxpool(const void *in, void *out, int N, int C, int H, int W, int K, int S)
{
    const int Ho = (H - K) / S + 1, Wo = (W - K) / S + 1, planes = N * ((C + 7) / 8);
    const long long total = (long long)planes * Ho * Wo;
    if (total >= (1ll << 31) || (long long)planes * H * W >= (1ll << 31)) return SQ_ERR_UNSUPPORTED;
    LaunchScope scope("maxpool_blocked", 0.0, 16.0 * ((double)planes * H * W + (double)total));
    auto kernel = maxpool_blocked_kernel<0, 0>;
    if (K == 3 && S == 2) kernel = maxpool_blocked_kernel<3, 2>;
    hipLaunchKernelGGL(kernel, dim3(grid_for(total, 256)), dim3(256), 0, current_stream(), (const u32x4 *)in, (u32x4 *)out,
                       planes, H, W, Ho, Wo, K, S, make_fastdiv(Wo), make_fastdiv(Ho * Wo));
    return check_launch();
}

int blocked_avgpool_global(const void *in, float *out, int N, int C, int H, int W)
{
    const int CB = (C + 7) / 8, planes = N * CB;
    if ((long long)planes * H * W >= (1ll << 31)) return SQ_ERR_UNSUPPORTED;
    LaunchScope scope("avgpool_blocked", 0.0, 16.0 * (double)planes * H * W + 4.0 * N * C);
    const int IT = (H * W + 63) / 64;
    auto kernel = avgpool_blocked_kernel<0>;
    if (IT == 1) kernel = avgpool_blocked_kernel<1>;
    else if (IT == 2) kernel = avgpool_blocked_kernel<2>;
    else if (IT == 3) kernel = avgpool_blocked_kernel<3>;
    else if (IT == 4) kernel = avgpool_blocked_kernel<4>;
    hipLaunchKernelGGL(kernel, dim3((planes + 3) / 4), dim3(256), 0, current_stream(), (const u32x4 *)in, out,
                       planes, C, CB, H * W, make_fastdiv(CB));
    return check_launch();
}

}  // namespace sq
