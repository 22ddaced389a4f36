// A whole fire layer in one launch, reduced-precision path (section "Convolutional Neural
// Networks": one squeeze and two expand convolutions; blocked bfloat16 maps and packed
// kernels as in blocked_bf16.hip).  For small batches, where a pass over the network is
// bound by the number of launches and by the latency of each, not by arithmetic.
//
// A workgroup owns a band of TH output rows of one image and one slice of 64 expand
// layers (of the 1x1 or of the 3x3 expand).
//   phase A: the squeeze map of the band plus one halo row above and below is computed
//            into LDS as a blocked map [Csq/8][(TH+2) x (W+2)][8] whose border (image
//            rows outside the image, one column left and right) is zero -- the zero padding
//            of the 3x3, so phase B needs no tests.  B operands come straight from global
//            memory, A operands (packed squeeze kernels) too: nothing is staged.
//   phase B: the slice's 1x1 or 3x3 expand of that map.  B operands are 16-byte LDS reads
//            at the tap's shift, A operands (packed expand kernels) come from global memory.
// Every slice recomputes the squeeze of its band (1/8 to 1/2 of the slice's own work) and
// every band its two halo rows; in exchange the squeeze map never goes to memory and the
// layer is one launch instead of two.  The arithmetic of every output is the same as in
// the separate kernels (same order of steps, bias as the start value, one rounding of the
// squeeze map), so the results are bit-identical to theirs.
#include "conv_mfma_common.h"

namespace sq {
namespace blocked {

using namespace mfma;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kFireThreads = 512, kFireWaves = kFireThreads / 64;
constexpr int kRing = 4;     // steps in flight; step counts are padded to a multiple with zero operands

struct FireParams {
    const void *in;                      // blocked [N][Cin/8][H][W][8]
    const void *wp_sq, *wp_e1, *wp_e3;   // packed kernels
    const float *b_sq, *b_e1, *b_e3;     // biases or nullptr
    void *out;                           // blocked [N][(Ce1+Ce3)/8][H][W][8]
    uint32_t in_bytes, out_bytes, wsq_bytes, we1_bytes, we3_bytes;
    int N, Cin, H, W, HW, Csq, Ce1, Ce3;
    int Gin, Gsq;          // Cin / 16, Csq / 16
    int TH, bands;         // output rows per band, bands per image
    int nsl1, nsl3;        // slices of 64 layers of the 1x1 and of the 3x3 expand
    int ldcb;              // (Ce1 + Ce3) / 8
    int Wp, Plds;          // W + 2, (TH + 2) * Wp
    FastDiv dW, dBands, dSlices;
};

// 16-byte load through a buffer resource as four adjacent dwords (merged by the compiler)
__device__ __forceinline__ bf16x8 ld16(rsrc_t r, uint32_t lane_off, uint32_t uni_off)
{
    asm volatile("" : "+v"(lane_off));
    f32x4 v = {buf_ld(r, lane_off, uni_off), buf_ld(r, lane_off + 4u, uni_off), buf_ld(r, lane_off + 8u, uni_off),
               buf_ld(r, lane_off + 12u, uni_off)};
    return __builtin_bit_cast(bf16x8, v);
}

// CBS = blocks of 32 squeeze layers (1: Csq <= 32, 2: Csq <= 64)
template <int CBS>
__global__ __launch_bounds__(kFireThreads, 1) void fire_blocked_kernel(const FireParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    u32x4 *const smap = reinterpret_cast<u32x4 *>(smem);       // [Csq/8][Plds] elements of 16 bytes

    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int j = lane & 31, h = lane >> 5;
    const int nsl = p.nsl1 + p.nsl3;
    const int tb = fdiv((int)blockIdx.x, p.dSlices), slice = (int)blockIdx.x - tb * nsl;   // (image, band), slice
    const int n = fdiv(tb, p.dBands), band = tb - n * p.bands;
    const int r0 = band * p.TH;                               // first output row of the band

    // ---- zero the LDS map (its border is the zero padding of the 3x3)
    {
        const int total = (p.Csq >> 3) * p.Plds;
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int e = t; e < total; e += kFireThreads) smap[e] = z;
    }
    __syncthreads();

    const rsrc_t rin = make_rsrc(p.in, p.in_bytes);
    const uint32_t hw16 = (uint32_t)p.HW * 16u;

    // ---- phase A: squeeze of rows r0-1 .. r0+TH into LDS -----------------------------------------
    {
        const rsrc_t rw = make_rsrc(p.wp_sq, p.wsq_bytes);
        const int steps = p.Gin, steps_pad = (steps + kRing - 1) / kRing * kRing;
        const int npix = (p.TH + 2) * p.W, nblk = (npix + 31) >> 5;
        for (int blk = wv; blk < nblk; blk += kFireWaves) {
            const int q = blk * 32 + j;
            const int i = fdiv(q < npix ? q : 0, p.dW), x = (q < npix ? q : 0) - i * p.W;
            const int row = r0 - 1 + i;                        // image row of LDS row i
            const bool ok = q < npix && row >= 0 && row < p.H;
            const uint32_t ibase = ok ? (uint32_t)((n * (p.Cin >> 3) + h) * p.HW + row * p.W + x) * 16u : kOob;

            bf16x8 bx[kRing], ax[kRing][CBS];
            auto issue = [&](int ring, int s_) {
                const int s = __builtin_amdgcn_readfirstlane(s_);
                const bool live = s < steps;                   // padded steps read zeros
                bx[ring] = ld16(rin, live ? ibase : kOob, live ? (uint32_t)s * 2u * hw16 : 0u);
#pragma unroll
                for (int cb = 0; cb < CBS; ++cb)
                    ax[ring][cb] = ld16(rw, live ? (uint32_t)lane * 16u : kOob, live ? (uint32_t)(cb * steps + s) * 1024u : 0u);
            };
#pragma unroll
            for (int r = 0; r < kRing; ++r) issue(r, r);
            f32x16 acc[CBS];
#pragma unroll
            for (int cb = 0; cb < CBS; ++cb)
#pragma unroll
                for (int qq = 0; qq < 4; ++qq)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int m = cb * 32 + 8 * qq + 4 * h + e;
                        acc[cb][4 * qq + e] = (p.b_sq && m < p.Csq) ? p.b_sq[m] : 0.f;
                    }
            for (int s0 = 0; s0 < steps_pad; s0 += kRing) {
#pragma unroll
                for (int r = 0; r < kRing; ++r) {
#pragma unroll
                    for (int cb = 0; cb < CBS; ++cb)
                        acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ax[r][cb], bx[r], acc[cb], 0, 0, 0);
                    issue(r, s0 + r + kRing);                  // past the last step: zeros, never used
                }
            }
            // ReLU, round, into the LDS map at (row i, column x + 1); rows outside the image stay zero
            if (ok) {
                const int lpix = i * p.Wp + x + 1;
#pragma unroll
                for (int cb = 0; cb < CBS; ++cb)
#pragma unroll
                    for (int qq = 0; qq < 4; ++qq) {
                        const int lb = cb * 4 + qq;
                        if (lb * 8 < p.Csq) {
                            const float v0 = fmaxf(acc[cb][4 * qq + 0], 0.f), v1 = fmaxf(acc[cb][4 * qq + 1], 0.f);
                            const float v2 = fmaxf(acc[cb][4 * qq + 2], 0.f), v3 = fmaxf(acc[cb][4 * qq + 3], 0.f);
                            uint32_t *dst = reinterpret_cast<uint32_t *>(smap + lb * p.Plds + lpix) + 2 * h;
                            dst[0] = pack_bf16x2(v0, v1);
                            dst[1] = pack_bf16x2(v2, v3);
                        }
                    }
            }
        }
    }
    __syncthreads();

    // ---- phase B: this slice's expand of the LDS map ---------------------------------------------
    {
        const bool is3 = slice >= p.nsl1;                       // uniform
        const int sl = is3 ? slice - p.nsl1 : slice;            // slice of 64 layers inside its convolution
        const rsrc_t rw = make_rsrc(is3 ? p.wp_e3 : p.wp_e1, is3 ? p.we3_bytes : p.we1_bytes);
        const rsrc_t rout = make_rsrc(p.out, p.out_bytes);
        const float *bias = is3 ? p.b_e3 : p.b_e1;
        const int Cout = is3 ? p.Ce3 : p.Ce1;
        const int coffb = is3 ? (p.Ce1 >> 3) : 0;
        const int K = is3 ? 3 : 1, KK = K * K;
        const int steps = KK * p.Gsq, steps_pad = (steps + kRing - 1) / kRing * kRing;
        const int npix = p.TH * p.W, nblk = (npix + 31) >> 5;
        for (int blk = wv; blk < nblk; blk += kFireWaves) {
            const int q = blk * 32 + j;
            const int y = fdiv(q < npix ? q : 0, p.dW), x = (q < npix ? q : 0) - y * p.W;
            const bool ok = q < npix && r0 + y < p.H;
            // LDS element of tap (0, 0) of this pixel, layer block h of a pair (the 1x1 reads the centre)
            const int lbase = h * p.Plds + (is3 ? y * p.Wp + x : (y + 1) * p.Wp + x + 1);
            const uint32_t obase = ok ? (uint32_t)((n * p.ldcb + coffb) * p.HW + (r0 + y) * p.W + x) * 16u + 8u * (uint32_t)h : kOob;

            // (the uniform offset is not part of the buffer range check, so a block of 32 layers past the
            // last one, or a padded step, must be turned away through the lane offset)
            const int nmb = (Cout + 31) >> 5;
            bf16x8 ax[kRing][2];
            auto issue = [&](int ring, int s_) {
                const int s = __builtin_amdgcn_readfirstlane(s_);
#pragma unroll
                for (int cb = 0; cb < 2; ++cb) {
                    const bool live = s < steps && sl * 2 + cb < nmb;
                    ax[ring][cb] = ld16(rw, live ? (uint32_t)lane * 16u : kOob, live ? (uint32_t)((sl * 2 + cb) * steps + s) * 1024u : 0u);
                }
            };
#pragma unroll
            for (int r = 0; r < kRing; ++r) issue(r, r);
            f32x16 acc[2];
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int qq = 0; qq < 4; ++qq)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int m = (sl * 2 + cb) * 32 + 8 * qq + 4 * h + e;
                        acc[cb][4 * qq + e] = (bias && m < Cout) ? bias[m] : 0.f;
                    }
            // position of the step whose B operand is read next: tap (ky, kx), pair of layer blocks g
            int g = 0, ky = 0, kx = 0;
            for (int s0 = 0; s0 < steps_pad; s0 += kRing) {
#pragma unroll
                for (int r = 0; r < kRing; ++r) {
                    // padded steps read a valid element (tap (0,0), pair 0) against zero kernels
                    const bool live = s0 + r < steps;
                    const int el = live ? lbase + 2 * g * p.Plds + ky * p.Wp + kx : lbase;
                    const bf16x8 b = __builtin_bit_cast(bf16x8, smap[el]);
#pragma unroll
                    for (int cb = 0; cb < 2; ++cb)
                        acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ax[r][cb], b, acc[cb], 0, 0, 0);
                    issue(r, s0 + r + kRing);
                    if (++g == p.Gsq) {
                        g = 0;
                        if (++kx == K) {
                            kx = 0;
                            ++ky;
                        }
                    }
                }
            }
#pragma unroll
            for (int cb = 0; cb < 2; ++cb)
#pragma unroll
                for (int qq = 0; qq < 4; ++qq) {
                    const int lb = (sl * 2 + cb) * 4 + qq;
                    if (lb * 8 < Cout) {
                        const float v0 = fmaxf(acc[cb][4 * qq + 0], 0.f), v1 = fmaxf(acc[cb][4 * qq + 1], 0.f);
                        const float v2 = fmaxf(acc[cb][4 * qq + 2], 0.f), v3 = fmaxf(acc[cb][4 * qq + 3], 0.f);
                        buf_st2(rout, obase, (uint32_t)lb * hw16, __builtin_bit_cast(float, pack_bf16x2(v0, v1)),
                                __builtin_bit_cast(float, pack_bf16x2(v2, v3)));
                    }
                }
        }
    }
}

}  // namespace
}  // namespace blocked

using namespace blocked;

// Whether the one-launch fire kernel covers this shape (no GPU needed).
bool blocked_fire_fused_supported(int Cin, int Csq, int Ce1, int Ce3, int W)
{
    if (Cin % 16 != 0 || Csq % 16 != 0 || Csq > 64 || Ce1 % 8 != 0 || Ce3 % 8 != 0) return false;
    // at least one output row plus its halo must fit the LDS
    return (size_t)3 * (W + 2) * Csq * 2 <= (size_t)mfma::kLdsBytes;
}

// Fire layer on blocked maps in one launch; SQ_ERR_UNSUPPORTED where the shape is not covered.
int blocked_fire_fused(const void *in, const void *wp_sq, const float *b_sq, const void *wp_e1, const float *b_e1,
                       const void *wp_e3, const float *b_e3, void *out, int N, int Cin, int H, int W, int Csq, int Ce1,
                       int Ce3)
{
    if (!blocked_fire_fused_supported(Cin, Csq, Ce1, Ce3, W)) return SQ_ERR_UNSUPPORTED;
    const long long in_bytes = (long long)blocked_map_bytes(N, Cin, H, W);
    const long long out_bytes = (long long)blocked_map_bytes(N, Ce1 + Ce3, H, W);
    if (in_bytes >= (1ll << 31) || out_bytes >= (1ll << 31)) return SQ_ERR_UNSUPPORTED;
    FireParams p;
    p.in = in; p.wp_sq = wp_sq; p.wp_e1 = wp_e1; p.wp_e3 = wp_e3; p.b_sq = b_sq; p.b_e1 = b_e1; p.b_e3 = b_e3; p.out = out;
    p.in_bytes = (uint32_t)in_bytes; p.out_bytes = (uint32_t)out_bytes;
    p.wsq_bytes = (uint32_t)blocked_packed_kernel_bytes(Csq, Cin, 1);
    p.we1_bytes = (uint32_t)blocked_packed_kernel_bytes(Ce1, Csq, 1);
    p.we3_bytes = (uint32_t)blocked_packed_kernel_bytes(Ce3, Csq, 3);
    p.N = N; p.Cin = Cin; p.H = H; p.W = W; p.HW = H * W; p.Csq = Csq; p.Ce1 = Ce1; p.Ce3 = Ce3;
    p.Gin = Cin / 16; p.Gsq = Csq / 16;
    p.Wp = W + 2;
    // band height: as many rows as give every CU a workgroup at this batch, within half the LDS
    const size_t row_bytes = (size_t)p.Wp * Csq * 2;
    int TH = (int)((size_t)mfma::kLdsBytes / 2 / row_bytes) - 2;
    if (TH < 1) TH = 1;
    p.nsl1 = (Ce1 + 63) / 64; p.nsl3 = (Ce3 + 63) / 64;
    const int want_bands = (num_cus() + N * (p.nsl1 + p.nsl3) - 1) / (N * (p.nsl1 + p.nsl3));
    int th_par = (H + want_bands - 1) / want_bands;
    if (th_par < 4) th_par = 4;                       // two halo rows per band: keep the recomputation under a half
    if (TH > th_par) TH = th_par;
    if (TH > H) TH = H;
    p.TH = TH;
    p.bands = (H + TH - 1) / TH;
    p.Plds = (TH + 2) * p.Wp;
    p.ldcb = (Ce1 + Ce3) / 8;
    p.dW = make_fastdiv(W); p.dBands = make_fastdiv(p.bands); p.dSlices = make_fastdiv(p.nsl1 + p.nsl3);
    const size_t lds = (size_t)(Csq / 8) * p.Plds * 16;
    if (lds > (size_t)mfma::kLdsBytes) return SQ_ERR_UNSUPPORTED;
    const long long wgs = (long long)N * p.bands * (p.nsl1 + p.nsl3);
    if (wgs >= (1ll << 31)) return SQ_ERR_UNSUPPORTED;
    typedef void (*FireFn)(const FireParams);
    FireFn fn = Csq > 32 ? fire_blocked_kernel<2> : fire_blocked_kernel<1>;
    if (!allow_big_lds((const void *)fn)) {
        const int e = check_launch();
        return e ? e : SQ_ERR_HIP;
    }
    const double px = (double)N * H * W;
    LaunchScope scope(Csq > 32 ? "fire1_bf16_sq64" : "fire1_bf16_sq32", 2.0 * px * ((double)Cin * Csq + (double)Csq * Ce1 + 9.0 * Csq * Ce3),
                      2.0 * (px * (Cin + Ce1 + Ce3) + (double)Cin * Csq + (double)Csq * Ce1 + 9.0 * Csq * Ce3));
    hipLaunchKernelGGL(fn, dim3((unsigned)wgs), dim3(kFireThreads), lds, current_stream(), p);
    return check_launch();
}

bool fire_bf16_register_kernels()
{
    return allow_big_lds((const void *)fire_blocked_kernel<1>) && allow_big_lds((const void *)fire_blocked_kernel<2>);
}

}  // namespace sq
