// conv1-type layer on the fp32 matrix cores: 7x7 kernels, stride 2, three input layers,
// at most 96 output layers (section "Convolutional Neural Networks": the first layer of
// the network reads the 224 x 224 RGB image).
//
// Why it has its own kernel.  The contraction length is 3*49 = 147, which the generic
// kernel can only cover by padding the three input layers to four (196, a third of the
// MFMA work wasted).  Here the two k-values of each v_mfma_f32_32x32x2_f32 are chosen so
// that the LDS offset between the pair is a per-lane constant and only one slot is padding
// (148 = 74 MFMA steps):
//     steps  0..48   tap (i,j) of input layer 0   with the same tap of input layer 1
//     steps 49..69   tap (i,j), i<3, of layer 2   with tap (i+3, j) of layer 2
//     steps 70..72   tap (6,j), j<3, of layer 2   with tap (6, j+3) of layer 2
//     step  73       tap (6,6) of layer 2         with a zero kernel value
// The kernels are stored in LDS in exactly that order (slot 2*step + pair member), so the
// A-operand address is uniform; the B operand uses four per-lane base offsets.
//
// The workgroup is persistent: it stages all 96 x 147 kernel values once, then walks over
// pixel tiles (BN consecutive output pixels of the batch-flattened image, which may
// straddle two images), prefetching the next tile's input patch into registers while the
// MFMAs of the current tile run, and double-buffering the patch in LDS.
#include "conv_mfma_common.h"

namespace sq {
namespace mfma {
namespace {

constexpr int kKS = 7, kS = 2, kKK = 49, kK = 147, kLDK = 149, kBM = 96, kTM = 3;

// LDS slot of kernel value k = (c, i, j) in the pairing order above.
__device__ __forceinline__ int pair_slot(int k)
{
    const int c = k / kKK, tap = k - c * kKK;
    if (c < 2) return 2 * tap + c;
    const int i = tap / kKS, j = tap - i * kKS;
    if (i < 3) return 2 * (49 + tap);
    if (i < 6) return 2 * (49 + tap - 21) + 1;
    if (j < 3) return 2 * (70 + j);
    if (j < 6) return 2 * (70 + j - 3) + 1;
    return 146;
}

template <int BN, int PE, int MINW>
__global__ __launch_bounds__(BN / 32 * 64, MINW) void conv7s2c3_kernel(const KParams p)
{
    using M = Mfma<32>;
    using Acc = typename M::Acc;
    constexpr int NW = BN / 32, NT = NW * 64;

    extern __shared__ float smem[];
    float *const Ws = smem;                 // [96][149]
    float *const Xs = Ws + kBM * kLDK;      // [2][3*plane]
    const int plane = p.plane, LWs = p.LWs;

    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
    const int li = lane & 31, kk = lane >> 5;

    // ---- kernels, once per workgroup -----------------------------------------------------
    for (int e = t; e < kBM * kK; e += NT) {
        const int m = e / kK, k = e - m * kK;
        Ws[m * kLDK + pair_slot(k)] = m < p.Cout ? p.w[e] : 0.f;
    }
    if (t < kBM) {
        Ws[t * kLDK + 147] = 0.f;
        Ws[t * kLDK + 148] = 0.f;
    }

    int aoff[kTM];
#pragma unroll
    for (int x = 0; x < kTM; ++x) aoff[x] = (x * 32 + li) * kLDK + kk;

    // bias of the 48 output layers this lane stores (layer = x*32 + row_reg(r) + row_lane)
    const int lrow = M::row_lane(lane);
    float bias[kTM][16];
#pragma unroll
    for (int x = 0; x < kTM; ++x)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = x * 32 + M::row_reg(r) + lrow;
            bias[x][r] = (p.b && m < p.Cout) ? p.b[m] : 0.f;
        }

    // ---- staging map: element e = t + NT*r of a [rows][LW] plane; row and column of e do
    // not depend on the tile, only the first virtual row va does -------------------------
    int evr[PE], epc[PE];
#pragma unroll
    for (int r = 0; r < PE; ++r) {
        const int e = t + NT * r;
        evr[r] = fdiv(e, p.dLW);
        epc[r] = e - evr[r] * p.LW;
    }

    int va = 0, PRt = 0;
    auto tile_geometry = [&](int tile) {  // uniform
        const int P0 = tile * BN;
        const int Ra = fdiv(P0, p.dWo);
        const int Rb = fdiv(min(P0 + BN, p.PT) - 1, p.dWo);
        const int na = fdiv(Ra, p.dHo), nb = fdiv(Rb, p.dHo);
        va = na * p.VH + (Ra - na * p.Ho) * kS;
        PRt = nb * p.VH + (Rb - nb * p.Ho) * kS + kKS - va;
    };

    float xreg[3 * PE];
    bool xstage[PE];
    auto load_patch = [&]() {  // uses va / PRt of the tile being fetched
#pragma unroll
        for (int r = 0; r < PE; ++r) {
            const int v = va + evr[r];
            const int n = fdiv(v, p.dVH), ih = v - n * p.VH - p.P, iw = epc[r] - p.P;
            xstage[r] = evr[r] < PRt;
            const bool inb = xstage[r] && n < p.N && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
            const uint32_t src = inb ? (uint32_t)(((n * 3 * p.H + ih) * p.W + iw) * 4) : 0u;
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                const float x = ld_f32(p.in + (size_t)c * p.HW, src);
                xreg[c * PE + r] = inb ? x : 0.f;
            }
        }
    };
    auto store_patch = [&](int buf) {
        float *xs = Xs + buf * (3 * plane);
#pragma unroll
        for (int r = 0; r < PE; ++r)
            if (xstage[r]) {
                const int d = evr[r] * LWs + epc[r];
#pragma unroll
                for (int c = 0; c < 3; ++c) xs[c * plane + d] = xreg[c * PE + r];
            }
    };

    int tile = blockIdx.x;
    if (tile < p.ntiles) {
        tile_geometry(tile);
        load_patch();
        store_patch(0);
    }
    __syncthreads();

    for (int it = 0; tile < p.ntiles; ++it, tile += gridDim.x) {
        // B-operand base of this lane's pixel in the current tile
        tile_geometry(tile);
        const int pp = tile * BN + wv * 32 + li;
        int base;
        {
            const int pc = min(pp, p.PT - 1);
            const int R = fdiv(pc, p.dWo), ow = pc - R * p.Wo;
            const int n = fdiv(R, p.dHo);
            base = (n * p.VH + (R - n * p.Ho) * kS - va) * LWs + ow * kS;
        }
        const int b1 = base + kk * plane;
        const int b2 = base + 2 * plane + kk * 3 * LWs;
        const int b3 = base + 2 * plane + 6 * LWs + kk * 3;
        const int b4 = base + 2 * plane + 6 * LWs + 6;

        const int next = tile + gridDim.x;
        const bool more = next < p.ntiles;
        if (more) {
            tile_geometry(next);
            load_patch();
        }

        const float *xs = Xs + (it & 1) * (3 * plane);
        Acc acc[kTM];
#pragma unroll
        for (int x = 0; x < kTM; ++x)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[x][r] = 0.f;

        // The operands of MFMA step s+1 are fetched from LDS before the MFMAs of step s are
        // issued, so the LDS latency hides behind three MFMAs.
        auto b_addr = [&](int s) -> int {
            if (s < 49) return b1 + (s / 7) * LWs + s % 7;
            if (s < 70) return b2 + ((s - 49) / 7) * LWs + (s - 49) % 7;
            if (s < 73) return b3 + (s - 70);
            return b4;
        };
        float av[2][kTM], bv[2];
        auto fetch = [&](int s, float *a, float &b) {
#pragma unroll
            for (int x = 0; x < kTM; ++x) a[x] = Ws[aoff[x] + 2 * s];
            b = xs[b_addr(s)];
        };
        fetch(0, av[0], bv[0]);
#pragma unroll
        for (int s = 0; s < 74; ++s) {
            if (s + 1 < 74) fetch(s + 1, av[(s + 1) & 1], bv[(s + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);  // reads of step s+1 stay ahead of the MFMAs of step s
#pragma unroll
            for (int x = 0; x < kTM; ++x) acc[x] = M::run(av[s & 1][x], bv[s & 1], acc[x]);
            __builtin_amdgcn_sched_barrier(0);
        }

        // The prefetched patch goes to the other LDS buffer BEFORE the output stores are
        // issued: the wait for its global loads would otherwise also wait for the stores.
        if (more) store_patch((it + 1) & 1);

        // epilogue: bias, ReLU, coalesced store of 32 consecutive pixels per register
        if (pp < p.PT) {
            const int n = fdiv(pp, p.dHoWo), q = pp - n * p.HoWo;
            const uint32_t lbase = (uint32_t)(((n * p.ldc + p.coff + lrow) * p.HoWo + q) * 4);
#pragma unroll
            for (int x = 0; x < kTM; ++x)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int mu = x * 32 + M::row_reg(r);
                    float v = acc[x][r] + bias[x][r];
                    if (p.relu) v = fmaxf(v, 0.f);
                    if (p.Cout == kBM || mu + lrow < p.Cout) st_f32(p.out + (size_t)mu * p.HoWo, lbase, v);
                }
        }
        __syncthreads();
    }
}

}  // namespace

KernelFn conv7s2c3_kernel_for(int BN)
{
    if (BN == 256) return conv7s2c3_kernel<256, 8, 1>;
    if (BN == 128) return conv7s2c3_kernel<128, 15, 1>;
    return nullptr;
}

}  // namespace mfma
}  // namespace sq
