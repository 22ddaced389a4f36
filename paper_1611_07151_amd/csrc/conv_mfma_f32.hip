// Instantiates every tiling of the matrix-core convolution kernel for fp32 inputs.
#include "conv_mfma_kernel.h"
#include "conv_mfma_variants.h"
#include "conv_wino_kernel.h"

namespace sq {
namespace mfma {

// The pooled-input form exists for those 1x1 tilings that can keep nine values per staged element in registers
// beside their accumulators without spilling (checked with -Rpass-analysis=kernel-resource-usage).
template <int KS, int S, int BM, int BN, int WM, int WN, int MT, int CC, int PE, int MINW> constexpr KernelFn pooled_kernel()
{
    constexpr int XREG = CC * BN / (WM * WN * 64);
    if constexpr (KS == 1 && S == 1 && MINW <= 2 && (XREG <= 8 || BM == 16 || (BM == 32 && CC == 16))) return conv_mfma_kernel<float, KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, false, false, 1>;
    else return nullptr;
}
// The form that pools the rows of a column-pooled map (six values per staged element): the same tilings.
template <int KS, int S, int BM, int BN, int WM, int WN, int MT, int CC, int PE, int MINW> constexpr KernelFn rowpool_kernel()
{
    constexpr int XREG = CC * BN / (WM * WN * 64);
    if constexpr (KS == 1 && S == 1 && MINW <= 2 && (XREG <= 8 || BM == 16 || (BM == 32 && CC == 16))) return conv_mfma_kernel<float, KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, false, false, 2>;
    else return nullptr;
}

// The averaging form exists for every 1x1 tiling (input layers a multiple of the chunk).
template <int KS, int S, int BM, int BN, int WM, int WN, int MT, int CC, int PE, int MINW> constexpr KernelFn avg_kernel()
{
    if constexpr (KS == 1 && S == 1) return conv_mfma_kernel<float, KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, false, false, 0, true>;
    else return nullptr;
}

#define SQ_V(KS, S, BM, BN, WM, WN, MT, CC, PE, MINW)                                                 \
    {conv_mfma_kernel<float, KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, false>,                       \
     conv_mfma_kernel<float, KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, true>, nullptr,               \
     pooled_kernel<KS, S, BM, BN, WM, WN, MT, CC, PE, MINW>(), avg_kernel<KS, S, BM, BN, WM, WN, MT, CC, PE, MINW>(),    \
     rowpool_kernel<KS, S, BM, BN, WM, WN, MT, CC, PE, MINW>()},
#define SQ_E(KS, S, BM, BN, WM, WN, MT, CC, PE, MINW)                                                 \
    {conv_mfma_kernel<float, KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, false>,                       \
     conv_mfma_kernel<float, KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, true>,                        \
     conv_mfma_kernel<float, KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, false, true>, nullptr, nullptr, nullptr},
#define SQ_C(NW) {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr},
#define SQ_W(BM, BT, CC) {conv_wino_kernel<float>, nullptr, nullptr, nullptr, nullptr, nullptr},
#define SQ_WA(BM, BT) {conv_wino_auto_kernel<float>, nullptr, nullptr, nullptr, nullptr, nullptr},
const KernelSet conv_mfma_kernels_f32[] = {SQ_VARIANT_LIST(SQ_V, SQ_E, SQ_C, SQ_W, SQ_C, SQ_WA)};

#define SQ_PAIR(BM, BN, WM, WN, MT, CC)                                                                 \
    {"k1s1_" #BM "x" #BN "_w" #WM "x" #WN "_m" #MT "_c" #CC "_o2",                                      \
     "k3s1_f2x2_64x32_c8+k1s1_" #BM "x" #BN "_w" #WM "x" #WN "_m" #MT "_c" #CC, expand_pair_kernel<BM, BN, WM, WN, MT, CC>,         \
     "k3s1_f2x2_64x32_c8", nullptr, nullptr},
const PairKernel expand_pair_kernels[] = {SQ_PAIR(64, 128, 2, 2, 32, 16) SQ_PAIR(64, 256, 1, 4, 32, 16)
                                          {nullptr, "k3s1_f2x2a_32x16+k1a", expand_pair_auto_kernel<float>, "k3s1_f2x2a_32x16",
                                           expand_pair_auto_kernel<float, true>, "k3s1_f2x2a_32x16+k1a+poolcols"}};
const int num_expand_pair_kernels = sizeof(expand_pair_kernels) / sizeof(expand_pair_kernels[0]);

}  // namespace mfma
}  // namespace sq
