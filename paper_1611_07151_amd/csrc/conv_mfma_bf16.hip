// Instantiates every tiling of the matrix-core convolution kernel for bfloat16 inputs.
#include "conv_mfma_kernel.h"
#include "conv_mfma_variants.h"
#include "conv_wino_kernel.h"

namespace sq {
namespace mfma {

#define SQ_V(KS, S, BM, BN, WM, WN, MT, CC, PE, MINW)                                                 \
    {conv_mfma_kernel<uint16_t, KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, false>,                       \
     conv_mfma_kernel<uint16_t, KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, true>, nullptr, nullptr, nullptr},
#define SQ_E(KS, S, BM, BN, WM, WN, MT, CC, PE, MINW)                                                 \
    {conv_mfma_kernel<uint16_t, KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, false>,                       \
     conv_mfma_kernel<uint16_t, KS, S, BM, BN, WM, WN, MT, CC, PE, MINW, true>,                        \
     nullptr, nullptr, nullptr},
#define SQ_C(NW) {nullptr, nullptr, nullptr, nullptr, nullptr},
#define SQ_W(BM, BT, CC) {conv_wino_kernel<uint16_t>, nullptr, nullptr, nullptr, nullptr},
#define SQ_WA(BM, BT) {conv_wino_auto_kernel<uint16_t>, nullptr, nullptr, nullptr, nullptr},
const KernelSet conv_mfma_kernels_bf16[] = {SQ_VARIANT_LIST(SQ_V, SQ_E, SQ_C, SQ_W, SQ_C, SQ_WA)};

}  // namespace mfma
}  // namespace sq
