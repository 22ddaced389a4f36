// placeholder until the matrix-core kernels land
#include "sq_internal.h"
namespace sq {
int conv_mfma(const ConvArgs &, int) { return SQ_ERR_UNSUPPORTED; }
int conv_mfma_variant_count() { return 0; }
const char *conv_mfma_variant_name(int) { return ""; }
}  // namespace sq
