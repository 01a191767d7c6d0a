// Part of the matrix-core engine's kernel instantiations (see qnn_gemm_mfma_kernel.h): single-plane products on the FP4 and int8 paths.
#include "qnn_gemm_mfma_kernel.h"

namespace qnn {
namespace mfma {

VariantList variants_fp4() {
    static const Variant k[] = {
        QNN_VARIANT_FP4(4, false, false),
        QNN_VARIANT_FP4(4, false, true),
    };
    return {k, (int)(sizeof(k) / sizeof(k[0]))};
}

}  // namespace mfma
}  // namespace qnn
