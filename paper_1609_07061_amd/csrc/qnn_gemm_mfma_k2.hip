// Part of the matrix-core engine's kernel instantiations (see qnn_gemm_mfma_kernel.h): multi-bit activations and weights (Sec. 3).
#include "qnn_gemm_mfma_kernel.h"

namespace qnn {
namespace mfma {

VariantList variants_multibit() {
    static const Variant k[] = {
        QNN_VARIANT(4, 4, 1, false, false),
        QNN_VARIANT(2, 1, 2, false, false),
        QNN_VARIANT(4, 1, 1, false, false),
        QNN_VARIANT(2, 2, 2, false, false),
    };
    return {k, (int)(sizeof(k) / sizeof(k[0]))};
}

}  // namespace mfma
}  // namespace qnn
