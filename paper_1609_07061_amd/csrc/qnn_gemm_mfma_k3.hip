// Part of the matrix-core engine's kernel instantiations (see qnn_gemm_mfma_kernel.h): convolution by implicit im2col, int32 sums.
#include "qnn_gemm_mfma_kernel.h"

namespace qnn {
namespace mfma {

VariantList variants_conv() {
    static const Variant k[] = {
        QNN_VARIANT_FP4(4, true, false),
        QNN_VARIANT(2, 1, 2, true, false),
    };
    return {k, (int)(sizeof(k) / sizeof(k[0]))};
}

}  // namespace mfma
}  // namespace qnn
