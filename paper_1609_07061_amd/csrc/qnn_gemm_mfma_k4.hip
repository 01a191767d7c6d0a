// Part of the matrix-core engine's kernel instantiations (see qnn_gemm_mfma_kernel.h): convolution by implicit im2col with Sign(BatchNorm(.)) fused (binarized ConvNet layers, App. A).
#include "qnn_gemm_mfma_kernel.h"

namespace qnn {
namespace mfma {

VariantList variants_conv_sign() {
    static const Variant k[] = {
        QNN_VARIANT_FP4(4, true, true),
        QNN_VARIANT(2, 1, 2, true, true),
    };
    return {k, (int)(sizeof(k) / sizeof(k[0]))};
}

}  // namespace mfma
}  // namespace qnn
