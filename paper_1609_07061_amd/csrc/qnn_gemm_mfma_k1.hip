// Part of the matrix-core engine's kernel instantiations (see qnn_gemm_mfma_kernel.h): first layer of Alg. 4 (8 input planes, or the 8-bit codes themselves).
#include "qnn_gemm_mfma_kernel.h"

namespace qnn {
namespace mfma {

VariantList variants_first_layer() {
    static const Variant k[] = {
        QNN_VARIANT(8, 1, 1, false, false),
        QNN_VARIANT(8, 1, 1, false, true),
    };
    return {k, (int)(sizeof(k) / sizeof(k[0]))};
}

const KernelFn *byte_kernels() {
    static const KernelFn k[2] = {gemm_mfma_kernel<1, 1, 1, true, false, false, false, true>,
                                  gemm_mfma_kernel<1, 1, 1, true, false, true, false, true>};
    return k;
}

}  // namespace mfma
}  // namespace qnn
