// Part of the staged matrix-core kernel's instantiations (see qnn_gemm_stage_kernel.h): convolution by implicit im2col with two-bit activations.
#include "qnn_gemm_stage_kernel.h"

namespace qnn {
namespace stage {

EntryList entries_conv() {
    static const Entry k[] = {
        QNN_STAGE_ENTRY(2, 1, kPixelPlanes, false),
        QNN_STAGE_ENTRY(2, 1, kPixelPlanes, true),
    };
    return {k, (int)(sizeof(k) / sizeof(k[0]))};
}

}  // namespace stage
}  // namespace qnn
