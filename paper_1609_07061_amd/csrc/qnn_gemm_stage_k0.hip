// Part of the staged matrix-core kernel's instantiations (see qnn_gemm_stage_kernel.h): eight input planes (first layer of Alg. 4 when the codes cannot be read directly).
#include "qnn_gemm_stage_kernel.h"

namespace qnn {
namespace stage {

EntryList entries_first_layer() {
    static const Entry k[] = {
        QNN_STAGE_ENTRY(8, 1, kPlanes, false),
        QNN_STAGE_ENTRY(8, 1, kPlanes, true),
    };
    return {k, (int)(sizeof(k) / sizeof(k[0]))};
}

}  // namespace stage
}  // namespace qnn
