// Instantiations of the panel-fed matrix-core kernel (see qnn_gemm_panel_kernel.h).
#include "qnn_gemm_panel_kernel.h"

namespace qnn {
namespace panel {

KernelFn find_kernel(bool sign, bool narrow, bool tail) {
    if (narrow) return sign ? gemm_panel_kernel<true, 2> : gemm_panel_kernel<false, 2>;
    if (tail) return sign ? gemm_panel_kernel<true, 4, true> : gemm_panel_kernel<false, 4, true>;
    return sign ? gemm_panel_kernel<true, 4> : gemm_panel_kernel<false, 4>;
}

}  // namespace panel
}  // namespace qnn
