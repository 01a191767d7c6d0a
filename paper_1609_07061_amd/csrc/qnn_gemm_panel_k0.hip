// Instantiations of the panel-fed matrix-core kernel (see qnn_gemm_panel_kernel.h).
#include "qnn_gemm_panel_kernel.h"

namespace qnn {
namespace panel {

KernelFn find_kernel(bool sign) { return sign ? gemm_panel_kernel<true> : gemm_panel_kernel<false>; }

}  // namespace panel
}  // namespace qnn
