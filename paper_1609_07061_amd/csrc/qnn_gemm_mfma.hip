// Matrix-core engine of the binary / bit-plane matrix product (placeholder: not yet available, the vector-ALU engine
// takes every job).
#include "qnn_internal.h"

namespace qnn {

bool mfma_supports(const GemmArgs &) { return false; }
bool mfma_preferred(const GemmArgs &) { return false; }

int launch_gemm_mfma(const GemmArgs &, hipStream_t) {
    return fail(QNN_ERR_UNSUPPORTED, "matrix-core engine is not built");
}

}  // namespace qnn
