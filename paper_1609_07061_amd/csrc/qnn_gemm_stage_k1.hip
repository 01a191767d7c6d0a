// Part of the staged matrix-core kernel's instantiations (see qnn_gemm_stage_kernel.h): multi-bit activations and weights (Sec. 3).
#include "qnn_gemm_stage_kernel.h"

namespace qnn {
namespace stage {

EntryList entries_multibit() {
    static const Entry k[] = {
        QNN_STAGE_ENTRY(4, 4, kPlanes, false),
        QNN_STAGE_ENTRY(4, 1, kPlanes, false),
        QNN_STAGE_ENTRY(2, 2, kPlanes, false),
    };
    return {k, (int)(sizeof(k) / sizeof(k[0]))};
}

KernelFn find_kernel(int PA, int PW, int kind, bool sign) {
    const EntryList lists[] = {entries_first_layer(), entries_multibit(), entries_conv()};
    for (const EntryList &l : lists)
        for (int i = 0; i < l.n; ++i) {
            const Entry &e = l.e[i];
            if (e.PA == PA && e.PW == PW && e.kind == kind && e.sign == sign) return e.fn;
        }
    return nullptr;
}

}  // namespace stage
}  // namespace qnn
