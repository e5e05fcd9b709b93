// Instantiations of the operand-staging contraction kernel for F(4,3).
#include "wq_contract_lds_kernel.h"

hipError_t wq_launch_lds_m4(const wq_plan *p, hipStream_t s, const void *args) {
    return launch_lds_m<4, false>(p, s, *static_cast<const LArgs *>(args));
}
