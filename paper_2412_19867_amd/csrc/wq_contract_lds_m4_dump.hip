// Instantiations of the operand-staging contraction kernel for F(4,3), with the int32 dump.
#include "wq_contract_lds_kernel.h"

hipError_t wq_launch_lds_m4_dump(const wq_plan *p, hipStream_t s, const void *args) {
    return launch_lds_m<4, true>(p, s, *static_cast<const LArgs *>(args));
}
