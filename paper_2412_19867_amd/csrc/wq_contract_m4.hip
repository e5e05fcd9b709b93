// Instantiations of the contraction + output-transform kernel for F(4,3).
#include "wq_contract_kernel.h"

hipError_t wq_launch_contract_m4(const wq_plan *p, hipStream_t s, const int8_t *Xq, const float *sX,
                                 const int8_t *Wq, const float *sW, const float *bias, float *y,
                                 const wq_dump &dump) {
    return launch_m<4>(p, s, Xq, sX, Wq, sW, bias, y, dump);
}
