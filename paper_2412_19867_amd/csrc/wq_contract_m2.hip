// Instantiations of the contraction + output-transform kernel for F(2,3).
#include "wq_contract_kernel.h"

hipError_t wq_launch_contract_m2(const wq_plan *p, hipStream_t s, const int8_t *Xq, const float *sX,
                                 const int8_t *Wq, const float *sW, const float *bias, float *y,
                                 const wq_dump &dump) {
    return launch_m<2>(p, s, Xq, sX, Wq, sW, bias, y, dump);
}
