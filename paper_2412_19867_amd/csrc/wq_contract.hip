// Dispatch of stages 2+3 by Winograd tile size; the kernel template lives in
// wq_contract_kernel.h and is instantiated per tile size in its own file.
#include "wq_internal.h"

hipError_t wq_launch_contract_m2(const wq_plan *, hipStream_t, const int8_t *, const float *,
                                 const int8_t *, const float *, const float *, float *, int32_t *);
hipError_t wq_launch_contract_m4(const wq_plan *, hipStream_t, const int8_t *, const float *,
                                 const int8_t *, const float *, const float *, float *, int32_t *);
hipError_t wq_launch_contract_m6(const wq_plan *, hipStream_t, const int8_t *, const float *,
                                 const int8_t *, const float *, const float *, float *, int32_t *);

hipError_t wq_launch_contract(const wq_plan *p, hipStream_t s, const int8_t *Xq, const float *sX,
                              const int8_t *Wq, const float *sW, const float *bias, float *Mbuf,
                              float *y, int32_t *P) {
    // the int32 dump exists only in the fused kernel
    if (!P && p->two_kernel) return wq_launch_contract_unfused(p, s, Xq, sX, Wq, sW, bias, Mbuf, y);
    switch (p->m) {
        case 2: return wq_launch_contract_m2(p, s, Xq, sX, Wq, sW, bias, y, P);
        case 4: return wq_launch_contract_m4(p, s, Xq, sX, Wq, sW, bias, y, P);
        default: return wq_launch_contract_m6(p, s, Xq, sX, Wq, sW, bias, y, P);
    }
}
