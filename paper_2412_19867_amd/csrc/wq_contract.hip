// Dispatch of stages 2+3 by the plan's kernel variant and Winograd tile size; the fused
// kernel template lives in wq_contract_kernel.h and is instantiated per tile size in its own
// file.
#include "wq_internal.h"

hipError_t wq_launch_contract_m2(const wq_plan *, hipStream_t, const int8_t *, const float *,
                                 const int8_t *, const float *, const float *, float *, const wq_dump &);
hipError_t wq_launch_contract_m4(const wq_plan *, hipStream_t, const int8_t *, const float *,
                                 const int8_t *, const float *, const float *, float *, const wq_dump &);
hipError_t wq_launch_contract_m6(const wq_plan *, hipStream_t, const int8_t *, const float *,
                                 const int8_t *, const float *, const float *, float *, const wq_dump &);

hipError_t wq_launch_contract(const wq_plan *p, hipStream_t s, const int8_t *Xq, const float *sX,
                              const int8_t *Wq, const float *sW, const float *bias, float *Mbuf,
                              float *y, const wq_dump &dump, int parts) {
    if (wq_is_gemm_variant(p->k2_variant))
        return wq_launch_contract_unfused(p, s, Xq, sX, Wq, sW, bias, Mbuf, y, parts, dump);
    if (wq_is_lds_variant(p->k2_variant))
        return wq_launch_contract_lds(p, s, Xq, sX, Wq, sW, bias, Mbuf, y, dump, parts);
    if (!(parts & 1)) return hipSuccess;   // the fused kernel is the variant's only one
    switch (p->m) {
        case 2: return wq_launch_contract_m2(p, s, Xq, sX, Wq, sW, bias, y, dump);
        case 4: return wq_launch_contract_m4(p, s, Xq, sX, Wq, sW, bias, y, dump);
        default: return wq_launch_contract_m6(p, s, Xq, sX, Wq, sW, bias, y, dump);
    }
}
