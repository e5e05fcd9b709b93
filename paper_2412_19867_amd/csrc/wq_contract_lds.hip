// Dispatch of the operand-staging (LDS) variants of stages 2+3 and the finishing kernel of
// their row form.  The contraction kernel template lives in wq_contract_lds_kernel.h and is
// instantiated per Winograd tile size, once plain and once with the int32 dump of the debug
// entry point, in files of their own (compile time).
#include "wq_contract_lds_kernel.h"

hipError_t wq_launch_lds_m4(const wq_plan *, hipStream_t, const void *args);
hipError_t wq_launch_lds_m4_dump(const wq_plan *, hipStream_t, const void *args);
hipError_t wq_launch_lds_m6(const wq_plan *, hipStream_t, const void *args);
hipError_t wq_launch_lds_m6_dump(const wq_plan *, hipStream_t, const void *args);

namespace {

struct FArgs {
    wq_xf xf;
    const float *Rbuf;
    const float *bias;
    float *y;
    int H, W, Cout, TH, TW, T, Cout_pad;
};

// y = sum_i A^T[a][i] R_i[b] + bias from the row sums R [T_pad][n][m][Cout_pad]: one thread per
// (tile, output column b, 4 output channels).
template <int M, bool ATSP>
__global__ __launch_bounds__(256) void k_row_finish(const FArgs a) {
    constexpr int n = M + 2;
    const int cq = a.Cout_pad >> 2;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    const int oq = (int)(idx % cq);
    const long rest = idx / cq;
    const int b = (int)(rest % M), tau = (int)(rest / M);
    const int o = oq * 4;
    if (tau >= a.T || o >= a.Cout) return;
    const int tw = tau % a.TW, th = (tau / a.TW) % a.TH, bb = tau / (a.TW * a.TH);
    const int hv = min(M, a.H - th * M), wv = min(M, a.W - tw * M);
    if (b >= wv) return;
    float vx[n], vy[n], vz[n], vw[n];
#pragma unroll
    for (int i = 0; i < n; ++i) {
        const float4 v = *reinterpret_cast<const float4 *>(a.Rbuf + (((size_t)tau * n + i) * M + b) * a.Cout_pad + o);
        vx[i] = v.x; vy[i] = v.y; vz[i] = v.z; vw[i] = v.w;
    }
    float ox[M], oy[M], oz[M], ow[M];
    wq_apply_at<M, ATSP>(a.xf, vx, ox);
    wq_apply_at<M, ATSP>(a.xf, vy, oy);
    wq_apply_at<M, ATSP>(a.xf, vz, oz);
    wq_apply_at<M, ATSP>(a.xf, vw, ow);
    const float4 bv4 = *reinterpret_cast<const float4 *>(a.bias + o);   // padded to Cout_pad
    float *base = a.y + ((size_t)(bb * a.H + th * M) * a.W + tw * M + b) * a.Cout + o;
    const bool vec = (a.Cout & 3) == 0;
#pragma unroll
    for (int aa = 0; aa < M; ++aa) {
        if (aa >= hv) continue;
        const v4f out = {ox[aa] + bv4.x, oy[aa] + bv4.y, oz[aa] + bv4.z, ow[aa] + bv4.w};
        float *dst = base + (size_t)aa * a.W * a.Cout;
        if (vec) {
            store_y(out, reinterpret_cast<v4f *>(dst));
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (o + r < a.Cout) store_y(out[r], dst + r);
        }
    }
}

template <int M>
hipError_t launch_finish(const wq_plan *p, hipStream_t s, const LArgs &a) {
    FArgs f;
    f.xf = p->xf; f.Rbuf = a.Rbuf; f.bias = a.bias; f.y = a.y;
    f.H = p->H; f.W = p->W; f.Cout = p->Cout; f.TH = p->TH; f.TW = p->TW; f.T = p->T; f.Cout_pad = p->Cout_pad;
    const long threads = (long)p->T * M * (p->Cout_pad / 4);
    const dim3 grid((unsigned)((threads + 255) / 256));
    if (p->sparse_at) hipLaunchKernelGGL((k_row_finish<M, true>), grid, dim3(256), 0, s, f);
    else hipLaunchKernelGGL((k_row_finish<M, false>), grid, dim3(256), 0, s, f);
    return hipGetLastError();
}

}  // namespace

hipError_t wq_launch_contract_lds(const wq_plan *p, hipStream_t s, const int8_t *Xq, const float *sX,
                                  const int8_t *Wq, const float *sW, const float *bias, float *Mbuf,
                                  float *y, const wq_dump &dump, int parts) {
    LArgs a;
    a.xf = p->xf;
    a.Xq = Xq; a.sX = sX; a.Wq = Wq; a.sW = sW; a.bias = bias; a.y = y; a.Rbuf = Mbuf; a.dump = dump;
    a.H = p->H; a.W = p->W; a.Cin = p->Cin; a.Cout = p->Cout; a.TH = p->TH; a.TW = p->TW;
    a.T = p->T; a.T_pad = p->T_pad; a.Cout_pad = p->Cout_pad;
    a.log2g = 0;
    while ((1 << a.log2g) < p->g) ++a.log2g;
    a.nOBt = a.nTBt = a.total = a.per_xcd = a.tb_fastest = 0;
    {   // bytes of the intermediate: n*n products per element for the tap form, n*m row sums for the row form
        const long long per_elem = wq_is_lds_tap_variant(p->k2_variant) ? p->n * p->n : p->n * p->m;
        a.plain_stores = per_elem * p->T_pad * p->Cout_pad * 4 >= (20LL << 20);
    }
    if (p->m != 4 && p->m != 6) return hipErrorInvalidValue;   // the plan never picks these variants for F(2,3)
    hipError_t e = hipSuccess;
    if (parts & 1) {
        if (p->m == 4) e = dump.P ? wq_launch_lds_m4_dump(p, s, &a) : wq_launch_lds_m4(p, s, &a);
        else e = dump.P ? wq_launch_lds_m6_dump(p, s, &a) : wq_launch_lds_m6(p, s, &a);
    }
    if (e != hipSuccess || !(parts & 2)) return e;
    if (wq_is_lds_tap_variant(p->k2_variant))   // the output-transform kernel of the GEMM form reads the same M
        return wq_launch_contract_unfused(p, s, Xq, sX, Wq, sW, bias, Mbuf, y, 2, dump);
    if (!wq_is_lds_row_variant(p->k2_variant)) return e;
    return p->m == 4 ? launch_finish<4>(p, s, a) : launch_finish<6>(p, s, a);
}
