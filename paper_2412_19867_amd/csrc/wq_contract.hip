// Stages 2+3 for gfx950: the Winograd-domain contraction as int8 MFMA GEMMs
// with per-group dequantization, and the output transform y = A^T Y A + bias
// fused behind it, so the n*n fp32 Winograd-domain planes never reach memory.
//
// A workgroup owns a 16-tile x 16-output-channel block for ALL n*n taps and
// has n waves; wave i owns tap row i (taps i*n .. i*n+n-1).  For one tap the
// wave walks the input channels one quantization group at a time:
//   int32 block  = MFMA(Wq rows, Xq rows)        exact, zero-initialised per group
//   M           += float(block) * (sW[o] * sX[tile])   fp32
// (A operand = 16 output channels, B operand = 16 tiles; both are K-contiguous
// int8 rows, each lane fetches the same K-chunk of its A row and its B row, so
// the exact integer sum does not depend on how the instruction orders K.)
// After each tap the wave folds M into R[b] += A^T[b][j] * M  (row i of Y A),
// after its n taps it parks R in LDS, and the whole workgroup finishes
// Y[a][b] = sum_i A^T[a][i] R_i[b], adds bias and stores NHWC with the ragged
// right/bottom edge masked.
#include "wq_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

template <int M, bool K64, bool ATSP, bool DUMP>
__global__ __launch_bounds__(64 * (M + 2)) void k_contract_output(
    wq_xf xf, const int8_t *__restrict__ Xq, const float *__restrict__ sX,
    const int8_t *__restrict__ Wq, const float *__restrict__ sW, const float *__restrict__ bias,
    float *__restrict__ y, int32_t *__restrict__ P, int H, int W, int Cin, int Cout, int TH, int TW,
    int T, int T_pad, int Cout_pad, int g) {
    constexpr int n = M + 2;
    constexpr int KB = K64 ? 16 : 8;   // operand bytes per lane per MFMA
    using Pat = wq_pattern<M>;
    __shared__ float Rs[n][M][256];
    __shared__ int tile_off[16];
    __shared__ int tile_lim[16];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int tau0 = blockIdx.x * 16, o0 = blockIdx.y * 16;
    const int groups = Cin / g;

    if (tid < 16) {
        const int tau = tau0 + tid;
        int off = 0, lim = 0;
        if (tau < T) {
            const int tw = tau % TW, th = (tau / TW) % TH, b = tau / (TW * TH);
            off = ((b * H + th * M) * W + tw * M) * Cout;
            const int hv = min(M, H - th * M), wv = min(M, W - tw * M);
            lim = hv | (wv << 8);
        }
        tile_off[tid] = off;
        tile_lim[tid] = lim;
    }

    float4 R[M];
#pragma unroll
    for (int b = 0; b < M; ++b) R[b] = make_float4(0.f, 0.f, 0.f, 0.f);

    const int i = wave;
#pragma unroll
    for (int j = 0; j < n; ++j) {
        const int t = i * n + j;
        const int8_t *wp = Wq + ((size_t)t * Cout_pad + o0 + l16) * Cin + q * KB;
        const int8_t *xp = Xq + ((size_t)t * T_pad + tau0 + l16) * Cin + q * KB;
        const float *swp = sW + (size_t)t * groups * Cout_pad + o0 + 4 * q;
        const float *sxp = sX + ((size_t)t * T_pad + tau0 + l16) * groups;
        // fp32 partial sums over chunks of 4 groups, chunk totals added in fp64:
        // keeps the rounding of long reductions (many groups) out of the
        // cancelling sums of the output transform.
        double Mt0 = 0.0, Mt1 = 0.0, Mt2 = 0.0, Mt3 = 0.0;
        for (int g0 = 0; g0 < groups; g0 += 4) {
            const int g1 = min(g0 + 4, groups);
            float4 Mc = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int gi = g0; gi < g1; ++gi) {
                v4i acc = {0, 0, 0, 0};
                if constexpr (K64) {
                    for (int kk = 0; kk < g; kk += 64) {
                        const v4i a = *reinterpret_cast<const v4i *>(wp + gi * g + kk);
                        const v4i b = *reinterpret_cast<const v4i *>(xp + gi * g + kk);
                        acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc, 0, 0, 0);
                    }
                } else {
                    for (int kk = 0; kk < g; kk += 32) {
                        const long a = *reinterpret_cast<const long *>(wp + gi * g + kk);
                        const long b = *reinterpret_cast<const long *>(xp + gi * g + kk);
                        acc = __builtin_amdgcn_mfma_i32_16x16x32_i8(a, b, acc, 0, 0, 0);
                    }
                }
                const float4 sw = *reinterpret_cast<const float4 *>(swp + (size_t)gi * Cout_pad);
                const float sx = sxp[gi];
                Mc.x = __builtin_fmaf((float)acc[0], sw.x * sx, Mc.x);
                Mc.y = __builtin_fmaf((float)acc[1], sw.y * sx, Mc.y);
                Mc.z = __builtin_fmaf((float)acc[2], sw.z * sx, Mc.z);
                Mc.w = __builtin_fmaf((float)acc[3], sw.w * sx, Mc.w);
                if constexpr (DUMP) {
                    const int tau = tau0 + l16;
                    if (tau < T) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int o = o0 + 4 * q + r;
                            if (o < Cout)
                                P[(((size_t)t * T + tau) * groups + gi) * Cout + o] = acc[r];
                        }
                    }
                }
            }
            Mt0 += (double)Mc.x;
            Mt1 += (double)Mc.y;
            Mt2 += (double)Mc.z;
            Mt3 += (double)Mc.w;
        }
        const float4 Mv = make_float4((float)Mt0, (float)Mt1, (float)Mt2, (float)Mt3);
#pragma unroll
        for (int b = 0; b < M; ++b)
            if (!ATSP || Pat::at(b, j)) {
                const float c = xf.AT[b * n + j];
                R[b].x = __builtin_fmaf(c, Mv.x, R[b].x);
                R[b].y = __builtin_fmaf(c, Mv.y, R[b].y);
                R[b].z = __builtin_fmaf(c, Mv.z, R[b].z);
                R[b].w = __builtin_fmaf(c, Mv.w, R[b].w);
            }
    }
    // element e = tile_local*16 + channel_local; the lane holds channels 4q..4q+3 of tile l16
#pragma unroll
    for (int b = 0; b < M; ++b)
        *reinterpret_cast<float4 *>(&Rs[i][b][l16 * 16 + 4 * q]) = R[b];
    __syncthreads();

    for (int idx = tid; idx < M * 256; idx += 64 * n) {
        const int bcol = idx >> 8, e = idx & 255, tl = e >> 4, ol = e & 15;
        float Yv[M];
#pragma unroll
        for (int a = 0; a < M; ++a) Yv[a] = 0.f;
#pragma unroll
        for (int ii = 0; ii < n; ++ii) {
            const float rv = Rs[ii][bcol][e];
#pragma unroll
            for (int a = 0; a < M; ++a)
                if (!ATSP || Pat::at(a, ii)) Yv[a] = __builtin_fmaf(xf.AT[a * n + ii], rv, Yv[a]);
        }
        const int lim = tile_lim[tl], hv = lim & 0xff, wv = lim >> 8;
        const int o = o0 + ol;
        if (bcol < wv && o < Cout) {
            const float bv = bias[o];
            float *dst = y + (size_t)tile_off[tl] + bcol * Cout + o;
#pragma unroll
            for (int a = 0; a < M; ++a)
                if (a < hv) dst[(size_t)a * W * Cout] = Yv[a] + bv;
        }
    }
}

template <int M, bool K64, bool ATSP>
hipError_t launch3(const wq_plan *p, hipStream_t s, const int8_t *Xq, const float *sX,
                   const int8_t *Wq, const float *sW, const float *bias, float *y, int32_t *P) {
    const dim3 grid(p->T_pad / 16, p->Cout_pad / 16), block(64 * (M + 2));
    if (P)
        hipLaunchKernelGGL((k_contract_output<M, K64, ATSP, true>), grid, block, 0, s, p->xf, Xq, sX,
                           Wq, sW, bias, y, P, p->H, p->W, p->Cin, p->Cout, p->TH, p->TW, p->T,
                           p->T_pad, p->Cout_pad, p->g);
    else
        hipLaunchKernelGGL((k_contract_output<M, K64, ATSP, false>), grid, block, 0, s, p->xf, Xq,
                           sX, Wq, sW, bias, y, P, p->H, p->W, p->Cin, p->Cout, p->TH, p->TW, p->T,
                           p->T_pad, p->Cout_pad, p->g);
    return hipGetLastError();
}

template <int M>
hipError_t launch1(const wq_plan *p, hipStream_t s, const int8_t *Xq, const float *sX,
                   const int8_t *Wq, const float *sW, const float *bias, float *y, int32_t *P) {
    const bool k64 = (p->g % 64) == 0;
    if (k64)
        return p->sparse_at ? launch3<M, true, true>(p, s, Xq, sX, Wq, sW, bias, y, P)
                            : launch3<M, true, false>(p, s, Xq, sX, Wq, sW, bias, y, P);
    return p->sparse_at ? launch3<M, false, true>(p, s, Xq, sX, Wq, sW, bias, y, P)
                        : launch3<M, false, false>(p, s, Xq, sX, Wq, sW, bias, y, P);
}

}  // namespace

hipError_t wq_launch_contract(const wq_plan *p, hipStream_t s, const int8_t *Xq, const float *sX,
                              const int8_t *Wq, const float *sW, const float *bias, float *y,
                              int32_t *P) {
    switch (p->m) {
        case 2: return launch1<2>(p, s, Xq, sX, Wq, sW, bias, y, P);
        case 4: return launch1<4>(p, s, Xq, sX, Wq, sW, bias, y, P);
        default: return launch1<6>(p, s, Xq, sX, Wq, sW, bias, y, P);
    }
}
