// Stage 1 (X = B^T d B + dynamic group-wise int8 quantization) and the offline
// stage (W = G w G^T + group-wise int8 quantization) for gfx950.
//
// Both kernels share one skeleton.  A workgroup of 256 threads is 16 DPP rows
// of 16 lanes; a row owns one "unit" = (tile or output channel, 32 consecutive
// input channels), a lane owns 2 of those channels.  Units are numbered so
// that unit u starts at byte 32*u of every tap plane of the int8 output, which
// makes all stores of a workgroup contiguous.
//   phase A  each lane transforms its two channels with fused-multiply-add
//            chains (left factor first, inner index ascending, from +0) and
//            reduces |value| over its row with four DPP steps per tap;
//   phase B  one lane per (tap, group) combines the rows of the group, does
//            the two correctly rounded divisions s = a/127, r = 127/a and
//            stores s; r goes through LDS;
//   phase C  every lane quantizes its values as rint(v*r) (rounded product,
//            then round-half-even via the 1.5*2^23 add) and stores two codes.
// The arithmetic order is part of the library's contract: the int8 codes and
// scales are reproducible bit for bit from the definition in include/wq.h.
#include <float.h>

#include "wq_internal.h"

namespace {

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xf, 0xf, false);
}

// max over the 16 lanes of a DPP row, result in every lane
__device__ __forceinline__ uint32_t row_max16(uint32_t v) {
    v = max(v, dpp_mov<0xB1>(v));   // quad_perm [1,0,3,2]
    v = max(v, dpp_mov<0x4E>(v));   // quad_perm [2,3,0,1]
    v = max(v, dpp_mov<0x141>(v));  // row_half_mirror
    v = max(v, dpp_mov<0x140>(v));  // row_mirror
    return v;
}

__device__ __forceinline__ uint32_t abs_bits(float v) { return __float_as_uint(v) & 0x7fffffffu; }

// rint(v*r) as the low byte of a two's-complement code; |v*r| <= 127 + ulp.
__device__ __forceinline__ uint32_t quant_code(float v, float r) {
    const float p = v * r;                   // one rounded product (contraction is off)
    const float z = p + 12582912.0f;         // 1.5*2^23: the add rounds p to nearest-even integer
    return __float_as_uint(z) & 0xffu;
}

// Phases B and C.  `vals` are the lane's transformed values [tap][2],
// `amax_s`/`r_s` LDS tables [n2][16].  log2k = log2(rows per group).
// scale_index(t, first_unit_of_group) gives the element index of the scale.
template <int N2, typename ScaleIndex>
__device__ __forceinline__ void quantize_and_store(const float2 (&vals)[N2], uint32_t (*amax_s)[16],
                                                   float (*r_s)[16], int log2k, long unit_base,
                                                   long n_units, long plane_bytes, int8_t *codes,
                                                   float *scales, ScaleIndex scale_index) {
    const int tid = threadIdx.x, row = tid >> 4, l16 = tid & 15;
    const int k = 1 << log2k, ng_log2 = 4 - log2k, ng = 1 << ng_log2;
    __syncthreads();
    for (int it = tid; it < N2 * ng; it += 256) {
        const int t = it >> ng_log2, gi = it & (ng - 1);
        uint32_t a = 0;
        for (int q = 0; q < k; ++q) a = max(a, amax_s[t][gi * k + q]);
        const float af = __uint_as_float(a);
        float s = 0.0f, r = 0.0f;
        if (af >= 127.0f * FLT_MIN) {
            s = af / 127.0f;   // correctly rounded (hipcc default for fp32 division)
            r = 127.0f / af;
        }
        r_s[t][gi] = r;
        const long u0 = unit_base + (long)gi * k;
        if (u0 < n_units) scales[scale_index(t, u0)] = s;
    }
    __syncthreads();
    const long u = unit_base + row;
    if (u < n_units) {
        int8_t *dst = codes + u * 32 + l16 * 2;
        const int gi = row >> log2k;
#pragma unroll
        for (int t = 0; t < N2; ++t) {
            const float r = r_s[t][gi];
            const uint32_t c = quant_code(vals[t].x, r) | (quant_code(vals[t].y, r) << 8);
            *reinterpret_cast<uint16_t *>(dst + (long)t * plane_bytes) = (uint16_t)c;
        }
    }
}

// ---------------------------------------------------------------- stage 1
template <int M, bool SPARSE>
__global__ __launch_bounds__(256) void k_input_transform(wq_xf xf, const float *__restrict__ x,
                                                         int8_t *__restrict__ Xq,
                                                         float *__restrict__ sX, int H, int W,
                                                         int Cin, int TH, int TW, int T, int T_pad,
                                                         int log2k) {
    constexpr int n = M + 2, n2 = n * n;
    using Pat = wq_pattern<M>;
    __shared__ uint32_t amax_s[n2][16];
    __shared__ float r_s[n2][16];
    const int tid = threadIdx.x, row = tid >> 4, l16 = tid & 15;
    const int CC = Cin >> 5;
    const long n_units = (long)T_pad * CC;
    const long unit_base = (long)blockIdx.x * 16;
    const long u = unit_base + row;
    const bool unit_ok = u < n_units;
    const int tau = unit_ok ? (int)(u / CC) : 0;
    const int chunk = unit_ok ? (int)(u % CC) : 0;
    const bool tile_ok = unit_ok && tau < T;
    const int tw = tau % TW, th = (tau / TW) % TH, b = tau / (TW * TH);
    const int h0 = th * M - 1, w0 = tw * M - 1;
    const float *xb = x + (size_t)b * H * W * Cin + chunk * 32 + l16 * 2;

    // first product Tm = B^T d, one input column at a time
    float2 Tm[n][n];
#pragma unroll
    for (int j = 0; j < n; ++j) {
        float2 d[n];
        const int ww = w0 + j;
#pragma unroll
        for (int k = 0; k < n; ++k) {
            const int hh = h0 + k;
            const bool ok = tile_ok && hh >= 0 && hh < H && ww >= 0 && ww < W;
            d[k] = ok ? *reinterpret_cast<const float2 *>(xb + ((size_t)hh * W + ww) * Cin)
                      : make_float2(0.0f, 0.0f);
        }
#pragma unroll
        for (int i = 0; i < n; ++i) {
            float ax = 0.0f, ay = 0.0f;
#pragma unroll
            for (int k = 0; k < n; ++k)
                if (!SPARSE || Pat::bt(i, k)) {
                    ax = __builtin_fmaf(xf.BT[i * n + k], d[k].x, ax);
                    ay = __builtin_fmaf(xf.BT[i * n + k], d[k].y, ay);
                }
            Tm[i][j] = make_float2(ax, ay);
        }
    }
    // second product X = Tm B, abs-max of each tap over the row's 32 channels
    float2 X[n2];
#pragma unroll
    for (int i = 0; i < n; ++i)
#pragma unroll
        for (int j = 0; j < n; ++j) {
            float ax = 0.0f, ay = 0.0f;
#pragma unroll
            for (int k = 0; k < n; ++k)
                if (!SPARSE || Pat::bt(j, k)) {
                    ax = __builtin_fmaf(Tm[i][k].x, xf.BT[j * n + k], ax);
                    ay = __builtin_fmaf(Tm[i][k].y, xf.BT[j * n + k], ay);
                }
            X[i * n + j] = make_float2(ax, ay);
            const uint32_t a = row_max16(max(abs_bits(ax), abs_bits(ay)));
            if (l16 == 0) amax_s[i * n + j][row] = a;
        }
    const int groups = CC >> log2k;
    const long sx_plane = (long)T_pad * groups;
    quantize_and_store<n2>(X, amax_s, r_s, log2k, unit_base, n_units, (long)T_pad * Cin, Xq, sX,
                           [=](int t, long u0) { return (long)t * sx_plane + (u0 >> log2k); });
}

// ----------------------------------------------------------- offline stage
template <int M, bool SPARSE>
__global__ __launch_bounds__(256) void k_weight_transform(wq_xf xf, const float *__restrict__ w,
                                                          int8_t *__restrict__ Wq,
                                                          float *__restrict__ sW, int Cin, int Cout,
                                                          int Cout_pad, int log2k) {
    constexpr int n = M + 2, n2 = n * n;
    using Pat = wq_pattern<M>;
    __shared__ uint32_t amax_s[n2][16];
    __shared__ float r_s[n2][16];
    const int tid = threadIdx.x, row = tid >> 4, l16 = tid & 15;
    const int CC = Cin >> 5;
    const long n_units = (long)Cout_pad * CC;
    const long unit_base = (long)blockIdx.x * 16;
    const long u = unit_base + row;
    const bool unit_ok = u < n_units;
    const int o = unit_ok ? (int)(u / CC) : 0;
    const int chunk = unit_ok ? (int)(u % CC) : 0;
    const bool ok = unit_ok && o < Cout;

    // the lane's two 3x3 filters are 18 consecutive floats
    float f[18];
    const float2 *src =
        reinterpret_cast<const float2 *>(w + ((size_t)o * Cin + chunk * 32 + l16 * 2) * 9);
#pragma unroll
    for (int e = 0; e < 9; ++e) {
        const float2 v = ok ? src[e] : make_float2(0.0f, 0.0f);
        f[2 * e] = v.x;
        f[2 * e + 1] = v.y;
    }
    float2 X[n2];
    {
        float2 U[n][3];
#pragma unroll
        for (int i = 0; i < n; ++i)
#pragma unroll
            for (int bcol = 0; bcol < 3; ++bcol) {
                float ax = 0.0f, ay = 0.0f;
#pragma unroll
                for (int k = 0; k < 3; ++k)
                    if (!SPARSE || Pat::g(i, k)) {
                        ax = __builtin_fmaf(xf.G[i * 3 + k], f[k * 3 + bcol], ax);
                        ay = __builtin_fmaf(xf.G[i * 3 + k], f[9 + k * 3 + bcol], ay);
                    }
                U[i][bcol] = make_float2(ax, ay);
            }
#pragma unroll
        for (int i = 0; i < n; ++i)
#pragma unroll
            for (int j = 0; j < n; ++j) {
                float ax = 0.0f, ay = 0.0f;
#pragma unroll
                for (int k = 0; k < 3; ++k)
                    if (!SPARSE || Pat::g(j, k)) {
                        ax = __builtin_fmaf(U[i][k].x, xf.G[j * 3 + k], ax);
                        ay = __builtin_fmaf(U[i][k].y, xf.G[j * 3 + k], ay);
                    }
                X[i * n + j] = make_float2(ax, ay);
                const uint32_t a = row_max16(max(abs_bits(ax), abs_bits(ay)));
                if (l16 == 0) amax_s[i * n + j][row] = a;
            }
    }
    const int groups = CC >> log2k;
    quantize_and_store<n2>(X, amax_s, r_s, log2k, unit_base, n_units, (long)Cout_pad * Cin, Wq, sW,
                           [=](int t, long u0) {
                               const long oo = u0 / CC, gam = (u0 % CC) >> log2k;
                               return ((long)t * groups + gam) * Cout_pad + oo;
                           });
}

__global__ void k_copy_bias(const float *__restrict__ bias, float *__restrict__ out, int Cout,
                            int Cout_pad) {
    const int o = blockIdx.x * blockDim.x + threadIdx.x;
    if (o < Cout_pad) out[o] = (bias && o < Cout) ? bias[o] : 0.0f;
}

int ilog2(int v) {
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

template <int M>
hipError_t launch_input_m(const wq_plan *p, hipStream_t s, const float *x, int8_t *Xq, float *sX) {
    const long units = (long)p->T_pad * (p->Cin / 32);
    const dim3 grid((unsigned)((units + 15) / 16)), block(256);
    const int log2k = ilog2(p->g / 32);
    if (p->sparse_bt)
        hipLaunchKernelGGL((k_input_transform<M, true>), grid, block, 0, s, p->xf, x, Xq, sX, p->H,
                           p->W, p->Cin, p->TH, p->TW, p->T, p->T_pad, log2k);
    else
        hipLaunchKernelGGL((k_input_transform<M, false>), grid, block, 0, s, p->xf, x, Xq, sX, p->H,
                           p->W, p->Cin, p->TH, p->TW, p->T, p->T_pad, log2k);
    return hipGetLastError();
}

template <int M>
hipError_t launch_weight_m(const wq_plan *p, hipStream_t s, const float *w, int8_t *Wq, float *sW) {
    const long units = (long)p->Cout_pad * (p->Cin / 32);
    const dim3 grid((unsigned)((units + 15) / 16)), block(256);
    const int log2k = ilog2(p->g / 32);
    if (p->sparse_g)
        hipLaunchKernelGGL((k_weight_transform<M, true>), grid, block, 0, s, p->xf, w, Wq, sW,
                           p->Cin, p->Cout, p->Cout_pad, log2k);
    else
        hipLaunchKernelGGL((k_weight_transform<M, false>), grid, block, 0, s, p->xf, w, Wq, sW,
                           p->Cin, p->Cout, p->Cout_pad, log2k);
    return hipGetLastError();
}

}  // namespace

hipError_t wq_launch_input(const wq_plan *p, hipStream_t s, const float *x, int8_t *Xq, float *sX) {
    switch (p->m) {
        case 2: return launch_input_m<2>(p, s, x, Xq, sX);
        case 4: return launch_input_m<4>(p, s, x, Xq, sX);
        default: return launch_input_m<6>(p, s, x, Xq, sX);
    }
}

hipError_t wq_launch_weight(const wq_plan *p, hipStream_t s, const float *w, const float *bias,
                            int8_t *Wq, float *sW, float *bias_out) {
    hipError_t e;
    switch (p->m) {
        case 2: e = launch_weight_m<2>(p, s, w, Wq, sW); break;
        case 4: e = launch_weight_m<4>(p, s, w, Wq, sW); break;
        default: e = launch_weight_m<6>(p, s, w, Wq, sW); break;
    }
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_copy_bias, dim3((p->Cout_pad + 255) / 256), dim3(256), 0, s, bias, bias_out,
                       p->Cout, p->Cout_pad);
    return hipGetLastError();
}
