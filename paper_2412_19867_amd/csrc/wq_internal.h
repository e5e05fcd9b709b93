// Internal declarations shared by the host side and the kernel launchers of
// the wq library (group-wise int8 quantized Winograd F(m,3) convolution).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "wq.h"

// Transform matrices as handed to kernels by value (kernarg segment -> SGPRs).
struct wq_xf {
    float BT[64];  // n x n, row-major, row stride n
    float G[24];   // n x 3
    float AT[48];  // m x n, row stride n
    // When A^T has the paired form (columns 2k-1 and 2k belong to points p and -p, up to a
    // column scale): AT[a][2k] = (-1)^a * ATr[k-1] * AT[a][2k-1].  Then a column pair costs
    // E = v1 + r v2, O = v1 - r v2 and one multiply-add per output row instead of two.
    float ATr[4];
};

// The int8 forms of B^T and A^T for the fully-integer transforms (first and third
// quantized-stage equations of Section "Learnable Winograd transform scales"): codes
// Q(M / s) with s = abs-max / 127 per matrix (or per row), and the products of the two scales
// that stand outside an integer product, sBB[i][j] = s_B[i] s_B[j], sAA[a][b] = s_A[a] s_A[b].
struct wq_xi {
    int QB[64];      // n x n, row stride n
    int QA[48];      // m x n, row stride n
    double sBB[64];  // n x n
    double sAA[36];  // m x m, row stride m
};

struct wq_plan {
    int N, H, W, Cin, Cout, m, n, g, groups;
    int TH, TW, T, T_pad, Cout_pad;
    int kstep;   // K bytes per MFMA step and per block of the operand layout: 32 (g = 32) or 64
    int wbits;   // width of the weight codes: 8, or 4 (two codes per byte; standard convolution and linear layers only)
    wq_xf xf;
    // true when the zero entries of the standard matrices are also zero here
    // (always the case for diagonal rescalings of the standard matrices), so
    // that kernels may skip those terms of the fused-multiply-add chains.
    // sparse_at additionally requires the paired form of A^T (see wq_xf::ATr); matrices
    // without it take the dense output-transform code.
    bool sparse_bt, sparse_g, sparse_at;
    // the kernel instance of stages 2+3 (a wq_k2_variant_t) and the tap rows per workgroup of the
    // input kernel, picked from the shape when the plan is made (wq_plan_tune overrides them)
    int k2_variant, k1_rows;
    // 0: fp32 transforms (the path of the second quantized-stage equation alone); 1 / 2: integer
    // input and output transforms with one scale per transform matrix / per matrix row
    int integer_transforms;
    wq_xi xi;
    wq_layout_t lay;
    std::atomic<int> prepared;
};

// Zero pattern of the standard F(m,3) matrices built from the points
// 0, +-1, +-2, +-1/2, infinity: the point 0 and the point at infinity give the
// first and last rows their sparse form.
template <int M>
struct wq_pattern {
    static constexpr int n = M + 2;
    static constexpr bool bt(int i, int k) {
        return i == 0 ? (k % 2 == 0 && k <= n - 2) : (i == n - 1 ? (k % 2 == 1) : (k >= 1 && k <= n - 2));
    }
    static constexpr bool g(int i, int k) { return i == 0 ? k == 0 : (i == n - 1 ? k == 2 : true); }
    static constexpr bool at(int a, int i) { return i == 0 ? a == 0 : (i == n - 1 ? a == M - 1 : true); }
};

// out[a] = sum_i A^T[a][i] * v[i].  PAIRED: the standard zero pattern and the paired form of
// A^T (wq_xf::ATr) are known to hold: 26 instead of 48 multiply-adds for F(6,3).
template <int M, bool PAIRED>
__device__ __forceinline__ void wq_apply_at(const wq_xf &xf, const float (&v)[M + 2], float (&out)[M]) {
    constexpr int n = M + 2;
#pragma unroll
    for (int a = 0; a < M; ++a) out[a] = 0.f;
    if constexpr (!PAIRED) {
#pragma unroll
        for (int i = 0; i < n; ++i)
#pragma unroll
            for (int a = 0; a < M; ++a) out[a] = __builtin_fmaf(xf.AT[a * n + i], v[i], out[a]);
    } else {
        out[0] = xf.AT[0] * v[0];
#pragma unroll
        for (int k = 1; k <= (n - 2) / 2; ++k) {
            const float r = xf.ATr[k - 1];
            const float E = __builtin_fmaf(r, v[2 * k], v[2 * k - 1]);
            const float O = __builtin_fmaf(-r, v[2 * k], v[2 * k - 1]);
#pragma unroll
            for (int a = 0; a < M; ++a)
                out[a] = __builtin_fmaf(xf.AT[a * n + 2 * k - 1], (a & 1) ? O : E, out[a]);
        }
        out[M - 1] = __builtin_fmaf(xf.AT[(M - 1) * n + n - 1], v[n - 1], out[M - 1]);
    }
}

inline bool wq_is_gemm_variant(int v) { return v >= WQ_K2_GEMM_64x64 && v <= WQ_K2_GEMM_128x128; }
inline bool wq_is_fused_variant(int v) { return v >= WQ_K2_FUSED_16x16 && v <= WQ_K2_FUSED_32x32; }
inline bool wq_is_lds_full_variant(int v) { return v >= WQ_K2_LDS_FULL_64x64 && v <= WQ_K2_LDS_FULL_32x32; }
inline bool wq_is_lds_row_variant(int v) { return v >= WQ_K2_LDS_ROW_64x64 && v <= WQ_K2_LDS_ROW_32x64; }
inline bool wq_is_lds_tap_variant(int v) { return v == WQ_K2_LDS_TAP_64x64 || v == WQ_K2_LDS_TAP_128x128; }
inline bool wq_is_lds_variant(int v) {
    return wq_is_lds_full_variant(v) || wq_is_lds_row_variant(v) || wq_is_lds_tap_variant(v);
}

// Which part of the int32 group sums a debug call stores: taps [tap0, tap0+ntaps) x tiles
// [tile0, tile0+ntiles), P [ntaps][ntiles][groups][Cout].  P == nullptr: no dump.
struct wq_dump {
    int32_t *P;
    int tap0, ntaps, tile0, ntiles;
};

// Store the 4 int32 sums a lane holds after an int8 MFMA block (output channels o..o+3 of
// tile tau, tap t, group gam) into the dump slab.  Called under a uniform `if (d.P)`.
__device__ __forceinline__ void wq_dump_store(const wq_dump &d, int t, int tau, int gam, int groups,
                                              int o, int Cout, int T, const int (&v)[4]) {
    const int tt = t - d.tap0, tl = tau - d.tile0;
    if (tt < 0 || tt >= d.ntaps || tl < 0 || tl >= d.ntiles || tau >= T || gam < 0 || gam >= groups) return;
    int32_t *dst = d.P + (((size_t)tt * d.ntiles + tl) * groups + gam) * (size_t)Cout;
#pragma unroll
    for (int r = 0; r < 4; ++r)
        if (o + r < Cout) dst[o + r] = v[r];
}

// Kernel launchers (each enqueues on `s` and returns the launch status).
hipError_t wq_launch_weight(const wq_plan *p, hipStream_t s, const float *w, const float *bias,
                            int8_t *Wq, float *sW, float *bias_out);
// w [Cout][Cin] without a transform (one tap): linear layers
hipError_t wq_launch_weight_rows(const wq_plan *p, hipStream_t s, const float *w, const float *bias,
                                 int8_t *Wq, float *sW, float *bias_out);
hipError_t wq_launch_input(const wq_plan *p, hipStream_t s, const float *x, int8_t *Xq, float *sX);
// Mbuf: fp32 scratch [T_pad][taps][Cout_pad] inside the workspace, used by the two-kernel path
// parts: bit 0 = the first kernel of the plan's variant, bit 1 = its second kernel (if it has one)
hipError_t wq_launch_contract(const wq_plan *p, hipStream_t s, const int8_t *Xq, const float *sX,
                              const int8_t *Wq, const float *sW, const float *bias, float *Mbuf,
                              float *y, const wq_dump &dump, int parts = 3);
// stages: bit 0 = tiled GEMM with group dequantization into Mbuf, bit 1 = output transform of Mbuf
hipError_t wq_launch_contract_unfused(const wq_plan *p, hipStream_t s, const int8_t *Xq,
                                      const float *sX, const int8_t *Wq, const float *sW,
                                      const float *bias, float *Mbuf, float *y, int stages,
                                      const wq_dump &dump);
// the operand-staging (LDS) kernels: full fusion, or tap-row sums + finishing kernel (Mbuf holds
// the row sums)
hipError_t wq_launch_contract_lds(const wq_plan *p, hipStream_t s, const int8_t *Xq, const float *sX,
                                  const int8_t *Wq, const float *sW, const float *bias, float *Mbuf,
                                  float *y, const wq_dump &dump, int parts);
