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
};

struct wq_plan {
    int N, H, W, Cin, Cout, m, n, g, groups;
    int TH, TW, T, T_pad, Cout_pad;
    int kstep;   // K bytes per MFMA step and per block of the operand layout: 32 (g = 32) or 64
    wq_xf xf;
    // true when the zero entries of the standard matrices are also zero here
    // (always the case for diagonal rescalings of the standard matrices), so
    // that kernels may skip those terms of the fused-multiply-add chains.
    bool sparse_bt, sparse_g, sparse_at;
    // stages 2+3 as GEMM + separate output transform (few tiles, many channels) instead of fused
    bool two_kernel;
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

// Kernel launchers (each enqueues on `s` and returns the launch status).
hipError_t wq_launch_weight(const wq_plan *p, hipStream_t s, const float *w, const float *bias,
                            int8_t *Wq, float *sW, float *bias_out);
hipError_t wq_launch_input(const wq_plan *p, hipStream_t s, const float *x, int8_t *Xq, float *sX);
// Mbuf: fp32 scratch [T_pad][taps][Cout_pad] inside the workspace, used by the two-kernel path
hipError_t wq_launch_contract(const wq_plan *p, hipStream_t s, const int8_t *Xq, const float *sX,
                              const int8_t *Wq, const float *sW, const float *bias, float *Mbuf,
                              float *y, int32_t *P);
// stages: bit 0 = tiled GEMM with group dequantization into Mbuf, bit 1 = output transform of Mbuf
hipError_t wq_launch_contract_unfused(const wq_plan *p, hipStream_t s, const int8_t *Xq,
                                      const float *sX, const int8_t *Wq, const float *sW,
                                      const float *bias, float *Mbuf, float *y, int stages = 3);
