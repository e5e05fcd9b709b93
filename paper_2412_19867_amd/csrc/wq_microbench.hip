// Issue-rate microbenchmark for the contraction's inner loop on gfx950: what a SIMD sustains
// when every int8 MFMA block must be followed by the per-group dequantization
//     M += float(P) * (sW * sX)        4 conversions, 4 multiplies, 4 multiply-adds per 16x16 block
// (the second quantized-stage equation of Section "Learnable Winograd transform scales" puts a
// pair of scales on every group of the reduction, so the int32 sums cannot be carried across
// groups).  No memory traffic: operands and scales live in registers, so the figure is the
// ceiling the matrix core and the vector ALU set together, per group size.
#include "wq_device.h"
#include "wq_internal.h"

namespace {

// MODE 0: MFMA only.  1: dequantization only (on a register that changes every iteration).
// 2: MFMA, then the dequantization of its result (as written in a straightforward loop).
// 3: software-pipelined - the MFMAs of group k+1 are issued before the dequantization of group k.
// KPG = MFMA K-steps per group (group size = 64 * KPG with the 16x16x64 instruction,
// 32 * KPG with the 16x16x32 one); NB = independent 16x16 blocks per wave.
// The compiler must not merge or hoist anything: every group gets operands, scales and (in the
// dequantization-only mode) int32 sums it cannot see through.
template <typename T>
__device__ __forceinline__ void opaque(T &v) {
    asm volatile("" : "+v"(v));
}

template <int MODE, bool K64, int KPG, int NB>
__global__ __launch_bounds__(256, 2) void k_h1(const int *__restrict__ seed, float *__restrict__ out,
                                           long long *__restrict__ cycles, int iters) {
    constexpr int NA = NB / 2;   // the wave's blocks are NA x 2: NA weight operands, 2 activation operands
    const int tid = threadIdx.x;
    v4i a[NA], b[2];
    v4f sw[NA];
    float sx[2];
#pragma unroll
    for (int k = 0; k < NA; ++k) {
        a[k] = v4i{seed[(tid + k) & 63], seed[(tid + 1) & 63], seed[(tid + 2) & 63], seed[(tid + 3) & 63]};
        sw[k] = v4f{1.0f + tid * 1e-3f, 1.1f + k, 1.2f, 1.3f};
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        b[k] = v4i{seed[(tid + 4 + k) & 63], seed[(tid + 5) & 63], seed[(tid + 6) & 63], seed[(tid + 7) & 63]};
        sx[k] = 0.5f + tid * 1e-4f + k;
    }
    v4i acc[2][NB];
    v4f M[NB];
#pragma unroll
    for (int k = 0; k < NB; ++k) {
        acc[0][k] = acc[1][k] = v4i{tid, 1, 2, 3};
        M[k] = v4f{0.f, 0.f, 0.f, 0.f};
    }
    auto mfma_group = [&](v4i (&ac)[NB]) {
#pragma unroll
        for (int s = 0; s < KPG; ++s) {
#pragma unroll
            for (int k = 0; k < NA; ++k) opaque(a[k]);   // "new" operands every K-step
#pragma unroll
            for (int k = 0; k < 2; ++k) opaque(b[k]);
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                const v4i c0 = s == 0 ? v4i{0, 0, 0, 0} : ac[k];
                const v4i av = a[k / 2], bv = b[k % 2];
                if constexpr (K64) {
                    ac[k] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av, bv, c0, 0, 0, 0);
                } else {
                    const long x = __builtin_bit_cast(long, v2i{av.x, av.y});
                    const long y = __builtin_bit_cast(long, v2i{bv.x, bv.y});
                    ac[k] = __builtin_amdgcn_mfma_i32_16x16x32_i8(x, y, c0, 0, 0, 0);
                }
            }
        }
    };
    auto dequant = [&](const v4i (&ac)[NB]) {
#pragma unroll
        for (int k = 0; k < NA; ++k) opaque(sw[k]);   // "new" scales every group
#pragma unroll
        for (int k = 0; k < 2; ++k) opaque(sx[k]);
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const v4f w = sw[k / 2];
            const float x = sx[k % 2];
            M[k].x = __builtin_fmaf((float)ac[k].x, w.x * x, M[k].x);
            M[k].y = __builtin_fmaf((float)ac[k].y, w.y * x, M[k].y);
            M[k].z = __builtin_fmaf((float)ac[k].z, w.z * x, M[k].z);
            M[k].w = __builtin_fmaf((float)ac[k].w, w.w * x, M[k].w);
        }
    };
    const long long w0 = wall_clock64();
    const long long t0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; it += 2) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if constexpr (MODE == 0) {
                mfma_group(acc[u]);
#pragma unroll
                for (int k = 0; k < NB; ++k) opaque(acc[u][k]);   // the result is "used"
            } else if constexpr (MODE == 1) {
#pragma unroll
                for (int k = 0; k < NB; ++k) opaque(acc[0][k]);   // "new" sums every group
                dequant(acc[0]);
            } else if constexpr (MODE == 2) {
                mfma_group(acc[0]);
                dequant(acc[0]);
            } else {
                mfma_group(acc[u]);
                dequant(acc[u ^ 1]);
            }
        }
    }
    const long long t1 = __builtin_readcyclecounter();
    const long long w1 = wall_clock64();
    float r = 0.f;
#pragma unroll
    for (int k = 0; k < NB; ++k) r += M[k].x + M[k].y + M[k].z + M[k].w + (float)(acc[0][k].x + acc[1][k].x);
    out[(size_t)blockIdx.x * 256 + tid] = r;
    if (tid == 0) {
        cycles[2 * blockIdx.x] = t1 - t0;
        cycles[2 * blockIdx.x + 1] = w1 - w0;   // the constant 100 MHz clock
    }
}

template <int MODE, bool K64, int NB>
hipError_t launch_kpg(int kpg, dim3 grid, hipStream_t s, const int *seed, float *out, long long *cyc, int iters) {
    switch (kpg) {
        case 1: hipLaunchKernelGGL((k_h1<MODE, K64, 1, NB>), grid, dim3(256), 0, s, seed, out, cyc, iters); break;
        case 2: hipLaunchKernelGGL((k_h1<MODE, K64, 2, NB>), grid, dim3(256), 0, s, seed, out, cyc, iters); break;
        case 4: hipLaunchKernelGGL((k_h1<MODE, K64, 4, NB>), grid, dim3(256), 0, s, seed, out, cyc, iters); break;
        case 8: hipLaunchKernelGGL((k_h1<MODE, K64, 8, NB>), grid, dim3(256), 0, s, seed, out, cyc, iters); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <bool K64, int NB>
hipError_t launch_mode(int mode, int kpg, dim3 grid, hipStream_t s, const int *seed, float *out, long long *cyc,
                       int iters) {
    switch (mode) {
        case 0: return launch_kpg<0, K64, NB>(kpg, grid, s, seed, out, cyc, iters);
        case 1: return launch_kpg<1, K64, NB>(kpg, grid, s, seed, out, cyc, iters);
        case 2: return launch_kpg<2, K64, NB>(kpg, grid, s, seed, out, cyc, iters);
        case 3: return launch_kpg<3, K64, NB>(kpg, grid, s, seed, out, cyc, iters);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

extern "C" wq_status_t wq_microbench_dequant(void *stream, int mode, int group_size, int blocks_per_wave,
                                             int workgroups, int iters, const int32_t *seed_dev,
                                             float *out_dev, long long *cycles_dev) {
    if (!seed_dev || !out_dev || !cycles_dev || workgroups <= 0 || iters <= 0 || (iters & 1))
        return WQ_ERR_INVALID_ARG;
    if (blocks_per_wave != 2 && blocks_per_wave != 4) return WQ_ERR_UNSUPPORTED;
    const bool k64 = group_size >= 64;
    const int kpg = k64 ? group_size / 64 : 1;
    if (group_size != 32 && group_size != 64 && group_size != 128 && group_size != 256 && group_size != 512)
        return WQ_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)workgroups);
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    if (blocks_per_wave == 2)
        e = k64 ? launch_mode<true, 2>(mode, kpg, grid, s, seed_dev, out_dev, cycles_dev, iters)
                : launch_mode<false, 2>(mode, kpg, grid, s, seed_dev, out_dev, cycles_dev, iters);
    else
        e = k64 ? launch_mode<true, 4>(mode, kpg, grid, s, seed_dev, out_dev, cycles_dev, iters)
                : launch_mode<false, 4>(mode, kpg, grid, s, seed_dev, out_dev, cycles_dev, iters);
    if (e == hipErrorInvalidValue) return WQ_ERR_INVALID_ARG;
    return e == hipSuccess ? WQ_OK : WQ_ERR_DEVICE;
}
