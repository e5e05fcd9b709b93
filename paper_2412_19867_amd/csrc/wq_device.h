// Device-side helpers shared by the kernels: vector types, buffer-resource constants, the
// cross-lane maximum and the quantizer's code (Section "Quantization": symmetric int8,
// round-half-to-even, one reciprocal per group).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kBufFlags = 0x00020000;   // raw buffer, 32-bit elements (gfx9 family)
// cache policy sc0 sc1 of a store: the data is written through to memory while the kernel runs
// instead of being flushed from the XCD's L2 when it ends
constexpr int kWriteThrough = 17;
// a buffer offset past the end of any buffer (all are below 2 GiB): such a load returns 0
constexpr unsigned kPastEnd = 1u << 31;

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_max(uint32_t v) {
    // bound_ctrl with a zero fill lets the compiler fold the move into v_max_u32_dpp
    return max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true));
}

// rint(v*r) as the low byte of a two's-complement code; |v*r| <= 127 + ulp.
__device__ __forceinline__ uint32_t quant_code(float v, float r) {
    const float p = v * r;                   // one rounded product (contraction is off)
    const float z = p + 12582912.0f;         // 1.5*2^23: the add rounds p to nearest-even integer
    return __float_as_uint(z) & 0xffu;
}

// Store of an output value: streaming (non-temporal), the layer does not read y again.  (Plain
// stores make the next layer's input kernel faster when it follows at once, and this layer's
// output stage slower by as much: measured equal on a chained stack, 4-8 % slower elsewhere.)
template <typename T>
__device__ __forceinline__ void store_y(T v, T *p) {
    __builtin_nontemporal_store(v, p);
}
