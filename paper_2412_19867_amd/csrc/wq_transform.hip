// Stage 1 (X = B^T d B + dynamic group-wise int8 quantization) and the offline
// stage (W = G w G^T + group-wise int8 quantization) for gfx950.
//
// Both kernels share one skeleton.  A workgroup of 256 threads is 16 DPP rows
// of 16 lanes; a row owns one "unit" = (tile or output channel, 32 consecutive
// input channels), a lane owns 2 of those channels.  With k = group_size/32,
// a workgroup holds 16/k consecutive tiles (output channels) times the k
// units of ONE quantization group, so every group is reduced inside one
// workgroup and the int8 codes of a workgroup land in whole cache lines of
// the blocked operand layout (see include/wq.h).
//   phase A  each lane transforms its two channels with fused-multiply-add
//            chains (left factor first, inner index ascending, from +0) and
//            reduces |value| over each 4-lane group with two DPP steps per tap
//            (the four partial maxima of a row go to LDS);
//   phase B  one lane per (tap, group) combines the partial maxima of the group, does
//            the two correctly rounded divisions s = a/127, r = 127/a and
//            stores s; r goes through LDS;
//   phase C  every lane quantizes its values as rint(v*r) (rounded product,
//            then round-half-even via the 1.5*2^23 add); the codes go through LDS
//            and leave as 16-byte stores that fill whole cache lines.
// The input kernel can additionally split the n tap rows over blockIdx.y:
// B^T d only has to be formed for the workgroup's rows, so the split costs
// nothing but re-reading the tile through L1, and it cuts the registers and
// the length of the per-wave instruction stream (the plan's k1_rows).
// The arithmetic order is part of the library's contract: the int8 codes and
// scales are reproducible bit for bit from the definition in include/wq.h.
#include <float.h>
#include <stdlib.h>

#include "wq_device.h"
#include "wq_internal.h"

namespace {

// added to a row or column offset to push the sum past the buffer end (two of them may add up)
constexpr unsigned kInvalid = 1u << 30;
// (writing the codes through, see kWriteThrough, measured 5-8 % of the input kernel)

// max over each aligned group of 4 lanes, result in all 4 lanes
__device__ __forceinline__ uint32_t quad_max(uint32_t v) {
    v = dpp_max<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_max<0x4E>(v);   // quad_perm [2,3,0,1]
    return v;
}

// bit pattern of max(|a|, |b|): one v_max_f32 with source modifiers.  The operands are
// finite results of fused multiply-adds, so the float maximum orders them like their bits.
__device__ __forceinline__ uint32_t abs_max_bits(float a, float b) {
    return __float_as_uint(__builtin_fmaxf(__builtin_fabsf(a), __builtin_fabsf(b)));
}

// Byte offset of a lane's two codes inside one 16-row block of the operand
// layout [K-step][q][row][KB]: `chunk` = 32-channel chunk index of the unit,
// `row16` = row inside the block.
__device__ __forceinline__ unsigned blocked_offset(int chunk, int row16, int l16, int kstep_log2) {
    if (kstep_log2 == 5)   // K-step 32: q = l16/4, 8 bytes per (q,row)
        return ((unsigned)chunk * 64u + (unsigned)(l16 >> 2) * 16u + (unsigned)row16) * 8u +
               (unsigned)((2 * l16) & 7);
    // K-step 64: two chunks per K-step, q = (chunk&1)*2 + l16/8, 16 bytes per (q,row)
    return ((unsigned)(chunk >> 1) * 64u + (unsigned)((chunk & 1) * 2 + (l16 >> 3)) * 16u +
            (unsigned)row16) * 16u + (unsigned)((2 * l16) & 15);
}

// Where a lane's two codes, and a thread's 16-byte piece, sit in the LDS staging area of one tap
// and in global memory.  The 256 lanes of a workgroup produce 512 code bytes per tap = 32 pieces
// of 16 bytes, each contiguous in the blocked layout:
//   K-step 32 (group 32): the workgroup's 512 bytes are one whole 16-row block; a piece is
//                         (K-quarter q, row pair); LDS pads 32 bytes per q against bank conflicts;
//   K-step 64:            a piece is (DPP row, half of its 16 lanes).
struct CodePlace {
    unsigned lane_pos;    // LDS byte position of the lane's two codes inside a tap
    unsigned piece_pos;   // LDS byte position of the thread's 16-byte piece inside a tap
    unsigned piece_off;   // global byte offset of that piece inside a tap plane
};
constexpr int kTapStride = 640;   // LDS bytes per tap (512 + padding)

// unit_of(r) gives (chunk, row16) of DPP row r; base = byte offset of the 16-row block row
template <typename UnitOf>
__device__ __forceinline__ CodePlace code_place(int tid, int kstep_log2, unsigned base, UnitOf unit_of) {
    const int row = tid >> 4, l16 = tid & 15, p = tid & 31;
    CodePlace c;
    if (kstep_log2 == 5) {
        int chunk, row16;
        unit_of(row, chunk, row16);            // groups of 32: one unit per row, row16 == row
        const int q = l16 >> 2;
        c.lane_pos = (unsigned)((q * 8 + (row16 >> 1)) * 16 + q * 32 + (row16 & 1) * 8 + ((2 * l16) & 7));
        c.piece_pos = (unsigned)(p * 16 + (p >> 3) * 32);
        c.piece_off = base + blocked_offset(chunk, 2 * (p & 7), 4 * (p >> 3), 5);
    } else {
        c.lane_pos = (unsigned)((row * 2 + (l16 >> 3)) * 16 + ((2 * l16) & 15));
        c.piece_pos = (unsigned)(p * 16);
        int chunk, row16;
        unit_of(p >> 1, chunk, row16);
        c.piece_off = base + blocked_offset(chunk, row16, 8 * (p & 1), 6);
    }
    return c;
}

// Phases B and C for NT consecutive taps starting at tap t0.
//   amax_s       LDS [NT][16 rows][4 quads]: partial maxima of the 4-lane groups of every row
//   r_s          LDS [NT][16]
//   codes_s      LDS [NT][kTapStride]: the workgroup's codes, staged so that they leave in
//                16-byte pieces that fill whole 128-byte lines (2-byte stores straight from the
//                lanes cost the input kernel a quarter of its time)
//   log2k        log2(units per group); the workgroup holds 16>>log2k rows-of-groups
//   code_rsrc    buffer over the int8 tensor
//   scale index  scale_base + t*scale_plane + item (item = row-of-group index inside the workgroup)
//   W4           4-bit codes in [-7, 7] (scale a/7), two per byte: the 16-byte piece of int8 codes
//                d0..d3 leaves as 8 bytes p0 p1 at half the byte offset, byte j of p0 holding byte j
//                of d0 in its low and byte j of d1 in its high nibble (p1 likewise from d2, d3)
template <int NT, bool W4 = false>
__device__ __forceinline__ void quantize_and_store(const float2 (&vals)[NT], uint4 (*amax_s)[16],
                                                   float (*r_s)[16], char *codes_s, int log2k, int t0,
                                                   __amdgpu_buffer_rsrc_t code_rsrc, CodePlace place,
                                                   unsigned plane_bytes,
                                                   float *__restrict__ scales, long scale_base,
                                                   long scale_plane, int items_ok) {
    const int tid = threadIdx.x, row = tid >> 4;
    const int k = 1 << log2k, ni_log2 = 4 - log2k, ni = 1 << ni_log2;   // ni items per tap
    __syncthreads();
    for (int it = tid; it < NT * ni; it += 256) {
        const int tl = it >> ni_log2, item = it & (ni - 1);
        uint32_t a = 0;
        for (int q = 0; q < k; ++q) {
            const uint4 v = amax_s[tl][item * k + q];
            a = max(max(a, max(v.x, v.y)), max(v.z, v.w));
        }
        const float af = __uint_as_float(a);
        constexpr float QMAX = W4 ? 7.0f : 127.0f;
        float s = 0.0f, r = 0.0f;
        if (af >= QMAX * FLT_MIN) {
            s = af / QMAX;   // correctly rounded (hipcc default for fp32 division)
            r = QMAX / af;
        }
        r_s[tl][item] = r;
        if (item < items_ok) scales[scale_base + (long)(t0 + tl) * scale_plane + item] = s;
    }
    __syncthreads();
    {
        const int item = row >> log2k;
#pragma unroll
        for (int tl = 0; tl < NT; ++tl) {
            const float r = r_s[tl][item];
            const uint32_t c = quant_code(vals[tl].x, r) | (quant_code(vals[tl].y, r) << 8);
            *reinterpret_cast<uint16_t *>(codes_s + tl * kTapStride + place.lane_pos) = (uint16_t)c;
        }
    }
    __syncthreads();
    // 32 pieces per tap: thread tid moves piece tid % 32 of taps tid / 32, tid / 32 + 8, ...
#pragma unroll
    for (int tl = tid >> 5; tl < NT; tl += 8) {
        const v4i v = *reinterpret_cast<const v4i *>(codes_s + tl * kTapStride + place.piece_pos);
        if constexpr (W4) {
            const v2i pk = {(int)(((unsigned)v.x & 0x0f0f0f0fu) | (((unsigned)v.y << 4) & 0xf0f0f0f0u)),
                            (int)(((unsigned)v.z & 0x0f0f0f0fu) | (((unsigned)v.w << 4) & 0xf0f0f0f0u))};
            __builtin_amdgcn_raw_buffer_store_b64(pk, code_rsrc, place.piece_off >> 1,
                                                  (unsigned)(t0 + tl) * (plane_bytes >> 1), kWriteThrough);
        } else {
            __builtin_amdgcn_raw_buffer_store_b128(v, code_rsrc, place.piece_off,
                                                   (unsigned)(t0 + tl) * plane_bytes, kWriteThrough);
        }
    }
}

// ---------------------------------------------------------------- stage 1
// The tap rows per workgroup of the input kernel are the plan's k1_rows (chosen from the
// layer's wave count when the plan is made).
template <int M, int TR, int I0, bool SPARSE>
__device__ __forceinline__ void input_body(const wq_xf &xf, const float *__restrict__ x,
                                           int8_t *__restrict__ Xq, float *__restrict__ sX, int H,
                                           int W, int Cin, int TH, int TW, int T, int T_pad,
                                           int log2k, int kstep_log2, unsigned x_bytes, int bid,
                                           uint4 (*amax_s)[16], float (*r_s)[16], char *codes_s) {
    constexpr int n = M + 2, NT = TR * n;
    using Pat = wq_pattern<M>;
    const int tid = threadIdx.x, row = tid >> 4, l16 = tid & 15;
    const int k = 1 << log2k;
    const int CC = Cin >> 5, groups = CC >> log2k;
    // workgroup -> (16-tile block rb, sub-block of 16/k tiles, group)
    const int rb = bid / CC, rem = bid % CC;
    const int sub = rem / groups, gam = rem % groups;
    const int row16 = sub * (16 >> log2k) + (row >> log2k);      // tile inside the 16-tile block
    const int chunk = gam * k + (row & (k - 1));
    const int tau = rb * 16 + row16;
    const bool tile_ok = tau < T;
    const int tw = tau % TW, th = (tau / TW) % TH, b = tau / (TW * TH);
    const int h0 = th * M - 1, w0 = tw * M - 1;

    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(x), 0, (int)x_bytes, kBufFlags);
    // byte offsets of the tile's rows and columns; anything outside the image
    // (or a padding tile) is pushed past the end of the buffer and loads as zero
    unsigned roff[n], coff[n];
#pragma unroll
    for (int e = 0; e < n; ++e) {
        const int hh = h0 + e, ww = w0 + e;
        roff[e] = (tile_ok && hh >= 0 && hh < H) ? (unsigned)((b * H + hh) * W) * (unsigned)Cin * 4u
                                                 : kInvalid;
        coff[e] = (ww >= 0 && ww < W) ? (unsigned)(ww * Cin + chunk * 32 + l16 * 2) * 4u : kInvalid;
    }

    // first product, rows I0..I0+TR-1 of Tm = B^T d, one input column at a time
    float2 Tm[TR][n];
#pragma unroll
    for (int j = 0; j < n; ++j) {
        float2 d[n];
#pragma unroll
        for (int kk = 0; kk < n; ++kk) {
            const v2i v = __builtin_amdgcn_raw_buffer_load_b64(rx, roff[kk] + coff[j], 0, 0);
            d[kk] = make_float2(__int_as_float(v.x), __int_as_float(v.y));
        }
#pragma unroll
        for (int r = 0; r < TR; ++r) {
            const int i = I0 + r;
            float ax = 0.0f, ay = 0.0f;
#pragma unroll
            for (int kk = 0; kk < n; ++kk)
                if (!SPARSE || Pat::bt(i, kk)) {
                    ax = __builtin_fmaf(xf.BT[i * n + kk], d[kk].x, ax);
                    ay = __builtin_fmaf(xf.BT[i * n + kk], d[kk].y, ay);
                }
            Tm[r][j] = make_float2(ax, ay);
        }
    }
    // second product X = Tm B, abs-max of each tap over the row's 32 channels
    float2 X[NT];
#pragma unroll
    for (int r = 0; r < TR; ++r) {
        uint32_t am[n];
#pragma unroll
        for (int j = 0; j < n; ++j) {
            float ax = 0.0f, ay = 0.0f;
#pragma unroll
            for (int kk = 0; kk < n; ++kk)
                if (!SPARSE || Pat::bt(j, kk)) {
                    ax = __builtin_fmaf(Tm[r][kk].x, xf.BT[j * n + kk], ax);
                    ay = __builtin_fmaf(Tm[r][kk].y, xf.BT[j * n + kk], ay);
                }
            X[r * n + j] = make_float2(ax, ay);
            am[j] = quad_max(abs_max_bits(ax, ay));
        }
        {   // all four lanes of a group store the same value to the same word
            uint32_t *dst = reinterpret_cast<uint32_t *>(&amax_s[r * n][row]) + (l16 >> 2);
#pragma unroll
            for (int j = 0; j < n; ++j) dst[j * 64] = am[j];   // 64 words per tap
        }
    }
    const int RB = T_pad >> 4;
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(
        Xq, 0, (int)((unsigned)(n * n) * (unsigned)T_pad * (unsigned)Cin), kBufFlags);
    const CodePlace place =
        code_place(tid, kstep_log2, (unsigned)rb * 16u * (unsigned)Cin, [&](int r, int &c, int &r16) {
            c = gam * k + (r & (k - 1));
            r16 = sub * (16 >> log2k) + (r >> log2k);
        });
    // sX [t][rb][group][16]: this workgroup owns 16/k consecutive entries per tap
    const long scale_base = ((long)rb * groups + gam) * 16 + sub * (16 >> log2k);
    quantize_and_store<NT>(X, amax_s, r_s, codes_s, log2k, I0 * n, rq, place,
                           (unsigned)T_pad * (unsigned)Cin, sX, scale_base,
                           (long)RB * groups * 16, 16);
}

template <int M, int TR, bool SPARSE>
__global__ __launch_bounds__(256) void k_input_transform(wq_xf xf, const float *__restrict__ x,
                                                         int8_t *__restrict__ Xq,
                                                         float *__restrict__ sX, int H, int W,
                                                         int Cin, int TH, int TW, int T, int T_pad,
                                                         int log2k, int kstep_log2,
                                                         unsigned x_bytes, int total, int per_xcd) {
    constexpr int n = M + 2;
    // Workgroup ids go round-robin over the 8 XCDs, whose L2s are private: XCD x takes the
    // workgroups [x * per_xcd, (x + 1) * per_xcd) of the tile order, a band of whole tile rows,
    // so that the two input rows that vertically adjacent tiles share are found in that L2.
    const int bid = (int)(blockIdx.x & 7u) * per_xcd + (int)(blockIdx.x >> 3);
    if (bid >= total) return;   // the whole workgroup leaves, before any barrier
    // The abs-max words are dead once the scales exist (the barrier behind the scale pass), the
    // codes are staged after it: both live in the same LDS bytes, which lets one more workgroup
    // onto a CU.
    __shared__ float r_s[TR * n][16];
    __shared__ __attribute__((aligned(16))) char codes_s[TR * n * kTapStride];
    static_assert(sizeof(uint4) * 16 <= kTapStride, "the abs-max rows fit under the code rows");
    uint4 (*amax_s)[16] = reinterpret_cast<uint4 (*)[16]>(codes_s);
#define WQ_BODY(I0)                                                                            \
    input_body<M, TR, (I0), SPARSE>(xf, x, Xq, sX, H, W, Cin, TH, TW, T, T_pad, log2k, kstep_log2, \
                                x_bytes, bid, amax_s, r_s, codes_s)
    // uniform branch: which block of TR tap rows this workgroup forms
    constexpr int NY = n / TR;
    static_assert(NY * TR == n && NY <= 8, "unsupported tap-row split");
    const int yb = blockIdx.y;
    if (yb == 0) WQ_BODY(0);
    if constexpr (NY > 1) { if (yb == 1) WQ_BODY(TR); }
    if constexpr (NY > 2) { if (yb == 2) WQ_BODY(2 * TR); }
    if constexpr (NY > 3) { if (yb == 3) WQ_BODY(3 * TR); }
    if constexpr (NY > 4) { if (yb == 4) WQ_BODY(4 * TR); }
    if constexpr (NY > 5) { if (yb == 5) WQ_BODY(5 * TR); }
    if constexpr (NY > 6) { if (yb == 6) WQ_BODY(6 * TR); }
    if constexpr (NY > 7) { if (yb == 7) WQ_BODY(7 * TR); }
#undef WQ_BODY
}

// ------------------------------------------- stage 1 with the integer transform
// First quantized-stage equation of Section "Learnable Winograd transform scales":
//     X~ = s_B[i] s_B[j] s_x  (Q_B Q(d / s_x) Q_B^T)[i][j]
// with the int8 matrix Q_B = Q(B^T / s_B) from the plan, one dynamic scale s_x = abs-max / 127 per
// (tile, group) over the group's n x n x g patch values, the integer product exact in int32
// (|.| <= n^2 127^3 < 2^31), and the scales applied in fp64 and rounded once to fp32; the result
// then takes the same group quantizer as the fp32 transform's.  Same thread mapping as
// k_input_transform with all n tap rows in one workgroup: a row of 16 lanes owns (tile, 32
// channels), a lane 2 channels, the k = g/32 rows of a group sit side by side.
template <int M>
__global__ __launch_bounds__(256) void k_input_transform_int(wq_xi xi, const float *__restrict__ x,
                                                             int8_t *__restrict__ Xq,
                                                             float *__restrict__ sX, int H, int W,
                                                             int Cin, int TH, int TW, int T, int T_pad,
                                                             int log2k, int kstep_log2,
                                                             unsigned x_bytes, int total, int per_xcd) {
    constexpr int n = M + 2, NT = n * n;
    const int bid = (int)(blockIdx.x & 7u) * per_xcd + (int)(blockIdx.x >> 3);
    if (bid >= total) return;   // the whole workgroup leaves, before any barrier
    __shared__ float r_s[NT][16];
    __shared__ __attribute__((aligned(16))) char codes_s[NT * kTapStride];
    __shared__ uint32_t patch_s[16][4];
    uint4 (*amax_s)[16] = reinterpret_cast<uint4 (*)[16]>(codes_s);

    const int tid = threadIdx.x, row = tid >> 4, l16 = tid & 15;
    const int k = 1 << log2k;
    const int CC = Cin >> 5, groups = CC >> log2k;
    const int rb = bid / CC, rem = bid % CC;
    const int sub = rem / groups, gam = rem % groups;
    const int row16 = sub * (16 >> log2k) + (row >> log2k);
    const int chunk = gam * k + (row & (k - 1));
    const int tau = rb * 16 + row16;
    const bool tile_ok = tau < T;
    const int tw = tau % TW, th = (tau / TW) % TH, b = tau / (TW * TH);
    const int h0 = th * M - 1, w0 = tw * M - 1;
    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(x), 0, (int)x_bytes, kBufFlags);
    unsigned roff[n], coff[n];
#pragma unroll
    for (int e = 0; e < n; ++e) {
        const int hh = h0 + e, ww = w0 + e;
        roff[e] = (tile_ok && hh >= 0 && hh < H) ? (unsigned)((b * H + hh) * W) * (unsigned)Cin * 4u
                                                 : kInvalid;
        coff[e] = (ww >= 0 && ww < W) ? (unsigned)(ww * Cin + chunk * 32 + l16 * 2) * 4u : kInvalid;
    }
    // the lane's two patches and the abs-max of the group's patch values
    float2 d[n][n];
    uint32_t pm = 0;
#pragma unroll
    for (int kk = 0; kk < n; ++kk)
#pragma unroll
        for (int j = 0; j < n; ++j) {
            const v2i v = __builtin_amdgcn_raw_buffer_load_b64(rx, roff[kk] + coff[j], 0, 0);
            d[kk][j] = make_float2(__int_as_float(v.x), __int_as_float(v.y));
            pm = max(pm, abs_max_bits(d[kk][j].x, d[kk][j].y));
        }
    pm = quad_max(pm);
    patch_s[row][l16 >> 2] = pm;   // the four lanes of a quad store the same word
    __syncthreads();
    uint32_t am_bits = 0;
    {
        const int r0 = row & ~(k - 1);
        for (int q = 0; q < k; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) am_bits = max(am_bits, patch_s[r0 + q][j]);
    }
    const double a_x = (double)__uint_as_float(am_bits);
    const double s_x = a_x > 0.0 ? a_x / 127.0 : 0.0, r_x = a_x > 0.0 ? 127.0 / a_x : 0.0;

    float2 X[NT];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        int q[n][n];
#pragma unroll
        for (int kk = 0; kk < n; ++kk)
#pragma unroll
            for (int j = 0; j < n; ++j) {
                const double v = (double)(c ? d[kk][j].y : d[kk][j].x) * r_x;
                q[kk][j] = (int)fmin(127.0, fmax(-127.0, rint(v)));
            }
        int t1[n][n];   // Q_B q
#pragma unroll
        for (int i = 0; i < n; ++i)
#pragma unroll
            for (int j = 0; j < n; ++j) {
                int acc = 0;
#pragma unroll
                for (int kk = 0; kk < n; ++kk) acc += xi.QB[i * n + kk] * q[kk][j];
                t1[i][j] = acc;
            }
#pragma unroll
        for (int i = 0; i < n; ++i)
#pragma unroll
            for (int j = 0; j < n; ++j) {
                int acc = 0;
#pragma unroll
                for (int l = 0; l < n; ++l) acc += t1[i][l] * xi.QB[j * n + l];
                const float v = (float)((xi.sBB[i * n + j] * s_x) * (double)acc);
                if (c) X[i * n + j].y = v; else X[i * n + j].x = v;
            }
    }
    __syncthreads();   // patch_s is read; amax_s (below) shares nothing with it, r_s neither
    // abs-max of each tap over the row's 32 channels, as in the fp32 kernel
#pragma unroll
    for (int i = 0; i < n; ++i) {
        uint32_t am[n];
#pragma unroll
        for (int j = 0; j < n; ++j) am[j] = quad_max(abs_max_bits(X[i * n + j].x, X[i * n + j].y));
        uint32_t *dst = reinterpret_cast<uint32_t *>(&amax_s[i * n][row]) + (l16 >> 2);
#pragma unroll
        for (int j = 0; j < n; ++j) dst[j * 64] = am[j];
    }
    const int RB = T_pad >> 4;
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(
        Xq, 0, (int)((unsigned)(n * n) * (unsigned)T_pad * (unsigned)Cin), kBufFlags);
    const CodePlace place =
        code_place(tid, kstep_log2, (unsigned)rb * 16u * (unsigned)Cin, [&](int r, int &cc, int &r16) {
            cc = gam * k + (r & (k - 1));
            r16 = sub * (16 >> log2k) + (r >> log2k);
        });
    const long scale_base = ((long)rb * groups + gam) * 16 + sub * (16 >> log2k);
    quantize_and_store<NT>(X, amax_s, r_s, codes_s, log2k, 0, rq, place,
                           (unsigned)T_pad * (unsigned)Cin, sX, scale_base,
                           (long)RB * groups * 16, 16);
}

// ----------------------------------------------------------- offline stage
template <int M, bool SPARSE, bool W4 = false>
__global__ __launch_bounds__(256) void k_weight_transform(wq_xf xf, const float *__restrict__ w,
                                                          int8_t *__restrict__ Wq,
                                                          float *__restrict__ sW, int Cin, int Cout,
                                                          int Cout_pad, int log2k, int kstep_log2) {
    constexpr int n = M + 2, n2 = n * n;
    using Pat = wq_pattern<M>;
    __shared__ uint4 amax_s[n2][16];
    __shared__ float r_s[n2][16];
    __shared__ __attribute__((aligned(16))) char codes_s[n2 * kTapStride];
    const int tid = threadIdx.x, row = tid >> 4, l16 = tid & 15;
    const int k = 1 << log2k;
    const int CC = Cin >> 5, groups = CC >> log2k;
    const int rb = blockIdx.x / CC, rem = blockIdx.x % CC;
    const int sub = rem / groups, gam = rem % groups;
    const int row16 = sub * (16 >> log2k) + (row >> log2k);
    const int chunk = gam * k + (row & (k - 1));
    const int o = rb * 16 + row16;
    const bool ok = o < Cout;

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
                for (int kk = 0; kk < 3; ++kk)
                    if (!SPARSE || Pat::g(i, kk)) {
                        ax = __builtin_fmaf(xf.G[i * 3 + kk], f[kk * 3 + bcol], ax);
                        ay = __builtin_fmaf(xf.G[i * 3 + kk], f[9 + kk * 3 + bcol], ay);
                    }
                U[i][bcol] = make_float2(ax, ay);
            }
#pragma unroll
        for (int i = 0; i < n; ++i) {
            uint32_t am[n];
#pragma unroll
            for (int j = 0; j < n; ++j) {
                float ax = 0.0f, ay = 0.0f;
#pragma unroll
                for (int kk = 0; kk < 3; ++kk)
                    if (!SPARSE || Pat::g(j, kk)) {
                        ax = __builtin_fmaf(U[i][kk].x, xf.G[j * 3 + kk], ax);
                        ay = __builtin_fmaf(U[i][kk].y, xf.G[j * 3 + kk], ay);
                    }
                X[i * n + j] = make_float2(ax, ay);
                am[j] = quad_max(abs_max_bits(ax, ay));
            }
            {   // all four lanes of a group store the same value to the same word
                uint32_t *dst = reinterpret_cast<uint32_t *>(&amax_s[i * n][row]) + (l16 >> 2);
#pragma unroll
                for (int j = 0; j < n; ++j) dst[j * 64] = am[j];   // 64 words per tap
            }
        }
    }
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(
        Wq, 0, (int)(((unsigned)n2 * (unsigned)Cout_pad * (unsigned)Cin) >> (W4 ? 1 : 0)), kBufFlags);
    const CodePlace place =
        code_place(tid, kstep_log2, (unsigned)rb * 16u * (unsigned)Cin, [&](int r, int &c, int &r16) {
            c = gam * k + (r & (k - 1));
            r16 = sub * (16 >> log2k) + (r >> log2k);
        });
    // sW [t][group][Cout_pad]: this workgroup owns 16/k consecutive output channels
    const long scale_base = (long)gam * Cout_pad + rb * 16 + sub * (16 >> log2k);
    quantize_and_store<n2, W4>(X, amax_s, r_s, codes_s, log2k, 0, rq, place,
                               (unsigned)Cout_pad * (unsigned)Cin, sW, scale_base,
                               (long)groups * Cout_pad, 16);
}

__global__ void k_copy_bias(const float *__restrict__ bias, float *__restrict__ out, int Cout,
                            int Cout_pad) {
    const int o = blockIdx.x * blockDim.x + threadIdx.x;
    if (o < Cout_pad) out[o] = (bias && o < Cout) ? bias[o] : 0.0f;
}

// Group-wise quantization of a plain weight matrix w [Cout][Cin] (a linear layer, or a 1x1
// convolution): the offline weight stage without a transform, one tap.
template <bool W4>
__global__ __launch_bounds__(256) void k_quantize_weight_rows(const float *__restrict__ w,
                                                              int8_t *__restrict__ Wq,
                                                              float *__restrict__ sW, int Cin, int Cout,
                                                              int Cout_pad, int log2k, int kstep_log2) {
    __shared__ uint4 amax_s[1][16];
    __shared__ float r_s[1][16];
    __shared__ __attribute__((aligned(16))) char codes_s[kTapStride];
    const int tid = threadIdx.x, row = tid >> 4, l16 = tid & 15;
    const int k = 1 << log2k;
    const int CC = Cin >> 5, groups = CC >> log2k;
    const int rb = blockIdx.x / CC, rem = blockIdx.x % CC;
    const int sub = rem / groups, gam = rem % groups;
    const int row16 = sub * (16 >> log2k) + (row >> log2k);
    const int chunk = gam * k + (row & (k - 1));
    const int o = rb * 16 + row16;
    float2 X[1];
    X[0] = o < Cout ? *reinterpret_cast<const float2 *>(w + (size_t)o * Cin + chunk * 32 + l16 * 2)
                    : make_float2(0.0f, 0.0f);
    reinterpret_cast<uint32_t *>(&amax_s[0][row])[l16 >> 2] = quad_max(abs_max_bits(X[0].x, X[0].y));
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(
        Wq, 0, (int)(((unsigned)Cout_pad * (unsigned)Cin) >> (W4 ? 1 : 0)), kBufFlags);
    const CodePlace place =
        code_place(tid, kstep_log2, (unsigned)rb * 16u * (unsigned)Cin, [&](int r, int &c, int &r16) {
            c = gam * k + (r & (k - 1));
            r16 = sub * (16 >> log2k) + (r >> log2k);
        });
    const long scale_base = (long)gam * Cout_pad + rb * 16 + sub * (16 >> log2k);
    quantize_and_store<1, W4>(X, amax_s, r_s, codes_s, log2k, 0, rq, place,
                              (unsigned)Cout_pad * (unsigned)Cin, sW, scale_base,
                              (long)groups * Cout_pad, 16);
}

int ilog2(int v) {
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

template <int M, int TR>
hipError_t launch_input_rows(const wq_plan *p, hipStream_t s, const float *x, int8_t *Xq, float *sX) {
    const int total = (p->T_pad / 16) * (p->Cin / 32), per_xcd = (total + 7) / 8;
    const dim3 grid((unsigned)per_xcd * 8u, (M + 2) / TR), block(256);
    const int log2k = ilog2(p->g / 32), kstep_log2 = p->kstep == 32 ? 5 : 6;
    const unsigned x_bytes = (unsigned)((size_t)p->N * p->H * p->W * p->Cin * 4);
    if (p->sparse_bt)
        hipLaunchKernelGGL((k_input_transform<M, TR, true>), grid, block, 0, s, p->xf, x, Xq, sX, p->H,
                           p->W, p->Cin, p->TH, p->TW, p->T, p->T_pad, log2k, kstep_log2, x_bytes, total, per_xcd);
    else
        hipLaunchKernelGGL((k_input_transform<M, TR, false>), grid, block, 0, s, p->xf, x, Xq, sX, p->H,
                           p->W, p->Cin, p->TH, p->TW, p->T, p->T_pad, log2k, kstep_log2, x_bytes, total, per_xcd);
    return hipGetLastError();
}

template <int M>
hipError_t launch_input_m(const wq_plan *p, hipStream_t s, const float *x, int8_t *Xq, float *sX) {
    constexpr int n = M + 2;
    if (p->integer_transforms) {
        const int total = (p->T_pad / 16) * (p->Cin / 32), per_xcd = (total + 7) / 8;
        const unsigned x_bytes = (unsigned)((size_t)p->N * p->H * p->W * p->Cin * 4);
        hipLaunchKernelGGL((k_input_transform_int<M>), dim3((unsigned)per_xcd * 8u), dim3(256), 0, s, p->xi, x, Xq,
                           sX, p->H, p->W, p->Cin, p->TH, p->TW, p->T, p->T_pad, ilog2(p->g / 32),
                           p->kstep == 32 ? 5 : 6, x_bytes, total, per_xcd);
        return hipGetLastError();
    }
    const int tr = p->k1_rows;   // n, n/2, 2 or 1
    if (tr == n) return launch_input_rows<M, n>(p, s, x, Xq, sX);
    if (tr == 1) return launch_input_rows<M, 1>(p, s, x, Xq, sX);
    if (tr == 2) return launch_input_rows<M, 2>(p, s, x, Xq, sX);
    return launch_input_rows<M, n / 2>(p, s, x, Xq, sX);
}

template <int M>
hipError_t launch_weight_m(const wq_plan *p, hipStream_t s, const float *w, int8_t *Wq, float *sW) {
    const dim3 grid((unsigned)((p->Cout_pad / 16) * (p->Cin / 32))), block(256);
    const int log2k = ilog2(p->g / 32), kstep_log2 = p->kstep == 32 ? 5 : 6;
    if constexpr (M == 1) {   // the untransformed taps of a standard convolution: also with 4-bit codes
        if (p->wbits == 4) {
            hipLaunchKernelGGL((k_weight_transform<M, false, true>), grid, block, 0, s, p->xf, w, Wq, sW,
                               p->Cin, p->Cout, p->Cout_pad, log2k, kstep_log2);
            return hipGetLastError();
        }
    }
    if (p->sparse_g)
        hipLaunchKernelGGL((k_weight_transform<M, true>), grid, block, 0, s, p->xf, w, Wq, sW,
                           p->Cin, p->Cout, p->Cout_pad, log2k, kstep_log2);
    else
        hipLaunchKernelGGL((k_weight_transform<M, false>), grid, block, 0, s, p->xf, w, Wq, sW,
                           p->Cin, p->Cout, p->Cout_pad, log2k, kstep_log2);
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

hipError_t wq_launch_weight_rows(const wq_plan *p, hipStream_t s, const float *w, const float *bias,
                                 int8_t *Wq, float *sW, float *bias_out) {
    const dim3 grid((unsigned)((p->Cout_pad / 16) * (p->Cin / 32))), block(256);
    if (p->wbits == 4)
        hipLaunchKernelGGL((k_quantize_weight_rows<true>), grid, block, 0, s, w, Wq, sW, p->Cin, p->Cout,
                           p->Cout_pad, ilog2(p->g / 32), p->kstep == 32 ? 5 : 6);
    else
        hipLaunchKernelGGL((k_quantize_weight_rows<false>), grid, block, 0, s, w, Wq, sW, p->Cin, p->Cout,
                           p->Cout_pad, ilog2(p->g / 32), p->kstep == 32 ? 5 : 6);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    hipLaunchKernelGGL(k_copy_bias, dim3((p->Cout_pad + 255) / 256), dim3(256), 0, s, bias, bias_out,
                       p->Cout, p->Cout_pad);
    return hipGetLastError();
}

hipError_t wq_launch_weight(const wq_plan *p, hipStream_t s, const float *w, const float *bias,
                            int8_t *Wq, float *sW, float *bias_out) {
    hipError_t e;
    switch (p->m) {
        case 1: e = launch_weight_m<1>(p, s, w, Wq, sW); break;   // F(1,3): the untransformed 3x3 taps
        case 2: e = launch_weight_m<2>(p, s, w, Wq, sW); break;
        case 4: e = launch_weight_m<4>(p, s, w, Wq, sW); break;
        default: e = launch_weight_m<6>(p, s, w, Wq, sW); break;
    }
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_copy_bias, dim3((p->Cout_pad + 255) / 256), dim3(256), 0, s, bias, bias_out,
                       p->Cout, p->Cout_pad);
    return hipGetLastError();
}
