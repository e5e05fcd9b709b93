// Group-wise int8 quantized STANDARD 3x3 convolution (stride 1, zero pad 1): the layer the
// paper's runtime section compares the quantized Winograd convolution against.  Same
// quantizer, same groups along the input channels, no transforms:
//   activations  one dynamic scale per (pixel, group)            k_quantize_pixels
//   weights      one scale per (filter tap, out-channel, group)  the offline weight kernel run
//                                                                 as F(1,3) with G = I
//   y[p][o] = bias[o] + sum over the 9 taps and the groups of
//             float(int32 dot product) * sx[shifted pixel][group] * sw[tap][group][o]
//                                                                 k_direct_conv
// k_direct_conv is an implicit GEMM: a workgroup owns 64 consecutive output pixels x 64 output
// channels; per K-step the 256 threads copy four 16-channel weight blocks (already in MFMA
// operand order) and gather the 64 input pixels of the current tap - shifted by the tap's
// offset, zero where the window leaves the image - into MFMA operand order in LDS, plus the
// 64+64 scales of the group.  Two K-steps are in flight in a statically indexed register
// ring; every wave computes a 2x2 arrangement of 16x16 int8 MFMA blocks into fresh int32
// accumulators per group and folds them into fp32 with the two scales.
#include <float.h>

#include <cstdlib>
#include <cstring>
#include <new>

#include "wq_device.h"
#include "wq_internal.h"

struct wq_direct_plan {
    wq_plan w;   // the offline weight stage as F(1,3): m = 1, n = 3, G = identity
    int N, H, W, Cin, Cout, g, groups, P, Cout_pad, kstep;
    int taps;     // 9 = 3x3 convolution, 1 = linear layer (every row is its own "image")
    int wbits;    // width of the weight codes: 8, or 4 (W4A8: two codes per byte)
    int splits;   // the 9 filter taps are shared out over this many workgroups per output tile (1, 3 or 9)
    wq_direct_layout_t lay;
    std::atomic<int> prepared;
};

namespace {

constexpr unsigned kInvalid = kPastEnd;

// ------------------------------------------------------------ activations
// 8 lanes per (pixel, group); a lane owns CPL = g/8 consecutive channels.
template <int CPL>
__global__ __launch_bounds__(256) void k_quantize_pixels(const float *__restrict__ x,
                                                         int8_t *__restrict__ xq,
                                                         float *__restrict__ sx, int units,
                                                         int Cin, int groups) {
    const int tid = threadIdx.x, l8 = tid & 7;
    const int unit = blockIdx.x * 32 + (tid >> 3);
    if (unit >= units) return;   // the 8 lanes of a unit leave together
    const int p = unit / groups, gi = unit - p * groups;
    const size_t e0 = (size_t)p * Cin + (size_t)gi * (CPL * 8) + (size_t)l8 * CPL;
    float v[CPL];
#pragma unroll
    for (int k = 0; k < CPL / 4; ++k) {
        const float4 t = *reinterpret_cast<const float4 *>(x + e0 + 4 * k);
        v[4 * k] = t.x; v[4 * k + 1] = t.y; v[4 * k + 2] = t.z; v[4 * k + 3] = t.w;
    }
    uint32_t a = 0;
#pragma unroll
    for (int k = 0; k < CPL; ++k) a = max(a, __float_as_uint(v[k]) & 0x7fffffffu);
    a = dpp_max<0xB1>(a);    // quad_perm [1,0,3,2]
    a = dpp_max<0x4E>(a);    // quad_perm [2,3,0,1]
    a = dpp_max<0x141>(a);   // row_half_mirror: the 8 lanes of the unit
    const float af = __uint_as_float(a);
    float s = 0.0f, r = 0.0f;
    if (af >= 127.0f * FLT_MIN) {
        s = af / 127.0f;   // correctly rounded
        r = 127.0f / af;
    }
    uint32_t words[CPL / 4];
#pragma unroll
    for (int k = 0; k < CPL / 4; ++k)
        words[k] = quant_code(v[4 * k], r) | (quant_code(v[4 * k + 1], r) << 8) |
                   (quant_code(v[4 * k + 2], r) << 16) | (quant_code(v[4 * k + 3], r) << 24);
    uint32_t *dst = reinterpret_cast<uint32_t *>(xq + e0);
    if constexpr (CPL == 4) {
        dst[0] = words[0];
    } else if constexpr (CPL == 8) {
        *reinterpret_cast<uint2 *>(dst) = make_uint2(words[0], words[1]);
    } else {
#pragma unroll
        for (int k = 0; k < CPL / 16; ++k)
            *reinterpret_cast<uint4 *>(dst + 4 * k) =
                make_uint4(words[4 * k], words[4 * k + 1], words[4 * k + 2], words[4 * k + 3]);
    }
    if (l8 == 0) sx[unit] = s;
}

// ------------------------------------------------------------ convolution
struct DArgs {
    const int8_t *xq;
    const float *sx;
    const int8_t *Wq;
    const float *sW;
    const float *bias;
    float *y;
    float *part;   // splits > 1: partial sums [split][P][Cout], summed (+ bias) by k_direct_reduce
    int N, H, W, Cin, Cout, Cout_pad, P, log2g, splits, taps;
};

// W4: the weight codes are 4 bits wide, two per byte (see the weight kernels for the packing of a
// 16-byte piece into 8).  A weight loader fetches the 8 packed bytes of its 16-byte LDS piece and
// unpacks them on the way into LDS as 16 * code (a nibble moved to the top of its byte), so the
// MFMA loop is the 8-bit one; the factor 16 leaves with the weight scales, which are staged as
// sw / 16 (exact), and 16 * |sum| stays below 2^24 for every group size.
template <bool K64, bool CPG1, bool W4>
__global__ __launch_bounds__(256, 2) void k_direct_conv(const DArgs a) {
    constexpr int KSTEP = K64 ? 64 : 32, KB = KSTEP / 4;
    constexpr int BLK = 16 * KSTEP;   // bytes of one K-step of a 16-row block
    constexpr int LPT = K64 ? 2 : 1;  // 16-byte loads per thread per K-step
    constexpr int PD = 2;             // K-steps in flight (deeper rings measured no faster)
    __shared__ __attribute__((aligned(16))) char opnd[2][8 * BLK];   // blocks 0-3 weights, 4-7 pixels
    __shared__ __attribute__((aligned(16))) float sc[2][128];        // 64 weight scales, 64 pixel scales

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), wm = w >> 1, wn = w & 1;
    const int ob0 = blockIdx.x * 4, p0 = blockIdx.y * 64;
    const int Cin = a.Cin, Cout_pad = a.Cout_pad, H = a.H, W = a.W, P = a.P;
    const int groups = Cin >> a.log2g, cps = Cin / KSTEP;
    const int cpg_mask = ((1 << a.log2g) / KSTEP) - 1;

    const __amdgpu_buffer_rsrc_t rW = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.Wq), 0,
        (int)(((unsigned)a.taps * (unsigned)Cout_pad * (unsigned)Cin) >> (W4 ? 1 : 0)), kBufFlags);
    const __amdgpu_buffer_rsrc_t rX = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.xq), 0, (int)((unsigned)P * (unsigned)Cin), kBufFlags);
    const __amdgpu_buffer_rsrc_t rSW = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(a.sW), 0, (int)((unsigned)a.taps * (unsigned)groups * (unsigned)Cout_pad * 4u), kBufFlags);
    const __amdgpu_buffer_rsrc_t rSX = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(a.sx), 0, (int)((unsigned)P * (unsigned)groups * 4u), kBufFlags);

    // What this thread copies per K-step.
    //   weights (K64: load 0 of every thread; K32: threads 0..127): a linear 16-byte piece of the
    //     four 16-channel blocks;
    //   pixels  (K64: load 1 of every thread; K32: threads 128..255): 16 bytes of one of the 64
    //     pixel rows; `nb` = which bits of the 3x3 neighbourhood of that pixel lie inside the image.
    const bool w_loader = K64 || w < 2;
    unsigned vW = kInvalid;
    {
        const int c = K64 ? tid : (tid & 127), blk = c / (BLK / 16), off = (c % (BLK / 16)) * 16;
        if ((ob0 + blk) * 16 < Cout_pad) vW = (unsigned)((ob0 + blk) * 16 * Cin + off) >> (W4 ? 1 : 0);
    }
    // pixel row and 16-byte piece of the gather, and where the piece goes in MFMA operand order
    const int xr = K64 ? (tid >> 2) : ((tid & 127) >> 1);   // row 0..63 inside the pixel tile
    const int xpc = K64 ? (tid & 3) : (tid & 1);            // 16-byte piece inside the row's K-step
    unsigned nb = 0;
    int prow = p0 + xr;
    {
        const int pc = min(prow, P - 1);
        const int ww = pc % W, hh = (pc / W) % H;
        if (prow < P) {
            if (a.taps == 1) nb = 1u;   // linear layer: the row itself
            else
#pragma unroll
            for (int u = 0; u < 3; ++u)
#pragma unroll
                for (int v = 0; v < 3; ++v)
                    if (hh + u - 1 >= 0 && hh + u - 1 < H && ww + v - 1 >= 0 && ww + v - 1 < W)
                        nb |= 1u << (u * 3 + v);
        }
    }
    // scales: wave 0 the 64 weight scales, wave 1 the 64 pixel scales (waves 2,3 repeat them
    // so that every wave issues the same loads; only waves 0 and 1 store them)
    const bool sc_w = (w & 1) == 0;
    unsigned nb_s = 0;
    int prow_s = p0 + lane;
    {
        const int pc = min(prow_s, P - 1);
        const int ww = pc % W, hh = (pc / W) % H;
        if (prow_s < P) {
            if (a.taps == 1) nb_s = 1u;
            else
#pragma unroll
            for (int u = 0; u < 3; ++u)
#pragma unroll
                for (int v = 0; v < 3; ++v)
                    if (hh + u - 1 >= 0 && hh + u - 1 < H && ww + v - 1 >= 0 && ww + v - 1 < W)
                        nb_s |= 1u << (u * 3 + v);
        }
    }
    const unsigned vSW = (ob0 * 16 + lane) < Cout_pad ? (unsigned)(ob0 * 16 + lane) * 4u : kInvalid;

    v4i pre[PD][LPT];
    float psc[PD];
    // the loader walks (tap t, K-step s) in order; its cursor is kept incrementally (uniform
    // scalars) and stops at the last step, which the tail of the ring fetches again
    // this workgroup's share of the reduction: taps [t_beg, t_end) (all 9, a row of the window, or
    // a single tap) times K-steps [s_beg, s_end) (all of them; a linear layer with few rows splits
    // its one tap along K instead, in whole groups)
    const bool ksplit = a.taps == 1;
    const int tps = ksplit ? 1 : a.taps / a.splits, t_beg = ksplit ? 0 : (int)blockIdx.z * tps, t_end = t_beg + tps;
    const int sps = ksplit ? cps / a.splits : cps, s_beg = ksplit ? (int)blockIdx.z * sps : 0, s_end = s_beg + sps;
    int t_f = t_beg, s_f = s_beg, dp_f = a.taps == 1 ? 0 : (t_beg / 3 - 1) * W + (t_beg % 3 - 1);
    auto fetch = [&](v4i (&dst)[LPT], float &dsc) {
        const int t = t_f, s = s_f, dp = dp_f;
        const unsigned gam = (unsigned)(s * KSTEP) >> a.log2g;
        // pixels: row (prow + dp), bytes s*KSTEP + piece*16 ..
        const unsigned vX = ((nb >> t) & 1u)
                                ? (unsigned)(prow + dp) * (unsigned)Cin + (unsigned)(s * KSTEP + xpc * 16)
                                : kInvalid;
        const unsigned soW = ((unsigned)t * Cout_pad * Cin + (unsigned)s * BLK) >> (W4 ? 1 : 0);
        if constexpr (K64) {
            if constexpr (W4) {
                const v2i pk = __builtin_amdgcn_raw_buffer_load_b64(rW, vW, soW, 0);
                dst[0] = v4i{pk.x, pk.y, 0, 0};
            } else {
                dst[0] = __builtin_amdgcn_raw_buffer_load_b128(rW, vW, soW, 0);
            }
            dst[1] = __builtin_amdgcn_raw_buffer_load_b128(rX, vX, 0, 0);
        } else {
            // (W4: a weight loader's 16 bytes are its 8 packed bytes and its neighbour's, which it
            // ignores: one load instruction for both kinds of loader keeps the waves in step)
            dst[0] = __builtin_amdgcn_raw_buffer_load_b128(w_loader ? rW : rX, w_loader ? vW : vX,
                                                           w_loader ? soW : 0u, 0);
        }
        const unsigned vs = sc_w ? vSW
                                 : (((nb_s >> t) & 1u) ? ((unsigned)(prow_s + dp) * (unsigned)groups + gam) * 4u
                                                       : kInvalid);
        const unsigned so = sc_w ? ((unsigned)t * groups + gam) * (unsigned)Cout_pad * 4u : 0u;
        dsc = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(sc_w ? rSW : rSX, vs, so, 0));
        if (!(t_f == t_end - 1 && s_f == s_end - 1)) {   // advance unless this was the last step
            if (++s_f == s_end) {
                s_f = s_beg;
                ++t_f;
                dp_f = (t_f == 3 || t_f == 6) ? dp_f + W - 2 : dp_f + 1;   // next row of the window, or next column
            }
        }
    };
    // LDS position of a gathered pixel piece in MFMA operand order [block][q][row16][KB bytes]
    const int xblk = 4 + (xr >> 4), xr16 = xr & 15;
    auto unpack = [](const v4i &pk) {   // 8 packed bytes -> 16 bytes of 16 * code
        if constexpr (!W4) return pk;
        const unsigned p0 = (unsigned)pk.x, p1 = (unsigned)pk.y;
        return v4i{(int)((p0 << 4) & 0xf0f0f0f0u), (int)(p0 & 0xf0f0f0f0u),
                   (int)((p1 << 4) & 0xf0f0f0f0u), (int)(p1 & 0xf0f0f0f0u)};
    };
    auto commit = [&](int buf, const v4i (&src)[LPT], float ssc) {
        if constexpr (K64) {
            *reinterpret_cast<v4i *>(&opnd[buf][tid * 16]) = unpack(src[0]);
            *reinterpret_cast<v4i *>(&opnd[buf][xblk * BLK + xpc * 256 + xr16 * 16]) = src[1];
        } else {
            if (w_loader) {
                *reinterpret_cast<v4i *>(&opnd[buf][tid * 16]) = unpack(src[0]);
            } else {   // 16 bytes = two K-quarters of 8 bytes
                char *d = &opnd[buf][xblk * BLK + (2 * xpc) * 128 + xr16 * 8];
                *reinterpret_cast<v2i *>(d) = v2i{src[0].x, src[0].y};
                *reinterpret_cast<v2i *>(d + 128) = v2i{src[0].z, src[0].w};
            }
        }
        if (w < 2) sc[buf][w * 64 + lane] = (W4 && w == 0) ? ssc * 0.0625f : ssc;
    };

    v4i acc[2][2];
    float4 Mc[2][2];
#pragma unroll
    for (int no = 0; no < 2; ++no)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            acc[no][nt] = v4i{0, 0, 0, 0};
            Mc[no][nt] = make_float4(0.f, 0.f, 0.f, 0.f);
        }

    const int NI = tps * sps;
#pragma unroll
    for (int u = 0; u < PD; ++u) fetch(pre[u], psc[u]);
    commit(0, pre[0], psc[0]);
    __syncthreads();
    for (int i0 = 0; i0 < NI; i0 += PD) {
#pragma unroll
      for (int u = 0; u < PD; ++u) {
        const int it = i0 + u;
        if (it >= NI) break;
        const int buf = u & 1;   // PD is even, so it & 1 == u & 1
        fetch(pre[u], psc[u]);   // step it + PD (or the last one again); slot u held step it, already in LDS
        v4i av[2], bv[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const char *pa = &opnd[buf][(2 * wn + e) * BLK + lane * KB];
            const char *pb = &opnd[buf][(4 + 2 * wm + e) * BLK + lane * KB];
            if constexpr (K64) {
                av[e] = *reinterpret_cast<const v4i *>(pa);
                bv[e] = *reinterpret_cast<const v4i *>(pb);
            } else {
                const v2i ta = *reinterpret_cast<const v2i *>(pa), tb = *reinterpret_cast<const v2i *>(pb);
                av[e] = v4i{ta.x, ta.y, 0, 0};
                bv[e] = v4i{tb.x, tb.y, 0, 0};
            }
        }
#pragma unroll
        for (int no = 0; no < 2; ++no)
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                const v4i c0 = CPG1 ? v4i{0, 0, 0, 0} : acc[no][nt];
                if constexpr (K64) {
                    acc[no][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av[no], bv[nt], c0, 0, 0, 0);
                } else {
                    const long x = __builtin_bit_cast(long, v2i{av[no].x, av[no].y});
                    const long y = __builtin_bit_cast(long, v2i{bv[nt].x, bv[nt].y});
                    acc[no][nt] = __builtin_amdgcn_mfma_i32_16x16x32_i8(x, y, c0, 0, 0, 0);
                }
            }
        if (CPG1 || ((it + 1) & cpg_mask) == 0) {   // last K-step of a group (a share is a whole number of groups)
#pragma unroll
            for (int no = 0; no < 2; ++no) {
                const v4f sw = *reinterpret_cast<const v4f *>(&sc[buf][(2 * wn + no) * 16 + 4 * q]);
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) {
                    const float sxv = sc[buf][64 + (2 * wm + nt) * 16 + l16];
                    Mc[no][nt].x = __builtin_fmaf((float)acc[no][nt][0], sw.x * sxv, Mc[no][nt].x);
                    Mc[no][nt].y = __builtin_fmaf((float)acc[no][nt][1], sw.y * sxv, Mc[no][nt].y);
                    Mc[no][nt].z = __builtin_fmaf((float)acc[no][nt][2], sw.z * sxv, Mc[no][nt].z);
                    Mc[no][nt].w = __builtin_fmaf((float)acc[no][nt][3], sw.w * sxv, Mc[no][nt].w);
                    if constexpr (!CPG1) acc[no][nt] = v4i{0, 0, 0, 0};
                }
            }
        }
        if (it + 1 < NI) commit(buf ^ 1, pre[(u + 1) % PD], psc[(u + 1) % PD]);
        __syncthreads();
      }
    }
    // + bias, NHWC store: the lane holds channels 4q..4q+3 of pixel l16 in each block
    const bool vec = (a.Cout & 3) == 0;   // rows of y are 16-byte aligned
    const bool final_sum = a.splits == 1;
    float *out = final_sum ? a.y : a.part + (size_t)blockIdx.z * P * a.Cout;
#pragma unroll
    for (int no = 0; no < 2; ++no) {
        const int o = (ob0 + 2 * wn + no) * 16 + 4 * q;
        float bv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) bv[r] = (final_sum && o + r < a.Cout) ? a.bias[o + r] : 0.f;
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const int p = p0 + (2 * wm + nt) * 16 + l16;
            if (p >= P || o >= a.Cout) continue;
            const float mv[4] = {Mc[no][nt].x + bv[0], Mc[no][nt].y + bv[1], Mc[no][nt].z + bv[2],
                                 Mc[no][nt].w + bv[3]};
            float *dst = out + (size_t)p * a.Cout + o;
            if (vec) {   // o is a multiple of 4, so o + 3 < Cout too
                __builtin_nontemporal_store(v4f{mv[0], mv[1], mv[2], mv[3]}, reinterpret_cast<v4f *>(dst));
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (o + r < a.Cout) __builtin_nontemporal_store(mv[r], dst + r);
            }
        }
    }
}

// y = bias + sum of the per-split partial sums (splits > 1)
__global__ __launch_bounds__(256) void k_direct_reduce(const float *__restrict__ part,
                                                       const float *__restrict__ bias,
                                                       float *__restrict__ y, int total, int Cout,
                                                       int splits) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    float acc = bias[e % Cout];
    for (int z = 0; z < splits; ++z) acc += part[(size_t)z * total + e];
    __builtin_nontemporal_store(acc, &y[e]);
}

int ilog2(int v) {
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

uint64_t align256(uint64_t v) { return (v + 255) / 256 * 256; }

}  // namespace

// ------------------------------------------------------------------ C ABI
extern "C" {

static wq_status_t make_plan(wq_direct_plan_t **out, int N, int H, int W, int Cin, int Cout,
                             int group_size, int taps, int weight_bits) {
    if (!out) return WQ_ERR_INVALID_ARG;
    *out = nullptr;
    if (weight_bits != 8 && weight_bits != 4) return WQ_ERR_UNSUPPORTED;
    if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || group_size <= 0) return WQ_ERR_INVALID_ARG;
    if (group_size != 32 && group_size != 64 && group_size != 128 && group_size != 256 && group_size != 512)
        return WQ_ERR_UNSUPPORTED;
    if (Cin % group_size != 0) return WQ_ERR_INVALID_ARG;
    const long long P = (long long)N * H * W, Cp = (Cout + 31) / 32 * 32, lim = (1LL << 31) - 1;
    if (P * Cin * 4 > lim || P * Cout * 4 > lim || taps * Cp * Cin > lim ||
        taps * Cp * (Cin / group_size) * 4 > lim)
        return WQ_ERR_UNSUPPORTED;
    if ((P + 63) / 64 > 65535) return WQ_ERR_UNSUPPORTED;   // pixel tiles are the grid's y dimension
    wq_direct_plan *p = new (std::nothrow) wq_direct_plan();
    if (!p) return WQ_ERR_INVALID_ARG;
    p->N = N; p->H = H; p->W = W; p->Cin = Cin; p->Cout = Cout; p->g = group_size;
    p->groups = Cin / group_size; p->P = (int)P; p->Cout_pad = (int)Cp;
    p->kstep = group_size == 32 ? 32 : 64;
    p->taps = taps;
    p->wbits = weight_bits;
    // the weight stage: the offline Winograd weight kernel as F(1,3) with G = I leaves the nine
    // filter taps untransformed and quantizes them per (tap, out-channel, group)
    wq_plan &w = p->w;
    w.N = N; w.H = H; w.W = W; w.Cin = Cin; w.Cout = Cout; w.m = 1; w.n = 3; w.g = group_size;
    w.groups = p->groups; w.TH = H; w.TW = W; w.T = (int)P; w.T_pad = (int)((P + 31) / 32 * 32);
    w.Cout_pad = p->Cout_pad; w.kstep = p->kstep; w.wbits = weight_bits;
    w.k1_rows = 1; w.k2_variant = WQ_K2_FUSED_16x16;
    std::memset(&w.xf, 0, sizeof(w.xf));
    w.xf.G[0] = w.xf.G[4] = w.xf.G[8] = 1.0f;
    w.sparse_bt = w.sparse_g = w.sparse_at = false;
    w.prepared.store(0);
    wq_direct_layout_t &L = p->lay;
    L.N = N; L.H = H; L.W = W; L.Cin = Cin; L.Cout = Cout; L.group_size = group_size;
    L.groups = p->groups; L.P = p->P; L.Cout_pad = p->Cout_pad; L.kstep = p->kstep;
    L.taps = taps;
    L.weight_bits = weight_bits;
    L.reserved = 0;
    L.blob_Wq_off = 0;
    L.blob_sW_off = align256(((uint64_t)taps * p->Cout_pad * Cin * weight_bits) / 8);
    L.blob_bias_off = L.blob_sW_off + align256((uint64_t)taps * p->groups * p->Cout_pad * 4);
    L.blob_bytes = L.blob_bias_off + align256((uint64_t)p->Cout_pad * 4);
    L.ws_xq_off = 0;
    L.ws_sx_off = align256((uint64_t)P * Cin);
    // few output tiles: share the taps out over 3 or 9 workgroups per tile (partial sums in the
    // workspace, one more small kernel adds them) so that the chip has enough waves
    const long long base = ((P + 63) / 64) * ((Cp + 63) / 64);
    p->splits = base >= 512 ? 1 : (base * 3 >= 512 ? 3 : 9);
    if (taps == 1) {
        // a linear layer with few rows: split K, in whole groups, until the chip has enough
        // workgroups (the partial sums are added by the same small kernel)
        p->splits = 1;
        while (base * p->splits < 512 && p->splits < 16 && p->groups % (p->splits * 2) == 0 &&
               Cin / (p->splits * 2) >= 256)
            p->splits *= 2;
    }
    L.splits = p->splits;
    L.ws_part_off = L.ws_sx_off + align256((uint64_t)P * p->groups * 4);
    L.ws_bytes = L.ws_part_off + (p->splits > 1 ? align256((uint64_t)p->splits * P * Cout * 4) : 0);
    p->prepared.store(0);
    *out = p;
    return WQ_OK;
}

wq_status_t wq_direct_plan_create(wq_direct_plan_t **out, int N, int H, int W, int Cin, int Cout,
                                  int group_size) {
    return make_plan(out, N, H, W, Cin, Cout, group_size, 9, 8);
}

wq_status_t wq_direct_plan_create_bits(wq_direct_plan_t **out, int N, int H, int W, int Cin, int Cout,
                                       int group_size, int weight_bits) {
    return make_plan(out, N, H, W, Cin, Cout, group_size, 9, weight_bits);
}

wq_status_t wq_linear_plan_create(wq_direct_plan_t **out, int R, int Cin, int Cout, int group_size) {
    return make_plan(out, R, 1, 1, Cin, Cout, group_size, 1, 8);
}

wq_status_t wq_linear_plan_create_bits(wq_direct_plan_t **out, int R, int Cin, int Cout, int group_size,
                                       int weight_bits) {
    return make_plan(out, R, 1, 1, Cin, Cout, group_size, 1, weight_bits);
}

wq_status_t wq_direct_plan_tune(wq_direct_plan_t *plan, int splits) {
    if (!plan || splits < 0) return WQ_ERR_INVALID_ARG;
    if (splits == 0) return WQ_OK;
    const bool ok = plan->taps == 9 ? (splits == 1 || splits == 3 || splits == 9)
                                    : (splits <= 16 && (splits & (splits - 1)) == 0 &&
                                       plan->groups % splits == 0);
    if (!ok) return WQ_ERR_UNSUPPORTED;
    plan->splits = splits;
    wq_direct_layout_t &L = plan->lay;
    L.splits = splits;
    L.ws_bytes = L.ws_part_off +
                 (splits > 1 ? align256((uint64_t)splits * plan->P * plan->Cout * 4) : 0);
    return WQ_OK;
}

wq_status_t wq_direct_plan_destroy(wq_direct_plan_t *plan) {
    if (!plan) return WQ_ERR_INVALID_ARG;
    delete plan;
    return WQ_OK;
}

wq_status_t wq_direct_plan_layout(const wq_direct_plan_t *plan, wq_direct_layout_t *out) {
    if (!plan || !out) return WQ_ERR_INVALID_ARG;
    *out = plan->lay;
    return WQ_OK;
}

wq_status_t wq_direct_weight_prepare(wq_direct_plan_t *plan, void *stream, const float *w_dev,
                                     const float *bias_dev, void *weight_blob_dev, size_t blob_bytes) {
    if (!plan || !w_dev || !weight_blob_dev) return WQ_ERR_INVALID_ARG;
    if (blob_bytes < plan->lay.blob_bytes) return WQ_ERR_WORKSPACE;
    char *b = (char *)weight_blob_dev;
    hipError_t e = (plan->taps == 1 ? wq_launch_weight_rows : wq_launch_weight)(
        &plan->w, (hipStream_t)stream, w_dev, bias_dev, (int8_t *)(b + plan->lay.blob_Wq_off),
        (float *)(b + plan->lay.blob_sW_off), (float *)(b + plan->lay.blob_bias_off));
    if (e != hipSuccess) return WQ_ERR_DEVICE;
    plan->prepared.store(1);
    return WQ_OK;
}

wq_status_t wq_direct_quantize(const wq_direct_plan_t *plan, void *stream, const float *x_dev,
                               void *workspace_dev, size_t workspace_bytes) {
    if (!plan || !x_dev || !workspace_dev) return WQ_ERR_INVALID_ARG;
    if (workspace_bytes < plan->lay.ws_bytes) return WQ_ERR_WORKSPACE;
    char *ws = (char *)workspace_dev;
    int8_t *xq = (int8_t *)(ws + plan->lay.ws_xq_off);
    float *sx = (float *)(ws + plan->lay.ws_sx_off);
    const int units = plan->P * plan->groups;
    const dim3 grid((unsigned)((units + 31) / 32)), block(256);
    hipStream_t s = (hipStream_t)stream;
    switch (plan->g) {
        case 32: hipLaunchKernelGGL((k_quantize_pixels<4>), grid, block, 0, s, x_dev, xq, sx, units, plan->Cin, plan->groups); break;
        case 64: hipLaunchKernelGGL((k_quantize_pixels<8>), grid, block, 0, s, x_dev, xq, sx, units, plan->Cin, plan->groups); break;
        case 128: hipLaunchKernelGGL((k_quantize_pixels<16>), grid, block, 0, s, x_dev, xq, sx, units, plan->Cin, plan->groups); break;
        case 256: hipLaunchKernelGGL((k_quantize_pixels<32>), grid, block, 0, s, x_dev, xq, sx, units, plan->Cin, plan->groups); break;
        default: hipLaunchKernelGGL((k_quantize_pixels<64>), grid, block, 0, s, x_dev, xq, sx, units, plan->Cin, plan->groups); break;
    }
    return hipGetLastError() == hipSuccess ? WQ_OK : WQ_ERR_DEVICE;
}

wq_status_t wq_direct_conv(const wq_direct_plan_t *plan, void *stream, void *workspace_dev,
                           size_t workspace_bytes, const void *weight_blob_dev, size_t blob_bytes,
                           float *y_dev) {
    if (!plan || !workspace_dev || !weight_blob_dev || !y_dev) return WQ_ERR_INVALID_ARG;
    if (workspace_bytes < plan->lay.ws_bytes || blob_bytes < plan->lay.blob_bytes) return WQ_ERR_WORKSPACE;
    if (!plan->prepared.load()) return WQ_ERR_NOT_PREPARED;
    const char *ws = (const char *)workspace_dev, *b = (const char *)weight_blob_dev;
    DArgs a;
    a.xq = (const int8_t *)(ws + plan->lay.ws_xq_off);
    a.sx = (const float *)(ws + plan->lay.ws_sx_off);
    a.Wq = (const int8_t *)(b + plan->lay.blob_Wq_off);
    a.sW = (const float *)(b + plan->lay.blob_sW_off);
    a.bias = (const float *)(b + plan->lay.blob_bias_off);
    a.y = y_dev;
    a.part = (float *)(const_cast<char *>(ws) + plan->lay.ws_part_off);
    a.splits = plan->splits;
    a.taps = plan->taps;
    a.N = plan->N; a.H = plan->H; a.W = plan->W; a.Cin = plan->Cin; a.Cout = plan->Cout;
    a.Cout_pad = plan->Cout_pad; a.P = plan->P; a.log2g = ilog2(plan->g);
    const dim3 grid((unsigned)((plan->Cout_pad + 63) / 64), (unsigned)((plan->P + 63) / 64),
                    (unsigned)plan->splits), block(256);
    hipStream_t s = (hipStream_t)stream;
    if (plan->wbits == 4) {
        if (plan->kstep == 32) hipLaunchKernelGGL((k_direct_conv<false, true, true>), grid, block, 0, s, a);
        else if (plan->g == 64) hipLaunchKernelGGL((k_direct_conv<true, true, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((k_direct_conv<true, false, true>), grid, block, 0, s, a);
    } else {
        if (plan->kstep == 32) hipLaunchKernelGGL((k_direct_conv<false, true, false>), grid, block, 0, s, a);
        else if (plan->g == 64) hipLaunchKernelGGL((k_direct_conv<true, true, false>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((k_direct_conv<true, false, false>), grid, block, 0, s, a);
    }
    if (hipGetLastError() != hipSuccess) return WQ_ERR_DEVICE;
    if (plan->splits > 1) {
        const int total = plan->P * plan->Cout;
        hipLaunchKernelGGL(k_direct_reduce, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           (const float *)a.part, a.bias, y_dev, total, plan->Cout, plan->splits);
    }
    return hipGetLastError() == hipSuccess ? WQ_OK : WQ_ERR_DEVICE;
}

wq_status_t wq_direct_forward(const wq_direct_plan_t *plan, void *stream, const float *x_dev,
                              const void *weight_blob_dev, size_t blob_bytes, void *workspace_dev,
                              size_t workspace_bytes, float *y_dev) {
    if (!plan || !x_dev || !y_dev || !weight_blob_dev || !workspace_dev) return WQ_ERR_INVALID_ARG;
    if (workspace_bytes < plan->lay.ws_bytes || blob_bytes < plan->lay.blob_bytes) return WQ_ERR_WORKSPACE;
    if (!plan->prepared.load()) return WQ_ERR_NOT_PREPARED;
    wq_status_t st = wq_direct_quantize(plan, stream, x_dev, workspace_dev, workspace_bytes);
    if (st != WQ_OK) return st;
    return wq_direct_conv(plan, stream, workspace_dev, workspace_bytes, weight_blob_dev, blob_bytes, y_dev);
}

}  // extern "C"
