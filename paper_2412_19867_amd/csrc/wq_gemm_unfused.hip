// Stages 2 and 3 as two kernels, for layers whose Winograd-domain result
// M [taps][tiles][Cout] (fp32) is small next to their operands: few tiles,
// many channels.  There the fused kernel's register tiles re-read each operand
// block from L2 many times and too few workgroups stream the weights; a
// conventional LDS-tiled GEMM per tap reads every operand block once per
// 64x64 output tile, and M is written once and read once.
//
//   k_gemm_dequant      grid (Cout/64, tiles/64, taps), 4 waves.  Per K-step the
//                       256 threads copy four 16-row weight blocks and four
//                       16-row activation blocks (already in MFMA operand
//                       order) plus the 64+64 scales of the group into LDS,
//                       double buffered, fed from a register ring that keeps two
//                       K-steps in flight; every wave owns a 32x32 quarter
//                       (2x2 int8 MFMA blocks, fresh int32 accumulators per
//                       group) and dequantizes into fp32 at each group end.
//   k_output_transform  one workgroup per (tile, 64 channels), one wave per output
//                       column: y = A^T M A + bias through LDS, NHWC store with the
//                       ragged edge masked.
#include <cstdlib>
#include <cstring>

#include "wq_device.h"
#include "wq_internal.h"

namespace {

// (writing M through, see kWriteThrough, measured 3 % of the ResNet layer set's step)

struct GArgs {
    const int8_t *Xq;
    const float *sX;
    const int8_t *Wq;
    const float *sW;
    float *Mbuf;
    wq_dump dump;   // debug calls: where to store the int32 group sums (P == nullptr otherwise)
    int Cin, T, Cout, T_pad, Cout_pad, log2g, n2;
    // workgroup tiles along channels and tiles, their product with the taps, and the share of
    // each XCD (set by the launcher)
    int nOBt, nTBt, total, per_xcd;
    int m_plain_stores;   // cache policy of the product tensor's stores (see the kernel's end)
};

// TBW = 16-tile blocks per workgroup (4: a 64x64 output tile, waves 2x2; 2: 32 tiles x 128
// channels, waves 1x4, for layers whose padded tile count is an odd multiple of 32).
template <bool K64, bool CPG1, bool WIDE, int TBW, bool DUMP>
__global__ __launch_bounds__(256, 2) void k_gemm_dequant(const GArgs a) {
    constexpr int KSTEP = K64 ? 64 : 32, KB = KSTEP / 4;
    constexpr int BLK = 16 * KSTEP;              // bytes of one K-step of a 16-row block
    constexpr int OBW = TBW == 4 ? 4 : 8;        // 16-channel weight blocks per workgroup
    constexpr int NB = OBW + TBW;                // blocks per stage: weights first, then activations
    constexpr int CPB = BLK / 16;                // 16-byte chunks per block
    constexpr int LPT = (NB * CPB + 255) / 256;  // 16-byte loads per thread per K-step
    constexpr int WN = TBW == 2 ? 4 : 2, WM = 4 / WN;   // waves along channels / along tiles
    constexpr int BN = OBW / WN, BM = TBW / WM;         // 16x16 blocks per wave along channels / tiles
    constexpr int NSW = OBW * 16, NSX = TBW * 16;       // scales per stage
    constexpr unsigned kInvalid = kPastEnd;
    __shared__ __attribute__((aligned(16))) char opnd[2][NB * BLK];
    __shared__ __attribute__((aligned(16))) float sc[2][NSW + NSX];   // weight scales, then activation scales

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), wm = w / WN, wn = w % WN;
    // Workgroup ids go round-robin over the 8 XCDs, whose L2s are private.  XCD x takes the
    // logical tiles [x * per_xcd, (x + 1) * per_xcd) in order, channel tiles fastest, so that
    // the workgroups resident on one XCD at a time are neighbours in (tap, tile, channel) and
    // share their operand tiles in that L2 instead of every XCD fetching every tile.
    const int logical = (int)(blockIdx.x & 7u) * a.per_xcd + (int)(blockIdx.x >> 3);
    if (logical >= a.total) return;   // the whole workgroup leaves, before any barrier
    const int t = logical / (a.nOBt * a.nTBt), rem = logical - t * (a.nOBt * a.nTBt);
    const int ob0 = (rem % a.nOBt) * OBW, tb0 = (rem / a.nOBt) * TBW;   // in 16-row blocks
    const int Cin = a.Cin, T_pad = a.T_pad, Cout_pad = a.Cout_pad;
    const int groups = Cin >> a.log2g, cps = Cin / KSTEP;
    const int cpg_mask = ((1 << a.log2g) / KSTEP) - 1;
    const unsigned n2 = (unsigned)a.n2;

    const __amdgpu_buffer_rsrc_t rW = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.Wq), 0, (int)(n2 * (unsigned)Cout_pad * (unsigned)Cin), kBufFlags);
    const __amdgpu_buffer_rsrc_t rX = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.Xq), 0, (int)(n2 * (unsigned)T_pad * (unsigned)Cin), kBufFlags);
    const __amdgpu_buffer_rsrc_t rSW = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(a.sW), 0, (int)(n2 * (unsigned)groups * (unsigned)Cout_pad * 4u), kBufFlags);
    const __amdgpu_buffer_rsrc_t rSX = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(a.sX), 0, (int)(n2 * (unsigned)T_pad * (unsigned)groups * 4u), kBufFlags);

    // which 16 bytes of the stage this thread copies with load u, as buffer offsets; a wave's
    // 64 chunks lie in one block (K-step 64) or two (K-step 32), all weights or all activations
    unsigned vop[LPT];
    bool is_w[LPT];
#pragma unroll
    for (int u = 0; u < LPT; ++u) {
        const int c = tid + u * 256, blk = c / CPB, off = (c % CPB) * 16;
        is_w[u] = (w * 64 + u * 256) / CPB < OBW;   // wave-uniform
        const int row = blk < OBW ? ob0 + blk : tb0 + blk - OBW;
        const bool ok = blk < NB && row * 16 < (blk < OBW ? Cout_pad : T_pad);
        vop[u] = ok ? (unsigned)(row * 16 * Cin + off) : kInvalid;
    }
    // scales of a group: threads 0..NSW-1 the weight scales, the next NSX the activation scales
    const bool sc_w = w * 64 < NSW;                 // wave-uniform
    unsigned vsc = kInvalid;
    if (tid < NSW) {
        if (ob0 * 16 + tid < Cout_pad) vsc = (unsigned)(ob0 * 16 + tid) * 4u;
    } else if (tid < NSW + NSX) {
        const int r = tid - NSW;                    // tile inside the workgroup's tile range
        if ((tb0 + (r >> 4)) * 16 < T_pad)
            vsc = (unsigned)((tb0 + (r >> 4)) * groups * 64 + (r & 15) * 4);
    }
    const unsigned baseW = (unsigned)t * Cout_pad * Cin, baseX = (unsigned)t * T_pad * Cin;
    const unsigned baseSW = (unsigned)t * groups * Cout_pad * 4, baseSX = (unsigned)t * T_pad * groups * 4;

    // A K-step costs one trip to memory (about a microsecond) unless it was requested long
    // before: PD K-steps are in flight in a register ring whose slots are compile-time
    // indices (the main loop is unrolled PD times), step s is consumed from LDS buffer
    // s & 1 while step s+1 moves from its ring slot into the other buffer.  Every wave
    // issues the same number of loads per K-step and no load sits under a branch, so the
    // wait before the move leaves the newer K-steps outstanding.
    constexpr int PD = 2;   // measured: 2, 4, 6, 8 K-steps in flight, on every tile variant; 2 is as fast as any and starts sooner
    v4i pre[PD][LPT];
    float psc[PD];
    auto fetch = [&](int s, v4i (&dst)[LPT], float &dsc) {   // global -> registers for K-step s
#pragma unroll
        for (int u = 0; u < LPT; ++u) {
            const unsigned so = (is_w[u] ? baseW : baseX) + (unsigned)s * BLK;
            dst[u] = __builtin_amdgcn_raw_buffer_load_b128(is_w[u] ? rW : rX, vop[u], so, 0);
        }
        const unsigned gam = (unsigned)(s * KSTEP) >> a.log2g;
        dsc = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                            sc_w ? rSW : rSX, vsc,
                                            sc_w ? baseSW + gam * (unsigned)Cout_pad * 4u : baseSX + gam * 64u, 0));
    };
    auto commit = [&](int buf, const v4i (&src)[LPT], float ssc) {   // registers -> LDS
#pragma unroll
        for (int u = 0; u < LPT; ++u)
            if ((u + 1) * 256 <= NB * CPB || tid + u * 256 < NB * CPB)
                *reinterpret_cast<v4i *>(&opnd[buf][(tid + u * 256) * 16]) = src[u];
        if (tid < NSW + NSX) sc[buf][tid] = ssc;
    };

    v4i acc[BN][BM];
    float4 Mc[BN][BM];
    double Mt[BN][BM][4];
#pragma unroll
    for (int no = 0; no < BN; ++no)
#pragma unroll
        for (int nt = 0; nt < BM; ++nt) {
            acc[no][nt] = v4i{0, 0, 0, 0};
            Mc[no][nt] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int r = 0; r < 4; ++r) Mt[no][nt][r] = 0.0;
        }
    int in_chunk = 0;

    const int last = cps - 1;
    // The K loop starts at a group that depends on the workgroup and wraps round: workgroups
    // that run side by side then read different K positions of their rows at any one time
    // (their rows are a multiple of 256 bytes apart, so equal K positions land on the same
    // few L2 channels; measured 4-7 % on layers with thousands of workgroups, nothing on
    // small ones).  The integer sums of a group do not depend on the order; the fp32 sum
    // over the groups is taken in the rotated order.
    const int k_rot = (logical % groups) * (cpg_mask + 1);
    auto kpos = [&](int k) { const int v = k + k_rot; return v >= cps ? v - cps : v; };
#pragma unroll
    for (int u = 0; u < PD; ++u) fetch(kpos(min(u, last)), pre[u], psc[u]);
    commit(0, pre[0], psc[0]);
    __syncthreads();
    for (int sb = 0; sb < cps; sb += PD) {
#pragma unroll
      for (int u = 0; u < PD; ++u) {
        const int s = sb + u;
        if (s >= cps) break;
        const int buf = u & 1;   // PD is even, so s & 1 == u & 1
        fetch(kpos(min(s + PD, last)), pre[u], psc[u]);   // slot u held step s, already in LDS
        // operands of this wave's BN x BM blocks
        v4i av[BN], bv[BM];
#pragma unroll
        for (int e = 0; e < BN; ++e) {
            const char *pa = &opnd[buf][(BN * wn + e) * BLK + lane * KB];
            if constexpr (K64) {
                av[e] = *reinterpret_cast<const v4i *>(pa);
            } else {
                const v2i ta = *reinterpret_cast<const v2i *>(pa);
                av[e] = v4i{ta.x, ta.y, 0, 0};
            }
        }
#pragma unroll
        for (int e = 0; e < BM; ++e) {
            const char *pb = &opnd[buf][(OBW + BM * wm + e) * BLK + lane * KB];
            if constexpr (K64) {
                bv[e] = *reinterpret_cast<const v4i *>(pb);
            } else {
                const v2i tb = *reinterpret_cast<const v2i *>(pb);
                bv[e] = v4i{tb.x, tb.y, 0, 0};
            }
        }
#pragma unroll
        for (int no = 0; no < BN; ++no)
#pragma unroll
            for (int nt = 0; nt < BM; ++nt) {
                const v4i c0 = CPG1 ? v4i{0, 0, 0, 0} : acc[no][nt];
                if constexpr (K64) {
                    acc[no][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av[no], bv[nt], c0, 0, 0, 0);
                } else {
                    const long x = __builtin_bit_cast(long, v2i{av[no].x, av[no].y});
                    const long y = __builtin_bit_cast(long, v2i{bv[nt].x, bv[nt].y});
                    acc[no][nt] = __builtin_amdgcn_mfma_i32_16x16x32_i8(x, y, c0, 0, 0, 0);
                }
            }
        if (CPG1 || ((s + 1) & cpg_mask) == 0) {   // last K-step of a group: dequantize
#pragma unroll
            for (int no = 0; no < BN; ++no) {
                const v4f sw = *reinterpret_cast<const v4f *>(&sc[buf][(BN * wn + no) * 16 + 4 * q]);
#pragma unroll
                for (int nt = 0; nt < BM; ++nt) {
                    const float sx = sc[buf][NSW + (BM * wm + nt) * 16 + l16];
                    Mc[no][nt].x = __builtin_fmaf((float)acc[no][nt][0], sw.x * sx, Mc[no][nt].x);
                    Mc[no][nt].y = __builtin_fmaf((float)acc[no][nt][1], sw.y * sx, Mc[no][nt].y);
                    Mc[no][nt].z = __builtin_fmaf((float)acc[no][nt][2], sw.z * sx, Mc[no][nt].z);
                    Mc[no][nt].w = __builtin_fmaf((float)acc[no][nt][3], sw.w * sx, Mc[no][nt].w);
                    if constexpr (DUMP) {   // the debug entry point's instance of this kernel
                        const int v[4] = {acc[no][nt][0], acc[no][nt][1], acc[no][nt][2], acc[no][nt][3]};
                        wq_dump_store(a.dump, t, (tb0 + BM * wm + nt) * 16 + l16,
                                      (kpos(s) * KSTEP) >> a.log2g, groups,
                                      (ob0 + BN * wn + no) * 16 + 4 * q, a.Cout, a.T, v);
                    }
                    if constexpr (!CPG1) acc[no][nt] = v4i{0, 0, 0, 0};
                }
            }
            if (WIDE && ++in_chunk == 4) {   // fp64 totals of 4-group fp32 chunks (long reductions)
                in_chunk = 0;
#pragma unroll
                for (int no = 0; no < BN; ++no)
#pragma unroll
                    for (int nt = 0; nt < BM; ++nt) {
                        Mt[no][nt][0] += (double)Mc[no][nt].x;
                        Mt[no][nt][1] += (double)Mc[no][nt].y;
                        Mt[no][nt][2] += (double)Mc[no][nt].z;
                        Mt[no][nt][3] += (double)Mc[no][nt].w;
                        Mc[no][nt] = make_float4(0.f, 0.f, 0.f, 0.f);
                    }
            }
        }
        if (s + 1 < cps) commit(buf ^ 1, pre[(u + 1) % PD], psc[(u + 1) % PD]);
        __syncthreads();
      }
    }
    // M is below 2 GiB (checked when the plan is made), so 32-bit offsets reach all of it
    const __amdgpu_buffer_rsrc_t rM = __builtin_amdgcn_make_buffer_rsrc(
        a.Mbuf, 0, (int)(n2 * (unsigned)T_pad * (unsigned)Cout_pad * 4u), kBufFlags);
    // store M [tile][tap][Cout_pad] (a tile's taps together: the output transform reads them
    // from one contiguous region); the lane holds channels 4q..4q+3 of tile l16 in each block
#pragma unroll
    for (int no = 0; no < BN; ++no)
#pragma unroll
        for (int nt = 0; nt < BM; ++nt) {
            float4 Mv = Mc[no][nt];
            if constexpr (WIDE)
                Mv = make_float4((float)(Mt[no][nt][0] + (double)Mv.x), (float)(Mt[no][nt][1] + (double)Mv.y),
                                 (float)(Mt[no][nt][2] + (double)Mv.z), (float)(Mt[no][nt][3] + (double)Mv.w));
            const int tau = (tb0 + BM * wm + nt) * 16 + l16, o = (ob0 + BN * wn + no) * 16 + 4 * q;
            if (tau < T_pad && o < Cout_pad) {
                const v4i bits = __builtin_bit_cast(v4i, v4f{Mv.x, Mv.y, Mv.z, Mv.w});
                const unsigned off =
                    (((unsigned)tau * n2 + (unsigned)t) * (unsigned)Cout_pad + (unsigned)o) * 4u;
                // a product tensor far larger than the caches: plain stores; otherwise written
                // through, which spares the flush at the kernel's end (each measured ~5 % better
                // on its side)
                if (a.m_plain_stores) __builtin_amdgcn_raw_buffer_store_b128(bits, rM, off, 0, 0);
                else __builtin_amdgcn_raw_buffer_store_b128(bits, rM, off, 0, kWriteThrough);
            }
        }
}

struct OArgs {
    wq_xf xf;
    const float *Mbuf;
    const float *bias;
    float *y;
    int H, W, Cout, TH, TW, T, T_pad, Cout_pad;
};

// One workgroup per (tile, 64 output channels): the tile's n*n x 64 slice of M goes
// through LDS once, then wave b (one per output column) forms column b of Y A and of
// A^T (Y A).  Splitting an element's work over M waves keeps several waves on every
// SIMD even for layers with few tiles; a lone wave per SIMD issues at a fraction of
// the vector-ALU rate.
template <int M, bool ATSP>
__global__ __launch_bounds__(64 * M) void k_output_transform(const OArgs a) {
    constexpr int n = M + 2, n2 = n * n;
    using Pat = wq_pattern<M>;
    __shared__ __attribute__((aligned(16))) float Ms[n2][64];
    const int tid = threadIdx.x, ol = tid & 63;
    const int b = __builtin_amdgcn_readfirstlane(tid >> 6);   // output column of this wave
    const int o0 = blockIdx.y * 64, tau = blockIdx.x;
    const float *src = a.Mbuf + (size_t)tau * n2 * a.Cout_pad + o0;   // M [tile][tap][Cout_pad]
    for (int idx = tid; idx < n2 * 16; idx += 64 * M) {
        const int t = idx >> 4, c4 = (idx & 15) * 4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (o0 + c4 < a.Cout_pad) v = *reinterpret_cast<const float4 *>(src + (size_t)t * a.Cout_pad + c4);
        *reinterpret_cast<float4 *>(&Ms[t][c4]) = v;
    }
    __syncthreads();
    // column pass R = M A^T[b][:] with the wave's (run-time) row b of A^T
    float atb[n];
#pragma unroll
    for (int j = 0; j < n; ++j) atb[j] = a.xf.AT[b * n + j];
    float R[n];
#pragma unroll
    for (int i = 0; i < n; ++i) {
        float r = 0.f;
#pragma unroll
        for (int j = 0; j < n; ++j) r = __builtin_fmaf(atb[j], Ms[i * n + j][ol], r);
        R[i] = r;
    }
    const int o = o0 + ol;
    const int tw = tau % a.TW, th = (tau / a.TW) % a.TH, bb = tau / (a.TW * a.TH);
    const int hv = min(M, a.H - th * M), wv = min(M, a.W - tw * M);
    if (o < a.Cout && b < wv) {
        const float bv = a.bias[o];
        float *dst = a.y + ((size_t)(bb * a.H + th * M) * a.W + tw * M + b) * a.Cout + o;
        float Yv[M];
        wq_apply_at<M, ATSP>(a.xf, R, Yv);
#pragma unroll
        for (int aa = 0; aa < M; ++aa) {
            const float yv = Yv[aa];
            if (aa < hv)   // streaming store: y is not read again by this layer
                store_y(yv + bv, &dst[(size_t)aa * a.W * a.Cout]);
        }
    }
}

// Third quantized-stage equation of Section "Learnable Winograd transform scales":
//     y = s_A[a] s_A[b] s_Y  (Q_A Q(Y / s_Y) Q_A^T)[a][b] + bias
// with the int8 matrix Q_A = Q(A^T / s_A) from the plan and one dynamic scale s_Y = abs-max / 127
// per (tile, output channel) over its n x n Winograd-domain values; the integer product is exact,
// scales and bias in fp64, one rounding to fp32 at the store.  One thread per (tile, channel):
// 4 tiles x 64 channels per workgroup, M [tile][tap][Cout_pad] read straight from the workspace
// (a wave's 64 lanes read 256 contiguous bytes per tap).
struct OIArgs {
    wq_xi xi;
    const float *Mbuf;
    const float *bias;
    float *y;
    int H, W, Cout, TH, TW, T, T_pad, Cout_pad;
};

template <int M>
__global__ __launch_bounds__(256) void k_output_transform_int(const OIArgs a) {
    constexpr int n = M + 2, n2 = n * n;
    const int tid = threadIdx.x, ol = tid & 63;
    const int tau = blockIdx.x * 4 + (tid >> 6), o = blockIdx.y * 64 + ol;
    if (tau >= a.T || o >= a.Cout) return;
    const float *src = a.Mbuf + (size_t)tau * n2 * a.Cout_pad + o;
    float Yv[n2];
    float am = 0.f;
#pragma unroll
    for (int t = 0; t < n2; ++t) {
        Yv[t] = src[(size_t)t * a.Cout_pad];
        am = __builtin_fmaxf(am, __builtin_fabsf(Yv[t]));
    }
    const double a_y = (double)am;
    const double s_y = a_y > 0.0 ? a_y / 127.0 : 0.0, r_y = a_y > 0.0 ? 127.0 / a_y : 0.0;
    int q[n][n];
#pragma unroll
    for (int i = 0; i < n; ++i)
#pragma unroll
        for (int j = 0; j < n; ++j)
            q[i][j] = (int)fmin(127.0, fmax(-127.0, rint((double)Yv[i * n + j] * r_y)));
    int u[M][n];   // Q_A q
#pragma unroll
    for (int aa = 0; aa < M; ++aa)
#pragma unroll
        for (int j = 0; j < n; ++j) {
            int acc = 0;
#pragma unroll
            for (int i = 0; i < n; ++i) acc += a.xi.QA[aa * n + i] * q[i][j];
            u[aa][j] = acc;
        }
    const int tw = tau % a.TW, th = (tau / a.TW) % a.TH, bb = tau / (a.TW * a.TH);
    const int hv = min(M, a.H - th * M), wv = min(M, a.W - tw * M);
    const double bv = (double)a.bias[o];
    float *base = a.y + ((size_t)(bb * a.H + th * M) * a.W + tw * M) * a.Cout + o;
#pragma unroll
    for (int aa = 0; aa < M; ++aa)
#pragma unroll
        for (int b = 0; b < M; ++b) {
            int acc = 0;
#pragma unroll
            for (int j = 0; j < n; ++j) acc += u[aa][j] * a.xi.QA[b * n + j];
            const double v = (a.xi.sAA[aa * M + b] * s_y) * (double)acc + bv;
            if (aa < hv && b < wv) store_y((float)v, base + ((size_t)aa * a.W + b) * a.Cout);
        }
}

// plain, or (debug entry point) the same kernel with the stores of the int32 sums compiled in
template <bool K64, bool CPG1, bool WIDE, int TBW>
void launch_one(dim3 grid, hipStream_t s, const GArgs &g) {
    if (g.dump.P) hipLaunchKernelGGL((k_gemm_dequant<K64, CPG1, WIDE, TBW, true>), grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL((k_gemm_dequant<K64, CPG1, WIDE, TBW, false>), grid, dim3(256), 0, s, g);
}

template <bool K64, bool CPG1>
void launch_gemm(const GArgs &g0, hipStream_t s, bool wide, bool narrow, bool big) {
    GArgs g = g0;
    auto shape = [&](int ch_per_wg, int tiles_per_wg) {
        g.nOBt = (g.Cout_pad + ch_per_wg - 1) / ch_per_wg;
        g.nTBt = (g.T_pad + tiles_per_wg - 1) / tiles_per_wg;
        g.total = g.nOBt * g.nTBt * g.n2;
        g.per_xcd = (g.total + 7) / 8;
        return dim3((unsigned)g.per_xcd * 8u);
    };
    if constexpr (K64 && !CPG1) {
        if (big && !wide) {
            const dim3 grid = shape(128, 128);
            launch_one<true, false, false, 8>(grid, s, g);
            return;
        }
    }
    if (narrow) {
        const dim3 grid = shape(128, 32);
        if (wide)
            launch_one<K64, CPG1, true, 2>(grid, s, g);
        else
            launch_one<K64, CPG1, false, 2>(grid, s, g);
    } else {
        const dim3 grid = shape(64, 64);
        if (wide)
            launch_one<K64, CPG1, true, 4>(grid, s, g);
        else
            launch_one<K64, CPG1, false, 4>(grid, s, g);
    }
}

template <int M>
void launch_out(const OArgs &o, dim3 grid, hipStream_t s, bool atsp) {
    if (atsp)
        hipLaunchKernelGGL((k_output_transform<M, true>), grid, dim3(64 * M), 0, s, o);
    else
        hipLaunchKernelGGL((k_output_transform<M, false>), grid, dim3(64 * M), 0, s, o);
}

}  // namespace

hipError_t wq_launch_contract_unfused(const wq_plan *p, hipStream_t s, const int8_t *Xq, const float *sX,
                                      const int8_t *Wq, const float *sW, const float *bias, float *Mbuf,
                                      float *y, int stages, const wq_dump &dump) {
    if (stages & 1) {
    GArgs g;
    g.Xq = Xq; g.sX = sX; g.Wq = Wq; g.sW = sW; g.Mbuf = Mbuf; g.dump = dump;
    g.Cin = p->Cin; g.T = p->T; g.Cout = p->Cout; g.T_pad = p->T_pad; g.Cout_pad = p->Cout_pad;
    g.n2 = p->n * p->n;
    g.log2g = 0;
    while ((1 << g.log2g) < p->g) ++g.log2g;
    g.m_plain_stores = (long long)g.n2 * p->T_pad * p->Cout_pad * 4 > (128LL << 20);
    const bool k64 = p->kstep == 64, cpg1 = p->g == p->kstep, wide = p->groups > 8;
    // the tile shape is the plan's variant when that is one of this kernel's; a plan of another
    // variant that calls this stage on its own (wq_contract) gets the 64x64 tiles
    const bool narrow = p->k2_variant == WQ_K2_GEMM_32x128;
    const bool big = p->k2_variant == WQ_K2_GEMM_128x128;
    if (!k64) launch_gemm<false, true>(g, s, wide, narrow, big);
    else if (cpg1) launch_gemm<true, true>(g, s, wide, narrow, big);
    else launch_gemm<true, false>(g, s, wide, narrow, big);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    }
    if (!(stages & 2)) return hipSuccess;

    OArgs o;
    o.xf = p->xf; o.Mbuf = Mbuf; o.bias = bias; o.y = y;
    o.H = p->H; o.W = p->W; o.Cout = p->Cout; o.TH = p->TH; o.TW = p->TW; o.T = p->T;
    o.T_pad = p->T_pad; o.Cout_pad = p->Cout_pad;
    if (p->integer_transforms) {
        OIArgs oi;
        oi.xi = p->xi; oi.Mbuf = Mbuf; oi.bias = bias; oi.y = y;
        oi.H = p->H; oi.W = p->W; oi.Cout = p->Cout; oi.TH = p->TH; oi.TW = p->TW; oi.T = p->T;
        oi.T_pad = p->T_pad; oi.Cout_pad = p->Cout_pad;
        const dim3 igrid((p->T + 3) / 4, (p->Cout + 63) / 64);
        switch (p->m) {
            case 2: hipLaunchKernelGGL((k_output_transform_int<2>), igrid, dim3(256), 0, s, oi); break;
            case 4: hipLaunchKernelGGL((k_output_transform_int<4>), igrid, dim3(256), 0, s, oi); break;
            default: hipLaunchKernelGGL((k_output_transform_int<6>), igrid, dim3(256), 0, s, oi); break;
        }
        return hipGetLastError();
    }
    const dim3 ogrid(p->T, (p->Cout + 63) / 64);   // tiles along x: y holds 65535 at most
    switch (p->m) {
        case 2: launch_out<2>(o, ogrid, s, p->sparse_at); break;
        case 4: launch_out<4>(o, ogrid, s, p->sparse_at); break;
        default: launch_out<6>(o, ogrid, s, p->sparse_at); break;
    }
    return hipGetLastError();
}
