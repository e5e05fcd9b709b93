// Stages 2+3 for gfx950: the Winograd-domain contraction as int8 MFMA GEMMs
// with per-group dequantization, and the output transform y = A^T Y A + bias
// fused behind it, so the n*n fp32 Winograd-domain planes never reach memory.
//
// Work decomposition
//   workgroup  = one (16*NT tiles) x (16*NO output channels) block, ALL n*n taps;
//   wave       = (tap row i, K slice ks): taps i*n .. i*n+n-1 over 1/KS of the
//                input channels (whole quantization groups);  n*KS waves.
// A wave walks a flat sequence of K-steps (tap-major, then channels):
//   int32 block  = MFMA(Wq block, Xq block)       exact, fresh per group
//   M           += float(block) * (sW[o] * sX[tile])     at the end of each group
// A operand = 16 output channels, B operand = 16 tiles.  Both tensors are stored
// in the blocked operand order (include/wq.h), so one K-step of one 16-row block
// is 16*KSTEP contiguous bytes and every lane fetches KB bytes at lane*KB; the
// exact integer sum does not depend on how the instruction orders K as long as
// A and B use the same order, which they do.  Operands and scales are fetched D
// K-steps ahead into registers with buffer loads whose running offsets are
// scalar.  At the end of a tap the wave folds M into R[b] += A^T[b][j] * M (its
// share of row i of Y A); after its n taps R goes through LDS and the workgroup
// finishes Y[a][b] = sum_i A^T[a][i] (sum_ks R_{i,ks}[b]), adds bias and stores
// NHWC with the ragged right/bottom edge masked.
//
// Workgroups are numbered so that the eight XCDs (which receive consecutive
// workgroup ids round-robin and have private L2s) each own a slice of the
// larger operand: with xcd_mode 0 an XCD owns every 8th block of output
// channels (weights stay in its L2), with xcd_mode 1 every 8th block of tiles,
// with xcd_mode 2 every 4th block of tiles and one half of the channels.
#pragma once

#include "wq_device.h"
#include "wq_internal.h"

namespace {   // every including file instantiates its own tile size; nothing here is exported

constexpr int kPrefetchBase = 4;         // K-steps in flight of the 16x16 configurations
constexpr int RS_STRIDE = 20;           // floats per tile row of the LDS exchange (16 + pad)

struct Args {
    wq_xf xf;
    const int8_t *Xq;
    const float *sX;
    const int8_t *Wq;
    const float *sW;
    const float *bias;
    float *y;
    wq_dump dump;   // debug calls: where to store the int32 group sums (P == nullptr otherwise)
    int H, W, Cin, Cout, TH, TW, T, T_pad, Cout_pad, log2g;
    int nTB, nOB, xcd_mode;
};

template <bool K64, int NT, int NO>
struct Stage {
    v4i a[NO], b[NT];   // K64: 16 operand bytes per lane; otherwise .xy only
    v4f sw[NO];         // weight scales of the lane's 4 output channels per sub-block
    float sx[NT];       // activation scale of the lane's tile per sub-block
};

template <int M, bool K64, bool CPG1, bool WIDE, bool ATSP, bool DUMP, int NT, int NO, int KS, int D>
__global__ __launch_bounds__(64 * (M + 2) * KS) void k_contract_output(const Args a) {
    constexpr int n = M + 2;
    constexpr int KSTEP = K64 ? 64 : 32;   // K per MFMA
    constexpr int KB = KSTEP / 4;          // operand bytes per lane per MFMA
    constexpr int NW = n * KS;             // waves
    // output columns per LDS pass: all M when the exchange area fits 64 KiB, else half of them
    constexpr int BP = NW * M * 16 * RS_STRIDE * 4 <= 65536 ? M : M / 2;
    constexpr int NTH = (64 * NW / 256) * 256;   // threads of the final phase: a multiple of 256,
                                                 // so that a thread keeps its (tile, channel) position
    using Pat = wq_pattern<M>;
    __shared__ float Rs[NW][BP][16 * RS_STRIDE];

    // ---- which block (uniform) ----
    int tb, ob;
    {
        const int id = blockIdx.x, xcd = id & 7, s = id >> 3;
        if (a.xcd_mode == 0) {
            ob = (s / a.nTB) * 8 + xcd;
            tb = s % a.nTB;
        } else if (a.xcd_mode == 1) {
            tb = (s / a.nOB) * 8 + xcd;
            ob = s % a.nOB;
        } else {   // 4 parts of the tiles x 2 halves of the channels
            const int hob = (a.nOB + 1) >> 1;
            tb = (s / hob) * 4 + (xcd >> 1);
            ob = (xcd & 1) * hob + s % hob;
        }
        if (tb >= a.nTB || ob >= a.nOB) return;
    }
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i = w % n, ks = w / n;   // tap row, K slice (uniform)
    const int tau0 = tb * 16 * NT, o0 = ob * 16 * NO;
    const int Cin = a.Cin, Cout_pad = a.Cout_pad, T_pad = a.T_pad;
    const int groups = Cin >> a.log2g;
    const int gps = groups / KS;                 // groups per K slice
    const int cps = (Cin / KSTEP) / KS;          // K-steps per tap for this wave
    const int cpg_mask = ((1 << a.log2g) / KSTEP) - 1;

    const unsigned n2 = n * n;
    const __amdgpu_buffer_rsrc_t rW = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.Wq), 0, (int)(n2 * (unsigned)Cout_pad * (unsigned)Cin), kBufFlags);
    const __amdgpu_buffer_rsrc_t rX = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.Xq), 0, (int)(n2 * (unsigned)T_pad * (unsigned)Cin), kBufFlags);
    const __amdgpu_buffer_rsrc_t rSW = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(a.sW), 0, (int)(n2 * (unsigned)groups * (unsigned)Cout_pad * 4u),
        kBufFlags);
    const __amdgpu_buffer_rsrc_t rSX = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(a.sX), 0, (int)(n2 * (unsigned)T_pad * (unsigned)groups * 4u),
        kBufFlags);
    // per-lane byte offsets inside a tap plane (sub-block 0); the tap/K position is scalar
    const int vW = o0 * Cin + lane * KB;
    const int vX = tau0 * Cin + lane * KB;
    const int vSW = (o0 + 4 * q) * 4;                       // sW [tap][group][Cout_pad]
    const int vSX = (tau0 >> 4) * groups * 64 + l16 * 4;    // sX [tap][16-tile block][group][16]
    const unsigned planeW = (unsigned)Cout_pad * Cin, planeX = (unsigned)T_pad * Cin;
    const unsigned planeSW = (unsigned)groups * Cout_pad * 4, planeSX = (unsigned)T_pad * groups * 4;
    constexpr unsigned stepOp = 16 * KSTEP;                 // bytes of one K-step of a 16-row block
    const unsigned stepSW = (unsigned)Cout_pad * 4;
    // scalar running offsets of the loader, and what to add when it wraps to the next tap
    const unsigned t0 = (unsigned)(i * n);
    unsigned oW = t0 * planeW + (unsigned)(ks * cps) * stepOp;
    unsigned oX = t0 * planeX + (unsigned)(ks * cps) * stepOp;
    unsigned oSW = t0 * planeSW + (unsigned)(ks * gps) * stepSW;
    unsigned oSX = t0 * planeSX + (unsigned)(ks * gps) * 64u;
    const unsigned dW = planeW - (unsigned)cps * stepOp, dX = planeX - (unsigned)cps * stepOp;
    const unsigned dSW = planeSW - (unsigned)gps * stepSW, dSX = planeSX - (unsigned)gps * 64u;
    int k_ld = cps, kg_ld = 0;

    auto load_stage = [&](Stage<K64, NT, NO> &s) {
#pragma unroll
        for (int no = 0; no < NO; ++no) {
            if constexpr (K64) {
                s.a[no] = __builtin_amdgcn_raw_buffer_load_b128(rW, vW + no * 16 * Cin, oW, 0);
            } else {
                const v2i t = __builtin_amdgcn_raw_buffer_load_b64(rW, vW + no * 16 * Cin, oW, 0);
                s.a[no] = v4i{t.x, t.y, 0, 0};
            }
            s.sw[no] = __builtin_bit_cast(
                v4f, __builtin_amdgcn_raw_buffer_load_b128(rSW, vSW + no * 64, oSW, 0));
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if constexpr (K64) {
                s.b[nt] = __builtin_amdgcn_raw_buffer_load_b128(rX, vX + nt * 16 * Cin, oX, 0);
            } else {
                const v2i t = __builtin_amdgcn_raw_buffer_load_b64(rX, vX + nt * 16 * Cin, oX, 0);
                s.b[nt] = v4i{t.x, t.y, 0, 0};
            }
            s.sx[nt] = __builtin_bit_cast(
                float, __builtin_amdgcn_raw_buffer_load_b32(rSX, vSX + nt * groups * 64, oSX, 0));
        }
        oW += stepOp;
        oX += stepOp;
        if (CPG1 || (++kg_ld & cpg_mask) == 0) {
            oSW += stepSW;
            oSX += 64u;
        }
        if (--k_ld == 0) {
            k_ld = cps;
            oW += dW;
            oX += dX;
            oSW += dSW;
            oSX += dSX;
        }
    };

    float4 R[M][NO][NT];
#pragma unroll
    for (int b = 0; b < M; ++b)
#pragma unroll
        for (int no = 0; no < NO; ++no)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) R[b][no][nt] = make_float4(0.f, 0.f, 0.f, 0.f);

    const int NI = n * cps;   // >= n >= 4 >= D
    Stage<K64, NT, NO> st[D];
#pragma unroll
    for (int d = 0; d < D; ++d) load_stage(st[d]);
    int loads_left = NI - D;

    // compute cursor (uniform)
    int j_cp = 0, k_left = cps, kg_cp = 0, gam_cp = 0, in_chunk = 0;
    v4i acc[NO][NT];
    float4 Mc[NO][NT];
    double Mt[NO][NT][4];
#pragma unroll
    for (int no = 0; no < NO; ++no)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            acc[no][nt] = v4i{0, 0, 0, 0};
            Mc[no][nt] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int r = 0; r < 4; ++r) Mt[no][nt][r] = 0.0;
        }
    float atc[M];
#pragma unroll
    for (int b = 0; b < M; ++b) atc[b] = a.xf.AT[b * n];   // column of tap j = 0

    for (int it = 0; it < NI; it += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (it + d < NI) {
                Stage<K64, NT, NO> &s = st[d];
#pragma unroll
                for (int no = 0; no < NO; ++no)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        const v4i c0 = CPG1 ? v4i{0, 0, 0, 0} : acc[no][nt];
                        if constexpr (K64) {
                            acc[no][nt] =
                                __builtin_amdgcn_mfma_i32_16x16x64_i8(s.a[no], s.b[nt], c0, 0, 0, 0);
                        } else {
                            const long av = __builtin_bit_cast(long, v2i{s.a[no].x, s.a[no].y});
                            const long bv = __builtin_bit_cast(long, v2i{s.b[nt].x, s.b[nt].y});
                            acc[no][nt] = __builtin_amdgcn_mfma_i32_16x16x32_i8(av, bv, c0, 0, 0, 0);
                        }
                    }
                const bool group_end = CPG1 || ((++kg_cp & cpg_mask) == 0);
                float4 c[NO][NT];
#pragma unroll
                for (int no = 0; no < NO; ++no)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        c[no][nt] = make_float4(s.sw[no].x * s.sx[nt], s.sw[no].y * s.sx[nt],
                                                s.sw[no].z * s.sx[nt], s.sw[no].w * s.sx[nt]);
                if (loads_left > 0) {   // the stage's registers are free again: refill them
                    load_stage(s);
                    --loads_left;
                }
                if (group_end) {
#pragma unroll
                    for (int no = 0; no < NO; ++no)
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt) {
                            Mc[no][nt].x = __builtin_fmaf((float)acc[no][nt][0], c[no][nt].x, Mc[no][nt].x);
                            Mc[no][nt].y = __builtin_fmaf((float)acc[no][nt][1], c[no][nt].y, Mc[no][nt].y);
                            Mc[no][nt].z = __builtin_fmaf((float)acc[no][nt][2], c[no][nt].z, Mc[no][nt].z);
                            Mc[no][nt].w = __builtin_fmaf((float)acc[no][nt][3], c[no][nt].w, Mc[no][nt].w);
                            if constexpr (DUMP) {   // the debug entry point's instance of this kernel
                                const int v[4] = {acc[no][nt][0], acc[no][nt][1], acc[no][nt][2],
                                                  acc[no][nt][3]};
                                wq_dump_store(a.dump, i * n + j_cp, tau0 + nt * 16 + l16,
                                              ks * gps + gam_cp, groups, o0 + no * 16 + 4 * q, a.Cout,
                                              a.T, v);
                            }
                            if constexpr (!CPG1) acc[no][nt] = v4i{0, 0, 0, 0};
                        }
                    ++gam_cp;
                    if (WIDE && ++in_chunk == 4) {   // fp64 totals of 4-group fp32 chunks (long reductions)
                        in_chunk = 0;
#pragma unroll
                        for (int no = 0; no < NO; ++no)
#pragma unroll
                            for (int nt = 0; nt < NT; ++nt) {
                                Mt[no][nt][0] += (double)Mc[no][nt].x;
                                Mt[no][nt][1] += (double)Mc[no][nt].y;
                                Mt[no][nt][2] += (double)Mc[no][nt].z;
                                Mt[no][nt][3] += (double)Mc[no][nt].w;
                                Mc[no][nt] = make_float4(0.f, 0.f, 0.f, 0.f);
                            }
                    }
                }
                if (--k_left == 0) {   // end of tap j_cp: fold into (this slice's share of) row i of Y A
                    k_left = cps;
                    gam_cp = 0;
                    in_chunk = 0;
                    // branch-free on purpose: entries of A^T that are zero simply add nothing
#pragma unroll
                    for (int no = 0; no < NO; ++no)
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt) {
                            float4 Mv = Mc[no][nt];
                            if constexpr (WIDE) {
                                Mv = make_float4((float)(Mt[no][nt][0] + (double)Mv.x),
                                                 (float)(Mt[no][nt][1] + (double)Mv.y),
                                                 (float)(Mt[no][nt][2] + (double)Mv.z),
                                                 (float)(Mt[no][nt][3] + (double)Mv.w));
#pragma unroll
                                for (int r = 0; r < 4; ++r) Mt[no][nt][r] = 0.0;
                            }
                            Mc[no][nt] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                            for (int b = 0; b < M; ++b) {
                                float4 &Rb = R[b][no][nt];
                                Rb.x = __builtin_fmaf(atc[b], Mv.x, Rb.x);
                                Rb.y = __builtin_fmaf(atc[b], Mv.y, Rb.y);
                                Rb.z = __builtin_fmaf(atc[b], Mv.z, Rb.z);
                                Rb.w = __builtin_fmaf(atc[b], Mv.w, Rb.w);
                            }
                        }
                    ++j_cp;
                    const int jn = j_cp < n ? j_cp : 0;
#pragma unroll
                    for (int b = 0; b < M; ++b) atc[b] = a.xf.AT[b * n + jn];
                }
            }
        }
    }

    // Every thread finishes the same (tile, channel) position of each sub-block: where
    // that tile's outputs start, how much of it lies inside the image, and the bias.
    const int tl = (tid >> 4) & 15, ol = tid & 15;
    int out_off[NT], out_lim[NT];
    float bias_v[NO];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int tau = tau0 + nt * 16 + tl;
        out_off[nt] = 0;
        out_lim[nt] = 0;
        if (tau < a.T) {
            const int tw = tau % a.TW, th = (tau / a.TW) % a.TH, bb = tau / (a.TW * a.TH);
            out_off[nt] = ((bb * a.H + th * M) * a.W + tw * M) * a.Cout;
            out_lim[nt] = min(M, a.H - th * M) | (min(M, a.W - tw * M) << 8);
        }
    }
#pragma unroll
    for (int no = 0; no < NO; ++no) {
        const int o = o0 + no * 16 + ol;
        bias_v[no] = o < a.Cout ? a.bias[o] : 0.f;
    }

    // ---- output transform across tap rows, one 16x16 sub-block and BP columns at a time ----
    bool first = true;
#pragma unroll
    for (int no = 0; no < NO; ++no)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int p = 0; p < M / BP; ++p) {
                if (!first) __syncthreads();
                first = false;
#pragma unroll
                for (int bp = 0; bp < BP; ++bp)
                    *reinterpret_cast<float4 *>(&Rs[w][bp][l16 * RS_STRIDE + 4 * q]) =
                        R[p * BP + bp][no][nt];
                __syncthreads();
                for (int idx = tid < NTH ? tid : BP * 256; idx < BP * 256; idx += NTH) {
                    const int bp = idx >> 8;   // idx & 255 == tid & 255 for every iteration
                    const int bcol = p * BP + bp;
                    float Yv[M], rv[n];
#pragma unroll
                    for (int ii = 0; ii < n; ++ii) {
                        rv[ii] = Rs[ii][bp][tl * RS_STRIDE + ol];
#pragma unroll
                        for (int k2 = 1; k2 < KS; ++k2) rv[ii] += Rs[k2 * n + ii][bp][tl * RS_STRIDE + ol];
                    }
                    wq_apply_at<M, ATSP>(a.xf, rv, Yv);
                    const int hv = out_lim[nt] & 0xff, wv = out_lim[nt] >> 8;
                    const int o = o0 + no * 16 + ol;
                    if (bcol < wv && o < a.Cout) {
                        float *dst = a.y + (size_t)out_off[nt] + bcol * a.Cout + o;
#pragma unroll
                        for (int aa = 0; aa < M; ++aa)
                            if (aa < hv)   // streaming store: y is not read again by this layer
                                store_y(Yv[aa] + bias_v[no],
                                                            &dst[(size_t)aa * a.W * a.Cout]);
                    }
                }
            }
}

template <int M, bool K64, bool CPG1, bool WIDE, bool ATSP, int NT, int NO, int KS, int D>
hipError_t launch_cfg(const Args &a, hipStream_t s) {
    // the debug entry point runs the same template with the stores of the int32 sums compiled in
    Args b = a;
    b.nTB = a.T_pad / (16 * NT);
    b.nOB = a.Cout_pad / (16 * NO);
    // the XCDs partition the blocks of the larger operand
    const long wbytes = (long)a.Cout_pad * a.Cin, xbytes = (long)a.T_pad * a.Cin;
    b.xcd_mode = wbytes >= xbytes ? 0 : 1;
    // tiles split over the XCDs, but all taps' weights would fill an XCD's 4 MB L2 on their own:
    // split the channels in two as well, so that half of the weights stays resident next to the
    // streaming activations
    const long wall = wbytes * (M + 2) * (M + 2);
    if (b.xcd_mode == 1 && wall > (5L << 19) && wall <= (8L << 20) && b.nOB >= 2) b.xcd_mode = 2;
    const int split = b.xcd_mode == 0 ? b.nOB : b.nTB, other = b.xcd_mode == 0 ? b.nTB : b.nOB;
    const unsigned grid = b.xcd_mode == 2 ? (unsigned)(((b.nTB + 3) / 4) * ((b.nOB + 1) / 2) * 8)
                                          : (unsigned)(((split + 7) / 8) * 8 * other);
    if (a.dump.P)
        hipLaunchKernelGGL((k_contract_output<M, K64, CPG1, WIDE, ATSP, true, NT, NO, KS, D>), dim3(grid),
                           dim3(64 * (M + 2) * KS), 0, s, b);
    else
        hipLaunchKernelGGL((k_contract_output<M, K64, CPG1, WIDE, ATSP, false, NT, NO, KS, D>), dim3(grid),
                           dim3(64 * (M + 2) * KS), 0, s, b);
    return hipGetLastError();
}

// fp64 chunk totals only where a wave reduces more than 8 groups per tap
template <int M, bool K64, bool CPG1, bool ATSP>
hipError_t launch_base(const Args &a, hipStream_t s, bool wide) {
    return wide ? launch_cfg<M, K64, CPG1, true, ATSP, 1, 1, 1, kPrefetchBase>(a, s)
                : launch_cfg<M, K64, CPG1, false, ATSP, 1, 1, 1, kPrefetchBase>(a, s);
}

// the register-tile variants: one K-step per group, paired form of A^T
template <int M, bool K64>
hipError_t launch_fast(const Args &a, hipStream_t s, int variant, bool wide) {
    if (variant == WQ_K2_FUSED_KSPLIT)
        return wide ? launch_cfg<M, K64, true, true, true, 1, 1, 2, kPrefetchBase>(a, s)
                    : launch_cfg<M, K64, true, false, true, 1, 1, 2, kPrefetchBase>(a, s);
    if (variant == WQ_K2_FUSED_32x16)
        return wide ? launch_cfg<M, K64, true, true, true, 2, 1, 1, 3>(a, s)
                    : launch_cfg<M, K64, true, false, true, 2, 1, 1, 3>(a, s);
    return wide ? launch_cfg<M, K64, true, true, true, 2, 2, 1, 2>(a, s)
                : launch_cfg<M, K64, true, false, true, 2, 2, 1, 2>(a, s);
}

template <int M>
hipError_t launch_m(const wq_plan *p, hipStream_t s, const int8_t *Xq, const float *sX,
                    const int8_t *Wq, const float *sW, const float *bias, float *y,
                    const wq_dump &dump) {
    Args a;
    a.xf = p->xf;
    a.Xq = Xq; a.sX = sX; a.Wq = Wq; a.sW = sW; a.bias = bias; a.y = y; a.dump = dump;
    a.H = p->H; a.W = p->W; a.Cin = p->Cin; a.Cout = p->Cout; a.TH = p->TH; a.TW = p->TW;
    a.T = p->T; a.T_pad = p->T_pad; a.Cout_pad = p->Cout_pad;
    a.log2g = 0;
    while ((1 << a.log2g) < p->g) ++a.log2g;
    a.nTB = a.nOB = a.xcd_mode = 0;
    const bool k64 = p->kstep == 64, cpg1 = p->g == p->kstep;
    const int variant = p->k2_variant;   // a fused one, checked for this plan when it was chosen
    const bool wide = p->groups / (variant == WQ_K2_FUSED_KSPLIT ? 2 : 1) > 8;
    if constexpr (M != 2) {
        if (variant != WQ_K2_FUSED_16x16)
            return k64 ? launch_fast<M, true>(a, s, variant, wide) : launch_fast<M, false>(a, s, variant, wide);
    }
    if (!k64)
        return p->sparse_at ? launch_base<M, false, true, true>(a, s, wide)
                            : launch_base<M, false, true, false>(a, s, wide);
    if (cpg1)
        return p->sparse_at ? launch_base<M, true, true, true>(a, s, wide)
                            : launch_base<M, true, true, false>(a, s, wide);
    return p->sparse_at ? launch_base<M, true, false, true>(a, s, wide)
                        : launch_base<M, true, false, false>(a, s, wide);
}

}  // namespace
