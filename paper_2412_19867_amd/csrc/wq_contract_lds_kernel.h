// Stages 2+3 with shared operand tiles for gfx950: the Winograd-domain contraction as int8
// MFMA blocks with per-group dequantization (the Hadamard-product equation of Section
// "Winograd convolution" summed over input channels, with the scales of the second
// quantized-stage equation of Section "Learnable Winograd transform scales"), and the output
// transform y = A^T Y A + bias (output-transform equation) folded in tap by tap.
//
// Every wave of a workgroup works on the SAME tap at the same time.  A workgroup owns a
// (16*TBW tiles) x (16*OBW output channels) block and walks a flat sequence of steps
// (tap-major, then K): per step the OBW weight blocks and TBW activation blocks of one K-step
// - both tensors are stored in the MFMA operand order (include/wq.h), so the copy is linear -
// and the scales of the K-step's group are loaded straight into LDS (buffer loads with the LDS
// destination, no registers in between) into a ring of NS stages that keeps NS-2 steps in
// flight: a step's operands are requested about a microsecond before they are used, which is
// what a trip to memory takes.  Every wave then reads the blocks of its BN x BM sub-tile from
// LDS, so an operand byte is fetched from L2 once per workgroup instead of once per wave.
// The compiler does not order LDS reads after such loads by itself: the loop does it by hand
// (a counted wait on the wave's own loads, then the workgroup barrier).
// A wave issues at most one instruction every four cycles or so, and with the output
// transform's state in registers only two or three waves fit a SIMD, so the loop is written to
// keep the instruction count per step down: the ring is unrolled (every LDS address is an immediate), the
// loader's cursor is branch-free scalar arithmetic, and the int32 dump of the debug entry point is
// a template switch of the same kernel, not a test inside the loop.
// A wave's state per output element is
//     int32 block (fresh per group)  ->  M += float(block) * sW[o] * sX[tile]    (group end)
//     R[b]    += A^T[b][j] * M                                                   (end of tap (i,j))
//     Y[a][b] += A^T[a][i] * R[b]                                                (end of tap row i)
// i.e. 1 + m + m*m floats, never the n*n Winograd-domain values.  A wave dequantizes a step's
// blocks right after their MFMAs; a second set of accumulators that would let the next step's
// MFMAs run under the dequantization costs 16 registers and measured slower than what the extra
// resident workgroup does with them (MFMA and vector-ALU time add up on a SIMD either way).
//
// Three forms:
//   FULL  a workgroup walks all n*n taps and stores y (NHWC, ragged edge masked): one kernel,
//         nothing but y leaves the chip.  Needs (tiles x channels)/(workgroup tile) workgroups
//         to fill the GPU, i.e. many tiles.
//   ROW   a workgroup walks the n taps of ONE tap row i and stores its row sums R_i[b]
//         (m floats per element instead of the n a row of M would take) to the workspace;
//         k_row_finish then forms y = sum_i A^T[a][i] R_i[b] + bias.  n times the workgroups,
//         for layers with few tiles.
//   TAP   a workgroup reduces ONE tap and stores its fp32 Winograd-domain products M
//         [T_pad][n*n][Cout_pad] to the workspace for the separate output-transform kernel:
//         n*n times the workgroups, each short and with no output-transform state in registers
//         (four waves per SIMD), for layers with very few tiles and long reductions.
#pragma once

#include "wq_device.h"
#include "wq_internal.h"

namespace {   // every including file instantiates its own tile size; nothing here is exported

constexpr unsigned kInvalid = kPastEnd;

struct LArgs {
    wq_xf xf;
    const int8_t *Xq;
    const float *sX;
    const int8_t *Wq;
    const float *sW;
    const float *bias;
    float *y;      // FULL: the layer's output
    float *Rbuf;   // ROW: row sums [T_pad][n][m][Cout_pad] in the workspace; TAP: M [T_pad][n*n][Cout_pad]
    wq_dump dump;  // debug calls: where to store the int32 group sums
    int H, W, Cin, Cout, TH, TW, T, T_pad, Cout_pad, log2g;
    // workgroup tiles along channels and tiles, the number of workgroups, the share of each XCD,
    // and which of the two tile indices runs fastest (set by the launcher)
    int nOBt, nTBt, total, per_xcd, tb_fastest;
    // row and tap forms: store the intermediate with plain (write-back) stores instead of writing
    // it through.  Written through, it is in memory before the kernel ends and nothing is left to
    // flush; written back, part of it is still in the caches when the second kernel reads it.
    // Measured inside a sequence of layers: from about 20 MB on the second effect wins (-2 % on a
    // whole step), below it the first (+1-2 %).
    int plain_stores;
};

#define WQ_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

// Buffer loads whose destination is LDS: lane l's 16 (4) bytes land at lds + 16 l (4 l); `lds` and
// `soff` are wave-uniform.  Completion is counted by the wave's vector-memory counter.  (Plain
// device functions on purpose: called from a lambda inside the kernel template, the builtin makes
// the host pass drop the kernel's launch stub without a diagnostic.)
__device__ __forceinline__ void lds_load16(__amdgpu_buffer_rsrc_t r, char *lds, unsigned voff, unsigned soff) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, WQ_LDS_PTR(lds), 16, voff, soff, 0, 0);
}
__device__ __forceinline__ void lds_load4(__amdgpu_buffer_rsrc_t r, char *lds, unsigned voff, unsigned soff) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(r, WQ_LDS_PTR(lds), 4, voff, soff, 0, 0);
}

// s_waitcnt until at most VM of the wave's vector-memory operations are outstanding (gfx9
// encoding: vmcnt in bits 3:0 and 15:14; the LDS/scalar counter is waited to zero as well, the
// export counter left alone), followed by the workgroup barrier.  The "memory" clobber keeps the
// compiler from moving LDS accesses across it.
template <int VM>
__device__ __forceinline__ void wait_loads_and_barrier() {
    static_assert(VM >= 0 && VM < 64, "vmcnt is a 6-bit counter");
    constexpr int imm = 0x0070 | (VM & 0xf) | ((VM >> 4) << 14);
    asm volatile("s_waitcnt %0\n\ts_barrier" ::"n"(imm) : "memory");
}

// NWO x NWT waves (along channels x along tiles), each a BN x BM arrangement of 16x16 blocks;
// NS = stages of the LDS ring.  DUMP: the debug entry point's instance, which also stores the
// int32 group sums.
template <int M, bool K64, bool CPG1, bool WIDE, bool FULL, bool DUMP, int NWO, int NWT, int BN, int BM, int NS, bool TAP = false>
__global__ __launch_bounds__(64 * NWO * NWT, 2) void k_wino_lds(const LArgs a) {
    static_assert(!(FULL && TAP), "one form at a time");
    constexpr int NTAPS = FULL ? (M + 2) * (M + 2) : (TAP ? 1 : M + 2);   // taps a workgroup walks
    constexpr int n = M + 2, NW = NWO * NWT;
    constexpr int KSTEP = K64 ? 64 : 32, KB = KSTEP / 4;
    constexpr int BLK = 16 * KSTEP;                    // bytes of one K-step of a 16-row block
    constexpr int OBW = NWO * BN, TBW = NWT * BM;      // 16-row blocks per workgroup: channels, tiles
    constexpr int NB = OBW + TBW;                      // blocks per stage: weights first
    constexpr int CPB = BLK / 16, CHUNKS = NB * CPB;   // 16-byte chunks per block / per stage
    constexpr int NWL = (CHUNKS + 63) / 64;            // wave-wide 1 KiB loads per stage
    constexpr int LW = (NWL + NW - 1) / NW;            // of which each wave issues this many
    constexpr int OPB = LW * NW * 1024;                // operand bytes per stage (rounded up to that)
    constexpr int NSW = OBW * 16, NSX = TBW * 16;      // scales per stage
    constexpr int NLW = (NSW + 63) / 64, NLX = (NSX + 63) / 64;   // wave-wide scale loads per stage
    // a stage: operands, the weight scales, the activation scales (64 words per wave-wide load),
    // 64 words nobody reads (the scale load of the waves that have none to fetch)
    constexpr int STAGE = OPB + (NLW + NLX + 1) * 256;
    constexpr int D = NS - 2;                          // steps in flight
    constexpr int LPS = LW + 1;                        // loads per wave and step
    static_assert(NS >= 4 && NS % 2 == 0, "ring size (the operand register sets alternate with the step's parity)");
    static_assert(NLW + NLX <= NW, "one scale load per wave and step: the first waves fetch the weight scales, the next the activation scales");
    static_assert(K64 || OBW % 2 == 0, "a wave's 64 chunks must not straddle weights and activations");
    static_assert(D * LPS < 64, "the wait counts loads");
    __shared__ __attribute__((aligned(16))) char ring[NS * STAGE];

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, q = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), wo = w % NWO, wt = w / NWO;
    // Workgroup ids go round-robin over the 8 XCDs, whose L2s are private: XCD x takes the
    // logical workgroups [x * per_xcd, (x + 1) * per_xcd) in order, so that the workgroups
    // resident on one XCD at a time are neighbours and share operand tiles in that L2.
    const int logical = (int)(blockIdx.x & 7u) * a.per_xcd + (int)(blockIdx.x >> 3);
    if (logical >= a.total) return;   // the whole workgroup leaves, before any barrier
    int row_i = 0, rem = logical;
    if constexpr (!FULL) {   // row_i: the tap row (ROW) or the tap (TAP) of this workgroup
        const int per_row = a.nOBt * a.nTBt;
        row_i = logical / per_row;
        rem = logical - row_i * per_row;
    }
    const int obi = a.tb_fastest ? rem / a.nTBt : rem % a.nOBt;
    const int tbi = a.tb_fastest ? rem % a.nTBt : rem / a.nOBt;
    const int ob0 = obi * OBW, tb0 = tbi * TBW;   // in 16-row blocks
    const int Cin = a.Cin, T_pad = a.T_pad, Cout_pad = a.Cout_pad;
    const int groups = Cin >> a.log2g, cps = Cin / KSTEP;
    const int cpg_mask = ((1 << a.log2g) / KSTEP) - 1;
    constexpr unsigned n2 = n * n;

    const __amdgpu_buffer_rsrc_t rW = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.Wq), 0, (int)(n2 * (unsigned)Cout_pad * (unsigned)Cin), kBufFlags);
    const __amdgpu_buffer_rsrc_t rX = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.Xq), 0, (int)(n2 * (unsigned)T_pad * (unsigned)Cin), kBufFlags);
    const __amdgpu_buffer_rsrc_t rSW = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(a.sW), 0, (int)(n2 * (unsigned)groups * (unsigned)Cout_pad * 4u), kBufFlags);
    const __amdgpu_buffer_rsrc_t rSX = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(a.sX), 0, (int)(n2 * (unsigned)T_pad * (unsigned)groups * 4u), kBufFlags);

    // ---- the loader ----
    // Wave-load k = w + u * NW of a stage covers its 16-byte chunks [64 k, 64 k + 64), all weights
    // or all activations, and lands at byte 1024 k of the stage.  Per load the wave keeps one
    // scalar cursor (the byte offset of the current (tap, K-step) inside its tensor) that advances
    // by a K-step, jumps to the next tap's plane at the end of a tap, and stops at the last step
    // (which the tail of the ring fetches again, into stages nobody reads any more).
    const unsigned planeW = (unsigned)Cout_pad * Cin, planeX = (unsigned)T_pad * Cin;
    const unsigned planeSX = (unsigned)T_pad * groups * 4;
    const unsigned stepSW = (unsigned)Cout_pad * 4;   // a tap's weight scales are groups * stepSW bytes: taps are contiguous
    const unsigned t_first = FULL ? 0u : (unsigned)(TAP ? row_i : row_i * n), t_last = t_first + NTAPS - 1;
    const int NSTEPS = NTAPS * cps;
    unsigned vop[LW], oOp[LW], jumpOp[LW], lastOp[LW];
    bool is_w[LW];
#pragma unroll
    for (int u = 0; u < LW; ++u) {
        const int c = (w + u * NW) * 64 + lane, blk = c / CPB, off = (c % CPB) * 16;
        is_w[u] = ((w + u * NW) * 64) / CPB < OBW;   // wave-uniform
        const int row = blk < OBW ? ob0 + blk : tb0 + blk - OBW;
        const bool ok = c < CHUNKS && row * 16 < (blk < OBW ? Cout_pad : T_pad);
        vop[u] = ok ? (unsigned)(row * 16 * Cin + off) : kInvalid;
        const unsigned plane = is_w[u] ? planeW : planeX;
        oOp[u] = t_first * plane;
        jumpOp[u] = plane - (unsigned)cps * BLK;
        lastOp[u] = t_last * plane + (unsigned)(cps - 1) * BLK;
    }
    // the scales of a group, one per lane: waves [0, NLW) fetch 64 weight scales each, waves
    // [NLW, NLW + NLX) 64 activation scales each (4 tile blocks of 16); the other waves issue the
    // same load past the end of the buffer (every wave has the same number of loads in flight per
    // step, which the counted wait relies on)
    const bool is_sw = w < NLW, is_sx = !is_sw && w < NLW + NLX;
    unsigned vsc = kInvalid;
    if (is_sw && 64 * w + lane < NSW && ob0 * 16 + 64 * w + lane < Cout_pad)
        vsc = (unsigned)(ob0 * 16 + 64 * w + lane) * 4u;
    if (is_sx && 64 * (w - NLW) + lane < NSX && (tb0 + 4 * (w - NLW) + (lane >> 4)) * 16 < T_pad)
        vsc = (unsigned)((tb0 + 4 * (w - NLW) + (lane >> 4)) * groups * 64 + (lane & 15) * 4);
    const int sc_slot = OPB + 256 * min(w, NLW + NLX);
    const __amdgpu_buffer_rsrc_t rSc = is_sw ? rSW : rSX;
    const unsigned stepSc = is_sw ? stepSW : 64u;                                  // per group
    const unsigned jumpSc = is_sw ? 0u : planeSX - (unsigned)groups * 64u;         // per tap
    unsigned oSc = is_sw ? t_first * (unsigned)groups * stepSW : t_first * planeSX;
    const unsigned lastSc = oSc + (is_sw ? (unsigned)NTAPS * groups * stepSW - stepSW
                                         : (unsigned)(NTAPS - 1) * planeSX + (unsigned)(groups - 1) * 64u);
    int k_ld = 0;

    auto issue = [&](int stage) {   // request the cursor's step into ring stage `stage` (a constant after unrolling)
        char *base = ring + stage * STAGE;
#pragma unroll
        for (int u = 0; u < LW; ++u)
            lds_load16(is_w[u] ? rW : rX, base + (w + u * NW) * 1024, vop[u], oOp[u]);
        lds_load4(rSc, base + sc_slot, vsc, oSc);
        // branch-free scalar bookkeeping
        ++k_ld;
        const bool wrap = k_ld == cps;
        k_ld = wrap ? 0 : k_ld;
#pragma unroll
        for (int u = 0; u < LW; ++u) oOp[u] = min(oOp[u] + BLK + (wrap ? jumpOp[u] : 0u), lastOp[u]);
        const bool next_group = CPG1 || (k_ld & cpg_mask) == 0;
        oSc = min(oSc + (next_group ? stepSc : 0u) + (wrap ? jumpSc : 0u), lastSc);
    };

    // ---- per-element state ----
    v4i acc[BN][BM];
    float4 Mc[BN][BM];
    double Mt[BN][BM][4];
    float4 R[TAP ? 1 : M][BN][BM];
    float4 Y[FULL ? M : 1][FULL ? M : 1][BN][BM];
#pragma unroll
    for (int no = 0; no < BN; ++no)
#pragma unroll
        for (int nt = 0; nt < BM; ++nt) {
            acc[no][nt] = v4i{0, 0, 0, 0};
            Mc[no][nt] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int r = 0; r < 4; ++r) Mt[no][nt][r] = 0.0;
#pragma unroll
            for (int b = 0; b < (TAP ? 1 : M); ++b) R[b][no][nt] = make_float4(0.f, 0.f, 0.f, 0.f);
            if constexpr (FULL) {
#pragma unroll
                for (int aa = 0; aa < M; ++aa)
#pragma unroll
                    for (int b = 0; b < M; ++b) Y[aa][b][no][nt] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    // The compute cursor (uniform).
    int g_left = groups, in_chunk = 0;        // groups left in the tap; groups in the fp32 chunk
    int i_cp = FULL ? 0 : (TAP ? row_i / n : row_i), j_cp = TAP ? row_i % n : 0;    // the tap being reduced
    int gam_cp = 0;                           // its group (the dump's index)
    float atc[M], atr[M];   // column j_cp of A^T (for R), column i_cp of A^T (for Y)
#pragma unroll
    for (int b = 0; b < M; ++b) {
        atc[b] = a.xf.AT[b * n];
        atr[b] = a.xf.AT[b * n + i_cp];
    }

    // A finished group: dequantize its int32 blocks into M; at the end of a tap fold M into R,
    // at the end of a tap row fold R into Y.
    auto finish_group = [&](v4i (&ac)[BN][BM], const v4f (&sw)[BN], const float (&sx)[BM]) {
#pragma unroll
        for (int no = 0; no < BN; ++no)
#pragma unroll
            for (int nt = 0; nt < BM; ++nt) {
                Mc[no][nt].x = __builtin_fmaf((float)ac[no][nt][0], sw[no].x * sx[nt], Mc[no][nt].x);
                Mc[no][nt].y = __builtin_fmaf((float)ac[no][nt][1], sw[no].y * sx[nt], Mc[no][nt].y);
                Mc[no][nt].z = __builtin_fmaf((float)ac[no][nt][2], sw[no].z * sx[nt], Mc[no][nt].z);
                Mc[no][nt].w = __builtin_fmaf((float)ac[no][nt][3], sw[no].w * sx[nt], Mc[no][nt].w);
                if constexpr (DUMP) {
                    const int v[4] = {ac[no][nt][0], ac[no][nt][1], ac[no][nt][2], ac[no][nt][3]};
                    wq_dump_store(a.dump, i_cp * n + j_cp, (tb0 + BM * wt + nt) * 16 + l16, gam_cp, groups,
                                      (ob0 + BN * wo + no) * 16 + 4 * q, a.Cout, a.T, v);
                }
            }
        if constexpr (DUMP) ++gam_cp;
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
        if (!TAP && --g_left == 0) {   // end of tap (i_cp, j_cp); the tap form keeps M for its epilogue
            g_left = groups;
            in_chunk = 0;
            if constexpr (DUMP) gam_cp = 0;
#pragma unroll
            for (int no = 0; no < BN; ++no)
#pragma unroll
                for (int nt = 0; nt < BM; ++nt) {
                    float4 Mv = Mc[no][nt];
                    if constexpr (WIDE) {
                        Mv = make_float4((float)(Mt[no][nt][0] + (double)Mv.x), (float)(Mt[no][nt][1] + (double)Mv.y),
                                         (float)(Mt[no][nt][2] + (double)Mv.z), (float)(Mt[no][nt][3] + (double)Mv.w));
#pragma unroll
                        for (int r = 0; r < 4; ++r) Mt[no][nt][r] = 0.0;
                    }
                    Mc[no][nt] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                    for (int b = 0; b < M; ++b) {   // branch-free: zero entries of A^T add nothing
                        float4 &Rb = R[b][no][nt];
                        Rb.x = __builtin_fmaf(atc[b], Mv.x, Rb.x);
                        Rb.y = __builtin_fmaf(atc[b], Mv.y, Rb.y);
                        Rb.z = __builtin_fmaf(atc[b], Mv.z, Rb.z);
                        Rb.w = __builtin_fmaf(atc[b], Mv.w, Rb.w);
                    }
                }
            if (++j_cp == n) {   // end of tap row i_cp
                j_cp = 0;
                if constexpr (FULL) {
#pragma unroll
                    for (int no = 0; no < BN; ++no)
#pragma unroll
                        for (int nt = 0; nt < BM; ++nt)
#pragma unroll
                            for (int b = 0; b < M; ++b) {
                                const float4 Rb = R[b][no][nt];
                                R[b][no][nt] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                                for (int aa = 0; aa < M; ++aa) {
                                    float4 &Yv = Y[aa][b][no][nt];
                                    Yv.x = __builtin_fmaf(atr[aa], Rb.x, Yv.x);
                                    Yv.y = __builtin_fmaf(atr[aa], Rb.y, Yv.y);
                                    Yv.z = __builtin_fmaf(atr[aa], Rb.z, Yv.z);
                                    Yv.w = __builtin_fmaf(atr[aa], Rb.w, Yv.w);
                                }
                            }
                    ++i_cp;
                    const int in = i_cp < n ? i_cp : 0;
#pragma unroll
                    for (int aa = 0; aa < M; ++aa) atr[aa] = a.xf.AT[aa * n + in];
                }
            }
#pragma unroll
            for (int b = 0; b < M; ++b) atc[b] = a.xf.AT[b * n + j_cp];
        }
    };

    // operands and scales of this wave's blocks out of ring stage `stage` (a constant after unrolling)
    auto read_operands = [&](int stage, v4i (&av)[BN], v4i (&bv)[BM]) {
        const char *base = ring + stage * STAGE + lane * KB;
#pragma unroll
        for (int e = 0; e < BN; ++e) {
            const char *pa = base + (BN * wo + e) * BLK;
            if constexpr (K64) {
                av[e] = *reinterpret_cast<const v4i *>(pa);
            } else {
                const v2i t = *reinterpret_cast<const v2i *>(pa);
                av[e] = v4i{t.x, t.y, 0, 0};
            }
        }
#pragma unroll
        for (int e = 0; e < BM; ++e) {
            const char *pb = base + (OBW + BM * wt + e) * BLK;
            if constexpr (K64) {
                bv[e] = *reinterpret_cast<const v4i *>(pb);
            } else {
                const v2i t = *reinterpret_cast<const v2i *>(pb);
                bv[e] = v4i{t.x, t.y, 0, 0};
            }
        }
    };
    auto read_scales = [&](int stage, v4f (&sw)[BN], float (&sx)[BM]) {
        const float *sc = reinterpret_cast<const float *>(ring + stage * STAGE + OPB);
#pragma unroll
        for (int e = 0; e < BN; ++e) sw[e] = *reinterpret_cast<const v4f *>(&sc[(BN * wo + e) * 16 + 4 * q]);
#pragma unroll
        for (int e = 0; e < BM; ++e) sx[e] = sc[64 * NLW + (BM * wt + e) * 16 + l16];
    };
    auto mfma_blocks = [&](v4i (&ac)[BN][BM], const v4i (&av)[BN], const v4i (&bv)[BM], bool fresh) {
#pragma unroll
        for (int no = 0; no < BN; ++no)
#pragma unroll
            for (int nt = 0; nt < BM; ++nt) {
                const v4i c0 = fresh ? v4i{0, 0, 0, 0} : ac[no][nt];
                if constexpr (K64) {
                    ac[no][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av[no], bv[nt], c0, 0, 0, 0);
                } else {
                    const long x = __builtin_bit_cast(long, v2i{av[no].x, av[no].y});
                    const long y = __builtin_bit_cast(long, v2i{bv[nt].x, bv[nt].y});
                    ac[no][nt] = __builtin_amdgcn_mfma_i32_16x16x32_i8(x, y, c0, 0, 0, 0);
                }
            }
    };

    // ---- the step loop ----
    // Step s: request step s + D into stage (s + D) % NS = (s - 2) % NS, which every wave
    // finished reading before it arrived at the barrier of step s - 1; wait until this wave's
    // loads of step s + 1 have landed (all but the D - 1 newer steps' loads); barrier:
    // everybody's have.  The operands (and, with one K-step per group, the scales) of step s + 1
    // are then read into the other register set while the MFMAs and the dequantization of step s run.
#pragma unroll
    for (int d = 0; d < D; ++d) issue(d);
    v4f swS[2][BN] = {};
    float sxS[2][BM] = {};
    v4i avS[2][BN], bvS[2][BM];
    wait_loads_and_barrier<DUMP ? 0 : (D - 1) * LPS>();   // (the dump's stores are counted too: wait for all)
    read_operands(0, avS[0], bvS[0]);
    if constexpr (CPG1) read_scales(0, swS[0], sxS[0]);
    for (int sb = 0; sb < NSTEPS; sb += NS) {
#pragma unroll
        for (int v = 0; v < NS; ++v) {
            if (sb + v >= NSTEPS) break;   // NSTEPS is even but need not be a multiple of NS
            const int u = v & 1;
            issue((v + D) % NS);
            wait_loads_and_barrier<DUMP ? 0 : (D - 1) * LPS>();
            read_operands((v + 1) % NS, avS[u ^ 1], bvS[u ^ 1]);   // past the last step: read, never used
            if constexpr (CPG1) {
                mfma_blocks(acc, avS[u], bvS[u], true);
                read_scales((v + 1) % NS, swS[u ^ 1], sxS[u ^ 1]);
                finish_group(acc, swS[u], sxS[u]);
            } else {
                // several K-steps per group: the MFMAs accumulate; the sums are cleared when the
                // group is done (a select on every step would cost one instruction per register)
                const bool last = ((sb + v + 1) & cpg_mask) == 0;
                mfma_blocks(acc, avS[u], bvS[u], false);
                if (last) {
                    read_scales(v, swS[0], sxS[0]);
                    finish_group(acc, swS[0], sxS[0]);
#pragma unroll
                    for (int no = 0; no < BN; ++no)
#pragma unroll
                        for (int nt = 0; nt < BM; ++nt) acc[no][nt] = v4i{0, 0, 0, 0};
                }
            }
        }
    }

    // ---- epilogue ----
    if constexpr (FULL) {
#pragma unroll
        for (int nt = 0; nt < BM; ++nt) {
            const int tau = (tb0 + BM * wt + nt) * 16 + l16;
            if (tau >= a.T) continue;
            const int tw = tau % a.TW, th = (tau / a.TW) % a.TH, bb = tau / (a.TW * a.TH);
            const int hv = min(M, a.H - th * M), wv = min(M, a.W - tw * M);
            float *base = a.y + ((size_t)(bb * a.H + th * M) * a.W + tw * M) * a.Cout;
#pragma unroll
            for (int no = 0; no < BN; ++no) {
                const int o = (ob0 + BN * wo + no) * 16 + 4 * q;
                if (o >= a.Cout) continue;
                const float4 bv4 = *reinterpret_cast<const float4 *>(a.bias + o);   // padded to Cout_pad
                const bool vec = (a.Cout & 3) == 0;   // then o + 3 < Cout and the address is 16-byte aligned
#pragma unroll
                for (int aa = 0; aa < M; ++aa)
#pragma unroll
                    for (int b = 0; b < M; ++b) {
                        if (aa >= hv || b >= wv) continue;
                        const float4 Yv = Y[aa][b][no][nt];
                        float *dst = base + ((size_t)aa * a.W + b) * a.Cout + o;
                        const v4f out = {Yv.x + bv4.x, Yv.y + bv4.y, Yv.z + bv4.z, Yv.w + bv4.w};
                        if (vec) {
                            // a plain store: this form runs on layers with many tiles, whose output the
                            // next layer's input kernel finds in the caches (measured on a chained
                            // stack: -0.9 % of the whole step against the streaming store)
                            *reinterpret_cast<v4f *>(dst) = out;
                        } else {
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                if (o + r < a.Cout) store_y(out[r], dst + r);
                        }
                    }
            }
        }
    } else if constexpr (TAP) {
        const __amdgpu_buffer_rsrc_t rM = __builtin_amdgcn_make_buffer_rsrc(
            a.Rbuf, 0, (int)(n2 * (unsigned)T_pad * (unsigned)Cout_pad * 4u), kBufFlags);
#pragma unroll
        for (int nt = 0; nt < BM; ++nt) {
            const int tau = (tb0 + BM * wt + nt) * 16 + l16;
#pragma unroll
            for (int no = 0; no < BN; ++no) {
                const int o = (ob0 + BN * wo + no) * 16 + 4 * q;
                if (tau >= T_pad || o >= Cout_pad) continue;
                float4 Mv = Mc[no][nt];
                if constexpr (WIDE)
                    Mv = make_float4((float)(Mt[no][nt][0] + (double)Mv.x), (float)(Mt[no][nt][1] + (double)Mv.y),
                                     (float)(Mt[no][nt][2] + (double)Mv.z), (float)(Mt[no][nt][3] + (double)Mv.w));
                const unsigned off = (((unsigned)tau * n2 + (unsigned)row_i) * (unsigned)Cout_pad + (unsigned)o) * 4u;
                const v4i bits = __builtin_bit_cast(v4i, v4f{Mv.x, Mv.y, Mv.z, Mv.w});
                if (a.plain_stores) __builtin_amdgcn_raw_buffer_store_b128(bits, rM, off, 0, 0);
                else __builtin_amdgcn_raw_buffer_store_b128(bits, rM, off, 0, kWriteThrough);
            }
        }
    } else {
        const __amdgpu_buffer_rsrc_t rR = __builtin_amdgcn_make_buffer_rsrc(
            a.Rbuf, 0, (int)((unsigned)T_pad * (unsigned)(n * M) * (unsigned)Cout_pad * 4u), kBufFlags);
#pragma unroll
        for (int nt = 0; nt < BM; ++nt) {
            const int tau = (tb0 + BM * wt + nt) * 16 + l16;
#pragma unroll
            for (int no = 0; no < BN; ++no) {
                const int o = (ob0 + BN * wo + no) * 16 + 4 * q;
                if (tau >= T_pad || o >= Cout_pad) continue;
#pragma unroll
                for (int b = 0; b < M; ++b) {
                    const float4 Rb = R[b][no][nt];
                    const unsigned off =
                        ((((unsigned)tau * n + (unsigned)row_i) * M + (unsigned)b) * (unsigned)Cout_pad + (unsigned)o) * 4u;
                    const v4i bits = __builtin_bit_cast(v4i, v4f{Rb.x, Rb.y, Rb.z, Rb.w});
                    if (a.plain_stores) __builtin_amdgcn_raw_buffer_store_b128(bits, rR, off, 0, 0);
                    else __builtin_amdgcn_raw_buffer_store_b128(bits, rR, off, 0, kWriteThrough);
                }
            }
        }
    }
}

template <int M, bool K64, bool CPG1, bool WIDE, bool FULL, bool DUMP, int NWO, int NWT, int BN, int BM, int NS, bool TAP = false>
void launch_tile(const LArgs &a0, hipStream_t s) {
    LArgs a = a0;
    constexpr int n = M + 2;
    a.nOBt = (a.Cout_pad + 16 * NWO * BN - 1) / (16 * NWO * BN);
    a.nTBt = (a.T_pad + 16 * NWT * BM - 1) / (16 * NWT * BM);
    a.total = a.nOBt * a.nTBt * (FULL ? 1 : (TAP ? n * n : n));
    a.per_xcd = (a.total + 7) / 8;
    // neighbours in launch order share the larger operand's tiles: with more weight bytes than
    // activation bytes the tile index runs fastest (the same weight tile for consecutive workgroups)
    a.tb_fastest = (long)a.Cout_pad > (long)a.T_pad ? 1 : 0;
    hipLaunchKernelGGL((k_wino_lds<M, K64, CPG1, WIDE, FULL, DUMP, NWO, NWT, BN, BM, NS, TAP>), dim3((unsigned)a.per_xcd * 8u),
                       dim3(64 * NWO * NWT), 0, s, a);
}

template <int M, bool K64, bool CPG1, bool WIDE, bool DUMP>
void launch_variant(const LArgs &a, hipStream_t s, int variant) {
    // wave tiles: the per-element state of the full form (1 + m + m*m floats) allows 8 elements
    // per lane for F(4,3) and 4 for F(6,3); the row form (1 + m floats) allows 16
    constexpr int FBM = M == 6 ? 1 : 2;
    switch (variant) {
        case WQ_K2_LDS_FULL_64x64:   // tiles x channels: 16*NWT*BM x 16*NWO*BN
            // (not offered for F(6,3): 16 waves of 4 elements per lane would need 128 registers each)
            if constexpr (M != 6) {
                launch_tile<M, K64, CPG1, WIDE, true, DUMP, 4, 2, 1, 2, 8>(a, s);
                break;
            }
            [[fallthrough]];
        case WQ_K2_LDS_FULL_32x64:
            launch_tile<M, K64, CPG1, WIDE, true, DUMP, 4, 2 / FBM, 1, FBM, 8>(a, s);
            break;
        case WQ_K2_LDS_FULL_32x32:   // one block per wave: four workgroups per CU, their waves interleave on a SIMD
            launch_tile<M, K64, CPG1, WIDE, true, DUMP, 2, 2, 1, 1, 8>(a, s);
            break;
        case WQ_K2_LDS_ROW_64x64:
            launch_tile<M, K64, CPG1, WIDE, false, DUMP, 2, 2, 2, 2, 6>(a, s);   // 3 workgroups' rings per CU
            break;
        case WQ_K2_LDS_TAP_64x64:   // 4 stages: four workgroups' rings per CU
            launch_tile<M, K64, CPG1, WIDE, false, DUMP, 2, 2, 2, 2, 4, true>(a, s);
            break;
        case WQ_K2_LDS_TAP_128x128:   // 64x64 per wave: 16 MFMAs per 8 operand blocks read from LDS
            if constexpr (!WIDE) {    // (with fp64 chunk totals 16 blocks per wave do not fit the registers)
                launch_tile<M, K64, CPG1, WIDE, false, DUMP, 2, 2, 4, 4, 4, true>(a, s);
                break;
            }
            launch_tile<M, K64, CPG1, WIDE, false, DUMP, 2, 2, 2, 2, 4, true>(a, s);
            break;
        default:   // WQ_K2_LDS_ROW_32x64
            launch_tile<M, K64, CPG1, WIDE, false, DUMP, 4, 1, 1, 2, 8>(a, s);
            break;
    }
}

// The contraction kernel of an LDS variant for tile size M; DUMP = the debug entry point's instance.
template <int M, bool DUMP>
hipError_t launch_lds_m(const wq_plan *p, hipStream_t s, const LArgs &a) {
    const bool k64 = p->kstep == 64, cpg1 = p->g == p->kstep;
    const bool wide = p->groups > 16;   // fp64 chunk totals where a tap reduces more than 16 groups
    const int v = p->k2_variant;
    if (!k64) {
        if (wide) launch_variant<M, false, true, true, DUMP>(a, s, v);
        else launch_variant<M, false, true, false, DUMP>(a, s, v);
    } else if (cpg1) {
        if (wide) launch_variant<M, true, true, true, DUMP>(a, s, v);
        else launch_variant<M, true, true, false, DUMP>(a, s, v);
    } else {
        if (wide) launch_variant<M, true, false, true, DUMP>(a, s, v);
        else launch_variant<M, true, false, false, DUMP>(a, s, v);
    }
    return hipGetLastError();
}

}  // namespace
