/*
 * wq - group-wise int8 quantized Winograd F(m,3) convolution for AMD MI355X (gfx950).
 *
 * C ABI of the library built from paper_2412_19867_amd/csrc.  The operation is
 * the 3x3, stride-1, zero-pad-1 cross-correlation of an NHWC fp32 activation
 * with OIHW fp32 weights, evaluated as the Winograd pipeline of the paper's
 * Section "Winograd convolution" (W = G w G^T, X = B^T x B, Y = W . X summed
 * over input channels, y = A^T Y A) with the Winograd-domain operands
 * quantized group-wise to int8 as in the second quantized-stage equation of
 * Section "Learnable Winograd transform scales" (Y ~ s_qW s_qX Q(W/s_qW)
 * Q(X/s_qX)), the quantizer being the uniform symmetric one of Section
 * "Related work" with dynamic abs-max scales for activations.
 *
 * Conventions
 *   - n = m+2; taps t = i*n+j (i,j < n); tile grid TH = ceil(H/m), TW = ceil(W/m),
 *     T = N*TH*TW, tile id (b*TH+th)*TW+tw; groups of `group_size` consecutive
 *     input channels, groups = Cin/group_size.
 *   - Every device buffer is owned by the caller.  The library allocates no
 *     device memory, never synchronises, and enqueues all work on the
 *     hipStream_t passed as `stream` (NULL = the default stream).
 *   - `*_dev` pointers are device pointers; everything else is host memory.
 *   - All functions return a wq_status_t; no exceptions.  The library keeps no
 *     state outside the objects it hands out and reads no environment
 *     variable (the one exception, wq_conv_forward_static, says so).  Distinct
 *     plans may be used from distinct threads.  Every argument check happens
 *     on the host before any kernel is launched.
 *   - Inputs containing NaN/Inf give unspecified outputs.
 */
#ifndef WQ_H
#define WQ_H

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#pragma GCC visibility push(default)   /* the library itself is built with hidden visibility */
#endif
#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    WQ_OK = 0,
    WQ_ERR_INVALID_ARG = 1,   /* NULL pointer, non-positive size, Cin % group_size != 0 */
    WQ_ERR_UNSUPPORTED = 2,   /* m not in {2,4,6}; group_size not in {32,64,128,256,512};
                                 a tensor of 2 GiB or more (input: more than 1 GiB); a tuning
                                 choice that does not apply to the plan's shape */
    WQ_ERR_BAD_TRANSFORM = 3, /* matrices non-finite or not a valid F(m,3) triple */
    WQ_ERR_NOT_PREPARED = 4,  /* forward called on a plan that never prepared weights (tracked per
                                 plan, not per blob: passing a blob that no wq_weight_prepare call
                                 of an identical plan has filled is the caller's error and is not
                                 detected) */
    WQ_ERR_WORKSPACE = 5,     /* a caller buffer is smaller than wq_plan_layout reports */
    WQ_ERR_DEVICE = 6         /* a kernel launch failed */
} wq_status_t;

typedef struct wq_plan wq_plan_t; /* opaque host object */

/* Sizes and offsets (bytes) of the library's device-side formats, so that a
 * caller can allocate the buffers and a test can read the intermediate tensors.
 *   weight blob : Wq int8, blocked            at blob_Wq_off
 *                 sW fp32 [n*n][groups][Cout_pad]  at blob_sW_off
 *                 bias fp32 [Cout_pad]             at blob_bias_off
 *   workspace   : Xq int8, blocked            at ws_Xq_off
 *                 sX fp32 [n*n][T_pad/16][groups][16]  at ws_sX_off  (last index = tile % 16)
 *                 M  fp32 [T_pad][n*n][Cout_pad]       at ws_M_off   (scratch of the two-kernel path)
 *   debug dump  : P int32 [n*n][T][groups][Cout]   (dense, no padding)
 * Blocked int8 layout (R = T_pad for Xq, Cout_pad for Wq; the MFMA operand order):
 *   [n*n][R/16][Cin/kstep][4][16][kstep/4]
 *   element (tap, row, c) sits at block (tap, row/16, c/kstep), then
 *   q = (c % kstep) / (kstep/4), then row % 16, then c % (kstep/4);
 *   kstep = 32 for group_size 32, else 64.
 * Rows T..T_pad-1 and Cout..Cout_pad-1 hold zeros. */
typedef struct {
    int32_t N, H, W, Cin, Cout, m, n, group_size, groups;
    int32_t TH, TW, T, T_pad, Cout_pad, kstep;
    int32_t k2_kernels; /* launches of wq_contract_output: 1 = fused kernel, 2 = GEMM + output transform */
    int32_t k2_variant; /* which kernel instance stages 2+3 run, a wq_k2_variant_t (see wq_plan_tune) */
    int32_t k1_rows;    /* tap rows per workgroup of the input kernel: n, n/2, 2 or 1 */
    uint64_t blob_bytes, blob_Wq_off, blob_sW_off, blob_bias_off;
    uint64_t ws_bytes, ws_Xq_off, ws_sX_off, ws_M_off;
    uint64_t debug_P_bytes;
} wq_layout_t;

/* The paper's standard F(m,3) matrices (supplementary Section "Standard
 * Winograd transforms" for m = 4, 6; the same construction with points
 * 0, 1, -1, infinity for m = 2), row-major fp64, host memory:
 * BT n*n, G n*3, AT m*n.  Any output pointer may be NULL. */
wq_status_t wq_standard_transforms(int m, double *BT, double *G, double *AT);

/* The scale-parametrised transforms of Section "Learnable Winograd transform
 * scales" (W = S_G V_G w V_G^T S_G, X = S_B V_B x V_B^T S_B, y = V_A S_A Y S_A V_A^T
 * with S_A S_B S_G = I): row i of the standard B^T times u_B[i], row i of the
 * standard G times u_G[i], column i of the standard A^T divided by
 * u_B[i]*u_G[i].  u_B, u_G: n finite non-zero host doubles each (else
 * INVALID_ARG).  Outputs are host, row-major fp32 (BT n*n, G n*3, AT m*n),
 * formed in fp64 and rounded once; any output pointer may be NULL.  The result
 * is what wq_plan_create expects. */
wq_status_t wq_scaled_transforms(int m, const double *u_B, const double *u_G,
                                 float *BT, float *G, float *AT);

/* Create a plan for one layer shape.  BT (n*n), G (n*3), AT (m*n) are host,
 * row-major fp32: the transform matrices WITH any learned diagonal scales
 * already applied (Section "Learnable Winograd transform scales": rows of B^T
 * and G scaled, columns of A^T scaled by the inverse product).  Pass all three
 * NULL for the standard matrices.  The matrices are copied.  They must satisfy
 * sum_i AT[a][i] G[i][k] BT[i][l] = [l == a+k] to 1e-4 relative.
 * On error *out is set to NULL. */
wq_status_t wq_plan_create(wq_plan_t **out, int N, int H, int W, int Cin, int Cout,
                           int m, int group_size,
                           const float *BT, const float *G, const float *AT);

wq_status_t wq_plan_destroy(wq_plan_t *plan);

wq_status_t wq_plan_layout(const wq_plan_t *plan, wq_layout_t *out);

/* Which kernel instance runs stages 2+3 (wq_layout_t::k2_variant).  The plan
 * picks one from the layer shape; wq_plan_tune overrides the pick.
 *   FUSED_*   one kernel, a wave per tap row, operands straight from L2 into
 *             registers, output transform behind the contraction
 *             (16x16 / 16x16 with K split over two waves / 32x16 / 32x32 register tiles);
 *   GEMM_*    a tiled GEMM per tap that writes the fp32 Winograd-domain products to
 *             the workspace (tiles x channels per workgroup), then an output-transform kernel;
 *   LDS_FULL_* one kernel, every wave of a workgroup on the same tap, operand tiles staged
 *             once per K-step in LDS and shared, the output transform accumulated tap row
 *             by tap row in registers (tiles x channels per workgroup; 32x32 = one 16x16
 *             block per wave and four workgroups per CU, for many tiles and short reductions);
 *   LDS_ROW_*  one workgroup per (tile block, channel block, tap row): the same staged
 *             contraction over the n taps of a row folded into row sums of Y A, which go
 *             to the workspace; a small second kernel applies A^T and the bias;
 *   LDS_TAP_*  one workgroup per (tile block, channel block, tap): the staged contraction of
 *             one tap, its fp32 products M written to the workspace like GEMM_* does, then the
 *             same output-transform kernel (128x128: 64x64 per wave, reductions of at most 16
 *             groups). */
typedef enum {
    WQ_K2_AUTO = -1,
    WQ_K2_FUSED_16x16 = 0,
    WQ_K2_FUSED_KSPLIT = 1,
    WQ_K2_FUSED_32x16 = 2,
    WQ_K2_FUSED_32x32 = 3,
    WQ_K2_GEMM_64x64 = 10,
    WQ_K2_GEMM_32x128 = 11,
    WQ_K2_GEMM_128x128 = 12,
    WQ_K2_LDS_FULL_64x64 = 20,
    WQ_K2_LDS_FULL_32x64 = 21,
    WQ_K2_LDS_FULL_32x32 = 22,
    WQ_K2_LDS_ROW_64x64 = 30,
    WQ_K2_LDS_ROW_32x64 = 31,
    WQ_K2_LDS_TAP_64x64 = 40,
    WQ_K2_LDS_TAP_128x128 = 41
} wq_k2_variant_t;

/* Tuning overrides (tests and sweeps; results stay within the documented
 * bounds: int8 codes, scales and int32 sums do not depend on them, the fp32
 * output only through its summation order).  Buffer sizes do not change.
 *   k1_rows    tap rows per workgroup of the input kernel: 0 = the plan's
 *              own choice, else one of 1, 2, n/2, n;
 *   k2_variant WQ_K2_AUTO = the plan's own choice, else a wq_k2_variant_t.
 * A value that is not listed -> INVALID_ARG; one that does not apply to this
 * plan's shape, group size or matrices -> UNSUPPORTED (the plan is unchanged). */
wq_status_t wq_plan_tune(wq_plan_t *plan, int k1_rows, int k2_variant);

/* Fully-integer input and output transforms (first and third quantized-stage
 * equations of Section "Learnable Winograd transform scales"; the Hadamard
 * stage between them is the one wq_conv_forward always runs):
 *   X~ = s_B s_B s_x  Q(B^T/s_B) Q(d/s_x) Q(B/s_B),   y = s_A s_A s_Y  Q(A^T/s_A) Q(Y/s_Y) Q(A/s_A) + bias.
 * mode 0: off (fp32 transforms, the default); 1: one scale per transform matrix
 * (abs-max/127); 2: one scale per matrix row.  The plan's fp32 B^T and A^T are
 * quantized to int8 on the host; s_x is dynamic, one per (tile, group of
 * group_size input channels) over the n x n x group_size patch; s_Y is dynamic,
 * one per (tile, output channel) over its n x n Winograd-domain values; the
 * integer products are exact; scales, the scaled products and the bias add are
 * evaluated in fp64 and rounded once to fp32 (X~ before the group quantizer of
 * stage 1, y at the store).  The paper leaves these granularities open; this is
 * the reading the CPU reference of the tests implements.  Stages 2+3 then run in
 * a variant that writes the Winograd-domain products to the workspace (GEMM_* or
 * LDS_TAP_*); wq_plan_tune refuses the others with WQ_ERR_UNSUPPORTED while the
 * mode is on.  Host call, no device work; call it before wq_weight_prepare or
 * after, the weight blob does not depend on it. */
wq_status_t wq_plan_set_integer_transforms(wq_plan_t *plan, int mode);

/* Offline stage (W = G w G^T, then group-wise quantization along Cin):
 * reads w_dev [Cout][Cin][3][3] fp32 and bias_dev [Cout] fp32 (NULL = zero
 * bias) and fills weight_blob_dev (blob_bytes, 256-byte aligned). */
wq_status_t wq_weight_prepare(wq_plan_t *plan, void *stream,
                              const float *w_dev, const float *bias_dev,
                              void *weight_blob_dev, size_t blob_bytes);

/* Stage 1 alone (X = B^T x B, dynamic group-wise quantization): reads x_dev
 * [N][H][W][Cin] fp32 and fills Xq and sX inside workspace_dev. */
wq_status_t wq_input_transform(const wq_plan_t *plan, void *stream, const float *x_dev,
                               void *workspace_dev, size_t workspace_bytes);

/* Stages 2+3 alone (int8 contraction with per-group dequantization, then
 * y = A^T Y A + bias): reads the workspace written by wq_input_transform and
 * the weight blob, writes y_dev [N][H][W][Cout] fp32.  May use the M scratch area of
 * the workspace. */
wq_status_t wq_contract_output(const wq_plan_t *plan, void *stream,
                               void *workspace_dev, size_t workspace_bytes,
                               const void *weight_blob_dev, size_t blob_bytes, float *y_dev);

/* For profilers: only the first (part = 1) or only the second (part = 2) kernel of
 * wq_contract_output (k2_kernels says how many there are; part 2 of a one-kernel variant
 * launches nothing).  Any other part -> INVALID_ARG. */
wq_status_t wq_contract_output_part(const wq_plan_t *plan, void *stream, void *workspace_dev,
                                    size_t workspace_bytes, const void *weight_blob_dev,
                                    size_t blob_bytes, float *y_dev, int part);

/* Stage 2 alone, in the two-kernel form (any plan may call it, whatever
 * k2_kernels says): the n*n int8 GEMMs over the workspace's Xq/sX and the
 * blob's Wq/sW with per-group dequantization (the Hadamard-product equation
 * of Section "Winograd convolution" summed over input channels, with the scales of the
 * second quantized-stage equation of Section "Learnable Winograd transform
 * scales"); writes M fp32 [T_pad][n*n][Cout_pad] at ws_M_off. */
wq_status_t wq_contract(const wq_plan_t *plan, void *stream, void *workspace_dev,
                        size_t workspace_bytes, const void *weight_blob_dev, size_t blob_bytes);

/* Stage 3 alone (the output-transform equation of Section "Winograd
 * convolution"): y = A^T M A + bias from the M that
 * wq_contract left in the workspace; writes y_dev [N][H][W][Cout] fp32. */
wq_status_t wq_output_transform(const wq_plan_t *plan, void *stream, const void *workspace_dev,
                                size_t workspace_bytes, const void *weight_blob_dev,
                                size_t blob_bytes, float *y_dev);

/* The whole forward pass: wq_input_transform followed by wq_contract_output. */
wq_status_t wq_conv_forward(const wq_plan_t *plan, void *stream, const float *x_dev,
                            const void *weight_blob_dev, size_t blob_bytes,
                            void *workspace_dev, size_t workspace_bytes, float *y_dev);

/* wq_conv_forward for callers that cannot allocate device memory or pass a
 * workspace along: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The workspace is a device array owned by
 * the library, WQ_STATIC_WORKSPACE_BYTES large, one copy per GPU, held until the
 * process ends; this call allocates nothing (its first call on a device looks
 * up the array's address there).  A plan whose ws_bytes exceeds
 * WQ_STATIC_WORKSPACE_BYTES -> WQ_ERR_WORKSPACE (checked on the host before any
 * device call).  All calls on one GPU share the array: calls that overlap in
 * time on the same GPU (two streams, two threads) race - serialise them or
 * use wq_conv_forward with separate workspaces.  The array keeps the previous
 * call's contents; nothing depends on them.  Inputs, weight blob and output
 * are the caller's, as for wq_conv_forward, and the result is the same bit
 * for bit. */
#define WQ_STATIC_WORKSPACE_BYTES (32u << 20)
wq_status_t wq_conv_forward_static(const wq_plan_t *plan, void *stream, const float *x_dev,
                                   const void *weight_blob_dev, size_t blob_bytes, float *y_dev);

/* wq_conv_forward with a dump of the exact int32 group partial sums
 * P[t][tile][group][o] = sum_{c in group} Xq[t][tile][c] * Wq[t][o][c] (the
 * integer product inside the second quantized-stage equation of Section
 * "Learnable Winograd transform scales").  It launches exactly the kernel
 * instances wq_conv_forward launches for this plan (wq_layout_t::k2_variant,
 * same tile configuration, same launch shape), compiled from the same kernel
 * templates with the stores of P switched on.
 * P_dev: int32 [n*n][T][groups][Cout], dense (debug_P_bytes).  For tests. */
wq_status_t wq_conv_forward_debug(const wq_plan_t *plan, void *stream, const float *x_dev,
                                  const void *weight_blob_dev, size_t blob_bytes,
                                  void *workspace_dev, size_t workspace_bytes, float *y_dev,
                                  int32_t *P_dev, size_t P_bytes);

/* The same with only a slab of P stored, for layers whose full P is too large
 * to keep: taps [tap0, tap0+ntaps) x tiles [tile0, tile0+ntiles), every group
 * and output channel.  P_dev: int32 [ntaps][ntiles][groups][Cout]
 * (ntaps*ntiles*groups*Cout*4 bytes, else WORKSPACE).  An empty or out-of-range
 * slab -> INVALID_ARG. */
wq_status_t wq_conv_forward_debug_slab(const wq_plan_t *plan, void *stream, const float *x_dev,
                                       const void *weight_blob_dev, size_t blob_bytes,
                                       void *workspace_dev, size_t workspace_bytes, float *y_dev,
                                       int32_t *P_dev, size_t P_bytes,
                                       int tap0, int ntaps, int tile0, int ntiles);

/* ---------------------------------------------------------------------------
 * The group-wise int8 quantized STANDARD 3x3 convolution (stride 1, zero pad 1)
 * that the paper's Section "Runtime improvements" measures the quantized
 * Winograd convolution against.  Same quantizer and the same groups along the
 * input channels; no transforms:
 *   activations: one dynamic scale per (pixel, group);
 *   weights:     one scale per (filter tap t = u*3+v, output channel, group);
 *   y[p][o] = bias[o] + sum_{t, group} float(int32 dot product over the group)
 *                                      * sx[pixel shifted by tap t][group] * sw[t][group][o].
 * Formats (device, sizes and offsets from wq_direct_plan_layout):
 *   weight blob : Wq int8, blocked like the Winograd blob with `taps` taps
 *                 [taps][Cout_pad/16][Cin/kstep][4][16][kstep/4]  at blob_Wq_off
 *                 sW fp32 [taps][groups][Cout_pad]                 at blob_sW_off
 *                 bias fp32 [Cout_pad]                             at blob_bias_off
 *   workspace   : xq int8 [N*H*W][Cin] (NHWC)                      at ws_xq_off
 *                 sx fp32 [N*H*W][groups]                          at ws_sx_off
 *                 partial sums fp32 [splits][N*H*W][Cout]          at ws_part_off (scratch, splits > 1)
 * Conventions as above: caller-owned device memory, calls enqueue on `stream`
 * and never synchronise, every argument is checked on the host.  Errors:
 * non-positive sizes, NULL pointers, Cin not a multiple of group_size ->
 * INVALID_ARG; group_size not in {32,64,128,256,512}, a tensor of 2 GiB or
 * more, or more than 4193280 pixels (rows) -> UNSUPPORTED; a buffer smaller than the layout says -> WORKSPACE;
 * conv before weight_prepare -> NOT_PREPARED. */
typedef struct wq_direct_plan wq_direct_plan_t;

typedef struct {
    int32_t N, H, W, Cin, Cout, group_size, groups, P, Cout_pad, kstep;
    int32_t splits, taps; /* splits: workgroups sharing the reduction of an output tile: the 9 taps
                             (1, 3 or 9) or, for a linear layer, its groups (a power of two up to 16);
                             taps: 9 for the 3x3 convolution, 1 for a linear layer */
    int32_t weight_bits;  /* 8, or 4 (W4A8) */
    int32_t reserved;     /* 0 */
    uint64_t blob_bytes, blob_Wq_off, blob_sW_off, blob_bias_off;
    uint64_t ws_bytes, ws_xq_off, ws_sx_off, ws_part_off;
} wq_direct_layout_t;

wq_status_t wq_direct_plan_create(wq_direct_plan_t **out, int N, int H, int W, int Cin, int Cout,
                                  int group_size);
/* The same plan type for a group-wise quantized LINEAR layer y = x W^T + bias (the paper
 * quantizes every linear layer and attention product the same way, Section "Experiments"):
 * x [R][Cin] fp32 with one dynamic scale per (row, group), W [Cout][Cin] fp32 with one scale
 * per (output row, group), y [R][Cout] fp32.  It is the one-tap case of the convolution above:
 * use wq_direct_weight_prepare (w_dev is then [Cout][Cin]), wq_direct_quantize,
 * wq_direct_conv and wq_direct_forward with N*H*W = R; the layout has taps = 1. */
wq_status_t wq_linear_plan_create(wq_direct_plan_t **out, int R, int Cin, int Cout, int group_size);
/* W4A8 (the 4/8-bit rows of the paper's result tables, which apply to standard convolutions
 * and linear layers): the same two plans with weight codes `weight_bits` wide, 8 or 4 (anything
 * else -> UNSUPPORTED).  4-bit codes come from the same symmetric abs-max quantizer with codes
 * in [-7, 7] and scale max|w|/7 per (tap, output channel, group); activations stay int8 with
 * dynamic scales.  The blob then holds two codes per byte in the same blocked order: each
 * aligned 16-byte piece d0 d1 d2 d3 (little-endian 32-bit words) of the int8 layout becomes
 * the 8 bytes p0 p1 at half its offset, byte j of p0 carrying byte j of d0 in its low nibble and
 * byte j of d1 in its high nibble (two's complement), p1 likewise from d2 and d3; Wq takes
 * taps*Cout_pad*Cin/2 bytes.  Scales, bias, workspace and every other call are unchanged. */
wq_status_t wq_direct_plan_create_bits(wq_direct_plan_t **out, int N, int H, int W, int Cin, int Cout,
                                       int group_size, int weight_bits);
wq_status_t wq_linear_plan_create_bits(wq_direct_plan_t **out, int R, int Cin, int Cout, int group_size,
                                       int weight_bits);
/* Tuning override for tests and sweeps: the number of workgroups that share the reduction of
 * an output tile (wq_direct_layout_t::splits).  0 keeps the plan's own choice; a 3x3 plan takes
 * 1, 3 or 9, a linear plan a power of two up to 16 that divides its group count; anything else
 * -> UNSUPPORTED.  Changes ws_bytes: call it before sizing the workspace. */
wq_status_t wq_direct_plan_tune(wq_direct_plan_t *plan, int splits);
wq_status_t wq_direct_plan_destroy(wq_direct_plan_t *plan);
wq_status_t wq_direct_plan_layout(const wq_direct_plan_t *plan, wq_direct_layout_t *out);

/* Offline: quantizes w_dev [Cout][Cin][3][3] fp32 per (tap, output channel,
 * group) into the blob and copies bias_dev [Cout] (NULL = zeros). */
wq_status_t wq_direct_weight_prepare(wq_direct_plan_t *plan, void *stream, const float *w_dev,
                                     const float *bias_dev, void *weight_blob_dev, size_t blob_bytes);

/* Dynamic activation quantization: x_dev [N][H][W][Cin] fp32 -> xq, sx in the workspace. */
wq_status_t wq_direct_quantize(const wq_direct_plan_t *plan, void *stream, const float *x_dev,
                               void *workspace_dev, size_t workspace_bytes);

/* The convolution proper on the quantized operands; writes y_dev [N][H][W][Cout] fp32.
 * May use the partial-sum area of the workspace. */
wq_status_t wq_direct_conv(const wq_direct_plan_t *plan, void *stream, void *workspace_dev,
                           size_t workspace_bytes, const void *weight_blob_dev, size_t blob_bytes,
                           float *y_dev);

/* wq_direct_quantize followed by wq_direct_conv. */
wq_status_t wq_direct_forward(const wq_direct_plan_t *plan, void *stream, const float *x_dev,
                              const void *weight_blob_dev, size_t blob_bytes, void *workspace_dev,
                              size_t workspace_bytes, float *y_dev);

/* Issue-rate microbenchmark of the contraction's inner loop, without memory traffic: every
 * wave repeats, `iters` times (even), the int8 MFMAs of one quantization group on
 * `blocks_per_wave` (2 or 4) 16x16 blocks followed by the per-group dequantization the second
 * quantized-stage equation of Section "Learnable Winograd transform scales" demands
 * (M += float(P) * sW * sX: 12 vector instructions per block).  mode 0 = MFMAs only, 1 =
 * dequantization only, 2 = each group's MFMAs then its dequantization, 3 = the MFMAs of the next
 * group issued before the dequantization of the previous one.  group_size in {32,64,128,256,512}
 * (32: the 16x16x32 instruction; otherwise group_size/64 16x16x64 instructions per block and
 * group).  `workgroups` workgroups of 4 waves are launched.  seed_dev: 64 int32 (any values);
 * out_dev: workgroups*256 floats (written so that nothing is optimised away); cycles_dev: two
 * int64 per workgroup, the cycle-counter ticks and the 100 MHz wall-clock ticks its first wave
 * spent in the loop. */
wq_status_t wq_microbench_dequant(void *stream, int mode, int group_size, int blocks_per_wave,
                                  int workgroups, int iters, const int32_t *seed_dev,
                                  float *out_dev, long long *cycles_dev);

const char *wq_status_string(wq_status_t status);

#ifdef __cplusplus
}
#endif
#if defined(__GNUC__)
#pragma GCC visibility pop
#endif
#endif /* WQ_H */
