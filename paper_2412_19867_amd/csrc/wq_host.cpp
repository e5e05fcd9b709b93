// Host side of the wq library: plan creation and validation, buffer layouts,
// the standard transform matrices, and the C-ABI entry points that check
// their arguments and enqueue the kernels.  Nothing here touches the device
// except through the launchers in the kernel files.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

#include "wq_internal.h"

namespace {

// Standard F(m,3) matrices (supplementary Section "Standard Winograd
// transforms"): B^T = diag(S_B) V^{-T}, G = diag(S_G) V, A^T = V^T diag(S_A)
// for the points 0, 1, -1, 2, -2, (1/2, -1/2,) infinity.
const double kBT2[16] = {1, 0, -1, 0, 0, 1, 1, 0, 0, -1, 1, 0, 0, 1, 0, -1};
const double kG2[12] = {1, 0, 0, 0.5, 0.5, 0.5, 0.5, -0.5, 0.5, 0, 0, 1};
const double kAT2[8] = {1, 1, 1, 0, 0, 1, -1, -1};

const double kBT4[36] = {4, 0,  -5, 0,  1, 0, 0, -4, -4, 1,  1, 0, 0, 4, -4, -1, 1, 0,
                         0, -2, -1, 2,  1, 0, 0, 2,  -1, -2, 1, 0, 0, 4, 0,  -5, 0, 1};
const double kG4[18] = {1.0 / 4,  0,        0,       -1.0 / 6, -1.0 / 6,  -1.0 / 6,
                        -1.0 / 6, 1.0 / 6,  -1.0 / 6, 1.0 / 24, 1.0 / 12, 1.0 / 6,
                        1.0 / 24, -1.0 / 12, 1.0 / 6, 0,        0,        1};
const double kAT4[24] = {1, 1, 1, 1, 1, 0, 0, 1, -1, 2, -2, 0, 0, 1, 1, 4, 4, 0, 0, 1, -1, 8, -8, 1};

const double kBT6[64] = {
    1, 0,    -5.25, 0,     5.25,  0,     -1, 0,   //
    0, 1,    1,     -4.25, -4.25, 1,     1,  0,   //
    0, -1,   1,     4.25,  -4.25, -1,    1,  0,   //
    0, 0.5,  0.25,  -2.5,  -1.25, 2,     1,  0,   //
    0, -0.5, 0.25,  2.5,   -1.25, -2,    1,  0,   //
    0, 2,    4,     -2.5,  -5,    0.5,   1,  0,   //
    0, -2,   4,     2.5,   -5,    -0.5,  1,  0,   //
    0, -1,   0,     5.25,  0,     -5.25, 0,  1};
const double kG6[24] = {1,         0,          0,        -2.0 / 9,  -2.0 / 9,  -2.0 / 9,
                        -2.0 / 9,  2.0 / 9,    -2.0 / 9, 1.0 / 90,  1.0 / 45,  2.0 / 45,
                        1.0 / 90,  -1.0 / 45,  2.0 / 45, 32.0 / 45, 16.0 / 45, 8.0 / 45,
                        32.0 / 45, -16.0 / 45, 8.0 / 45, 0,         0,         1};
const double kAT6[48] = {
    1, 1, 1,  1,  1,   1,        1,         0,  //
    0, 1, -1, 2,  -2,  0.5,      -0.5,      0,  //
    0, 1, 1,  4,  4,   0.25,     0.25,      0,  //
    0, 1, -1, 8,  -8,  0.125,    -0.125,    0,  //
    0, 1, 1,  16, 16,  0.0625,   0.0625,    0,  //
    0, 1, -1, 32, -32, 0.03125,  -0.03125,  1};

bool std_tables(int m, const double **bt, const double **g, const double **at) {
    switch (m) {
        case 2: *bt = kBT2; *g = kG2; *at = kAT2; return true;
        case 4: *bt = kBT4; *g = kG4; *at = kAT4; return true;
        case 6: *bt = kBT6; *g = kG6; *at = kAT6; return true;
        default: return false;
    }
}

uint64_t align256(uint64_t v) { return (v + 255) & ~uint64_t(255); }

template <int M>
void detect_patterns(wq_plan *p) {
    constexpr int n = M + 2;
    p->sparse_bt = p->sparse_g = p->sparse_at = true;
    for (int i = 0; i < n; ++i)
        for (int k = 0; k < n; ++k)
            if (!wq_pattern<M>::bt(i, k) && p->xf.BT[i * n + k] != 0.0f) p->sparse_bt = false;
    for (int i = 0; i < n; ++i)
        for (int k = 0; k < 3; ++k)
            if (!wq_pattern<M>::g(i, k) && p->xf.G[i * 3 + k] != 0.0f) p->sparse_g = false;
    for (int a = 0; a < M; ++a)
        for (int i = 0; i < n; ++i)
            if (!wq_pattern<M>::at(a, i) && p->xf.AT[a * n + i] != 0.0f) p->sparse_at = false;
    // paired columns: AT[a][2k] = (-1)^a r_k AT[a][2k-1] to within one unit in the last place of
    // fp32 (the entries of a rescaled matrix were rounded one by one, so exact equality is too
    // much to ask; a difference of one ulp in a coefficient is of the size of the roundings the
    // fp32 evaluation makes anyway).  Anything further off takes the dense code, which uses
    // every entry as given.
    for (int k = 1; k <= (n - 2) / 2 && p->sparse_at; ++k) {
        const int i1 = 2 * k - 1, i2 = 2 * k;
        int best = 0;
        for (int a = 1; a < M; ++a)
            if (std::fabs(p->xf.AT[a * n + i1]) > std::fabs(p->xf.AT[best * n + i1])) best = a;
        const double d = p->xf.AT[best * n + i1];
        if (d == 0.0) { p->sparse_at = false; break; }
        const double r = ((best & 1) ? -1.0 : 1.0) * (double)p->xf.AT[best * n + i2] / d;
        for (int a = 0; a < M; ++a) {
            const double want = ((a & 1) ? -1.0 : 1.0) * r * (double)p->xf.AT[a * n + i1];
            const double got = p->xf.AT[a * n + i2];
            if (std::fabs(got - want) > 1.1920929e-7 * std::fabs(got) + 1e-37) p->sparse_at = false;
        }
        p->xf.ATr[k - 1] = (float)r;
    }
}

// 1-D minimal-filtering identity: the triple computes y[a] = sum_k d[a+k] g[k].
bool valid_triple(const wq_xf &xf, int m) {
    const int n = m + 2;
    for (int i = 0; i < n * n; ++i)
        if (!std::isfinite(xf.BT[i])) return false;
    for (int i = 0; i < n * 3; ++i)
        if (!std::isfinite(xf.G[i])) return false;
    for (int i = 0; i < m * n; ++i)
        if (!std::isfinite(xf.AT[i])) return false;
    for (int a = 0; a < m; ++a)
        for (int k = 0; k < 3; ++k)
            for (int l = 0; l < n; ++l) {
                double s = 0.0, mag = 0.0;
                for (int i = 0; i < n; ++i) {
                    double term = (double)xf.AT[a * n + i] * xf.G[i * 3 + k] * xf.BT[i * n + l];
                    s += term;
                    mag += std::fabs(term);
                }
                const double want = (l == a + k) ? 1.0 : 0.0;
                if (std::fabs(s - want) > 1e-4 * (mag > 1.0 ? mag : 1.0)) return false;
            }
    return true;
}

enum { CHECK_BLOB = 1, CHECK_WS = 2 };
wq_status_t check_buffers(const wq_plan *p, int which, const void *blob, size_t blob_bytes,
                          const void *ws, size_t ws_bytes) {
    if (!p) return WQ_ERR_INVALID_ARG;
    if (which & CHECK_BLOB) {
        if (!blob) return WQ_ERR_INVALID_ARG;
        if (blob_bytes < p->lay.blob_bytes) return WQ_ERR_WORKSPACE;
    }
    if (which & CHECK_WS) {
        if (!ws) return WQ_ERR_INVALID_ARG;
        if (ws_bytes < p->lay.ws_bytes) return WQ_ERR_WORKSPACE;
    }
    return WQ_OK;
}

// ---- which kernel instances a plan runs (all measured on MI355X) ----

// Tap rows per workgroup of the input kernel.  A workgroup that forms all n rows reads its
// tiles once and has the longest instruction stream per wave; splitting the rows over
// blockIdx.y re-reads the tiles through L1/L2 but shortens the stream and multiplies the
// waves.  Over layers from 32 to 20480 waves (counted with all rows in one workgroup): big
// layers want all rows together, mid-sized ones halves, small ones two rows (one row only when
// the layer is a handful of waves).
int default_k1_rows(const wq_plan *p) {
    const int n = p->n;
    const long waves_all_rows = (long)(p->T_pad / 16) * (p->Cin / 32) * 4;
    if (waves_all_rows >= 1536) return n;
    if (n == 8 || waves_all_rows >= 1024) return n / 2;
    if (waves_all_rows >= 128) return 2;
    return 1;
}

bool k1_rows_ok(const wq_plan *p, int rows) {
    return rows == 1 || rows == 2 || rows == p->n / 2 || rows == p->n;
}

bool variant_applicable(const wq_plan *p, int v) {
    // the integer output transform quantizes whole n x n tiles of the Winograd-domain result: only
    // the forms that write it to the workspace can feed it
    if (p->integer_transforms && !wq_is_gemm_variant(v) && !wq_is_lds_tap_variant(v)) return false;
    const bool fast_fused_ok = p->sparse_at && p->m != 2 && p->g <= 64;   // instantiated for one K-step per group
    switch (v) {
        case WQ_K2_FUSED_16x16: return true;
        case WQ_K2_FUSED_KSPLIT: return fast_fused_ok && p->groups % 2 == 0;
        case WQ_K2_FUSED_32x16:
        case WQ_K2_FUSED_32x32: return fast_fused_ok;
        case WQ_K2_GEMM_64x64:
        case WQ_K2_GEMM_32x128: return true;
        case WQ_K2_GEMM_128x128: return p->g >= 128 && p->groups <= 8;
        case WQ_K2_LDS_FULL_64x64: return p->m == 4;   // 16 waves of F(6,3) state do not fit the registers
        case WQ_K2_LDS_FULL_32x64:
        case WQ_K2_LDS_FULL_32x32:
        case WQ_K2_LDS_ROW_64x64:
        case WQ_K2_LDS_ROW_32x64:
        case WQ_K2_LDS_TAP_64x64: return p->m != 2;    // instantiated for F(4,3) and F(6,3)
        case WQ_K2_LDS_TAP_128x128: return p->m != 2 && p->groups <= 16;   // no fp64 chunk totals at this wave tile
        default: return false;
    }
}

int default_k2_variant(const wq_plan *p) {
    if (p->integer_transforms) {
        if (p->T_pad <= 32 || ((p->T_pad % 64) == 32 && p->T_pad <= 160)) return WQ_K2_GEMM_32x128;
        return (p->g < 128 && p->m != 2) ? WQ_K2_LDS_TAP_64x64 : WQ_K2_GEMM_64x64;
    }
    // The row form with operand tiles shared through LDS: measured ahead of the others where its
    // workgroups (64 tiles x 64 channels x one tap row) fill the GPU once at two to three per CU
    // and each of them walks a reduction long enough to pay for the second kernel.
    if (variant_applicable(p, WQ_K2_LDS_ROW_64x64) && p->g == p->kstep && p->groups >= 8) {
        const long wgs = (long)((p->T_pad + 63) / 64) * ((p->Cout_pad + 63) / 64) * (p->m + 2);
        // also layers large in tiles AND output channels, where the Winograd-domain product the
        // two-kernel forms write would reach hundreds of MB
        if (wgs >= 384 && (wgs <= 768 || (p->T_pad >= 1024 && p->Cout_pad >= 512))) return WQ_K2_LDS_ROW_64x64;
    }
    // With few tiles the Winograd-domain result is small next to the operands, and a tiled GEMM
    // per tap plus a separate output transform beats the fused kernel; so it does for very wide
    // layers and for groups of 128 and more, where the fused kernel's register tiles re-read the
    // operands too often.
    const bool two_kernel = (p->T_pad <= 512 && (p->Cin >= 512 || (p->g == 32 && p->Cin >= 128))) ||
                            p->Cin >= 1024 || p->g >= 128;
    if (two_kernel) {
        // 128x128 tiles: groups of 128 and more on layers with at least 1024 tiles and 256 channels
        if (p->g >= 128 && p->groups <= 8 && p->T_pad >= 1024 && p->Cout_pad >= 256)
            return variant_applicable(p, WQ_K2_LDS_TAP_128x128) ? WQ_K2_LDS_TAP_128x128 : WQ_K2_GEMM_128x128;
        // 32-tile workgroups when 64-tile ones would leave half a tile row of blocks empty
        if ((p->T_pad % 64) == 32 && p->T_pad <= 160) return WQ_K2_GEMM_32x128;
        // two to eight 64-tile blocks: the same tiling with the operands staged in LDS measures ahead
        if (p->T_pad >= 128 && p->T_pad <= 512 && p->g < 128 && variant_applicable(p, WQ_K2_LDS_TAP_64x64))
            return WQ_K2_LDS_TAP_64x64;
        return WQ_K2_GEMM_64x64;
    }
    // Many tiles and a short reduction (the 128 x 128, 320-channel layer): one 16x16 block per wave with
    // the operands shared through LDS, four workgroups of 32 tiles x 32 channels per CU.  A workgroup
    // walks all n*n taps in sequence, so the reduction must be short and the workgroups must fill
    // the GPU at least twice over; the fused kernel below has the same traffic but fewer, fatter waves.
    if (p->m == 4 && p->g == p->kstep && variant_applicable(p, WQ_K2_LDS_FULL_32x32)) {
        const long wgs = (long)((p->T_pad + 31) / 32) * ((p->Cout_pad + 31) / 32);
        if (wgs >= 512 && p->groups <= 6) return WQ_K2_LDS_FULL_32x32;
    }
    if (!variant_applicable(p, WQ_K2_FUSED_32x16)) return WQ_K2_FUSED_16x16;
    // few tile blocks -> split K over more waves; many blocks -> taller or bigger register tiles
    const long tb = p->T_pad / 16, ob = p->Cout_pad / 16;
    const bool can_split = p->groups % 2 == 0 && p->groups >= 4;
    if (tb <= 2) return can_split ? WQ_K2_FUSED_KSPLIT : WQ_K2_FUSED_16x16;
    if (tb * ob >= 640) return ob >= 40 ? WQ_K2_FUSED_32x32 : WQ_K2_FUSED_32x16;
    if (tb >= 16) return WQ_K2_FUSED_32x16;
    return (can_split && p->groups >= 16) ? WQ_K2_FUSED_KSPLIT : WQ_K2_FUSED_16x16;
}

void publish_choices(wq_plan *p) {
    p->lay.k2_variant = p->k2_variant;
    p->lay.k1_rows = p->k1_rows;
    p->lay.k2_kernels = (wq_is_gemm_variant(p->k2_variant) || wq_is_lds_row_variant(p->k2_variant) ||
                         wq_is_lds_tap_variant(p->k2_variant)) ? 2 : 1;
}

struct Blob {
    const int8_t *Wq;
    const float *sW;
    const float *bias;
};
Blob blob_of(const wq_plan *p, const void *blob) {
    const char *b = (const char *)blob;
    return {(const int8_t *)(b + p->lay.blob_Wq_off), (const float *)(b + p->lay.blob_sW_off),
            (const float *)(b + p->lay.blob_bias_off)};
}

}  // namespace

extern "C" {

wq_status_t wq_standard_transforms(int m, double *BT, double *G, double *AT) {
    const double *bt, *g, *at;
    if (!std_tables(m, &bt, &g, &at)) return WQ_ERR_UNSUPPORTED;
    const int n = m + 2;
    if (BT) std::memcpy(BT, bt, sizeof(double) * n * n);
    if (G) std::memcpy(G, g, sizeof(double) * n * 3);
    if (AT) std::memcpy(AT, at, sizeof(double) * m * n);
    return WQ_OK;
}

wq_status_t wq_scaled_transforms(int m, const double *u_B, const double *u_G, float *BT, float *G,
                                 float *AT) {
    const double *bt, *g, *at;
    if (!std_tables(m, &bt, &g, &at)) return WQ_ERR_UNSUPPORTED;
    if (!u_B || !u_G) return WQ_ERR_INVALID_ARG;
    const int n = m + 2;
    for (int i = 0; i < n; ++i)
        if (!std::isfinite(u_B[i]) || !std::isfinite(u_G[i]) || u_B[i] * u_G[i] == 0.0 ||
            !std::isfinite(1.0 / (u_B[i] * u_G[i])))
            return WQ_ERR_INVALID_ARG;
    // S_B and S_G scale rows; S_A = (S_B S_G)^-1 scales the columns of A^T
    if (BT)
        for (int i = 0; i < n; ++i)
            for (int k = 0; k < n; ++k) BT[i * n + k] = (float)(bt[i * n + k] * u_B[i]);
    if (G)
        for (int i = 0; i < n; ++i)
            for (int k = 0; k < 3; ++k) G[i * 3 + k] = (float)(g[i * 3 + k] * u_G[i]);
    if (AT)
        for (int a = 0; a < m; ++a)
            for (int i = 0; i < n; ++i) AT[a * n + i] = (float)(at[a * n + i] / (u_B[i] * u_G[i]));
    return WQ_OK;
}

wq_status_t wq_plan_create(wq_plan_t **out, int N, int H, int W, int Cin, int Cout, int m,
                           int group_size, const float *BT, const float *G, const float *AT) {
    if (!out) return WQ_ERR_INVALID_ARG;
    *out = nullptr;
    if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || group_size <= 0)
        return WQ_ERR_INVALID_ARG;
    const bool any = BT || G || AT, all = BT && G && AT;
    if (any && !all) return WQ_ERR_INVALID_ARG;
    if (m != 2 && m != 4 && m != 6) return WQ_ERR_UNSUPPORTED;
    if (group_size != 32 && group_size != 64 && group_size != 128 && group_size != 256 &&
        group_size != 512)
        return WQ_ERR_UNSUPPORTED;
    if (Cin % group_size != 0) return WQ_ERR_INVALID_ARG;
    const int n = m + 2;
    const long long TH = (H + m - 1) / m, TW = (W + m - 1) / m, T = (long long)N * TH * TW;
    // 32-bit byte offsets inside the kernels (buffer addressing): every tensor below 2 GiB,
    // the input below 1 GiB (its out-of-image offsets are pushed past the end by adding 2^30)
    {
        const long long n2 = (long long)n * n, Tp = (T + 31) / 32 * 32, Cp = (Cout + 31) / 32 * 32;
        const long long lim = (1LL << 31) - 1;
        if ((long long)N * H * W * Cin * 4 > (1LL << 30) || (long long)N * H * W * Cout * 4 > lim ||
            n2 * Tp * Cin > lim || n2 * Cp * Cin > lim || n2 * Tp * Cp * 4 > lim || n2 * Tp * (Cin / group_size) * 4 > lim ||
            n2 * Cp * (Cin / group_size) * 4 > lim)
            return WQ_ERR_UNSUPPORTED;
    }

    wq_plan *p = new (std::nothrow) wq_plan();
    if (!p) return WQ_ERR_INVALID_ARG;
    p->N = N; p->H = H; p->W = W; p->Cin = Cin; p->Cout = Cout; p->m = m; p->n = n;
    p->g = group_size; p->groups = Cin / group_size;
    p->TH = (int)TH; p->TW = (int)TW; p->T = (int)T;
    p->T_pad = (int)((T + 31) / 32 * 32);
    p->Cout_pad = (Cout + 31) / 32 * 32;
    p->kstep = group_size == 32 ? 32 : 64;
    p->wbits = 8;
    p->prepared.store(0);
    p->integer_transforms = 0;
    std::memset(&p->xi, 0, sizeof(p->xi));
    std::memset(&p->xf, 0, sizeof(p->xf));
    if (all) {
        std::memcpy(p->xf.BT, BT, sizeof(float) * n * n);
        std::memcpy(p->xf.G, G, sizeof(float) * n * 3);
        std::memcpy(p->xf.AT, AT, sizeof(float) * m * n);
    } else {
        const double *bt, *g, *at;
        std_tables(m, &bt, &g, &at);
        for (int i = 0; i < n * n; ++i) p->xf.BT[i] = (float)bt[i];
        for (int i = 0; i < n * 3; ++i) p->xf.G[i] = (float)g[i];
        for (int i = 0; i < m * n; ++i) p->xf.AT[i] = (float)at[i];
    }
    if (!valid_triple(p->xf, m)) {
        delete p;
        return WQ_ERR_BAD_TRANSFORM;
    }
    if (m == 2) detect_patterns<2>(p);
    else if (m == 4) detect_patterns<4>(p);
    else detect_patterns<6>(p);

    wq_layout_t &L = p->lay;
    L.N = N; L.H = H; L.W = W; L.Cin = Cin; L.Cout = Cout; L.m = m; L.n = n;
    L.group_size = group_size; L.groups = p->groups;
    L.TH = p->TH; L.TW = p->TW; L.T = p->T; L.T_pad = p->T_pad; L.Cout_pad = p->Cout_pad;
    L.kstep = p->kstep;
    const uint64_t n2 = (uint64_t)n * n;
    L.blob_Wq_off = 0;
    L.blob_sW_off = align256(n2 * p->Cout_pad * Cin);
    L.blob_bias_off = L.blob_sW_off + align256(n2 * p->groups * p->Cout_pad * 4);
    L.blob_bytes = L.blob_bias_off + align256((uint64_t)p->Cout_pad * 4);
    L.ws_Xq_off = 0;
    L.ws_sX_off = align256(n2 * p->T_pad * Cin);
    L.ws_M_off = L.ws_sX_off + align256(n2 * p->T_pad * p->groups * 4);
    L.ws_bytes = L.ws_M_off + align256(n2 * p->T_pad * p->Cout_pad * 4);
    L.debug_P_bytes = n2 * (uint64_t)T * p->groups * Cout * 4;
    p->k1_rows = default_k1_rows(p);
    p->k2_variant = default_k2_variant(p);
    publish_choices(p);
    *out = p;
    return WQ_OK;
}

wq_status_t wq_plan_destroy(wq_plan_t *plan) {
    if (!plan) return WQ_ERR_INVALID_ARG;
    delete plan;
    return WQ_OK;
}

wq_status_t wq_plan_tune(wq_plan_t *plan, int k1_rows, int k2_variant) {
    if (!plan) return WQ_ERR_INVALID_ARG;
    if (k1_rows < 0 || k1_rows > 8) return WQ_ERR_INVALID_ARG;
    switch (k2_variant) {
        case WQ_K2_AUTO:
        case WQ_K2_FUSED_16x16: case WQ_K2_FUSED_KSPLIT: case WQ_K2_FUSED_32x16: case WQ_K2_FUSED_32x32:
        case WQ_K2_GEMM_64x64: case WQ_K2_GEMM_32x128: case WQ_K2_GEMM_128x128:
        case WQ_K2_LDS_FULL_64x64: case WQ_K2_LDS_FULL_32x64: case WQ_K2_LDS_FULL_32x32:
        case WQ_K2_LDS_ROW_64x64: case WQ_K2_LDS_ROW_32x64: case WQ_K2_LDS_TAP_64x64: case WQ_K2_LDS_TAP_128x128: break;
        default: return WQ_ERR_INVALID_ARG;
    }
    if (k1_rows != 0 && !k1_rows_ok(plan, k1_rows)) return WQ_ERR_UNSUPPORTED;
    if (plan->integer_transforms && k1_rows != 0 && k1_rows != plan->n) return WQ_ERR_UNSUPPORTED;
    if (k2_variant != WQ_K2_AUTO && !variant_applicable(plan, k2_variant)) return WQ_ERR_UNSUPPORTED;
    plan->k1_rows = k1_rows ? k1_rows : (plan->integer_transforms ? plan->n : default_k1_rows(plan));
    plan->k2_variant = k2_variant != WQ_K2_AUTO ? k2_variant : default_k2_variant(plan);
    publish_choices(plan);
    return WQ_OK;
}

// Q(M / s), s = abs-max / 127, over a whole matrix or per row; in double on the host.
static void quantize_matrix(const float *Mx, int rows, int cols, int stride, bool per_row, int *Q, double *s) {
    double a_all = 0.0;
    for (int r = 0; r < rows; ++r)
        for (int c = 0; c < cols; ++c) a_all = std::fmax(a_all, std::fabs((double)Mx[r * stride + c]));
    for (int r = 0; r < rows; ++r) {
        double a = a_all;
        if (per_row) {
            a = 0.0;
            for (int c = 0; c < cols; ++c) a = std::fmax(a, std::fabs((double)Mx[r * stride + c]));
        }
        s[r] = a > 0.0 ? a / 127.0 : 0.0;
        const double rcp = a > 0.0 ? 127.0 / a : 0.0;
        for (int c = 0; c < cols; ++c) {
            double q = std::nearbyint((double)Mx[r * stride + c] * rcp);   // round half to even
            q = std::fmin(127.0, std::fmax(-127.0, q));
            Q[r * stride + c] = (int)q;
        }
    }
}

wq_status_t wq_plan_set_integer_transforms(wq_plan_t *plan, int mode) {
    if (!plan || mode < 0 || mode > 2) return WQ_ERR_INVALID_ARG;
    plan->integer_transforms = mode;
    if (mode) {
        const int n = plan->n, m = plan->m;
        double sB[8], sA[8];
        quantize_matrix(plan->xf.BT, n, n, n, mode == 2, plan->xi.QB, sB);
        quantize_matrix(plan->xf.AT, m, n, n, mode == 2, plan->xi.QA, sA);
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) plan->xi.sBB[i * n + j] = sB[i] * sB[j];
        for (int a = 0; a < m; ++a)
            for (int b = 0; b < m; ++b) plan->xi.sAA[a * m + b] = sA[a] * sA[b];
        plan->k1_rows = n;   // the patch scale needs the whole patch in one workgroup
    } else {
        plan->k1_rows = default_k1_rows(plan);
    }
    plan->k2_variant = default_k2_variant(plan);
    publish_choices(plan);
    return WQ_OK;
}

wq_status_t wq_plan_layout(const wq_plan_t *plan, wq_layout_t *out) {
    if (!plan || !out) return WQ_ERR_INVALID_ARG;
    *out = plan->lay;
    return WQ_OK;
}

wq_status_t wq_weight_prepare(wq_plan_t *plan, void *stream, const float *w_dev,
                              const float *bias_dev, void *weight_blob_dev, size_t blob_bytes) {
    if (!plan || !w_dev) return WQ_ERR_INVALID_ARG;
    wq_status_t st = check_buffers(plan, CHECK_BLOB, weight_blob_dev, blob_bytes, nullptr, 0);
    if (st != WQ_OK) return st;
    char *b = (char *)weight_blob_dev;
    hipError_t e = wq_launch_weight(plan, (hipStream_t)stream, w_dev, bias_dev,
                                    (int8_t *)(b + plan->lay.blob_Wq_off),
                                    (float *)(b + plan->lay.blob_sW_off),
                                    (float *)(b + plan->lay.blob_bias_off));
    if (e != hipSuccess) return WQ_ERR_DEVICE;
    plan->prepared.store(1);
    return WQ_OK;
}

wq_status_t wq_input_transform(const wq_plan_t *plan, void *stream, const float *x_dev,
                               void *workspace_dev, size_t workspace_bytes) {
    if (!plan || !x_dev) return WQ_ERR_INVALID_ARG;
    wq_status_t st = check_buffers(plan, CHECK_WS, nullptr, 0, workspace_dev, workspace_bytes);
    if (st != WQ_OK) return st;
    char *ws = (char *)workspace_dev;
    hipError_t e = wq_launch_input(plan, (hipStream_t)stream, x_dev,
                                   (int8_t *)(ws + plan->lay.ws_Xq_off),
                                   (float *)(ws + plan->lay.ws_sX_off));
    return e == hipSuccess ? WQ_OK : WQ_ERR_DEVICE;
}

static wq_status_t contract_impl(const wq_plan_t *plan, void *stream, void *workspace_dev,
                                 size_t workspace_bytes, const void *weight_blob_dev,
                                 size_t blob_bytes, float *y_dev, const wq_dump &dump, int parts = 3) {
    if (!plan || !y_dev) return WQ_ERR_INVALID_ARG;
    wq_status_t st = check_buffers(plan, CHECK_BLOB | CHECK_WS, weight_blob_dev, blob_bytes, workspace_dev, workspace_bytes);
    if (st != WQ_OK) return st;
    if (!plan->prepared.load()) return WQ_ERR_NOT_PREPARED;
    char *ws = (char *)workspace_dev;
    Blob bl = blob_of(plan, weight_blob_dev);
    hipError_t e = wq_launch_contract(plan, (hipStream_t)stream,
                                      (const int8_t *)(ws + plan->lay.ws_Xq_off),
                                      (const float *)(ws + plan->lay.ws_sX_off), bl.Wq, bl.sW,
                                      bl.bias, (float *)(ws + plan->lay.ws_M_off), y_dev, dump, parts);
    return e == hipSuccess ? WQ_OK : WQ_ERR_DEVICE;
}

static const wq_dump kNoDump = {nullptr, 0, 0, 0, 0};

wq_status_t wq_contract_output(const wq_plan_t *plan, void *stream, void *workspace_dev,
                               size_t workspace_bytes, const void *weight_blob_dev,
                               size_t blob_bytes, float *y_dev) {
    return contract_impl(plan, stream, workspace_dev, workspace_bytes, weight_blob_dev, blob_bytes,
                         y_dev, kNoDump);
}

wq_status_t wq_contract_output_part(const wq_plan_t *plan, void *stream, void *workspace_dev,
                                    size_t workspace_bytes, const void *weight_blob_dev,
                                    size_t blob_bytes, float *y_dev, int part) {
    if (part != 1 && part != 2) return WQ_ERR_INVALID_ARG;
    return contract_impl(plan, stream, workspace_dev, workspace_bytes, weight_blob_dev, blob_bytes,
                         y_dev, kNoDump, part);
}

static wq_status_t split_stage(const wq_plan_t *plan, void *stream, void *workspace_dev,
                               size_t workspace_bytes, const void *weight_blob_dev,
                               size_t blob_bytes, float *y_dev, int stages) {
    if (!plan || ((stages & 2) && !y_dev)) return WQ_ERR_INVALID_ARG;
    wq_status_t st = check_buffers(plan, CHECK_BLOB | CHECK_WS, weight_blob_dev, blob_bytes, workspace_dev, workspace_bytes);
    if (st != WQ_OK) return st;
    if (!plan->prepared.load()) return WQ_ERR_NOT_PREPARED;
    char *ws = (char *)workspace_dev;
    Blob bl = blob_of(plan, weight_blob_dev);
    hipError_t e = wq_launch_contract_unfused(plan, (hipStream_t)stream,
                                              (const int8_t *)(ws + plan->lay.ws_Xq_off),
                                              (const float *)(ws + plan->lay.ws_sX_off), bl.Wq,
                                              bl.sW, bl.bias, (float *)(ws + plan->lay.ws_M_off),
                                              y_dev, stages, kNoDump);
    return e == hipSuccess ? WQ_OK : WQ_ERR_DEVICE;
}

wq_status_t wq_contract(const wq_plan_t *plan, void *stream, void *workspace_dev,
                        size_t workspace_bytes, const void *weight_blob_dev, size_t blob_bytes) {
    return split_stage(plan, stream, workspace_dev, workspace_bytes, weight_blob_dev, blob_bytes,
                       nullptr, 1);
}

wq_status_t wq_output_transform(const wq_plan_t *plan, void *stream, const void *workspace_dev,
                                size_t workspace_bytes, const void *weight_blob_dev,
                                size_t blob_bytes, float *y_dev) {
    return split_stage(plan, stream, const_cast<void *>(workspace_dev), workspace_bytes,
                       weight_blob_dev, blob_bytes, y_dev, 2);
}

wq_status_t wq_conv_forward(const wq_plan_t *plan, void *stream, const float *x_dev,
                            const void *weight_blob_dev, size_t blob_bytes, void *workspace_dev,
                            size_t workspace_bytes, float *y_dev) {
    if (!plan || !x_dev || !y_dev) return WQ_ERR_INVALID_ARG;
    wq_status_t st = check_buffers(plan, CHECK_BLOB | CHECK_WS, weight_blob_dev, blob_bytes, workspace_dev, workspace_bytes);
    if (st != WQ_OK) return st;
    if (!plan->prepared.load()) return WQ_ERR_NOT_PREPARED;
    st = wq_input_transform(plan, stream, x_dev, workspace_dev, workspace_bytes);
    if (st != WQ_OK) return st;
    return contract_impl(plan, stream, workspace_dev, workspace_bytes, weight_blob_dev, blob_bytes,
                         y_dev, kNoDump);
}

wq_status_t wq_conv_forward_debug_slab(const wq_plan_t *plan, void *stream, const float *x_dev,
                                       const void *weight_blob_dev, size_t blob_bytes,
                                       void *workspace_dev, size_t workspace_bytes, float *y_dev,
                                       int32_t *P_dev, size_t P_bytes, int tap0, int ntaps, int tile0,
                                       int ntiles) {
    if (!plan || !x_dev || !y_dev || !P_dev) return WQ_ERR_INVALID_ARG;
    wq_status_t st = check_buffers(plan, CHECK_BLOB | CHECK_WS, weight_blob_dev, blob_bytes, workspace_dev, workspace_bytes);
    if (st != WQ_OK) return st;
    const int n2 = plan->n * plan->n;
    if (tap0 < 0 || ntaps <= 0 || tap0 > n2 - ntaps || tile0 < 0 || ntiles <= 0 ||
        tile0 > plan->T - ntiles)
        return WQ_ERR_INVALID_ARG;
    if (P_bytes < (size_t)ntaps * ntiles * plan->groups * plan->Cout * 4) return WQ_ERR_WORKSPACE;
    if (!plan->prepared.load()) return WQ_ERR_NOT_PREPARED;
    st = wq_input_transform(plan, stream, x_dev, workspace_dev, workspace_bytes);
    if (st != WQ_OK) return st;
    const wq_dump dump = {P_dev, tap0, ntaps, tile0, ntiles};
    return contract_impl(plan, stream, workspace_dev, workspace_bytes, weight_blob_dev, blob_bytes,
                         y_dev, dump);
}

wq_status_t wq_conv_forward_debug(const wq_plan_t *plan, void *stream, const float *x_dev,
                                  const void *weight_blob_dev, size_t blob_bytes,
                                  void *workspace_dev, size_t workspace_bytes, float *y_dev,
                                  int32_t *P_dev, size_t P_bytes) {
    if (!plan) return WQ_ERR_INVALID_ARG;
    return wq_conv_forward_debug_slab(plan, stream, x_dev, weight_blob_dev, blob_bytes, workspace_dev,
                                      workspace_bytes, y_dev, P_dev, P_bytes, 0, plan->n * plan->n, 0,
                                      plan->T);
}

const char *wq_status_string(wq_status_t status) {
    switch (status) {
        case WQ_OK: return "ok";
        case WQ_ERR_INVALID_ARG: return "invalid argument";
        case WQ_ERR_UNSUPPORTED: return "unsupported configuration";
        case WQ_ERR_BAD_TRANSFORM: return "transform matrices are not a valid F(m,3) triple";
        case WQ_ERR_NOT_PREPARED: return "weights were never prepared on this plan";
        case WQ_ERR_WORKSPACE: return "caller buffer too small";
        case WQ_ERR_DEVICE: return "kernel launch failed";
    }
    return "unknown status";
}

}  // extern "C"
