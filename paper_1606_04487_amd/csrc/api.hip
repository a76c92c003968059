// C ABI of the library: argument checks, workspace carving and the launch sequence of each pass.
// Everything before the first launch is plain host code, so every error path can be exercised on a
// machine without a GPU.
#include <cmath>
#include <mutex>

#include "common.h"
#include "pack_jobs.h"

namespace omni {

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int make_geom(const omni_conv_desc *d, ConvGeom *g)
{
    if (d == nullptr) return OMNI_INVALID_ARGUMENT;
    if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->F <= 0 || d->kh <= 0 || d->kw <= 0 ||
        d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0)
        return OMNI_INVALID_ARGUMENT;
    int64_t eh = (int64_t)d->H + 2 * (int64_t)d->pad_h - d->kh;
    int64_t ew = (int64_t)d->W + 2 * (int64_t)d->pad_w - d->kw;
    if (eh < 0 || ew < 0) return OMNI_INVALID_ARGUMENT;  // the window does not fit: empty output
    if (d->dtype != OMNI_F32 && d->dtype != OMNI_BF16) return OMNI_UNSUPPORTED;
    if (d->flags & ~(OMNI_FLAG_RELU | OMNI_FLAG_DHAT_CACHED | OMNI_FLAG_FUSED | OMNI_FLAG_SPLIT_K)) return OMNI_UNSUPPORTED;
    int64_t Ho = eh / d->stride_h + 1, Wo = ew / d->stride_w + 1;
    int64_t M = (int64_t)d->N * Ho * Wo;
    int64_t K = (int64_t)d->C * d->kh * d->kw;
    const int64_t lim = 0x7fffffffll - 4096;  // indices are decoded with 32-bit multiply-high divisions
    if (M > lim || K > lim || (int64_t)d->H * d->W > lim || (int64_t)d->N * d->C > lim ||
        (int64_t)d->N * d->F > lim || d->F > 65535 || (int64_t)d->pad_h + d->H > lim ||
        (int64_t)d->pad_w + d->W > lim)
        return OMNI_UNSUPPORTED;
    g->N = d->N; g->C = d->C; g->H = d->H; g->W = d->W; g->F = d->F;
    g->kh = d->kh; g->kw = d->kw; g->sh = d->stride_h; g->sw = d->stride_w; g->ph = d->pad_h; g->pw = d->pad_w;
    g->Ho = (int32_t)Ho; g->Wo = (int32_t)Wo; g->K = (int32_t)K; g->M = (int32_t)M; g->HoWo = (int32_t)(Ho * Wo);
    g->flags = d->flags;
    g->div_Wo = FastDiv((uint32_t)Wo);
    g->div_HoWo = FastDiv((uint32_t)(Ho * Wo));
    g->div_kw = FastDiv((uint32_t)d->kw);
    g->div_khkw = FastDiv((uint32_t)(d->kh * d->kw));
    g->div_W = FastDiv((uint32_t)d->W);
    g->div_HW = FastDiv((uint32_t)(d->H * d->W));
    g->div_sh = FastDiv((uint32_t)d->stride_h);
    g->div_sw = FastDiv((uint32_t)d->stride_w);
    return OMNI_OK;
}

static size_t align256(size_t b) { return (b + 255) / 256 * 256; }

// OMNI_FLAG_SPLIT_K: a forward / data-gradient product of rows x cols results over a reduction of `red`
// (a multiple of the LDS tile).  Split when its tiles fill at most half the compute units, into as many
// chunks as bring the work items to about one per unit, each chunk at least four steps long.
static void plan_split_k(const ConvGeom &g, int dtype, int64_t rows, int64_t cols, int64_t red, int *splits, int64_t *chunk)
{
    int64_t bk = gemm_red_tile(dtype);
    *splits = 1;
    *chunk = round_up(red, bk);
    if (!(g.flags & OMNI_FLAG_SPLIT_K)) return;
    int bm, bn;
    gemm_split_tile((int)rows, (int)cols, &bm, &bn);
    int64_t tiles = ((rows + bm - 1) / bm) * ((cols + bn - 1) / bn);
    int64_t steps = (red + bk - 1) / bk;
    if (tiles > 128 || steps < 8) return;
    int64_t want = 256 / tiles, most = steps / 4;
    int64_t n = want < most ? want : most;
    if (n < 2) return;
    *chunk = round_up((red + n - 1) / n, bk);
    *splits = (int)((red + *chunk - 1) / *chunk);
}

void plan_forward(const ConvGeom &g, int dtype, ForwardWs *w)
{
    size_t e = elem_size(dtype);
    w->ld = dhat_ld(g);
    w->Fp = g.F;
    w->Kp = round_up(g.K, 64);  // zero padded to whole reduction steps
    w->dhat = 0;
    w->khat = align256((size_t)g.K * w->ld * e);
    w->partials = w->khat + align256((size_t)w->Fp * w->Kp * e);
    plan_split_k(g, dtype, g.F, w->ld, g.K, &w->splits, &w->chunk);
    w->total = w->partials + align256(w->splits > 1 ? (size_t)w->splits * g.F * w->ld * sizeof(float) : 0);
    w->explicit_total = w->total;
    // the fused path keeps only its repacked weights here
    if (fused_supported(g, dtype, false) && fused_weight_bytes(g, false) > w->total) w->total = align256(fused_weight_bytes(g, false));
    if (strided_supported(g, dtype) && strided_weight_bytes(g) > w->total) w->total = align256(strided_weight_bytes(g));
}

void plan_backward_data(const ConvGeom &g, int dtype, BwdDataWs *w)
{
    size_t e = elem_size(dtype);
    w->ld = dhat_ld(g);
    w->Kp = g.K;
    w->Fp = round_up(g.F, 64);  // zero padded to whole reduction steps
    w->ddhat = 0;
    w->dyhat = align256((size_t)g.K * w->ld * e);
    w->khat_t = w->dyhat + align256((size_t)g.F * w->ld * e);
    w->partials = w->khat_t + align256((size_t)w->Kp * w->Fp * e);
    if (dgrad_dense_supported(g)) {
        // whole-image window: one product dX [N][K] = dY [N][F] * W [F][K]; the workspace holds only its partial sums
        plan_split_k(g, dtype, g.N, g.K, g.F, &w->splits, &w->chunk);
        w->partials = 0;
        w->total = align256(w->splits > 1 ? (size_t)w->splits * g.N * g.K * sizeof(float) : 16);
        return;
    }
    plan_split_k(g, dtype, g.K, w->ld, g.F, &w->splits, &w->chunk);
    w->total = w->partials + align256(w->splits > 1 ? (size_t)w->splits * g.K * w->ld * sizeof(float) : 0);
    if (fused_supported(g, dtype, true) && fused_weight_bytes(g, true) > w->total) w->total = align256(fused_weight_bytes(g, true));
    if (strided_dgrad_supported(g, dtype) && strided_dgrad_bytes(g) > w->total) w->total = align256(strided_dgrad_bytes(g));
}

// Split the long reduction (extent ld) over the chip: one round of 256 x 256 workgroups on the 256 compute
// units or two rounds of 128 x 128 ones (just under, so that the last round is full), each with at least
// four steps.  More splits would balance better but every split writes, and the reduction re-reads, a
// whole fp32 copy of the gradient (measured: twice as many splits cost 4 % of the training step).
static void plan_splits(const ConvGeom &g, int dtype, int64_t ld, int *splits_out, int64_t *chunk_out)
{
    int64_t bk = gemm_red_tile(dtype);
    int bm, bn;
    gemm_wgrad_tile(g.F, g.K, &bm, &bn);
    int64_t tiles = ((g.F + bm - 1) / bm) * (int64_t)((g.K + bn - 1) / bn);
    int64_t steps = (ld + bk - 1) / bk;
    int64_t rounds = bm * bn >= 192 * 256 ? 1 : 2;
    int64_t want = (256 * rounds) / tiles;
    int64_t max_splits = steps / 4 > 0 ? steps / 4 : 1;
    int64_t splits = want < max_splits ? want : max_splits;
    if (splits < 1) splits = 1;
    int64_t chunk = round_up((ld + splits - 1) / splits, bk);
    *splits_out = (int)((ld + chunk - 1) / chunk);
    *chunk_out = chunk;
}

void plan_backward_weights(const ConvGeom &g, int dtype, BwdWeightsWs *w)
{
    size_t e = elem_size(dtype);
    w->ld = dhat_ld(g);
    plan_splits(g, dtype, w->ld, &w->splits, &w->chunk);
    w->bias_blocks = pack_dyhat_blocks(g);
    // the direct model gradient uses a row-padded dY-hat; the regions are sized for whichever is larger
    const bool direct = wgrad_direct_supported(g, dtype);
    w->ld_rows = direct ? dyhat_rows_ld(g) : w->ld;
    w->splits_rows = w->splits, w->chunk_rows = w->chunk, w->bias_blocks_rows = w->bias_blocks;
    if (direct) {
        plan_splits(g, dtype, w->ld_rows, &w->splits_rows, &w->chunk_rows);
        w->bias_blocks_rows = pack_dyhat_rows_blocks(g);
    }
    // the phase-split model gradient of a stride-4 layer: one result tile, so a workgroup per split
    const bool phase = !direct && wgrad_phase_supported(g, dtype);
    int64_t k_max = g.K;
    size_t x4_bytes = 0;
    if (phase) {
        w->ld_rows = dyhat_rows_ld(g);
        int64_t bk = gemm_red_tile(dtype), steps = (w->ld_rows + bk - 1) / bk;
        int64_t splits = steps / 4 < 256 ? steps / 4 : 256;
        if (splits < 1) splits = 1;
        w->chunk_rows = round_up((w->ld_rows + splits - 1) / splits, bk);
        w->splits_rows = (int)((w->ld_rows + w->chunk_rows - 1) / w->chunk_rows);
        w->bias_blocks_rows = pack_dyhat_rows_blocks(g);
        k_max = wgrad_phase_kp(g) + 1 > g.K ? wgrad_phase_kp(g) + 1 : g.K;  // + 1: the bias gradient's column
        x4_bytes = (size_t)g.N * g.C * 4 * g.H * wgrad_phase_wp(g) * e;
    }
    // the LDS-patch model gradient: its own split count over images, always through the partial sums
    w->splits_patch = !phase && wgrad_patch_supported(g, dtype) ? wgrad_patch_splits(g) : 0;
    if (w->splits_patch > 0) {
        w->ld_rows = dyhat_rows_ld(g);
        w->bias_blocks_rows = pack_dyhat_rows_blocks(g);
    }
    w->splits_wide = !phase && w->splits_patch == 0 && wgrad_wide_supported(g, dtype) ? wgrad_wide_splits(g) : 0;
    if (w->splits_wide > 0) {
        w->ld_rows = dyhat_rows_ld(g);
        w->bias_blocks_rows = pack_dyhat_rows_blocks(g);
    }
    int64_t ld_max = w->ld > w->ld_rows ? w->ld : w->ld_rows;
    int splits_max = w->splits > w->splits_rows ? w->splits : w->splits_rows;
    if (w->splits_wide > 0 && splits_max < w->splits_wide + 1) splits_max = w->splits_wide + 1;
    if (w->splits_patch > 0 && splits_max < w->splits_patch + 1) splits_max = w->splits_patch + 1;  // + 1: kept even when it is 1
    int bb_max = w->bias_blocks > w->bias_blocks_rows ? w->bias_blocks : w->bias_blocks_rows;
    w->dhat = 0;
    size_t dhat_bytes = (size_t)g.K * w->ld * e;
    w->dyhat = align256(dhat_bytes > x4_bytes ? dhat_bytes : x4_bytes);
    w->partials = w->dyhat + align256((size_t)g.F * ld_max * e);
    w->bias_partials = w->partials + align256(splits_max > 1 || phase ? (size_t)splits_max * g.F * k_max * sizeof(float) : 0);
    w->total = w->bias_partials + align256((size_t)g.F * bb_max * sizeof(float));
}

}  // namespace omni

using namespace omni;

extern "C" {

const char *omni_status_string(int status)
{
    switch (status) {
    case OMNI_OK: return "ok";
    case OMNI_INVALID_ARGUMENT: return "invalid argument";
    case OMNI_UNSUPPORTED: return "unsupported dtype, flag or extent";
    case OMNI_WORKSPACE_TOO_SMALL: return "workspace too small";
    case OMNI_MISALIGNED: return "device pointer not 16-byte aligned";
    case OMNI_HIP_ERROR: return "HIP launch error";
    default: return "unknown status";
    }
}

const char *omni_version(void) { return "0.1"; }

int omni_tuning_set(int knob, int value)
{
    switch (knob) {
    case OMNI_TUNE_GEMM_TILE: set_gemm_tile_override(value); return OMNI_OK;
    case OMNI_TUNE_FUSED_BN:
        if (value != 0 && value != 256 && value != 384 && value != 512) return OMNI_INVALID_ARGUMENT;
        set_fused_tile_override(value, -1);
        return OMNI_OK;
    case OMNI_TUNE_FUSED_BM:
        if (value != 0 && value != 96 && value != 128) return OMNI_INVALID_ARGUMENT;
        set_fused_tile_override(-1, value);
        return OMNI_OK;
    case OMNI_TUNE_FUSED_PITCH:
        if (value != 0 && value != 1) return OMNI_INVALID_ARGUMENT;
        set_fused_pitch_override(value);
        return OMNI_OK;
    case OMNI_TUNE_POOL_LDS:
        if (value != 0 && value != 1) return OMNI_INVALID_ARGUMENT;
        set_pool_override(value);
        return OMNI_OK;
    case OMNI_TUNE_WGRAD_SPLITS:
        if (value < 0) return OMNI_INVALID_ARGUMENT;
        set_wgrad_patch_override(value, -1);
        set_wgrad_wide_override(value, -1);
        return OMNI_OK;
    case OMNI_TUNE_WGRAD_PATCH:
        if (value != 0 && value != 1) return OMNI_INVALID_ARGUMENT;
        set_wgrad_patch_override(-1, value);
        set_wgrad_wide_override(-1, value);
        return OMNI_OK;
    default: return OMNI_INVALID_ARGUMENT;
    }
}

int omni_conv_output_dims(const omni_conv_desc *desc, int32_t *Ho, int32_t *Wo)
{
    if (Ho == nullptr || Wo == nullptr) return OMNI_INVALID_ARGUMENT;
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    *Ho = g.Ho;
    *Wo = g.Wo;
    return OMNI_OK;
}

int omni_conv_dhat_ld(const omni_conv_desc *desc, int64_t *ld)
{
    if (ld == nullptr) return OMNI_INVALID_ARGUMENT;
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    *ld = dhat_ld(g);
    return OMNI_OK;
}

int omni_conv_workspace_bytes(const omni_conv_desc *desc, int pass, size_t *bytes)
{
    if (bytes == nullptr) return OMNI_INVALID_ARGUMENT;
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    if (pass == OMNI_PASS_FORWARD) {
        ForwardWs w;
        plan_forward(g, desc->dtype, &w);
        *bytes = w.total;
    } else if (pass == OMNI_PASS_BACKWARD_DATA) {
        BwdDataWs w;
        plan_backward_data(g, desc->dtype, &w);
        *bytes = w.total;
    } else if (pass == OMNI_PASS_BACKWARD_WEIGHTS) {
        BwdWeightsWs w;
        plan_backward_weights(g, desc->dtype, &w);
        *bytes = w.total;
    } else {
        return OMNI_INVALID_ARGUMENT;
    }
    return OMNI_OK;
}

int omni_conv_fused_supported(const omni_conv_desc *desc, int pass)
{
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    if (pass == OMNI_PASS_FORWARD) {
        ForwardWs w;
        plan_forward(g, desc->dtype, &w);
        if (strided_supported(g, desc->dtype) && strided_weight_bytes(g) <= w.total) return 1;
        return fused_supported(g, desc->dtype, false) && fused_weight_bytes(g, false) <= w.total ? 1 : 0;
    }
    if (pass == OMNI_PASS_BACKWARD_DATA) {
        BwdDataWs w;
        plan_backward_data(g, desc->dtype, &w);
        if (strided_dgrad_supported(g, desc->dtype) && strided_dgrad_bytes(g) <= w.total) return 1;
        return fused_supported(g, desc->dtype, true) && fused_weight_bytes(g, true) <= w.total ? 1 : 0;
    }
    if (pass == OMNI_PASS_BACKWARD_WEIGHTS)
        return wgrad_patch_supported(g, desc->dtype) || wgrad_wide_supported(g, desc->dtype) || wgrad_direct_supported(g, desc->dtype) || wgrad_phase_supported(g, desc->dtype) ? 1 : 0;
    return OMNI_INVALID_ARGUMENT;
}

// The forward pass on checked arguments.  `avail` bytes of scratch at `ws`: each path checks what IT needs
// (the fused kernels only their repacked weights, the explicit path D-hat, K-hat and the split partials).
static int forward_on_scratch(const omni_conv_desc *desc, const ConvGeom &g, const ForwardWs &w, const void *X, const void *W,
                              const float *bias, void *Y, char *ws, size_t avail, hipStream_t s, const void *prepacked = nullptr)
{
    const int relu = (desc->flags & OMNI_FLAG_RELU) ? 1 : 0;
    if ((desc->flags & OMNI_FLAG_FUSED) && fused_supported(g, desc->dtype, false)) {
        if (avail < fused_weight_bytes(g, false)) return OMNI_WORKSPACE_TOO_SMALL;
        return launch_fused_conv(g, false, X, W, bias, relu, Y, ws, s, -1, prepacked);
    }
    if ((desc->flags & OMNI_FLAG_FUSED) && strided_supported(g, desc->dtype)) {
        if (avail < strided_weight_bytes(g)) return OMNI_WORKSPACE_TOO_SMALL;
        return launch_strided_conv(g, X, W, bias, relu, Y, ws, s, prepacked);
    }
    if (prepacked != nullptr) return OMNI_UNSUPPORTED;  // the explicit path reads W itself
    if (avail < w.explicit_total) return OMNI_WORKSPACE_TOO_SMALL;
    void *Dhat = ws + w.dhat, *Khat = ws + w.khat;
    int st = launch_lower(g, desc->dtype, X, Dhat, w.ld, s);
    if (st != OMNI_OK) return st;
    // K-hat is W with every row zero-padded to whole reduction steps: where there is nothing to pad, W itself
    const bool w_is_khat = w.Kp == g.K && w.Fp == g.F;
    if (!w_is_khat) {
        st = launch_pack_khat(g, desc->dtype, W, Khat, w.Fp, w.Kp, s);
        if (st != OMNI_OK) return st;
    }
    GemmFwdArgs a{w_is_khat ? W : Khat, w.Kp, Dhat, w.ld, bias, Y, relu, (float *)(ws + w.partials), w.splits, w.chunk};
    return launch_gemm_forward(g, desc->dtype, a, s);
}

int omni_conv_forward(const omni_conv_desc *desc, const void *X, const void *W, const float *bias, void *Y,
                      void *workspace, size_t workspace_bytes, void *hip_stream)
{
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    if (X == nullptr || W == nullptr || Y == nullptr || workspace == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(X) || !aligned16(W) || !aligned16(Y) || !aligned16(workspace) || (bias && !aligned16(bias)))
        return OMNI_MISALIGNED;
    ForwardWs w;
    plan_forward(g, desc->dtype, &w);
    if (workspace_bytes < w.total) return OMNI_WORKSPACE_TOO_SMALL;
    return forward_on_scratch(desc, g, w, X, W, bias, Y, (char *)workspace, workspace_bytes, (hipStream_t)hip_stream);
}

// ---------------------------------------------------------------- the forward pass on the library's own scratch
// One array per GPU, part of the loaded code object: it exists from the moment the library is loaded on a
// device until the process ends, and no call ever allocates it.  In host code the array's name is only a
// handle for hipGetSymbolAddress; kernels and copies get the device address looked up below.
static __device__ __align__(256) unsigned char scratch[OMNI_STATIC_SCRATCH_BYTES];

static const int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[kMaxDevices];  // per device: the address of that GPU's copy of the array

// The current device's copy of the array (looked up once per device), or null if HIP refuses.
static char *static_scratch_base()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return (char *)g_scratch_ptr[dev];
}

int omni_conv_forward_static(const omni_conv_desc *desc, const void *X, const void *W, const float *bias, void *Y,
                             void *hip_stream)
{
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    if (X == nullptr || W == nullptr || Y == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(X) || !aligned16(W) || !aligned16(Y) || (bias && !aligned16(bias))) return OMNI_MISALIGNED;
    ForwardWs w;
    plan_forward(g, desc->dtype, &w);
    size_t need = 0;
    st = omni_conv_static_scratch_need(desc, &need);
    if (st != OMNI_OK) return st;
    if (need > (size_t)OMNI_STATIC_SCRATCH_BYTES) return OMNI_WORKSPACE_TOO_SMALL;  // before any HIP call
    char *ws = static_scratch_base();
    if (ws == nullptr) return OMNI_HIP_ERROR;
    // Nothing in the scratch has to start at zero: every path writes each byte it later reads (D-hat with its
    // padded columns, K-hat with its padding, the repacked weights with their padded rows) in this very call.
    return forward_on_scratch(desc, g, w, X, W, bias, Y, ws, (size_t)OMNI_STATIC_SCRATCH_BYTES, (hipStream_t)hip_stream);
}

int omni_conv_static_scratch_need(const omni_conv_desc *desc, size_t *bytes)
{
    if (bytes == nullptr) return OMNI_INVALID_ARGUMENT;
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    ForwardWs w;
    plan_forward(g, desc->dtype, &w);
    if ((desc->flags & OMNI_FLAG_FUSED) && fused_supported(g, desc->dtype, false)) *bytes = fused_weight_bytes(g, false);
    else if ((desc->flags & OMNI_FLAG_FUSED) && strided_supported(g, desc->dtype)) *bytes = strided_weight_bytes(g);
    else *bytes = w.explicit_total;
    return OMNI_OK;
}

int omni_conv_forward_partial(const omni_conv_desc *desc, int32_t b_p, const void *X, const void *W,
                              const float *bias, void *Y, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    if (b_p < 1 || b_p > desc->N || X == nullptr || Y == nullptr) return OMNI_INVALID_ARGUMENT;
    const size_t e = elem_size(desc->dtype);
    const size_t x_image = (size_t)g.C * g.H * g.W * e, y_image = (size_t)g.F * g.HoWo * e;
    if (b_p < desc->N && ((x_image * (size_t)b_p) % 16 != 0 || (y_image * (size_t)b_p) % 16 != 0)) return OMNI_MISALIGNED;
    omni_conv_desc part = *desc;
    part.flags &= ~(uint32_t)OMNI_FLAG_FUSED;
    // check every group's arguments before the first launch: a failed call launches nothing
    part.N = b_p;
    ForwardWs w;
    ConvGeom gp;
    st = make_geom(&part, &gp);
    if (st != OMNI_OK) return st;
    plan_forward(gp, part.dtype, &w);
    if (W == nullptr || workspace == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(X) || !aligned16(W) || !aligned16(Y) || !aligned16(workspace) || (bias && !aligned16(bias)))
        return OMNI_MISALIGNED;
    if (workspace_bytes < w.total) return OMNI_WORKSPACE_TOO_SMALL;
    if (desc->N % b_p != 0) {  // the smaller last group plans for itself (its split may differ): check it now too
        omni_conv_desc last = part;
        last.N = desc->N % b_p;
        ForwardWs wl;
        ConvGeom gl;
        st = make_geom(&last, &gl);
        if (st != OMNI_OK) return st;
        plan_forward(gl, last.dtype, &wl);
        if (workspace_bytes < wl.total) return OMNI_WORKSPACE_TOO_SMALL;
    }
    for (int32_t n0 = 0; n0 < desc->N; n0 += b_p) {
        part.N = desc->N - n0 < b_p ? desc->N - n0 : b_p;
        st = omni_conv_forward(&part, (const char *)X + (size_t)n0 * x_image, W, bias, (char *)Y + (size_t)n0 * y_image,
                               workspace, workspace_bytes, hip_stream);
        if (st != OMNI_OK) return st;
    }
    return OMNI_OK;
}

int omni_conv_backward_data(const omni_conv_desc *desc, const void *dY, const void *W, void *dX, void *workspace,
                            size_t workspace_bytes, void *hip_stream)
{
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    if (dY == nullptr || W == nullptr || dX == nullptr || workspace == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(dY) || !aligned16(W) || !aligned16(dX) || !aligned16(workspace)) return OMNI_MISALIGNED;
    BwdDataWs w;
    plan_backward_data(g, desc->dtype, &w);
    if (workspace_bytes < w.total) return OMNI_WORKSPACE_TOO_SMALL;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    void *dDhat = ws + w.ddhat, *dYhat = ws + w.dyhat, *KhatT = ws + w.khat_t;

    if ((desc->flags & OMNI_FLAG_FUSED) && fused_supported(g, desc->dtype, true) &&
        fused_weight_bytes(g, true) <= w.total)
        return launch_fused_conv(g, true, dY, W, nullptr, 0, dX, ws, s);
    if ((desc->flags & OMNI_FLAG_FUSED) && strided_dgrad_supported(g, desc->dtype) && strided_dgrad_bytes(g) <= w.total)
        return launch_strided_dgrad(g, dY, W, dX, ws, s);

    if (dgrad_dense_supported(g))
        return launch_gemm_dgrad_dense(g, desc->dtype, dY, W, dX, (float *)(ws + w.partials), w.splits, w.chunk, s);

    st = launch_pack_dyhat(g, desc->dtype, dY, dYhat, w.ld, nullptr, 0, nullptr, s);
    if (st != OMNI_OK) return st;
    st = launch_pack_khat_t(g, desc->dtype, W, KhatT, w.Kp, w.Fp, s);
    if (st != OMNI_OK) return st;
    GemmDgradArgs a{KhatT, w.Fp, dYhat, w.ld, dDhat, (float *)(ws + w.partials), w.splits, w.chunk};
    st = launch_gemm_dgrad(g, desc->dtype, a, s);
    if (st != OMNI_OK) return st;
    return launch_col2im(g, desc->dtype, dDhat, w.ld, dX, s);
}

// Which repacking (if any) `pass` of this layer reads with OMNI_FLAG_FUSED: fills `job` (when not null) and `bytes`.
static bool packed_weights_job(const omni_conv_desc *desc, const ConvGeom &g, int pass, const void *W, void *packed, PackJob *job,
                               size_t *bytes)
{
    *bytes = 0;
    if (!(desc->flags & OMNI_FLAG_FUSED)) return false;
    if (pass == OMNI_PASS_FORWARD) {
        if (fused_supported(g, desc->dtype, false)) return fused_pack_job(g, false, W, packed, job, bytes);
        if (strided_supported(g, desc->dtype)) return strided_pack_job(g, W, packed, job, bytes);
        return false;
    }
    if (pass == OMNI_PASS_BACKWARD_DATA && fused_supported(g, desc->dtype, true)) return fused_pack_job(g, true, W, packed, job, bytes);
    return false;
}

int omni_conv_packed_weights_bytes(const omni_conv_desc *desc, int pass, size_t *bytes)
{
    if (bytes == nullptr) return OMNI_INVALID_ARGUMENT;
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    if (pass != OMNI_PASS_FORWARD && pass != OMNI_PASS_BACKWARD_DATA) return OMNI_INVALID_ARGUMENT;
    packed_weights_job(desc, g, pass, nullptr, nullptr, nullptr, bytes);
    return OMNI_OK;
}

int omni_conv_pack_weights(int32_t n, const omni_conv_desc *descs, const int32_t *passes, const void *const *W,
                           void *const *packed, void *hip_stream)
{
    if (n < 0 || n > MAX_PACK_JOBS) return OMNI_INVALID_ARGUMENT;
    if (n == 0) return OMNI_OK;
    if (descs == nullptr || passes == nullptr || W == nullptr || packed == nullptr) return OMNI_INVALID_ARGUMENT;
    PackJobTable t;
    t.n = n;
    t.first_block[0] = 0;
    for (int i = 0; i < n; ++i) {
        ConvGeom g;
        int st = make_geom(&descs[i], &g);
        if (st != OMNI_OK) return st;
        if (passes[i] != OMNI_PASS_FORWARD && passes[i] != OMNI_PASS_BACKWARD_DATA) return OMNI_INVALID_ARGUMENT;
        if (W[i] == nullptr || packed[i] == nullptr) return OMNI_INVALID_ARGUMENT;
        if (!aligned16(W[i]) || !aligned16(packed[i])) return OMNI_MISALIGNED;
        size_t bytes;
        if (!packed_weights_job(&descs[i], g, passes[i], W[i], packed[i], &t.job[i], &bytes)) return OMNI_UNSUPPORTED;
        t.first_block[i + 1] = t.first_block[i] + (t.job[i].total + 255) / 256;
    }
    return launch_pack_jobs(t, (hipStream_t)hip_stream);
}

int omni_conv_forward_packed(const omni_conv_desc *desc, const void *X, const void *packed, const float *bias, void *Y,
                             void *workspace, size_t workspace_bytes, void *hip_stream)
{
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    if (X == nullptr || packed == nullptr || Y == nullptr || workspace == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(X) || !aligned16(packed) || !aligned16(Y) || !aligned16(workspace) || (bias && !aligned16(bias)))
        return OMNI_MISALIGNED;
    size_t pbytes;
    if (!packed_weights_job(desc, g, OMNI_PASS_FORWARD, nullptr, nullptr, nullptr, &pbytes)) return OMNI_UNSUPPORTED;
    ForwardWs w;
    plan_forward(g, desc->dtype, &w);
    if (workspace_bytes < w.total) return OMNI_WORKSPACE_TOO_SMALL;
    return forward_on_scratch(desc, g, w, X, nullptr, bias, Y, (char *)workspace, workspace_bytes, (hipStream_t)hip_stream, packed);
}

int omni_conv_backward_data_packed(const omni_conv_desc *desc, const void *dY, const void *packed, void *dX, void *workspace,
                                   size_t workspace_bytes, void *hip_stream)
{
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    if (dY == nullptr || packed == nullptr || dX == nullptr || workspace == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(dY) || !aligned16(packed) || !aligned16(dX) || !aligned16(workspace)) return OMNI_MISALIGNED;
    size_t pbytes;
    if (!packed_weights_job(desc, g, OMNI_PASS_BACKWARD_DATA, nullptr, nullptr, nullptr, &pbytes)) return OMNI_UNSUPPORTED;
    BwdDataWs w;
    plan_backward_data(g, desc->dtype, &w);
    if (workspace_bytes < w.total) return OMNI_WORKSPACE_TOO_SMALL;
    if (fused_weight_bytes(g, true) > w.total) return OMNI_UNSUPPORTED;
    return launch_fused_conv(g, true, dY, nullptr, nullptr, 0, dX, workspace, (hipStream_t)hip_stream, -1, packed);
}

int omni_conv_backward_weights(const omni_conv_desc *desc, const void *X, const void *dY, float *dW, float *dbias,
                               void *workspace, size_t workspace_bytes, void *hip_stream)
{
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    bool cached = (desc->flags & OMNI_FLAG_DHAT_CACHED) != 0;
    if ((X == nullptr && !cached) || dY == nullptr || dW == nullptr || workspace == nullptr)
        return OMNI_INVALID_ARGUMENT;
    if ((X && !aligned16(X)) || !aligned16(dY) || !aligned16(dW) || !aligned16(workspace) ||
        (dbias && !aligned16(dbias)))
        return OMNI_MISALIGNED;
    BwdWeightsWs w;
    plan_backward_weights(g, desc->dtype, &w);
    if (workspace_bytes < w.total) return OMNI_WORKSPACE_TOO_SMALL;
    hipStream_t s = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    void *Dhat = ws + w.dhat, *dYhat = ws + w.dyhat;
    float *partials = (float *)(ws + w.partials), *bias_partials = (float *)(ws + w.bias_partials);

    if ((desc->flags & OMNI_FLAG_FUSED) && !cached && w.splits_patch > 0) {
        // 3 x 3 layer on small planes: dY as a plane-padded matrix, the lowered operand from an LDS copy of X
        st = launch_pack_dyhat_rows(g, dY, dYhat, w.ld_rows, dbias ? bias_partials : nullptr, w.bias_blocks_rows, nullptr, s);
        if (st != OMNI_OK) return st;
        st = launch_wgrad_patch(g, X, dYhat, w.ld_rows, partials, w.splits_patch, s);
        if (st != OMNI_OK) return st;
        return launch_wgrad_reduce(g, partials, w.splits_patch, dW, bias_partials, w.bias_blocks_rows, dbias, s);
    }
    if ((desc->flags & OMNI_FLAG_FUSED) && !cached && w.splits_wide > 0) {
        // 5-wide window: dY as a plane-padded matrix, the lowered operand from LDS copies of windows of X's planes
        st = launch_pack_dyhat_rows(g, dY, dYhat, w.ld_rows, dbias ? bias_partials : nullptr, w.bias_blocks_rows, nullptr, s);
        if (st != OMNI_OK) return st;
        return launch_wgrad_wide(g, X, dYhat, w.ld_rows, partials, w.splits_wide, dW, bias_partials, w.bias_blocks_rows, dbias, s);
    }
    const bool direct = (desc->flags & OMNI_FLAG_FUSED) && !cached && wgrad_direct_supported(g, desc->dtype);
    // with a split product the ordered reduction finishes the bias gradient too (one launch fewer)
    if (direct) {
        const bool defer = dbias != nullptr && w.splits_rows > 1;
        st = launch_pack_dyhat_rows(g, dY, dYhat, w.ld_rows, dbias ? bias_partials : nullptr, w.bias_blocks_rows,
                                    defer ? nullptr : dbias, s);
        if (st != OMNI_OK) return st;
        GemmWgradArgs a{dYhat, nullptr, w.ld_rows, partials, w.splits_rows, w.chunk_rows, dW, X,
                        bias_partials, w.bias_blocks_rows, defer ? dbias : nullptr};
        return launch_gemm_wgrad(g, desc->dtype, a, s);
    }
    if ((desc->flags & OMNI_FLAG_FUSED) && !cached && wgrad_phase_supported(g, desc->dtype)) {
        // stride-4 layer: X split into its four phase images; the product reads those and dY as they are
        st = launch_phase_split(g, wgrad_phase_wp(g), X, Dhat, s);
        if (st != OMNI_OK) return st;
        return launch_gemm_wgrad_phase(g, Dhat, dY, w.ld_rows, partials, w.splits_rows, w.chunk_rows, dW, dbias, s);
    }
    const bool defer = dbias != nullptr && w.splits > 1;
    st = launch_pack_dyhat(g, desc->dtype, dY, dYhat, w.ld, dbias ? bias_partials : nullptr, w.bias_blocks,
                           defer ? nullptr : dbias, s);
    if (st != OMNI_OK) return st;
    if (!cached) {  // after the packing: dY is usually fresh in the last-level cache, which D-hat would flush
        st = launch_lower(g, desc->dtype, X, Dhat, w.ld, s);
        if (st != OMNI_OK) return st;
    }
    GemmWgradArgs a{dYhat, Dhat, w.ld, partials, w.splits, w.chunk, dW, nullptr, bias_partials, w.bias_blocks,
                    defer ? dbias : nullptr};
    return launch_gemm_wgrad(g, desc->dtype, a, s);
}

// Whether the layer's model gradient reads dY in the rows form, and that form's extents.
static bool dy_rows_layout(const omni_conv_desc *desc, const ConvGeom &g, const BwdWeightsWs &w, int64_t *ld, int64_t *pitch)
{
    if (!(desc->flags & OMNI_FLAG_FUSED) || (desc->flags & OMNI_FLAG_DHAT_CACHED)) return false;
    if (w.splits_patch <= 0 && w.splits_wide <= 0) return false;
    const int64_t p = ((int64_t)g.Ho * g.Wo + 7) / 8 * 8;
    if (w.ld_rows != (int64_t)g.N * p) return false;  // no round-up at the rows' ends: every element belongs to a plane
    *ld = w.ld_rows, *pitch = p;
    return true;
}

int omni_conv_dy_rows_layout(const omni_conv_desc *desc, int64_t *ld, int64_t *plane_pitch)
{
    if (ld == nullptr || plane_pitch == nullptr) return OMNI_INVALID_ARGUMENT;
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    BwdWeightsWs w;
    plan_backward_weights(g, desc->dtype, &w);
    return dy_rows_layout(desc, g, w, ld, plane_pitch) ? OMNI_OK : OMNI_UNSUPPORTED;
}

int omni_conv_backward_weights_rows(const omni_conv_desc *desc, const void *X, const void *dY_rows, const float *plane_sums,
                                    int32_t sums_per_filter, float *dW, float *dbias, void *workspace, size_t workspace_bytes,
                                    void *hip_stream)
{
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    if (X == nullptr || dY_rows == nullptr || dW == nullptr || workspace == nullptr ||
        (dbias != nullptr && (plane_sums == nullptr || sums_per_filter <= 0)))
        return OMNI_INVALID_ARGUMENT;
    if (!aligned16(X) || !aligned16(dY_rows) || !aligned16(dW) || !aligned16(workspace) || (dbias && !aligned16(dbias)) ||
        (plane_sums && !aligned16(plane_sums)))
        return OMNI_MISALIGNED;
    BwdWeightsWs w;
    plan_backward_weights(g, desc->dtype, &w);
    int64_t ld, pitch;
    if (!dy_rows_layout(desc, g, w, &ld, &pitch)) return OMNI_UNSUPPORTED;
    if (workspace_bytes < w.total) return OMNI_WORKSPACE_TOO_SMALL;
    hipStream_t s = (hipStream_t)hip_stream;
    float *partials = (float *)((char *)workspace + w.partials);
    if (w.splits_patch > 0) {
        st = launch_wgrad_patch(g, X, dY_rows, ld, partials, w.splits_patch, s);
        if (st != OMNI_OK) return st;
        return launch_wgrad_reduce(g, partials, w.splits_patch, dW, plane_sums, sums_per_filter, dbias, s);
    }
    return launch_wgrad_wide(g, X, dY_rows, ld, partials, w.splits_wide, dW, plane_sums, sums_per_filter, dbias, s);
}

// the rows forms of both ends of a data gradient: checks shared by the two entry points below
static int backward_data_rows_checks(const omni_conv_desc *desc, ConvGeom *g, int64_t *ld, size_t workspace_bytes)
{
    int st = make_geom(desc, g);
    if (st != OMNI_OK) return st;
    size_t pbytes;
    if (!packed_weights_job(desc, *g, OMNI_PASS_BACKWARD_DATA, nullptr, nullptr, nullptr, &pbytes)) return OMNI_UNSUPPORTED;
    BwdWeightsWs ww;
    plan_backward_weights(*g, desc->dtype, &ww);
    int64_t pitch;
    if (!dy_rows_layout(desc, *g, ww, ld, &pitch)) return OMNI_UNSUPPORTED;
    BwdDataWs w;
    plan_backward_data(*g, desc->dtype, &w);
    if (workspace_bytes < w.total) return OMNI_WORKSPACE_TOO_SMALL;
    if (fused_weight_bytes(*g, true) > w.total) return OMNI_UNSUPPORTED;
    return OMNI_OK;
}

int omni_conv_backward_data_rows(const omni_conv_desc *desc, const void *dY_rows, const void *packed, void *dX, void *workspace,
                                 size_t workspace_bytes, void *hip_stream)
{
    if (dY_rows == nullptr || packed == nullptr || dX == nullptr || workspace == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(dY_rows) || !aligned16(packed) || !aligned16(dX) || !aligned16(workspace)) return OMNI_MISALIGNED;
    ConvGeom g;
    int64_t ld;
    int st = backward_data_rows_checks(desc, &g, &ld, workspace_bytes);
    if (st != OMNI_OK) return st;
    FusedIO io{ld, nullptr, 0, nullptr};
    return launch_fused_conv(g, true, dY_rows, nullptr, nullptr, 0, dX, workspace, (hipStream_t)hip_stream, -1, packed, &io);
}

int omni_conv_backward_data_relu_rows_sums(const omni_conv_desc *desc, int32_t *sums_per_channel)
{
    if (sums_per_channel == nullptr) return OMNI_INVALID_ARGUMENT;
    ConvGeom g;
    int64_t ld;
    int st = backward_data_rows_checks(desc, &g, &ld, (size_t)-1);
    if (st != OMNI_OK) return st;
    const int tiles = fused_column_tiles(g, true);
    if (tiles <= 0) return OMNI_UNSUPPORTED;
    *sums_per_channel = tiles;
    return OMNI_OK;
}

int omni_conv_backward_data_relu_rows(const omni_conv_desc *desc, const void *dY_rows, const void *packed, const void *y_front,
                                      void *dX_rows, int64_t ld_out, float *col_sums, void *workspace, size_t workspace_bytes,
                                      void *hip_stream)
{
    if (dY_rows == nullptr || packed == nullptr || y_front == nullptr || dX_rows == nullptr || workspace == nullptr)
        return OMNI_INVALID_ARGUMENT;
    if (!aligned16(dY_rows) || !aligned16(packed) || !aligned16(y_front) || !aligned16(dX_rows) || !aligned16(workspace) ||
        (col_sums && !aligned16(col_sums)))
        return OMNI_MISALIGNED;
    ConvGeom g;
    int64_t ld;
    int st = backward_data_rows_checks(desc, &g, &ld, workspace_bytes);
    if (st != OMNI_OK) return st;
    if (fused_column_tiles(g, true) <= 0) return OMNI_UNSUPPORTED;
    if (ld_out % 8 != 0 || ld_out < (int64_t)g.N * (((int64_t)g.H * g.W + 7) / 8 * 8)) return OMNI_INVALID_ARGUMENT;
    FusedIO io{ld, y_front, ld_out, col_sums};
    return launch_fused_conv(g, true, dY_rows, nullptr, nullptr, 0, dX_rows, workspace, (hipStream_t)hip_stream, -1, packed, &io);
}

int omni_sgd_momentum_step(int32_t n_tensors, float *const *W, float *const *V, const float *const *G,
                           const int64_t *counts, void *const *W_shadow, float lr, float momentum, float weight_decay,
                           void *hip_stream)
{
    if (n_tensors < 0) return OMNI_INVALID_ARGUMENT;
    if (n_tensors == 0) return OMNI_OK;
    if (W == nullptr || V == nullptr || G == nullptr || counts == nullptr) return OMNI_INVALID_ARGUMENT;
    for (int32_t i = 0; i < n_tensors; ++i) {
        if (counts[i] < 0) return OMNI_INVALID_ARGUMENT;
        if (counts[i] == 0) continue;
        if (W[i] == nullptr || V[i] == nullptr || G[i] == nullptr) return OMNI_INVALID_ARGUMENT;
        if (!aligned16(W[i]) || !aligned16(V[i]) || !aligned16(G[i]) || (W_shadow && W_shadow[i] && !aligned16(W_shadow[i])))
            return OMNI_MISALIGNED;
    }
    return launch_sgd(n_tensors, W, V, G, counts, W_shadow, lr, momentum, weight_decay, (hipStream_t)hip_stream);
}

int omni_lower(const omni_conv_desc *desc, const void *X, void *Dhat, int64_t ld, void *hip_stream)
{
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    if (X == nullptr || Dhat == nullptr || ld < g.M) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(X) || !aligned16(Dhat)) return OMNI_MISALIGNED;
    return launch_lower(g, desc->dtype, X, Dhat, ld, (hipStream_t)hip_stream);
}

int omni_col2im(const omni_conv_desc *desc, const void *dDhat, int64_t ld, void *dX, void *hip_stream)
{
    ConvGeom g;
    int st = make_geom(desc, &g);
    if (st != OMNI_OK) return st;
    if (dDhat == nullptr || dX == nullptr || ld < g.M) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(dDhat) || !aligned16(dX)) return OMNI_MISALIGNED;
    return launch_col2im(g, desc->dtype, dDhat, ld, dX, (hipStream_t)hip_stream);
}

static int check_dtype(int32_t dtype) { return (dtype == OMNI_F32 || dtype == OMNI_BF16) ? OMNI_OK : OMNI_UNSUPPORTED; }

int omni_relu_forward(int32_t dtype, int64_t count, const void *x, void *y, void *hip_stream)
{
    if (check_dtype(dtype) != OMNI_OK) return OMNI_UNSUPPORTED;
    if (count < 0) return OMNI_INVALID_ARGUMENT;
    if (count == 0) return OMNI_OK;
    if (x == nullptr || y == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(x) || !aligned16(y)) return OMNI_MISALIGNED;
    return launch_relu(dtype, false, count, x, nullptr, y, (hipStream_t)hip_stream);
}

int omni_relu_backward(int32_t dtype, int64_t count, const void *y, const void *dy, void *dx, void *hip_stream)
{
    if (check_dtype(dtype) != OMNI_OK) return OMNI_UNSUPPORTED;
    if (count < 0) return OMNI_INVALID_ARGUMENT;
    if (count == 0) return OMNI_OK;
    if (y == nullptr || dy == nullptr || dx == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(y) || !aligned16(dy) || !aligned16(dx)) return OMNI_MISALIGNED;
    return launch_relu(dtype, true, count, y, dy, dx, (hipStream_t)hip_stream);
}

int omni_relu_backward_rows(int32_t dtype, int32_t N, int32_t C, int64_t plane, const void *y, const void *dy, void *dx_rows,
                            int64_t ld, float *plane_sums, void *hip_stream)
{
    if (dtype != OMNI_BF16) return OMNI_UNSUPPORTED;
    if (N < 0 || C <= 0 || plane <= 0) return OMNI_INVALID_ARGUMENT;
    if (!relu_bwd_rows_supported(N, C, plane)) return OMNI_UNSUPPORTED;
    if (ld % 8 != 0 || ld < (int64_t)N * ((plane + 7) / 8 * 8)) return OMNI_INVALID_ARGUMENT;
    if (N == 0) return OMNI_OK;
    if (y == nullptr || dy == nullptr || dx_rows == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(y) || !aligned16(dy) || !aligned16(dx_rows) || (plane_sums && !aligned16(plane_sums))) return OMNI_MISALIGNED;
    return launch_relu_bwd_rows(N, C, plane, y, dy, dx_rows, ld, plane_sums, (hipStream_t)hip_stream);
}

int omni_pool_output_dim(int32_t in, int32_t k, int32_t stride, int32_t ceil_mode)
{
    if (in <= 0 || k <= 0 || stride <= 0 || in < k) return OMNI_INVALID_ARGUMENT;
    int32_t span = in - k;
    return (ceil_mode ? (span + stride - 1) / stride : span / stride) + 1;
}

static int check_pool(int32_t dtype, int64_t planes, int32_t H, int32_t W, int32_t k, int32_t stride)
{
    if (check_dtype(dtype) != OMNI_OK) return OMNI_UNSUPPORTED;
    if (planes < 0 || H <= 0 || W <= 0 || k <= 0 || stride <= 0 || H < k || W < k) return OMNI_INVALID_ARGUMENT;
    if (k > 15) return OMNI_UNSUPPORTED;  // the winner's window position is stored in one byte
    if ((int64_t)H * W > 0x7fffffffll - 4096) return OMNI_UNSUPPORTED;
    return OMNI_OK;
}

int omni_maxpool_forward(int32_t dtype, int64_t planes, int32_t H, int32_t W, int32_t k, int32_t stride,
                         int32_t ceil_mode, const void *x, void *y, uint8_t *argmax, void *hip_stream)
{
    int st = check_pool(dtype, planes, H, W, k, stride);
    if (st != OMNI_OK) return st;
    if (planes == 0) return OMNI_OK;
    if (x == nullptr || y == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(x) || !aligned16(y)) return OMNI_MISALIGNED;
    return launch_maxpool_fwd(dtype, planes, H, W, k, stride, ceil_mode, x, y, argmax, (hipStream_t)hip_stream);
}

int omni_maxpool_backward(int32_t dtype, int64_t planes, int32_t H, int32_t W, int32_t k, int32_t stride,
                          int32_t ceil_mode, const void *dy, const uint8_t *argmax, void *dx, void *hip_stream)
{
    int st = check_pool(dtype, planes, H, W, k, stride);
    if (st != OMNI_OK) return st;
    if (planes == 0) return OMNI_OK;
    if (dy == nullptr || argmax == nullptr || dx == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(dy) || !aligned16(dx)) return OMNI_MISALIGNED;
    return launch_maxpool_bwd(dtype, planes, H, W, k, stride, ceil_mode, dy, argmax, nullptr, dx, (hipStream_t)hip_stream);
}

int omni_maxpool_relu_backward(int32_t dtype, int64_t planes, int32_t H, int32_t W, int32_t k, int32_t stride,
                               int32_t ceil_mode, const void *dy, const uint8_t *argmax, const void *y, void *dx,
                               void *hip_stream)
{
    int st = check_pool(dtype, planes, H, W, k, stride);
    if (st != OMNI_OK) return st;
    if (planes == 0) return OMNI_OK;
    if (dy == nullptr || argmax == nullptr || y == nullptr || dx == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(dy) || !aligned16(y) || !aligned16(dx)) return OMNI_MISALIGNED;
    return launch_maxpool_bwd(dtype, planes, H, W, k, stride, ceil_mode, dy, argmax, y, dx, (hipStream_t)hip_stream);
}

int omni_maxpool_backward_rows(int32_t dtype, int32_t N, int32_t C, int32_t H, int32_t W, int32_t k, int32_t stride,
                               int32_t ceil_mode, const void *dy, const uint8_t *argmax, const void *y, void *dx_rows,
                               int64_t ld, float *plane_sums, void *hip_stream)
{
    if (N < 0 || C <= 0) return OMNI_INVALID_ARGUMENT;
    int st = check_pool(dtype, (int64_t)N * C, H, W, k, stride);
    if (st != OMNI_OK) return st;
    if (dtype != OMNI_BF16 || !maxpool_bwd_rows_supported(N > 0 ? N : 1, C, H, W, k, stride, ceil_mode)) return OMNI_UNSUPPORTED;
    if (ld % 8 != 0 || ld < (int64_t)N * (((int64_t)H * W + 7) / 8 * 8)) return OMNI_INVALID_ARGUMENT;
    if (N == 0) return OMNI_OK;
    if (dy == nullptr || argmax == nullptr || dx_rows == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(dy) || !aligned16(dx_rows) || (y && !aligned16(y)) || (plane_sums && !aligned16(plane_sums)))
        return OMNI_MISALIGNED;
    return launch_maxpool_bwd_rows(N, C, H, W, k, stride, ceil_mode, dy, argmax, y, dx_rows, ld, plane_sums,
                                   (hipStream_t)hip_stream);
}

static int check_lrn(int32_t dtype, int64_t N, int32_t C, int64_t plane, int32_t size, float alpha, float beta, float k)
{
    if (check_dtype(dtype) != OMNI_OK) return OMNI_UNSUPPORTED;
    if (N < 0 || C <= 0 || plane <= 0 || size <= 0 || !(k > 0.f) || !(alpha >= 0.f) || !(beta >= 0.f)) return OMNI_INVALID_ARGUMENT;
    if (size % 2 != 1 || size > 9) return OMNI_UNSUPPORTED;  // symmetric window, held in registers
    if (plane > 0x7fffffffll - 4096 || (double)N * (double)plane > 2147479551.0) return OMNI_UNSUPPORTED;
    return OMNI_OK;
}

int omni_lrn_forward(int32_t dtype, int64_t N, int32_t C, int64_t plane, int32_t size, float alpha, float beta, float k,
                     const void *x, void *y, float *scale, void *hip_stream)
{
    int st = check_lrn(dtype, N, C, plane, size, alpha, beta, k);
    if (st != OMNI_OK) return st;
    if (N == 0) return OMNI_OK;
    if (x == nullptr || y == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(x) || !aligned16(y) || (scale && !aligned16(scale))) return OMNI_MISALIGNED;
    return launch_lrn(dtype, false, N, C, plane, size, alpha, beta, k, x, nullptr, scale, y, (hipStream_t)hip_stream);
}

int omni_lrn_backward(int32_t dtype, int64_t N, int32_t C, int64_t plane, int32_t size, float alpha, float beta, float k,
                      const void *x, const void *dy, const float *scale, void *dx, void *hip_stream)
{
    int st = check_lrn(dtype, N, C, plane, size, alpha, beta, k);
    if (st != OMNI_OK) return st;
    if (N == 0) return OMNI_OK;
    if (x == nullptr || dy == nullptr || scale == nullptr || dx == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(scale) || !aligned16(dx)) return OMNI_MISALIGNED;
    return launch_lrn(dtype, true, N, C, plane, size, alpha, beta, k, x, dy, const_cast<float *>(scale), dx,
                      (hipStream_t)hip_stream);
}

// floor(p * 2^32), at most 2^32 - 1: an element is kept iff its 32-bit draw is at least this
static uint32_t dropout_threshold(float p)
{
    double t = floor((double)p * 4294967296.0);
    return t > 4294967295.0 ? 4294967295u : (uint32_t)t;
}

static int dropout_call(int32_t dtype, int64_t count, float p, uint64_t seed, uint64_t stream_id, const void *in, void *out,
                        void *hip_stream)
{
    if (check_dtype(dtype) != OMNI_OK) return OMNI_UNSUPPORTED;
    if (count < 0 || !(p >= 0.f) || !(p < 1.f)) return OMNI_INVALID_ARGUMENT;
    if (count == 0) return OMNI_OK;
    if (in == nullptr || out == nullptr) return OMNI_INVALID_ARGUMENT;
    if (!aligned16(in) || !aligned16(out)) return OMNI_MISALIGNED;
    return launch_dropout(dtype, count, dropout_threshold(p), 1.0f / (1.0f - p), seed, stream_id, in, out,
                          (hipStream_t)hip_stream);
}

int omni_dropout_forward(int32_t dtype, int64_t count, float p, uint64_t seed, uint64_t stream_id, const void *x, void *y,
                         void *hip_stream)
{
    return dropout_call(dtype, count, p, seed, stream_id, x, y, hip_stream);
}

int omni_dropout_backward(int32_t dtype, int64_t count, float p, uint64_t seed, uint64_t stream_id, const void *dy, void *dx,
                          void *hip_stream)
{
    return dropout_call(dtype, count, p, seed, stream_id, dy, dx, hip_stream);
}

}  // extern "C"
