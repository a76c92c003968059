// Internal declarations shared by the HIP sources of the library (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "omniconv.h"

namespace omni {

typedef uint16_t bf16_t;  // raw bf16 bit pattern

// ---------------------------------------------------------------- bf16 <-> fp32, device side
__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// Round to nearest, ties to even; NaN stays a (quiet) NaN.  gfx950 converts in hardware
// (v_cvt_pk_bf16_f32, two values per instruction), which is what the casts below compile to.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }

// (lo, hi) -> two bf16 in one 32-bit word, lo in bits 0..15
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi)
{
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
    static __device__ __forceinline__ float to_f32(float v) { return v; }
    static __device__ __forceinline__ float from_f32(float v) { return v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float to_f32(bf16_t v) { return bf16_to_f32(v); }
    static __device__ __forceinline__ bf16_t from_f32(float v) { return f32_to_bf16(v); }
};

// ---------------------------------------------------------------- division by a run-time constant
// q = n / d for 0 <= n < 2^31 and 1 <= d < 2^31 as a multiply-high, an add and a shift
// (the round-up method of Granlund & Montgomery); the multiplier is computed once on the host.
struct FastDiv {
    uint32_t d, mul, shift;
    FastDiv() : d(1), mul(0), shift(0) {}
    explicit FastDiv(uint32_t div) : d(div)
    {
        shift = 0;
        while ((1ull << shift) < div) ++shift;
        mul = (uint32_t)((((1ull << shift) - div) << 32) / div + 1);
    }
    __host__ __device__ __forceinline__ uint32_t div(uint32_t n) const
    {
#if defined(__HIP_DEVICE_COMPILE__)
        return (__umulhi(n, mul) + n) >> shift;
#else
        return (uint32_t)((((uint64_t)n * mul) >> 32) + n) >> shift;
#endif
    }
    __host__ __device__ __forceinline__ void divmod(uint32_t n, uint32_t &q, uint32_t &r) const
    {
        q = div(n);
        r = n - q * d;
    }
};

// ---------------------------------------------------------------- geometry of one layer
struct ConvGeom {
    int32_t N, C, H, W, F, kh, kw, sh, sw, ph, pw, Ho, Wo;
    int32_t K;     // C*kh*kw   rows of D-hat
    int32_t M;     // N*Ho*Wo   columns of D-hat
    int32_t HoWo;  // Ho*Wo
    uint32_t flags;  // the descriptor's OMNI_FLAG_* bits
    FastDiv div_Wo, div_HoWo, div_kw, div_khkw, div_W, div_HW, div_sh, div_sw;
};

inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

// Host-side checks; fill `g` from a descriptor.  Pure host code (no HIP calls).
int make_geom(const omni_conv_desc *desc, ConvGeom *g);

// Leading dimension of D-hat / dY-hat inside a workspace.
// A multiple of 64 so that a reduction along M can be walked in whole steps without a ragged tail.
inline int64_t dhat_ld(const ConvGeom &g) { return round_up(g.M, 64); }

// ---------------------------------------------------------------- workspace carving
// splits > 1 (OMNI_FLAG_SPLIT_K): the reduction is cut into `splits` chunks of `chunk` whose fp32 partial
// results [splits][rows][ld] live at `partials`
// explicit_total: what lowering + GEMM alone need (total also covers the fused kernels' repacked weights)
struct ForwardWs { size_t dhat, khat, partials, total, explicit_total; int64_t ld, Fp, Kp; int splits; int64_t chunk; };
struct BwdDataWs { size_t ddhat, dyhat, khat_t, partials, total; int64_t ld, Kp, Fp; int splits; int64_t chunk; };
// *_rows: the same plan for the row-padded dY-hat of the direct model gradient (reduction extent ld_rows)
struct BwdWeightsWs {
    size_t dhat, dyhat, partials, bias_partials, total;  // dhat also holds X4 of the phase-split model gradient
    int64_t ld; int splits; int64_t chunk; int bias_blocks;
    int64_t ld_rows; int splits_rows; int64_t chunk_rows; int bias_blocks_rows;
    int splits_patch;  // > 0: the layer's fused model gradient is wgrad_patch.hip's, over this many image ranges
    int splits_wide;   // > 0: ... is wgrad_wide.hip's, over this many ranges of stages
};
void plan_forward(const ConvGeom &g, int dtype, ForwardWs *w);
void plan_backward_data(const ConvGeom &g, int dtype, BwdDataWs *w);
void plan_backward_weights(const ConvGeom &g, int dtype, BwdWeightsWs *w);

inline size_t elem_size(int dtype) { return dtype == OMNI_BF16 ? 2 : 4; }

#define OMNI_LAUNCH_CHECK()                                   \
    do {                                                      \
        if (hipGetLastError() != hipSuccess) return OMNI_HIP_ERROR; \
    } while (0)

// ---------------------------------------------------------------- optional event timing (profile.hip)
enum KernelId {
    KID_LOWER = 0, KID_PACK_KHAT, KID_PACK_DYHAT, KID_BIAS_REDUCE, KID_GEMM_FWD, KID_GEMM_DGRAD, KID_GEMM_WGRAD,
    KID_REDUCE_PARTIALS, KID_COL2IM, KID_SGD, KID_RELU, KID_POOL_FWD, KID_POOL_BWD, KID_FUSED_FWD, KID_FUSED_DGRAD, KID_STRIDED_FWD,
    KID_LRN, KID_DROPOUT,
    KID_COUNT
};
// Brackets the launches made during its lifetime with two events on `s` when profiling is on.
// flops / bytes are the algorithmic work of the bracketed launch.
class ProfScope {
  public:
    ProfScope(int kernel_id, hipStream_t s, double flops, double bytes);
    ~ProfScope();
    ProfScope(const ProfScope &) = delete;
    ProfScope &operator=(const ProfScope &) = delete;

  private:
    long slot_;
    hipStream_t stream_;
};

// ---------------------------------------------------------------- launchers (one per source file)
// lowering.hip
int launch_lower(const ConvGeom &g, int dtype, const void *X, void *Dhat, int64_t ld, hipStream_t s);
int launch_col2im(const ConvGeom &g, int dtype, const void *dDhat, int64_t ld, void *dX, hipStream_t s);
int launch_pack_khat(const ConvGeom &g, int dtype, const void *W, void *Khat, int64_t Fp, int64_t Kp, hipStream_t s);
int launch_pack_khat_t(const ConvGeom &g, int dtype, const void *W, void *KhatT, int64_t Kp, int64_t Fp, hipStream_t s);
// dY [N][F][Ho][Wo] -> dY-hat [F][ld]; if bias_partials != null also writes per-block sums
// [F][bias_blocks] and then reduces them into dbias.
// (dbias == null with bias_partials != null: the per-block sums are left for the caller to reduce)
int launch_pack_dyhat(const ConvGeom &g, int dtype, const void *dY, void *dYhat, int64_t ld,
                      float *bias_partials, int bias_blocks, float *dbias, hipStream_t s);
int pack_dyhat_blocks(const ConvGeom &g);
// row-padded variant (bf16): every output row padded to a multiple of 8 columns
int64_t dyhat_rows_ld(const ConvGeom &g);
int pack_dyhat_rows_blocks(const ConvGeom &g);
int launch_pack_dyhat_rows(const ConvGeom &g, const void *dY, void *dYhat, int64_t ld, float *bias_partials,
                           int bias_blocks, float *dbias, hipStream_t s);

// gemm.hip
// splits > 1: partial products into `partials`, then the ordered sum with the epilogue
struct GemmFwdArgs { const void *Khat; int64_t ldk; const void *Dhat; int64_t ldd; const float *bias; void *Y; int relu; float *partials; int splits; int64_t chunk; };
int launch_gemm_forward(const ConvGeom &g, int dtype, const GemmFwdArgs &a, hipStream_t s);
struct GemmDgradArgs { const void *KhatT; int64_t ldk; const void *dYhat; int64_t ldd; void *dDhat; float *partials; int splits; int64_t chunk; };
int launch_gemm_dgrad(const ConvGeom &g, int dtype, const GemmDgradArgs &a, hipStream_t s);
// whole-image windows (fully connected layers): one product on the tensors as they are
bool dgrad_dense_supported(const ConvGeom &g);
int launch_gemm_dgrad_dense(const ConvGeom &g, int dtype, const void *dY, const void *W, void *dX, float *partials,
                            int splits, int64_t chunk, hipStream_t s);
// X_direct != null: D-hat is not in memory, its entries are read from X (wgrad_direct_supported layers)
// dbias != null (only with splits > 1): the ordered reduction also finishes the bias gradient from bias_partials
struct GemmWgradArgs { const void *dYhat; const void *Dhat; int64_t ldd; float *partials; int splits; int64_t chunk; float *dW; const void *X_direct;
                       const float *bias_partials; int bias_blocks; float *dbias; };
int launch_gemm_wgrad(const ConvGeom &g, int dtype, const GemmWgradArgs &a, hipStream_t s);
bool wgrad_direct_supported(const ConvGeom &g, int dtype);
bool wgrad_direct_planes(const ConvGeom &g);  // its padded unit is the image plane, not the output row
int gemm_red_tile(int dtype);  // reduction extent of one LDS tile (elements)
void gemm_wgrad_tile(int F, int K, int *bm, int *bn);
void gemm_split_tile(int rows, int cols, int *bm, int *bn);  // tile of a split forward / data-gradient product

// implicit.hip: the convolution with lowering (forward) or col2im (data gradient) fused into the matrix
// product; bf16, stride 1, shapes whose column tiles fit the kernel's LDS patch.  wt_scratch receives the
// repacked weights (fused_weight_bytes).
bool fused_supported(const ConvGeom &g, int dtype, bool data_gradient);
size_t fused_weight_bytes(const ConvGeom &g, bool data_gradient);
// Optional forms of the fused kernel's operands: in_ld > 0 = the input is given in its rows form [C][in_ld] (plane of
// image n at column n * (plane rounded up to 8)) instead of the dense tensor; mask != null = the output goes out in
// the rows form as well (leading dimension out_ld), zero where the dense tensor mask [N][F][Ho][Wo] is not positive,
// and col_sums [F][fused_column_tiles] (nullable) receives the sums of what every column tile stored per row.
struct FusedIO { int64_t in_ld; const void *mask; int64_t out_ld; float *col_sums; };
int fused_column_tiles(const ConvGeom &g, bool data_gradient);  // 0: not fused, or the reduction is split
// kid: kernel class the launch is timed under (-1: by data_gradient)
int launch_fused_conv(const ConvGeom &g, bool data_gradient, const void *X, const void *W, const float *bias,
                      int relu, void *Y, void *wt_scratch, hipStream_t s, int kid = -1, const void *prepacked = nullptr,
                      const FusedIO *io = nullptr);

// strided.hip: the forward convolution of a layer with horizontal stride 4, no padding, at most 96 filters and
// a short reduction (CaffeNet's conv1) without D-hat; bf16.  wt_scratch receives the repacked weights.
bool strided_supported(const ConvGeom &g, int dtype);
size_t strided_weight_bytes(const ConvGeom &g);
int launch_strided_conv(const ConvGeom &g, const void *X, const void *W, const float *bias, int relu, void *Y,
                        void *wt_scratch, hipStream_t s, const void *prepacked = nullptr);

// Data gradient of a strided, unpadded layer as one stride-1 convolution over dY with C*sh*sw output channels
// (run by the fused kernel of implicit.hip) plus the interleaving of the phase images into dX; bf16.
// `workspace` needs strided_dgrad_bytes().
bool strided_dgrad_supported(const ConvGeom &g, int dtype);
size_t strided_dgrad_bytes(const ConvGeom &g);
int launch_strided_dgrad(const ConvGeom &g, const void *dY, const void *W, void *dX, void *workspace, hipStream_t s);

// The model gradient of such a layer without D-hat: phase_split writes X4 [N][4C][H][WP] (strided.hip), the
// product reads its lowered operand from X4 and its other operand from dY itself (gemm.hip); the bias
// gradient comes out of the same product.
bool wgrad_phase_supported(const ConvGeom &g, int dtype);
int wgrad_phase_kp(const ConvGeom &g);  // columns of the phase-ordered gradient [F][K']
int wgrad_phase_wp(const ConvGeom &g);  // row pitch of X4 in elements
int launch_phase_split(const ConvGeom &g, int WP, const void *X, void *X4, hipStream_t s);
int launch_gemm_wgrad_phase(const ConvGeom &g, const void *X4, const void *dY, int64_t ld, float *partials, int splits,
                            int64_t chunk, float *dW, float *dbias, hipStream_t s);

// wgrad_patch.hip: the model gradient of a 3 x 3, stride-1, same-size layer on small planes (bf16) with the
// lowered operand read from an LDS copy of the input planes; dY-hat in the plane-padded layout of
// launch_pack_dyhat_rows, partial sums [splits][F][K] (splits = wgrad_patch_splits) for launch_wgrad_reduce.
bool wgrad_patch_supported(const ConvGeom &g, int dtype);
int wgrad_patch_splits(const ConvGeom &g);
int launch_wgrad_patch(const ConvGeom &g, const void *X, const void *dYhat, int64_t ld, float *partials, int splits,
                       hipStream_t s);
// wgrad_wide.hip: the same for a 5-wide window on planes too large for LDS (one window row per workgroup, stages of
// 128 positions); partial sums [splits][kh][F][C][kw], added in order by its own reduction (with the bias gradient)
bool wgrad_wide_supported(const ConvGeom &g, int dtype);
int wgrad_wide_splits(const ConvGeom &g);
int launch_wgrad_wide(const ConvGeom &g, const void *X, const void *dYhat, int64_t ld, float *partials, int splits, float *dW,
                      const float *bias_partials, int bias_blocks, float *dbias, hipStream_t s);
void set_wgrad_wide_override(int max_splits, int off);
// gemm.hip: ordered sum of the split partial results [splits][F][K] into dW; with dbias != null the same launch
// finishes the bias gradient from the per-block sums of the dY packing kernel
int launch_wgrad_reduce(const ConvGeom &g, const float *partials, int splits, float *dW, const float *bias_partials,
                        int bias_blocks, float *dbias, hipStream_t s);

// tile overrides for sweeps (omni_tuning_set); -1 leaves a value as it is
void set_gemm_tile_override(int tile);
void set_fused_tile_override(int bn, int bm);
void set_fused_pitch_override(int bare);
void set_wgrad_patch_override(int max_splits, int off);

// elementwise.hip
int launch_sgd(int32_t n, float *const *W, float *const *V, const float *const *G, const int64_t *counts,
               void *const *shadow, float lr, float mu, float wd, hipStream_t s);
int launch_relu(int dtype, bool backward, int64_t count, const void *ref, const void *dy, void *out, hipStream_t s);
int launch_maxpool_fwd(int dtype, int64_t planes, int32_t H, int32_t W, int32_t k, int32_t stride, int32_t ceil_mode,
                       const void *x, void *y, uint8_t *argmax, hipStream_t s);
int launch_maxpool_bwd(int dtype, int64_t planes, int32_t H, int32_t W, int32_t k, int32_t stride, int32_t ceil_mode,
                       const void *dy, const uint8_t *argmax, const void *y, void *dx, hipStream_t s);
void set_pool_override(int lds);  // omni_tuning_set(OMNI_TUNE_POOL_LDS)
// The two producers of a layer's output gradient writing its "rows" form directly (bf16): a matrix [C][ld], plane
// (n, c) at column n * pitch with pitch = the plane rounded up to 8 elements (the round-up zero), plus the sum of
// every plane's values, plane_sums [C][N] (optional).  Columns from N * pitch to ld are not written.
bool maxpool_bwd_rows_supported(int32_t N, int32_t C, int32_t H, int32_t W, int32_t k, int32_t stride, int32_t ceil_mode);
int launch_maxpool_bwd_rows(int32_t N, int32_t C, int32_t H, int32_t W, int32_t k, int32_t stride, int32_t ceil_mode,
                            const void *dy, const uint8_t *argmax, const void *y, void *dx_rows, int64_t ld, float *plane_sums,
                            hipStream_t s);
bool relu_bwd_rows_supported(int32_t N, int32_t C, int64_t plane);
int launch_relu_bwd_rows(int32_t N, int32_t C, int64_t plane, const void *y, const void *dy, void *dx_rows, int64_t ld,
                         float *plane_sums, hipStream_t s);

// normdrop.hip: normalisation across channels (x, dy, out [N][C][plane]; scale fp32, same shape) and dropout
int launch_lrn(int dtype, bool backward, int64_t N, int32_t C, int64_t plane, int32_t size, float alpha, float beta, float k,
               const void *x, const void *dy, float *scale, void *out, hipStream_t s);
int launch_dropout(int dtype, int64_t count, uint32_t threshold, float scale, uint64_t seed, uint64_t stream_id, const void *x,
                   void *y, hipStream_t s);

}  // namespace omni
