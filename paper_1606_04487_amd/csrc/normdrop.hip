// Local response normalisation across channels and dropout (gfx950): the remaining non-GEMM layers of the
// paper's CaffeNet runs (App. C, "Data Parallelism in non-GEMM Kernels").  Both are bound by HBM traffic and
// data-parallel over the batch; the grid over (image, pixel) resp. over blocks of eight elements is that
// partitioning.
#include "common.h"

namespace omni {

template <typename T> __device__ __forceinline__ float ld_f32(const T *p);
template <> __device__ __forceinline__ float ld_f32<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ld_f32<bf16_t>(const bf16_t *p) { return bf16_to_f32(*p); }
template <typename T> __device__ __forceinline__ void st_f32(T *p, float v);
template <> __device__ __forceinline__ void st_f32<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void st_f32<bf16_t>(bf16_t *p, float v) { *p = f32_to_bf16(v); }

// ------------------------------------------------------------------------------------------------
// Normalisation: s = k + alpha/size * sum_{|c'-c| <= size/2} x[c']^2,  y = x * s^-beta.
// One thread per (image, pixel, block of LRN_CB channels) walks its channels; consecutive threads hold
// consecutive pixels, so every access of a wavefront is one contiguous run of a channel plane.  The window's
// squares live in registers (a shift register of HALF*2+1 values), so x is read once plus the block's halo.
// s is optionally stored (fp32) for the backward pass, which needs it at every channel of the window.
// s^-beta = exp2(-beta * log2(s)) on the hardware's exp2 / log2 units (s >= k > 0).
// ------------------------------------------------------------------------------------------------
constexpr int LRN_CB = 8;  // channels per thread

__device__ __forceinline__ float pow_neg(float s, float beta) { return __builtin_amdgcn_exp2f(-beta * __builtin_amdgcn_logf(s)); }

template <typename T, int HALF>
__global__ __launch_bounds__(256) void lrn_forward_kernel(const T *__restrict__ x, T *__restrict__ y, float *__restrict__ scale,
                                                          int64_t pixels, int32_t C, int64_t plane, FastDiv div_plane,
                                                          float alpha_over_size, float beta, float k)
{
    int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= pixels) return;
    uint32_t n, p;
    div_plane.divmod((uint32_t)t, n, p);
    const int64_t base = (int64_t)n * C * plane + p;
    float sq[2 * HALF + 1], xv[HALF + 1];  // squares of channels c-HALF .. c+HALF; values of c .. c+HALF
#pragma unroll
    for (int j = 0; j < 2 * HALF + 1; ++j) sq[j] = 0.f;
#pragma unroll
    for (int j = 0; j <= HALF; ++j) xv[j] = 0.f;
    // preload channels c0 - HALF .. c0 + HALF - 1: the window of channel c0 minus its newest member
    const int c0 = blockIdx.y * LRN_CB, c1 = c0 + LRN_CB < C ? c0 + LRN_CB : C;
#pragma unroll
    for (int j = 0; j < 2 * HALF; ++j) {
        int cc = c0 - HALF + j;
        float v = (cc >= 0 && cc < C) ? ld_f32(x + base + (int64_t)cc * plane) : 0.f;
        sq[j + 1] = v * v;
        if (j >= HALF) xv[j - HALF + 1] = v;
    }
    for (int c = c0; c < c1; ++c) {
        // shift the window by one channel and take in channel c + HALF
#pragma unroll
        for (int j = 0; j < 2 * HALF; ++j) sq[j] = sq[j + 1];
#pragma unroll
        for (int j = 0; j < HALF; ++j) xv[j] = xv[j + 1];
        float v = c + HALF < C ? ld_f32(x + base + (int64_t)(c + HALF) * plane) : 0.f;
        xv[HALF] = v;
        sq[2 * HALF] = v * v;
        float acc = 0.f;
#pragma unroll
        for (int j = 0; j < 2 * HALF + 1; ++j) acc += sq[j];
        float s = k + alpha_over_size * acc;
        if (scale != nullptr) scale[base + (int64_t)c * plane] = s;
        st_f32(y + base + (int64_t)c * plane, xv[0] * pow_neg(s, beta));
    }
}

// dx[c] = dy[c] * s[c]^-beta - (2 alpha beta / size) * x[c] * sum_{|c'-c| <= HALF} dy[c'] x[c'] s[c']^(-beta-1)
// Same walk; the window now holds r[c'] = dy[c'] x[c'] s[c']^(-beta-1).
template <typename T, int HALF>
__global__ __launch_bounds__(256) void lrn_backward_kernel(const T *__restrict__ x, const T *__restrict__ dy,
                                                           const float *__restrict__ scale, T *__restrict__ dx, int64_t pixels,
                                                           int32_t C, int64_t plane, FastDiv div_plane, float coef, float beta)
{
    int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= pixels) return;
    uint32_t n, p;
    div_plane.divmod((uint32_t)t, n, p);
    const int64_t base = (int64_t)n * C * plane + p;
    float r[2 * HALF + 1], xv[HALF + 1], own[HALF + 1];  // own[j] = dy * s^-beta of channel c + j
#pragma unroll
    for (int j = 0; j < 2 * HALF + 1; ++j) r[j] = 0.f;
#pragma unroll
    for (int j = 0; j <= HALF; ++j) xv[j] = 0.f, own[j] = 0.f;
    auto take = [&](int c, float &xo, float &oo, float &ro) {
        if (c >= 0 && c < C) {
            int64_t i = base + (int64_t)c * plane;
            float xx = ld_f32(x + i), g = ld_f32(dy + i), s = scale[i];
            float pw = pow_neg(s, beta);
            xo = xx, oo = g * pw, ro = g * xx * pw / s;
        } else {
            xo = 0.f, oo = 0.f, ro = 0.f;
        }
    };
    const int c0 = blockIdx.y * LRN_CB, c1 = c0 + LRN_CB < C ? c0 + LRN_CB : C;
#pragma unroll
    for (int j = 0; j < 2 * HALF; ++j) {
        float xo, oo;
        take(c0 - HALF + j, xo, oo, r[j + 1]);
        if (j >= HALF) xv[j - HALF + 1] = xo, own[j - HALF + 1] = oo;
    }
    for (int c = c0; c < c1; ++c) {
#pragma unroll
        for (int j = 0; j < 2 * HALF; ++j) r[j] = r[j + 1];
#pragma unroll
        for (int j = 0; j < HALF; ++j) xv[j] = xv[j + 1], own[j] = own[j + 1];
        take(c + HALF, xv[HALF], own[HALF], r[2 * HALF]);
        float acc = 0.f;
#pragma unroll
        for (int j = 0; j < 2 * HALF + 1; ++j) acc += r[j];
        st_f32(dx + base + (int64_t)c * plane, own[0] - coef * xv[0] * acc);
    }
}

template <typename T, int HALF>
static int lrn_launch(bool backward, int64_t N, int32_t C, int64_t plane, int32_t size, float alpha, float beta, float k,
                      const void *x, const void *dy, float *scale, void *out, hipStream_t s)
{
    const int64_t pixels = N * plane;
    const double elems = (double)pixels * C, e = sizeof(T);
    dim3 grid((unsigned)((pixels + 255) / 256), (unsigned)((C + LRN_CB - 1) / LRN_CB)), block(256);
    FastDiv dp((uint32_t)plane);
    if (!backward) {
        ProfScope prof(KID_LRN, s, 0.0, elems * (2.0 * e + (scale ? 4.0 : 0.0)));
        hipLaunchKernelGGL((lrn_forward_kernel<T, HALF>), grid, block, 0, s, (const T *)x, (T *)out, scale, pixels, C, plane, dp,
                           alpha / (float)size, beta, k);
    } else {
        ProfScope prof(KID_LRN, s, 0.0, elems * (3.0 * e + 4.0));
        hipLaunchKernelGGL((lrn_backward_kernel<T, HALF>), grid, block, 0, s, (const T *)x, (const T *)dy, (const float *)scale,
                           (T *)out, pixels, C, plane, dp, 2.0f * alpha * beta / (float)size, beta);
    }
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

int launch_lrn(int dtype, bool backward, int64_t N, int32_t C, int64_t plane, int32_t size, float alpha, float beta, float k,
               const void *x, const void *dy, float *scale, void *out, hipStream_t s)
{
#define OMNI_LRN_CASE(H)                                                                                               \
    case H:                                                                                                            \
        return dtype == OMNI_BF16 ? lrn_launch<bf16_t, H>(backward, N, C, plane, size, alpha, beta, k, x, dy, scale, out, s) \
                                  : lrn_launch<float, H>(backward, N, C, plane, size, alpha, beta, k, x, dy, scale, out, s);
    switch (size / 2) {
        OMNI_LRN_CASE(0)
        OMNI_LRN_CASE(1)
        OMNI_LRN_CASE(2)
        OMNI_LRN_CASE(3)
        OMNI_LRN_CASE(4)
    default: return OMNI_UNSUPPORTED;
    }
#undef OMNI_LRN_CASE
}

// ------------------------------------------------------------------------------------------------
// Dropout: keep an element with probability 1 - p and scale it by 1 / (1 - p).  The mask is never stored:
// element i is kept iff draw i mod 8 of Philox4x64-10 block i / 8 (counter {block, 0, 0, 0}, key {seed,
// stream}; low 32-bit half of each 64-bit word first) is at least floor(p * 2^32), so the backward pass
// regenerates it from the same seed.  One thread per block of eight elements.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void philox4x64_10(uint64_t c0, uint64_t c1, uint64_t c2, uint64_t c3, uint64_t k0, uint64_t k1,
                                              uint64_t out[4])
{
    const uint64_t M0 = 0xD2E7470EE14C6C93ull, M1 = 0xCA5A826395121157ull;
    const uint64_t W0 = 0x9E3779B97F4A7C15ull, W1 = 0xBB67AE8584CAA73Bull;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint64_t hi0 = __umul64hi(M0, c0), lo0 = M0 * c0;
        uint64_t hi1 = __umul64hi(M1, c2), lo1 = M1 * c2;
        uint64_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0, c1 = lo1, c2 = n2, c3 = lo0;
        k0 += W0, k1 += W1;
    }
    out[0] = c0, out[1] = c1, out[2] = c2, out[3] = c3;
}

template <typename T>
__global__ __launch_bounds__(256) void dropout_kernel(const T *__restrict__ x, T *__restrict__ y, int64_t count, uint32_t threshold,
                                                      float scale, uint64_t seed, uint64_t stream_id)
{
    int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t i0 = b * 8;
    if (i0 >= count) return;
    uint64_t w[4];
    philox4x64_10((uint64_t)b, 0, 0, 0, seed, stream_id, w);
    uint32_t draw[8] = {(uint32_t)w[0], (uint32_t)(w[0] >> 32), (uint32_t)w[1], (uint32_t)(w[1] >> 32),
                        (uint32_t)w[2], (uint32_t)(w[2] >> 32), (uint32_t)w[3], (uint32_t)(w[3] >> 32)};
    if (i0 + 8 <= count) {
        T v[8];
        __builtin_memcpy(v, x + i0, sizeof(v));  // 8 elements: i0 * sizeof(T) is a multiple of 16
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float f = Elem<T>::to_f32(v[j]) * scale;
            v[j] = Elem<T>::from_f32(draw[j] >= threshold ? f : 0.f);
        }
        __builtin_memcpy(y + i0, v, sizeof(v));
    } else {
        for (int j = 0; i0 + j < count; ++j) {
            float f = Elem<T>::to_f32(x[i0 + j]) * scale;
            y[i0 + j] = Elem<T>::from_f32(draw[j] >= threshold ? f : 0.f);
        }
    }
}

int launch_dropout(int dtype, int64_t count, uint32_t threshold, float scale, uint64_t seed, uint64_t stream_id, const void *x,
                   void *y, hipStream_t s)
{
    const int64_t blocks8 = (count + 7) / 8;
    dim3 grid((unsigned)((blocks8 + 255) / 256)), block(256);
    ProfScope prof(KID_DROPOUT, s, 0.0, 2.0 * (double)count * elem_size(dtype));
    if (dtype == OMNI_BF16)
        hipLaunchKernelGGL(dropout_kernel<bf16_t>, grid, block, 0, s, (const bf16_t *)x, (bf16_t *)y, count, threshold, scale, seed, stream_id);
    else
        hipLaunchKernelGGL(dropout_kernel<float>, grid, block, 0, s, (const float *)x, (float *)y, count, threshold, scale, seed, stream_id);
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

}  // namespace omni
