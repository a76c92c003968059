// Data-movement kernels of the lowered convolution (gfx950): batched lowering X -> D-hat, its
// transpose col2im dD-hat -> dX, the reshaping of the model into K-hat / K-hat^T, and the packing
// of an output-shaped gradient into the matrix dY-hat (with the bias gradient as a by-product).
//
// All of them are bound by HBM traffic, so the rules are: every thread writes 16 bytes, lanes of a
// wavefront touch consecutive addresses, indices are decoded once per thread with multiply-high
// divisions, and nothing is reduced with floating point atomics.
#include "common.h"

namespace omni {

// ------------------------------------------------------------------------------------------------
// Batched lowering (App. C, lowering phase; Sec. III-B: all N images before any GEMM)
//   D-hat[(c,ky,kx)][(n,oy,ox)] = X[n,c,oy*sh-ph+ky,ox*sw-pw+kx]   or 0 in the padding
// U is an unsigned integer of the element's width: lowering copies bit patterns.
// Each thread produces VEC consecutive columns of one row; columns in [M, ld) are written as zero.
// ------------------------------------------------------------------------------------------------
template <typename U, int VEC> struct alignas(sizeof(U) * VEC) VecOf { U v[VEC]; };

template <typename U, int VEC>
__global__ __launch_bounds__(256) void lower_kernel(ConvGeom g, const U *__restrict__ X, U *__restrict__ D,
                                                    int64_t ld, int64_t vecs_per_row)
{
    int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= vecs_per_row) return;
    uint32_t m0 = (uint32_t)(v * VEC);
    uint32_t n, rem, oy, ox;
    g.div_HoWo.divmod(m0 < (uint32_t)g.M ? m0 : 0u, n, rem);
    g.div_Wo.divmod(rem, oy, ox);

    for (int k = blockIdx.y; k < g.K; k += gridDim.y) {
        uint32_t c, r2, ky, kx;
        g.div_khkw.divmod((uint32_t)k, c, r2);
        g.div_kw.divmod(r2, ky, kx);
        VecOf<U, VEC> out;
        uint32_t nn = n, yy = oy, xx = ox;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            U val = 0;
            if (m0 + e < (uint32_t)g.M) {
                int iy = (int)yy * g.sh - g.ph + (int)ky;
                int ix = (int)xx * g.sw - g.pw + (int)kx;
                if (iy >= 0 && iy < g.H && ix >= 0 && ix < g.W)
                    val = X[(((int64_t)nn * g.C + c) * g.H + iy) * g.W + ix];
            }
            out.v[e] = val;
            if (++xx == (uint32_t)g.Wo) {
                xx = 0;
                if (++yy == (uint32_t)g.Ho) {
                    yy = 0;
                    ++nn;
                }
            }
        }
        *reinterpret_cast<VecOf<U, VEC> *>(D + (int64_t)k * ld + m0) = out;
    }
}

template <typename U>
static int run_lower(const ConvGeom &g, const U *X, U *D, int64_t ld, hipStream_t s)
{
    constexpr int VEC = 16 / sizeof(U);
    unsigned gy = (unsigned)(g.K < 65535 ? g.K : 65535);
    ProfScope prof(KID_LOWER, s, 0.0, ((double)g.N * g.C * g.H * g.W + (double)g.K * g.M) * sizeof(U));
    if (ld % VEC == 0) {
        int64_t vpr = ld / VEC;
        dim3 grid((unsigned)((vpr + 255) / 256), gy, 1);
        hipLaunchKernelGGL((lower_kernel<U, VEC>), grid, dim3(256), 0, s, g, X, D, ld, vpr);
    } else {
        dim3 grid((unsigned)((ld + 255) / 256), gy, 1);
        hipLaunchKernelGGL((lower_kernel<U, 1>), grid, dim3(256), 0, s, g, X, D, ld, ld);
    }
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

int launch_lower(const ConvGeom &g, int dtype, const void *X, void *Dhat, int64_t ld, hipStream_t s)
{
    if (dtype == OMNI_BF16) return run_lower<uint16_t>(g, (const uint16_t *)X, (uint16_t *)Dhat, ld, s);
    return run_lower<uint32_t>(g, (const uint32_t *)X, (uint32_t *)Dhat, ld, s);
}

// ------------------------------------------------------------------------------------------------
// col2im (transpose of the lowering map), gather form: one thread per input pixel sums the entries
// of dD-hat that were copies of that pixel, in ascending (ky, kx) order, in fp32.  No atomics.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void col2im_kernel(ConvGeom g, const T *__restrict__ D, int64_t ld,
                                                     T *__restrict__ dX, uint32_t plane0, uint32_t count)
{
    // One launch covers `count` < 2^31 pixels starting at plane (n*C + c) = plane0.
    uint32_t local = blockIdx.x * 256u + threadIdx.x;
    if (local >= count) return;
    uint32_t pl, pix, iy, ix;
    g.div_HW.divmod(local, pl, pix);
    g.div_W.divmod(pix, iy, ix);
    uint32_t plane = plane0 + pl;
    uint32_t n = plane / (uint32_t)g.C, c = plane - n * (uint32_t)g.C;

    float acc = 0.f;
    for (int ky = 0; ky < g.kh; ++ky) {
        int ty = (int)iy + g.ph - ky;
        if (ty < 0) break;  // larger ky only moves further up
        int oy = ty / g.sh;
        if (oy * g.sh != ty || oy >= g.Ho) continue;
        for (int kx = 0; kx < g.kw; ++kx) {
            int tx = (int)ix + g.pw - kx;
            if (tx < 0) break;
            int ox = tx / g.sw;
            if (ox * g.sw != tx || ox >= g.Wo) continue;
            int64_t row = ((int64_t)c * g.kh + ky) * g.kw + kx;
            int64_t col = ((int64_t)n * g.Ho + oy) * g.Wo + ox;
            acc += Elem<T>::to_f32(D[row * ld + col]);
        }
    }
    dX[(int64_t)plane * g.H * g.W + pix] = Elem<T>::from_f32(acc);
}

int launch_col2im(const ConvGeom &g, int dtype, const void *dDhat, int64_t ld, void *dX, hipStream_t s)
{
    int64_t planes = (int64_t)g.N * g.C, hw = (int64_t)g.H * g.W;
    int64_t planes_per_launch = (0x7fffffffll - 4096) / hw;
    ProfScope prof(KID_COL2IM, s, 0.0, ((double)planes * hw + (double)g.K * g.M) * elem_size(dtype));
    for (int64_t p0 = 0; p0 < planes; p0 += planes_per_launch) {
        int64_t np = planes - p0 < planes_per_launch ? planes - p0 : planes_per_launch;
        uint32_t count = (uint32_t)(np * hw);
        dim3 grid((count + 255u) / 256u);
        if (dtype == OMNI_BF16)
            hipLaunchKernelGGL(col2im_kernel<bf16_t>, grid, dim3(256), 0, s, g, (const bf16_t *)dDhat, ld, (bf16_t *)dX, (uint32_t)p0, count);
        else
            hipLaunchKernelGGL(col2im_kernel<float>, grid, dim3(256), 0, s, g, (const float *)dDhat, ld, (float *)dX, (uint32_t)p0, count);
        OMNI_LAUNCH_CHECK();
    }
    return OMNI_OK;
}

// ------------------------------------------------------------------------------------------------
// K-hat: the model as a matrix (App. C: "the kernel does not require any replication").
// W [F][K] -> K-hat [Fp][Kp] zero padded;  K-hat^T [Kp][Fp] zero padded.
// ------------------------------------------------------------------------------------------------
template <typename U>
__global__ void pack_khat_kernel(const U *__restrict__ W, U *__restrict__ out, int F, int K, int64_t rows,
                                 int64_t cols, int transpose)
{
    int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * cols) return;
    int64_t r = idx / cols, c = idx - r * cols;
    int64_t f = transpose ? c : r, k = transpose ? r : c;
    out[idx] = (f < F && k < K) ? W[f * K + k] : (U)0;
}

static int run_pack_khat(int dtype, const void *W, void *out, int F, int K, int64_t rows, int64_t cols,
                         int transpose, hipStream_t s)
{
    dim3 grid((unsigned)((rows * cols + 255) / 256));
    ProfScope prof(KID_PACK_KHAT, s, 0.0, 2.0 * F * K * elem_size(dtype));
    if (dtype == OMNI_BF16)
        hipLaunchKernelGGL(pack_khat_kernel<uint16_t>, grid, dim3(256), 0, s, (const uint16_t *)W, (uint16_t *)out, F, K, rows, cols, transpose);
    else
        hipLaunchKernelGGL(pack_khat_kernel<uint32_t>, grid, dim3(256), 0, s, (const uint32_t *)W, (uint32_t *)out, F, K, rows, cols, transpose);
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

int launch_pack_khat(const ConvGeom &g, int dtype, const void *W, void *Khat, int64_t Fp, int64_t Kp, hipStream_t s)
{
    return run_pack_khat(dtype, W, Khat, g.F, g.K, Fp, Kp, 0, s);
}

int launch_pack_khat_t(const ConvGeom &g, int dtype, const void *W, void *KhatT, int64_t Kp, int64_t Fp, hipStream_t s)
{
    return run_pack_khat(dtype, W, KhatT, g.F, g.K, Kp, Fp, 1, s);
}

// ------------------------------------------------------------------------------------------------
// dY [N][F][Ho][Wo] -> dY-hat [F][ld] (the inverse of lifting), columns in [M, ld) zero.
// Each block covers PACK_COLS columns of one row f; with bias_partials != null it also leaves the
// fp32 sum of its columns in bias_partials[f][block], reduced in block order by the second kernel.
// ------------------------------------------------------------------------------------------------
constexpr int PACK_VEC = 8;
constexpr int PACK_COLS = 256 * PACK_VEC;

template <typename T, typename U>
__global__ __launch_bounds__(256) void pack_dyhat_kernel(ConvGeom g, const T *__restrict__ dY, U *__restrict__ out,
                                                         int64_t ld, float *__restrict__ bias_partials)
{
    int f = blockIdx.y;
    int64_t m0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * PACK_VEC;
    float sum = 0.f;
    if (m0 < ld) {
        uint32_t n, r;
        g.div_HoWo.divmod(m0 < g.M ? (uint32_t)m0 : 0u, n, r);
        VecOf<U, PACK_VEC> o;
#pragma unroll
        for (int e = 0; e < PACK_VEC; ++e) {
            U bits = 0;
            if (m0 + e < g.M) {
                const T *src = dY + ((int64_t)n * g.F + f) * g.HoWo + r;
                bits = *reinterpret_cast<const U *>(src);
                sum += Elem<T>::to_f32(*src);
            }
            o.v[e] = bits;
            if (++r == (uint32_t)g.HoWo) {
                r = 0;
                ++n;
            }
        }
        // 8 x 4 bytes does not fit one 16-byte store: write two halves for fp32
        if constexpr (sizeof(U) == 2) {
            *reinterpret_cast<VecOf<U, 8> *>(out + (int64_t)f * ld + m0) = o;
        } else {
            VecOf<U, 4> a, b;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                a.v[e] = o.v[e];
                b.v[e] = o.v[4 + e];
            }
            *reinterpret_cast<VecOf<U, 4> *>(out + (int64_t)f * ld + m0) = a;
            *reinterpret_cast<VecOf<U, 4> *>(out + (int64_t)f * ld + m0 + 4) = b;
        }
    }
    if (bias_partials != nullptr) {
        // fixed-shape tree: lanes, then the four wavefronts in order
        __shared__ float wave_sum[4];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) sum += __shfl_down(sum, off, 64);
        if ((threadIdx.x & 63) == 0) wave_sum[threadIdx.x >> 6] = sum;
        __syncthreads();
        if (threadIdx.x == 0)
            bias_partials[(int64_t)f * gridDim.x + blockIdx.x] = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
    }
}

__global__ __launch_bounds__(64) void bias_reduce_kernel(const float *__restrict__ partials, int blocks, float *__restrict__ dbias)
{
    // one wavefront per filter: strided partial sums per lane (fixed order), then a fixed tree
    int f = blockIdx.x;
    float acc = 0.f;
    for (int b = threadIdx.x; b < blocks; b += 64) acc += partials[(int64_t)f * blocks + b];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    if (threadIdx.x == 0) dbias[f] = acc;
}

int pack_dyhat_blocks(const ConvGeom &g) { return (int)((dhat_ld(g) + PACK_COLS - 1) / PACK_COLS); }

int launch_pack_dyhat(const ConvGeom &g, int dtype, const void *dY, void *dYhat, int64_t ld, float *bias_partials,
                      int bias_blocks, float *dbias, hipStream_t s)
{
    int blocks = (int)((ld + PACK_COLS - 1) / PACK_COLS);
    if (bias_partials != nullptr && bias_blocks != blocks) return OMNI_INVALID_ARGUMENT;
    dim3 grid((unsigned)blocks, (unsigned)g.F, 1);
    {
        ProfScope prof(KID_PACK_DYHAT, s, 0.0, 2.0 * g.F * (double)g.M * elem_size(dtype));
        if (dtype == OMNI_BF16)
            hipLaunchKernelGGL((pack_dyhat_kernel<bf16_t, uint16_t>), grid, dim3(256), 0, s, g, (const bf16_t *)dY, (uint16_t *)dYhat, ld, bias_partials);
        else
            hipLaunchKernelGGL((pack_dyhat_kernel<float, uint32_t>), grid, dim3(256), 0, s, g, (const float *)dY, (uint32_t *)dYhat, ld, bias_partials);
    }
    OMNI_LAUNCH_CHECK();
    if (bias_partials != nullptr) {
        ProfScope prof(KID_BIAS_REDUCE, s, 0.0, 4.0 * g.F * (blocks + 1));
        hipLaunchKernelGGL(bias_reduce_kernel, dim3((unsigned)g.F), dim3(64), 0, s, bias_partials, blocks, dbias);
        OMNI_LAUNCH_CHECK();
    }
    return OMNI_OK;
}

}  // namespace omni
