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

// LDS-staged variant.  A workgroup takes one input channel c of a group of images (small planes) or
// of a band of output rows of one image (large planes), copies the zero-padded patch it needs into
// LDS once with coalesced reads, and then writes all kh*kw rows of D-hat that stem from that patch:
// for each row the columns of the group are one contiguous range, written 16 bytes per lane.  Columns
// at the ragged ends of the range (ranges need not start on a 16-byte boundary) are stored one by one.
// X is read from HBM once; every store instruction of a wavefront covers 1 KiB of consecutive bytes.
struct LowerPlan {
    int nb;        // images per workgroup (1 in banded mode)
    int br;        // output rows per band (Ho when nb > 1)
    int bands;     // bands per image
    int groups;    // image groups
    int rows_in;   // input rows held per image: (br-1)*sh + kh
    int wp;        // padded row pitch: W + 2*pw
    FastDiv div_wp, div_rows_in;
};

template <typename U, int VEC, int KW>  // KW > 0: window width known at compile time (inner loop unrolled)
__global__ __launch_bounds__(256) void lower_lds_kernel(ConvGeom g, LowerPlan p, const U *__restrict__ X,
                                                        U *__restrict__ D, int64_t ld)
{
    extern __shared__ __align__(16) unsigned char lower_smem[];
    U *tile = reinterpret_cast<U *>(lower_smem);
    const int tid = threadIdx.x;
    const int c = blockIdx.y;
    const int band = blockIdx.x % p.bands, grp = blockIdx.x / p.bands;
    const int n0 = grp * p.nb;
    const int nb = g.N - n0 < p.nb ? g.N - n0 : p.nb;
    const int oy0 = band * p.br;
    const int br = g.Ho - oy0 < p.br ? g.Ho - oy0 : p.br;
    const int rows_used = (br - 1) * g.sh + g.kh;
    const int kw = KW > 0 ? KW : g.kw;
    constexpr int VECL = 16 / sizeof(U);  // elements per 16-byte global load

    // patch -> LDS.  The padding is zeroed first; then the pixels, which for one image are one
    // contiguous run of whole input rows, are fetched 16 bytes per lane (the run need not be 16-byte
    // aligned) and dropped into the padded layout one element at a time.
    {
        const int patch16 = (nb * p.rows_in * p.wp * (int)sizeof(U) + 15) / 16;
        uint4 *t16 = reinterpret_cast<uint4 *>(lower_smem);
        for (int i = tid; i < patch16; i += 256) t16[i] = make_uint4(0, 0, 0, 0);
    }
    __syncthreads();
    {
        int iy_lo = oy0 * g.sh - g.ph, iy_hi = iy_lo + rows_used;  // input rows the patch covers
        const int ry0 = iy_lo < 0 ? -iy_lo : 0;                     // first patch row that lies in the image
        if (iy_lo < 0) iy_lo = 0;
        if (iy_hi > g.H) iy_hi = g.H;
        const int run = (iy_hi - iy_lo) * g.W;                      // elements per image
        const int chunks = (run + VECL - 1) / VECL;
        for (int t = tid; t < nb * chunks; t += 256) {
            int inb = t / chunks, ch = t - inb * chunks;
            const U *src = X + (((int64_t)(n0 + inb) * g.C + c) * g.H + iy_lo) * g.W + ch * VECL;
            U vals[VECL];
            if ((ch + 1) * VECL <= run) {
                __builtin_memcpy(vals, src, sizeof(vals));
            } else {
#pragma unroll
                for (int e = 0; e < VECL; ++e) vals[e] = ch * VECL + e < run ? src[e] : (U)0;
            }
            uint32_t ry, ix;
            g.div_W.divmod((uint32_t)(ch * VECL), ry, ix);
            U *drow = tile + (inb * p.rows_in + ry0 + (int)ry) * p.wp + g.pw;
#pragma unroll
            for (int e = 0; e < VECL; ++e) {
                if (ch * VECL + e < run) drow[ix] = vals[e];
                if (++ix == (uint32_t)g.W) {
                    ix = 0;
                    drow += p.wp;
                }
            }
        }
    }
    __syncthreads();

    // the contiguous column range of this workgroup
    const int seg = p.nb > 1 ? g.HoWo : br * g.Wo;  // columns per image
    const int64_t m_lo = (int64_t)n0 * g.HoWo + (int64_t)oy0 * g.Wo;
    const int64_t m_hi = m_lo + (int64_t)(p.nb > 1 ? nb : 1) * seg;
    const int64_t v_lo = (m_lo + VEC - 1) / VEC, v_hi = m_hi / VEC;  // slots that lie entirely inside the range
    const int khkw = g.kh * kw;
    auto locate = [&](int64_t m) -> int {  // LDS index of the window origin of column m
        uint32_t t = (uint32_t)(m - m_lo), inb = 0, rem = t, oy, ox;
        if (p.nb > 1) g.div_HoWo.divmod(t, inb, rem);
        g.div_Wo.divmod(rem, oy, ox);
        return ((int)inb * p.rows_in + (int)oy * g.sh) * p.wp + (int)ox * g.sw;
    };

    for (int64_t v = v_lo + tid; v < v_hi; v += 256) {
        int a[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) a[e] = locate(v * VEC + e);
        U *dst = D + (int64_t)c * khkw * ld + v * VEC;
        for (int ky = 0; ky < g.kh; ++ky) {
            const U *src[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) src[e] = tile + a[e] + ky * p.wp;
            if constexpr (KW > 0) {
#pragma unroll
                for (int kx = 0; kx < KW; ++kx) {
                    VecOf<U, VEC> out;
#pragma unroll
                    for (int e = 0; e < VEC; ++e) out.v[e] = src[e][kx];
                    *reinterpret_cast<VecOf<U, VEC> *>(dst) = out;
                    dst += ld;
                }
            } else {
                for (int kx = 0; kx < kw; ++kx) {
                    VecOf<U, VEC> out;
#pragma unroll
                    for (int e = 0; e < VEC; ++e) out.v[e] = src[e][kx];
                    *reinterpret_cast<VecOf<U, VEC> *>(dst) = out;
                    dst += ld;
                }
            }
        }
    }
    // ragged ends: the columns before the first and after the last whole slot, one (row, column) per thread
    const int head = (int)(v_lo * VEC - m_lo < m_hi - m_lo ? v_lo * VEC - m_lo : m_hi - m_lo);
    const int tail = v_hi >= v_lo ? (int)(m_hi - v_hi * VEC) : 0;
    const int edge = head + tail;
    for (int idx = tid; idx < edge * khkw; idx += 256) {
        int r = idx / edge, j = idx - r * edge;
        int64_t m = j < head ? m_lo + j : v_hi * VEC + (j - head);
        int ky = r / kw, kx = r - ky * kw;
        D[((int64_t)c * khkw + r) * ld + m] = tile[locate(m) + ky * p.wp + kx];
    }
    // columns in [M, ld) of this channel's rows are zero; the workgroup that owns the last column writes them
    if (m_hi == g.M && ld > g.M) {
        const int padc = (int)(ld - g.M);
        for (int idx = tid; idx < khkw * padc; idx += 256) {
            int r = idx / padc, cc = idx - r * padc;
            D[((int64_t)c * khkw + r) * ld + g.M + cc] = 0;
        }
    }
}

// Choose the staging plan; returns false when not even one output row's patch fits in LDS.
static bool make_lower_plan(const ConvGeom &g, size_t elem, LowerPlan *p, size_t *lds_bytes)
{
    const size_t small_budget = 32 * 1024, band_budget = 40 * 1024;
    p->wp = g.W + 2 * g.pw;
    int rows_full = (g.Ho - 1) * g.sh + g.kh;
    size_t plane = (size_t)rows_full * p->wp * elem;
    if (2 * plane <= small_budget) {
        int nb = (int)(small_budget / plane);
        if (nb > 32) nb = 32;
        if (nb > g.N) nb = g.N;
        p->nb = nb;
        p->br = g.Ho;
        p->bands = 1;
        p->rows_in = rows_full;
    } else {
        size_t row_bytes = (size_t)p->wp * elem;
        if ((size_t)g.kh * row_bytes > 64 * 1024) return false;
        int64_t rows_fit = (int64_t)(band_budget / row_bytes);
        int br = rows_fit >= g.kh ? (int)((rows_fit - g.kh) / g.sh + 1) : 1;
        if (br > g.Ho) br = g.Ho;
        p->nb = 1;
        p->br = br;
        p->bands = (g.Ho + br - 1) / br;
        p->rows_in = (br - 1) * g.sh + g.kh;
    }
    p->groups = (g.N + p->nb - 1) / p->nb;
    p->div_wp = FastDiv((uint32_t)p->wp);
    p->div_rows_in = FastDiv((uint32_t)p->rows_in);
    *lds_bytes = (size_t)p->nb * p->rows_in * p->wp * elem;
    if ((int64_t)p->bands * p->groups > 0x7fffffffll || g.C > 65535) return false;
    return true;
}

template <typename U>
static int run_lower(const ConvGeom &g, const U *X, U *D, int64_t ld, hipStream_t s)
{
    constexpr int VEC = 16 / sizeof(U);
    ProfScope prof(KID_LOWER, s, 0.0, ((double)g.N * g.C * g.H * g.W + (double)g.K * g.M) * sizeof(U));
    LowerPlan plan;
    size_t lds = 0;
    if (make_lower_plan(g, sizeof(U), &plan, &lds)) {
        dim3 grid((unsigned)(plan.bands * plan.groups), (unsigned)g.C, 1);
        const int vec = ld % VEC != 0 ? 1 : VEC;
#define OMNI_LOWER_CASE(V, KWT) hipLaunchKernelGGL((lower_lds_kernel<U, V, KWT>), grid, dim3(256), lds, s, g, plan, X, D, ld)
#define OMNI_LOWER_KW(V)                                  \
    do {                                                  \
        if (g.kw == 3) OMNI_LOWER_CASE(V, 3);             \
        else if (g.kw == 5) OMNI_LOWER_CASE(V, 5);        \
        else if (g.kw == 11) OMNI_LOWER_CASE(V, 11);      \
        else OMNI_LOWER_CASE(V, 0);                       \
    } while (0)
        if (vec == 1) OMNI_LOWER_CASE(1, 0);
        else OMNI_LOWER_KW(VEC);
#undef OMNI_LOWER_KW
#undef OMNI_LOWER_CASE
        OMNI_LAUNCH_CHECK();
        return OMNI_OK;
    }
    unsigned gy = (unsigned)(g.K < 65535 ? g.K : 65535);
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
// The window positions that cover input coordinate i along one axis: k = first, first+s, ... <= last,
// with output coordinate o(first) = (i + pad - first)/s decreasing by one per step.  No per-tap division.
struct TapRange { int first, last, o_first; };
__device__ __forceinline__ TapRange tap_range(int i, int pad, int k, int s, int out, const FastDiv &div_s)
{
    TapRange t;
    int top = i + pad;                       // k = top gives o = 0
    int lo = top - (out - 1) * s;            // smallest k with o <= out-1
    if (lo < 0) lo = 0;
    uint32_t q, r;
    div_s.divmod((uint32_t)(top - lo), q, r);  // top - lo >= 0 whenever the range is non-empty
    t.first = lo + (int)r;                   // same residue as top modulo s
    t.o_first = (int)q;
    t.last = top < k - 1 ? top : k - 1;
    if (top < lo) t.last = -1;               // empty
    return t;
}

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
    const TapRange ry = tap_range((int)iy, g.ph, g.kh, g.sh, g.Ho, g.div_sh);
    const TapRange rx = tap_range((int)ix, g.pw, g.kw, g.sw, g.Wo, g.div_sw);
    for (int ky = ry.first, oy = ry.o_first; ky <= ry.last; ky += g.sh, --oy)
        for (int kx = rx.first, ox = rx.o_first; kx <= rx.last; kx += g.sw, --ox) {
            int64_t row = ((int64_t)c * g.kh + ky) * g.kw + kx;
            int64_t col = ((int64_t)n * g.Ho + oy) * g.Wo + ox;
            acc += Elem<T>::to_f32(D[row * ld + col]);
        }
    dX[(int64_t)plane * g.H * g.W + pix] = Elem<T>::from_f32(acc);
}

// Strided layers whose segments do not fit in LDS (CaffeNet's conv1: 11 x 11 window, stride 4).  With stride S an
// input pixel meets only the taps of its own residue class, kx = (ix + pw) mod S + S*j, and for one such tap the
// pixels ix, ix + S, ix + 2S, ... of a row read consecutive columns of one row of dD-hat.  So a thread takes the S
// consecutive pixels S*b .. S*b + S - 1 of an input row and neighbouring lanes take neighbouring b: every load
// instruction of a wavefront then reads one run of consecutive elements (the per-pixel form above reads S runs with
// gaps, and fetched three times the matrix on conv1), and every thread stores S consecutive pixels at once.
// At most JY x JX taps per pixel (ceil(kh / S), ceil(kw / S)), all issued together with the absent ones masked;
// each pixel's terms are added in ascending (ky, kx), as above.
template <typename T, int S, int JY, int JX>
__global__ __launch_bounds__(256) void col2im_strided_kernel(ConvGeom g, const T *__restrict__ D, int64_t ld,
                                                             T *__restrict__ dX, uint32_t plane0, uint32_t count,
                                                             FastDiv div_rows, FastDiv div_bw)
{
    // One launch covers `count` < 2^31 (plane, row, group of S pixels) triples starting at plane plane0.
    const uint32_t local = blockIdx.x * 256u + threadIdx.x;
    if (local >= count) return;
    uint32_t pl, rest, iy, b;
    div_rows.divmod(local, pl, rest);  // rows of groups per plane: H * ceil(W / S)
    div_bw.divmod(rest, iy, b);
    const uint32_t plane = plane0 + pl;
    const uint32_t n = plane / (uint32_t)g.C, c = plane - n * (uint32_t)g.C;
    const TapRange ry = tap_range((int)iy, g.ph, g.kh, S, g.Ho, g.div_sh);
    TapRange rx[S];
#pragma unroll
    for (int px = 0; px < S; ++px) {
        const int ix = S * (int)b + px;
        rx[px] = tap_range(ix < g.W ? ix : g.W - 1, g.pw, g.kw, S, g.Wo, g.div_sw);
        if (ix >= g.W) rx[px].last = -1;
    }
    float v[JY][S][JX];
    bool ok[JY][S][JX];
#pragma unroll
    for (int jy = 0; jy < JY; ++jy) {
        const int ky = ry.first + jy * S, oy = ry.o_first - jy;
        const bool vy = ky <= ry.last;
        const int64_t col0 = ((int64_t)n * g.Ho + oy) * g.Wo;
#pragma unroll
        for (int px = 0; px < S; ++px)
#pragma unroll
            for (int jx = 0; jx < JX; ++jx) {
                const int kx = rx[px].first + jx * S, ox = rx[px].o_first - jx;
                ok[jy][px][jx] = vy && kx <= rx[px].last;
                const int64_t at = ok[jy][px][jx] ? (((int64_t)c * g.kh + ky) * g.kw + kx) * ld + col0 + ox : 0;
                v[jy][px][jx] = Elem<T>::to_f32(D[at]);
            }
    }
    T res[S];
#pragma unroll
    for (int px = 0; px < S; ++px) {
        float acc = 0.f;
#pragma unroll
        for (int jy = 0; jy < JY; ++jy)
#pragma unroll
            for (int jx = 0; jx < JX; ++jx) acc += ok[jy][px][jx] ? v[jy][px][jx] : 0.f;
        res[px] = Elem<T>::from_f32(acc);
    }
    T *out = dX + ((int64_t)plane * g.H + iy) * g.W + S * (int64_t)b;
    if (S * (int)b + S <= g.W) {
        __builtin_memcpy(out, res, sizeof(res));  // element-aligned store of S pixels
    } else {
#pragma unroll
        for (int px = 0; px < S; ++px)
            if (S * (int)b + px < g.W) out[px] = res[px];
    }
}

// LDS-staged variant.  A workgroup takes channel c of a group of nb images.  Step 1 copies, for each of
// the kh*kw rows of that channel, the column range of the group from dD-hat into LDS with 16-byte loads
// (all loads are in flight together).  Step 2 is the same gather as above, served from LDS: one thread
// per input pixel, ascending (ky, kx), fp32.  dD-hat is read from HBM exactly once, in full vectors.
struct Col2imPlan {
    int nb;      // images per workgroup
    int groups;  // image groups
    int pitch;   // LDS elements per row segment (multiple of the vector width)
};

// KH, KW > 0: stride 1 and a window known at compile time.  Pixel (iy, ix) then receives tap (ky, kx) from output
// position (iy + ph - ky, ix + pw - kx), i.e. from LDS element  base - ky * Wo - kx  of row ky * KW + kx: one
// address per pixel, constant offsets per tap, and the taps that fall outside the output are masked instead of
// being skipped by loops with data-dependent bounds (the vector ALU, not memory, is what bounded this kernel).
template <typename T, int KH, int KW>
__global__ __launch_bounds__(256) void col2im_lds_kernel(ConvGeom g, Col2imPlan p, const T *__restrict__ D,
                                                         int64_t ld, T *__restrict__ dX)
{
    constexpr int VEC = 16 / sizeof(T);
    extern __shared__ __align__(16) unsigned char col2im_smem[];
    T *seg = reinterpret_cast<T *>(col2im_smem);
    const int tid = threadIdx.x;
    const int c = blockIdx.y;
    const int n0 = blockIdx.x * p.nb;
    const int nb = g.N - n0 < p.nb ? g.N - n0 : p.nb;
    const int khkw = g.kh * g.kw;
    const int64_t m_lo = (int64_t)n0 * g.HoWo, m_hi = m_lo + (int64_t)nb * g.HoWo;
    const int64_t v_lo = m_lo / VEC, v_hi = (m_hi + VEC - 1) / VEC;  // 16-byte slots covering the range
    const int slots = (int)(v_hi - v_lo);
    const int skew = (int)(m_lo - v_lo * VEC);                        // position of column m_lo inside its slot

    const uint4 *src = reinterpret_cast<const uint4 *>(D + (int64_t)c * khkw * ld) + v_lo;
    const int64_t row_slots = ld / VEC;
    uint4 *dst = reinterpret_cast<uint4 *>(col2im_smem);
    const int pitch_slots = p.pitch / VEC;
    {
        // batches of loads into registers, then into LDS: a plain copy loop waits for each load before it
        // issues the next one, and a workgroup's whole segment is only about ten loads per thread
        constexpr int BATCH = 12;
        const int total = khkw * slots;
        for (int i0 = tid; i0 < total; i0 += 256 * BATCH) {
            uint4 regs[BATCH];
            int where[BATCH];
            // branch-free: indices past the end repeat the last slot (the same bytes land in the same place twice)
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                int i = i0 + 256 * u;
                i = i < total ? i : total - 1;
                const int r = i / slots, v = i - r * slots;
                regs[u] = src[r * row_slots + v];
                where[u] = r * pitch_slots + v;
            }
#pragma unroll
            for (int u = 0; u < BATCH; ++u) dst[where[u]] = regs[u];
        }
    }
    __syncthreads();

    const int hw = g.H * g.W;
    for (int px = tid; px < nb * hw; px += 256) {
        uint32_t inb, pix, iy, ix;
        g.div_HW.divmod((uint32_t)px, inb, pix);
        g.div_W.divmod(pix, iy, ix);
        float acc = 0.f;
        if constexpr (KH > 0) {
            const int oy0 = (int)iy + g.ph, ox0 = (int)ix + g.pw;     // output position of tap (0, 0)
            const int base = skew + (int)inb * g.HoWo + oy0 * g.Wo + ox0;
            bool vx[KW];
#pragma unroll
            for (int kx = 0; kx < KW; ++kx) vx[kx] = (unsigned)(ox0 - kx) < (unsigned)g.Wo;
#pragma unroll
            for (int ky = 0; ky < KH; ++ky) {
                const bool vy = (unsigned)(oy0 - ky) < (unsigned)g.Ho;
#pragma unroll
                for (int kx = 0; kx < KW; ++kx) {
                    const bool ok = vy && vx[kx];
                    const int idx = ok ? (ky * KW + kx) * p.pitch + base - ky * g.Wo - kx : 0;
                    const float v = Elem<T>::to_f32(seg[idx]);
                    acc += ok ? v : 0.f;
                }
            }
        } else {
            const T *base = seg + skew + (int)inb * g.HoWo;
            const TapRange ry = tap_range((int)iy, g.ph, g.kh, g.sh, g.Ho, g.div_sh);
            const TapRange rx = tap_range((int)ix, g.pw, g.kw, g.sw, g.Wo, g.div_sw);
            for (int ky = ry.first, oy = ry.o_first; ky <= ry.last; ky += g.sh, --oy) {
                const T *row = base + ky * g.kw * p.pitch + oy * g.Wo;
                for (int kx = rx.first, ox = rx.o_first; kx <= rx.last; kx += g.sw, --ox)
                    acc += Elem<T>::to_f32(row[kx * p.pitch + ox]);
            }
        }
        dX[((int64_t)(n0 + inb) * g.C + c) * hw + pix] = Elem<T>::from_f32(acc);
    }
}

static bool make_col2im_plan(const ConvGeom &g, size_t elem, int64_t ld, Col2imPlan *p, size_t *lds_bytes)
{
    const int vec = (int)(16 / elem);
    if (ld % vec != 0 || g.C > 65535) return false;
    const size_t budget = 40 * 1024, hard_limit = 80 * 1024;  // two workgroups per compute unit at the limit
    const int khkw = g.kh * g.kw;
    size_t per_image = (size_t)khkw * g.HoWo * elem;
    int nb = (int)(budget / per_image);
    if (nb < 1) nb = 1;
    if (nb > 32) nb = 32;
    if (nb > g.N) nb = g.N;
    p->nb = nb;
    p->groups = (g.N + nb - 1) / nb;
    p->pitch = (int)round_up((int64_t)nb * g.HoWo + vec, vec) + vec;  // room for the skew at both ends
    *lds_bytes = (size_t)khkw * p->pitch * elem;
    return *lds_bytes <= hard_limit;
}

int launch_col2im(const ConvGeom &g, int dtype, const void *dDhat, int64_t ld, void *dX, hipStream_t s)
{
    int64_t planes = (int64_t)g.N * g.C, hw = (int64_t)g.H * g.W;
    ProfScope prof(KID_COL2IM, s, 0.0, ((double)planes * hw + (double)g.K * g.M) * elem_size(dtype));
    Col2imPlan plan;
    size_t lds = 0;
    if (make_col2im_plan(g, elem_size(dtype), ld, &plan, &lds)) {
        dim3 grid((unsigned)plan.groups, (unsigned)g.C, 1);
        const bool unit = g.sh == 1 && g.sw == 1;
#define OMNI_COL2IM_CASE(KH, KW)                                                                                              \
    do {                                                                                                                      \
        if (dtype == OMNI_BF16)                                                                                               \
            hipLaunchKernelGGL((col2im_lds_kernel<bf16_t, KH, KW>), grid, dim3(256), lds, s, g, plan, (const bf16_t *)dDhat,   \
                               ld, (bf16_t *)dX);                                                                              \
        else                                                                                                                  \
            hipLaunchKernelGGL((col2im_lds_kernel<float, KH, KW>), grid, dim3(256), lds, s, g, plan, (const float *)dDhat, ld, \
                               (float *)dX);                                                                                   \
    } while (0)
        if (unit && g.kh == 3 && g.kw == 3) OMNI_COL2IM_CASE(3, 3);
        else if (unit && g.kh == 5 && g.kw == 5) OMNI_COL2IM_CASE(5, 5);
        else OMNI_COL2IM_CASE(0, 0);
#undef OMNI_COL2IM_CASE
        OMNI_LAUNCH_CHECK();
        return OMNI_OK;
    }
    // strided layers: the form whose loads are contiguous per wavefront, when the window has at most 3 x 3 taps per pixel
    const int S = g.sh;
    if (g.sh == g.sw && (S == 2 || S == 4) && (g.kh + S - 1) / S <= 3 && (g.kw + S - 1) / S <= 3) {
        const int64_t bw = (g.W + S - 1) / S, rows = (int64_t)g.H * bw;
        const int64_t per_launch = (0x7fffffffll - 4096) / rows;
        const FastDiv div_rows((uint32_t)rows), div_bw((uint32_t)bw);
        for (int64_t p0 = 0; p0 < planes; p0 += per_launch) {
            const int64_t np = planes - p0 < per_launch ? planes - p0 : per_launch;
            const uint32_t count = (uint32_t)(np * rows);
            dim3 grid((count + 255u) / 256u);
#define OMNI_COL2IM_STRIDED(T_, S_)                                                                                       \
    hipLaunchKernelGGL((col2im_strided_kernel<T_, S_, 3, 3>), grid, dim3(256), 0, s, g, (const T_ *)dDhat, ld, (T_ *)dX,   \
                       (uint32_t)p0, count, div_rows, div_bw)
            if (dtype == OMNI_BF16 && S == 4) OMNI_COL2IM_STRIDED(bf16_t, 4);
            else if (dtype == OMNI_BF16) OMNI_COL2IM_STRIDED(bf16_t, 2);
            else if (S == 4) OMNI_COL2IM_STRIDED(float, 4);
            else OMNI_COL2IM_STRIDED(float, 2);
#undef OMNI_COL2IM_STRIDED
            OMNI_LAUNCH_CHECK();
        }
        return OMNI_OK;
    }
    int64_t planes_per_launch = (0x7fffffffll - 4096) / hw;
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
constexpr int PACK_UNR = 4;                          // packs per thread
constexpr int PACK_COLS = 256 * PACK_VEC * PACK_UNR;  // columns per workgroup

template <typename T, typename U>
__global__ __launch_bounds__(256) void pack_dyhat_kernel(ConvGeom g, const T *__restrict__ dY, U *__restrict__ out,
                                                         int64_t ld, float *__restrict__ bias_partials)
{
    // PACK_UNR packs per thread, 256 packs apart.  Their loads are issued together and unconditionally: a
    // pack that cannot be read with one load (it straddles two images or the end of the matrix) reads the
    // first bytes of dY instead and is then assembled element by element.
    const int f = blockIdx.y;
    const bool can_vec = (int64_t)g.N * g.F * g.HoWo >= PACK_VEC;
    float sum = 0.f;
    int64_t m0[PACK_UNR];
    uint32_t n[PACK_UNR], r[PACK_UNR];
    bool fast[PACK_UNR];
    VecOf<U, PACK_VEC> o[PACK_UNR];
#pragma unroll
    for (int u = 0; u < PACK_UNR; ++u) {
        m0[u] = (((int64_t)blockIdx.x * PACK_UNR + u) * 256 + threadIdx.x) * PACK_VEC;
        g.div_HoWo.divmod(m0[u] < g.M ? (uint32_t)m0[u] : 0u, n[u], r[u]);
        fast[u] = can_vec && m0[u] + PACK_VEC <= g.M && r[u] + PACK_VEC <= (uint32_t)g.HoWo;
        const T *src = fast[u] ? dY + ((int64_t)n[u] * g.F + f) * g.HoWo + r[u] : dY;
        if (can_vec) __builtin_memcpy(&o[u], src, sizeof(o[u]));
    }
#pragma unroll
    for (int u = 0; u < PACK_UNR; ++u) {
        if (m0[u] >= ld) continue;
        if (fast[u]) {
#pragma unroll
            for (int e = 0; e < PACK_VEC; ++e) {
                T v;
                __builtin_memcpy(&v, &o[u].v[e], sizeof(T));
                sum += Elem<T>::to_f32(v);
            }
        } else {
            uint32_t nn = n[u], rr = r[u];
#pragma unroll
            for (int e = 0; e < PACK_VEC; ++e) {
                U bits = 0;
                if (m0[u] + e < g.M) {
                    const T *src = dY + ((int64_t)nn * g.F + f) * g.HoWo + rr;
                    bits = *reinterpret_cast<const U *>(src);
                    sum += Elem<T>::to_f32(*src);
                }
                o[u].v[e] = bits;
                if (++rr == (uint32_t)g.HoWo) {
                    rr = 0;
                    ++nn;
                }
            }
        }
        // 8 x 4 bytes does not fit one 16-byte store: write two halves for fp32
        if constexpr (sizeof(U) == 2) {
            *reinterpret_cast<VecOf<U, 8> *>(out + (int64_t)f * ld + m0[u]) = o[u];
        } else {
            VecOf<U, 4> a, b;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                a.v[e] = o[u].v[e];
                b.v[e] = o[u].v[4 + e];
            }
            *reinterpret_cast<VecOf<U, 4> *>(out + (int64_t)f * ld + m0[u]) = a;
            *reinterpret_cast<VecOf<U, 4> *>(out + (int64_t)f * ld + m0[u] + 4) = b;
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

// The same matrix with every output row padded with zeros to a multiple of 8 columns:
// column ((n*Ho + oy) * P8 + i) * 8 + e holds dY[n][f][oy][8i + e], P8 = ceil(Wo / 8).  A pack of 8 columns
// then never leaves its output row, which is what lets the model-gradient product read the matching
// entries of D-hat straight from X with one load per pack.  One thread per pack; bias partial sums as above.
__global__ __launch_bounds__(256) void pack_dyhat_rows_kernel(ConvGeom g, FastDiv div_p8, FastDiv div_Ho,
                                                              const bf16_t *__restrict__ dY, uint16_t *__restrict__ out,
                                                              int64_t ld, float *__restrict__ bias_partials)
{
    const int f = blockIdx.y;
    const bool can_vec = (int64_t)g.N * g.F * g.Ho * g.Wo >= 8;
    float sum = 0.f;
    int64_t pack[PACK_UNR];
    uint32_t i[PACK_UNR];
    const bf16_t *src[PACK_UNR];
    bool live[PACK_UNR], fast[PACK_UNR];
    int back[PACK_UNR];
    VecOf<uint16_t, 8> o[PACK_UNR];
#pragma unroll
    for (int u = 0; u < PACK_UNR; ++u) {
        pack[u] = ((int64_t)blockIdx.x * PACK_UNR + u) * 256 + threadIdx.x;
        uint32_t row, n, oy;
        div_p8.divmod((uint32_t)(pack[u] * 8 < ld ? pack[u] : 0), row, i[u]);
        div_Ho.divmod(row, n, oy);
        live[u] = pack[u] * 8 < ld && (int)n < g.N;
        src[u] = dY + (((int64_t)(live[u] ? n : 0) * g.F + f) * g.Ho + oy) * g.Wo + 8 * i[u];
        // a row's ragged last pack is read so that the 16 bytes END at the row's end (inside the tensor) and
        // shifted down afterwards, which zeroes its padding
        const int valid = g.Wo - 8 * (int)i[u];
        back[u] = valid < 8 ? 8 - valid : 0;
        fast[u] = can_vec && live[u] && (back[u] == 0 || g.Wo >= 8);
        if (can_vec) __builtin_memcpy(&o[u], fast[u] ? src[u] - back[u] : dY, 16);  // element-aligned 16-byte loads, issued together
    }
#pragma unroll
    for (int u = 0; u < PACK_UNR; ++u) {
        if (pack[u] * 8 >= ld) continue;
        if (fast[u]) {
            if (back[u]) {
                unsigned __int128 x;
                __builtin_memcpy(&x, &o[u], 16);
                x >>= 16 * back[u];
                __builtin_memcpy(&o[u], &x, 16);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) sum += bf16_to_f32(o[u].v[e]);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                uint16_t bits = 0;
                if (live[u] && 8 * (int)i[u] + e < g.Wo) {
                    bits = src[u][e];
                    sum += bf16_to_f32(bits);
                }
                o[u].v[e] = bits;
            }
        }
        *reinterpret_cast<VecOf<uint16_t, 8> *>(out + (int64_t)f * ld + pack[u] * 8) = o[u];
    }
    if (bias_partials != nullptr) {
        __shared__ float wave_sum[4];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) sum += __shfl_down(sum, off, 64);
        if ((threadIdx.x & 63) == 0) wave_sum[threadIdx.x >> 6] = sum;
        __syncthreads();
        if (threadIdx.x == 0)
            bias_partials[(int64_t)f * gridDim.x + blockIdx.x] = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
    }
}

// The padded unit is the output row, or the whole plane of an image where the direct model gradient
// works on planes: a plane is then handled as one long row.
static ConvGeom padded_unit_view(const ConvGeom &g)
{
    ConvGeom v = g;
    if (wgrad_direct_planes(g)) v.Wo = g.Ho * g.Wo, v.Ho = 1;
    return v;
}

int64_t dyhat_rows_ld(const ConvGeom &g)
{
    ConvGeom v = padded_unit_view(g);
    return round_up((int64_t)v.N * v.Ho * ((v.Wo + 7) / 8) * 8, 64);
}
int pack_dyhat_rows_blocks(const ConvGeom &g) { return (int)((dyhat_rows_ld(g) + PACK_COLS - 1) / PACK_COLS); }

int launch_pack_dyhat_rows(const ConvGeom &geom, const void *dY, void *dYhat, int64_t ld, float *bias_partials,
                           int bias_blocks, float *dbias, hipStream_t s)
{
    const ConvGeom g = padded_unit_view(geom);
    int blocks = (int)((ld + PACK_COLS - 1) / PACK_COLS);
    if (bias_partials != nullptr && bias_blocks != blocks) return OMNI_INVALID_ARGUMENT;
    dim3 grid((unsigned)blocks, (unsigned)g.F, 1);
    {
        ProfScope prof(KID_PACK_DYHAT, s, 0.0, 2.0 * g.F * (double)g.M * 2.0);
        hipLaunchKernelGGL(pack_dyhat_rows_kernel, grid, dim3(256), 0, s, g, FastDiv((uint32_t)((g.Wo + 7) / 8)),
                           FastDiv((uint32_t)g.Ho), (const bf16_t *)dY, (uint16_t *)dYhat, ld, bias_partials);
    }
    OMNI_LAUNCH_CHECK();
    if (bias_partials != nullptr && dbias != nullptr) {
        ProfScope prof(KID_BIAS_REDUCE, s, 0.0, 4.0 * g.F * (blocks + 1));
        hipLaunchKernelGGL(bias_reduce_kernel, dim3((unsigned)g.F), dim3(64), 0, s, bias_partials, blocks, dbias);
        OMNI_LAUNCH_CHECK();
    }
    return OMNI_OK;
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
    if (bias_partials != nullptr && dbias != nullptr) {
        ProfScope prof(KID_BIAS_REDUCE, s, 0.0, 4.0 * g.F * (blocks + 1));
        hipLaunchKernelGGL(bias_reduce_kernel, dim3((unsigned)g.F), dim3(64), 0, s, bias_partials, blocks, dbias);
        OMNI_LAUNCH_CHECK();
    }
    return OMNI_OK;
}

}  // namespace omni
