// Element-wise and window kernels (gfx950): the fused momentum-SGD update over a list of tensors,
// ReLU, and 2-D max-pooling.  All are bound by HBM traffic; each thread moves 16 bytes where the
// layout allows it and nothing uses floating point atomics.
#include <type_traits>

#include "common.h"

namespace omni {

// ------------------------------------------------------------------------------------------------
// Momentum SGD (Sec. II-B, Eq. (update2) then Eq. (update1)), many tensors per launch:
//   V <- mu*V - lr*(G + lambda*W);   W <- W + V;   optionally W_shadow <- bf16(W)
// The tensor table travels in the kernel arguments, so no device memory is needed for it.
// ------------------------------------------------------------------------------------------------
constexpr int SGD_MAX_TENSORS = 24;
constexpr int SGD_BLOCK_ELEMS = 256 * 4 * 4;  // 4 float4 per thread

struct SgdTable {
    float *W[SGD_MAX_TENSORS];
    float *V[SGD_MAX_TENSORS];
    const float *G[SGD_MAX_TENSORS];
    bf16_t *S[SGD_MAX_TENSORS];
    int64_t count[SGD_MAX_TENSORS];
    int32_t first_block[SGD_MAX_TENSORS + 1];  // prefix sum of blocks per tensor
    int32_t n;
};

__device__ __forceinline__ void sgd_one(float &w, float &v, float g, float lr, float mu, float wd)
{
    float step = g + wd * w;
    v = mu * v - lr * step;
    w = w + v;
}

__global__ __launch_bounds__(256) void sgd_kernel(SgdTable t, float lr, float mu, float wd)
{
    int b = blockIdx.x;
    int ti = 0;
    while (ti + 1 < t.n && b >= t.first_block[ti + 1]) ++ti;
    int64_t base = (int64_t)(b - t.first_block[ti]) * SGD_BLOCK_ELEMS;
    float *W = t.W[ti];
    float *V = t.V[ti];
    const float *G = t.G[ti];
    bf16_t *S = t.S[ti];
    int64_t count = t.count[ti];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        int64_t i = base + ((int64_t)q * 256 + threadIdx.x) * 4;
        if (i + 4 <= count) {
            float4 w = *reinterpret_cast<float4 *>(W + i);
            float4 v = *reinterpret_cast<float4 *>(V + i);
            float4 g = *reinterpret_cast<const float4 *>(G + i);
            sgd_one(w.x, v.x, g.x, lr, mu, wd);
            sgd_one(w.y, v.y, g.y, lr, mu, wd);
            sgd_one(w.z, v.z, g.z, lr, mu, wd);
            sgd_one(w.w, v.w, g.w, lr, mu, wd);
            *reinterpret_cast<float4 *>(W + i) = w;
            *reinterpret_cast<float4 *>(V + i) = v;
            if (S != nullptr) {
                uint2 p;
                p.x = f32x2_to_bf16x2(w.x, w.y);
                p.y = f32x2_to_bf16x2(w.z, w.w);
                *reinterpret_cast<uint2 *>(S + i) = p;
            }
        } else {
            for (int64_t j = i; j < count; ++j) {
                float w = W[j], v = V[j];
                sgd_one(w, v, G[j], lr, mu, wd);
                W[j] = w;
                V[j] = v;
                if (S != nullptr) S[j] = f32_to_bf16(w);
            }
        }
    }
}

int launch_sgd(int32_t n, float *const *W, float *const *V, const float *const *G, const int64_t *counts,
               void *const *shadow, float lr, float mu, float wd, hipStream_t s)
{
    int32_t done = 0;
    while (done < n) {
        SgdTable t;
        t.n = 0;
        t.first_block[0] = 0;
        while (done < n && t.n < SGD_MAX_TENSORS) {
            int64_t c = counts[done];
            if (c > 0) {
                int64_t blocks = (c + SGD_BLOCK_ELEMS - 1) / SGD_BLOCK_ELEMS;
                if (t.first_block[t.n] + blocks > 0x7fffffff) {
                    if (t.n == 0) return OMNI_UNSUPPORTED;
                    break;  // launch what is collected so far; this tensor starts the next table
                }
                t.W[t.n] = W[done];
                t.V[t.n] = V[done];
                t.G[t.n] = G[done];
                t.S[t.n] = shadow ? (bf16_t *)shadow[done] : nullptr;
                t.count[t.n] = c;
                t.first_block[t.n + 1] = t.first_block[t.n] + (int32_t)blocks;
                ++t.n;
            }
            ++done;
        }
        if (t.n == 0) continue;
        for (int i = t.n; i < SGD_MAX_TENSORS; ++i) {
            t.W[i] = t.V[i] = nullptr;
            t.G[i] = nullptr;
            t.S[i] = nullptr;
            t.count[i] = 0;
            t.first_block[i + 1] = t.first_block[t.n];
        }
        double params = 0, shadowed = 0;
        for (int i = 0; i < t.n; ++i) {
            params += (double)t.count[i];
            if (t.S[i]) shadowed += (double)t.count[i];
        }
        ProfScope prof(KID_SGD, s, 4.0 * params, 20.0 * params + 2.0 * shadowed);
        hipLaunchKernelGGL(sgd_kernel, dim3((unsigned)t.first_block[t.n]), dim3(256), 0, s, t, lr, mu, wd);
        OMNI_LAUNCH_CHECK();
    }
    return OMNI_OK;
}

// ------------------------------------------------------------------------------------------------
// ReLU
// ------------------------------------------------------------------------------------------------
template <typename T, bool BACKWARD>
__global__ __launch_bounds__(256) void relu_kernel(int64_t count, const T *ref, const T *dy, T *out)  // in place allowed: no restrict
{
    constexpr int VEC = 16 / sizeof(T);
    int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * VEC;
    if (i >= count) return;
    if (i + VEC <= count) {
        struct alignas(16) V { T v[VEC]; };
        V r = *reinterpret_cast<const V *>(ref + i);
        V o;
        if constexpr (BACKWARD) {
            V d = *reinterpret_cast<const V *>(dy + i);
#pragma unroll
            for (int e = 0; e < VEC; ++e) o.v[e] = Elem<T>::to_f32(r.v[e]) > 0.f ? d.v[e] : (T)0;
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) o.v[e] = Elem<T>::to_f32(r.v[e]) > 0.f ? r.v[e] : (T)0;
        }
        *reinterpret_cast<V *>(out + i) = o;
    } else {
        for (int64_t j = i; j < count; ++j) {
            bool pos = Elem<T>::to_f32(ref[j]) > 0.f;
            out[j] = pos ? (BACKWARD ? dy[j] : ref[j]) : (T)0;
        }
    }
}

int launch_relu(int dtype, bool backward, int64_t count, const void *ref, const void *dy, void *out, hipStream_t s)
{
    if (count == 0) return OMNI_OK;
    int vec = dtype == OMNI_BF16 ? 8 : 4;
    dim3 grid((unsigned)((count + 256 * (int64_t)vec - 1) / (256 * (int64_t)vec)));
    ProfScope prof(KID_RELU, s, 0.0, (backward ? 3.0 : 2.0) * count * elem_size(dtype));
    if (dtype == OMNI_BF16) {
        if (backward)
            hipLaunchKernelGGL((relu_kernel<bf16_t, true>), grid, dim3(256), 0, s, count, (const bf16_t *)ref, (const bf16_t *)dy, (bf16_t *)out);
        else
            hipLaunchKernelGGL((relu_kernel<bf16_t, false>), grid, dim3(256), 0, s, count, (const bf16_t *)ref, (const bf16_t *)nullptr, (bf16_t *)out);
    } else {
        if (backward)
            hipLaunchKernelGGL((relu_kernel<float, true>), grid, dim3(256), 0, s, count, (const float *)ref, (const float *)dy, (float *)out);
        else
            hipLaunchKernelGGL((relu_kernel<float, false>), grid, dim3(256), 0, s, count, (const float *)ref, (const float *)nullptr, (float *)out);
    }
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

// ------------------------------------------------------------------------------------------------
// Max-pool, k x k window, stride s, no padding, last window clipped at the border in ceil mode.
// ------------------------------------------------------------------------------------------------
static int g_pool_fwd_direct = 1;  // 0: the LDS kernel also for bf16 3 x 3 / stride 2 (tuning knob, for comparisons)

void set_pool_override(int lds) { g_pool_fwd_direct = lds ? 0 : 1; }

struct PoolGeom {
    int32_t H, W, Ho, Wo, k, s;
    FastDiv div_Wo, div_HoWo, div_W, div_HW, div_s;
    FastDiv div_rp, div_xb;  // row pairs per plane, 8-pixel blocks per row (backward, 3 x 3 / stride 2)
};

// Output as the "rows" form of a gradient [N][C][plane] that the model-gradient kernels read: a matrix
// [C][ld] in which plane (n, c) starts at column n * pitch (pitch = the plane's size rounded up to 8
// elements, the round-up zero).  sums (optional): [C][N], the sum of every plane's stored values.
struct RowsOut {
    int64_t ld;
    int32_t pitch, N;
    FastDiv div_C;
    float *sums;
};

template <typename T>
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(PoolGeom g, int64_t plane0, uint32_t count,
                                                          const T *__restrict__ x, T *__restrict__ y,
                                                          uint8_t *__restrict__ argmax)
{
    // One launch covers `count` < 2^31 outputs starting at plane plane0.
    uint32_t local = blockIdx.x * 256u + threadIdx.x;
    if (local >= count) return;
    uint32_t pl, o, oy, ox;
    g.div_HoWo.divmod(local, pl, o);
    g.div_Wo.divmod(o, oy, ox);
    int64_t plane = plane0 + pl;
    const T *src = x + plane * g.H * g.W;
    int best = -1;
    float bv = 0.f;
    T braw = (T)0;
    for (int ky = 0; ky < g.k; ++ky) {
        int iy = (int)oy * g.s + ky;
        if (iy >= g.H) break;
        for (int kx = 0; kx < g.k; ++kx) {
            int ix = (int)ox * g.s + kx;
            if (ix >= g.W) break;
            T raw = src[iy * g.W + ix];
            float v = Elem<T>::to_f32(raw);
            if (best < 0 || v > bv) {  // strict: the first maximum in scan order wins
                best = ky * g.k + kx;
                bv = v;
                braw = raw;
            }
        }
    }
    int64_t out = plane * g.Ho * g.Wo + o;
    y[out] = braw;
    if (argmax != nullptr) argmax[out] = (uint8_t)best;
}

// Gather form: each input pixel collects the gradient of every window that elected it, in
// ascending (oy, ox) order, in fp32.
template <typename T, bool RELU>  // RELU: a window routes its gradient only if its pooled value y is > 0
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(PoolGeom g, int64_t plane0, uint32_t count,
                                                          const T *__restrict__ dy, const uint8_t *__restrict__ argmax,
                                                          const T *__restrict__ y, T *__restrict__ dx)
{
    uint32_t local = blockIdx.x * 256u + threadIdx.x;
    if (local >= count) return;
    uint32_t pl, p, iy, ix;
    g.div_HW.divmod(local, pl, p);
    g.div_W.divmod(p, iy, ix);
    int64_t plane = plane0 + pl;
    // windows oy with oy*s <= iy <= oy*s + k - 1, clipped to the pooled extent (multiply-high divisions)
    int oy_lo = (int)iy - g.k + 1;
    oy_lo = oy_lo <= 0 ? 0 : (int)g.div_s.div((uint32_t)(oy_lo + g.s - 1));
    int oy_hi = (int)g.div_s.div(iy);
    if (oy_hi > g.Ho - 1) oy_hi = g.Ho - 1;
    int ox_lo = (int)ix - g.k + 1;
    ox_lo = ox_lo <= 0 ? 0 : (int)g.div_s.div((uint32_t)(ox_lo + g.s - 1));
    int ox_hi = (int)g.div_s.div(ix);
    if (ox_hi > g.Wo - 1) ox_hi = g.Wo - 1;
    const int64_t obase = plane * g.Ho * g.Wo;
    float acc = 0.f;
    for (int oy = oy_lo; oy <= oy_hi; ++oy)
        for (int ox = ox_lo; ox <= ox_hi; ++ox) {
            int code = ((int)iy - oy * g.s) * g.k + ((int)ix - ox * g.s);
            int64_t o = obase + (int64_t)oy * g.Wo + ox;
            bool hit = argmax[o] == (uint8_t)code;
            if constexpr (RELU) hit = hit && Elem<T>::to_f32(y[o]) > 0.f;
            if (hit) acc += Elem<T>::to_f32(dy[o]);
        }
    dx[plane * g.H * g.W + p] = Elem<T>::from_f32(acc);
}

// LDS-staged variants.  A workgroup takes a few whole planes; their pixels are one contiguous run in
// memory, fetched 16 bytes per lane into LDS (the run need not be 16-byte aligned; dst must be), and every window is
// then evaluated from LDS.  Global traffic is each operand once, in full vectors.
template <typename T>
__device__ __forceinline__ void run_to_lds(const T *__restrict__ src, int count, T *dst, int tid)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr int VEC = 16 / (int)sizeof(T);
    constexpr int U = 4;  // loads in flight per thread
    const int full = count / VEC;
    if (full == 0) {
        if (tid < count) dst[tid] = src[tid];
        return;
    }
    // The ragged end: the last VEC elements once more, as a piece moved back to end at the run's end.
    // Issued first, stored last (the same values land on the bytes it shares with the last whole piece).
    u32x4 tail = {0, 0, 0, 0};
    const bool ragged = full * VEC < count && tid == 255;
    if (ragged) __builtin_memcpy(&tail, src + (count - VEC), 16);
    // Whole pieces, ceil(full / 256) per thread, in batches of up to U: all loads of a batch are issued
    // before the first is waited for.  A piece index past the end is clamped to the last piece (the
    // duplicate rewrites the same bytes), so neither the loads nor the LDS stores sit behind a per-thread
    // branch; the batch size is the same for the whole workgroup.
    auto batch = [&](auto n_tag, int first) {
        constexpr int N = decltype(n_tag)::value;
        u32x4 v[N];
        int c[N];
#pragma unroll
        for (int u = 0; u < N; ++u) {
            c[u] = tid + 256 * (first + u) < full ? tid + 256 * (first + u) : full - 1;
            __builtin_memcpy(&v[u], src + c[u] * VEC, 16);
        }
#pragma unroll
        for (int u = 0; u < N; ++u) *reinterpret_cast<u32x4 *>(dst + c[u] * VEC) = v[u];
    };
    const int per = (full + 255) / 256;
    for (int b = 0; b < per; b += U) {
        switch (per - b < U ? per - b : U) {
        case 1: batch(std::integral_constant<int, 1>(), b); break;
        case 2: batch(std::integral_constant<int, 2>(), b); break;
        case 3: batch(std::integral_constant<int, 3>(), b); break;
        default: batch(std::integral_constant<int, 4>(), b); break;
        }
    }
    if (ragged) {
        T t[VEC];
        __builtin_memcpy(t, &tail, 16);
#pragma unroll
        for (int e = 0; e < VEC; ++e) dst[count - VEC + e] = t[e];
    }
}

// K3S2: the 3 x 3 / stride 2 pool of the paper's networks with its loops unrolled and its divisions as shifts
template <typename T, bool K3S2>
__global__ __launch_bounds__(256) void maxpool_fwd_lds_kernel(PoolGeom g, int64_t planes, int pb,
                                                              const T *__restrict__ x, T *__restrict__ y,
                                                              uint8_t *__restrict__ argmax)
{
    extern __shared__ __align__(16) unsigned char pool_smem[];
    T *tile = reinterpret_cast<T *>(pool_smem);
    const int64_t p0 = (int64_t)blockIdx.x * pb;
    const int np = (int)(planes - p0 < pb ? planes - p0 : pb);
    const int hw = g.H * g.W, howo = g.Ho * g.Wo;
    run_to_lds(x + p0 * hw, np * hw, tile, threadIdx.x);
    __syncthreads();
    for (int o = threadIdx.x; o < np * howo; o += 256) {
        uint32_t pl, r, oy, ox;
        g.div_HoWo.divmod((uint32_t)o, pl, r);
        g.div_Wo.divmod(r, oy, ox);
        const T *src = tile + pl * hw;
        int best = -1;
        float bv = 0.f;
        T braw = (T)0;
        if constexpr (K3S2) {
            // nine reads at coordinates clamped into the plane (no read sits behind a branch), then the scan
            // in window order over the pixels that are really inside; the first pixel always is
            const int y0 = (int)oy * 2, x0 = (int)ox * 2;
            T raw[9];

#pragma unroll
            for (int ky = 0; ky < 3; ++ky)
#pragma unroll
                for (int kx = 0; kx < 3; ++kx) {
                    const int iy = y0 + ky < g.H ? y0 + ky : g.H - 1, ix = x0 + kx < g.W ? x0 + kx : g.W - 1;
                    raw[ky * 3 + kx] = src[iy * g.W + ix];
                }
            best = 0;
            braw = raw[0];
            bv = Elem<T>::to_f32(raw[0]);
#pragma unroll
            for (int k = 1; k < 9; ++k) {
                const bool in = y0 + k / 3 < g.H && x0 + k % 3 < g.W;
                const float v = Elem<T>::to_f32(raw[k]);
                const bool take = in && v > bv;  // strict: the first maximum in scan order wins
                best = take ? k : best;
                bv = take ? v : bv;
                braw = take ? raw[k] : braw;
            }
        } else {
            for (int ky = 0; ky < g.k; ++ky) {
                int iy = (int)oy * g.s + ky;
                if (iy >= g.H) break;
                for (int kx = 0; kx < g.k; ++kx) {
                    int ix = (int)ox * g.s + kx;
                    if (ix >= g.W) break;
                    T raw = src[iy * g.W + ix];
                    float v = Elem<T>::to_f32(raw);
                    if (best < 0 || v > bv) {  // strict: the first maximum in scan order wins
                        best = ky * g.k + kx;
                        bv = v;
                        braw = raw;
                    }
                }
            }
        }
        y[p0 * howo + o] = braw;
        if (argmax != nullptr) argmax[p0 * howo + o] = (uint8_t)best;
    }
}

// 3 x 3 / stride 2 forward pool on bf16 planes without LDS.  One thread = 2 output rows x 3 output columns of a
// plane: the 5 input rows x 7 input columns under them arrive as five element-aligned 16-byte loads (all issued
// before the first is used; neighbouring threads' loads overlap in the cache, not in memory), positions outside the
// plane (clipped last windows, missing rows) become -inf, every value is widened once, and each window is scanned
// in window order with a strict comparison, so the first maximum wins as in the definition.  About 83 vector
// instructions per output against 117 in the LDS kernel; both are bound by issuing them.
__global__ __launch_bounds__(256) void maxpool_fwd_k3s2_bf16_kernel(PoolGeom g, FastDiv div_tasks, FastDiv div_tx, uint32_t total_tasks,
                                                                    int64_t total_elems, const bf16_t *__restrict__ x,
                                                                    bf16_t *__restrict__ y, uint8_t *__restrict__ argmax)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const uint32_t task = blockIdx.x * 256u + threadIdx.x;
    if (task >= total_tasks) return;
    uint32_t pl, rest, ty, tx;
    div_tasks.divmod(task, pl, rest);
    div_tx.divmod(rest, ty, tx);
    const int iy0 = 4 * (int)ty, ix0 = 6 * (int)tx;
    const int64_t base = (int64_t)pl * g.H * g.W + (int64_t)iy0 * g.W + ix0;
    // loads; a piece that would run past the end of the tensor is moved back to end there and shifted down afterwards
    u32x4 w[5];
    int shift[5];
#pragma unroll
    for (int j = 0; j < 5; ++j) {
        int64_t at = base + (int64_t)j * g.W;
        const bool row_ok = iy0 + j < g.H;
        if (!row_ok) at = base;
        const int64_t last = total_elems - 8;
        shift[j] = at > last ? (int)(at - last) : 0;
        at = at > last ? last : at;
        __builtin_memcpy(&w[j], x + at, 16);
    }
    // 16-bit lanes of columns inside the plane
    uint32_t keep[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
        keep[q] = (ix0 + 2 * q < g.W ? 0x0000ffffu : 0u) | (ix0 + 2 * q + 1 < g.W && 2 * q + 1 < 7 ? 0xffff0000u : 0u);
    constexpr uint32_t NINF2 = 0xff80ff80u;  // two bf16 -inf
    float v[5][7];
#pragma unroll
    for (int j = 0; j < 5; ++j) {
        if (shift[j] != 0) {  // last rows of the last plane only
            unsigned __int128 t;
            __builtin_memcpy(&t, &w[j], 16);
            t >>= 16 * shift[j];
            __builtin_memcpy(&w[j], &t, 16);
        }
        const bool row_ok = iy0 + j < g.H;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t m = row_ok ? keep[q] : 0u;
            const uint32_t word = (w[j][q] & m) | (NINF2 & ~m);
            v[j][2 * q] = __uint_as_float(word << 16);
            if (2 * q + 1 < 7) v[j][2 * q + 1] = __uint_as_float(word & 0xffff0000u);
        }
    }
    const int howo = g.Ho * g.Wo;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int oy = 2 * (int)ty + r;
        if (oy >= g.Ho) break;
        uint32_t bits[3], code[3];
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            float bv = v[2 * r][2 * c];
            int best = 0;
#pragma unroll
            for (int k = 1; k < 9; ++k) {
                const float cand = v[2 * r + k / 3][2 * c + k % 3];
                const bool take = cand > bv;  // strict: the first maximum in scan order wins; -inf is never taken
                best = take ? k : best;
                bv = take ? cand : bv;
            }
            bits[c] = __float_as_uint(bv) >> 16;
            code[c] = (uint32_t)best;
        }
        const int ox0 = 3 * (int)tx, n = g.Wo - ox0 < 3 ? g.Wo - ox0 : 3;
        bf16_t *yo = y + (int64_t)pl * howo + oy * g.Wo + ox0;
        if (n >= 2) {
            const uint32_t two = bits[0] | (bits[1] << 16);
            __builtin_memcpy(yo, &two, 4);
            if (n == 3) yo[2] = (bf16_t)bits[2];
        } else {
            yo[0] = (bf16_t)bits[0];
        }
        if (argmax != nullptr) {
            uint8_t *ao = argmax + (int64_t)pl * howo + oy * g.Wo + ox0;
            if (n >= 2) {
                const uint16_t two = (uint16_t)(code[0] | (code[1] << 8));
                __builtin_memcpy(ao, &two, 2);
                if (n == 3) ao[2] = (uint8_t)code[2];
            } else {
                ao[0] = (uint8_t)code[0];
            }
        }
    }
}

// N consecutive results to element-aligned memory in as few store instructions as possible.  16-bit
// results are first packed two to a register: left to itself the compiler stores some of them one by one
// (to save the packing), which multiplies the write requests the memory system has to merge again.
template <int N, typename T>
__device__ __forceinline__ void store_packed(T *dst, const T *src)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    if constexpr (sizeof(T) == 2 && N == 8) {
        u32x4 w;
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = (uint32_t)src[2 * i] | ((uint32_t)src[2 * i + 1] << 16);
        __builtin_memcpy(dst, &w, 16);
    } else if constexpr (sizeof(T) == 2 && N == 4) {
        u32x2 w;
#pragma unroll
        for (int i = 0; i < 2; ++i) w[i] = (uint32_t)src[2 * i] | ((uint32_t)src[2 * i + 1] << 16);
        __builtin_memcpy(dst, &w, 8);
    } else if constexpr (sizeof(T) == 2 && N == 2) {
        uint32_t w = (uint32_t)src[0] | ((uint32_t)src[1] << 16);
        __builtin_memcpy(dst, &w, 4);
    } else {
        __builtin_memcpy(dst, src, N * sizeof(T));
    }
}

// 3 x 3 / stride 2 backward from the staged gradients and winners of np planes.
// One task = input rows 2t, 2t+1 x pixels 8b .. 8b+7 of a plane.  The windows that can hold them
// are output rows t-1, t x columns 4b-1 .. 4b+3: ten (winner, gradient) pairs read once, and for
// every pixel the candidate windows and the winner code each would have follow from the pixel's
// parities, known at compile time.  Contributions are added in ascending (oy, ox).
// ROWS: `out` is the rows matrix, the group's first plane is plane0 (plane = n * C + c), every task leaves the
// sum of what it stored in tsum[task], and the planes' zero round-ups are written as well.
template <typename T, bool ROWS = false>
__device__ __forceinline__ void pool_bwd_k3s2_tasks(const PoolGeom &g, int np, const T *gdy, const uint8_t *gam,
                                                    T *__restrict__ out, int hw, int howo, const RowsOut *ro = nullptr,
                                                    int64_t plane0 = 0, float *tsum = nullptr)
{
    const int rp = (g.H + 1) >> 1, xb = (g.W + 7) >> 3;
    const int tasks = np * rp * xb;
    auto plane_ptr = [&](int pl) -> T * {
        if constexpr (ROWS) {
            uint32_t n, c;
            ro->div_C.divmod((uint32_t)(plane0 + pl), n, c);
            return out + (int64_t)c * ro->ld + (int64_t)n * ro->pitch;
        } else {
            return out + pl * hw;
        }
    };
    if constexpr (ROWS) {
        const int tail = ro->pitch - hw;
        for (int i = threadIdx.x; i < np * tail; i += 256) plane_ptr(i / tail)[hw + i % tail] = (T)0;
    }
    for (int task = threadIdx.x; task < tasks; task += 256) {
        uint32_t rest, b, pl, t;
        g.div_xb.divmod((uint32_t)task, rest, b);
        g.div_rp.divmod(rest, pl, t);
        const int obase = (int)pl * howo, ox0 = 4 * (int)b - 1;
        float d[2][5];
        int code[2][5];
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int q = 0; q < 5; ++q) {
                const int oy = (int)t - 1 + r, ox = ox0 + q;
                const bool ok = oy >= 0 && oy < g.Ho && ox >= 0 && ox < g.Wo;
                const int o = ok ? obase + oy * g.Wo + ox : obase;
                code[r][q] = ok ? (int)gam[o] : 255;
                d[r][q] = Elem<T>::to_f32(gdy[o]);
            }
        T res[2][8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int q = (e >> 1) + 1;  // the window column that starts at or just left of this pixel
            float top = 0.f, bot = 0.f;  // input rows 2t and 2t+1
            if ((e & 1) == 0) {
                top += code[0][q - 1] == 8 ? d[0][q - 1] : 0.f;
                top += code[0][q] == 6 ? d[0][q] : 0.f;
                top += code[1][q - 1] == 2 ? d[1][q - 1] : 0.f;
                top += code[1][q] == 0 ? d[1][q] : 0.f;
                bot += code[1][q - 1] == 5 ? d[1][q - 1] : 0.f;
                bot += code[1][q] == 3 ? d[1][q] : 0.f;
            } else {
                top += code[0][q] == 7 ? d[0][q] : 0.f;
                top += code[1][q] == 1 ? d[1][q] : 0.f;
                bot += code[1][q] == 4 ? d[1][q] : 0.f;
            }
            res[0][e] = Elem<T>::from_f32(top);
            res[1][e] = Elem<T>::from_f32(bot);
        }
        const int x0 = 8 * (int)b, nv = g.W - x0 < 8 ? g.W - x0 : 8;
        if constexpr (ROWS) {
            float ts = 0.f;  // of the stored (rounded) values, in the order row, pixel
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (2 * (int)t + r < g.H && e < nv) ts += Elem<T>::to_f32(res[r][e]);
            tsum[task] = ts;
        }
        T *plane = plane_ptr((int)pl);
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int iy = 2 * (int)t + r;
            if (iy >= g.H) break;
            T *row = plane + iy * g.W + x0;
            if (nv == 8) {
                store_packed<8>(row, res[r]);  // element-aligned stores
            } else {
                // 4, 2 and 1 pixels as nv's bits say; positions spelled out so that res stays in registers
                if (nv & 4) store_packed<4>(row, res[r]);
                if ((nv & 6) == 6) store_packed<2>(row + 4, res[r] + 4);
                if ((nv & 6) == 2) store_packed<2>(row, res[r]);
#pragma unroll
                for (int at = 0; at < 8; at += 2)
                    if ((nv & 1) && (nv & 6) == at) row[at] = res[r][at];
            }
        }
    }
}

// Persistent form of the 3 x 3 / stride 2 backward pass.  A workgroup walks groups of pb planes with the
// grid's stride; the loads of its next group (gradient, pooled values, winners: 16-byte pieces held in
// registers) are issued before the current group is computed and stored, so every resident workgroup has
// reads in flight all the time instead of only during its load phase.  Requires 16 <= pb * Ho*Wo <= 4096
// for every group (the host checks, also for the last, smaller group).
template <typename T, bool RELU, bool ROWS = false>
__global__ __launch_bounds__(256) void maxpool_bwd_k3s2_kernel(PoolGeom g, int64_t planes, int pb,
                                                               const T *__restrict__ dy, const uint8_t *__restrict__ argmax,
                                                               const T *__restrict__ y, T *__restrict__ dx, RowsOut ro)
{
    extern __shared__ __align__(16) unsigned char pool_smem[];
    constexpr int VEC = 16 / (int)sizeof(T);
    constexpr int MAXC = 4096 / VEC / 256;
    const int hw = g.H * g.W, howo = g.Ho * g.Wo;
    const int64_t groups = (planes + pb - 1) / pb;
    T *gdy = reinterpret_cast<T *>(pool_smem);
    uint8_t *gam = pool_smem + (((size_t)pb * howo * sizeof(T) + 15) / 16) * 16;
    float *tsum = reinterpret_cast<float *>(gam + (((size_t)pb * howo + 15) / 16) * 16);  // ROWS: one float per task
    T d[MAXC][VEC], v[MAXC][VEC];
    uint8_t a[16];
    int at[MAXC], aat = 0, n = 0;
    // A piece that would stick out of the group's run is moved back to end at the run's end: it then
    // overlaps its neighbour, and both write the same values to the same LDS bytes.
    auto load = [&](int64_t grp) {
        const int64_t p0 = grp * pb;
        n = (int)(planes - p0 < pb ? planes - p0 : pb) * howo;
        const T *dp = dy + p0 * howo, *yp = y + p0 * howo;
#pragma unroll
        for (int u = 0; u < MAXC; ++u) {
            const int c = (int)threadIdx.x + 256 * u;
            at[u] = c * VEC + VEC <= n ? c * VEC : n - VEC;
            __builtin_memcpy(d[u], dp + at[u], sizeof(d[u]));
            if constexpr (RELU) __builtin_memcpy(v[u], yp + at[u], sizeof(v[u]));
        }
        aat = (int)threadIdx.x * 16 + 16 <= n ? (int)threadIdx.x * 16 : n - 16;
        __builtin_memcpy(a, argmax + p0 * howo + aat, 16);
    };
    int64_t grp = blockIdx.x;
    if (grp >= groups) return;
    load(grp);
    for (;;) {
        const int np = n / howo;
#pragma unroll
        for (int u = 0; u < MAXC; ++u) {
            const int c = (int)threadIdx.x + 256 * u;
            if (c * VEC >= n) continue;
            // the pooled value is the winner's value: where it is not positive the ReLU under the pool
            // passes nothing, so that window's gradient is dropped while it is staged
            if constexpr (RELU) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) d[u][e] = Elem<T>::to_f32(v[u][e]) > 0.f ? d[u][e] : (T)0;
            }
            if (at[u] == c * VEC) {
                __builtin_memcpy(__builtin_assume_aligned(gdy + c * VEC, 16), d[u], sizeof(d[u]));
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) gdy[at[u] + e] = d[u][e];
            }
        }
        if ((int)threadIdx.x * 16 < n) {
            if (aat == (int)threadIdx.x * 16) {
                __builtin_memcpy(__builtin_assume_aligned(gam + aat, 16), a, 16);
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) gam[aat + e] = a[e];
            }
        }
        __syncthreads();
        const int64_t next = grp + gridDim.x;
        if (next < groups) load(next);
        if constexpr (ROWS) {
            pool_bwd_k3s2_tasks<T, true>(g, np, gdy, gam, dx, hw, howo, &ro, grp * pb, tsum);
            __syncthreads();  // the staged group has been read by everyone, and every task's sum is there
            if (ro.sums != nullptr) {
                // 16 lanes per plane: lane k adds the plane's tasks k, k + 16, ... in that order, then a fixed tree
                // over the 16 lanes (the same order every run; one thread per plane would walk all tasks alone
                // while the workgroup waits)
                const int per = ((g.H + 1) >> 1) * ((g.W + 7) >> 3);
                const int k = threadIdx.x & 15;
                for (int pl0 = 0; pl0 < np; pl0 += 16) {   // uniform trip count: the shuffles need every lane
                    const int pl = pl0 + (int)(threadIdx.x >> 4);
                    float acc = 0.f;
                    if (pl < np)
                        for (int j = k; j < per; j += 16) acc += tsum[pl * per + j];
#pragma unroll
                    for (int off = 8; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 16);
                    if (pl < np && k == 0) {
                        uint32_t nn, c;
                        ro.div_C.divmod((uint32_t)(grp * pb + pl), nn, c);
                        ro.sums[(int64_t)c * ro.N + nn] = acc;
                    }
                }
            }
            // tsum is next written after the next group's staging barrier, which the summing threads join
            if (next >= groups) break;
        } else {
            pool_bwd_k3s2_tasks<T>(g, np, gdy, gam, dx + grp * pb * hw, hw, howo);
            if (next >= groups) break;
            __syncthreads();  // the staged group has been read by everyone
        }
        grp = next;
    }
}

template <typename T, bool RELU, bool K3S2>
__global__ __launch_bounds__(256) void maxpool_bwd_lds_kernel(PoolGeom g, int64_t planes, int pb,
                                                              const T *__restrict__ dy, const uint8_t *__restrict__ argmax,
                                                              const T *__restrict__ y, T *__restrict__ dx)
{
    extern __shared__ __align__(16) unsigned char pool_smem[];
    constexpr int VEC = 16 / (int)sizeof(T);
    const int64_t p0 = (int64_t)blockIdx.x * pb;
    const int np = (int)(planes - p0 < pb ? planes - p0 : pb);
    const int hw = g.H * g.W, howo = g.Ho * g.Wo;
    T *gdy = reinterpret_cast<T *>(pool_smem);
    uint8_t *gam = pool_smem + (((size_t)pb * howo * sizeof(T) + 15) / 16) * 16;
    const int n = np * howo;
    constexpr int MAXC = 4096 / VEC / 256;  // 16-byte pieces of dy (and y) per thread when n <= 4096
    if (n <= 4096 && n >= 16) {
        // All of the run's loads go out before the first is waited for (one memory latency, not one per
        // operand and loop trip).  A piece that would stick out of the run is moved back to end at the
        // run's end: it then overlaps its neighbour, and both write the same values to the same LDS bytes.
        const T *dp = dy + p0 * howo, *yp = y + p0 * howo;
        const uint8_t *ap = argmax + p0 * howo;
        T d[MAXC][VEC], v[MAXC][VEC];
        uint8_t a[16];
        int at[MAXC];
#pragma unroll
        for (int u = 0; u < MAXC; ++u) {
            const int c = (int)threadIdx.x + 256 * u;
            at[u] = c * VEC + VEC <= n ? c * VEC : n - VEC;
            __builtin_memcpy(d[u], dp + at[u], sizeof(d[u]));
            if constexpr (RELU) __builtin_memcpy(v[u], yp + at[u], sizeof(v[u]));
        }
        const int aat = (int)threadIdx.x * 16 + 16 <= n ? (int)threadIdx.x * 16 : n - 16;
        __builtin_memcpy(a, ap + aat, 16);
#pragma unroll
        for (int u = 0; u < MAXC; ++u) {
            const int c = (int)threadIdx.x + 256 * u;
            if (c * VEC >= n) continue;
            // the pooled value is the winner's value: where it is not positive the ReLU under the pool
            // passes nothing, so that window's gradient is dropped while it is staged
            if constexpr (RELU) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) d[u][e] = Elem<T>::to_f32(v[u][e]) > 0.f ? d[u][e] : (T)0;
            }
            if (at[u] == c * VEC) {
                __builtin_memcpy(__builtin_assume_aligned(gdy + c * VEC, 16), d[u], sizeof(d[u]));
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) gdy[at[u] + e] = d[u][e];
            }
        }
        if ((int)threadIdx.x * 16 < n) {
            if (aat == (int)threadIdx.x * 16) {
                __builtin_memcpy(__builtin_assume_aligned(gam + aat, 16), a, 16);
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) gam[aat + e] = a[e];
            }
        }
    } else {
        run_to_lds(argmax + p0 * howo, n, gam, threadIdx.x);
        if constexpr (RELU) {
            const T *yp = y + p0 * howo, *dp = dy + p0 * howo;
            const int chunks = (n + VEC - 1) / VEC;
            for (int c = threadIdx.x; c < chunks; c += 256) {
                if ((c + 1) * VEC <= n) {
                    T v[VEC], d[VEC];
                    __builtin_memcpy(v, yp + c * VEC, sizeof(v));
                    __builtin_memcpy(d, dp + c * VEC, sizeof(d));
#pragma unroll
                    for (int e = 0; e < VEC; ++e) d[e] = Elem<T>::to_f32(v[e]) > 0.f ? d[e] : (T)0;
                    __builtin_memcpy(__builtin_assume_aligned(gdy + c * VEC, 16), d, sizeof(d));
                } else {
                    for (int e = 0; c * VEC + e < n; ++e)
                        gdy[c * VEC + e] = Elem<T>::to_f32(yp[c * VEC + e]) > 0.f ? dp[c * VEC + e] : (T)0;
                }
            }
        } else {
            run_to_lds(dy + p0 * howo, n, gdy, threadIdx.x);
        }
    }
    __syncthreads();
    if constexpr (K3S2) {
        pool_bwd_k3s2_tasks<T>(g, np, gdy, gam, dx + p0 * hw, hw, howo);
        return;
    }
    // each thread produces VEC consecutive pixels of the workgroup's run of planes and stores them at once
    T *out = dx + p0 * hw;
    const int total = np * hw;
    for (int v0 = threadIdx.x * VEC; v0 < total; v0 += 256 * VEC) {
        uint32_t pl, p, iy, ix;
        g.div_HW.divmod((uint32_t)v0, pl, p);
        g.div_W.divmod(p, iy, ix);
        T res[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            float acc = 0.f;
            if (v0 + e < total) {
                const int obase = (int)pl * howo;
                {
                    int oy_lo = (int)iy - g.k + 1;
                    oy_lo = oy_lo <= 0 ? 0 : (int)g.div_s.div((uint32_t)(oy_lo + g.s - 1));
                    int oy_hi = (int)g.div_s.div(iy);
                    if (oy_hi > g.Ho - 1) oy_hi = g.Ho - 1;
                    int ox_lo = (int)ix - g.k + 1;
                    ox_lo = ox_lo <= 0 ? 0 : (int)g.div_s.div((uint32_t)(ox_lo + g.s - 1));
                    int ox_hi = (int)g.div_s.div(ix);
                    if (ox_hi > g.Wo - 1) ox_hi = g.Wo - 1;
                    for (int oy = oy_lo; oy <= oy_hi; ++oy)
                        for (int ox = ox_lo; ox <= ox_hi; ++ox) {
                            int code = ((int)iy - oy * g.s) * g.k + ((int)ix - ox * g.s);
                            int o = obase + oy * g.Wo + ox;
                            if (gam[o] == (uint8_t)code) acc += Elem<T>::to_f32(gdy[o]);
                        }
                }
            }
            res[e] = Elem<T>::from_f32(acc);
            if (++ix == (uint32_t)g.W) {
                ix = 0;
                if (++iy == (uint32_t)g.H) iy = 0, ++pl;
            }
        }
        if (v0 + VEC <= total) {
            store_packed<VEC>(out + v0, res);  // element-aligned 16-byte store
        } else {
            for (int e = 0; v0 + e < total; ++e) out[v0 + e] = res[e];
        }
    }
}

// planes per workgroup for the LDS variants (0: a single plane does not fit, use the direct kernels)
static int pool_planes_per_block(int64_t plane_bytes, int64_t plane_elems, int64_t target_elems = 4096)
{
    const int64_t budget = 32 * 1024;
    if (plane_bytes > 2 * budget) return 0;
    int64_t pb = target_elems / plane_elems;
    if (pb < 1) pb = 1;
    while (pb > 1 && pb * plane_bytes > budget) --pb;
    return (int)pb;
}

// 3 x 3 / stride 2 backward: the planes per workgroup that keep its 256 threads busiest (a plane is
// ceil(H/2) * ceil(W/8) tasks), within the LDS budget and four passes of the threads.
static int pool_bwd_planes_k3s2(int H, int W, int64_t plane_bytes, int64_t howo)
{
    const int tasks = ((H + 1) / 2) * ((W + 7) / 8);
    int best = 0;
    double best_fill = 0.0;
    for (int pb = 1; pb <= 64; ++pb) {
        if (pb * plane_bytes > 32 * 1024 || (pb > 1 && (pb * tasks > 1024 || pb * howo > 4096))) break;
        double fill = (double)(pb * tasks) / (double)((pb * tasks + 255) / 256 * 256);
        if (fill >= best_fill) best = pb, best_fill = fill;
    }
    return best;
}

static PoolGeom make_pool_geom(int32_t H, int32_t W, int32_t k, int32_t stride, int32_t ceil_mode)
{
    PoolGeom g;
    g.H = H;
    g.W = W;
    g.k = k;
    g.s = stride;
    g.Ho = omni_pool_output_dim(H, k, stride, ceil_mode);
    g.Wo = omni_pool_output_dim(W, k, stride, ceil_mode);
    g.div_Wo = FastDiv((uint32_t)g.Wo);
    g.div_HoWo = FastDiv((uint32_t)(g.Ho * g.Wo));
    g.div_W = FastDiv((uint32_t)W);
    g.div_HW = FastDiv((uint32_t)(H * W));
    g.div_s = FastDiv((uint32_t)stride);
    g.div_rp = FastDiv((uint32_t)((H + 1) / 2));
    g.div_xb = FastDiv((uint32_t)((W + 7) / 8));
    return g;
}

int launch_maxpool_fwd(int dtype, int64_t planes, int32_t H, int32_t W, int32_t k, int32_t stride, int32_t ceil_mode,
                       const void *x, void *y, uint8_t *argmax, hipStream_t s)
{
    PoolGeom g = make_pool_geom(H, W, k, stride, ceil_mode);
    int64_t per = (int64_t)g.Ho * g.Wo;
    int64_t planes_per_launch = (0x7fffffffll - 4096) / per;
    ProfScope prof(KID_POOL_FWD, s, 0.0, (double)planes * ((double)H * W + per) * elem_size(dtype) + (argmax ? (double)planes * per : 0.0));
    const int64_t hw = (int64_t)H * W;
    if (dtype == OMNI_BF16 && k == 3 && stride == 2 && g_pool_fwd_direct) {
        const int64_t txn = (g.Wo + 2) / 3, tasks = txn * ((g.Ho + 1) / 2), total = planes * tasks;
        if (total <= 0x7fffffffll && planes * hw >= 8) {
            hipLaunchKernelGGL(maxpool_fwd_k3s2_bf16_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, g,
                               FastDiv((uint32_t)tasks), FastDiv((uint32_t)txn), (uint32_t)total, planes * hw, (const bf16_t *)x,
                               (bf16_t *)y, argmax);
            OMNI_LAUNCH_CHECK();
            return OMNI_OK;
        }
    }
    // about 16 KB of input per workgroup (measured best on the 55 x 55 planes: 8192 elements 60 us, 4096 72 us)
    int pb = pool_planes_per_block(hw * (int64_t)elem_size(dtype), hw, 8192);
    if (pb > 0 && (planes + pb - 1) / pb <= 0x7fffffffll) {
        dim3 grid((unsigned)((planes + pb - 1) / pb));
        size_t lds = (size_t)pb * hw * elem_size(dtype) + 16;
        if (dtype == OMNI_BF16)
            if (k == 3 && stride == 2)
                hipLaunchKernelGGL((maxpool_fwd_lds_kernel<bf16_t, true>), grid, dim3(256), lds, s, g, planes, pb, (const bf16_t *)x, (bf16_t *)y, argmax);
            else
                hipLaunchKernelGGL((maxpool_fwd_lds_kernel<bf16_t, false>), grid, dim3(256), lds, s, g, planes, pb, (const bf16_t *)x, (bf16_t *)y, argmax);
        else
            if (k == 3 && stride == 2)
                hipLaunchKernelGGL((maxpool_fwd_lds_kernel<float, true>), grid, dim3(256), lds, s, g, planes, pb, (const float *)x, (float *)y, argmax);
            else
                hipLaunchKernelGGL((maxpool_fwd_lds_kernel<float, false>), grid, dim3(256), lds, s, g, planes, pb, (const float *)x, (float *)y, argmax);
        OMNI_LAUNCH_CHECK();
        return OMNI_OK;
    }
    for (int64_t p0 = 0; p0 < planes; p0 += planes_per_launch) {
        int64_t np = planes - p0 < planes_per_launch ? planes - p0 : planes_per_launch;
        uint32_t count = (uint32_t)(np * per);
        dim3 grid((count + 255u) / 256u);
        if (dtype == OMNI_BF16)
            hipLaunchKernelGGL(maxpool_fwd_kernel<bf16_t>, grid, dim3(256), 0, s, g, p0, count, (const bf16_t *)x, (bf16_t *)y, argmax);
        else
            hipLaunchKernelGGL(maxpool_fwd_kernel<float>, grid, dim3(256), 0, s, g, p0, count, (const float *)x, (float *)y, argmax);
        OMNI_LAUNCH_CHECK();
    }
    return OMNI_OK;
}

int launch_maxpool_bwd(int dtype, int64_t planes, int32_t H, int32_t W, int32_t k, int32_t stride, int32_t ceil_mode,
                       const void *dy, const uint8_t *argmax, const void *y, void *dx, hipStream_t s)
{
    PoolGeom g = make_pool_geom(H, W, k, stride, ceil_mode);
    int64_t per = (int64_t)H * W;
    int64_t planes_per_launch = (0x7fffffffll - 4096) / per;
    ProfScope prof(KID_POOL_BWD, s, 0.0,
                   (double)planes * (per * (y ? 2.0 : 1.0) + (double)g.Ho * g.Wo) * elem_size(dtype) + (double)planes * g.Ho * g.Wo);
    {
        const int64_t howo = (int64_t)g.Ho * g.Wo;
        int pb = pool_planes_per_block(howo * (int64_t)(elem_size(dtype) + 1), per);
        if (pb > 0 && k == 3 && stride == 2) pb = pool_bwd_planes_k3s2(H, W, howo * (int64_t)(elem_size(dtype) + 1), howo);
        if (pb > 0 && (planes + pb - 1) / pb <= 0x7fffffffll) {
            dim3 grid((unsigned)((planes + pb - 1) / pb));
            size_t lds = (((size_t)pb * howo * elem_size(dtype) + 15) / 16) * 16 + (size_t)pb * howo + 16;
            const int64_t last = planes % pb == 0 ? pb : planes % pb;
            if (k == 3 && stride == 2 && (int64_t)pb * howo <= 4096 && last * howo >= 16) {
                // persistent: a few workgroups per compute unit, each walking the groups with the grid's stride (four:
                // measured inside the training step, where the tensors come from memory, 3 / 4 / 6 / 8 per unit give
                // 179 / 172 / 176 / 180 us for the step's three pools; back to back from a warm cache six are best)
                const unsigned resident = 256u * 4u;
                dim3 pgrid(grid.x < resident ? grid.x : resident);
                if (dtype == OMNI_BF16) {
                    if (y) hipLaunchKernelGGL((maxpool_bwd_k3s2_kernel<bf16_t, true>), pgrid, dim3(256), lds, s, g, planes, pb, (const bf16_t *)dy, argmax, (const bf16_t *)y, (bf16_t *)dx, RowsOut{});
                    else hipLaunchKernelGGL((maxpool_bwd_k3s2_kernel<bf16_t, false>), pgrid, dim3(256), lds, s, g, planes, pb, (const bf16_t *)dy, argmax, (const bf16_t *)nullptr, (bf16_t *)dx, RowsOut{});
                } else {
                    if (y) hipLaunchKernelGGL((maxpool_bwd_k3s2_kernel<float, true>), pgrid, dim3(256), lds, s, g, planes, pb, (const float *)dy, argmax, (const float *)y, (float *)dx, RowsOut{});
                    else hipLaunchKernelGGL((maxpool_bwd_k3s2_kernel<float, false>), pgrid, dim3(256), lds, s, g, planes, pb, (const float *)dy, argmax, (const float *)nullptr, (float *)dx, RowsOut{});
                }
                OMNI_LAUNCH_CHECK();
                return OMNI_OK;
            }
#define OMNI_POOL_BWD(T, R)                                                                                              \
    do {                                                                                                             \
        if (k == 3 && stride == 2)                                                                                   \
            hipLaunchKernelGGL((maxpool_bwd_lds_kernel<T, R, true>), grid, dim3(256), lds, s, g, planes, pb, (const T *)dy, argmax, (const T *)y, (T *)dx); \
        else                                                                                                         \
            hipLaunchKernelGGL((maxpool_bwd_lds_kernel<T, R, false>), grid, dim3(256), lds, s, g, planes, pb, (const T *)dy, argmax, (const T *)y, (T *)dx); \
    } while (0)
            if (dtype == OMNI_BF16) {
                if (y) OMNI_POOL_BWD(bf16_t, true); else OMNI_POOL_BWD(bf16_t, false);
            } else {
                if (y) OMNI_POOL_BWD(float, true); else OMNI_POOL_BWD(float, false);
            }
#undef OMNI_POOL_BWD
            OMNI_LAUNCH_CHECK();
            return OMNI_OK;
        }
    }
    for (int64_t p0 = 0; p0 < planes; p0 += planes_per_launch) {
        int64_t np = planes - p0 < planes_per_launch ? planes - p0 : planes_per_launch;
        uint32_t count = (uint32_t)(np * per);
        dim3 grid((count + 255u) / 256u);
        if (dtype == OMNI_BF16) {
            if (y)
                hipLaunchKernelGGL((maxpool_bwd_kernel<bf16_t, true>), grid, dim3(256), 0, s, g, p0, count, (const bf16_t *)dy, argmax, (const bf16_t *)y, (bf16_t *)dx);
            else
                hipLaunchKernelGGL((maxpool_bwd_kernel<bf16_t, false>), grid, dim3(256), 0, s, g, p0, count, (const bf16_t *)dy, argmax, (const bf16_t *)nullptr, (bf16_t *)dx);
        } else {
            if (y)
                hipLaunchKernelGGL((maxpool_bwd_kernel<float, true>), grid, dim3(256), 0, s, g, p0, count, (const float *)dy, argmax, (const float *)y, (float *)dx);
            else
                hipLaunchKernelGGL((maxpool_bwd_kernel<float, false>), grid, dim3(256), 0, s, g, p0, count, (const float *)dy, argmax, (const float *)nullptr, (float *)dx);
        }
        OMNI_LAUNCH_CHECK();
    }
    return OMNI_OK;
}


// The same backward pass writing the rows form (RowsOut) instead of the dense tensor: bf16, 3 x 3 / stride 2
// windows on planes the persistent kernel can stage; anything else is reported as unsupported.
bool maxpool_bwd_rows_supported(int32_t N, int32_t C, int32_t H, int32_t W, int32_t k, int32_t stride, int32_t ceil_mode)
{
    if (k != 3 || stride != 2 || H < k || W < k || (int64_t)N * C > 0x7fffffffll) return false;
    PoolGeom g = make_pool_geom(H, W, k, stride, ceil_mode);
    const int64_t howo = (int64_t)g.Ho * g.Wo, per = (int64_t)H * W, planes = (int64_t)N * C;
    if (howo * 3 > 32 * 1024 || per > 0x7fffffffll - 4096) return false;
    int pb = pool_planes_per_block(howo * 3, per);
    if (pb > 0) pb = pool_bwd_planes_k3s2(H, W, howo * 3, howo);
    if (pb <= 0) return false;
    const int64_t last = planes % pb == 0 ? pb : planes % pb;
    const int64_t tasks = (int64_t)pb * ((H + 1) / 2) * ((W + 7) / 8);
    return (int64_t)pb * howo <= 4096 && last * howo >= 16 && tasks <= 1024;
}

int launch_maxpool_bwd_rows(int32_t N, int32_t C, int32_t H, int32_t W, int32_t k, int32_t stride, int32_t ceil_mode,
                            const void *dy, const uint8_t *argmax, const void *y, void *dx_rows, int64_t ld, float *plane_sums,
                            hipStream_t s)
{
    if (!maxpool_bwd_rows_supported(N, C, H, W, k, stride, ceil_mode)) return OMNI_UNSUPPORTED;
    PoolGeom g = make_pool_geom(H, W, k, stride, ceil_mode);
    const int64_t howo = (int64_t)g.Ho * g.Wo, per = (int64_t)H * W, planes = (int64_t)N * C;
    const int pb = pool_bwd_planes_k3s2(H, W, howo * 3, howo);
    RowsOut ro;
    ro.ld = ld, ro.pitch = (int32_t)((per + 7) / 8 * 8), ro.N = N, ro.div_C = FastDiv((uint32_t)C), ro.sums = plane_sums;
    const int64_t groups = (planes + pb - 1) / pb;
    const int tasks = pb * ((H + 1) / 2) * ((W + 7) / 8);
    size_t lds = (((size_t)pb * howo * 2 + 15) / 16) * 16 + (((size_t)pb * howo + 15) / 16) * 16 + (size_t)tasks * sizeof(float) + 16;
    ProfScope prof(KID_POOL_BWD, s, 0.0,
                   (double)planes * ((double)ro.pitch + (y ? 2.0 : 1.0) * (double)howo) * 2.0 + (double)planes * (howo + 4.0));
    const unsigned resident = 256u * 4u;  // as in launch_maxpool_bwd
    dim3 pgrid((unsigned)(groups < resident ? groups : resident));
    if (y)
        hipLaunchKernelGGL((maxpool_bwd_k3s2_kernel<bf16_t, true, true>), pgrid, dim3(256), lds, s, g, planes, pb, (const bf16_t *)dy,
                           argmax, (const bf16_t *)y, (bf16_t *)dx_rows, ro);
    else
        hipLaunchKernelGGL((maxpool_bwd_k3s2_kernel<bf16_t, false, true>), pgrid, dim3(256), lds, s, g, planes, pb, (const bf16_t *)dy,
                           argmax, (const bf16_t *)nullptr, (bf16_t *)dx_rows, ro);
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

// ReLU backward from dense [N][C][hw] tensors into the rows form: out[c][n * 8 p8 + j] = y > 0 ? dy : 0 for
// j < hw and zero up to 8 p8 = the plane rounded up to 8 elements.  A workgroup takes pp consecutive images of one
// channel (pp * p8 <= 256 threads, one 8-element pack each); plane sums as in RowsOut.
__global__ __launch_bounds__(256) void relu_bwd_rows_kernel(int hw, int p8, int pp, int N, int C, FastDiv div_p8,
                                                            const bf16_t *__restrict__ y, const bf16_t *__restrict__ dy,
                                                            uint16_t *__restrict__ out, int64_t ld, float *__restrict__ sums)
{
    __shared__ float psum[256];
    const int c = blockIdx.y, n0 = blockIdx.x * pp;
    uint32_t pl, i;
    div_p8.divmod(threadIdx.x, pl, i);
    const int n = n0 + (int)pl;
    const bool live = (int)pl < pp && n < N;
    float sum = 0.f;
    if (live) {
        const int valid = hw - 8 * (int)i, back = valid < 8 ? 8 - valid : 0;
        // a plane's ragged last pack is read so that its 16 bytes END at the plane's end and shifted down
        // afterwards, which zeroes the round-up
        const int64_t at = ((int64_t)n * C + c) * hw + 8 * (int)i - back;
        struct alignas(16) Pack8 { uint16_t v[8]; } d, v;
        __builtin_memcpy(&d, dy + at, 16);
        __builtin_memcpy(&v, y + at, 16);
#pragma unroll
        for (int e = 0; e < 8; ++e) d.v[e] = bf16_to_f32(v.v[e]) > 0.f ? d.v[e] : (uint16_t)0;
        if (back) {
            unsigned __int128 x;
            __builtin_memcpy(&x, &d, 16);
            x >>= 16 * back;
            __builtin_memcpy(&d, &x, 16);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) sum += bf16_to_f32(d.v[e]);
        __builtin_memcpy(__builtin_assume_aligned(out + (int64_t)c * ld + ((int64_t)n * p8 + i) * 8, 16), &d, 16);
    }
    if (sums != nullptr) {
        psum[threadIdx.x] = sum;
        __syncthreads();
        if ((int)threadIdx.x < pp && n0 + (int)threadIdx.x < N) {
            float acc = 0.f;
            for (int j = 0; j < p8; ++j) acc += psum[threadIdx.x * p8 + j];
            sums[(int64_t)c * N + n0 + threadIdx.x] = acc;
        }
    }
}

bool relu_bwd_rows_supported(int32_t N, int32_t C, int64_t plane)
{
    return plane >= 8 && plane <= 2048 && C <= 65535 && (int64_t)N * C <= 0x7fffffffll;
}

int launch_relu_bwd_rows(int32_t N, int32_t C, int64_t plane, const void *y, const void *dy, void *dx_rows, int64_t ld,
                         float *plane_sums, hipStream_t s)
{
    if (!relu_bwd_rows_supported(N, C, plane)) return OMNI_UNSUPPORTED;
    const int p8 = (int)((plane + 7) / 8), pp = 256 / p8;
    dim3 grid((unsigned)((N + pp - 1) / pp), (unsigned)C, 1);
    ProfScope prof(KID_RELU, s, 0.0, (double)N * C * (2.0 * plane + 8.0 * p8) * 2.0 + 4.0 * N * C);
    hipLaunchKernelGGL(relu_bwd_rows_kernel, grid, dim3(256), 0, s, (int)plane, p8, pp, N, C, FastDiv((uint32_t)p8),
                       (const bf16_t *)y, (const bf16_t *)dy, (uint16_t *)dx_rows, ld, plane_sums);
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

}  // namespace omni
