// MFMA step, GEMM epilogues and result-tile stores shared by the lowered-GEMM kernels (gemm.hip) and the
// fused convolution kernel (implicit.hip).  Device code only; not part of the C ABI.
#pragma once

#include <type_traits>

#include "common.h"

namespace omni {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// ------------------------------------------------------------------------------------------------
// MFMA on a pair of packs (one "slab" of the reduction)
// ------------------------------------------------------------------------------------------------
template <typename T> struct Mma;
template <> struct Mma<float> {
    static __device__ __forceinline__ void run(const uint4 &a, const uint4 &b, f32x16 &acc)
    {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
    }
};
template <> struct Mma<bf16_t> {
    static __device__ __forceinline__ void run(const uint4 &a, const uint4 &b, f32x16 &acc)
    {
        union U { uint4 u; bf16x8 v; };
        U ua, ub;
        ua.u = a;
        ub.u = b;
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua.v, ub.v, acc, 0, 0, 0);
    }
};

// ------------------------------------------------------------------------------------------------
// Epilogues: receive result element (i, j) in fp32
// ------------------------------------------------------------------------------------------------

// forward: i = filter f, j = column m = (n, pixel).  "Lifting" (App. C) is this address map.
template <typename T> struct FwdEpilogue {
    T *Y;
    const float *bias;
    int F, M, HoWo;
    FastDiv div_HoWo;
    int relu;
    struct Col { int64_t base; bool ok; };
    __device__ __forceinline__ Col column(int j) const
    {
        Col c;
        c.ok = j < M;
        uint32_t n, r;
        div_HoWo.divmod(c.ok ? (uint32_t)j : 0u, n, r);
        c.base = (int64_t)n * F * HoWo + r;
        return c;
    }
    __device__ __forceinline__ float row_add(int i) const { return (bias != nullptr && i < F) ? bias[i] : 0.f; }
    __device__ __forceinline__ void store(int i, const Col &c, float v, float add, int) const
    {
        if (i < F && c.ok) {
            v += add;
            if (relu) v = v > 0.f ? v : 0.f;
            Y[c.base + (int64_t)i * HoWo] = Elem<T>::from_f32(v);
        }
    }
    // 32-bit addressing form: address(i, j) = base + i * row_stride + col_off(j), all in bytes
    typedef T Out;
    __device__ __forceinline__ char *base32(int) const { return reinterpret_cast<char *>(Y); }
    __device__ __forceinline__ uint32_t row_stride32() const { return (uint32_t)HoWo * (uint32_t)sizeof(T); }
    __device__ __forceinline__ int n_rows() const { return F; }
    __device__ __forceinline__ uint32_t col_off32(int j, bool &ok) const
    {
        ok = j < M;
        uint32_t n, r;
        div_HoWo.divmod(ok ? (uint32_t)j : 0u, n, r);
        return (n * (uint32_t)F * (uint32_t)HoWo + r) * (uint32_t)sizeof(T);
    }
    static constexpr bool HAS_ROW_ADD = true;
    __device__ __forceinline__ float apply(float v, float add) const
    {
        v += add;
        if (relu) v = v > 0.f ? v : 0.f;
        return v;
    }
    __device__ __forceinline__ T finish(float v, float add) const { return Elem<T>::from_f32(apply(v, add)); }
    bool fits32() const { return (double)M * F * sizeof(T) < 4.0e9; }
};

// data gradient handed to the layer in front in the form its model gradient multiplies: i = channel c, j = column
// m = (n, pixel); element (i, j) goes to out[i * ld + n * pitch + pixel] (the rows matrix) if mask[n][i][pixel] > 0
// (the ReLU of that layer, mask = its dense output [N][F][HoWo]), else zero goes there.
struct RowsMaskEpilogue {
    bf16_t *out;
    const bf16_t *mask;
    float *sums;  // [F][column tiles]: sum of what each column tile stored per row (nullable)
    int F, M, HoWo;
    FastDiv div_HoWo;
    uint32_t pitch, ld;
    typedef bf16_t Out;
    static constexpr bool MASKED = true;
    static constexpr bool HAS_ROW_ADD = false;
    __device__ __forceinline__ float row_add(int) const { return 0.f; }
    __device__ __forceinline__ char *base32(int) const { return reinterpret_cast<char *>(out); }
    __device__ __forceinline__ uint32_t row_stride32() const { return ld * 2u; }
    __device__ __forceinline__ int n_rows() const { return F; }
    __device__ __forceinline__ uint32_t col_off32(int j, bool &ok) const
    {
        ok = j < M;
        uint32_t n, r;
        div_HoWo.divmod(ok ? (uint32_t)j : 0u, n, r);
        return (n * pitch + r) * 2u;
    }
    __device__ __forceinline__ const char *mask_base() const { return reinterpret_cast<const char *>(mask); }
    __device__ __forceinline__ uint32_t mask_row_stride32() const { return (uint32_t)HoWo * 2u; }
    __device__ __forceinline__ uint32_t mask_col_off32(int j, bool &ok) const
    {
        ok = j < M;
        uint32_t n, r;
        div_HoWo.divmod(ok ? (uint32_t)j : 0u, n, r);
        return (n * (uint32_t)F * (uint32_t)HoWo + r) * 2u;
    }
    // columns from j to the end of j's image (j < M)
    __device__ __forceinline__ int columns_left_in_image(int j) const
    {
        uint32_t n, r;
        div_HoWo.divmod((uint32_t)j, n, r);
        return HoWo - (int)r;
    }
    __device__ __forceinline__ float apply(float v, float) const { return v; }
};

// dgrad: i = row k of dD-hat, j = column m; row-major with leading dimension ld.
template <typename T> struct RowMajorEpilogue {
    T *out;
    int64_t ld;
    int rows, cols;
    struct Col { int64_t base; bool ok; };
    __device__ __forceinline__ Col column(int j) const { return Col{(int64_t)j, j < cols}; }
    __device__ __forceinline__ float row_add(int) const { return 0.f; }
    __device__ __forceinline__ void store(int i, const Col &c, float v, float, int) const
    {
        if (i < rows && c.ok) out[(int64_t)i * ld + c.base] = Elem<T>::from_f32(v);
    }
    typedef T Out;
    __device__ __forceinline__ char *base32(int) const { return reinterpret_cast<char *>(out); }
    __device__ __forceinline__ uint32_t row_stride32() const { return (uint32_t)ld * (uint32_t)sizeof(T); }
    __device__ __forceinline__ int n_rows() const { return rows; }
    __device__ __forceinline__ uint32_t col_off32(int j, bool &ok) const
    {
        ok = j < cols;
        return (uint32_t)j * (uint32_t)sizeof(T);
    }
    static constexpr bool HAS_ROW_ADD = false;
    __device__ __forceinline__ float apply(float v, float) const { return v; }
    __device__ __forceinline__ T finish(float v, float) const { return Elem<T>::from_f32(v); }
    bool fits32() const { return (double)rows * ld * sizeof(T) < 4.0e9; }
};

// wgrad: i = filter f, j = k; fp32 partial sums, one [rows][cols] slice per split z.
struct PartialEpilogue {
    float *out;
    int rows, cols;
    struct Col { int64_t base; bool ok; };
    __device__ __forceinline__ Col column(int j) const { return Col{(int64_t)j, j < cols}; }
    __device__ __forceinline__ float row_add(int) const { return 0.f; }
    __device__ __forceinline__ void store(int i, const Col &c, float v, float, int z) const
    {
        if (i < rows && c.ok) out[((int64_t)z * rows + i) * cols + c.base] = v;
    }
    typedef float Out;
    __device__ __forceinline__ char *base32(int z) const { return reinterpret_cast<char *>(out + (int64_t)z * rows * cols); }
    __device__ __forceinline__ uint32_t row_stride32() const { return (uint32_t)cols * 4u; }
    __device__ __forceinline__ int n_rows() const { return rows; }
    __device__ __forceinline__ uint32_t col_off32(int j, bool &ok) const
    {
        ok = j < cols;
        return (uint32_t)j * 4u;
    }
    static constexpr bool HAS_ROW_ADD = false;
    __device__ __forceinline__ float apply(float v, float) const { return v; }
    __device__ __forceinline__ float finish(float v, float) const { return v; }
    bool fits32() const { return (double)rows * cols * 4.0 < 4.0e9; }
};

// Stores a wavefront's TI x TJ grid of 32 x 32 MFMA result tiles.  Result layout of one tile: lane holds
// column lane%32; register v holds row 8*(v/4) + 4*(lane/32) + v%4.  The address of an element is a
// wave-uniform 64-bit base (row part, scalar registers) plus a 32-bit per-lane offset (column part and
// the lane's share of the row), so one element costs a convert, an add and a store.
template <int TI, int TJ, typename Epi>
__device__ __forceinline__ void store_tile32(f32x16 (&acc)[TI][TJ], int i_wave, int j_wave, int li, int h, int z,
                                             const Epi &epi)
{
    typedef typename Epi::Out Out;
    const uint32_t rs = epi.row_stride32();
    char *base = epi.base32(z);
    uint32_t voff[TJ];
    bool ok[TJ];
#pragma unroll
    for (int u = 0; u < TJ; ++u) voff[u] = epi.col_off32(j_wave + u * 32 + li, ok[u]) + (uint32_t)(4 * h) * rs;
    const int rows = epi.n_rows();
#pragma unroll
    for (int t = 0; t < TI; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int iu = i_wave + t * 32 + 8 * (v / 4) + (v % 4);  // wave-uniform part of the row
            const int i = iu + 4 * h;
            if (iu >= rows) continue;                                 // uniform: nothing of this row exists
            const float add = epi.row_add(i);
            char *row = base + (int64_t)iu * rs;                      // uniform 64-bit
#pragma unroll
            for (int u = 0; u < TJ; ++u)
                if (ok[u] && i < rows) *reinterpret_cast<Out *>(row + voff[u]) = epi.finish(acc[t][u][v], add);
        }
}


// Same job staged through LDS.  The wavefront drops SR rows x (32*TJ) columns of raw fp32 results into
// a private LDS strip, then reads the strip back one 16-byte output piece per lane (4 fp32 or 8 bf16
// results of one row), applies the epilogue (row term, ReLU, rounding: two results per conversion
// instruction) and stores whole row segments instead of one element per lane.  A piece whose columns
// are not consecutive in memory (it straddles two images in the forward pass) or not all valid falls
// back to element stores.  `strip` is this wavefront's LDS region of SR * staged_pitch(TJ) bytes; only
// this wavefront touches it, and LDS operations of one wavefront complete in order, so no workgroup
// barrier is involved.  `row_add` is an LDS table of the tile's row terms indexed by (row - i_tile),
// read only if the epilogue has one.
// The pitch makes the two half-waves (rows r and r + 4) land 32 banks apart.
constexpr int staged_pitch(int TJ) { return 32 * TJ * 4 + 32; }

// An epilogue with Epi::MASKED (RowsMaskEpilogue) also zeroes every result whose entry in a second tensor is not
// positive and leaves, in wave_sums[(row - i_tile) * wave_cols + wave_col], the sum of the values this wavefront
// stored to that row (as rounded; fixed order: per 16-byte piece, then the row's pieces left to right).
template <typename Epi, typename = void> struct epilogue_is_masked : std::false_type {};
template <typename Epi> struct epilogue_is_masked<Epi, std::enable_if_t<Epi::MASKED>> : std::true_type {};

template <int TI, int TJ, int SR, typename Epi>
__device__ __forceinline__ void store_tile_staged(f32x16 (&acc)[TI][TJ], int i_wave, int j_wave, int lane, int z,
                                                  const Epi &epi, char *strip, const float *row_add, int i_tile,
                                                  float *wave_sums = nullptr, int wave_cols = 1, int wave_col = 0)
{
    constexpr bool MASKED = epilogue_is_masked<Epi>::value;
    typedef typename Epi::Out Out;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    static_assert(SR == 16 || SR == 32, "a strip holds half or all of a 32-row MFMA tile");
    constexpr int COLS = 32 * TJ;
    constexpr int VEC = 16 / (int)sizeof(Out);   // results per 16-byte output piece
    constexpr int GPR = COLS / VEC;              // pieces per row
    constexpr int RPP = 64 / GPR;                // rows per pass of the wavefront
    constexpr int PASSES = (SR + RPP - 1) / RPP;
    constexpr bool EXACT = RPP * GPR == 64 && SR % RPP == 0;  // else some lanes or pass rows are idle
    constexpr int PITCH = staged_pitch(TJ);
    static_assert(GPR <= 64, "pass shape");
    const int li = lane % 32, h = lane / 32;
    const uint32_t rs = epi.row_stride32();
    char *base = epi.base32(z);
    const int rows = epi.n_rows();
    // this lane's piece in the read-back phase
    const int cg = lane % GPR, rr = lane / GPR;
    bool ok_first, ok_last;
    const uint32_t off_first = epi.col_off32(j_wave + cg * VEC, ok_first);
    const uint32_t off_last = epi.col_off32(j_wave + cg * VEC + VEC - 1, ok_last);
    const bool whole = ok_first && ok_last && off_last - off_first == (uint32_t)((VEC - 1) * sizeof(Out));
    // MASKED: the mask entries of a piece are fetched as 16 bytes starting at its first column; a piece that runs
    // from image n into image n + 1 (its first `mk_first` columns in n) takes a second fetch that ends where the
    // piece ends, and picks per element.  Both stay inside the mask tensor because all the piece's columns exist;
    // a piece with columns past the end (last column tile only) reads its mask element by element instead.
    uint32_t moff_first = 0, moff_second = 0, mrs = 0;
    int mk_first = VEC;
    bool mask_vec = false;
    const char *mbase = nullptr;
    if constexpr (MASKED) {
        static_assert(sizeof(Out) == 2, "masked stores are bf16");
        bool ok;
        moff_first = epi.mask_col_off32(j_wave + cg * VEC, ok);
        mrs = epi.mask_row_stride32();
        mbase = epi.mask_base();
        mask_vec = ok_first && ok_last;
        if (mask_vec && !whole) {
            mk_first = epi.columns_left_in_image(j_wave + cg * VEC);  // 1 .. VEC - 1 here
            moff_second = epi.mask_col_off32(j_wave + cg * VEC + mk_first, ok) - (uint32_t)(mk_first * 2);
        }
    }
    // MASKED: the mask fetches of a group of passes (one strip) go out one group ahead, so that their latency passes
    // under the previous group's work; two sets of registers take turns
    u32x4 mask_a[2][MASKED ? PASSES : 1], mask_b[2][MASKED ? PASSES : 1];
    auto fetch_masks = [&](int gi, u32x4 *ma, u32x4 *mb) {
        if constexpr (MASKED) {
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                const int r = p * RPP + rr;
                const int i = i_wave + gi * SR + r;   // gi * SR = t * 32 + half * SR
                ma[p] = mb[p] = u32x4{0, 0, 0, 0};
                if ((!EXACT && (rr >= RPP || r >= SR)) || i >= rows || !mask_vec) continue;
                __builtin_memcpy(&ma[p], mbase + ((uint32_t)i * mrs + moff_first), 16);
                if (!whole) __builtin_memcpy(&mb[p], mbase + ((uint32_t)i * mrs + moff_second), 16);
            }
        }
    };
    fetch_masks(0, mask_a[0], mask_b[0]);
#pragma unroll
    for (int t = 0; t < TI; ++t) {
#pragma unroll
        for (int half = 0; half < 32 / SR; ++half) {
#pragma unroll
            for (int vv = 0; vv < SR / 2; ++vv) {
                const int v = half * (SR / 2) + vv;
                const int r = 8 * (vv / 4) + 4 * h + (vv % 4);
                float *row = reinterpret_cast<float *>(strip + r * PITCH);
#pragma unroll
                for (int u = 0; u < TJ; ++u) row[u * 32 + li] = acc[t][u][v];
            }
            if constexpr (MASKED) {
                const int gi = t * (32 / SR) + half;          // compile-time after unrolling
                if (gi + 1 < TI * (32 / SR)) fetch_masks(gi + 1, mask_a[(gi + 1) & 1], mask_b[(gi + 1) & 1]);
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                const int r = p * RPP + rr;
                if (!EXACT && (rr >= RPP || r >= SR)) continue;
                const int i = i_wave + t * 32 + half * SR + r;
                float x[VEC];
#pragma unroll
                for (int q = 0; q < VEC / 4; ++q) {
                    f32x4 f = *reinterpret_cast<const f32x4 *>(strip + r * PITCH + cg * (VEC * 4) + q * 16);
                    x[4 * q] = f[0], x[4 * q + 1] = f[1], x[4 * q + 2] = f[2], x[4 * q + 3] = f[3];
                }
                float add = 0.f;
                if constexpr (Epi::HAS_ROW_ADD) add = row_add[i - i_tile];
#pragma unroll
                for (int e = 0; e < VEC; ++e) x[e] = epi.apply(x[e], add);
                float stored = 0.f;  // MASKED: sum of this piece's stored values
                if (i < rows) {
                    if constexpr (MASKED) {
                        if (mask_vec) {
#pragma unroll
                            for (int e = 0; e < VEC; ++e) {
                                const int cur = (t * (32 / SR) + half) & 1;
                                const uint32_t word = e < mk_first ? mask_a[cur][p][e / 2] : mask_b[cur][p][e / 2];
                                const uint32_t bits = (e & 1) ? (word & 0xffff0000u) : (word << 16);
                                x[e] = __uint_as_float(bits) > 0.f ? x[e] : 0.f;
                            }
                        }
                    }
                    if (whole) {
                        u32x4 piece;
                        if constexpr (sizeof(Out) == 4)
                            piece = u32x4{__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3])};
                        else
                            piece = u32x4{f32x2_to_bf16x2(x[0], x[1]), f32x2_to_bf16x2(x[2], x[3]),
                                          f32x2_to_bf16x2(x[4], x[5]), f32x2_to_bf16x2(x[6], x[7])};
                        __builtin_memcpy(base + ((uint32_t)i * rs + off_first), &piece, 16);  // element-aligned 16-byte store
                        if constexpr (MASKED) {
#pragma unroll
                            for (int e = 0; e < VEC; ++e)
                                stored += __uint_as_float((e & 1) ? (piece[e / 2] & 0xffff0000u) : (piece[e / 2] << 16));
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < VEC; ++e) {
                            bool ok;
                            uint32_t off = epi.col_off32(j_wave + cg * VEC + e, ok);
                            if constexpr (MASKED) {
                                if (ok) {
                                    float xv = x[e];  // masked above unless the piece has columns past the end
                                    if (!mask_vec) {
                                        bool mok;
                                        const uint32_t moff = epi.mask_col_off32(j_wave + cg * VEC + e, mok);
                                        const bf16_t mbits = *reinterpret_cast<const bf16_t *>(mbase + ((uint32_t)i * mrs + moff));
                                        xv = bf16_to_f32(mbits) > 0.f ? xv : 0.f;
                                    }
                                    const Out o = Elem<Out>::from_f32(xv);
                                    *reinterpret_cast<Out *>(base + ((uint32_t)i * rs + off)) = o;
                                    stored += Elem<Out>::to_f32(o);
                                }
                            } else {
                                if (ok) *reinterpret_cast<Out *>(base + ((uint32_t)i * rs + off)) = Elem<Out>::from_f32(x[e]);
                            }
                        }
                    }
                }
                // the row's raw results have been read by all its lanes (same instructions, LDS in order): its
                // first floats now hold the pieces' sums
                if constexpr (MASKED) reinterpret_cast<float *>(strip + r * PITCH)[cg] = stored;
            }
            if constexpr (MASKED) {
                __builtin_amdgcn_wave_barrier();
                if (lane < SR) {
                    const float *ps = reinterpret_cast<const float *>(strip + lane * PITCH);
                    float acc_row = 0.f;
#pragma unroll
                    for (int c = 0; c < GPR; ++c) acc_row += ps[c];
                    wave_sums[(i_wave + t * 32 + half * SR + lane - i_tile) * wave_cols + wave_col] = acc_row;
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// Ordered sum of the split partial results [splits][rows][cols] of a forward or data-gradient product,
// handed to the product's own epilogue (address map, bias, ReLU, rounding).  One thread per result.
template <typename Epi>
__global__ __launch_bounds__(256) void reduce_store_kernel(const float *__restrict__ partials, int splits, int rows,
                                                           int cols, Epi epi)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x, count = (int64_t)rows * cols;
    if (idx >= count) return;
    const int i = (int)(idx / cols), j = (int)(idx - (int64_t)i * cols);
    float acc = 0.f;
    for (int z = 0; z < splits; ++z) acc += partials[(int64_t)z * count + idx];
    epi.store(i, epi.column(j), acc, epi.row_add(i), 0);
}

}  // namespace omni
