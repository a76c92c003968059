// MFMA GEMM for the three matrix products of a lowered convolution layer (gfx950).
//
// One kernel template serves the paper's "multiply phase" (App. C, "Convolution by Lowering and
// GEMM") in its three uses:
//   forward : Y-hat [F x M] = K-hat   [F x K] * D-hat  [K x M]      epilogue: +bias, ReLU, lifting
//   dgrad   : dD-hat[K x M] = K-hat^T [K x F] * dY-hat [F x M]      epilogue: plain row-major store
//   wgrad   : dK-hat[F x K] = dY-hat  [F x M] * D-hat^T[M x K]      split along M, fp32 partials
// In every use the "row operand" (index i of the result) is contiguous along the reduction index,
// and the "column operand" (index j, the contiguous index of the result) is either contiguous
// along j (forward, dgrad: D-hat and dY-hat have M as their fastest index) or along the reduction
// (wgrad).
//
// Tiling: a workgroup of 256 threads (4 wavefronts of 64 lanes, 2 x 2) owns a 128 x 128 tile of
// the result; each wavefront owns 64 x 64 = 2 x 2 MFMA tiles of 32 x 32, accumulated in fp32.
// The reduction is walked in steps of 128 bytes per row (64 bf16 or 32 fp32).  Both operands are
// staged in LDS as [pack][row] arrays of 16-byte packs, a pack being 8 (bf16) or 4 (fp32)
// consecutive reduction indices of one row, so that an MFMA fragment is one 16-byte LDS read per
// lane and 32 consecutive lanes read 512 consecutive bytes.  A column operand that is contiguous
// along j is transposed in registers on its way into LDS.  Global loads of the next step are
// issued before the MFMAs of the current one and land in the other LDS buffer.
//
// fp32 uses v_mfma_f32_32x32x2_f32 four times per pack: within one instruction lane-half h
// supplies reduction index 4*(2s+h)+e for both operands, which is a permutation of the slab's 8
// indices -- a sum does not care about the order of its terms.  bf16 uses
// v_mfma_f32_32x32x16_bf16, one instruction per pair of packs.
#include <cstdlib>
#include <type_traits>

#include "common.h"
#include "mma_epilogue.h"

namespace omni {

constexpr int NPACK = 8;  // 16-byte packs along the reduction per LDS tile (128 bytes of every row)

template <typename T> struct Pack;
template <> struct Pack<float> { static constexpr int KP = 4; };
template <> struct Pack<bf16_t> { static constexpr int KP = 8; };

int gemm_red_tile(int dtype) { return dtype == OMNI_BF16 ? NPACK * 8 : NPACK * 4; }

// ------------------------------------------------------------------------------------------------
// Operand loaders: global memory -> registers (issue()), registers -> LDS (commit()).
// An LDS tile of R rows is uint4[NPACK][R + 1]: pack g of row r at g*(R+1) + r.  The extra pack of
// padding per group spreads the 8 packs of one row over the banks when they are written together.
// ------------------------------------------------------------------------------------------------

// Operand stored [rows][ld] with the reduction index contiguous.  Element (r, k) is valid for
// r < rows and k < red; ld and red are multiples of the pack size and the base is 16-byte aligned.
template <typename T, int TILE_ROWS, int NT> struct RedContigLoader {
    static constexpr int KP = Pack<T>::KP;
    static constexpr int TASKS = TILE_ROWS * NPACK;
    static constexpr int PER_THREAD = (TASKS + NT - 1) / NT;
    static constexpr bool RAGGED = TASKS % NT != 0;  // the last round of tasks covers only part of the threads
    uint4 regs[PER_THREAD];

    __device__ __forceinline__ void issue(const T *base, int64_t ld, int rows, int64_t red, int row0,
                                          int64_t k0, int tid)
    {
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q) {
            int t = tid + q * NT;
            int g = t % NPACK, r = t / NPACK;
            int64_t k = k0 + (int64_t)g * KP;
            uint4 v = make_uint4(0, 0, 0, 0);
            if ((!RAGGED || t < TASKS) && row0 + r < rows && k < red)
                v = *reinterpret_cast<const uint4 *>(base + (int64_t)(row0 + r) * ld + k);
            regs[q] = v;
        }
    }
    __device__ __forceinline__ void commit(uint4 *lds, int tid) const
    {
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q) {
            int t = tid + q * NT;
            int g = t % NPACK, r = t / NPACK;
            if (!RAGGED || t < TASKS) lds[g * (TILE_ROWS + 1) + r] = regs[q];
        }
    }
};

// Operand stored [red][ld] with the result's column index j contiguous.  Element (k, j) is valid
// for k < red and j < cols; ld and cols are multiples of 8 and the base is 16-byte aligned.
// One task = one pack group g (KP reduction rows) x 4 consecutive columns, transposed in registers.
template <typename T, int TILE_COLS, int NT> struct OuterContigLoader;

template <int TILE_COLS, int NT> struct OuterContigLoader<float, TILE_COLS, NT> {
    static constexpr int CHUNKS = TILE_COLS / 4;
    static constexpr int PER_THREAD = NPACK * CHUNKS / NT;
    static_assert(NPACK * CHUNKS % NT == 0, "tile must divide over the threads");
    uint4 regs[PER_THREAD][4];
    __device__ __forceinline__ void issue(const float *base, int64_t ld, int64_t red, int cols,
                                          int64_t k0, int col0, int tid)
    {
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q) {
            int t = tid + q * NT;
            int jc = t % CHUNKS, g = t / CHUNKS;
            int j = col0 + jc * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int64_t k = k0 + g * 4 + e;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (k < red && j < cols) v = *reinterpret_cast<const uint4 *>(base + k * ld + j);
                regs[q][e] = v;
            }
        }
    }
    __device__ __forceinline__ void commit(uint4 *lds, int tid) const
    {
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q) {
            int t = tid + q * NT;
            int jc = t % CHUNKS, g = t / CHUNKS;
            uint4 *dst = lds + g * (TILE_COLS + 1) + jc * 4;
            const uint4 *r = regs[q];
            dst[0] = make_uint4(r[0].x, r[1].x, r[2].x, r[3].x);
            dst[1] = make_uint4(r[0].y, r[1].y, r[2].y, r[3].y);
            dst[2] = make_uint4(r[0].z, r[1].z, r[2].z, r[3].z);
            dst[3] = make_uint4(r[0].w, r[1].w, r[2].w, r[3].w);
        }
    }
};

template <int TILE_COLS, int NT> struct OuterContigLoader<bf16_t, TILE_COLS, NT> {
    static constexpr int CHUNKS = TILE_COLS / 4;
    static constexpr int PER_THREAD = NPACK * CHUNKS / NT;
    static_assert(NPACK * CHUNKS % NT == 0, "tile must divide over the threads");
    uint2 regs[PER_THREAD][8];
    __device__ __forceinline__ void issue(const bf16_t *base, int64_t ld, int64_t red, int cols,
                                          int64_t k0, int col0, int tid)
    {
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q) {
            int t = tid + q * NT;
            int jc = t % CHUNKS, g = t / CHUNKS;
            int j = col0 + jc * 4;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                int64_t k = k0 + g * 8 + e;
                uint2 v = make_uint2(0, 0);
                if (k < red && j < cols) v = *reinterpret_cast<const uint2 *>(base + k * ld + j);
                regs[q][e] = v;
            }
        }
    }
    static __device__ __forceinline__ uint32_t lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
    static __device__ __forceinline__ uint32_t hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }
    __device__ __forceinline__ void commit(uint4 *lds, int tid) const
    {
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q) {
            int t = tid + q * NT;
            int jc = t % CHUNKS, g = t / CHUNKS;
            uint4 *dst = lds + g * (TILE_COLS + 1) + jc * 4;
            const uint2 *r = regs[q];
            // column j = 2d + h of the 8 x 4 block becomes one pack: 8 reduction indices of column j
            dst[0] = make_uint4(lo(r[0].x, r[1].x), lo(r[2].x, r[3].x), lo(r[4].x, r[5].x), lo(r[6].x, r[7].x));
            dst[1] = make_uint4(hi(r[0].x, r[1].x), hi(r[2].x, r[3].x), hi(r[4].x, r[5].x), hi(r[6].x, r[7].x));
            dst[2] = make_uint4(lo(r[0].y, r[1].y), lo(r[2].y, r[3].y), lo(r[4].y, r[5].y), lo(r[6].y, r[7].y));
            dst[3] = make_uint4(hi(r[0].y, r[1].y), hi(r[2].y, r[3].y), hi(r[4].y, r[5].y), hi(r[6].y, r[7].y));
        }
    }
};

// ------------------------------------------------------------------------------------------------
// The lowered matrix read straight from the input tensor (stride-1 layers, bf16), for the model gradient.
// The reduction runs over padded columns.  Row mode: column ((n*Ho + oy) * P8 + i) * 8 + e stands for output
// position (n, oy, 8i + e), P8 = ceil(Wo / 8); plane mode (further down): only whole image planes are
// padded.  dY-hat is packed the same way with zeros in the padding (a sum does not care about the order or
// about zero terms).  A pack of 8 columns of row k = (c, ky, kx) of D-hat is then 8 consecutive input
// pixels: one 16-byte load at element granularity plus a mask for pixels in the zero padding or outside
// the image.  The same input bytes serve the kh*kw
// window taps of a channel, so nearly all of these loads hit in L1/L2; D-hat is never written or read.
// ------------------------------------------------------------------------------------------------
struct DirectSrc {
    const bf16_t *X;
    int32_t C, H, W, HW, K, ph, pw;
    int32_t rows;   // padded units in the batch: N * Ho output rows, or N image planes
    int32_t total;  // elements of X (< 2^31)
    FastDiv div_p8, div_Ho, div_khkw, div_kw;
    int32_t HoWo, KK;  // plane mode: output positions per image, window taps
    FastDiv div_W;
    int32_t sh;        // row mode: vertical stride (input rows per output row)
    int32_t F, Wo;     // DIRECT_ROWS_ONES: dY is [N][F][Ho][Wo], read by DyLoader
};

// Plane mode.  When the output is as wide as the input (stride 1, 2*pw = kw - 1), output position q of an
// image and window tap (ky, kx) meet input element q + (ky - ph) * W + (kx - pw) of the channel's plane,
// also where q wraps from one output row to the next.  So only each image's whole plane is padded to a
// multiple of 8 positions (not every row), a pack is still one 16-byte load, and which of its 8 elements
// are real pixels depends on (pack within the plane, tap) alone: a table in LDS, one byte per element,
// built when the workgroup starts.  Row (pack j, tap KK) of the table is zero: result columns beyond K.
constexpr int DIRECT_TAB = 2560;  // table entries (8 bytes each) a workgroup can hold beside its tiles
enum { DIRECT_ROWS = 1, DIRECT_ROWS_FIXED = 2, DIRECT_PLANES = 3, DIRECT_ROWS_ONES = 4, DIRECT_PHASE3 = 5 };
// DIRECT_ROWS_ONES: row mode in which (a) row K of the operand -- the first result column beyond the gradient
// -- is all ones, so that result column K is the sum of dY over every position: the bias gradient, from the
// same MFMAs; and (b) the row operand is read from dY as it lies in memory (DyLoader), not from a packed copy.

__device__ __forceinline__ void build_plane_table(const DirectSrc &d, uint2 *tab, int tid, int nt)
{
    const int p8 = (int)d.div_p8.d, kw = (int)d.div_kw.d;
    for (int idx = tid; idx < p8 * (d.KK + 1); idx += nt) {
        const int j = idx / (d.KK + 1), tap = idx - j * (d.KK + 1);
        uint32_t ky, kx;
        d.div_kw.divmod((uint32_t)(tap < d.KK ? tap : 0), ky, kx);
        uint32_t w[2] = {0u, 0u};
        for (int e = 0; e < 8; ++e) {
            const int q = 8 * j + e;
            uint32_t oy, ox;
            d.div_W.divmod((uint32_t)q, oy, ox);
            const bool ok = tap < d.KK && q < d.HoWo && (unsigned)((int)oy + (int)ky - d.ph) < (unsigned)d.H &&
                            (unsigned)((int)ox + (int)kx - d.pw) < (unsigned)d.W;
            if (ok) w[e / 4] |= 0xffu << (8 * (e % 4));
        }
        tab[idx] = make_uint2(w[0], w[1]);
    }
    (void)kw;
}

// MODE DIRECT_ROWS_FIXED: the row-padded rows are 1, 2, 4 or 8 packs long, so a reduction step (8 packs)
// moves every thread by whole output rows and the pack's place in its row -- hence which of its 8 elements
// fall beside the image for a given window column -- is the same in every step: those masks are built once.
template <int TILE_ROWS, int NT, int MODE> struct DirectLoader {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    static constexpr bool FIXED = MODE == DIRECT_ROWS_FIXED, PLANES = MODE == DIRECT_PLANES, ONES = MODE == DIRECT_ROWS_ONES;
    static constexpr int PER_THREAD = TILE_ROWS * NPACK / NT;
    static_assert(TILE_ROWS * NPACK % NT == 0 && NT % NPACK == 0, "tile must divide over the threads");
    u32x4 v[PER_THREAD];
    uint32_t ones[ONES ? PER_THREAD : 1];   // 0x3f803f80 (two bf16 ones) for the row of ones, else 0
    // rows: bits 0..7: which elements are real pixels (FIXED: bit 0: the input row exists).
    // bits 8..11: signed element shift (non-zero only where the 16 bytes had to be moved to stay inside
    // the tensor: first and last row of X)
    uint32_t masks[PER_THREAD];
    int kbase[PER_THREAD];
    int dky[PLANES ? 1 : PER_THREAD], dkx[FIXED || PLANES ? 1 : PER_THREAD];
    u32x4 colmask[FIXED ? PER_THREAD : 1];
    int tap[PLANES ? PER_THREAD : 1];       // planes: column of the mask table
    uint2 emask[PLANES ? PER_THREAD : 1];   // planes: this step's table entries

    static __device__ __forceinline__ uint32_t spread(uint32_t m, int bit)  // two mask bits -> two 16-bit fields
    {
        uint32_t lo = (uint32_t)((int32_t)(m << (31 - bit)) >> 31), hi = (uint32_t)((int32_t)(m << (30 - bit)) >> 31);
        return (lo & 0xffffu) | (hi & 0xffff0000u);
    }
    __device__ __forceinline__ void init(const DirectSrc &d, int col0, int tid)
    {
        uint32_t row_unused, i;
        d.div_p8.divmod((uint32_t)(tid % NPACK), row_unused, i);  // FIXED: this thread's pack within its row
        const int ox0 = 8 * (int)i;
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q) {
            int k = col0 + (tid + q * NT) / NPACK;
            uint32_t c, rem, ky, kx;
            d.div_khkw.divmod((uint32_t)(k < d.K ? k : 0), c, rem);
            d.div_kw.divmod(rem, ky, kx);
            const int dx = (int)kx - d.pw;
            kbase[q] = (int)c * d.HW + ((int)ky - d.ph) * d.W + dx;
            if constexpr (PLANES) {
                tap[q] = k < d.K ? (int)rem : d.KK;
            } else {
                if constexpr (ONES) ones[q] = k == d.K ? 0x3f803f80u : 0u;
                dky[q] = k < d.K ? (int)ky - d.ph : -(1 << 24);  // rows beyond K: no input row is ever valid
                if constexpr (FIXED) {
                    const int ix = ox0 + dx;
                    const int lo = ix < 0 ? -ix : 0, hi = d.W - ix < 8 ? d.W - ix : 8;
                    const uint32_t m = hi > lo ? (1u << hi) - (1u << lo) : 0u;
                    if (m == 0u) dky[q] = -(1 << 24);
#pragma unroll
                    for (int w = 0; w < 4; ++w) colmask[q][w] = spread(m, 2 * w);
                } else {
                    dkx[q] = dx;
                }
            }
        }
    }
    // m0: first padded column of this thread's packs -- the same for all of them, NT being a multiple of
    // NPACK.  tab: the plane mode's mask table.
    __device__ __forceinline__ void issue(const DirectSrc &d, int m0, const uint2 *tab)
    {
        const int top = d.total - 8;
        const char *xb = reinterpret_cast<const char *>(d.X);
        if constexpr (PLANES) {
            uint32_t n, j;
            d.div_p8.divmod((uint32_t)m0 >> 3, n, j);
            const bool live = (int)n < d.rows;
            const int base = (live ? (int)n : 0) * d.C * d.HW + 8 * (int)j;
            const int trow = (int)j * (d.KK + 1);
#pragma unroll
            for (int p = 0; p < PER_THREAD; ++p) {
                // element offset of the load, moved inside [0, total - 8] where it sticks out (by at most 7
                // elements if any element of the pack is a real pixel; else the mask is zero anyway)
                const int e = base + kbase[p];
                const int c = e < 0 ? 0 : (e > top ? top : e);
                __builtin_memcpy(&v[p], xb + 2u * (uint32_t)c, 16);
                masks[p] = (uint32_t)(e - c) & 15u;
                emask[p] = tab[live ? trow + tap[p] : d.KK];
            }
        } else {
            uint32_t row, i, n, oy;
            d.div_p8.divmod((uint32_t)m0 >> 3, row, i);
            const bool live = (int)row < d.rows;
            d.div_Ho.divmod(live ? row : 0u, n, oy);
            const int ox0 = 8 * (int)i;
            const int iy = (int)oy * d.sh;
            const int base = (int)n * d.C * d.HW + iy * d.W + ox0;
#pragma unroll
            for (int p = 0; p < PER_THREAD; ++p) {
                bool ok = live && (unsigned)(iy + dky[p]) < (unsigned)d.H;
                uint32_t m = 1u;
                if constexpr (!FIXED) {
                    const int ix = ox0 + dkx[p];
                    const int lo = ix < 0 ? -ix : 0, hi = d.W - ix < 8 ? d.W - ix : 8;
                    ok = ok && hi > lo;
                    m = (1u << hi) - (1u << lo);
                }
                // element offset of the load, moved inside [0, total - 8] where it sticks out
                const int e = base + kbase[p];
                const int c = ok ? (e < 0 ? 0 : (e > top ? top : e)) : 0;
                const uint32_t sft = ok ? (uint32_t)(e - c) & 15u : 0u;
                __builtin_memcpy(&v[p], xb + 2u * (uint32_t)c, 16);
                masks[p] = (ok ? m : 0u) | (sft << 8);
            }
        }
    }
    // element j of the result = element j + s of x (s = 4-bit two's complement, |s| <= 7 where it matters)
    static __device__ __forceinline__ u32x4 shifted(u32x4 x4, uint32_t s4)
    {
        unsigned __int128 x = ((unsigned __int128)(((uint64_t)x4[3] << 32) | x4[2]) << 64) | (((uint64_t)x4[1] << 32) | x4[0]);
        const int up = 16 - (int)s4 > 7 ? 7 : 16 - (int)s4;
        x = (s4 & 8u) ? x << (16 * up) : x >> (16 * (int)s4);
        uint64_t lo = (uint64_t)x, hi = (uint64_t)(x >> 64);
        return u32x4{(uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32)};
    }
    __device__ __forceinline__ void commit(uint4 *lds, int tid) const
    {
#pragma unroll
        for (int p = 0; p < PER_THREAD; ++p) {
            int t = tid + p * NT;
            int g = t % NPACK, r = t / NPACK;
            u32x4 a = v[p];
            u32x4 o;
            if constexpr (PLANES) {
                if (masks[p]) a = shifted(a, masks[p]);  // first or last few elements of the tensor only
                // one mask byte per element -> 16 bits per element (both operands the same word: either
                // half of the selector range picks from it)
                o[0] = a[0] & __builtin_amdgcn_perm(emask[p].x, emask[p].x, 0x01010000u);
                o[1] = a[1] & __builtin_amdgcn_perm(emask[p].x, emask[p].x, 0x03030202u);
                o[2] = a[2] & __builtin_amdgcn_perm(emask[p].y, emask[p].y, 0x01010000u);
                o[3] = a[3] & __builtin_amdgcn_perm(emask[p].y, emask[p].y, 0x03030202u);
            } else {
                if (masks[p] >> 8) a = shifted(a, (masks[p] >> 8) & 15u);
                if constexpr (FIXED) {
                    const uint32_t row_ok = 0u - (masks[p] & 1u);
#pragma unroll
                    for (int w = 0; w < 4; ++w) o[w] = a[w] & colmask[p][w] & row_ok;
                } else {
#pragma unroll
                    for (int w = 0; w < 4; ++w) o[w] = a[w] & spread(masks[p], 2 * w);
                    if constexpr (ONES) {
#pragma unroll
                        for (int w = 0; w < 4; ++w) o[w] |= ones[p];  // the masks of a row beyond K are zero
                    }
                }
            }
            reinterpret_cast<u32x4 *>(lds)[g * (TILE_ROWS + 1) + r] = o;
        }
    }
};

// DIRECT_PHASE3: the lowered operand of the phase-split stride-4 model gradient (launch_gemm_wgrad_phase) when a
// window row has three groups (kw = 9 .. 12).  Rows 3t, 3t + 1, 3t + 2 of the operand are then the same ten
// consecutive elements of phase image (c', ky) shifted by 0, 1 and 2: one 16-byte load and one 4-byte load
// (both aligned: X4's rows are 16-byte multiples and a pack starts at a multiple of 8) serve three packs, and
// only the K' / 3 real triples are loaded.  Nothing needs a mask: every address is inside X4 (8 * P8 + 2 <= WP),
// columns beyond the batch meet zeros of the other operand, rows beyond K' + 1 are never written (their
// results are columns the epilogue does not store), and row K' is the row of ones.
template <int TILE_ROWS, int NT> struct Phase3Loader {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    static constexpr int ROUNDS = (TILE_ROWS / 3 + NT / NPACK - 1) / (NT / NPACK);  // triples per thread
    u32x4 w[ROUNDS];
    uint32_t x[ROUNDS];
    int kbase[ROUNDS];  // element offset of the triple's input row from the pack's base; -1: no such triple

    __device__ __forceinline__ void init(const DirectSrc &d, int, int tid)
    {
        const int kh = (int)d.div_khkw.d / 3;
#pragma unroll
        for (int q = 0; q < ROUNDS; ++q) {
            const int tr = tid / NPACK + q * (NT / NPACK);
            const int c = tr / kh, ky = tr - c * kh;
            kbase[q] = 3 * tr < d.K ? c * d.HW + ky * d.W : -1;
        }
    }
    __device__ __forceinline__ void issue(const DirectSrc &d, int m0, const uint2 *)
    {
        uint32_t row, i, n, oy;
        d.div_p8.divmod((uint32_t)m0 >> 3, row, i);
        const bool live = (int)row < d.rows;
        d.div_Ho.divmod(live ? row : 0u, n, oy);
        const int base = (int)n * d.C * d.HW + (int)oy * d.sh * d.W + 8 * (int)i;
        const char *xb = reinterpret_cast<const char *>(d.X);
#pragma unroll
        for (int q = 0; q < ROUNDS; ++q) {
            const int e = live && kbase[q] >= 0 ? base + kbase[q] : 0;
            __builtin_memcpy(&w[q], xb + 2u * (uint32_t)e, 16);
            __builtin_memcpy(&x[q], xb + 2u * (uint32_t)e + 16, 4);
        }
    }
    __device__ __forceinline__ void commit(uint4 *lds, int tid) const
    {
        u32x4 *dst = reinterpret_cast<u32x4 *>(lds) + (tid % NPACK) * (TILE_ROWS + 1);
#pragma unroll
        for (int q = 0; q < ROUNDS; ++q) {
            const int tr = tid / NPACK + q * (NT / NPACK);
            if (kbase[q] >= 0) {
                const u32x4 a = w[q];
                dst[3 * tr] = a;
                dst[3 * tr + 1] = u32x4{__builtin_amdgcn_alignbit(a[1], a[0], 16), __builtin_amdgcn_alignbit(a[2], a[1], 16),
                                        __builtin_amdgcn_alignbit(a[3], a[2], 16), __builtin_amdgcn_alignbit(x[q], a[3], 16)};
                dst[3 * tr + 2] = u32x4{a[1], a[2], a[3], x[q]};
            }
        }
    }
    // the row of ones (row K of the operand), rewritten with every tile by the first NPACK threads
    __device__ __forceinline__ void commit_ones(uint4 *lds, int tid, int K) const
    {
        if (tid < NPACK) reinterpret_cast<u32x4 *>(lds)[tid * (TILE_ROWS + 1) + K] = u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
    }
};

// The row operand of the model gradient read from dY [N][F][Ho][Wo] itself: row f, padded column
// ((n * Ho + oy) * P8 + i) * 8 + e is dY(n, f, oy, 8 i + e), zero for 8 i + e >= Wo and for columns beyond the
// batch.  The 16 bytes of a row's ragged last pack are read so that they END at the row's end (always inside
// the tensor, Wo >= 8) and are shifted down, which also zeroes the padding.
template <int TILE_ROWS, int NT> struct DyLoader {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    static constexpr int TASKS = TILE_ROWS * NPACK;
    static constexpr int PER_THREAD = (TASKS + NT - 1) / NT;
    static constexpr bool RAGGED = TASKS % NT != 0;
    u32x4 regs[PER_THREAD];
    uint32_t okbits;
    int back;  // elements the loads were moved back by

    // m0: first padded column of this thread's packs (the same for all of them)
    __device__ __forceinline__ void issue(const bf16_t *dY, const DirectSrc &d, int row0, int m0, int tid)
    {
        uint32_t row, i, n, oy;
        d.div_p8.divmod((uint32_t)m0 >> 3, row, i);
        const bool live = (int)row < d.rows;
        d.div_Ho.divmod(live ? row : 0u, n, oy);
        const int valid = d.Wo - 8 * (int)i < 8 ? d.Wo - 8 * (int)i : 8;
        back = 8 - valid;
        const int base = (int)n * d.F * d.HoWo + (int)oy * d.Wo + 8 * (int)i - back;
        okbits = 0u;
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q) {
            const int t = tid + q * NT;
            const int f = row0 + t / NPACK;
            const bool ok = live && f < d.F && (!RAGGED || t < TASKS);
            const int e = ok ? base + f * d.HoWo : 0;
            __builtin_memcpy(&regs[q], reinterpret_cast<const char *>(dY) + 2u * (uint32_t)e, 16);
            okbits |= (ok ? 1u : 0u) << q;
        }
    }
    __device__ __forceinline__ void commit(uint4 *lds, int tid) const
    {
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q) {
            const int t = tid + q * NT;
            const int g = t % NPACK, r = t / NPACK;
            u32x4 v = regs[q];
            if (back) {
                unsigned __int128 x = ((unsigned __int128)(((uint64_t)v[3] << 32) | v[2]) << 64) | (((uint64_t)v[1] << 32) | v[0]);
                x >>= 16 * back;
                const uint64_t lo = (uint64_t)x, hi = (uint64_t)(x >> 64);
                v = u32x4{(uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32)};
            }
            const uint32_t keep = 0u - ((okbits >> q) & 1u);
#pragma unroll
            for (int w = 0; w < 4; ++w) v[w] &= keep;
            if (!RAGGED || t < TASKS) reinterpret_cast<u32x4 *>(lds)[g * (TILE_ROWS + 1) + r] = v;
        }
    }
};

// ------------------------------------------------------------------------------------------------
// The kernel
// ------------------------------------------------------------------------------------------------
struct GemmShape {
    int rows;         // extent of i
    int cols;         // extent of j (valid columns of the column operand)
    int64_t red;      // extent of the reduction index (what the loaders may touch)
    int64_t chunk;    // reduction extent handled by one split (multiple of the LDS tile)
    int tiles_i, tiles_j;
    int n_blocks;     // tiles_i * tiles_j
    int n_items;      // n_blocks * splits: work items of the launch
    int per_xcd;      // ceil(n_items / 8); the launch has 8 * per_xcd workgroups
    int fast_store;   // the result is below 4 GB: 32-bit store offsets
};

// Tile configuration: BM x BN result tile, WM x WN wavefronts, PF reduction steps of global loads in
// flight (register staging sets).
template <int BM_, int BN_, int WM_, int WN_, int PF_> struct Tile {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, PF = PF_;
    static constexpr int NT = 64 * WM * WN;
    static constexpr int TI = BM / WM / 32, TJ = BN / WN / 32;  // 32 x 32 MFMA tiles per wavefront
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "wavefront tiles are multiples of 32");
};

template <typename T, typename Cfg, bool COL_OUTER, typename Epi, int DIRECT = 0>  // DIRECT_ROWS ... DIRECT_PLANES
__global__ __launch_bounds__(Cfg::NT) void gemm_kernel(const T *__restrict__ A, int64_t lda,
                                                       const T *__restrict__ B, int64_t ldb,
                                                       GemmShape sh, Epi epi, DirectSrc direct)
{
    static_assert(!DIRECT || (!COL_OUTER && std::is_same<T, bf16_t>::value), "direct operand: bf16 model gradient only");
    constexpr int KP = Pack<T>::KP;
    constexpr int BK = NPACK * KP;
    constexpr int BM = Cfg::BM, BN = Cfg::BN, NT = Cfg::NT, TI = Cfg::TI, TJ = Cfg::TJ, PF = Cfg::PF;
    constexpr int LA = BM + 1, LB = BN + 1;
    __shared__ uint4 lds_all[2 * NPACK * (LA + LB)];  // A buffers 0, 1 then B buffers 0, 1
    __shared__ float lds_add[Epi::HAS_ROW_ADD ? BM : 1];
    auto lds_a = [&](int buf) { return lds_all + buf * (NPACK * LA); };
    auto lds_b = [&](int buf) { return lds_all + 2 * NPACK * LA + buf * (NPACK * LB); };

    // Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous range of the work
    // items (tile, split), tiles fastest: neighbouring tiles share operand panels and each XCD has its
    // own L2.  The launch is one-dimensional and padded to a multiple of 8.
    int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    int item = xcd * sh.per_xcd + slot;
    if (item >= sh.n_items) return;
    int z = item / sh.n_blocks, tile = item - z * sh.n_blocks;
    int ti = tile % sh.tiles_i, tj = tile / sh.tiles_i;  // row tiles fastest: they share the big column panel
    int row0 = ti * BM, col0 = tj * BN;
    int64_t k_begin = (int64_t)z * sh.chunk;
    int64_t k_end = k_begin + sh.chunk < sh.red ? k_begin + sh.chunk : sh.red;
    int steps = k_end > k_begin ? (int)((k_end - k_begin + BK - 1) / BK) : 0;

    int tid = threadIdx.x;
    int lane = tid % 64, wave = tid / 64;
    int wm = wave / Cfg::WN, wn = wave % Cfg::WN;
    int li = lane % 32, h = lane / 32;
    if constexpr (Epi::HAS_ROW_ADD)  // read back after the main loop's barriers
        for (int i = tid; i < BM; i += NT) lds_add[i] = epi.row_add(row0 + i);

    f32x16 acc[TI][TJ];
#pragma unroll
    for (int t = 0; t < TI; ++t)
#pragma unroll
        for (int u = 0; u < TJ; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][u][v] = 0.f;

    constexpr bool DY_DIRECT = DIRECT == DIRECT_ROWS_ONES || DIRECT == DIRECT_PHASE3;  // the row operand comes from dY as it is
    typename std::conditional<DY_DIRECT, DyLoader<BM, NT>, RedContigLoader<T, BM, NT>>::type la[PF];
    struct Unused {};  // only the column loader in use is instantiated: not every tile suits every loader
    typename std::conditional<!COL_OUTER && !DIRECT, RedContigLoader<T, BN, NT>, Unused>::type lb_red[PF];
    typename std::conditional<COL_OUTER, OuterContigLoader<T, BN, NT>, Unused>::type lb_out[PF];
    typename std::conditional<DIRECT == DIRECT_PHASE3, Phase3Loader<BN, NT>, DirectLoader<BN, NT, DIRECT>>::type lb_dir[DIRECT ? PF : 1];
    __shared__ uint2 plane_tab[DIRECT == DIRECT_PLANES ? DIRECT_TAB : 1];
    if constexpr (DIRECT != 0) {
#pragma unroll
        for (int p = 0; p < PF; ++p) lb_dir[p].init(direct, col0, tid);
        if constexpr (DIRECT == DIRECT_PLANES) {
            build_plane_table(direct, plane_tab, tid, NT);
            __syncthreads();
        }
    }

    auto issue = [&](int set, int64_t k0) {
        if constexpr (DY_DIRECT)
            la[set].issue(A, direct, row0, (int)k0 + (tid % NPACK) * 8, tid);
        else
            la[set].issue(A, lda, sh.rows, sh.red, row0, k0, tid);
        if constexpr (DIRECT)
            lb_dir[set].issue(direct, (int)k0 + (tid % NPACK) * 8, plane_tab);
        else if constexpr (COL_OUTER)
            lb_out[set].issue(B, ldb, sh.red, sh.cols, k0, col0, tid);
        else
            lb_red[set].issue(B, ldb, sh.cols, sh.red, col0, k0, tid);
    };
    auto commit = [&](int set, int buf) {
        la[set].commit(lds_a(buf), tid);
        if constexpr (DIRECT) {
            lb_dir[set].commit(lds_b(buf), tid);
            if constexpr (DIRECT == DIRECT_PHASE3) lb_dir[set].commit_ones(lds_b(buf), tid, direct.K);
        } else if constexpr (COL_OUTER)
            lb_out[set].commit(lds_b(buf), tid);
        else
            lb_red[set].commit(lds_b(buf), tid);
    };
    auto compute = [&](int buf, auto s0c, auto s1c) {
        constexpr int S0 = decltype(s0c)::value, S1 = decltype(s1c)::value;
        const uint4 *pa = lds_a(buf) + wm * (BM / Cfg::WM) + li;
        const uint4 *pb = lds_b(buf) + wn * (BN / Cfg::WN) + li;
#pragma unroll
        for (int slab = S0; slab < S1; ++slab) {
            int g = slab * 2 + h;
            uint4 a[TI], b[TJ];
#pragma unroll
            for (int t = 0; t < TI; ++t) a[t] = pa[g * LA + 32 * t];
#pragma unroll
            for (int u = 0; u < TJ; ++u) b[u] = pb[g * LB + 32 * u];
#pragma unroll
            for (int t = 0; t < TI; ++t)
#pragma unroll
                for (int u = 0; u < TJ; ++u) Mma<T>::run(a[t], b[u], acc[t][u]);
        }
    };

    // Step s computes tile s from LDS buffer s&1.  Global loads of tile s+PF are issued at the start
    // of step s into register set s%PF; the set holding tile s+1 is written to the other LDS buffer during
    // step s.  The loop is unrolled by PF so that set indices are compile-time constants.
#pragma unroll
    for (int p = 0; p < PF; ++p)
        if (p < steps) issue(p, k_begin + (int64_t)p * BK);
    if (steps > 0) commit(0, 0);
    __syncthreads();

    for (int s0 = 0; s0 < steps; s0 += PF) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            int s = s0 + p;
            if (s < steps) {
                if (s + PF < steps) issue(p, k_begin + (int64_t)(s + PF) * BK);
                // The next tile goes to LDS after the first of the step's four slabs (it lands in the other
                // buffer, which every wavefront left before the last barrier): the loads have had a slab's
                // MFMAs to arrive, and the stores and their address and mask arithmetic run under the
                // remaining three slabs of the other wavefronts (measured over the CaffeNet model gradients:
                // after 1 / 2 / 3 / 4 slabs 699 / 708 / 712 / 740 us in total).
                typedef std::integral_constant<int, 0> I0;
                typedef std::integral_constant<int, 1> I1;
                typedef std::integral_constant<int, NPACK / 2> I2;
                compute(s & 1, I0{}, I1{});
                if (s + 1 < steps) commit((p + 1) % PF, (s + 1) & 1);
                compute(s & 1, I1{}, I2{});
                __syncthreads();
            }
        }
    }

    if (sh.fast_store) {
        if constexpr (std::is_same<Epi, PartialEpilogue>::value) {
            store_tile32<TI, TJ>(acc, row0 + wm * (BM / Cfg::WM), col0 + wn * (BN / Cfg::WN), li, h, z, epi);
        } else {
            __syncthreads();  // every wavefront is done with the operand tiles (and with none, if steps == 0)
            constexpr int STRIP = 16 * staged_pitch(TJ);
            static_assert((NT / 64) * STRIP <= (int)sizeof(lds_all), "staging strips fit in the operand buffers");
            store_tile_staged<TI, TJ, 16>(acc, row0 + wm * (BM / Cfg::WM), col0 + wn * (BN / Cfg::WN), lane, z, epi,
                                          reinterpret_cast<char *>(lds_all) + wave * STRIP, lds_add, row0);
        }
        return;
    }
    // 64-bit addressing for results beyond 4 GB
#pragma unroll
    for (int u = 0; u < TJ; ++u) {
        int j = col0 + wn * (BN / Cfg::WN) + u * 32 + li;
        typename Epi::Col col = epi.column(j);
#pragma unroll
        for (int t = 0; t < TI; ++t) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int i = row0 + wm * (BM / Cfg::WM) + t * 32 + 8 * (v / 4) + 4 * h + (v % 4);
                epi.store(i, col, acc[t][u][v], epi.row_add(i), z);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Software-pipelined 256 x 256 kernel (4 wavefronts, 128 x 128 each, one workgroup per compute unit).
//
// With one wavefront per SIMD nothing hides latency unless the instruction stream itself interleaves
// MFMAs with LDS and global traffic.  A reduction step is four slabs of 16 MFMAs per wavefront; each
// slab is cut into four chunks of 4 MFMAs, and between chunks (fenced so the compiler keeps the order)
// the wavefront issues, in this rotation:
//   slab 0,1,2 : the 8 fragment reads of the next slab into the other fragment register set
//   slab 2     : the LDS writes of the next step's tile (its global loads were issued a step earlier)
//   slab 3     : barrier, the fragment reads of the next step's first slab, and the global loads of
//                the tile two steps ahead
// LDS rows are XOR-swizzled (row ^ ((row >> 3) & 7)) so that both the transposing writes of a
// column-contiguous operand and the fragment reads are free of bank conflicts.
// ------------------------------------------------------------------------------------------------
namespace pipe {

constexpr int BM = 256, BN = 256, NT = 256, LROWS = 257;

// Compile-time loop: the body receives std::integral_constant<int, I>, so every register-array index
// derived from it is a constant for the front end (arrays indexed that way stay in registers).
template <int I, int N, typename F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}
__device__ __forceinline__ int swz(int row) { return row ^ ((row >> 3) & 7); }

// The loaders of this kernel are unpredicated: row, column and reduction indices beyond the operand
// are clamped to the last valid one (their products only reach results the epilogue discards, or meet
// the zero padding of the other operand), and the row operand is zero-padded along the reduction to a
// multiple of the step.  No branch, no zero fill, nothing for the compiler to serialise on.
// Addresses are a wave-uniform 64-bit base (kept in scalar registers) plus a 32-bit per-lane byte
// offset that does not change from step to step, which keeps the vector register budget for data.
template <typename T> struct RedLoader {  // 256 rows x 8 packs: pack g = tid%8 of rows tid/8 + 32q, q = 0..7
    static constexpr int KP = Pack<T>::KP;
    // named members instead of arrays: each one is its own SSA value, nothing can end up in scratch
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 r0, r1, r2, r3, r4, r5, r6, r7;
    uint32_t o0, o1, o2, o3, o4, o5, o6, o7;  // byte offset of (row, pack) from the first row of the tile
    template <int Q> __device__ __forceinline__ u32x4 &reg()
    {
        if constexpr (Q == 0) return r0; else if constexpr (Q == 1) return r1; else if constexpr (Q == 2) return r2;
        else if constexpr (Q == 3) return r3; else if constexpr (Q == 4) return r4; else if constexpr (Q == 5) return r5;
        else if constexpr (Q == 6) return r6; else return r7;
    }
    template <int Q> __device__ __forceinline__ uint32_t &off()
    {
        if constexpr (Q == 0) return o0; else if constexpr (Q == 1) return o1; else if constexpr (Q == 2) return o2;
        else if constexpr (Q == 3) return o3; else if constexpr (Q == 4) return o4; else if constexpr (Q == 5) return o5;
        else if constexpr (Q == 6) return o6; else return o7;
    }
    __device__ __forceinline__ void init(int64_t ld, int rows, int row0, int tid)
    {
        int g = tid % NPACK, rr = tid / NPACK;
        static_for<0, 8>([&](auto q) {
            constexpr int Q = decltype(q)::value;
            int r = row0 + rr + 32 * Q;
            r = (r < rows ? r : rows - 1) - row0;
            off<Q>() = (uint32_t)(((int64_t)r * ld + g * KP) * (int64_t)sizeof(T));
        });
    }
    // tile_k: address of element (row0, k0) of the operand, wave-uniform
    template <int C> __device__ __forceinline__ void issue_part(const char *tile_k)
    {
        reg<2 * C>() = *reinterpret_cast<const u32x4 *>(tile_k + off<2 * C>());
        reg<2 * C + 1>() = *reinterpret_cast<const u32x4 *>(tile_k + off<2 * C + 1>());
    }
    template <int C> __device__ __forceinline__ void commit_part(uint4 *lds, int tid)
    {
        int g = tid % NPACK, rr = tid / NPACK;
        u32x4 *l = reinterpret_cast<u32x4 *>(lds);
        l[g * LROWS + swz(rr + 32 * (2 * C))] = reg<2 * C>();
        l[g * LROWS + swz(rr + 32 * (2 * C + 1))] = reg<2 * C + 1>();
    }
};

template <typename T> struct OuterLoader;
template <> struct OuterLoader<float> {  // columns 4*(tid%64)..+3, pack groups wave + 4q, q = 0, 1
    uint4 regs[2][4];
    uint32_t joff;
    __device__ __forceinline__ void init(int cols, int col0, int tid)
    {
        int j = col0 + (tid % 64) * 4;
        joff = (uint32_t)(j < cols ? j : cols - 4) * 4u;
    }
    template <int C> __device__ __forceinline__ void issue_part(const char *base, int64_t ld, int64_t red, int64_t k0, int wave)
    {
        int64_t ka = k0 + wave * 4 + C, kb = ka + 16;
        ka = ka < red ? ka : red - 1;
        kb = kb < red ? kb : red - 1;
        regs[0][C] = *reinterpret_cast<const uint4 *>(base + ka * ld * 4 + joff);
        regs[1][C] = *reinterpret_cast<const uint4 *>(base + kb * ld * 4 + joff);
    }
    template <int C, int Q> __device__ __forceinline__ uint4 column() const
    {
        if constexpr (C == 0) return make_uint4(regs[Q][0].x, regs[Q][1].x, regs[Q][2].x, regs[Q][3].x);
        else if constexpr (C == 1) return make_uint4(regs[Q][0].y, regs[Q][1].y, regs[Q][2].y, regs[Q][3].y);
        else if constexpr (C == 2) return make_uint4(regs[Q][0].z, regs[Q][1].z, regs[Q][2].z, regs[Q][3].z);
        else return make_uint4(regs[Q][0].w, regs[Q][1].w, regs[Q][2].w, regs[Q][3].w);
    }
    template <int C> __device__ __forceinline__ void commit_part(uint4 *lds, int tid) const
    {
        int jc = tid % 64, g = tid / 64;
        lds[g * LROWS + swz(jc * 4 + C)] = column<C, 0>();
        lds[(g + 4) * LROWS + swz(jc * 4 + C)] = column<C, 1>();
    }
};
template <> struct OuterLoader<bf16_t> {
    // one task per thread: 8 reduction rows (pack group tid/32) x 8 consecutive columns (16 bytes per row)
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 r0, r1, r2, r3, r4, r5, r6, r7;
    uint32_t joff;
    template <int E> __device__ __forceinline__ u32x4 &reg()
    {
        if constexpr (E == 0) return r0; else if constexpr (E == 1) return r1; else if constexpr (E == 2) return r2;
        else if constexpr (E == 3) return r3; else if constexpr (E == 4) return r4; else if constexpr (E == 5) return r5;
        else if constexpr (E == 6) return r6; else return r7;
    }
    __device__ __forceinline__ void init(int cols, int col0, int tid)
    {
        int j = col0 + (tid % 32) * 8;
        joff = (uint32_t)(j < cols ? j : cols - 8) * 2u;
    }
    template <int E> __device__ __forceinline__ void load_one(const char *base, uint32_t row_bytes, int red, int k0, int tid)
    {
        int k = k0 + (tid / 32) * 8 + E;
        k = k < red ? k : red - 1;
        reg<E>() = *reinterpret_cast<const u32x4 *>(base + ((uint32_t)k * row_bytes + joff));
    }
    template <int C> __device__ __forceinline__ void issue_part(const char *base, int64_t ld, int64_t red, int64_t k0, int tid)
    {
        load_one<2 * C>(base, (uint32_t)ld * 2u, (int)red, (int)k0, tid);
        load_one<2 * C + 1>(base, (uint32_t)ld * 2u, (int)red, (int)k0, tid);
    }
    static __device__ __forceinline__ uint32_t lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
    static __device__ __forceinline__ uint32_t hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }
    // column J (0..7) of the 8 x 8 block as one pack: the 8 reduction indices of that column
    template <int J> __device__ __forceinline__ u32x4 column() const
    {
        constexpr int D = J / 2;
        if constexpr (J % 2 == 0) return u32x4{lo(r0[D], r1[D]), lo(r2[D], r3[D]), lo(r4[D], r5[D]), lo(r6[D], r7[D])};
        else return u32x4{hi(r0[D], r1[D]), hi(r2[D], r3[D]), hi(r4[D], r5[D]), hi(r6[D], r7[D])};
    }
    template <int C> __device__ __forceinline__ void commit_part(uint4 *lds, int tid) const
    {
        int jc = tid % 32, g = tid / 32;
        u32x4 *l = reinterpret_cast<u32x4 *>(lds) + g * LROWS;
        l[swz(jc * 8 + 2 * C)] = column<2 * C>();
        l[swz(jc * 8 + 2 * C + 1)] = column<2 * C + 1>();
    }
};

}  // namespace pipe

template <typename T, bool COL_OUTER, typename Epi>
__global__ __launch_bounds__(256) void gemm_pipe_kernel(const T *__restrict__ A, int64_t lda,
                                                        const T *__restrict__ B, int64_t ldb, GemmShape sh, Epi epi)
{
    using namespace pipe;
    constexpr int KP = Pack<T>::KP;
    constexpr int BK = NPACK * KP;
    __shared__ uint4 lds_all[4 * NPACK * LROWS];  // A buffers 0, 1 then B buffers 0, 1
    __shared__ float lds_add[Epi::HAS_ROW_ADD ? BM : 1];
    auto lds_a = [&](int buf) { return lds_all + buf * (NPACK * LROWS); };
    auto lds_b = [&](int buf) { return lds_all + (2 + buf) * (NPACK * LROWS); };

    int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    int item = xcd * sh.per_xcd + slot;  // contiguous ranges of (tile, split) per XCD, tiles fastest
    if (item >= sh.n_items) return;
    int z = item / sh.n_blocks, tile = item - z * sh.n_blocks;
    int ti = tile % sh.tiles_i, tj = tile / sh.tiles_i;
    int row0 = ti * BM, col0 = tj * BN;
    int64_t k_begin = (int64_t)z * sh.chunk;
    int64_t k_end = k_begin + sh.chunk < sh.red ? k_begin + sh.chunk : sh.red;
    int steps = k_end > k_begin ? (int)((k_end - k_begin + BK - 1) / BK) : 0;

    int tid = threadIdx.x;
    int lane = tid % 64, wave = tid / 64;
    int wm = wave / 2, wn = wave % 2;
    int li = lane % 32, h = lane / 32;

    f32x16 acc[4][4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][u][v] = 0.f;

    if constexpr (Epi::HAS_ROW_ADD) lds_add[tid] = epi.row_add(row0 + tid);  // read back after the main loop's barriers

    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    RedLoader<T> la;
    RedLoader<T> lb_red;
    OuterLoader<T> lb_out;
    la.init(lda, sh.rows, row0, tid);
    if constexpr (COL_OUTER)
        lb_out.init(sh.cols, col0, tid);
    else
        lb_red.init(ldb, sh.cols, col0, tid);
    const char *a_tile = reinterpret_cast<const char *>(A + (int64_t)row0 * lda);
    const char *b_tile = reinterpret_cast<const char *>(COL_OUTER ? B : B + (int64_t)col0 * ldb);
    auto issue_part = [&](auto c, int64_t k0) {
        constexpr int C = decltype(c)::value;
        la.template issue_part<C>(a_tile + k0 * (int64_t)sizeof(T));
        if constexpr (COL_OUTER)
            lb_out.template issue_part<C>(b_tile, ldb, sh.red, k0, std::is_same<T, float>::value ? wave_s : tid);
        else
            lb_red.template issue_part<C>(b_tile + k0 * (int64_t)sizeof(T));
    };
    auto commit_part = [&](auto c, int buf) {
        constexpr int C = decltype(c)::value;
        la.template commit_part<C>(lds_a(buf), tid);
        if constexpr (COL_OUTER)
            lb_out.template commit_part<C>(lds_b(buf), tid);
        else
            lb_red.template commit_part<C>(lds_b(buf), tid);
    };

    uint4 fa[2][4], fb[2][4];
    // fragment rows of this lane (swizzled), relative to the tile
    int ra[4], rb[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        ra[t] = swz(wm * 128 + 32 * t + li);
        rb[t] = swz(wn * 128 + 32 * t + li);
    }
    // reads 2 of the 8 fragments of a slab: part 0 -> b0 b1, 1 -> b2 b3, 2 -> a0 a1, 3 -> a2 a3
    auto read_part = [&](auto c, auto set, int buf, int slab) {
        constexpr int C = decltype(c)::value, S = decltype(set)::value;
        int g = slab * 2 + h;
        if constexpr (C < 2) {
            fb[S][2 * C] = lds_b(buf)[g * LROWS + rb[2 * C]];
            fb[S][2 * C + 1] = lds_b(buf)[g * LROWS + rb[2 * C + 1]];
        } else {
            fa[S][2 * (C - 2)] = lds_a(buf)[g * LROWS + ra[2 * (C - 2)]];
            fa[S][2 * (C - 2) + 1] = lds_a(buf)[g * LROWS + ra[2 * (C - 2) + 1]];
        }
    };
    auto mma_chunk = [&](auto set, auto t) {
        constexpr int S = decltype(set)::value, Tt = decltype(t)::value;
        Mma<T>::run(fa[S][Tt], fb[S][0], acc[Tt][0]);
        Mma<T>::run(fa[S][Tt], fb[S][1], acc[Tt][1]);
        Mma<T>::run(fa[S][Tt], fb[S][2], acc[Tt][2]);
        Mma<T>::run(fa[S][Tt], fb[S][3], acc[Tt][3]);
    };
    using I0 = std::integral_constant<int, 0>;

    if (steps > 0) {
        static_for<0, 4>([&](auto c) { issue_part(c, k_begin); });
        static_for<0, 4>([&](auto c) { commit_part(c, 0); });
    }
    __syncthreads();
    if (steps > 1) static_for<0, 4>([&](auto c) { issue_part(c, k_begin + BK); });
    if (steps > 0) static_for<0, 4>([&](auto c) { read_part(c, I0{}, 0, 0); });

    for (int s = 0; s < steps; ++s) {
        const int buf = s & 1;
        const bool more = s + 1 < steps, more2 = s + 2 < steps;
        static_for<0, 4>([&](auto q) {
            constexpr int Q = decltype(q)::value;
            static_for<0, 4>([&](auto c) {
                constexpr int C = decltype(c)::value;
                mma_chunk(std::integral_constant<int, (Q & 1)>{}, c);
                if constexpr (Q < 3) {
                    read_part(c, std::integral_constant<int, ((Q + 1) & 1)>{}, buf, Q + 1);
                    if constexpr (Q == 2) {
                        if (more) commit_part(c, buf ^ 1);
                    }
                } else {
                    if constexpr (C == 0) __syncthreads();  // every wavefront has read `buf` and written `buf ^ 1`
                    if (more) read_part(c, I0{}, buf ^ 1, 0);
                    if (more2) issue_part(c, k_begin + (int64_t)(s + 2) * BK);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        });
    }

    if constexpr (std::is_same<Epi, PartialEpilogue>::value) {
        store_tile32<4, 4>(acc, row0 + wm * 128, col0 + wn * 128, li, h, z, epi);
    } else {
        __syncthreads();  // every wavefront is done with the operand tiles: LDS becomes staging space
        constexpr int STRIP = 32 * staged_pitch(4);
        static_assert(4 * STRIP <= (int)sizeof(lds_all), "staging strips fit in the operand buffers");
        store_tile_staged<4, 4, 32>(acc, row0 + wm * 128, col0 + wn * 128, lane, z, epi,
                                    reinterpret_cast<char *>(lds_all) + wave * STRIP, lds_add, row0);
    }
}

// Sum the per-split partial results into the final fp32 tensor, in a fixed order (deterministic): a
// workgroup takes 64 consecutive elements; wavefront l adds splits l, l+4, l+8, ... in that order, four
// loads in flight, and the four sums are then added as (s0 + s1) + (s2 + s3).
// The launch may carry extra workgroups (blockIdx >= main_blocks) that finish the bias gradient: one
// wavefront per filter adds that filter's per-block sums left by the dY packing kernel (strided per lane in
// block order, then a fixed tree) -- the same arithmetic as bias_reduce_kernel, without a launch of its own.
// PHASED: the partial results are [F][K' + 1] in the phase-split order of a stride-4 layer (see
// launch_gemm_wgrad_phase), K' index ((c * 4 + ph) * kh + ky) * kwq + kq standing for window column
// kx = 4 kq + ph; entries with kx >= kw are padding and are dropped, the others go to [F][C][kh][kw];
// column K' is the bias gradient.
struct PhaseMap { int32_t C, kh, kw; FastDiv div_Kp, div_khkwq, div_kwq; };

template <bool PHASED>
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ partials, int splits,
                                                              int64_t count, float *__restrict__ out, unsigned main_blocks,
                                                              const float *__restrict__ bias_partials, int bias_blocks,
                                                              int F, float *__restrict__ dbias, PhaseMap pm)
{
    __shared__ float part[4][64];
    const int c = threadIdx.x % 64, l = threadIdx.x / 64;
    if (blockIdx.x >= main_blocks) {
        const int f = (int)(blockIdx.x - main_blocks) * 4 + l;
        if (f < F) {
            float acc = 0.f;
            for (int b = c; b < bias_blocks; b += 64) acc += bias_partials[(int64_t)f * bias_blocks + b];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
            if (c == 0) dbias[f] = acc;
        }
        return;
    }
    const int64_t i = (int64_t)blockIdx.x * 64 + c;
    float acc = 0.f;
    if (i < count) {
        const float *p = partials + i;
        int z = l;
        for (; z + 12 < splits; z += 16) {
            float a0 = p[(int64_t)z * count], a1 = p[(int64_t)(z + 4) * count];
            float a2 = p[(int64_t)(z + 8) * count], a3 = p[(int64_t)(z + 12) * count];
            acc += a0, acc += a1, acc += a2, acc += a3;
        }
        for (; z < splits; z += 4) acc += p[(int64_t)z * count];
    }
    part[l][c] = acc;
    __syncthreads();
    if (l == 0 && i < count) {
        const float sum = (part[0][c] + part[1][c]) + (part[2][c] + part[3][c]);
        if constexpr (PHASED) {
            uint32_t f, kp, cp, rem, ky, kq;
            pm.div_Kp.divmod((uint32_t)i, f, kp);  // columns per row: K' + 1, the last one the bias gradient
            pm.div_khkwq.divmod(kp, cp, rem);
            pm.div_kwq.divmod(rem, ky, kq);
            const int kx = 4 * (int)kq + (int)(cp % 4u);
            if (kp + 1u == pm.div_Kp.d) {
                if (dbias != nullptr) dbias[f] = sum;
            } else if (kx < pm.kw) {
                out[(((int64_t)f * pm.C + cp / 4u) * pm.kh + ky) * pm.kw + kx] = sum;
            }
        } else {
            out[i] = sum;
        }
    }
}

// The same ordered sum for element counts that are a multiple of 4: a thread owns four consecutive elements and adds
// the splits in ascending order, eight 16-byte loads in flight (the 4-byte loads of the kernel above keep too few
// bytes in flight to reach the memory system's rate).  Extra workgroups finish the bias gradient as above.
__global__ __launch_bounds__(256) void reduce_partials_vec_kernel(const float4 *__restrict__ partials, int splits, int64_t count4,
                                                                  float4 *__restrict__ out, unsigned main_blocks,
                                                                  const float *__restrict__ bias_partials, int bias_blocks,
                                                                  int F, float *__restrict__ dbias)
{
    if (blockIdx.x >= main_blocks) {
        const int c = threadIdx.x % 64, f = (int)(blockIdx.x - main_blocks) * 4 + threadIdx.x / 64;
        if (f < F) {
            float acc = 0.f;
            for (int b = c; b < bias_blocks; b += 64) acc += bias_partials[(int64_t)f * bias_blocks + b];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
            if (c == 0) dbias[f] = acc;
        }
        return;
    }
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count4) return;
    const float4 *p = partials + i;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    int z = 0;
    for (; z + 8 <= splits; z += 8) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p[(int64_t)(z + u) * count4];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc.x += v[u].x, acc.y += v[u].y, acc.z += v[u].z, acc.w += v[u].w;
    }
    for (; z < splits; ++z) {
        const float4 v = p[(int64_t)z * count4];
        acc.x += v.x, acc.y += v.y, acc.z += v.z, acc.w += v.w;
    }
    out[i] = acc;
}

static GemmShape make_shape(int rows, int cols, int64_t red, int64_t chunk, int bm, int bn, int splits)
{
    GemmShape s;
    s.rows = rows;
    s.cols = cols;
    s.red = red;
    s.chunk = chunk;
    s.tiles_i = (rows + bm - 1) / bm;
    s.tiles_j = (cols + bn - 1) / bn;
    s.n_blocks = s.tiles_i * s.tiles_j;
    s.n_items = s.n_blocks * splits;
    s.per_xcd = (s.n_items + 7) / 8;
    s.fast_store = 0;
    return s;
}

// Tile configurations compiled in.  Index = the tuning override (omni_tuning_set, for sweeps) or
// the choice of pick_tile().
typedef Tile<128, 128, 2, 2, 1> Tile0;
typedef Tile<128, 128, 2, 2, 2> Tile1;
typedef Tile<256, 128, 2, 2, 1> Tile2;
typedef Tile<256, 128, 2, 2, 2> Tile3;
typedef Tile<128, 256, 2, 2, 1> Tile4;
typedef Tile<256, 256, 2, 2, 1> Tile5;
typedef Tile<256, 256, 4, 2, 1> Tile6;
typedef Tile<256, 256, 2, 4, 1> Tile7;
constexpr int TILE_PIPE = 8;  // the software-pipelined 256 x 256 kernel
typedef Tile<192, 256, 2, 4, 1> Tile9;
typedef Tile<384, 128, 4, 2, 1> Tile10;
constexpr int N_TILES = 11;

static int g_tile_override = -1;  // omni_tuning_set(OMNI_TUNE_GEMM_TILE, ...): sweeps and tests only
void set_gemm_tile_override(int v) { g_tile_override = (v >= 0 && v < N_TILES) ? v : -1; }
static int tile_override() { return g_tile_override; }

// Tile choice: the 256 x 256 tile halves the operand traffic per flop, so it wins whenever the result
// fills its tiles about as well as it fills 128 x 128 ones (measured on the CaffeNet-shaped layers: 256
// and 2400/3456-wide results take it, 96- and 384-wide ones lose a quarter or more of the tile to padding).
static int pick_tile(int rows, int cols)
{
    int o = tile_override();
    if (o >= 0) return o;
    auto fill = [](int n, int t) { return (double)n / (double)(((n + t - 1) / t) * t); };
    double u256 = fill(rows, 256) * fill(cols, 256), u128 = fill(rows, 128) * fill(cols, 128);
    return u256 >= 0.9 * u128 ? 6 : 0;
}

// The model gradient has a third candidate: 384 x 128, which takes a 384-row result (F = 384) in one row tile.
static int pick_wgrad_tile(int rows, int cols)
{
    int o = tile_override();
    if (o >= 0) return o;
    auto fill = [](int n, int t) { return (double)n / (double)(((n + t - 1) / t) * t); };
    double u256 = fill(rows, 256) * fill(cols, 256), u128 = fill(rows, 128) * fill(cols, 128);
    double u384 = fill(rows, 384) * fill(cols, 128);
    if (u384 > u256 && u384 >= 0.9 * u128) return 10;
    return u256 >= 0.9 * u128 ? 6 : 0;
}

static bool direct_tile(int tile) { return tile == 6 || tile == 9 || tile == 10; }

static void tile_dims(int tile, int *bm, int *bn)
{
    static const int dims[N_TILES][2] = {{128, 128}, {128, 128}, {256, 128}, {256, 128}, {128, 256},
                                         {256, 256}, {256, 256}, {256, 256}, {256, 256}, {192, 256}, {384, 128}};
    *bm = dims[tile][0];
    *bn = dims[tile][1];
}

// Whether the model gradient of this layer takes its column operand straight from X.  Assembling a pack
// costs vector ALU work that is shared by the rows of the result tile, so this pays only with the
// 256 x 256 tile (measured: with 128-row tiles lowering first and streaming D-hat is faster).
bool wgrad_direct_supported(const ConvGeom &g, int dtype)
{
    return dtype == OMNI_BF16 && g.sh == 1 && g.sw == 1 && g.pw < 24 && direct_tile(pick_wgrad_tile(g.F, g.K)) &&
           (int64_t)g.N * g.C * g.H * g.W < 0x7fffffffll - 16 && (int64_t)g.N * g.C * g.H * g.W >= 8;
}

// Whether the direct model gradient pads whole image planes (see DIRECT_PLANES) rather than output rows.
bool wgrad_direct_planes(const ConvGeom &g)
{
    return g.sh == 1 && g.sw == 1 && g.Wo == g.W &&
           (int64_t)((g.Ho * g.Wo + 7) / 8) * (g.kh * g.kw + 1) <= DIRECT_TAB;
}

// Result tile of the model-gradient GEMM for a layer (the split planner needs the tile count).
void gemm_wgrad_tile(int F, int K, int *bm, int *bn) { tile_dims(pick_wgrad_tile(F, K), bm, bn); }

template <typename T, typename Cfg, bool COL_OUTER, typename Epi>
static void launch_cfg(const T *A, int64_t lda, const T *B, int64_t ldb, int rows, int cols, int64_t red,
                       int64_t chunk, int splits, const Epi &epi, hipStream_t s)
{
    GemmShape sh = make_shape(rows, cols, red, chunk, Cfg::BM, Cfg::BN, splits);
    sh.fast_store = epi.fits32() ? 1 : 0;
    dim3 grid(sh.per_xcd * 8, 1, 1);
    hipLaunchKernelGGL((gemm_kernel<T, Cfg, COL_OUTER, Epi>), grid, dim3(Cfg::NT), 0, s, A, lda, B, ldb, sh, epi,
                       DirectSrc{});
}

// Model gradient with the column operand read from X (see DirectLoader), in the mode the geometry allows.
template <typename Cfg>
static void launch_direct(const bf16_t *A, int64_t lda, const DirectSrc &d, int rows, int cols, int64_t red,
                          int64_t chunk, int splits, const PartialEpilogue &epi, hipStream_t s)
{
    GemmShape sh = make_shape(rows, cols, red, chunk, Cfg::BM, Cfg::BN, splits);
    sh.fast_store = epi.fits32() ? 1 : 0;
    dim3 grid(sh.per_xcd * 8, 1, 1);
    const int p8 = (int)d.div_p8.d;
    if (d.KK > 0)
        hipLaunchKernelGGL((gemm_kernel<bf16_t, Cfg, false, PartialEpilogue, DIRECT_PLANES>), grid, dim3(Cfg::NT), 0, s, A,
                           lda, (const bf16_t *)nullptr, (int64_t)0, sh, epi, d);
    else if (p8 == 1 || p8 == 2 || p8 == 4 || p8 == 8)
        hipLaunchKernelGGL((gemm_kernel<bf16_t, Cfg, false, PartialEpilogue, DIRECT_ROWS_FIXED>), grid, dim3(Cfg::NT), 0, s,
                           A, lda, (const bf16_t *)nullptr, (int64_t)0, sh, epi, d);
    else
        hipLaunchKernelGGL((gemm_kernel<bf16_t, Cfg, false, PartialEpilogue, DIRECT_ROWS>), grid, dim3(Cfg::NT), 0, s, A, lda,
                           (const bf16_t *)nullptr, (int64_t)0, sh, epi, d);
}

template <typename T, bool COL_OUTER, typename Epi>
static void launch_any(int tile, const T *A, int64_t lda, const T *B, int64_t ldb, int rows, int cols, int64_t red,
                       int64_t chunk, int splits, const Epi &epi, hipStream_t s)
{
    // the pipelined kernel only has 32-bit load and store offsets
    if (tile == TILE_PIPE && (!epi.fits32() || (double)lda * sizeof(T) * 256 >= 4.0e9 || (double)ldb * sizeof(T) * 256 >= 4.0e9 ||
                              (COL_OUTER && (double)ldb * sizeof(T) * (double)red >= 4.0e9)))
        tile = 6;
    if (tile == TILE_PIPE) {
        GemmShape sh = make_shape(rows, cols, red, chunk, pipe::BM, pipe::BN, splits);
        dim3 grid(sh.per_xcd * 8, 1, 1);
        hipLaunchKernelGGL((gemm_pipe_kernel<T, COL_OUTER, Epi>), grid, dim3(pipe::NT), 0, s, A, lda, B, ldb, sh, epi);
        return;
    }
    switch (tile) {
    case 1: launch_cfg<T, Tile1, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    case 2: launch_cfg<T, Tile2, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    case 3: launch_cfg<T, Tile3, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    case 4: launch_cfg<T, Tile4, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    case 5: launch_cfg<T, Tile5, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    case 6: launch_cfg<T, Tile6, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    case 7: launch_cfg<T, Tile7, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    case 9: launch_cfg<T, Tile9, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    case 10:
        if constexpr (!COL_OUTER) {  // too few columns for the column-contiguous loader's tasks
            launch_cfg<T, Tile10, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s);
            break;
        }
        [[fallthrough]];
    default: launch_cfg<T, Tile0, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    }
}

// Tile of a split product: the 256 x 256 one where the result fills it about as well, else 128 x 128
static int split_tile(int rows, int cols) { return pick_tile(rows, cols) == 6 ? 6 : 0; }
void gemm_split_tile(int rows, int cols, int *bm, int *bn) { tile_dims(split_tile(rows, cols), bm, bn); }

template <typename T, typename Epi>
static void launch_split(const T *A, int64_t lda, const T *B, int64_t ldb, int rows, int cols, int64_t red, int64_t chunk,
                         int splits, float *partials, const Epi &epi, hipStream_t s)
{
    PartialEpilogue pe{partials, rows, cols};
    if (split_tile(rows, cols) == 6)
        launch_cfg<T, Tile6, true, PartialEpilogue>(A, lda, B, ldb, rows, cols, red, chunk, splits, pe, s);
    else
        launch_cfg<T, Tile0, true, PartialEpilogue>(A, lda, B, ldb, rows, cols, red, chunk, splits, pe, s);
    const int64_t count = (int64_t)rows * cols;
    hipLaunchKernelGGL((reduce_store_kernel<Epi>), dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, partials, splits,
                       rows, cols, epi);
}

template <typename T>
static int run_forward(const ConvGeom &g, const GemmFwdArgs &a, hipStream_t s)
{
    constexpr int BK = NPACK * Pack<T>::KP;
    // K-hat is zero-padded along K to a multiple of the pack size; rows of D-hat beyond K read as zero.
    FwdEpilogue<T> epi{(T *)a.Y, a.bias, g.F, g.M, g.HoWo, g.div_HoWo, a.relu};
    ProfScope prof(KID_GEMM_FWD, s, 2.0 * g.M * (double)g.K * g.F,
                   ((double)g.F * g.K + (double)g.K * g.M + (double)g.F * g.M) * sizeof(T));
    if (a.splits > 1)
        launch_split<T>((const T *)a.Khat, a.ldk, (const T *)a.Dhat, a.ldd, g.F, (int)a.ldd, g.K, a.chunk, a.splits, a.partials,
                        epi, s);
    else
        launch_any<T, true, FwdEpilogue<T>>(pick_tile(g.F, (int)a.ldd), (const T *)a.Khat, a.ldk, (const T *)a.Dhat, a.ldd,
                                            g.F, (int)a.ldd, g.K, round_up(g.K, BK), 1, epi, s);
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

int launch_gemm_forward(const ConvGeom &g, int dtype, const GemmFwdArgs &a, hipStream_t s)
{
    return dtype == OMNI_BF16 ? run_forward<bf16_t>(g, a, s) : run_forward<float>(g, a, s);
}

template <typename T>
static int run_dgrad(const ConvGeom &g, const GemmDgradArgs &a, hipStream_t s)
{
    constexpr int BK = NPACK * Pack<T>::KP;
    RowMajorEpilogue<T> epi{(T *)a.dDhat, a.ldd, g.K, (int)a.ldd};
    ProfScope prof(KID_GEMM_DGRAD, s, 2.0 * g.M * (double)g.K * g.F,
                   ((double)g.F * g.K + (double)g.K * g.M + (double)g.F * g.M) * sizeof(T));
    if (a.splits > 1)
        launch_split<T>((const T *)a.KhatT, a.ldk, (const T *)a.dYhat, a.ldd, g.K, (int)a.ldd, g.F, a.chunk, a.splits,
                        a.partials, epi, s);
    else
        launch_any<T, true, RowMajorEpilogue<T>>(pick_tile(g.K, (int)a.ldd), (const T *)a.KhatT, a.ldk, (const T *)a.dYhat,
                                                 a.ldd, g.K, (int)a.ldd, g.F, round_up(g.F, BK), 1, epi, s);
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

int launch_gemm_dgrad(const ConvGeom &g, int dtype, const GemmDgradArgs &a, hipStream_t s)
{
    return dtype == OMNI_BF16 ? run_dgrad<bf16_t>(g, a, s) : run_dgrad<float>(g, a, s);
}

// Data gradient of a layer whose window is the whole, unpadded image (a fully connected layer, Sec. II-C):
// dX [N][K] = dY [N][F] * W [F][K] with all three tensors in their natural layouts -- dY's rows run along the
// reduction, W's rows along the result's columns -- so nothing is packed, transposed or scattered back.
bool dgrad_dense_supported(const ConvGeom &g)
{
    return g.Ho == 1 && g.Wo == 1 && g.ph == 0 && g.pw == 0 && g.kh == g.H && g.kw == g.W && g.F % 8 == 0 && g.K % 8 == 0;
}

template <typename T>
static int run_dgrad_dense(const ConvGeom &g, const void *dY, const void *W, void *dX, float *partials, int splits,
                           int64_t chunk, hipStream_t s)
{
    constexpr int BK = NPACK * Pack<T>::KP;
    RowMajorEpilogue<T> epi{(T *)dX, (int64_t)g.K, g.N, g.K};
    ProfScope prof(KID_GEMM_DGRAD, s, 2.0 * g.N * (double)g.K * g.F,
                   ((double)g.F * g.K + (double)g.K * g.N + (double)g.F * g.N) * sizeof(T));
    if (splits > 1)
        launch_split<T>((const T *)dY, (int64_t)g.F, (const T *)W, (int64_t)g.K, g.N, g.K, g.F, chunk, splits, partials, epi, s);
    else
        launch_any<T, true, RowMajorEpilogue<T>>(pick_tile(g.N, g.K), (const T *)dY, (int64_t)g.F, (const T *)W, (int64_t)g.K,
                                                 g.N, g.K, g.F, round_up(g.F, BK), 1, epi, s);
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

int launch_gemm_dgrad_dense(const ConvGeom &g, int dtype, const void *dY, const void *W, void *dX, float *partials,
                            int splits, int64_t chunk, hipStream_t s)
{
    return dtype == OMNI_BF16 ? run_dgrad_dense<bf16_t>(g, dY, W, dX, partials, splits, chunk, s)
                              : run_dgrad_dense<float>(g, dY, W, dX, partials, splits, chunk, s);
}

template <typename T>
static int run_wgrad(const ConvGeom &g, const GemmWgradArgs &a, hipStream_t s)
{
    float *target = a.splits == 1 ? a.dW : a.partials;
    PartialEpilogue epi{target, g.F, g.K};
    {
        ProfScope prof(KID_GEMM_WGRAD, s, 2.0 * g.M * (double)g.K * g.F,
                       ((double)g.K * g.M + (double)g.F * g.M) * sizeof(T) + 4.0 * g.F * g.K * a.splits);
        if (a.X_direct != nullptr) {
            if constexpr (std::is_same<T, bf16_t>::value) {
                const bool planes = wgrad_direct_planes(g);
                const int unit = planes ? g.Ho * g.Wo : g.Wo;  // what is padded to a multiple of 8 positions
                DirectSrc d{(const bf16_t *)a.X_direct, g.C, g.H, g.W, g.H * g.W, g.K, g.ph, g.pw,
                            planes ? g.N : g.N * g.Ho, (int32_t)((int64_t)g.N * g.C * g.H * g.W),
                            FastDiv((uint32_t)((unit + 7) / 8)), FastDiv((uint32_t)g.Ho), g.div_khkw, g.div_kw,
                            g.Ho * g.Wo, planes ? g.kh * g.kw : 0, FastDiv((uint32_t)g.W), 1, g.F, g.Wo};
                switch (pick_wgrad_tile(g.F, g.K)) {
                case 9: launch_direct<Tile9>((const bf16_t *)a.dYhat, a.ldd, d, g.F, g.K, a.ldd, a.chunk, a.splits, epi, s); break;
                case 10: launch_direct<Tile10>((const bf16_t *)a.dYhat, a.ldd, d, g.F, g.K, a.ldd, a.chunk, a.splits, epi, s); break;
                default: launch_direct<Tile6>((const bf16_t *)a.dYhat, a.ldd, d, g.F, g.K, a.ldd, a.chunk, a.splits, epi, s); break;
                }
            }
        } else {
            launch_any<T, false, PartialEpilogue>(pick_wgrad_tile(g.F, g.K), (const T *)a.dYhat, a.ldd, (const T *)a.Dhat,
                                                  a.ldd, g.F, g.K, a.ldd, a.chunk, a.splits, epi, s);
        }
    }
    OMNI_LAUNCH_CHECK();
    if (a.splits > 1) return launch_wgrad_reduce(g, a.partials, a.splits, a.dW, a.bias_partials, a.bias_blocks, a.dbias, s);
    return OMNI_OK;
}

int launch_wgrad_reduce(const ConvGeom &g, const float *partials, int splits, float *dW, const float *bias_partials,
                        int bias_blocks, float *dbias, hipStream_t s)
{
    int64_t count = (int64_t)g.F * g.K;
    ProfScope prof(KID_REDUCE_PARTIALS, s, 0.0, 4.0 * count * (splits + 1));
    const unsigned bias_wgs = dbias != nullptr ? (unsigned)((g.F + 3) / 4) : 0u;
    if (count % 4 == 0) {
        const unsigned vec_blocks = (unsigned)((count / 4 + 255) / 256);
        hipLaunchKernelGGL(reduce_partials_vec_kernel, dim3(vec_blocks + bias_wgs), dim3(256), 0, s, (const float4 *)partials, splits,
                           count / 4, (float4 *)dW, vec_blocks, bias_partials, bias_blocks, g.F, dbias);
        OMNI_LAUNCH_CHECK();
        return OMNI_OK;
    }
    const unsigned main_blocks = (unsigned)((count + 63) / 64);
    hipLaunchKernelGGL(reduce_partials_kernel<false>, dim3(main_blocks + bias_wgs), dim3(256), 0, s, partials, splits, count, dW,
                       main_blocks, bias_partials, bias_blocks, g.F, dbias, PhaseMap{});
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

// ------------------------------------------------------------------------------------------------
// Model gradient of a layer with horizontal stride 4 and no padding (CaffeNet's conv1) without D-hat.
// The input is first split by x mod 4 into four phase images, X4 [N][C * 4][H][WP] with
// X4(n, 4c + ph, y, xq) = X(n, c, y, 4 xq + ph) (zero where that column does not exist).  Window column
// kx = 4 kq + ph of output column ox then meets phase image ph at xq = ox + kq: the layer is a convolution
// of X4 with horizontal stride 1, 4C channels and a window of kh x ceil(kw / 4), which the row mode of
// DirectLoader reads as it stands (8 consecutive output columns = 8 consecutive xq).  The result is
// [F][K'] in that order, K' = 4C * kh * ceil(kw / 4), window columns beyond kw being padding; the ordered
// reduction of the split partial results puts it back into [F][C][kh][kw].
// One 96 x 512 result tile (8 wavefronts, 96 x 64 each) holds the whole gradient, so the launch is one
// workgroup per split of the reduction.
// ------------------------------------------------------------------------------------------------
typedef Tile<96, 512, 1, 8, 1> TilePhase;

static int phase_kwq(const ConvGeom &g) { return (g.kw + 3) / 4; }
int wgrad_phase_kp(const ConvGeom &g) { return 4 * g.C * g.kh * phase_kwq(g); }
int wgrad_phase_wp(const ConvGeom &g) { return (int)round_up((g.W + 3) / 4, 8); }

bool wgrad_phase_supported(const ConvGeom &g, int dtype)
{
    if (dtype != OMNI_BF16 || g.sw != 4 || g.ph != 0 || g.pw != 0 || g.F > TilePhase::BM || g.Wo < 8) return false;
    if (wgrad_phase_kp(g) + 1 > TilePhase::BN) return false;  // + 1: the column of the bias gradient
    int64_t total4 = (int64_t)g.N * g.C * 4 * g.H * wgrad_phase_wp(g);
    return total4 < 0x7fffffffll - 16 && total4 >= 8 && (int64_t)g.N * g.C * g.H * g.W < 0x7fffffffll - 64 &&
           (int64_t)g.N * g.F * g.HoWo < 0x7fffffffll - 16;
}

// partials: [splits][F][K' + 1] floats; `ld` = the padded reduction extent (dyhat_rows_ld)
int launch_gemm_wgrad_phase(const ConvGeom &g, const void *X4, const void *dY, int64_t ld, float *partials, int splits,
                            int64_t chunk, float *dW, float *dbias, hipStream_t s)
{
    const int kwq = phase_kwq(g), Kp = wgrad_phase_kp(g), WP = wgrad_phase_wp(g);
    PartialEpilogue epi{partials, g.F, Kp + 1};
    {
        ProfScope prof(KID_GEMM_WGRAD, s, 2.0 * g.M * (double)g.K * g.F,
                       ((double)g.N * g.C * 4 * g.H * WP + (double)g.F * g.M) * 2.0 + 4.0 * g.F * (Kp + 1) * splits);
        DirectSrc d{(const bf16_t *)X4, 4 * g.C, g.H, WP, g.H * WP, Kp, 0, 0, g.N * g.Ho,
                    (int32_t)((int64_t)g.N * g.C * 4 * g.H * WP), FastDiv((uint32_t)((g.Wo + 7) / 8)), FastDiv((uint32_t)g.Ho),
                    FastDiv((uint32_t)(g.kh * kwq)), FastDiv((uint32_t)kwq), g.Ho * g.Wo, 0, FastDiv((uint32_t)WP), g.sh,
                    g.F, g.Wo};
        GemmShape sh = make_shape(g.F, Kp + 1, ld, chunk, TilePhase::BM, TilePhase::BN, splits);
        sh.fast_store = epi.fits32() ? 1 : 0;
        // three groups per window row and every pack's ten elements inside its row of X4: one load per three rows
        const bool triples = kwq == 3 && 8 * ((g.Wo + 7) / 8) + 2 <= WP;
        if (triples)
            hipLaunchKernelGGL((gemm_kernel<bf16_t, TilePhase, false, PartialEpilogue, DIRECT_PHASE3>), dim3(sh.per_xcd * 8),
                               dim3(TilePhase::NT), 0, s, (const bf16_t *)dY, (int64_t)0, (const bf16_t *)nullptr, (int64_t)0, sh, epi, d);
        else
            hipLaunchKernelGGL((gemm_kernel<bf16_t, TilePhase, false, PartialEpilogue, DIRECT_ROWS_ONES>), dim3(sh.per_xcd * 8),
                               dim3(TilePhase::NT), 0, s, (const bf16_t *)dY, (int64_t)0, (const bf16_t *)nullptr, (int64_t)0, sh, epi, d);
    }
    OMNI_LAUNCH_CHECK();
    const int64_t count = (int64_t)g.F * (Kp + 1);
    ProfScope prof(KID_REDUCE_PARTIALS, s, 0.0, 4.0 * count * (splits + 1));
    const unsigned main_blocks = (unsigned)((count + 63) / 64);
    PhaseMap pm{g.C, g.kh, g.kw, FastDiv((uint32_t)(Kp + 1)), FastDiv((uint32_t)(g.kh * kwq)), FastDiv((uint32_t)kwq)};
    hipLaunchKernelGGL(reduce_partials_kernel<true>, dim3(main_blocks), dim3(256), 0, s, partials, splits, count, dW,
                       main_blocks, (const float *)nullptr, 0, g.F, dbias, pm);
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

int launch_gemm_wgrad(const ConvGeom &g, int dtype, const GemmWgradArgs &a, hipStream_t s)
{
    return dtype == OMNI_BF16 ? run_wgrad<bf16_t>(g, a, s) : run_wgrad<float>(g, a, s);
}

}  // namespace omni
