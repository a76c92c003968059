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
#include "common.h"

namespace omni {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int BM = 128;        // rows of the result tile
constexpr int BN = 128;        // columns of the result tile
constexpr int NPACK = 8;       // 16-byte packs along the reduction per LDS tile
constexpr int LDS_ROWS = 129;  // 128 rows + 1 pack of padding: spreads the 8 packs of a row over the banks
constexpr int NTHREADS = 256;

template <typename T> struct Pack;
template <> struct Pack<float> { static constexpr int KP = 4; };
template <> struct Pack<bf16_t> { static constexpr int KP = 8; };

int gemm_red_tile(int dtype) { return dtype == OMNI_BF16 ? NPACK * 8 : NPACK * 4; }

// ------------------------------------------------------------------------------------------------
// Operand loaders: global memory -> registers (issue()), registers -> LDS (commit()).
// ------------------------------------------------------------------------------------------------

// Operand stored [rows][ld] with the reduction index contiguous.  Element (r, k) is valid for
// r < rows and k < red; ld and red are multiples of the pack size and the base is 16-byte aligned.
template <typename T, int TILE_ROWS> struct RedContigLoader {
    static constexpr int KP = Pack<T>::KP;
    static constexpr int PER_THREAD = TILE_ROWS * NPACK / NTHREADS;
    uint4 regs[PER_THREAD];

    __device__ __forceinline__ void issue(const T *base, int64_t ld, int rows, int64_t red, int row0,
                                          int64_t k0, int tid)
    {
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q) {
            int t = tid + q * NTHREADS;
            int g = t % NPACK, r = t / NPACK;
            int64_t k = k0 + (int64_t)g * KP;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (row0 + r < rows && k < red)
                v = *reinterpret_cast<const uint4 *>(base + (int64_t)(row0 + r) * ld + k);
            regs[q] = v;
        }
    }
    __device__ __forceinline__ void commit(uint4 *lds, int tid) const
    {
#pragma unroll
        for (int q = 0; q < PER_THREAD; ++q) {
            int t = tid + q * NTHREADS;
            int g = t % NPACK, r = t / NPACK;
            lds[g * LDS_ROWS + r] = regs[q];
        }
    }
};

// Operand stored [red][ld] with the result's column index j contiguous.  Element (k, j) is valid
// for k < red and j < cols; ld and cols are multiples of 8 and the base is 16-byte aligned.
template <typename T> struct OuterContigLoader;

template <> struct OuterContigLoader<float> {
    // one task per thread: pack g (4 reduction rows) x 4 consecutive columns
    uint4 regs[4];
    __device__ __forceinline__ void issue(const float *base, int64_t ld, int64_t red, int cols,
                                          int64_t k0, int col0, int tid)
    {
        int jc = tid % 32, g = tid / 32;
        int j = col0 + jc * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            int64_t k = k0 + g * 4 + e;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (k < red && j < cols) v = *reinterpret_cast<const uint4 *>(base + k * ld + j);
            regs[e] = v;
        }
    }
    __device__ __forceinline__ void commit(uint4 *lds, int tid) const
    {
        int jc = tid % 32, g = tid / 32;
        uint4 *dst = lds + g * LDS_ROWS + jc * 4;
        dst[0] = make_uint4(regs[0].x, regs[1].x, regs[2].x, regs[3].x);
        dst[1] = make_uint4(regs[0].y, regs[1].y, regs[2].y, regs[3].y);
        dst[2] = make_uint4(regs[0].z, regs[1].z, regs[2].z, regs[3].z);
        dst[3] = make_uint4(regs[0].w, regs[1].w, regs[2].w, regs[3].w);
    }
};

template <> struct OuterContigLoader<bf16_t> {
    // one task per thread: pack g (8 reduction rows) x 4 consecutive columns (8 bytes per row)
    uint2 regs[8];
    __device__ __forceinline__ void issue(const bf16_t *base, int64_t ld, int64_t red, int cols,
                                          int64_t k0, int col0, int tid)
    {
        int jc = tid % 32, g = tid / 32;
        int j = col0 + jc * 4;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int64_t k = k0 + g * 8 + e;
            uint2 v = make_uint2(0, 0);
            if (k < red && j < cols) v = *reinterpret_cast<const uint2 *>(base + k * ld + j);
            regs[e] = v;
        }
    }
    static __device__ __forceinline__ uint32_t lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
    static __device__ __forceinline__ uint32_t hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }
    __device__ __forceinline__ void commit(uint4 *lds, int tid) const
    {
        int jc = tid % 32, g = tid / 32;
        uint4 *dst = lds + g * LDS_ROWS + jc * 4;
        // column j = 2d + h of the 8 x 4 block becomes one pack: 8 reduction indices of column j
        dst[0] = make_uint4(lo(regs[0].x, regs[1].x), lo(regs[2].x, regs[3].x), lo(regs[4].x, regs[5].x), lo(regs[6].x, regs[7].x));
        dst[1] = make_uint4(hi(regs[0].x, regs[1].x), hi(regs[2].x, regs[3].x), hi(regs[4].x, regs[5].x), hi(regs[6].x, regs[7].x));
        dst[2] = make_uint4(lo(regs[0].y, regs[1].y), lo(regs[2].y, regs[3].y), lo(regs[4].y, regs[5].y), lo(regs[6].y, regs[7].y));
        dst[3] = make_uint4(hi(regs[0].y, regs[1].y), hi(regs[2].y, regs[3].y), hi(regs[4].y, regs[5].y), hi(regs[6].y, regs[7].y));
    }
};

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
    int n_blocks;     // tiles_i * tiles_j (the launch is padded to a multiple of 8)
    int per_xcd;      // ceil(n_blocks / 8)
};

template <typename T, bool COL_OUTER, typename Epi>
__global__ __launch_bounds__(NTHREADS) void gemm_kernel(const T *__restrict__ A, int64_t lda,
                                                        const T *__restrict__ B, int64_t ldb,
                                                        GemmShape sh, Epi epi)
{
    constexpr int KP = Pack<T>::KP;
    constexpr int BK = NPACK * KP;
    __shared__ uint4 lds_a[2][NPACK * LDS_ROWS];
    __shared__ uint4 lds_b[2][NPACK * LDS_ROWS];

    // Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous range of tiles
    // (neighbouring tiles share operand panels, and each XCD has its own L2).
    int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    int tile = xcd * sh.per_xcd + slot;
    if (tile >= sh.n_blocks) return;
    int ti = tile % sh.tiles_i, tj = tile / sh.tiles_i;  // row tiles fastest: they share the big column panel
    int row0 = ti * BM, col0 = tj * BN;
    int z = blockIdx.y;
    int64_t k_begin = (int64_t)z * sh.chunk;
    int64_t k_end = k_begin + sh.chunk < sh.red ? k_begin + sh.chunk : sh.red;
    int steps = k_end > k_begin ? (int)((k_end - k_begin + BK - 1) / BK) : 0;

    int tid = threadIdx.x;
    int lane = tid % 64, wave = tid / 64;
    int wm = wave / 2, wn = wave % 2;
    int li = lane % 32, h = lane / 32;

    f32x16 acc[2][2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][u][v] = 0.f;

    RedContigLoader<T, BM> la;
    RedContigLoader<T, BN> lb_red;
    OuterContigLoader<T> lb_out;

    auto issue = [&](int64_t k0) {
        la.issue(A, lda, sh.rows, sh.red, row0, k0, tid);
        if constexpr (COL_OUTER)
            lb_out.issue(B, ldb, sh.red, sh.cols, k0, col0, tid);
        else
            lb_red.issue(B, ldb, sh.cols, sh.red, col0, k0, tid);
    };
    auto commit = [&](int buf) {
        la.commit(lds_a[buf], tid);
        if constexpr (COL_OUTER)
            lb_out.commit(lds_b[buf], tid);
        else
            lb_red.commit(lds_b[buf], tid);
    };

    if (steps > 0) {
        issue(k_begin);
        commit(0);
    }
    __syncthreads();

    for (int s = 0; s < steps; ++s) {
        int buf = s & 1;
        bool more = s + 1 < steps;
        if (more) issue(k_begin + (int64_t)(s + 1) * BK);

        const uint4 *pa = lds_a[buf] + wm * 64 + li;
        const uint4 *pb = lds_b[buf] + wn * 64 + li;
#pragma unroll
        for (int slab = 0; slab < NPACK / 2; ++slab) {
            int g = slab * 2 + h;
            uint4 a0 = pa[g * LDS_ROWS], a1 = pa[g * LDS_ROWS + 32];
            uint4 b0 = pb[g * LDS_ROWS], b1 = pb[g * LDS_ROWS + 32];
            Mma<T>::run(a0, b0, acc[0][0]);
            Mma<T>::run(a0, b1, acc[0][1]);
            Mma<T>::run(a1, b0, acc[1][0]);
            Mma<T>::run(a1, b1, acc[1][1]);
        }

        if (more) commit(buf ^ 1);
        __syncthreads();
    }

    // Result layout of a 32 x 32 MFMA tile: lane holds column lane%32; register v holds row
    // 8*(v/4) + 4*(lane/32) + v%4.
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        int j = col0 + wn * 64 + u * 32 + li;
        typename Epi::Col col = epi.column(j);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int i = row0 + wm * 64 + t * 32 + 8 * (v / 4) + 4 * h + (v % 4);
                epi.store(i, col, acc[t][u][v], epi.row_add(i), z);
            }
        }
    }
}

// Sum the per-split partial results in split order (deterministic) into the final fp32 tensor.
__global__ void reduce_partials_kernel(const float *__restrict__ partials, int splits, int64_t count,
                                       float *__restrict__ out)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    float acc = 0.f;
    for (int z = 0; z < splits; ++z) acc += partials[(int64_t)z * count + i];
    out[i] = acc;
}

static GemmShape make_shape(int rows, int cols, int64_t red, int64_t chunk)
{
    GemmShape s;
    s.rows = rows;
    s.cols = cols;
    s.red = red;
    s.chunk = chunk;
    s.tiles_i = (rows + BM - 1) / BM;
    s.tiles_j = (cols + BN - 1) / BN;
    s.n_blocks = s.tiles_i * s.tiles_j;
    s.per_xcd = (s.n_blocks + 7) / 8;
    return s;
}

template <typename T>
static int run_forward(const ConvGeom &g, const GemmFwdArgs &a, hipStream_t s)
{
    constexpr int BK = NPACK * Pack<T>::KP;
    // K-hat is zero-padded along K to a multiple of the pack size; rows of D-hat beyond K read as zero.
    GemmShape sh = make_shape(g.F, (int)a.ldd, g.K, round_up(g.K, BK));
    FwdEpilogue<T> epi{(T *)a.Y, a.bias, g.F, g.M, g.HoWo, g.div_HoWo, a.relu};
    dim3 grid(sh.per_xcd * 8, 1, 1);
    ProfScope prof(KID_GEMM_FWD, s, 2.0 * g.M * (double)g.K * g.F,
                   ((double)g.F * g.K + (double)g.K * g.M + (double)g.F * g.M) * sizeof(T));
    hipLaunchKernelGGL((gemm_kernel<T, true, FwdEpilogue<T>>), grid, dim3(NTHREADS), 0, s, (const T *)a.Khat,
                       a.ldk, (const T *)a.Dhat, a.ldd, sh, epi);
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
    GemmShape sh = make_shape(g.K, (int)a.ldd, g.F, round_up(g.F, BK));
    RowMajorEpilogue<T> epi{(T *)a.dDhat, a.ldd, g.K, (int)a.ldd};
    dim3 grid(sh.per_xcd * 8, 1, 1);
    ProfScope prof(KID_GEMM_DGRAD, s, 2.0 * g.M * (double)g.K * g.F,
                   ((double)g.F * g.K + (double)g.K * g.M + (double)g.F * g.M) * sizeof(T));
    hipLaunchKernelGGL((gemm_kernel<T, true, RowMajorEpilogue<T>>), grid, dim3(NTHREADS), 0, s,
                       (const T *)a.KhatT, a.ldk, (const T *)a.dYhat, a.ldd, sh, epi);
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

int launch_gemm_dgrad(const ConvGeom &g, int dtype, const GemmDgradArgs &a, hipStream_t s)
{
    return dtype == OMNI_BF16 ? run_dgrad<bf16_t>(g, a, s) : run_dgrad<float>(g, a, s);
}

template <typename T>
static int run_wgrad(const ConvGeom &g, const GemmWgradArgs &a, hipStream_t s)
{
    GemmShape sh = make_shape(g.F, g.K, a.ldd, a.chunk);
    float *target = a.splits == 1 ? a.dW : a.partials;
    PartialEpilogue epi{target, g.F, g.K};
    dim3 grid(sh.per_xcd * 8, a.splits, 1);
    {
        ProfScope prof(KID_GEMM_WGRAD, s, 2.0 * g.M * (double)g.K * g.F,
                       ((double)g.K * g.M + (double)g.F * g.M) * sizeof(T) + 4.0 * g.F * g.K * a.splits);
        hipLaunchKernelGGL((gemm_kernel<T, false, PartialEpilogue>), grid, dim3(NTHREADS), 0, s, (const T *)a.dYhat,
                           a.ldd, (const T *)a.Dhat, a.ldd, sh, epi);
    }
    OMNI_LAUNCH_CHECK();
    if (a.splits > 1) {
        int64_t count = (int64_t)g.F * g.K;
        ProfScope prof(KID_REDUCE_PARTIALS, s, 0.0, 4.0 * count * (a.splits + 1));
        hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s,
                           a.partials, a.splits, count, a.dW);
        OMNI_LAUNCH_CHECK();
    }
    return OMNI_OK;
}

int launch_gemm_wgrad(const ConvGeom &g, int dtype, const GemmWgradArgs &a, hipStream_t s)
{
    return dtype == OMNI_BF16 ? run_wgrad<bf16_t>(g, a, s) : run_wgrad<float>(g, a, s);
}

}  // namespace omni
