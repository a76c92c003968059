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

#include "common.h"

namespace omni {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

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
    static constexpr int PER_THREAD = TILE_ROWS * NPACK / NT;
    static_assert(TILE_ROWS * NPACK % NT == 0, "tile must divide over the threads");
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
            if (row0 + r < rows && k < red)
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
            lds[g * (TILE_ROWS + 1) + r] = regs[q];
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

// Tile configuration: BM x BN result tile, WM x WN wavefronts, PF reduction steps of global loads in
// flight (register staging sets).
template <int BM_, int BN_, int WM_, int WN_, int PF_> struct Tile {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, PF = PF_;
    static constexpr int NT = 64 * WM * WN;
    static constexpr int TI = BM / WM / 32, TJ = BN / WN / 32;  // 32 x 32 MFMA tiles per wavefront
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "wavefront tiles are multiples of 32");
};

template <typename T, typename Cfg, bool COL_OUTER, typename Epi>
__global__ __launch_bounds__(Cfg::NT) void gemm_kernel(const T *__restrict__ A, int64_t lda,
                                                       const T *__restrict__ B, int64_t ldb,
                                                       GemmShape sh, Epi epi)
{
    constexpr int KP = Pack<T>::KP;
    constexpr int BK = NPACK * KP;
    constexpr int BM = Cfg::BM, BN = Cfg::BN, NT = Cfg::NT, TI = Cfg::TI, TJ = Cfg::TJ, PF = Cfg::PF;
    constexpr int LA = BM + 1, LB = BN + 1;
    __shared__ uint4 lds_a[2][NPACK * LA];
    __shared__ uint4 lds_b[2][NPACK * LB];

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
    int wm = wave / Cfg::WN, wn = wave % Cfg::WN;
    int li = lane % 32, h = lane / 32;

    f32x16 acc[TI][TJ];
#pragma unroll
    for (int t = 0; t < TI; ++t)
#pragma unroll
        for (int u = 0; u < TJ; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][u][v] = 0.f;

    RedContigLoader<T, BM, NT> la[PF];
    RedContigLoader<T, BN, NT> lb_red[PF];
    OuterContigLoader<T, BN, NT> lb_out[PF];

    auto issue = [&](int set, int64_t k0) {
        la[set].issue(A, lda, sh.rows, sh.red, row0, k0, tid);
        if constexpr (COL_OUTER)
            lb_out[set].issue(B, ldb, sh.red, sh.cols, k0, col0, tid);
        else
            lb_red[set].issue(B, ldb, sh.cols, sh.red, col0, k0, tid);
    };
    auto commit = [&](int set, int buf) {
        la[set].commit(lds_a[buf], tid);
        if constexpr (COL_OUTER)
            lb_out[set].commit(lds_b[buf], tid);
        else
            lb_red[set].commit(lds_b[buf], tid);
    };
    auto compute = [&](int buf) {
        const uint4 *pa = lds_a[buf] + wm * (BM / Cfg::WM) + li;
        const uint4 *pb = lds_b[buf] + wn * (BN / Cfg::WN) + li;
#pragma unroll
        for (int slab = 0; slab < NPACK / 2; ++slab) {
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
    // of step s into register set s%PF; the set holding tile s+1 is written to the other LDS buffer at
    // the end of step s.  The loop is unrolled by PF so that set indices are compile-time constants.
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
                compute(s & 1);
                if (s + 1 < steps) commit((p + 1) % PF, (s + 1) & 1);
                __syncthreads();
            }
        }
    }

    // Result layout of a 32 x 32 MFMA tile: lane holds column lane%32; register v holds row
    // 8*(v/4) + 4*(lane/32) + v%4.
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

static GemmShape make_shape(int rows, int cols, int64_t red, int64_t chunk, int bm, int bn)
{
    GemmShape s;
    s.rows = rows;
    s.cols = cols;
    s.red = red;
    s.chunk = chunk;
    s.tiles_i = (rows + bm - 1) / bm;
    s.tiles_j = (cols + bn - 1) / bn;
    s.n_blocks = s.tiles_i * s.tiles_j;
    s.per_xcd = (s.n_blocks + 7) / 8;
    return s;
}

// Tile configurations compiled in.  Index = OMNI_GEMM_TILE environment override (for tuning runs) or
// the choice of pick_tile().
typedef Tile<128, 128, 2, 2, 1> Tile0;
typedef Tile<128, 128, 2, 2, 2> Tile1;
typedef Tile<256, 128, 2, 2, 1> Tile2;
typedef Tile<256, 128, 2, 2, 2> Tile3;
typedef Tile<128, 256, 2, 2, 1> Tile4;
typedef Tile<256, 256, 2, 2, 1> Tile5;
typedef Tile<256, 256, 4, 2, 1> Tile6;
typedef Tile<256, 256, 2, 4, 1> Tile7;
constexpr int N_TILES = 8;

static int tile_override()
{
    const char *e = getenv("OMNI_GEMM_TILE");
    int v = e ? atoi(e) : -1;
    return (v >= 0 && v < N_TILES) ? v : -1;
}

static int pick_tile(int rows, int cols)
{
    int o = tile_override();
    if (o >= 0) return o;
    (void)rows;
    (void)cols;
    return 0;
}

template <typename T, typename Cfg, bool COL_OUTER, typename Epi>
static void launch_cfg(const T *A, int64_t lda, const T *B, int64_t ldb, int rows, int cols, int64_t red,
                       int64_t chunk, int splits, const Epi &epi, hipStream_t s)
{
    GemmShape sh = make_shape(rows, cols, red, chunk, Cfg::BM, Cfg::BN);
    dim3 grid(sh.per_xcd * 8, splits, 1);
    hipLaunchKernelGGL((gemm_kernel<T, Cfg, COL_OUTER, Epi>), grid, dim3(Cfg::NT), 0, s, A, lda, B, ldb, sh, epi);
}

template <typename T, bool COL_OUTER, typename Epi>
static void launch_any(int tile, const T *A, int64_t lda, const T *B, int64_t ldb, int rows, int cols, int64_t red,
                       int64_t chunk, int splits, const Epi &epi, hipStream_t s)
{
    switch (tile) {
    case 1: launch_cfg<T, Tile1, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    case 2: launch_cfg<T, Tile2, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    case 3: launch_cfg<T, Tile3, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    case 4: launch_cfg<T, Tile4, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    case 5: launch_cfg<T, Tile5, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    case 6: launch_cfg<T, Tile6, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    case 7: launch_cfg<T, Tile7, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    default: launch_cfg<T, Tile0, COL_OUTER, Epi>(A, lda, B, ldb, rows, cols, red, chunk, splits, epi, s); break;
    }
}

template <typename T>
static int run_forward(const ConvGeom &g, const GemmFwdArgs &a, hipStream_t s)
{
    constexpr int BK = NPACK * Pack<T>::KP;
    // K-hat is zero-padded along K to a multiple of the pack size; rows of D-hat beyond K read as zero.
    FwdEpilogue<T> epi{(T *)a.Y, a.bias, g.F, g.M, g.HoWo, g.div_HoWo, a.relu};
    ProfScope prof(KID_GEMM_FWD, s, 2.0 * g.M * (double)g.K * g.F,
                   ((double)g.F * g.K + (double)g.K * g.M + (double)g.F * g.M) * sizeof(T));
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
    launch_any<T, true, RowMajorEpilogue<T>>(pick_tile(g.K, (int)a.ldd), (const T *)a.KhatT, a.ldk, (const T *)a.dYhat,
                                             a.ldd, g.K, (int)a.ldd, g.F, round_up(g.F, BK), 1, epi, s);
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
    float *target = a.splits == 1 ? a.dW : a.partials;
    PartialEpilogue epi{target, g.F, g.K};
    {
        ProfScope prof(KID_GEMM_WGRAD, s, 2.0 * g.M * (double)g.K * g.F,
                       ((double)g.K * g.M + (double)g.F * g.M) * sizeof(T) + 4.0 * g.F * g.K * a.splits);
        launch_any<T, false, PartialEpilogue>(pick_tile(g.F, g.K), (const T *)a.dYhat, a.ldd, (const T *)a.Dhat, a.ldd,
                                              g.F, g.K, a.ldd, a.chunk, a.splits, epi, s);
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
