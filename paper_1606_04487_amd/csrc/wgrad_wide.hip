// Model gradient of a stride-1, same-size layer with a 5-wide window (CaffeNet's conv2) with the lowered operand read
// from an LDS copy of windows of the input planes (gfx950, bf16).
//
// The product is dK-hat [F x K] = dY-hat [F x M] * D-hat^T [M x K] (Sec. II-B; App. C, "Convolution by Lowering
// and GEMM").  As in wgrad_patch.hip, output position q of an image plane and window tap (ky, kx) meet input element
// q + (ky - ph) W + (kx - pw) of the same plane, also across a row wrap, except where the window column leaves the
// row: row (c, ky, kx) of D-hat restricted to one image is plane c of X shifted by a constant, with pixel columns
// blanked.  The planes here are too large to sit in LDS whole (27 x 27: 92 groups of 8 positions), and 25 taps are
// too many accumulators for one wavefront, so
//   * a workgroup owns ONE window row ky of the gradient of 128 filters x 96 channels and walks a range of stages,
//     a stage being up to 128 consecutive positions (16 groups) of one image; the reduction is split over the chip by
//     stages, the partial sums [ky][F][C][kw] are added in a fixed order afterwards;
//   * per stage it holds the dY-hat rows of its filters for those positions (global memory straight into LDS) and
//     the window of its channels' planes that the row's taps can touch (16 + 2 groups starting at the group of
//     element q0 + (ky - ph) W - pw; through registers: the pieces are only element-aligned in memory, and what
//     lies above or below the plane, or behind its last element, is zero-filled on the way), double buffered;
//   * a wavefront (12: 2 filter halves x 6 channel groups) accumulates 64 filters x 16 channels x 5 taps = 20 tiles
//     of v_mfma_f32_16x16x32_bf16; per slab of 32 positions it reads 4 fragments of dY-hat, the two or three
//     aligned groups that cover the five taps, and per tap off the centre a mask that blanks the positions whose
//     window column lies outside the row.  A tap is a shift by a compile-time number of elements: the row's offset
//     mod 8 is a template parameter.
#include <type_traits>

#include "common.h"
#include "mma_epilogue.h"

namespace omni {
namespace wwide {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int KW = 5;          // window width
constexpr int FT = 128;        // filters per workgroup
constexpr int CQ = 6;          // channel groups of 16 per workgroup
constexpr int CT = 16 * CQ;
constexpr int NW = 2 * CQ;     // wavefronts
constexpr int NT = 64 * NW;
constexpr int S = 4;           // slabs of 32 positions per stage
constexpr int SG = 4 * S;      // groups of 8 positions per stage
constexpr int YP = SG + 2;     // row pitches in groups, 2 mod 4: free of bank conflicts for the lane map row = lane % 16,
constexpr int XG = SG + 2;     // group = lane / 16 (see wgrad_patch.hip); XG: groups of a plane a stage's taps can touch
constexpr int XP = XG;
constexpr int Y_LOADS = FT * YP / 64;  // wavefront loads (64 groups each) of a dY-hat tile
constexpr int X_ITERS = (CT * XG + NT - 1) / NT;
constexpr int Y_BUF = FT * YP, X_BUF = CT * XP;
constexpr int MAX_P8 = 128;    // groups per plane the mask table holds
static_assert(YP % 4 == 2 && XP % 4 == 2, "conflict-free pitches");
static_assert(FT * YP % 64 == 0, "the dY-hat tile is a whole number of wavefront loads");
static_assert((2 * (Y_BUF + X_BUF) + MAX_P8 * (KW - 1)) * 16 <= 160 * 1024, "two buffers and the masks fit in LDS");

struct Args {
    const bf16_t *X;      // [N][C][H][W]
    const bf16_t *dYhat;  // [F][ld], image n at columns n * P8 * 8 .., zeros in the padding
    float *partials;      // [splits][kh][F][C][KW]
    int64_t ld;
    int32_t N, C, F, kh, ph, pw, W, HW, P8;
    int32_t stages_per_image, total_stages;
    int32_t tiles_f, n_tiles, splits, n_items, per_xcd;
    FastDiv div_W;
};

template <int I, int N, typename F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

__device__ __forceinline__ f32x4 mma16(const uint4 &a, const uint4 &b, const f32x4 &c)
{
    union U { uint4 u; bf16x8 v; };
    U ua, ub;
    ua.u = a;
    ub.u = b;
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(ua.v, ub.v, c, 0, 0, 0);
}

// SK: element offset of the window row's first tap inside an aligned group, ((ky - ph) W - pw) mod 8;
// ga: the group that offset falls into, floor(((ky - ph) W - pw) / 8)
template <int SK>
__device__ __forceinline__ void wgrad_wide_body(const Args &a, uint4 *ybuf, uint4 *xbuf, const uint4 *mtab, int z, int tf, int tc,
                                                int ky, int ga)
{
    constexpr int NR = (SK + KW - 1 + 7) / 8 + 1;  // aligned groups that cover the taps of 8 positions
    static_assert(NR <= XG - SG + 1, "the window holds every group a lane reads");
    const int f0 = tf * FT, c0 = tc * CT;
    const int t_lo = (int)((int64_t)z * a.total_stages / a.splits), t_hi = (int)((int64_t)(z + 1) * a.total_stages / a.splits);
    const int slabs_per_image = a.P8 / 4;

    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int fh = wave / CQ, cq = wave % CQ;
    const int r16 = lane % 16, lg = lane / 16;

    // ---- dY-hat rows: global memory -> LDS, 16 bytes per lane, linear in (row, group) order with the row pitch YP
    // (groups beyond the stage's, or beyond the plane, repeat the plane's last group: nobody reads them).
    // Wavefront w issues loads w, w + NW, ...
    const char *ybase = reinterpret_cast<const char *>(a.dYhat + (int64_t)f0 * a.ld);
    auto issue_y = [&](int n, int g0, int buf) {
        const char *py = ybase + (int64_t)n * a.P8 * 16;
#pragma unroll
        for (int it = 0; it < (Y_LOADS + NW - 1) / NW; ++it) {
            const int w = it * NW + wave;
            if (w < Y_LOADS) {
                const int idx = w * 64 + lane;
                const int row = idx / YP;
                int grp = g0 + (idx - row * YP);
                grp = grp < a.P8 ? grp : a.P8 - 1;
                const uint32_t off = (uint32_t)row * (uint32_t)(a.ld * 2) + (uint32_t)(grp * 16);
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(py + off),
                                                 (__attribute__((address_space(3))) void *)(ybuf + buf * Y_BUF + w * 64), 16, 0, 0);
            }
        }
    };
    auto wait_loads = [&]() { __builtin_amdgcn_s_waitcnt(0x0f70); };  // vmcnt(0): this wavefront's groups are in LDS

    // ---- plane windows: global memory -> registers -> LDS.  Piece (c, j) is group g0 + ga + j of plane c: zero when
    // that group lies outside the plane, and the plane's ragged last group is read so that its 16 bytes END at the
    // plane's end and shifted down (which zero-fills it).
    u32x4 xr[X_ITERS];
    const char *xbase = reinterpret_cast<const char *>(a.X);
    const int tail = a.HW - 8 * (a.P8 - 1);  // real elements of a plane's last group
    auto issue_x = [&](int n, int g0) {
        const char *p = xbase + (uint32_t)((n * a.C + c0) * a.HW) * 2u;
#pragma unroll
        for (int k = 0; k < X_ITERS; ++k) {
            const int idx = k * NT + tid;
            const bool in_tile = idx < CT * XG;
            const int c = in_tile ? idx / XG : 0, j = in_tile ? idx - c * XG : 0;
            const int G = g0 + ga + j;
            const bool inside = G >= 0 && G < a.P8;
            const int e0 = !inside ? 0 : (G == a.P8 - 1 ? a.HW - 8 : 8 * G);
            __builtin_memcpy(&xr[k], p + (uint32_t)((c * a.HW + e0) * 2), 16);  // element-aligned 16-byte load
        }
    };
    auto commit_x = [&](int g0, int buf) {
#pragma unroll
        for (int k = 0; k < X_ITERS; ++k) {
            const int idx = k * NT + tid;
            const int c = idx / XG, j = idx - c * XG;
            const int G = g0 + ga + j;
            u32x4 v = xr[k];
            if (G == a.P8 - 1) {
                unsigned __int128 x;
                __builtin_memcpy(&x, &v, 16);
                x >>= 16 * (8 - tail);  // tail = 8: nothing moves
                __builtin_memcpy(&v, &x, 16);
            }
            if (G < 0 || G >= a.P8) v = u32x4{0, 0, 0, 0};
            if (idx < CT * XG) *reinterpret_cast<u32x4 *>(xbuf + buf * X_BUF + c * XP + j) = v;
        }
    };

    const char *ylane = reinterpret_cast<const char *>(ybuf + (fh * 64 + r16) * YP + lg);
    const char *xlane = reinterpret_cast<const char *>(xbuf + (cq * 16 + r16) * XP + lg);
    const char *mlane = reinterpret_cast<const char *>(mtab + lg * (KW - 1));

    f32x4 acc[4][KW];
#pragma unroll
    for (int fi = 0; fi < 4; ++fi)
#pragma unroll
        for (int t = 0; t < KW; ++t) acc[fi][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // One slab: yp, xp, mp point at this lane's group in its dY-hat row, its plane window and the mask table.
    auto slab = [&](const char *yp, const char *xp, const char *mp) {
        uint4 A[4], R[NR];
#pragma unroll
        for (int fi = 0; fi < 4; ++fi) A[fi] = *reinterpret_cast<const uint4 *>(yp + fi * (16 * YP * 16));
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            // whole 16-byte reads, not the single words a tap uses (those would put four lanes on every bank)
            R[j] = *reinterpret_cast<const uint4 *>(xp + j * 16);
            asm volatile("" : "+v"(R[j].x), "+v"(R[j].y), "+v"(R[j].z), "+v"(R[j].w));
        }
        static_for<0, KW>([&](auto tt) {
            constexpr int kx = decltype(tt)::value;
            constexpr int o = SK + kx, rb = o / 8, s = o % 8;
            static_assert(rb + (s ? 1 : 0) < NR, "the groups read cover every tap");
            uint32_t D[8] = {R[rb].x, R[rb].y, R[rb].z, R[rb].w, 0, 0, 0, 0};
            if constexpr (s != 0) D[4] = R[rb + 1].x, D[5] = R[rb + 1].y, D[6] = R[rb + 1].z, D[7] = R[rb + 1].w;
            uint4 b;
            if constexpr (s % 2 == 0) {
                b = make_uint4(D[s / 2], D[s / 2 + 1], D[s / 2 + 2], D[s / 2 + 3]);
            } else {
                constexpr int q = (s - 1) / 2;
                b = make_uint4(__builtin_amdgcn_alignbit(D[q + 1], D[q], 16), __builtin_amdgcn_alignbit(D[q + 2], D[q + 1], 16),
                               __builtin_amdgcn_alignbit(D[q + 3], D[q + 2], 16), __builtin_amdgcn_alignbit(D[q + 4], D[q + 3], 16));
            }
            if constexpr (kx != KW / 2) {
                constexpr int mi = kx < KW / 2 ? kx : kx - 1;  // masks of the window columns off the centre
                const uint4 m = *reinterpret_cast<const uint4 *>(mp + mi * 16);
                b = make_uint4(b.x & m.x, b.y & m.y, b.z & m.z, b.w & m.w);
            }
#pragma unroll
            for (int fi = 0; fi < 4; ++fi) acc[fi][kx] = mma16(A[fi], b, acc[fi][kx]);
        });
    };

    auto stage_of = [&](int t, int &n, int &g0, int &nsl) {
        n = t / a.stages_per_image;
        const int st = t - n * a.stages_per_image;
        g0 = st * SG;
        nsl = slabs_per_image - st * S < S ? slabs_per_image - st * S : S;
    };

    int n, g0, nsl;
    stage_of(t_lo, n, g0, nsl);
    issue_y(n, g0, 0);
    issue_x(n, g0);
    commit_x(g0, 0);
    wait_loads();
    __syncthreads();
    for (int t = t_lo; t < t_hi; ++t) {
        const int buf = (t - t_lo) & 1;
        const bool more = t + 1 < t_hi;
        int n1 = 0, g1 = 0, nsl1 = 0;
        if (more) {
            stage_of(t + 1, n1, g1, nsl1);
            issue_y(n1, g1, buf ^ 1);  // that buffer was left by every wavefront before the last barrier
            issue_x(n1, g1);
        }
        const char *yp = ylane + buf * (Y_BUF * 16), *xp = xlane + buf * (X_BUF * 16), *mp = mlane + g0 * ((KW - 1) * 16);
#pragma unroll 1
        for (int sl = 0; sl < nsl; ++sl) slab(yp + sl * 64, xp + sl * 64, mp + sl * (4 * (KW - 1) * 16));
        if (more) commit_x(g1, buf ^ 1);
        wait_loads();
        __syncthreads();
        g0 = g1, nsl = nsl1;
    }

    // ---- epilogue: a wavefront's 16 filters x (16 channels x KW taps) are 16 runs of 16 KW consecutive floats of the
    // partial result [ky][F][C][KW]; they pass through an LDS strip so that the stores are whole 16-byte pieces.
    // Result layout of a 16 x 16 tile: lane holds column (channel) lane % 16, register r row (filter) 4 (lane / 16) + r.
    constexpr int RUN = 16 * KW, SP = RUN + 4;  // floats per run, strip pitch
    static_assert(RUN % 4 == 0, "runs are whole 16-byte pieces");
    static_assert(NW * 16 * SP * 4 <= 2 * Y_BUF * 16, "staging strips fit in ybuf");
    float *strip = reinterpret_cast<float *>(ybuf) + wave * (16 * SP);
    float *out = a.partials + ((((int64_t)z * a.kh + ky) * a.F + f0 + fh * 64) * a.C + c0 + cq * 16) * KW;
#pragma unroll
    for (int fi = 0; fi < 4; ++fi) {
#pragma unroll
        for (int t = 0; t < KW; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) strip[(4 * lg + r) * SP + r16 * KW + t] = acc[fi][t][r];
        __builtin_amdgcn_wave_barrier();
        constexpr int Q4 = RUN / 4;
#pragma unroll
        for (int p = 0; p < (16 * Q4 + 63) / 64; ++p) {
            const int idx = p * 64 + lane;
            if (idx < 16 * Q4) {
                const int row = idx / Q4, q4 = idx - row * Q4;
                const f32x4 v = *reinterpret_cast<const f32x4 *>(strip + row * SP + 4 * q4);
                *reinterpret_cast<f32x4 *>(out + (int64_t)(fi * 16 + row) * a.C * KW + 4 * q4) = v;
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

__global__ __launch_bounds__(NT) void wgrad_wide_kernel(Args a)
{
    __shared__ uint4 ybuf[2 * Y_BUF];
    __shared__ uint4 xbuf[2 * X_BUF];
    __shared__ uint4 mtab[MAX_P8 * (KW - 1)];
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int item = xcd * a.per_xcd + slot;  // contiguous ranges of items per XCD: the tiles of a split share stages
    if (item >= a.n_items) return;
    const int z = item / a.n_tiles, tile = item - z * a.n_tiles;
    const int tck = tile / a.tiles_f, tf = tile - tck * a.tiles_f;
    const int tc = tck / a.kh, ky = tck - tc * a.kh;
    // mask (g, kx off the centre): the positions 8g .. 8g + 7 whose window column ox + kx - pw lies inside the row
    for (int i = threadIdx.x; i < a.P8 * (KW - 1); i += NT) {
        const int g = i / (KW - 1), mi = i - g * (KW - 1), kx = mi < KW / 2 ? mi : mi + 1;
        uint32_t m[4] = {0, 0, 0, 0};
        for (int e = 0; e < 8; ++e) {
            uint32_t oy, ox;
            a.div_W.divmod((uint32_t)(8 * g + e), oy, ox);
            const int x = (int)ox + kx - a.pw;
            if (x >= 0 && x < a.W) m[e / 2] |= 0xffffu << (16 * (e % 2));
        }
        mtab[i] = make_uint4(m[0], m[1], m[2], m[3]);
    }
    __syncthreads();
    const int o0 = (ky - a.ph) * a.W - a.pw;                      // element offset of the row's first tap
    const int ga = o0 >= 0 ? o0 / 8 : -((-o0 + 7) / 8), sk = o0 - 8 * ga;  // uniform over the workgroup
    switch (sk) {
    case 0: wgrad_wide_body<0>(a, ybuf, xbuf, mtab, z, tf, tc, ky, ga); break;
    case 1: wgrad_wide_body<1>(a, ybuf, xbuf, mtab, z, tf, tc, ky, ga); break;
    case 2: wgrad_wide_body<2>(a, ybuf, xbuf, mtab, z, tf, tc, ky, ga); break;
    case 3: wgrad_wide_body<3>(a, ybuf, xbuf, mtab, z, tf, tc, ky, ga); break;
    case 4: wgrad_wide_body<4>(a, ybuf, xbuf, mtab, z, tf, tc, ky, ga); break;
    case 5: wgrad_wide_body<5>(a, ybuf, xbuf, mtab, z, tf, tc, ky, ga); break;
    case 6: wgrad_wide_body<6>(a, ybuf, xbuf, mtab, z, tf, tc, ky, ga); break;
    default: wgrad_wide_body<7>(a, ybuf, xbuf, mtab, z, tf, tc, ky, ga); break;
    }
}

// Ordered sum of the partial results [splits][kh][F][C][kw] into dW [F][C][kh][kw]: one thread per element, the
// splits added in order (four chains by split index mod 4, then (s0 + s1) + (s2 + s3)).  Extra workgroups
// (blockIdx >= main_blocks) finish the bias gradient from the per-block sums of the dY packing kernel, one
// wavefront per filter.
__global__ __launch_bounds__(256) void reduce_wide_kernel(const float *__restrict__ partials, int splits, int F, int C, int kh,
                                                          int kw, float *__restrict__ dW, unsigned main_blocks,
                                                          const float *__restrict__ bias_partials, int bias_blocks,
                                                          float *__restrict__ dbias)
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
    // thread -> element of the partial layout (a wavefront's reads are consecutive), written to its place in dW
    const int64_t count = (int64_t)F * C * kh * kw, i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    const int kx = (int)(i % kw);
    int64_t r = i / kw;
    const int c = (int)(r % C);
    r /= C;
    const int f = (int)(r % F), ky = (int)(r / F);
    const float *p = partials + i;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int zz = 0;
    for (; zz + 3 < splits; zz += 4) {
        s0 += p[(int64_t)zz * count], s1 += p[(int64_t)(zz + 1) * count];
        s2 += p[(int64_t)(zz + 2) * count], s3 += p[(int64_t)(zz + 3) * count];
    }
    if (zz < splits) s0 += p[(int64_t)zz * count];
    if (zz + 1 < splits) s1 += p[(int64_t)(zz + 1) * count];
    if (zz + 2 < splits) s2 += p[(int64_t)(zz + 2) * count];
    dW[(((int64_t)f * C + c) * kh + ky) * kw + kx] = (s0 + s1) + (s2 + s3);
}

static int g_off = 0, g_max_splits = 0;  // omni_tuning_set(OMNI_TUNE_WGRAD_*): sweeps and tests only

static int groups_per_plane(const ConvGeom &g) { return (g.H * g.W + 7) / 8; }
static int stages_per_image(const ConvGeom &g) { return (groups_per_plane(g) / 4 + S - 1) / S; }

}  // namespace wwide

void set_wgrad_wide_override(int max_splits, int off)
{
    if (max_splits >= 0) wwide::g_max_splits = max_splits;
    if (off >= 0) wwide::g_off = off;
}

bool wgrad_wide_supported(const ConvGeom &g, int dtype)
{
    using namespace wwide;
    if (g_off) return false;
    if (dtype != OMNI_BF16 || g.kw != KW || g.kh > 9 || g.sh != 1 || g.sw != 1) return false;
    if (2 * g.ph != g.kh - 1 || 2 * g.pw != g.kw - 1) return false;  // same-size output
    if (g.C % CT != 0 || g.F % FT != 0 || g.H * g.W < 8 || g.W < KW) return false;
    const int P8 = groups_per_plane(g);
    if (P8 % 4 != 0 || P8 > MAX_P8) return false;  // whole slabs of 32 positions; the mask table
    if (!wgrad_direct_planes(g)) return false;     // the dY-hat layout this kernel reads
    const double ld = (double)dyhat_rows_ld(g);
    return (double)g.N * g.C * g.H * g.W * 2.0 < 4.0e9 && FT * ld * 2.0 < 4.0e9;
}

// Splits of the reduction (ranges of stages): one round of workgroups on the 256 compute units.
int wgrad_wide_splits(const ConvGeom &g)
{
    using namespace wwide;
    const int64_t n_tiles = (int64_t)(g.F / FT) * (g.C / CT) * g.kh;
    const int64_t total = (int64_t)g.N * stages_per_image(g);
    int64_t splits = 256 / n_tiles;
    if (splits < 1) splits = 1;
    if (g_max_splits > 0 && splits > g_max_splits) splits = g_max_splits;
    return (int)(splits < total ? splits : total);
}

// dYhat in the plane-padded layout of launch_pack_dyhat_rows (leading dimension ld); partials: splits * F * K floats
int launch_wgrad_wide(const ConvGeom &g, const void *X, const void *dYhat, int64_t ld, float *partials, int splits, float *dW,
                      const float *bias_partials, int bias_blocks, float *dbias, hipStream_t s)
{
    using namespace wwide;
    Args a;
    a.X = (const bf16_t *)X, a.dYhat = (const bf16_t *)dYhat, a.partials = partials, a.ld = ld;
    a.N = g.N, a.C = g.C, a.F = g.F, a.kh = g.kh, a.ph = g.ph, a.pw = g.pw, a.W = g.W, a.HW = g.H * g.W;
    a.P8 = groups_per_plane(g);
    a.stages_per_image = stages_per_image(g);
    a.total_stages = g.N * a.stages_per_image;
    a.tiles_f = g.F / FT;
    a.n_tiles = a.tiles_f * g.kh * (g.C / CT);
    a.splits = splits;
    a.n_items = a.n_tiles * splits;
    a.per_xcd = (a.n_items + 7) / 8;
    a.div_W = FastDiv((uint32_t)g.W);
    {
        ProfScope prof(KID_GEMM_WGRAD, s, 2.0 * g.M * (double)g.K * g.F,
                       ((double)g.N * g.C * g.H * g.W + (double)g.F * g.M) * 2.0 + 4.0 * g.F * (double)g.K * splits);
        hipLaunchKernelGGL(wgrad_wide_kernel, dim3((unsigned)a.per_xcd * 8), dim3(NT), 0, s, a);
        OMNI_LAUNCH_CHECK();
    }
    const int64_t count = (int64_t)g.F * g.K;
    ProfScope prof(KID_REDUCE_PARTIALS, s, 0.0, 4.0 * count * (splits + 1));
    const unsigned main_blocks = (unsigned)((count + 255) / 256);
    const unsigned bias_wgs = dbias != nullptr ? (unsigned)((g.F + 3) / 4) : 0u;
    hipLaunchKernelGGL(reduce_wide_kernel, dim3(main_blocks + bias_wgs), dim3(256), 0, s, partials, splits, g.F, g.C, g.kh, g.kw, dW,
                       main_blocks, bias_partials, bias_blocks, dbias);
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

}  // namespace omni
