// Model gradient of a 3 x 3, stride-1, same-size layer on small image planes with the lowered operand read
// from an LDS copy of the input planes (gfx950, bf16).
//
// The product is dK-hat [F x K] = dY-hat [F x M] * D-hat^T [M x K] (Sec. II-B; App. C, "Convolution by Lowering
// and GEMM"), reduced over the columns m = (n, oy, ox) of the lowered matrix.  Where the output is as wide and
// as high as the input, output position q of an image plane and window tap (ky, kx) meet input element
// q + (ky - 1) W + (kx - 1) of the same plane, also across a row wrap, except where the window column leaves the
// row (then the entry of D-hat is a zero of the padding).  So row (c, ky, kx) of D-hat, restricted to one image, is
// plane c of X shifted by a constant and with one pixel column blanked: nothing of D-hat has to exist anywhere.
//
// A workgroup owns the gradient of 128 filters x 64 channels x all 9 taps and walks a range of images (the
// reduction is split over the chip by images; the partial sums are added in a fixed order afterwards).  Per
// image it holds in LDS
//   ybuf: dY-hat rows of its 128 filters, the plane padded to whole 16-byte groups of 8 positions (P8 groups),
//   xbuf: the planes of its 64 channels in the same padding, between two zeroed margins of W + 1 elements that
//         stand for the rows above and below the image,
// both double buffered: the next image's dY-hat rows go from global memory straight into LDS, its planes
// through registers (their 16-byte pieces are only element-aligned in memory and the ragged last piece of a
// plane is zero-filled on the way).  A wavefront (8 per workgroup: 2 filter halves x 4 channel quarters)
// accumulates 64 filters x 16 channels x 9 taps = 36 MFMA tiles of 16 x 16 (v_mfma_f32_16x16x32_bf16: a lane
// holds 8 consecutive reduction indices = one group of 8 positions; the four lane groups of an instruction take
// four consecutive groups).  Per slab of 32 positions it reads 4 fragments of dY-hat, the 5 aligned groups of
// its channel's plane around its positions and two masks, and derives all 9 taps' operands from those five
// reads in registers: a tap is a shift by a compile-time number of elements (register picks for even shifts, one
// funnel shift per word for odd ones) and, for the outer window columns, an AND with the mask that blanks the
// positions whose window column lies outside the row.  9 x 4 MFMAs follow from 11 LDS reads.
//
// P8 is 22 for 13 x 13 planes: 5.5 slabs.  Two consecutive images are therefore walked as 11 slabs: five of the
// first image, one that takes the first image's last two groups and the second image's first two (the lane
// groups read different buffers), five of the second image.
#include <type_traits>

#include "common.h"
#include "mma_epilogue.h"

namespace omni {
namespace wpatch {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int FT = 128;  // filters per workgroup
constexpr int CT = 64;   // channels per workgroup
constexpr int NT = 512;  // 8 wavefronts
constexpr int KH = 3, KW = 3, TAPS = KH * KW;

constexpr int floor_div(int a, int b) { return a >= 0 ? a / b : -((-a + b - 1) / b); }

template <int H_, int W_> struct Plane {
    static constexpr int H = H_, W = W_, HW = H * W;
    static constexpr int P8 = (HW + 7) / 8;          // 16-byte groups per plane
    static constexpr int TAIL = HW - 8 * (P8 - 1);   // real elements of a plane's last group
    static constexpr int MG = 2;                     // zero groups on either side of a plane in xbuf
    // Row pitches in groups.  A lane of a fragment read takes row lane % 16 at group lane / 16, and the LDS serves
    // the 64 lanes of a 16-byte read in four passes of 16 (lanes 0-3, 12-15, 20-27 | 4-11, 16-19, 28-31 | the same of
    // the upper half), a pass being free of bank conflicts when its 16-byte slots differ mod 16.  With slot =
    // pitch * row + group that holds exactly for pitch = 2, 6, 10 or 14 mod 16 (an odd pitch, which spreads any 16
    // CONSECUTIVE lanes over all slots, puts two lanes on half of the slots of every pass: measured twice the cycles).
    static constexpr int conflict_free_pitch(int n) { return n % 4 == 2 ? n : n + (6 - n % 4) % 4; }
    static constexpr int XP = conflict_free_pitch(P8 + 2 * MG);
    static constexpr int YP = conflict_free_pitch(P8);
    static_assert(XP % 4 == 2 && YP % 4 == 2 && XP >= P8 + 2 * MG && YP >= P8, "pitches");
    static constexpr int Y_ITERS = (FT * YP + NT - 1) / NT;
    static constexpr int Y_BUF = Y_ITERS * NT;       // groups per ybuf buffer (every thread writes one per iteration)
    static constexpr int X_PIECES = CT * P8;
    static constexpr int X_ITERS = (X_PIECES + NT - 1) / NT;
    static constexpr int X_BUF = CT * XP;
    static constexpr int SLABS = P8 / 4;             // whole slabs of an image
    static_assert(W + 1 <= 8 * MG && W >= 8, "a tap's shift stays within two groups on either side");
    static_assert(P8 % 4 == 2, "an image is SLABS slabs and half a slab");
    static_assert(HW >= 8, "the ragged last piece is read backwards from the plane's end");
};

struct Args {
    const bf16_t *X;       // [N][C][H][W]
    const bf16_t *dYhat;   // [F][ld], image n at columns n * P8 * 8 .. , zeros in the padding
    float *partials;       // [splits][F][K]
    int64_t ld;
    int32_t N, C, F, K;
    int32_t tiles_f, n_tiles, splits, n_items, per_xcd;
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

template <typename PL> __global__ __launch_bounds__(NT) void wgrad_patch_kernel(Args a)
{
    constexpr int P8 = PL::P8, XP = PL::XP, YP = PL::YP, MG = PL::MG, W = PL::W, HW = PL::HW;
    __shared__ uint4 ybuf[2][PL::Y_BUF];
    __shared__ uint4 xbuf[2][PL::X_BUF];
    __shared__ uint4 mtab[P8][2];

    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int item = xcd * a.per_xcd + slot;  // contiguous ranges of items per XCD: the tiles of a split share images
    if (item >= a.n_items) return;
    const int z = item / a.n_tiles, tile = item - z * a.n_tiles;
    const int tc = tile / a.tiles_f, tf = tile - tc * a.tiles_f;
    const int f0 = tf * FT, c0 = tc * CT;
    const int n_lo = (int)((int64_t)z * a.N / a.splits), n_hi = (int)((int64_t)(z + 1) * a.N / a.splits);

    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int fh = wave / 4, cq = wave % 4;
    const int r16 = lane % 16, lg = lane / 16;

    // ---- dY-hat rows: global memory -> LDS, 16 bytes per lane and iteration, linear in (row, group) order with
    // the row pitch YP (the padding group of a row repeats the row's last group; rows beyond the tile repeat
    // the last row: they land in the slack at the buffer's end).
    // The offsets are recomputed at every use instead of kept: registers are what this kernel is short of.
    const char *ybase = reinterpret_cast<const char *>(a.dYhat + (int64_t)f0 * a.ld);
    auto issue_y = [&](int n, int buf) {
        const char *p = ybase + (int64_t)n * (P8 * 16);
#pragma unroll
        for (int it = 0; it < PL::Y_ITERS; ++it) {
            int idx = it * NT + tid;
            int row = idx / YP, pc = idx - row * YP;
            row = row < FT ? row : FT - 1;
            pc = pc < P8 ? pc : P8 - 1;
            const uint32_t off = (uint32_t)row * (uint32_t)(a.ld * 2) + (uint32_t)(pc * 16);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p + off),
                                             (__attribute__((address_space(3))) void *)(&ybuf[buf][it * NT + wave * 64]), 16, 0, 0);
        }
    };
    auto wait_y = [&]() { __builtin_amdgcn_s_waitcnt(0x0f70); };  // vmcnt(0): this wavefront's groups are in LDS

    // ---- planes: global memory -> registers -> LDS; piece j of channel c holds plane elements 8j .. 8j + 7
    u32x4 xr[PL::X_ITERS];
    const char *xbase = reinterpret_cast<const char *>(a.X);
    auto issue_x = [&](int n) {
        const char *p = xbase + (uint32_t)((n * a.C + c0) * HW) * 2u;
#pragma unroll
        for (int k = 0; k < PL::X_ITERS; ++k) {
            const int idx = k * NT + tid;
            const bool valid = idx < PL::X_PIECES;
            const int c = valid ? idx / P8 : 0, j = valid ? idx - c * P8 : 0;
            // the ragged last piece is read so that its 16 bytes END at the plane's end, and shifted down in commit_x
            const bool tail = PL::TAIL < 8 && j == P8 - 1;
            __builtin_memcpy(&xr[k], p + (uint32_t)((c * HW + (tail ? HW - 8 : 8 * j)) * 2), 16);  // element-aligned 16-byte load
        }
    };
    auto commit_x = [&](int buf) {
#pragma unroll
        for (int k = 0; k < PL::X_ITERS; ++k) {
            const int idx = k * NT + tid;
            const int c = idx / P8, j = idx - c * P8;
            u32x4 v = xr[k];
            if (PL::TAIL < 8 && j == P8 - 1) {
                unsigned __int128 x;
                __builtin_memcpy(&x, &v, 16);
                x >>= 16 * (8 - PL::TAIL);
                __builtin_memcpy(&v, &x, 16);
            }
            if (idx < PL::X_PIECES) *reinterpret_cast<u32x4 *>(&xbuf[buf][c * XP + MG + j]) = v;
        }
    };

    // ---- this lane's rows
    const char *ylane = reinterpret_cast<const char *>(&ybuf[0][(fh * 64 + r16) * YP]);
    const char *xlane = reinterpret_cast<const char *>(&xbuf[0][(cq * 16 + r16) * XP + MG - 2]);
    constexpr int YB = PL::Y_BUF * 16, XB = PL::X_BUF * 16;  // bytes from buffer 0 to buffer 1
    const char *mlane = reinterpret_cast<const char *>(&mtab[0][0]);

    f32x4 acc[4][TAPS];
#pragma unroll
    for (int fi = 0; fi < 4; ++fi)
#pragma unroll
        for (int t = 0; t < TAPS; ++t) acc[fi][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // One slab: yp, xp, mp point at this lane's group in its dY-hat row, plane row and the mask table.
    auto slab = [&](const char *yp, const char *xp, const char *mp) {
        uint4 A[4], R[5], M0, M2;
#pragma unroll
        for (int fi = 0; fi < 4; ++fi) A[fi] = *reinterpret_cast<const uint4 *>(yp + fi * (16 * YP * 16));
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            // whole 16-byte reads (one bank group per lane, 16 lanes at a time): read as single words the compiler
            // fetches only the words a tap uses, and the row pitch then puts four lanes on every bank
            R[j] = *reinterpret_cast<const uint4 *>(xp + j * 16);
            asm volatile("" : "+v"(R[j].x), "+v"(R[j].y), "+v"(R[j].z), "+v"(R[j].w));
        }
        M0 = *reinterpret_cast<const uint4 *>(mp);
        M2 = *reinterpret_cast<const uint4 *>(mp + 16);
        static_for<0, TAPS>([&](auto tt) {
            constexpr int T = decltype(tt)::value, ky = T / KW, kx = T % KW;
            constexpr int o = (ky - 1) * W + (kx - 1);       // element shift of the tap
            constexpr int ga = floor_div(o, 8), s = o - 8 * ga, rb = ga + 2;
            static_assert(rb >= 0 && rb + (s ? 1 : 0) <= 4, "five groups cover every tap");
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
            if constexpr (kx == 0) b = make_uint4(b.x & M0.x, b.y & M0.y, b.z & M0.z, b.w & M0.w);
            if constexpr (kx == KW - 1) b = make_uint4(b.x & M2.x, b.y & M2.y, b.z & M2.z, b.w & M2.w);
#pragma unroll
            for (int fi = 0; fi < 4; ++fi) acc[fi][T] = mma16(A[fi], b, acc[fi][T]);
        });
    };

    // ---- prologue: first image requested, margins cleared, mask table built under the loads' latency
    issue_y(n_lo, 0);
    issue_x(n_lo);
    for (int i = tid; i < 2 * PL::X_BUF; i += NT) (&xbuf[0][0])[i] = make_uint4(0, 0, 0, 0);
    for (int i = tid; i < P8 * 2; i += NT) {
        // side 0: the tap's column is ox - 1 (blank where ox == 0); side 1: ox + 1 (blank where ox == W - 1)
        const int g = i / 2, side = i % 2;
        uint32_t m[4] = {0, 0, 0, 0};
        for (int e = 0; e < 8; ++e) {
            const int ox = (8 * g + e) % W;
            const bool blank = side == 0 ? ox == 0 : ox == W - 1;
            if (!blank) m[e / 2] |= 0xffffu << (16 * (e % 2));
        }
        mtab[g][side] = make_uint4(m[0], m[1], m[2], m[3]);
    }
    __syncthreads();
    commit_x(0);
    wait_y();
    __syncthreads();

    // A pair of images (buffers 0 and 1) is P8 / 2 slabs: lane group lg of slab `step` takes group 4 step + lg of
    // the pair, i.e. the middle slab takes the first image's last two groups and the second image's first two.
    constexpr int PAIR_SLABS = P8 / 2, MID = PL::SLABS;
    for (int n = n_lo; n < n_hi; n += 2) {
        const bool has_b = n + 1 < n_hi, has_next = n + 2 < n_hi;
        if (has_b) {
            issue_y(n + 1, 1);
            issue_x(n + 1);
        } else {
            // no second image: the middle slab's upper lane groups must add nothing -- their dY-hat groups are
            // cleared (and what they read of xbuf, so that no stale bit pattern meets those zeros)
            for (int i = tid; i < FT * 2; i += NT) ybuf[1][(i / 2) * YP + i % 2] = make_uint4(0, 0, 0, 0);
            for (int i = tid; i < PL::X_BUF; i += NT) xbuf[1][i] = make_uint4(0, 0, 0, 0);
        }
        const int steps = has_b ? PAIR_SLABS : MID + 1;
#pragma unroll 1
        for (int step = 0; step < steps; ++step) {
            if (step == MID) {
                if (has_b) commit_x(1);
                wait_y();
                __syncthreads();  // the second image is in LDS
            }
            if (step == MID + 1) {
                __syncthreads();  // buffer 0 is free
                if (has_next) {
                    issue_y(n + 2, 0);
                    issue_x(n + 2);
                }
            }
            const int G = 4 * step + lg, second = G >= P8 ? 1 : 0, g = G - second * P8;
            slab(ylane + second * YB + g * 16, xlane + second * XB + g * 16, mlane + g * 32);
        }
        if (has_b) {
            if (has_next) commit_x(0);
            wait_y();
            __syncthreads();
        }
    }
    __syncthreads();  // every wavefront is done with the buffers: ybuf becomes staging space

    // ---- epilogue: a wavefront's 16 filters x (16 channels x 9 taps) are 16 runs of 144 consecutive floats of the
    // gradient; they pass through an LDS strip so that the stores are whole 16-byte pieces of those runs.
    // Result layout of a 16 x 16 tile: lane holds column (channel) lane % 16, register r row (filter) 4 (lane / 16) + r.
    constexpr int SP = 16 * TAPS + 4;  // strip pitch in floats
    static_assert(8 * 16 * SP * 4 <= (int)sizeof(ybuf), "staging strips fit in ybuf");
    float *strip = reinterpret_cast<float *>(&ybuf[0][0]) + wave * (16 * SP);
    float *out = a.partials + ((int64_t)z * a.F + f0 + fh * 64) * a.K + (int64_t)(c0 + cq * 16) * TAPS;
#pragma unroll
    for (int fi = 0; fi < 4; ++fi) {
#pragma unroll
        for (int t = 0; t < TAPS; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) strip[(4 * lg + r) * SP + r16 * TAPS + t] = acc[fi][t][r];
        __builtin_amdgcn_wave_barrier();
        constexpr int Q4 = 16 * TAPS / 4;  // 16-byte pieces per row
#pragma unroll
        for (int p = 0; p < (16 * Q4 + 63) / 64; ++p) {
            const int idx = p * 64 + lane;
            if (idx < 16 * Q4) {
                const int row = idx / Q4, q4 = idx - row * Q4;
                const f32x4 v = *reinterpret_cast<const f32x4 *>(strip + row * SP + 4 * q4);
                *reinterpret_cast<f32x4 *>(out + (int64_t)(fi * 16 + row) * a.K + 4 * q4) = v;
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

typedef Plane<13, 13> Plane13;

static bool plane_supported(const ConvGeom &g) { return g.H == 13 && g.W == 13; }

static int g_max_splits = 0, g_off = 0;  // omni_tuning_set(OMNI_TUNE_WGRAD_*): sweeps and tests only

}  // namespace wpatch

void set_wgrad_patch_override(int max_splits, int off)
{
    if (max_splits >= 0) wpatch::g_max_splits = max_splits;
    if (off >= 0) wpatch::g_off = off;
}

bool wgrad_patch_supported(const ConvGeom &g, int dtype)
{
    using namespace wpatch;
    if (g_off) return false;
    if (dtype != OMNI_BF16 || g.kh != KH || g.kw != KW || g.sh != 1 || g.sw != 1 || g.ph != 1 || g.pw != 1) return false;
    if (!plane_supported(g) || g.C % CT != 0 || g.F % FT != 0) return false;
    if (!wgrad_direct_planes(g)) return false;  // the dY-hat layout this kernel reads
    const double ld = (double)dyhat_rows_ld(g);
    return (double)g.N * g.C * g.H * g.W * 2.0 < 4.0e9 && FT * ld * 2.0 < 4.0e9;
}

// Splits of the reduction (ranges of images): one round of workgroups on the 256 compute units.
int wgrad_patch_splits(const ConvGeom &g)
{
    using namespace wpatch;
    const int n_tiles = (g.F / FT) * (g.C / CT);
    int splits = 256 / n_tiles;
    if (splits < 1) splits = 1;
    if (g_max_splits > 0 && splits > g_max_splits) splits = g_max_splits;
    return splits < g.N ? splits : g.N;
}

int launch_wgrad_patch(const ConvGeom &g, const void *X, const void *dYhat, int64_t ld, float *partials, int splits,
                       hipStream_t s)
{
    using namespace wpatch;
    Args a;
    a.X = (const bf16_t *)X, a.dYhat = (const bf16_t *)dYhat, a.partials = partials, a.ld = ld;
    a.N = g.N, a.C = g.C, a.F = g.F, a.K = g.K;
    a.tiles_f = g.F / FT;
    a.n_tiles = a.tiles_f * (g.C / CT);
    a.splits = splits;
    a.n_items = a.n_tiles * splits;
    a.per_xcd = (a.n_items + 7) / 8;
    ProfScope prof(KID_GEMM_WGRAD, s, 2.0 * g.M * (double)g.K * g.F,
                   ((double)g.N * g.C * g.H * g.W + (double)g.F * g.M) * 2.0 + 4.0 * g.F * (double)g.K * splits);
    hipLaunchKernelGGL((wgrad_patch_kernel<Plane13>), dim3((unsigned)a.per_xcd * 8), dim3(NT), 0, s, a);
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

}  // namespace omni
