// Forward convolution of a wide-stride layer with few input channels (CaffeNet's conv1: 3 channels, 11 x 11
// window, stride 4) with the lowering fused into the matrix product (gfx950, bf16).
//
// Such a layer has a short reduction (K = 363) and a huge number of columns, so on the explicit path
// (App. C, "Convolution by Lowering and GEMM") writing and re-reading D-hat costs far more than the
// arithmetic.  Here D-hat never exists: a workgroup owns 512 consecutive output positions of one image and
// all (up to 96) filters, copies the input rows those positions touch into LDS as they are ([channel][row]
// [x], row pitch a multiple of 8 elements) and reads its MFMA operand straight out of that patch.
//
// The reduction index is reordered as (c, ky, kx) with the window row padded from kw to 4 * ceil(kw / 4)
// columns, in groups of 4 window columns.  With horizontal stride 4, group (c, ky, 4j .. 4j+3) of output
// column ox is the 8 aligned bytes at patch element (c, row, 4 * ox + 4 * j): consecutive lanes (consecutive
// ox) read consecutive 8-byte words, so the reads are free of bank conflicts.  An MFMA fragment (8 reduction
// indices) is two such groups.  Window columns beyond kw meet zero weights and are masked to zero in the
// fragment as well, so whatever pixel lies there never enters a sum.
//
// The weights (F x K', K' = 16 * steps <= 400) stay in LDS for the whole (persistent) workgroup: [pack][row]
// 16-byte packs as in the GEMM kernels.  Results leave through the staged epilogue (bias, ReLU, rounding,
// 16-byte stores), which borrows the patch's LDS space.
#include "common.h"
#include "mma_epilogue.h"
#include "pack_jobs.h"

namespace omni {
namespace strided {

constexpr int NT = 512;                  // 8 wavefronts, two per SIMD: one's LDS and store latencies hide under the other's MFMAs
constexpr int BM = 96, TI = BM / 32;     // every wavefront owns all filter rows
constexpr int TJ = 2;                    // 64 columns per wavefront
constexpr int BN = (NT / 64) * 32 * TJ;  // 512 columns per workgroup
constexpr int LA = BM + 1;
constexpr int MAX_PACKS = 50;            // 16-byte weight packs per row: K' <= 400
constexpr int MAX_GROUPS = 2 * MAX_PACKS;
constexpr int PATCH_ELEMS = 35584;       // bf16 elements of the LDS patch
constexpr int SLOTS = 9;                 // 16-byte patch pieces a thread moves per tile

struct Geom {
    int32_t N, C, H, W, F, Ho, Wo, kh, kw, sh;
    int32_t kwq;     // groups of 4 window columns per window row
    int32_t groups;  // C * kh * kwq
    int32_t steps;   // MFMA reduction steps of 16 = 4 groups
    int32_t PW;      // patch row pitch in elements: 4 * (Wo - 1 + kwq) rounded up to a multiple of 8
    int32_t CS;      // patch channel stride in elements (rows of the tallest tile times PW)
    int32_t tpc;     // pieces per thread and channel in the tallest tile
    int32_t HoWo, tiles_q, n_items;
    int32_t total;   // elements of X (< 2^31)
    FastDiv div_Wo, div_khkwq, div_kwq, div_tiles, div_PW8;
};

// result element (i = filter, j = output position inside the workgroup's image)
struct TileEpilogue {
    bf16_t *Yn;
    int F, HoWo, relu;
    typedef bf16_t Out;
    __device__ __forceinline__ char *base32(int) const { return reinterpret_cast<char *>(Yn); }
    __device__ __forceinline__ uint32_t row_stride32() const { return (uint32_t)HoWo * 2u; }
    __device__ __forceinline__ int n_rows() const { return F; }
    __device__ __forceinline__ uint32_t col_off32(int j, bool &ok) const
    {
        ok = j < HoWo;
        return (uint32_t)j * 2u;
    }
    static constexpr bool HAS_ROW_ADD = true;
    __device__ __forceinline__ float apply(float v, float add) const
    {
        v += add;
        if (relu) v = v > 0.f ? v : 0.f;
        return v;
    }
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// element j of the result = element j + s of x, zeros shifted in (0 < s < 8)
__device__ __forceinline__ u32x4 shifted_down(u32x4 x4, int s)
{
    unsigned __int128 x = ((unsigned __int128)(((uint64_t)x4[3] << 32) | x4[2]) << 64) | (((uint64_t)x4[1] << 32) | x4[0]);
    x >>= 16 * s;
    uint64_t lo = (uint64_t)x, hi = (uint64_t)(x >> 64);
    return u32x4{(uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32)};
}

// The workgroups are persistent: each loads the weights once and then walks its share of the tiles.  While a
// tile is being multiplied, the next tile's input rows are in flight into registers (16-byte pieces
// (c, row, 8 x8 .. 8 x8 + 7), read at element granularity); they go to LDS after the current tile's results
// have left through the same LDS space.
__global__ __launch_bounds__(NT) void strided_conv_kernel(const bf16_t *__restrict__ X, const uint4 *__restrict__ Wt,
                                                          bf16_t *__restrict__ Y, const float *__restrict__ bias,
                                                          int relu, Geom g)
{
    __shared__ uint4 atile[MAX_PACKS * LA];
    __shared__ uint4 patch[PATCH_ELEMS / 8];
    __shared__ uint4 gtab[MAX_GROUPS];  // per group: byte offset in the patch, masks of its two 32-bit halves
    __shared__ float lds_add[BM];

    const int tid = threadIdx.x;
    const int lane = tid % 64, wave = tid / 64;
    const int li = lane % 32, h = lane / 32;

    for (int gi = tid; gi < 4 * g.steps; gi += NT) {
        uint4 e = make_uint4(0u, 0u, 0u, 0u);
        if (gi < g.groups) {
            uint32_t c, rem, ky, kq;
            g.div_khkwq.divmod((uint32_t)gi, c, rem);
            g.div_kwq.divmod(rem, ky, kq);
            const int vc = g.kw - 4 * (int)kq;  // window columns of this group that exist (>= 1)
            e.x = (uint32_t)(((int)c * g.CS + (int)ky * g.PW + 4 * (int)kq) * 2);
            e.y = vc >= 2 ? 0xffffffffu : 0xffffu;
            e.z = vc >= 4 ? 0xffffffffu : (vc == 3 ? 0xffffu : 0u);
        }
        gtab[gi] = e;
    }
    for (int i = tid; i < BM; i += NT) lds_add[i] = (bias != nullptr && i < g.F) ? bias[i] : 0.f;
    {
        const int n_packs = 2 * g.steps * BM;
        for (int i0 = tid; i0 < n_packs; i0 += 8 * NT) {
            uint4 w[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * NT;
                w[u] = Wt[i < n_packs ? i : n_packs - 1];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + u * NT;
                const int p = i / BM, f = i - p * BM;
                if (i < n_packs) atile[p * LA + f] = w[u];
            }
        }
    }

    // this thread's pieces: slot s = (channel s / tpc, piece tid + (s % tpc) * NT of the channel's rows)
    uint32_t rx[SLOTS];  // row | x8 << 16
    {
        int j = 0;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            uint32_t r, x8;
            g.div_PW8.divmod((uint32_t)(tid + j * NT), r, x8);
            rx[s] = r | (x8 << 16);
            if (++j == g.tpc) j = 0;
        }
    }
    u32x4 pre[SLOTS];
    const char *xb = reinterpret_cast<const char *>(X);
    const int top = g.total - 8;
    // tile -> image n, first position q0, first output row oy_a, patch rows PH
    auto tile_of = [&](int item, int &n, int &q0, int &oy_a, int &PH) {
        uint32_t nn, tq;
        g.div_tiles.divmod((uint32_t)item, nn, tq);
        n = (int)nn;
        q0 = (int)tq * BN;
        const int q_last = (q0 + BN < g.HoWo ? q0 + BN : g.HoWo) - 1;
        oy_a = (int)g.div_Wo.div((uint32_t)q0);
        const int oy_b = (int)g.div_Wo.div((uint32_t)q_last);
        PH = (oy_b - oy_a) * g.sh + g.kh;  // input rows oy_a * sh .. + PH - 1, all inside the image (no padding)
    };
    auto issue_patch = [&](int n, int oy_a, int PH) {
        int c = 0, j = 0;
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            uint32_t q = rx[s];
            asm volatile("" : "+v"(q));  // opaque: what follows is recomputed per tile instead of kept (and spilled) across tiles
            const int r = (int)(q & 0xffffu), x8 = (int)(q >> 16);
            const bool ok = c < g.C && r < PH;
            const int e = ((n * g.C + c) * g.H + oy_a * g.sh + r) * g.W + 8 * x8;
            const int ec = ok ? (e < top ? e : top) : 0;
            __builtin_memcpy(&pre[s], xb + 2u * (uint32_t)ec, 16);
            if (++j == g.tpc) j = 0, ++c;
        }
    };
    auto commit_patch = [&](int n, int oy_a, int PH) {
        int c = 0, j = 0;
        u32x4 *dst = reinterpret_cast<u32x4 *>(patch);
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            uint32_t q = rx[s];
            asm volatile("" : "+v"(q));  // opaque: what follows is recomputed per tile instead of kept (and spilled) across tiles
            const int r = (int)(q & 0xffffu), x8 = (int)(q >> 16);
            if (c < g.C && r < PH) {
                u32x4 w = pre[s];
                const int e = ((n * g.C + c) * g.H + oy_a * g.sh + r) * g.W + 8 * x8;
                if (e > top) w = shifted_down(w, e - top);  // the tensor's last few elements only
                const int valid = g.W - 8 * x8;             // elements of the piece inside the row (>= 1)
                if (valid < 8) {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        w[i] &= valid >= 2 * i + 2 ? 0xffffffffu : (valid == 2 * i + 1 ? 0xffffu : 0u);
                }
                dst[(c * g.CS + r * g.PW) / 8 + x8] = w;
            }
            if (++j == g.tpc) j = 0, ++c;
        }
    };

    int item = blockIdx.x;
    int n, q0, oy_a, PH;
    if (item < g.n_items) {
        tile_of(item, n, q0, oy_a, PH);
        issue_patch(n, oy_a, PH);
    }
    const char *pb = reinterpret_cast<const char *>(patch);
    for (; item < g.n_items; item += gridDim.x) {
        commit_patch(n, oy_a, PH);
        __syncthreads();  // the patch (and, the first time, weights and tables) are in LDS
        const int cur_n = n, cur_q0 = q0, cur_oy_a = oy_a;
        if (item + (int)gridDim.x < g.n_items) {
            tile_of(item + (int)gridDim.x, n, q0, oy_a, PH);
            issue_patch(n, oy_a, PH);
        }

        // byte offset in the patch of window tap (0, 0) of each of this lane's columns
        uint32_t pp0[TJ];
#pragma unroll
        for (int u = 0; u < TJ; ++u) {
            int q = cur_q0 + wave * (32 * TJ) + 32 * u + li;
            q = q < g.HoWo ? q : g.HoWo - 1;
            uint32_t oy, ox;
            g.div_Wo.divmod((uint32_t)q, oy, ox);
            pp0[u] = (uint32_t)((((int)oy - cur_oy_a) * g.sh * g.PW + 4 * (int)ox) * 2);
        }

        f32x16 acc[TI][TJ];
#pragma unroll
        for (int t = 0; t < TI; ++t)
#pragma unroll
            for (int u = 0; u < TJ; ++u)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[t][u][v] = 0.f;

        // fragments of step st: this half-wave's pack p = 2 st + h holds reduction indices 16 st + 8 h .. + 7
        auto load_frags = [&](int st, uint4 (&a)[TI], uint4 (&b)[TJ]) {
            const int p = 2 * st + h;
#pragma unroll
            for (int t = 0; t < TI; ++t) a[t] = atile[p * LA + 32 * t + li];
            const uint4 e0 = gtab[2 * p], e1 = gtab[2 * p + 1];
#pragma unroll
            for (int u = 0; u < TJ; ++u) {
                const uint2 lo = *reinterpret_cast<const uint2 *>(pb + (pp0[u] + e0.x));
                const uint2 hi = *reinterpret_cast<const uint2 *>(pb + (pp0[u] + e1.x));
                b[u] = make_uint4(lo.x & e0.y, lo.y & e0.z, hi.x & e1.y, hi.y & e1.z);
            }
        };
        auto mma = [&](const uint4 (&a)[TI], const uint4 (&b)[TJ]) {
#pragma unroll
            for (int t = 0; t < TI; ++t)
#pragma unroll
                for (int u = 0; u < TJ; ++u) Mma<bf16_t>::run(a[t], b[u], acc[t][u]);
        };
        for (int st = 0; st < g.steps; ++st) {
            uint4 a0[TI], b0[TJ];
            load_frags(st, a0, b0);
            mma(a0, b0);
        }

        __syncthreads();  // every wavefront is done with the patch: it becomes staging space
        TileEpilogue epi{Y + (int64_t)cur_n * g.F * g.HoWo, g.F, g.HoWo, relu};
        constexpr int STRIP = 16 * staged_pitch(TJ);
        static_assert((NT / 64) * STRIP <= PATCH_ELEMS * 2, "staging strips fit in the patch");
        store_tile_staged<TI, TJ, 16>(acc, 0, cur_q0 + wave * (32 * TJ), lane, 0, epi,
                                      reinterpret_cast<char *>(patch) + wave * STRIP, lds_add, 0);
        __syncthreads();  // the strips are free again
    }
}

// The kernel's weights: W [F][C][kh][kw] -> [pack p][row f (96)] 16-byte packs: pack p holds groups 2p and 2p + 1,
// group (c, ky, j) the window columns 4j .. 4j + 3 (zero beyond kw, beyond the last group and for rows beyond F);
// written by pack_one (pack_jobs.h), kind 1.

static bool make_strided_geom(const ConvGeom &c, Geom *g)
{
    if (c.sw != 4 || c.ph != 0 || c.pw != 0 || c.F > BM) return false;
    g->N = c.N, g->C = c.C, g->H = c.H, g->W = c.W, g->F = c.F, g->Ho = c.Ho, g->Wo = c.Wo;
    g->kh = c.kh, g->kw = c.kw, g->sh = c.sh;
    g->kwq = (c.kw + 3) / 4;
    int64_t groups = (int64_t)c.C * c.kh * g->kwq;
    if (groups > MAX_GROUPS) return false;
    g->groups = (int32_t)groups;
    g->steps = (g->groups + 3) / 4;
    if (2 * g->steps > MAX_PACKS) return false;
    g->PW = (int32_t)round_up(4 * (c.Wo - 1 + g->kwq), 8);
    int rows_max = (c.Wo - 1 + BN - 1) / c.Wo + 1;  // output rows a tile of BN positions can touch
    if (rows_max > c.Ho) rows_max = c.Ho;
    int64_t ph_max = (int64_t)(rows_max - 1) * c.sh + c.kh;
    int64_t cs = ph_max * g->PW;
    if (cs * c.C > PATCH_ELEMS || ph_max > 0xffff) return false;
    g->CS = (int32_t)cs;
    g->tpc = (int32_t)((cs / 8 + NT - 1) / NT);
    if ((int64_t)g->tpc * c.C > SLOTS) return false;
    int64_t total = (int64_t)c.N * c.C * c.H * c.W;
    if (total < 8 || total > 0x7fffffffll - 4096) return false;
    g->total = (int32_t)total;
    g->HoWo = c.HoWo;
    g->tiles_q = (c.HoWo + BN - 1) / BN;
    int64_t items = (int64_t)c.N * g->tiles_q;
    if (items > 0x7fffffffll - 4096 || (double)c.F * c.HoWo * 2.0 >= 4.0e9) return false;
    g->n_items = (int32_t)items;
    g->div_Wo = FastDiv((uint32_t)c.Wo);
    g->div_khkwq = FastDiv((uint32_t)(c.kh * g->kwq));
    g->div_kwq = FastDiv((uint32_t)g->kwq);
    g->div_tiles = FastDiv((uint32_t)g->tiles_q);
    g->div_PW8 = FastDiv((uint32_t)(g->PW / 8));
    return true;
}

// X [planes][H][W] -> X4 [planes][4][H][WP]: X4(p, ph, y, xq) = X(p, y, 4 xq + ph), zero where 4 xq + ph >= W
// (the phase images of the stride-4 model gradient).  One thread per 32 consecutive input columns of a row:
// four 16-byte reads (element by element in a row's ragged last group), 16 half-word shuffles, one 16-byte
// piece of every phase image.
__global__ __launch_bounds__(256) void phase_split_kernel(const bf16_t *__restrict__ X, uint4 *__restrict__ X4, int planes,
                                                          int H, int W, FastDiv div_G, FastDiv div_H)
{
    const int G = (int)div_G.d;  // groups per row = WP / 8
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)planes * H * G) return;
    uint32_t row, gq, pl, y;
    div_G.divmod((uint32_t)idx, row, gq);
    div_H.divmod(row, pl, y);
    const bf16_t *src = X + ((int64_t)row * W + 32 * (int)gq);
    uint32_t w[16];
    if (32 * (int)gq + 32 <= W) {
        __builtin_memcpy(w, src, 64);
    } else {
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int x = 32 * (int)gq + 2 * k;
            const uint32_t lo = x < W ? (uint32_t)src[2 * k] : 0u, hi = x + 1 < W ? (uint32_t)src[2 * k + 1] : 0u;
            w[k] = lo | (hi << 16);
        }
    }
#pragma unroll
    for (int ph = 0; ph < 4; ++ph) {
        uint32_t o[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const uint32_t a = w[4 * t + ph / 2], b = w[4 * t + 2 + ph / 2];  // elements 8t + ph and 8t + 4 + ph
            o[t] = (ph % 2 == 0) ? ((a & 0xffffu) | (b << 16)) : ((a >> 16) | (b & 0xffff0000u));
        }
        X4[(((int64_t)pl * 4 + ph) * H + y) * G + gq] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

}  // namespace strided

int launch_phase_split(const ConvGeom &c, int WP, const void *X, void *X4, hipStream_t s)
{
    const int planes = c.N * c.C, G = WP / 8;
    const int64_t total = (int64_t)planes * c.H * G;
    if (total > 0x7fffffffll - 4096) return OMNI_UNSUPPORTED;
    ProfScope prof(KID_LOWER, s, 0.0, 2.0 * ((double)planes * c.H * c.W + (double)planes * 4 * c.H * WP));
    hipLaunchKernelGGL(strided::phase_split_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                       (const bf16_t *)X, (uint4 *)X4, planes, c.H, c.W, FastDiv((uint32_t)G), FastDiv((uint32_t)c.H));
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

// ------------------------------------------------------------------------------------------------
// Data gradient of a strided, unpadded layer without dD-hat or a scatter step.  Input pixel
// (y, x) = (sh yq + py, sw xq + px) receives dY(oy, ox) W(ky, kx) from the taps ky = py + sh kr, kx = px + sw kq
// at oy = yq - kr, ox = xq - kq: for a fixed phase (py, px) that is a stride-1 correlation of dY (F channels) with
// a window of ceil(kh / sh) x ceil(kw / sw) taps and full padding.  So the gradient is ONE stride-1 convolution
// with C sh sw output channels (c, py, px), run by the fused stride-1 kernel (implicit.hip) on dY as it is, followed
// by the interleaving of the phase images into dX (the inverse of phase_split).
//   Wc[(c, py, px)][f][a][b] = W[f][c][py + sh (khq - 1 - a)][px + sw (kwq - 1 - b)]   (0 beyond the window)
// ------------------------------------------------------------------------------------------------
namespace strided {

struct DgradPlan {
    ConvGeom gs;        // the stride-1 convolution: input dY [N][F][Ho][Wo], output [N][C sh sw][Hq][Wq]
    int khq, kwq, Hq, Wq, Co;
    size_t wt, wc, x4, total;  // workspace regions: packed weights of the fused kernel, Wc, the phase images
};

static bool make_dgrad_plan(const ConvGeom &c, int dtype, DgradPlan *p)
{
    if (dtype != OMNI_BF16 || c.ph != 0 || c.pw != 0 || (c.sh == 1 && c.sw == 1)) return false;
    p->khq = (c.kh + c.sh - 1) / c.sh, p->kwq = (c.kw + c.sw - 1) / c.sw;
    p->Hq = c.Ho + p->khq - 1, p->Wq = c.Wo + p->kwq - 1;
    int64_t co = (int64_t)c.C * c.sh * c.sw;
    if (co > 65535) return false;
    p->Co = (int)co;
    omni_conv_desc d{};
    d.N = c.N, d.C = c.F, d.H = c.Ho, d.W = c.Wo, d.F = p->Co, d.kh = p->khq, d.kw = p->kwq;
    d.stride_h = d.stride_w = 1, d.pad_h = p->khq - 1, d.pad_w = p->kwq - 1, d.dtype = OMNI_BF16, d.flags = 0;
    if (make_geom(&d, &p->gs) != OMNI_OK || p->gs.Ho != p->Hq || p->gs.Wo != p->Wq) return false;
    if (!fused_supported(p->gs, OMNI_BF16, false)) return false;
    if ((double)c.N * p->Co * p->Hq * p->Wq * 2.0 >= 4.0e9) return false;
    auto al = [](size_t b) { return (b + 255) / 256 * 256; };
    p->wt = 0;
    p->wc = al(fused_weight_bytes(p->gs, false));
    p->x4 = p->wc + al((size_t)p->Co * c.F * p->khq * p->kwq * 2);
    p->total = p->x4 + al((size_t)c.N * p->Co * p->Hq * p->Wq * 2);
    return true;
}

__global__ __launch_bounds__(256) void dgrad_phase_weights_kernel(const bf16_t *__restrict__ W, bf16_t *__restrict__ Wc, int C,
                                                                  int F, int kh, int kw, int sh, int sw, int khq, int kwq)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int taps = khq * kwq, total = C * sh * sw * F * taps;
    if (idx >= total) return;
    const int tap = idx % taps, f = (idx / taps) % F, co = idx / (taps * F);
    const int a = tap / kwq, b = tap - a * kwq;
    const int px = co % sw, py = (co / sw) % sh, c = co / (sw * sh);
    const int ky = py + sh * (khq - 1 - a), kx = px + sw * (kwq - 1 - b);
    Wc[idx] = (ky < kh && kx < kw) ? W[((f * C + c) * kh + ky) * kw + kx] : (bf16_t)0;
}

// dX(n, c, y, x) = X4(n, (c sh + y % sh) sw + x % sw, y / sh, x / sw), zero where that entry does not exist (rows and
// columns no window reaches).  One thread per 8 consecutive x of a row.
__global__ __launch_bounds__(256) void phase_merge_kernel(const bf16_t *__restrict__ X4, bf16_t *__restrict__ dX, int planes,
                                                          int H, int W, int sh, int sw, int Hq, int Wq, FastDiv div_G,
                                                          FastDiv div_H, FastDiv div_sh, FastDiv div_sw)
{
    const int G = (int)div_G.d;  // 8-element groups per row
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)planes * H * G) return;
    uint32_t row, gq, pl, y, yq, py;
    div_G.divmod((uint32_t)idx, row, gq);
    div_H.divmod(row, pl, y);
    div_sh.divmod(y, yq, py);
    const bf16_t *src = X4 + (((int64_t)pl * sh + py) * sw * Hq + yq) * Wq;  // phase px adds px * Hq * Wq
    const int64_t phase = (int64_t)Hq * Wq;
    uint32_t v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int x = 8 * (int)gq + e;
        uint32_t xq, px;
        div_sw.divmod((uint32_t)x, xq, px);
        v[e] = (x < W && (int)yq < Hq && (int)xq < Wq) ? (uint32_t)src[px * phase + xq] : 0u;
    }
    bf16_t *dst = dX + (int64_t)row * W + 8 * (int)gq;
    if (8 * (int)gq + 8 <= W) {
        const uint4 o = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
        __builtin_memcpy(dst, &o, 16);  // element-aligned 16-byte store
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (8 * (int)gq + e < W) dst[e] = (bf16_t)v[e];
    }
}

}  // namespace strided

bool strided_dgrad_supported(const ConvGeom &c, int dtype)
{
    strided::DgradPlan p;
    return strided::make_dgrad_plan(c, dtype, &p);
}

size_t strided_dgrad_bytes(const ConvGeom &c)
{
    strided::DgradPlan p;
    return strided::make_dgrad_plan(c, OMNI_BF16, &p) ? p.total : 0;
}

int launch_strided_dgrad(const ConvGeom &c, const void *dY, const void *W, void *dX, void *workspace, hipStream_t s)
{
    using namespace strided;
    DgradPlan p;
    if (!make_dgrad_plan(c, OMNI_BF16, &p)) return OMNI_UNSUPPORTED;
    char *ws = (char *)workspace;
    bf16_t *Wc = (bf16_t *)(ws + p.wc), *X4 = (bf16_t *)(ws + p.x4);
    {
        ProfScope prof(KID_PACK_KHAT, s, 0.0, 2.0 * (double)c.F * c.K * 2.0);
        const int total = p.Co * c.F * p.khq * p.kwq;
        hipLaunchKernelGGL(dgrad_phase_weights_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const bf16_t *)W, Wc,
                           c.C, c.F, c.kh, c.kw, c.sh, c.sw, p.khq, p.kwq);
        OMNI_LAUNCH_CHECK();
    }
    int st = launch_fused_conv(p.gs, false, dY, Wc, nullptr, 0, X4, ws + p.wt, s, KID_FUSED_DGRAD);
    if (st != OMNI_OK) return st;
    const int planes = c.N * c.C, G = (c.W + 7) / 8;
    const int64_t total = (int64_t)planes * c.H * G;
    if (total > 0x7fffffffll - 4096) return OMNI_UNSUPPORTED;
    ProfScope prof(KID_COL2IM, s, 0.0, 2.0 * ((double)planes * c.H * c.W + (double)c.N * p.Co * p.Hq * p.Wq));
    hipLaunchKernelGGL(phase_merge_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const bf16_t *)X4, (bf16_t *)dX,
                       planes, c.H, c.W, c.sh, c.sw, p.Hq, p.Wq, FastDiv((uint32_t)G), FastDiv((uint32_t)c.H),
                       FastDiv((uint32_t)c.sh), FastDiv((uint32_t)c.sw));
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

bool strided_supported(const ConvGeom &c, int dtype)
{
    strided::Geom g;
    return dtype == OMNI_BF16 && strided::make_strided_geom(c, &g);
}

size_t strided_weight_bytes(const ConvGeom &c)
{
    strided::Geom g;
    if (!strided::make_strided_geom(c, &g)) return 0;
    return (size_t)2 * g.steps * strided::BM * 16;
}

static void fill_strided_job(const strided::Geom &g, const void *W, void *packed, PackJob *job)
{
    job->kind = 1;
    job->W = (const bf16_t *)W, job->Wt = (uint4 *)packed;
    job->total = (int64_t)2 * g.steps * strided::BM;
    job->F = g.F, job->Fp = job->KK = job->n_chunks = job->flip = 0, job->stride_out = job->stride_in = 0;
    job->C = g.C, job->kh = g.kh, job->kw = g.kw, job->kwq = g.kwq, job->groups = g.groups, job->BM = strided::BM;
}

bool strided_pack_job(const ConvGeom &c, const void *W, void *packed, PackJob *job, size_t *bytes)
{
    strided::Geom g;
    *bytes = 0;
    if (!strided::make_strided_geom(c, &g)) return false;
    *bytes = strided_weight_bytes(c);
    if (job != nullptr) fill_strided_job(g, W, packed, job);
    return true;
}

// `prepacked` != null: the repacked weights already exist there (strided_pack_job) and W is not read
int launch_strided_conv(const ConvGeom &c, const void *X, const void *W, const float *bias, int relu, void *Y,
                        void *wt_scratch, hipStream_t s, const void *prepacked)
{
    using namespace strided;
    Geom g;
    if (!make_strided_geom(c, &g)) return OMNI_UNSUPPORTED;
    if (prepacked == nullptr) {
        PackJobTable t;
        fill_strided_job(g, W, wt_scratch, &t.job[0]);
        t.first_block[0] = 0, t.first_block[1] = (t.job[0].total + 255) / 256, t.n = 1;
        int st = launch_pack_jobs(t, s);
        if (st != OMNI_OK) return st;
    }
    const uint4 *wt = (const uint4 *)(prepacked != nullptr ? prepacked : wt_scratch);
    ProfScope prof(KID_STRIDED_FWD, s, 2.0 * (double)c.M * c.K * c.F,
                   2.0 * ((double)c.N * c.C * c.H * c.W + (double)c.M * c.F));
    hipLaunchKernelGGL(strided_conv_kernel, dim3((unsigned)(g.n_items < 256 ? g.n_items : 256)), dim3(NT), 0, s, (const bf16_t *)X,
                       wt, (bf16_t *)Y, bias, relu, g);
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

}  // namespace omni
