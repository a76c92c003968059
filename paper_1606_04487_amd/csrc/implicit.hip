// Convolution with the lowering fused into the matrix product (gfx950, bf16, stride 1).
//
// The lowered matrix D-hat repeats every input element kh*kw times (App. C: the replication factor of
// the lowering phase), and the explicit path moves it through HBM several times per training step.
// This kernel computes the same product  Y-hat[F x M] = K-hat[F x K] * D-hat[K x M]  without D-hat ever
// existing in memory: a workgroup that owns 256 consecutive columns m = (n, oy, ox) keeps the zero-padded
// input pixels those columns touch in LDS, one 32-channel chunk at a time, and reads its MFMA operand
// straight out of that patch -- entry ((c, ky, kx), m) of D-hat is the patch pixel (oy + ky, ox + kx) of
// channel c, so a window tap is a constant LDS offset.  The reduction runs over (chunk, tap, channel in
// chunk); a sum does not care about the order of its terms, and the weights are repacked to match.
//
// The data gradient of a stride-1 layer is the same computation with the roles of the two channel
// counts exchanged, the window flipped and padding k - 1 - p (the col2im sum, written as a gather), so
// it runs on the same kernel and needs neither dD-hat nor a scatter step.
//
// LDS layout: patch[g][pixel] and atile[tap][g][row] of 16-byte packs, pack g holding channels
// 8g .. 8g+7 of the chunk, so a fragment is one 16-byte read per lane and consecutive lanes (consecutive
// pixels or rows) read consecutive packs.  Pixels are transposed from the input's [channel][pixel]
// order in registers on their way into LDS (8 channels x 8 pixels per thread).  Padding pixels are
// zeroed once: the patch layout is the same for every chunk, and loads only ever write real pixels.
//
// Schedule: the weights of up to TG window taps are staged in LDS together, in one of two buffers, so a
// workgroup runs TG taps (TG x 8 MFMAs per wavefront) between barriers.  While it does, the next group's
// weights and -- during a chunk's first group -- the next chunk's pixels are in flight into registers.  The
// weights go to the other buffer before the group's last tap (every wavefront left that buffer before the last
// barrier), so those stores run under the other wavefronts' MFMAs and one barrier per group publishes them;
// only the pixels, once per chunk, need a barrier of their own before they overwrite the patch.
#include <cstdlib>
#include <type_traits>

#include "common.h"
#include "mma_epilogue.h"
#include "pack_jobs.h"

namespace omni {
namespace fused {

constexpr int CH = 32;           // channels per reduction chunk
constexpr int NG = CH / 8;       // 16-byte packs per pixel and chunk
constexpr int NT = 512;          // 8 wavefronts
// Columns (output positions) per workgroup and the patch capacity in pixels that goes with them.  The wide
// tile gives each wavefront 64 x 128 results: 6 instead of 8 LDS fragment reads per 8 MFMAs, and LDS
// bandwidth is what caps this kernel.
constexpr int BN_NARROW = 256, PATCH_NARROW = 672;
constexpr int BN_MID = 384, PATCH_MID = 960;
constexpr int BN_WIDE = 512, PATCH_WIDE = 1040;
constexpr int TG = 5;            // window taps whose weights are staged in LDS together (two such buffers)
constexpr int MAX_SLOTS = 8;     // images a column tile may touch
constexpr uint32_t NO_PIX = 0xffffu;

static int g_fused_bn = 0, g_fused_bm = 0, g_fused_bare_pitch = 0;  // omni_tuning_set(OMNI_TUNE_FUSED_*): sweeps and tests only

struct Geom {
    int32_t N, C, H, W;      // input  [N][C][H][W]
    int32_t F, Ho, Wo;       // output [N][F][Ho][Wo],  Ho = H + 2*ph - kh + 1
    int32_t kh, kw, ph, pw;  // window, zero padding
    int32_t Wp;              // row pitch of the patch: at least W + 2*pw, the width of a padded row
    int32_t HW, HoWo, M, KK;
    uint32_t sn, sc;         // elements from an input image to the next and from a channel's plane to the next
    int32_t n_chunks;        // C / CH
    int32_t Fp;              // F rounded up to the row tile
    int32_t tiles_f, tiles_m, n_items, per_xcd;
    int32_t splits, chunks_per_split;  // the reduction's chunks cut into `splits` ranges (1: not split)
    int32_t bn;              // columns per workgroup: BN_NARROW, BN_MID or BN_WIDE
    int32_t bm;              // filter rows per workgroup: 128, or 96 (with BN_WIDE) for layers of few filters
    FastDiv div_HoWo, div_Wo, div_W;
};

// What a column tile [col0, m_last] needs of image n: padded rows [ra, ra + nrows) of which the real
// input rows are [ya, ya + len / W).
struct SlotSpan { int ra, nrows, ya, len; };
__host__ __device__ inline SlotSpan slot_span(const Geom &g, int col0, int m_last, int n)
{
    int base = n * g.HoWo;
    int qa = col0 > base ? col0 - base : 0;
    int qb = m_last - base < g.HoWo - 1 ? m_last - base : g.HoWo - 1;
    int oya = (int)g.div_Wo.div((uint32_t)qa), oyb = (int)g.div_Wo.div((uint32_t)qb);
    SlotSpan s;
    s.ra = oya;
    s.nrows = oyb - oya + g.kh;
    int ya = s.ra - g.ph, yb = s.ra + s.nrows - g.ph;
    if (ya < 0) ya = 0;
    if (yb > g.H) yb = g.H;
    s.ya = ya;
    s.len = yb > ya ? (yb - ya) * g.W : 0;
    return s;
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Patch pixels are stored at swz(pixel): a loader thread writes 8 consecutive pixels and its neighbour the
// next 8, so without the permutation every lane of a store would fall on the same two bank groups.  The
// permutation stays inside aligned blocks of 8, so a run of consecutive pixels read by consecutive lanes
// still covers all banks.
__device__ __forceinline__ int swz(int pix) { return pix ^ ((pix >> 4) & 7); }

__device__ __forceinline__ uint32_t lo16(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
__device__ __forceinline__ uint32_t hi16(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }

// Compile-time loop: the body receives std::integral_constant<int, I>.
template <int I, int N, typename F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Epi: FwdEpilogue<bf16_t> (bias, ReLU, rounding, store into Y), or PartialEpilogue when few column tiles
// exist (small batches): the reduction's chunks are then split over `g.splits` workgroups per tile, each
// leaving its raw fp32 sums in a slice [F][M] of the scratch, which reduce_store_kernel adds in split order
// and hands to the forward epilogue.
// RIN: the input is read with the strides g.sn, g.sc (its rows form) instead of as the dense tensor.
template <int BM, int WM, int WN, int BN, int PATCH_PIX, typename Epi, bool RIN = false>
__global__ __launch_bounds__(NT) void fused_conv_kernel(const bf16_t *__restrict__ X, const bf16_t *__restrict__ Wt,
                                                        Geom g, Epi epi)
{
    static_assert(WM * WN * 64 == NT, "eight wavefronts");
    static_assert(BM * NG <= NT, "at most one 16-byte piece of a tap's weight tile per thread");
    constexpr int TI = BM / WM / 32, TJ = BN / WN / 32;
    constexpr int LA = BM + 1;
    __shared__ uint4 patch[NG * PATCH_PIX];
    __shared__ uint4 atile[2 * TG * NG * LA];
    __shared__ float lds_add[BM];
    __shared__ int slot_so[MAX_SLOTS], slot_ra[MAX_SLOTS], slot_p0[MAX_SLOTS], slot_ya[MAX_SLOTS], slot_len[MAX_SLOTS];
    __shared__ int total_pieces;

    const int xcd = blockIdx.x % 8, slot_id = blockIdx.x / 8;
    const int item = xcd * g.per_xcd + slot_id;  // contiguous ranges of tiles per XCD, row tiles fastest
    if (item >= g.n_items) return;
    const int n_tiles = g.tiles_f * g.tiles_m;
    const int z = item / n_tiles, tile_id = item - z * n_tiles;   // splits of one tile are far apart in time
    const int chunk_lo = z * g.chunks_per_split;
    const int chunk_hi = chunk_lo + g.chunks_per_split < g.n_chunks ? chunk_lo + g.chunks_per_split : g.n_chunks;
    const int tm = tile_id / g.tiles_f, tf = tile_id - tm * g.tiles_f;
    const int row0 = tf * BM, col0 = tm * BN;
    const int m_last = (col0 + BN < g.M ? col0 + BN : g.M) - 1;
    const int n0 = (int)g.div_HoWo.div((uint32_t)col0);
    const int nslots = (int)g.div_HoWo.div((uint32_t)m_last) - n0 + 1;

    const int tid = threadIdx.x;
    const int lane = tid % 64, wave = tid / 64;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane % 32, h = lane / 32;

    if (tid == 0) {
        int so = 0, p0 = 0;
        for (int i = 0; i < nslots; ++i) {
            SlotSpan s = slot_span(g, col0, m_last, n0 + i);
            slot_so[i] = so, slot_ra[i] = s.ra, slot_p0[i] = p0, slot_ya[i] = s.ya, slot_len[i] = s.len;
            so += s.nrows;
            p0 += (s.len + 7) / 8;
        }
        total_pieces = p0;
    }
    __syncthreads();

    // patch pixel of each of this lane's columns at tap (0, 0)
    int pp0[TJ];
#pragma unroll
    for (int u = 0; u < TJ; ++u) {
        int m = col0 + wn * (BN / WN) + 32 * u + li;
        m = m < g.M ? m : g.M - 1;
        uint32_t n, q, oy, ox;
        g.div_HoWo.divmod((uint32_t)m, n, q);
        g.div_Wo.divmod(q, oy, ox);
        int i = (int)n - n0;
        pp0[u] = (slot_so[i] + (int)oy - slot_ra[i]) * g.Wp + (int)ox;
    }

    // This thread's share of a chunk: 8 channels (pack tg) x 8 consecutive elements of one image's rows.
    const int PT = total_pieces;
    const bool has_task = tid < NG * PT;
    uint32_t goff = 0;                        // byte offset of the task's first element in chunk 0
    uint32_t l01 = NO_PIX | (NO_PIX << 16), l23 = l01, l45 = l01, l67 = l01;  // patch index of each element
    if (has_task) {
        int tg = tid / PT, jj = tid - tg * PT;
        int i = nslots - 1;
        while (i > 0 && jj < slot_p0[i]) --i;
        int ea = slot_ya[i] * g.W, eb = ea + slot_len[i];
        int e0 = ea + 8 * (jj - slot_p0[i]);
        e0 = e0 < g.HW - 8 ? e0 : g.HW - 8;  // stay inside the plane: the overlap rewrites equal values
        if constexpr (RIN) goff = ((uint32_t)(n0 + i) * g.sn + (uint32_t)(8 * tg) * g.sc + (uint32_t)e0) * 2u;
        else goff = ((uint32_t)((n0 + i) * g.C + 8 * tg) * (uint32_t)g.HW + (uint32_t)e0) * 2u;
        uint32_t l[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int flat = e0 + e;
            uint32_t y, x;
            g.div_W.divmod((uint32_t)flat, y, x);
            int pp = (slot_so[i] + (int)y + g.ph - slot_ra[i]) * g.Wp + (int)x + g.pw;
            l[e] = (flat >= ea && flat < eb) ? (uint32_t)(tg * PATCH_PIX + swz(pp)) : NO_PIX;
        }
        l01 = l[0] | (l[1] << 16), l23 = l[2] | (l[3] << 16), l45 = l[4] | (l[5] << 16), l67 = l[6] | (l[7] << 16);
    }

    u32x4 r0, r1, r2, r3, r4, r5, r6, r7;  // 8 channels x 8 elements
    const char *xb = reinterpret_cast<const char *>(X);
    const uint32_t plane_b = (RIN ? g.sc : (uint32_t)g.HW) * 2u, chunk_b = plane_b * CH;
    auto issue_patch = [&](int chunk) {
        const char *p = xb + (goff + (uint32_t)chunk * chunk_b);  // threads without a task read a valid address too
        __builtin_memcpy(&r0, p, 16);
        __builtin_memcpy(&r1, p + plane_b, 16);
        __builtin_memcpy(&r2, p + 2 * plane_b, 16);
        __builtin_memcpy(&r3, p + 3 * plane_b, 16);
        __builtin_memcpy(&r4, p + 4 * plane_b, 16);
        __builtin_memcpy(&r5, p + 5 * plane_b, 16);
        __builtin_memcpy(&r6, p + 6 * plane_b, 16);
        __builtin_memcpy(&r7, p + 7 * plane_b, 16);
    };
    auto commit_patch = [&]() {
        u32x4 *dst = reinterpret_cast<u32x4 *>(patch);
        uint32_t l;
        // element e of the 8 x 8 block as one pack: the 8 channels of that pixel
        l = l01 & 0xffffu; if (l != NO_PIX) dst[l] = u32x4{lo16(r0[0], r1[0]), lo16(r2[0], r3[0]), lo16(r4[0], r5[0]), lo16(r6[0], r7[0])};
        l = l01 >> 16;     if (l != NO_PIX) dst[l] = u32x4{hi16(r0[0], r1[0]), hi16(r2[0], r3[0]), hi16(r4[0], r5[0]), hi16(r6[0], r7[0])};
        l = l23 & 0xffffu; if (l != NO_PIX) dst[l] = u32x4{lo16(r0[1], r1[1]), lo16(r2[1], r3[1]), lo16(r4[1], r5[1]), lo16(r6[1], r7[1])};
        l = l23 >> 16;     if (l != NO_PIX) dst[l] = u32x4{hi16(r0[1], r1[1]), hi16(r2[1], r3[1]), hi16(r4[1], r5[1]), hi16(r6[1], r7[1])};
        l = l45 & 0xffffu; if (l != NO_PIX) dst[l] = u32x4{lo16(r0[2], r1[2]), lo16(r2[2], r3[2]), lo16(r4[2], r5[2]), lo16(r6[2], r7[2])};
        l = l45 >> 16;     if (l != NO_PIX) dst[l] = u32x4{hi16(r0[2], r1[2]), hi16(r2[2], r3[2]), hi16(r4[2], r5[2]), hi16(r6[2], r7[2])};
        l = l67 & 0xffffu; if (l != NO_PIX) dst[l] = u32x4{lo16(r0[3], r1[3]), lo16(r2[3], r3[3]), lo16(r4[3], r5[3]), lo16(r6[3], r7[3])};
        l = l67 >> 16;     if (l != NO_PIX) dst[l] = u32x4{hi16(r0[3], r1[3]), hi16(r2[3], r3[3]), hi16(r4[3], r5[3]), hi16(r6[3], r7[3])};
    };

    // The weight tile of reduction step st = chunk * KK + tap is [g][Fp] packs, contiguous per g; this
    // thread moves pack (tid / BM, row0 + tid % BM) of each of a group's TG tiles.  Requests are
    // unconditional: steps past the group's (or the reduction's) end repeat a valid tile that nobody reads.
    static_assert(TG <= 9, "named staging registers below");
    u32x4 a0, a1, a2, a3, a4, a5, a6, a7, a8;  // named so that each stays a register
    auto areg = [&](auto q) -> u32x4 & {
        constexpr int Q = decltype(q)::value;
        if constexpr (Q == 0) return a0; else if constexpr (Q == 1) return a1; else if constexpr (Q == 2) return a2;
        else if constexpr (Q == 3) return a3; else if constexpr (Q == 4) return a4; else if constexpr (Q == 5) return a5;
        else if constexpr (Q == 6) return a6; else if constexpr (Q == 7) return a7; else return a8;
    };
    const int KK = g.KK, n_steps = g.n_chunks * KK;
    const bool has_piece = tid < BM * NG;            // a 96-row tile has fewer pieces than threads
    const int wtid = has_piece ? tid : BM * NG - 1;  // the others repeat the last one's (valid) requests
    const u32x4 *wt = reinterpret_cast<const u32x4 *>(Wt) + (row0 + (wtid / BM) * g.Fp + wtid % BM);
    const int step_stride = NG * g.Fp;  // packs from one step's tile to the next
    u32x4 *const at = reinterpret_cast<u32x4 *>(atile) + (wtid / BM) * LA + wtid % BM;
    // Tiles whose pieces are one per thread (BM * NG == NT, BM a multiple of 64) go from global memory straight
    // into LDS: a wavefront's 64 pieces are 64 consecutive packs of one channel pack, in memory and in the tile,
    // so one global-to-LDS load per tap and wavefront (LDS address = a wave-uniform base + lane * 16) replaces a
    // load into registers, the registers themselves and an LDS store.  The loads are asynchronous: they are waited
    // for (memory counter at zero) before the barrier that publishes the buffer.
    constexpr bool DMA = BM * NG == NT && BM % 64 == 0;
    u32x4 *const at_wave = reinterpret_cast<u32x4 *>(atile) + __builtin_amdgcn_readfirstlane((wave * 64 / BM) * LA + (wave * 64) % BM);
    auto issue_a = [&](int st0, int buf) {
        static_for<0, TG>([&](auto q) {
            int st = st0 + decltype(q)::value;
            st = st < n_steps ? st : n_steps - 1;
            if constexpr (DMA)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(wt + st * step_stride),
                                                 (__attribute__((address_space(3))) void *)(at_wave + (buf * TG + decltype(q)::value) * (NG * LA)),
                                                 16, 0, 0);
            else
                areg(q) = wt[st * step_stride];
        });
    };
    auto commit_a = [&](int buf) {
        if constexpr (!DMA)
            if (has_piece)
                static_for<0, TG>([&](auto q) { at[(buf * TG + decltype(q)::value) * (NG * LA)] = areg(q); });
    };
    auto wait_a = [&]() {
        if constexpr (DMA) __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0) only: the tiles are in LDS
    };

    f32x16 acc[TI][TJ];
#pragma unroll
    for (int t = 0; t < TI; ++t)
#pragma unroll
        for (int u = 0; u < TJ; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][u][v] = 0.f;

    // A tap is two slabs of MFMAs (channel packs 0, 1 and 2, 3 of the chunk).  The fragments of a slab are read
    // from LDS one slab ahead, into the other of two register sets, so that a wavefront's LDS latency runs
    // under its own MFMAs and not only under the other wavefront's.
    uint4 fa0[TI], fb0[TJ], fa1[TI], fb1[TJ];
    int pix[TJ];
    auto set_pix = [&](int tapoff) {
#pragma unroll
        for (int u = 0; u < TJ; ++u) pix[u] = swz(pp0[u] + tapoff);
    };
    auto load_frag = [&](uint4 (&fa)[TI], uint4 (&fb)[TJ], int buf, int slot, int s2) {
        const int g2 = 2 * s2 + h;
        const uint4 *pa = atile + (buf * TG + slot) * (NG * LA) + wm * (BM / WM) + li + g2 * LA;
#pragma unroll
        for (int t = 0; t < TI; ++t) fa[t] = pa[32 * t];
#pragma unroll
        for (int u = 0; u < TJ; ++u) fb[u] = patch[g2 * PATCH_PIX + pix[u]];
    };
    auto mma_frag = [&](const uint4 (&fa)[TI], const uint4 (&fb)[TJ]) {
#pragma unroll
        for (int t = 0; t < TI; ++t)
#pragma unroll
            for (int u = 0; u < TJ; ++u) Mma<bf16_t>::run(fa[t], fb[u], acc[t][u]);
    };

    // The first chunk's pixels and weights are requested before the patch is cleared, so that the clearing (the
    // padding stays zero for the whole kernel: loads only ever write real pixels) runs under their latency.
    issue_patch(chunk_lo);
    issue_a(chunk_lo * KK, 0);
    for (int i = tid; i < NG * PATCH_PIX; i += NT) patch[i] = make_uint4(0, 0, 0, 0);
    if constexpr (Epi::HAS_ROW_ADD)
        for (int i = tid; i < BM; i += NT) lds_add[i] = epi.row_add(row0 + i);
    __syncthreads();
    commit_patch();
    commit_a(0);
    wait_a();
    __syncthreads();
    int ky = 0, kx = 0, buf = 0;
    for (int chunk = chunk_lo; chunk < chunk_hi; ++chunk) {
        const bool more_chunks = chunk + 1 < chunk_hi;
        for (int t0 = 0; t0 < KK; t0 += TG) {
            const int nt = KK - t0 < TG ? KK - t0 : TG;
            const bool last_group = t0 + TG >= KK;
            issue_a(chunk * KK + t0 + nt, buf ^ 1);            // the next group (of this chunk or the next)
            if (t0 == 0 && more_chunks) issue_patch(chunk + 1);
            // The next group's weights go to the other buffer (free since the last barrier) before this
            // group's last tap, so that those stores run under the other wavefronts' MFMAs.
            set_pix(ky * g.Wp + kx);
            load_frag(fa0, fb0, buf, 0, 0);
            for (int t = 0; t < nt; ++t) {
                load_frag(fa1, fb1, buf, t, 1);
                if (t == nt - 1) commit_a(buf ^ 1);
                mma_frag(fa0, fb0);
                if (++kx == g.kw) kx = 0, ++ky;
                if (t + 1 < nt) {
                    set_pix(ky * g.Wp + kx);
                    load_frag(fa0, fb0, buf, t + 1, 0);
                }
                mma_frag(fa1, fb1);
            }
            if (last_group) ky = 0;
            if (last_group && more_chunks) {
                __syncthreads();  // every wavefront has read this chunk's pixels
                commit_patch();
            }
            wait_a();
            __syncthreads();      // this group's weights are free, the next group's (and chunk's pixels) are in LDS
            buf ^= 1;
        }
    }

    // every wavefront is past the loop's last barrier: the weight tiles become staging space
    constexpr int STRIP = 16 * staged_pitch(TJ);
    static_assert((NT / 64) * STRIP <= (int)sizeof(atile), "staging strips fit in the weight tiles");
    if constexpr (epilogue_is_masked<Epi>::value) {
        // the patch is free as well: [BM][WN] sums of what each wavefront stored per row, added in wavefront order
        float *wave_sums = reinterpret_cast<float *>(patch);
        static_assert(BM * WN * 4 <= (int)sizeof(patch), "row sums fit in the patch");
        store_tile_staged<TI, TJ, 16>(acc, row0 + wm * (BM / WM), col0 + wn * (BN / WN), lane, z, epi,
                                      reinterpret_cast<char *>(atile) + wave * STRIP, lds_add, row0, wave_sums, WN, wn);
        __syncthreads();
        if (epi.sums != nullptr && tid < BM && row0 + tid < g.F) {
            float total = 0.f;
#pragma unroll
            for (int w = 0; w < WN; ++w) total += wave_sums[tid * WN + w];
            epi.sums[(int64_t)(row0 + tid) * g.tiles_m + tm] = total;
        }
    } else {
        store_tile_staged<TI, TJ, 16>(acc, row0 + wm * (BM / WM), col0 + wn * (BN / WN), lane, z, epi,
                                      reinterpret_cast<char *>(atile) + wave * STRIP, lds_add, row0);
    }
}

// Weights [out][in][kh][kw] (forward) or [in][out][kh][kw] read flipped (data gradient) -> the kernel's
// order [chunk][tap][g][Fp][8]: pack (chunk, tap, g, row) = input channels chunk*32 + 8g .. +7 of output
// channel `row` at window tap `tap`; rows beyond F are zero.  One thread per pack (pack_one, pack_jobs.h); a launch
// carries a table of such jobs, block b belonging to the job whose block range holds it.
__global__ __launch_bounds__(256) void pack_jobs_kernel(PackJobTable t)
{
    int j = 0;
    while (j + 1 < t.n && (int64_t)blockIdx.x >= t.first_block[j + 1]) ++j;
    const int64_t p = ((int64_t)blockIdx.x - t.first_block[j]) * 256 + threadIdx.x;
    if (p < t.job[j].total) pack_one(t.job[j], p);
}

// The convolution as this kernel sees it; for the data gradient the layer's output gradient is the
// input and the window is flipped.
static bool make_fused_geom(const ConvGeom &c, bool data_gradient, Geom *g)
{
    if (c.sh != 1 || c.sw != 1) return false;
    if (!data_gradient) {
        g->N = c.N, g->C = c.C, g->H = c.H, g->W = c.W, g->F = c.F, g->Ho = c.Ho, g->Wo = c.Wo;
        g->ph = c.ph, g->pw = c.pw;
    } else {
        g->N = c.N, g->C = c.F, g->H = c.Ho, g->W = c.Wo, g->F = c.C, g->Ho = c.H, g->Wo = c.W;
        g->ph = c.kh - 1 - c.ph, g->pw = c.kw - 1 - c.pw;
        if (g->ph < 0 || g->pw < 0) return false;
    }
    g->kh = c.kh, g->kw = c.kw;
    g->Wp = g->W + 2 * g->pw;  // replaced below by the pitch chosen with the tile
    g->HW = g->H * g->W, g->HoWo = g->Ho * g->Wo, g->KK = c.kh * c.kw;
    g->sn = (uint32_t)g->C * (uint32_t)g->HW, g->sc = (uint32_t)g->HW;  // dense [N][C][H][W]; launch_fused_conv may replace them
    int64_t M = (int64_t)g->N * g->HoWo;
    if (g->C % CH != 0 || g->HW < 8 || M > 0x7fffffffll - 4096) return false;
    if ((double)g->N * g->C * g->HW * 2.0 >= 4.0e9 || (double)M * g->F * 2.0 >= 4.0e9) return false;
    g->M = (int32_t)M;
    g->n_chunks = g->C / CH;
    g->bm = 128;
    g->Fp = (int32_t)round_up(g->F, 128);
    g->tiles_f = g->Fp / 128;
    g->div_HoWo = FastDiv((uint32_t)g->HoWo);
    g->div_Wo = FastDiv((uint32_t)g->Wo);
    g->div_W = FastDiv((uint32_t)g->W);
    // Every column tile must fit the kernel's fixed LDS patch and its one-task-per-thread loader.
    // (The tiles' positions inside an image repeat with period HoWo / gcd(bn, HoWo).)
    auto fits = [&](int bn, int patch_pix, int pitch) {
        int tiles_m = (g->M + bn - 1) / bn;
        int a = bn, b = g->HoWo;
        while (b != 0) { int t = a % b; a = b, b = t; }
        int period = g->HoWo / a + 1;
        for (int tm = 0; tm < tiles_m && tm < period; ++tm) {
            int col0 = tm * bn, m_last = (col0 + bn < g->M ? col0 + bn : g->M) - 1;
            int n0 = col0 / g->HoWo, n1 = m_last / g->HoWo;
            if (n1 - n0 + 1 > MAX_SLOTS) return false;
            int rows = 0, pieces = 0;
            for (int n = n0; n <= n1; ++n) {
                SlotSpan s = slot_span(*g, col0, m_last, n);
                rows += s.nrows;
                pieces += (s.len + 7) / 8;
            }
            if (rows * pitch > patch_pix || NG * pieces > NT) return false;
        }
        return true;
    };
    // Row pitch of the patch.  A fragment read takes its 64 lanes in four passes of 16 (lanes 0-3, 12-15, 20-27;
    // 4-11, 16-19, 28-31; the same of the upper half), each free of bank conflicts when its 16-byte slots differ
    // mod 16.  A lane's slot is the patch pixel of its output position, so with a pitch that equals the output
    // width mod 16 the slot is (position + constant) mod 16 also across row wraps, and consecutive positions never
    // collide; with the bare padded width every row wrap inside a pass shifts some lanes onto others' banks.
    const int wp_min = g->W + 2 * g->pw;
    int wp_free = wp_min;
    while ((wp_free - g->Wo) % 16 != 0) ++wp_free;
    // Few tiles (small batches): the reduction is cut into ranges of chunks so that about one workgroup per
    // compute unit exists; the ranges' fp32 sums are added in a fixed order afterwards.
    auto splits_for = [&](int64_t n_tiles, int64_t F_rows) {
        int splits = 1;
        if (n_tiles <= 128 && g->n_chunks >= 2 && (double)F_rows * g->M * 4.0 * 16.0 < 4.0e9) {
            int want = (int)(256 / n_tiles);
            splits = want < g->n_chunks ? want : g->n_chunks;
        }
        const int per = (g->n_chunks + splits - 1) / splits;
        return (g->n_chunks + per - 1) / per;
    };
    // Among the tiles that fit, the one with the least estimated time: rounds of the 256 compute units times the
    // tile's width times what a workgroup does per column -- the chunks of the reduction it walks plus its fixed
    // part (prologue and epilogue cost about as much as 14 window taps; a split reduction also writes fp32 partial
    // sums that are added afterwards) -- the narrower tiles a few per cent dearer per column (their weights are
    // staged for fewer columns, and they read more LDS fragments per MFMA).
    auto estimate = [&](int64_t tiles, int bn, double per_column, int64_t F_rows) {
        const int splits = splits_for(tiles, F_rows);
        const int per = (g->n_chunks + splits - 1) / splits;
        const double fixed = 14.0 / g->KK + (splits > 1 ? 0.5 : 0.0);
        return (double)((tiles * splits + 255) / 256) * bn * per_column * (per + fixed);
    };
    const int want = g_fused_bn;  // tuning override: 256, 384 or 512 (0: choose)
    const struct { int bn, patch; double per_column; } tiles[3] = {
        {BN_WIDE, PATCH_WIDE, 1.0}, {BN_MID, PATCH_MID, 1.03}, {BN_NARROW, PATCH_NARROW, 1.06}};
    constexpr double CONFLICTS = 1.15;  // what the bare pitch costs per column (measured on the 27-wide layer)
    double best = 0.0;
    g->bn = 0;
    for (const auto &t : tiles) {
        if (want != 0 && want != t.bn) continue;
        const bool free_fits = !g_fused_bare_pitch && fits(t.bn, t.patch, wp_free);
        if (!free_fits && !fits(t.bn, t.patch, wp_min)) continue;
        const double cost = estimate((int64_t)g->tiles_f * ((g->M + t.bn - 1) / t.bn), t.bn,
                                     t.per_column * (free_fits ? 1.0 : CONFLICTS), g->F);
        if (g->bn == 0 || cost < best) g->bn = t.bn, g->Wp = free_fits ? wp_free : wp_min, best = cost;
    }
    // A layer of at most 64 filters takes a 96-row tile (8 wavefronts of 96 x 64 on 512 columns): three quarters
    // of the MFMAs for a few more fragment reads per MFMA.  (Measured: 48 filters 287 -> 192 us; with 96 filters
    // the two tiles take the same time, the kernel being bound by its LDS reads, so those keep the 128-row tile.)
    const int bm_want = g_fused_bm;  // tuning override: 128 keeps the 128-row tile, 96 forces the other up to 96 filters
    const int f_max = bm_want == 96 ? 96 : 64;
    if (g->F <= f_max && (bm_want == 0 || bm_want == 96) && (want == 0 || want == BN_WIDE)) {
        const bool free_fits = !g_fused_bare_pitch && fits(BN_WIDE, PATCH_WIDE, wp_free);
        if (free_fits || fits(BN_WIDE, PATCH_WIDE, wp_min)) {
            const double cost = estimate((g->M + BN_WIDE - 1) / BN_WIDE, BN_WIDE, 0.8 * (free_fits ? 1.0 : CONFLICTS), g->F);
            if (g->bn == 0 || cost < best)
                g->bn = BN_WIDE, g->bm = 96, g->Fp = 96, g->tiles_f = 1, g->Wp = free_fits ? wp_free : wp_min, best = cost;
        }
    }
    if (g->bn == 0) return false;
    g->tiles_m = (g->M + g->bn - 1) / g->bn;
    const int n_tiles = g->tiles_f * g->tiles_m;
    g->splits = splits_for(n_tiles, g->F);
    g->chunks_per_split = (g->n_chunks + g->splits - 1) / g->splits;
    g->splits = (g->n_chunks + g->chunks_per_split - 1) / g->chunks_per_split;
    g->n_items = n_tiles * g->splits;
    g->per_xcd = (g->n_items + 7) / 8;
    return true;
}

}  // namespace fused

void set_fused_tile_override(int bn, int bm)
{
    if (bn >= 0) fused::g_fused_bn = bn;
    if (bm >= 0) fused::g_fused_bm = bm;
}
void set_fused_pitch_override(int bare) { fused::g_fused_bare_pitch = bare; }

bool fused_supported(const ConvGeom &c, int dtype, bool data_gradient)
{
    fused::Geom g;
    return dtype == OMNI_BF16 && fused::make_fused_geom(c, data_gradient, &g);
}

static size_t fused_packed_bytes(const fused::Geom &g)
{
    return ((size_t)g.n_chunks * g.KK * fused::NG * g.Fp * 16 + 255) / 256 * 256;
}

// the repacked weights, then (split reductions only) the fp32 partial results [splits][F][M]
size_t fused_weight_bytes(const ConvGeom &c, bool data_gradient)
{
    fused::Geom g;
    if (!fused::make_fused_geom(c, data_gradient, &g)) return 0;
    return fused_packed_bytes(g) + (g.splits > 1 ? (size_t)g.splits * g.F * g.M * sizeof(float) : 0);
}

static void fill_fused_job(const fused::Geom &g, bool data_gradient, const void *W, void *packed, PackJob *job)
{
    job->kind = 0;
    job->W = (const bf16_t *)W, job->Wt = (uint4 *)packed;
    job->total = (int64_t)g.n_chunks * g.KK * fused::NG * g.Fp;
    job->F = g.F, job->Fp = g.Fp, job->KK = g.KK, job->n_chunks = g.n_chunks, job->flip = data_gradient ? 1 : 0;
    job->stride_out = data_gradient ? g.KK : (int64_t)g.C * g.KK;
    job->stride_in = data_gradient ? (int64_t)g.F * g.KK : g.KK;
    job->C = job->kh = job->kw = job->kwq = job->groups = job->BM = 0;
}

bool fused_pack_job(const ConvGeom &c, bool data_gradient, const void *W, void *packed, PackJob *job, size_t *bytes)
{
    fused::Geom g;
    *bytes = 0;
    if (!fused::make_fused_geom(c, data_gradient, &g)) return false;
    *bytes = fused_packed_bytes(g);
    if (job != nullptr) fill_fused_job(g, data_gradient, W, packed, job);
    return true;
}

int launch_pack_jobs(const PackJobTable &t, hipStream_t s)
{
    if (t.n <= 0) return OMNI_OK;
    double bytes = 0.0;
    for (int j = 0; j < t.n; ++j) bytes += 2.0 * 16.0 * (double)t.job[j].total;
    ProfScope prof(KID_PACK_KHAT, s, 0.0, bytes);
    hipLaunchKernelGGL(fused::pack_jobs_kernel, dim3((unsigned)t.first_block[t.n]), dim3(256), 0, s, t);
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

int fused_column_tiles(const ConvGeom &c, bool data_gradient)
{
    fused::Geom g;
    if (!fused::make_fused_geom(c, data_gradient, &g) || g.splits > 1) return 0;
    return g.tiles_m;
}

// `prepacked` != null: the repacked weights already exist there (fused_pack_job) and W is not read.
// io (optional): in_ld > 0 = the input is not the dense tensor but its rows form, a matrix [C][in_ld] with image n's
// plane of channel c at column n * (the plane rounded up to 8 elements); mask != null = the output is written in
// the rows form too (leading dimension out_ld), zero where the dense tensor `mask` [N][F][Ho][Wo] is not positive,
// with col_sums [F][fused_column_tiles] (nullable) receiving every column tile's sums of the stored values.
int launch_fused_conv(const ConvGeom &c, bool data_gradient, const void *X, const void *W, const float *bias,
                      int relu, void *Y, void *wt_scratch, hipStream_t s, int kid, const void *prepacked, const FusedIO *io)
{
    using namespace fused;
    Geom g;
    if (!make_fused_geom(c, data_gradient, &g)) return OMNI_UNSUPPORTED;
    const int64_t in_ld = io != nullptr ? io->in_ld : 0;
    const bool masked = io != nullptr && io->mask != nullptr;
    const int64_t out_pitch = ((int64_t)g.HoWo + 7) / 8 * 8;
    if (masked && (in_ld <= 0 || g.splits > 1 || bias != nullptr || relu || io->out_ld < g.N * out_pitch ||
                   (double)io->out_ld * g.F * 2.0 >= 4.0e9))
        return OMNI_UNSUPPORTED;
    if (in_ld > 0) {
        const int64_t pitch = ((int64_t)g.HW + 7) / 8 * 8;
        if (in_ld < g.N * pitch || (double)in_ld * g.C * 2.0 >= 4.0e9) return OMNI_UNSUPPORTED;
        g.sn = (uint32_t)pitch, g.sc = (uint32_t)in_ld;
    }
    if (prepacked == nullptr) {
        PackJobTable t;
        fill_fused_job(g, data_gradient, W, wt_scratch, &t.job[0]);
        t.first_block[0] = 0, t.first_block[1] = (t.job[0].total + 255) / 256, t.n = 1;
        int st = launch_pack_jobs(t, s);
        if (st != OMNI_OK) return st;
    }
    const bf16_t *wt = (const bf16_t *)(prepacked != nullptr ? prepacked : wt_scratch);
    FwdEpilogue<bf16_t> epi{(bf16_t *)Y, bias, g.F, g.M, g.HoWo, g.div_HoWo, relu};
    ProfScope prof(kid >= 0 ? kid : (data_gradient ? KID_FUSED_DGRAD : KID_FUSED_FWD), s, 2.0 * (double)c.M * c.K * c.F, 0.0);
    dim3 grid((unsigned)(g.per_xcd * 8)), block(NT);
    float *partials = reinterpret_cast<float *>(reinterpret_cast<char *>(wt_scratch) + fused_packed_bytes(g));
    PartialEpilogue pe{partials, g.F, g.M};
    RowsMaskEpilogue me{(bf16_t *)Y, masked ? (const bf16_t *)io->mask : nullptr, masked ? io->col_sums : nullptr, g.F, g.M, g.HoWo,
                        g.div_HoWo, (uint32_t)out_pitch, masked ? (uint32_t)io->out_ld : 0u};
#define OMNI_FUSED_LAUNCH_IN(BM_, WM_, WN_, BN_, PATCH_, RIN_)                                                               \
    do {                                                                                                                    \
        if (g.splits > 1)                                                                                                   \
            hipLaunchKernelGGL((fused_conv_kernel<BM_, WM_, WN_, BN_, PATCH_, PartialEpilogue, RIN_>), grid, block, 0, s,    \
                               (const bf16_t *)X, wt, g, pe);                                                               \
        else                                                                                                                \
            hipLaunchKernelGGL((fused_conv_kernel<BM_, WM_, WN_, BN_, PATCH_, FwdEpilogue<bf16_t>, RIN_>), grid, block, 0,  \
                               s, (const bf16_t *)X, wt, g, epi);                                                           \
    } while (0)
#define OMNI_FUSED_LAUNCH(BM_, WM_, WN_, BN_, PATCH_)                                                                       \
    do {                                                                                                                    \
        if (masked)                                                                                                         \
            hipLaunchKernelGGL((fused_conv_kernel<BM_, WM_, WN_, BN_, PATCH_, RowsMaskEpilogue, true>), grid, block, 0, s,   \
                               (const bf16_t *)X, wt, g, me);                                                               \
        else if (in_ld > 0) OMNI_FUSED_LAUNCH_IN(BM_, WM_, WN_, BN_, PATCH_, true);                                         \
        else OMNI_FUSED_LAUNCH_IN(BM_, WM_, WN_, BN_, PATCH_, false);                                                       \
    } while (0)
    if (g.bm == 96) OMNI_FUSED_LAUNCH(96, 1, 8, BN_WIDE, PATCH_WIDE);
    else if (g.bn == BN_WIDE) OMNI_FUSED_LAUNCH(128, 2, 4, BN_WIDE, PATCH_WIDE);
    else if (g.bn == BN_MID) OMNI_FUSED_LAUNCH(128, 2, 4, BN_MID, PATCH_MID);
    else OMNI_FUSED_LAUNCH(128, 2, 4, BN_NARROW, PATCH_NARROW);
#undef OMNI_FUSED_LAUNCH
#undef OMNI_FUSED_LAUNCH_IN
    OMNI_LAUNCH_CHECK();
    if (g.splits > 1) {
        const int64_t count = (int64_t)g.F * g.M;
        hipLaunchKernelGGL((reduce_store_kernel<FwdEpilogue<bf16_t>>), dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s,
                           partials, g.splits, g.F, g.M, epi);
    }
    OMNI_LAUNCH_CHECK();
    return OMNI_OK;
}

}  // namespace omni
