// Weight repacking jobs of the fused kernels, so that one launch can repack the weights of many layers and passes
// (omni_conv_pack_weights).  Device code and the job record; not part of the C ABI.
#pragma once

#include "common.h"

namespace omni {

// One layer-and-pass's repacking: `total` 16-byte packs written to Wt, pack p by pack_one(job, p).
struct PackJob {
    int32_t kind;            // 0: fused stride-1 convolution (forward or data gradient), 1: stride-4 forward
    const bf16_t *W;         // [F][C][kh][kw]
    uint4 *Wt;
    int64_t total;
    // kind 0: [chunk][tap][g][Fp][8], see pack_weights_kernel in implicit.hip
    int32_t F, Fp, KK, n_chunks, flip;
    int64_t stride_out, stride_in;
    // kind 1: [pack][row (BM)] of window-column groups, see strided.hip
    int32_t C, kh, kw, kwq, groups, BM;
};

constexpr int MAX_PACK_JOBS = 16;
struct PackJobTable {
    PackJob job[MAX_PACK_JOBS];
    int64_t first_block[MAX_PACK_JOBS + 1];  // job j owns blocks [first_block[j], first_block[j + 1]) of 256 packs
    int32_t n;
};

__device__ __forceinline__ void pack_one(const PackJob &j, int64_t p)
{
    uint32_t v[8];
    if (j.kind == 0) {
        // pack (chunk, tap, g, row) = input channels chunk*32 + 8g .. +7 of output channel `row` at window tap `tap`.
        // Forward weights: a row's 8 channels x KK taps are contiguous in W, so the threads of a group of 4 rows x KK
        // taps share the lines they read (thread order: row % 4 fastest, then tap, then the other row bits) and
        // still write whole 64-byte lines; data-gradient weights are read with the row fastest as they are written
        // (consecutive rows are KK elements apart in W there).
        int row, gq, tap, chunk;
        if (j.flip) {
            row = (int)(p % j.Fp);
            int64_t t = p / j.Fp;
            gq = (int)(t % 4);
            t /= 4;
            tap = (int)(t % j.KK), chunk = (int)(t / j.KK);
        } else {
            const int row_lo = (int)(p % 4);
            int64_t t = p / 4;
            tap = (int)(t % j.KK);
            t /= j.KK;
            const int quads = j.Fp / 4;
            row = (int)(t % quads) * 4 + row_lo;
            t /= quads;
            gq = (int)(t % 4), chunk = (int)(t / 4);
            p = (((int64_t)chunk * j.KK + tap) * 4 + gq) * j.Fp + row;
        }
        const int src_tap = j.flip ? j.KK - 1 - tap : tap;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int c = chunk * 32 + gq * 8 + e;
            v[e] = row < j.F ? (uint32_t)j.W[row * j.stride_out + c * j.stride_in + src_tap] : 0u;
        }
    } else {
        // pack p holds groups 2p and 2p + 1, group (c, ky, kq) the window columns 4 kq .. 4 kq + 3
        const int pk = (int)(p / j.BM), f = (int)(p - (int64_t)pk * j.BM);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int gi = 2 * pk + e / 4, i = e % 4;
            v[e] = 0u;
            if (gi < j.groups && f < j.F) {
                const int c = gi / (j.kh * j.kwq), rem = gi - c * (j.kh * j.kwq);
                const int ky = rem / j.kwq, kq = rem - ky * j.kwq;
                const int kx = 4 * kq + i;
                if (kx < j.kw) v[e] = (uint32_t)j.W[((f * j.C + c) * j.kh + ky) * j.kw + kx];
            }
        }
    }
    j.Wt[p] = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
}

// implicit.hip / strided.hip: the job that writes what launch_fused_conv / launch_strided_conv read as their
// repacked weights, and its size in bytes (0 with `false`: the layer and pass do not take that kernel)
bool fused_pack_job(const ConvGeom &g, bool data_gradient, const void *W, void *packed, PackJob *job, size_t *bytes);
bool strided_pack_job(const ConvGeom &g, const void *W, void *packed, PackJob *job, size_t *bytes);
// implicit.hip: all jobs of the table in one launch
int launch_pack_jobs(const PackJobTable &t, hipStream_t s);

}  // namespace omni
