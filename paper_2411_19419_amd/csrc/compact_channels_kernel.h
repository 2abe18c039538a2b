// Sum over input channels from the structure-aware storage, in one launch (gfx950).
//
// A convolution layer adds the products of all its input channels: y = sum_c T_c x_c, every
// T_c with the row descriptors of Section 2 / Theorem 2.1 and its own k*k table.  One launch
// per channel (each adding to y) is bound by launches and by re-reading y when the planes are
// small and the channels many.  Here a wave keeps the sums of a 4 x 16 tile of outputs, VB
// batch columns each, in registers while it walks the channels:
//   - the W = 4, 8 or 16 waves of a workgroup share the tile and split the channels (wave w
//     takes channels w, w + W, ...); at the end their partial sums are added in wave order, so
//     the summation order is fixed;
//   - per channel a wave copies the (3 s + k) x (15 s + k) input pixels its tile touches, zero outside
//     the image, into LDS of its own (no workgroup barrier inside the walk: the LDS
//     instructions of a wave execute in order), then every lane adds the k x k taps of its
//     output over that padded patch, while the next channel's pixels are on their way from
//     memory to registers;
//   - this full k x k sum is a row's sum only when the row is described exactly as Theorem 2.1
//     says the window at its position must be.  A wave checks that on the descriptors it read;
//     if one differs (an edited descriptor), the whole wave walks the rectangles its
//     descriptors describe instead, reading x from global memory.
#pragma once
#include "compact_kernels.h"

namespace convspmv {

constexpr int kChanTileX = 4;         // output lines and
constexpr int kChanTileY = 16;        // output columns of a tile; 64 lanes = one tile
constexpr int kChanMinWaves = 4;      // waves per workgroup = ways the channels are split: 4, 8 or 16
constexpr int kChanItems = 16;        // float4 of a patch per lane, at most (16 KiB of patch per wave)
// Most waves per workgroup: a lane that carries more than 8 patch items needs more than the 128
// registers a thread of a 1024-thread workgroup can have.
constexpr int chan_max_waves(int items_per_lane) { return items_per_lane <= 8 ? 16 : 8; }

struct CompactChannelsGeom {
    int m, n, m_out, n_out, s, p, k;
    int batch, channels;
    int tiles_y;          // tiles per line of tiles
    int tiles, tiles_per_xcd;
    int phx, phy;         // patch lines, pixels per patch line: 3 s + k, 15 s + k
    int wave_vec4;        // float4 of LDS per wave: patch (or one partial sum per lane) + the channel's table
    float inv_phy;
    long long plane;      // floats per channel of x: m * n * batch
};

// The descriptor Theorem 2.1 gives row (x, y); {0, 0} for a row without entries.
__device__ __forceinline__ int2 described_by_position(int m, int n, int k, int s, int p, int x, int y) {
    const int r1 = axis_taps(x, m, k, s, p), r2 = axis_taps(y, n, k, s, p);
    int2 d = make_int2(0, 0);
    if (r1 > 0 && r2 > 0) {
        const long long sx = (long long)s * x, sy = (long long)s * y;
        const int a_lo = p > sx ? (int)(p - sx) : 0, b_lo = p > sy ? (int)(p - sy) : 0;
        d.x = (int)((sx + a_lo - p) * n + (sy + b_lo - p));
        d.y = (int)((unsigned)a_lo | (unsigned)r1 << 8 | (unsigned)b_lo << 16 | (unsigned)r2 << 24);
    }
    return d;
}

// VB batch columns per lane; NI float4 of a patch per lane (at least (3 s + k)(15 s + k) VB / 256); KK: the
// kernel size the tap loops are unrolled for, with the channel's table in scalar registers (0: any
// k, table in LDS).
template <int VB, int NI, int KK>
__global__ __launch_bounds__(chan_max_waves(NI) * kWave) void spmm_compact_channels_kernel(
    const int2 *__restrict__ desc, const float *__restrict__ ktab, const float *__restrict__ x, float *__restrict__ y,
    const CompactChannelsGeom g) {
    static_assert(VB == 4 || VB == 8 || VB == 16, "batch columns per lane");
    static_assert(NI >= 1 && NI <= kChanItems, "patch items per lane");
    constexpr int Q = VB / 4;
    extern __shared__ float4 chan_lds[];
    const int tid = (int)threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave), lane = tid % kWave;
    const int ways = (int)blockDim.x / kWave;
    float4 *const patch = chan_lds + wave * g.wave_vec4;
    float *const table = reinterpret_cast<float *>(patch + max(g.phx * g.phy, kWave) * Q);
    // consecutive workgroups go to different XCDs; a band of neighbouring tiles to one, so that the pixels
    // two tiles share are fetched into one L2
    const int tile = ((int)blockIdx.x % kXcds) * g.tiles_per_xcd + (int)blockIdx.x / kXcds;
    if ((int)blockIdx.x / kXcds >= g.tiles_per_xcd || tile >= g.tiles) return;      // uniform over the workgroup
    const int tile_x = tile / g.tiles_y, tile_y = tile - tile_x * g.tiles_y;
    const int lx = lane / kChanTileY, ly = lane % kChanTileY;
    const int ox = tile_x * kChanTileX + lx, oy = tile_y * kChanTileY + ly;
    const bool live = ox < g.m_out && oy < g.n_out;
    const long long row = (long long)ox * g.n_out + oy;
    const int c0 = (int)blockIdx.y * VB;
    const int kk = g.k * g.k;

    const int2 d = live ? desc[row] : make_int2(0, 0);
    const int2 want = described_by_position(g.m, g.n, g.k, g.s, g.p, ox, oy);
    const bool as_expected = __builtin_amdgcn_ballot_w64(live && (d.x != want.x || d.y != want.y)) == 0;

    float4 acc[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) acc[q] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    auto fma4 = [](float4 &a, float w, const float4 &e) {
        a.x = fmaf(w, e.x, a.x);
        a.y = fmaf(w, e.y, a.y);
        a.z = fmaf(w, e.z, a.z);
        a.w = fmaf(w, e.w, a.w);
    };

    if (as_expected) {
        const int i_lo = g.s * tile_x * kChanTileX - g.p, j_lo = g.s * tile_y * kChanTileY - g.p;   // patch origin
        const int items = g.phx * g.phy * Q;         // float4 of a patch; at most NI * 64
        // where this lane's items lie in a channel's plane (floats; -1: outside the image, a zero)
        int at[NI];
#pragma unroll
        for (int u = 0; u < NI; ++u) {
            const int it = min(u * kWave + lane, items - 1);
            const int pix = it / Q, q = it % Q;
            const int pi = div_small(pix, g.inv_phy), pj = pix - pi * g.phy;
            const int i = i_lo + pi, j = j_lo + pj;
            at[u] = i >= 0 && i < g.m && j >= 0 && j < g.n ? (i * g.n + j) * g.batch + 4 * q : -1;
        }
        // the next channel's patch travels from memory to registers while this channel's taps are summed
        float4 next[NI];
        auto ask = [&](int c) {
            const float *xc = x + min(c, g.channels - 1) * g.plane + c0;      // past the last channel: loaded, never used
#pragma unroll
            for (int u = 0; u < NI; ++u)
                if (u * kWave < items) next[u] = *reinterpret_cast<const float4 *>(xc + max(at[u], 0));
        };
        // The patch is kept as Q planes of one float4 per pixel: neighbouring lanes then read neighbouring
        // 16-byte words (pixel-major with 64 bytes per pixel, 16 lanes met in 4 banks).
        const int npix = g.phx * g.phy;
        const float4 *const mine = patch + lx * g.s * g.phy + ly * g.s;     // this lane's window in plane 0
        ask(wave);
        for (int c = wave; c < g.channels; c += ways) {
#pragma unroll
            for (int u = 0; u < NI; ++u)
                if (u * kWave < items && u * kWave + lane < items) {
                    const int it = u * kWave + lane;
                    patch[(it % Q) * npix + it / Q] = at[u] >= 0 ? next[u] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                }
            if constexpr (KK > 0) {
                float w[KK * KK];               // the same for every lane: scalar loads, scalar operands
                const float *tc = ktab + (long long)c * (KK * KK);
#pragma unroll
                for (int t = 0; t < KK * KK; ++t) w[t] = tc[t];
                ask(c + ways);
                wave_lds_order();
#pragma unroll
                for (int a = 0; a < KK; ++a) {
                    const float4 *line = mine + a * g.phy;
#pragma unroll
                    for (int b = 0; b < KK; ++b) {
#pragma unroll
                        for (int q = 0; q < Q; ++q) fma4(acc[q], w[a * KK + b], line[q * npix + b]);
                    }
                }
            } else {
                for (int t = lane; t < kk; t += kWave) table[t] = ktab[(long long)c * kk + t];
                ask(c + ways);
                wave_lds_order();
                for (int a = 0; a < g.k; ++a) {
                    const float4 *line = mine + a * g.phy;
                    const float *tl = table + a * g.k;
                    for (int b = 0; b < g.k; ++b) {
                        const float w = tl[b];
#pragma unroll
                        for (int q = 0; q < Q; ++q) fma4(acc[q], w, line[q * npix + b]);
                    }
                }
            }
            wave_lds_order();
        }
    } else if (live) {
        const unsigned w = (unsigned)d.y;
        const int a_lo = w & 255u, r1 = (w >> 8) & 255u, b_lo = (w >> 16) & 255u, r2 = w >> 24;
        for (int c = wave; c < g.channels; c += ways) {
            const float *xc = x + c * g.plane + c0;
            const float *tc = ktab + (long long)c * kk;
            for (int da = 0; da < r1; ++da)
                for (int db = 0; db < r2; ++db) {
                    const float wt = tc[(a_lo + da) * g.k + b_lo + db];
                    const float4 *e = reinterpret_cast<const float4 *>(xc + ((long long)d.x + (long long)da * g.n + db) * g.batch);
#pragma unroll
                    for (int q = 0; q < Q; ++q) fma4(acc[q], wt, e[q]);
                }
        }
    }
    // partial sums of the waves, added in wave order
    wave_lds_order();
#pragma unroll
    for (int q = 0; q < Q; ++q) patch[lane * Q + q] = acc[q];
    __syncthreads();
    if (wave == 0 && live) {
        float4 *out = reinterpret_cast<float4 *>(y + row * g.batch + c0);
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            float4 sum = chan_lds[lane * Q + q];
            for (int wv = 1; wv < ways; ++wv) {
                const float4 e = chan_lds[wv * g.wave_vec4 + lane * Q + q];
                sum.x += e.x;
                sum.y += e.y;
                sum.z += e.z;
                sum.w += e.w;
            }
            out[q] = sum;
        }
    }
}

}  // namespace convspmv
