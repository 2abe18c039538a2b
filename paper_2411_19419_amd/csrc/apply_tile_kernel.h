// Tiled SpMM over the stored CSR arrays: x staged in LDS, T streamed once.
//
// The entries of T are 3/4 of all bytes at batch 16 and are used exactly once,
// while every x row is used by about (k/s)^2 rows of T.  So a workgroup takes
// a TH x TW tile of output pixels (TH runs of TW consecutive rows of T),
// copies the input pixels those windows can touch into LDS once, and then
// streams its part of col_idx / vals straight from global memory.
//
// Work mapping inside the tile: G consecutive lanes share one row of T, lane l
// takes entries l, l+G, ...; a wave covers 64/G neighbouring rows per pass, so
// its loads of col_idx and vals sweep one contiguous span.  Each lane keeps
// 4*NV batch columns of partial sums; x is fetched from LDS as NV 16-byte
// reads whose addresses are consecutive across the lanes of a group (entries
// of a row are runs of neighbouring columns).  The G partial sums of a row are
// then combined with a DPP reduce-scatter, after which lane l of the group
// holds the finished columns [l*4*NV/G, (l+1)*4*NV/G) and the wave stores
// 64/G complete, contiguous y rows.
//
// The kernel stays a CSR product: a stored column is located in the LDS tile
// by arithmetic on its value, and a column that falls outside the tile is
// read from global memory instead.
#pragma once
#include "device_util.h"

namespace convspmv {

struct TileGeom {
    int m, n, m_out, n_out, s, p;
    int batch;            // x / y row pitch, in floats
    int th, tw;           // output tile: th lines of tw pixels (tw a multiple of 64/G)
    int tiles_x, tiles_y, n_tiles, tiles_per_xcd;
    int ih, iw;           // input extent a full tile can touch: (th-1)*s+k, (tw-1)*s+k
    int iw_pitch;         // LDS pixels per input line (>= iw)
    int chunk_stride;     // LDS pixels between the planes of successive float4 column chunks (>= ih*iw_pitch)
    float inv_n;          // 1.0f / n
};

constexpr int kXcds = 8;  // MI355X: workgroups are dealt round-robin to 8 XCDs, each with its own L2

// One combining step over lane pairs (l, l ^ mask), acting on the first N
// values of a[].  With N >= 2 it is a reduce-scatter step: the lane whose `hi`
// bit is clear keeps the lower half and adds the partner's lower half, the
// other lane does the same with the upper halves, and N/2 values remain.  With
// N == 1 both lanes end up with the sum.
template <int N, int CTRL, int LEN>
__device__ __forceinline__ void combine_step(float (&a)[LEN], bool hi) {
    if constexpr (N >= 2) {
#pragma unroll
        for (int i = 0; i < N / 2; ++i) {
            const float keep = hi ? a[N / 2 + i] : a[i];
            const float send = hi ? a[i] : a[N / 2 + i];
            a[i] = keep + dpp_move<CTRL>(send);
        }
    } else {
        a[0] += dpp_move<CTRL>(a[0]);
    }
}

constexpr int ilog2(int v) { return v <= 1 ? 0 : 1 + ilog2(v / 2); }
constexpr int imax(int a, int b) { return a > b ? a : b; }

// Non-temporal 4-byte loads for the entry stream (used once, keep it out of
// the way of x in the caches).
__device__ __forceinline__ int stream_load(const int *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ float stream_load(const float *p) { return __builtin_nontemporal_load(p); }

template <int G, int NIT, int NV>
__global__ __launch_bounds__(512) void spmm_tile_kernel(const int *__restrict__ row_ptr,
                                                        const int *__restrict__ col_idx,
                                                        const float *__restrict__ vals,
                                                        const float *__restrict__ x, float *__restrict__ y,
                                                        TileGeom g) {
    constexpr int RW = kWave / G;        // rows per wave pass
    constexpr int NVAL = 4 * NV;         // batch columns per lane
    // The combine runs log2(G) steps; the first SCAT of them halve the value
    // count (reduce-scatter), any left over are plain pair sums.
    constexpr int SCAT = ilog2(G) < ilog2(NVAL) ? ilog2(G) : ilog2(NVAL);
    constexpr int CNT = NVAL >> SCAT;             // finished columns per storing lane
    constexpr int DUP = ilog2(G) - SCAT;          // low lane bits that end up with copies
    static_assert(G == 4 || G == 8 || G == 16, "group width");
    extern __shared__ float4 smem[];
    float4 *xs = smem;
    int *rp_s = reinterpret_cast<int *>(smem + (size_t)NV * g.chunk_stride);

    // ---- which tile (XCD-aware: each XCD walks one contiguous band of tiles)
    const int local = blockIdx.x / kXcds;
    const int tile = (blockIdx.x % kXcds) * g.tiles_per_xcd + local;
    if (tile >= g.n_tiles) return;       // uniform over the block
    const int ty = tile / g.tiles_x, tx = tile - ty * g.tiles_x;
    const int x0 = ty * g.th, y0 = tx * g.tw;
    const int thc = min(g.th, g.m_out - x0), twc = min(g.tw, g.n_out - y0);
    const int c0 = blockIdx.y * NVAL;

    // ---- input window of the tile, clipped to the image
    const int i_lo = g.s * x0 - g.p, j_lo = g.s * y0 - g.p;
    const int i0 = max(i_lo, 0), j0 = max(j_lo, 0);
    const int ihc = max(min(i_lo + g.ih, g.m) - i0, 0);
    const int iwc = max(min(j_lo + g.iw, g.n) - j0, 0);
    const int cbase = i0 * g.n + j0;
    const int nthreads = blockDim.x, tid = threadIdx.x;

    {   // x window -> LDS, plane v holds columns [c0 + 4v, c0 + 4v + 4) of every pixel
        const int items = ihc * iwc * NV;
        const float inv_iwc = 1.0f / (float)max(iwc, 1);
#pragma unroll 4
        for (int item = tid; item < items; item += nthreads) {
            const int q = item / NV, v = item % NV;
            const int di = div_small(q, inv_iwc), dj = q - di * iwc;
            const float4 *src = reinterpret_cast<const float4 *>(
                x + ((long long)(i0 + di) * g.n + (j0 + dj)) * g.batch + c0);
            xs[v * g.chunk_stride + di * g.iw_pitch + dj] = src[v];
        }
        // row_ptr of the tile: tw + 1 values per output line
        const int rp_items = g.th * (g.tw + 1);
        for (int item = tid; item < rp_items; item += nthreads) {
            const int line = item / (g.tw + 1), yy = item - line * (g.tw + 1);
            int v = 0;
            if (line < thc && yy <= twc) v = row_ptr[(long long)(x0 + line) * g.n_out + y0 + yy];
            rp_s[item] = v;
        }
    }
    __syncthreads();

    const int lane = tid % kWave, wave = tid / kWave, nwaves = nthreads / kWave;
    const int gl = lane % G, gr = lane / G;
    const int groups_per_line = g.tw / RW;
    const int npass = g.th * groups_per_line;
    const unsigned lim = (unsigned)(ihc * g.n);      // deltas below this are on a tile line

    int cur_c[NIT], nxt_c[NIT];
    float cur_v[NIT], nxt_v[NIT];
    int beg = 0, end = 0, nbeg = 0, nend = 0;

    auto bounds = [&](int pid, int &b, int &e) {
        const int line = pid / groups_per_line, yy = (pid - line * groups_per_line) * RW + gr;
        b = e = 0;
        if (line < thc && yy < twc) {
            b = rp_s[line * (g.tw + 1) + yy];
            e = rp_s[line * (g.tw + 1) + yy + 1];
        }
    };
    auto fetch = [&](int b, int e, int (&c)[NIT], float (&v)[NIT]) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int idx = b + gl + it * G;
            c[it] = 0;
            v[it] = 0.0f;
            if (idx < e) {
                c[it] = stream_load(col_idx + idx);
                v[it] = stream_load(vals + idx);
            }
        }
    };

    int pid = wave;
    if (pid < npass) {
        bounds(pid, beg, end);
        fetch(beg, end, cur_c, cur_v);
    }
    for (; pid < npass; pid += nwaves) {
        const int npid = pid + nwaves;
        if (npid < npass) {              // uniform over the wave
            bounds(npid, nbeg, nend);
            fetch(nbeg, nend, nxt_c, nxt_v);
        }

        float acc[NVAL];
#pragma unroll
        for (int i = 0; i < NVAL; ++i) acc[i] = 0.0f;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            if (beg + gl + it * G < end) {
                const int col = cur_c[it];
                const float w = cur_v[it];
                const int delta = col - cbase;
                const int di = div_small(delta, g.inv_n);
                const int dj = delta - di * g.n;
                float4 xv[NV];
                if ((unsigned)delta < lim && (unsigned)dj < (unsigned)iwc) {
                    const float4 *src = xs + (di * g.iw_pitch + dj);
#pragma unroll
                    for (int v = 0; v < NV; ++v) xv[v] = src[v * g.chunk_stride];
                } else {                 // stored column outside the staged window
                    const float4 *src = reinterpret_cast<const float4 *>(x + (long long)col * g.batch + c0);
#pragma unroll
                    for (int v = 0; v < NV; ++v) xv[v] = src[v];
                }
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    acc[4 * v + 0] = fmaf(w, xv[v].x, acc[4 * v + 0]);
                    acc[4 * v + 1] = fmaf(w, xv[v].y, acc[4 * v + 1]);
                    acc[4 * v + 2] = fmaf(w, xv[v].z, acc[4 * v + 2]);
                    acc[4 * v + 3] = fmaf(w, xv[v].w, acc[4 * v + 3]);
                }
            }
        }

        // ---- combine the G partial sums of each row; all 64 lanes are active here
        if constexpr (G == 16) {
            combine_step<NVAL, kDppXor15>(acc, (gl & 8) != 0);
            combine_step<imax(NVAL / 2, 1), kDppXor7>(acc, (gl & 4) != 0);
            combine_step<imax(NVAL / 4, 1), kDppXor2>(acc, (gl & 2) != 0);
            combine_step<imax(NVAL / 8, 1), kDppXor1>(acc, (gl & 1) != 0);
        } else if constexpr (G == 8) {
            combine_step<NVAL, kDppXor7>(acc, (gl & 4) != 0);
            combine_step<imax(NVAL / 2, 1), kDppXor2>(acc, (gl & 2) != 0);
            combine_step<imax(NVAL / 4, 1), kDppXor1>(acc, (gl & 1) != 0);
        } else {
            combine_step<NVAL, kDppXor2>(acc, (gl & 2) != 0);
            combine_step<imax(NVAL / 2, 1), kDppXor1>(acc, (gl & 1) != 0);
        }

        {   // lanes whose DUP low bits are clear hold CNT finished columns of their row,
            // starting at column (gl >> DUP) * CNT of this launch's column block
            const int line = pid / groups_per_line, yy = (pid - line * groups_per_line) * RW + gr;
            if (line < thc && yy < twc && (gl & ((1 << DUP) - 1)) == 0) {
                float *dst = y + ((long long)(x0 + line) * g.n_out + (y0 + yy)) * g.batch + c0 + (gl >> DUP) * CNT;
                if constexpr (CNT == 1) {
                    dst[0] = acc[0];
                } else if constexpr (CNT == 2) {
                    *reinterpret_cast<float2 *>(dst) = make_float2(acc[0], acc[1]);
                } else {
#pragma unroll
                    for (int i = 0; i < CNT; i += 4)
                        *reinterpret_cast<float4 *>(dst + i) = make_float4(acc[i], acc[i + 1], acc[i + 2], acc[i + 3]);
                }
            }
        }

        beg = nbeg;
        end = nend;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            cur_c[it] = nxt_c[it];
            cur_v[it] = nxt_v[it];
        }
    }
}

}  // namespace convspmv
