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
// The entry loads of pass i+1 are issued before the arithmetic of pass i
// (two register sets used alternately), and the arithmetic of a pass is one
// straight-line block: a lane whose slot is past the end of its row, or whose
// stored column is not in the staged window, reads a zero pixel kept in LDS
// with weight 0.  The kernel stays a CSR product: a stored column is located
// in the LDS tile by arithmetic on its value, and any column that falls
// outside the tile is picked up afterwards from global memory.
#pragma once
#include "device_util.h"

namespace convspmv {

struct TileGeom {
    int m, n, m_out, n_out, s, p;
    int batch;            // x / y row pitch, in floats
    int nnz;
    int th;               // output lines per tile (pixels per line: template TW)
    int tiles_x, tiles_y, n_tiles, tiles_per_xcd;
    int ih, iw;           // input extent a full tile can touch: (th-1)*s+k, (TW-1)*s+k
    int iw_pitch;         // LDS pixels per input line (>= iw); ih*iw_pitch < CS (template)
    float inv_n;          // 1.0f / n
    int accum;            // 1: add to y instead of storing
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

// 4-byte loads of the entry stream; base is wave-uniform, off a byte offset.
// Plain (temporal) loads on purpose: a group reads 32-byte pieces, so each
// 128-byte line is touched by four consecutive loads of the same wave and has
// to stay in the vector L1 between them.  With non-temporal loads every touch
// became its own L2 request (measured: 85 % of L1 accesses went to L2 and the
// kernel took 1.65x longer).
__device__ __forceinline__ int stream_load_i(const int *base, unsigned off) {
    return *reinterpret_cast<const int *>(reinterpret_cast<const char *>(base) + off);
}
__device__ __forceinline__ float stream_load_f(const float *base, unsigned off) {
    return *reinterpret_cast<const float *>(reinterpret_cast<const char *>(base) + off);
}

// Store CNT (1, 2 or a multiple of 4) finished columns of one y row.  y is
// written once and not read again by this kernel: non-temporal stores, which
// on this part cost about a quarter less time than plain ones next to the
// entry stream (measured with a traffic-only probe: 67 MB of y add 22 us
// instead of 30 us to a 66 us read stream).
//
// accum: add to y instead (one hardware float add per element, no return value, so the wave
// does not wait for it).  Used for the second and later channels of a multi-channel sum, one
// launch per channel on one stream: every element of y then receives exactly one add per
// launch, in launch order, and the result does not depend on timing.
template <int CNT, int LEN>
__device__ __forceinline__ void store_row(float *dst, const float (&a)[LEN], bool accum = false) {
    typedef float vec2 __attribute__((ext_vector_type(2)));
    typedef float vec4 __attribute__((ext_vector_type(4)));
    if (accum) {
#pragma unroll
        for (int i = 0; i < CNT; ++i) unsafeAtomicAdd(dst + i, a[i]);
        return;
    }
    if constexpr (CNT == 1) {
        __builtin_nontemporal_store(a[0], dst);
    } else if constexpr (CNT == 2) {
        vec2 t;
        t.x = a[0];
        t.y = a[1];
        __builtin_nontemporal_store(t, reinterpret_cast<vec2 *>(dst));
    } else {
#pragma unroll
        for (int i = 0; i < CNT; i += 4) {
            vec4 t;
            t.x = a[i];
            t.y = a[i + 1];
            t.z = a[i + 2];
            t.w = a[i + 3];
            __builtin_nontemporal_store(t, reinterpret_cast<vec4 *>(dst + i));
        }
    }
}

// CS: LDS pixels per plane (one plane per float4 column chunk), a compile-time
// constant so that the NV reads of a pixel differ only by an immediate offset.
template <int G, int NIT, int NV, int TW, int CS>
__global__ __launch_bounds__(TW * 8) void spmm_tile_kernel(const int *__restrict__ row_ptr,
                                                           const int *__restrict__ col_idx,
                                                           const float *__restrict__ vals,
                                                           const float *__restrict__ x, float *__restrict__ y,
                                                           TileGeom g) {
    constexpr int RW = kWave / G;        // rows per wave pass
    constexpr int GPL = TW / RW;         // wave passes per output line of the tile
    constexpr int NVAL = 4 * NV;         // batch columns per lane
    // The combine runs log2(G) steps; the first SCAT of them halve the value
    // count (reduce-scatter), any left over are plain pair sums.
    constexpr int SCAT = ilog2(G) < ilog2(NVAL) ? ilog2(G) : ilog2(NVAL);
    constexpr int CNT = NVAL >> SCAT;             // finished columns per storing lane
    constexpr int DUP = ilog2(G) - SCAT;          // low lane bits that end up with copies
    static_assert(G == 2 || G == 4 || G == 8 || G == 16, "group width");
    static_assert(TW % RW == 0, "a wave pass must not straddle two output lines");
    extern __shared__ float4 smem[];
    float4 *xs = smem;
    int *rp_s = reinterpret_cast<int *>(smem + (size_t)NV * CS);

    // ---- which tile (XCD-aware: each XCD walks one contiguous band of tiles)
    const int local = blockIdx.x / kXcds;
    const int tile = (blockIdx.x % kXcds) * g.tiles_per_xcd + local;
    if (tile >= g.n_tiles) return;       // uniform over the block
    const int ty = tile / g.tiles_x, tx = tile - ty * g.tiles_x;
    const int x0 = ty * g.th, y0 = tx * TW;
    const int thc = min(g.th, g.m_out - x0), twc = min(TW, g.n_out - y0);
    const int c0 = blockIdx.y * NVAL;

    // ---- input window of the tile, clipped to the image
    const int i_lo = g.s * x0 - g.p, j_lo = g.s * y0 - g.p;
    const int i0 = max(i_lo, 0), j0 = max(j_lo, 0);
    const int ihc = max(min(i_lo + g.ih, g.m) - i0, 0);
    const int iwc = max(min(j_lo + g.iw, g.n) - j0, 0);
    const int cbase = i0 * g.n + j0;
    const int zslot = g.ih * g.iw_pitch;          // a pixel of zeros in every plane
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
            xs[v * CS + di * g.iw_pitch + dj] = src[v];
        }
        if (tid < NV) xs[tid * CS + zslot] = make_float4(0.f, 0.f, 0.f, 0.f);
        // row_ptr of the tile: TW + 1 values per output line
        const int rp_items = g.th * (TW + 1);
        for (int item = tid; item < rp_items; item += nthreads) {
            const int line = item / (TW + 1), yy = item - line * (TW + 1);
            int v = 0;
            if (line < thc && yy <= twc) v = row_ptr[(long long)(x0 + line) * g.n_out + y0 + yy];
            rp_s[item] = v;
        }
    }
    __syncthreads();

    const int lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int gl = lane % G, gr = lane / G;
    // Window geometry in LDS bytes (16 per pixel).  The host guarantees
    // m*n <= 2^27 (so col*16 fits an int), n < 2^20 and ih*n < 2^21 (so that
    // d16 < 2^25 is a multiple of 16, exact in fp32, and the quotient by n comes
    // out exact from one fused multiply-add and a truncation).
    const int cbase16 = cbase * 16, n16 = g.n * 16, pitch16 = g.iw_pitch * 16, zslot16 = zslot * 16;
    const unsigned lim16 = (unsigned)(ihc * g.n) * 16u, iwc16 = (unsigned)iwc * 16u;
    const float inv_n16 = g.inv_n * 0.0625f, half_inv_n = 0.5f * g.inv_n;

    struct Pass {
        int c[NIT];
        float v[NIT];
        int beg, end;
    };

    // Row bounds of this lane's row in pass pid and the entry loads for it.
    auto fetch = [&](int pid, Pass &ps) {
        const int line = pid / GPL, yy0 = (pid % GPL) * RW;          // wave-uniform
        const int yy = yy0 + gr;
        const int *rp_line = rp_s + line * (TW + 1);
        ps.beg = ps.end = 0;
        if (line < thc && yy < twc) {
            ps.beg = rp_line[yy];
            ps.end = rp_line[yy + 1];
        }
        // wave-uniform base: first entry of the tile line; lane offsets from it stay small
        const int line_base = __builtin_amdgcn_readfirstlane(rp_line[0]);
        const int span_end = __builtin_amdgcn_readfirstlane(rp_line[min(yy0 + RW, twc)]);
        const int *cb = col_idx + line_base;
        const float *vb = vals + line_base;
        const unsigned off = (unsigned)(max(ps.beg - line_base, 0) + gl) * 4u;
        // Both branches issue exactly 2*NIT loads and contain no lane-dependent
        // control flow, so the number of loads in flight is the same on every
        // path and later waits can leave the newest pass outstanding.
        if (line < thc && (long long)span_end + NIT * G <= g.nnz) {
            // every slot of every lane lies inside the arrays: slots past the end of
            // a row fetch entries of later rows, which the arithmetic ignores
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                ps.c[it] = stream_load_i(cb, off + it * G * 4);
                ps.v[it] = stream_load_f(vb, off + it * G * 4);
            }
        } else {
            // the last rows of T (or a tile line below the image): clamp to the last entry
            const unsigned last = (unsigned)(g.nnz - 1 - line_base) * 4u;
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const unsigned o = min(off + it * G * 4, last);
                ps.c[it] = stream_load_i(cb, o);
                ps.v[it] = stream_load_f(vb, o);
            }
        }
    };

    auto compute = [&](int pid, const Pass &ps) {
        float acc[NVAL];
#pragma unroll
        for (int i = 0; i < NVAL; ++i) acc[i] = 0.0f;
        bool stray = false;              // an in-row entry whose column is outside the window
        const int rem = ps.end - ps.beg - gl;     // slot it belongs to the row iff it*G < rem
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            // All offsets in bytes of LDS (16 per pixel): d16 = 16 * (col - first column of the
            // window) = 16 * (di * n + dj) for a column on window line di at window pixel dj.
            const bool act = it * G < rem;
            const int d16 = (ps.c[it] << 4) - cbase16;
            const int di = (int)fmaf((float)d16, inv_n16, half_inv_n);
            const int dj16 = d16 - __mul24(di, n16);
            const bool in = (unsigned)d16 < lim16 && (unsigned)dj16 < iwc16;
            stray |= act && !in;
            const int addr = (act && in) ? __mul24(di, pitch16) + dj16 : zslot16;
            const float w = (act && in) ? ps.v[it] : 0.0f;
            const float4 *src = reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(xs) + addr);
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const float4 xv = src[v * CS];
                acc[4 * v + 0] = fmaf(w, xv.x, acc[4 * v + 0]);
                acc[4 * v + 1] = fmaf(w, xv.y, acc[4 * v + 1]);
                acc[4 * v + 2] = fmaf(w, xv.z, acc[4 * v + 2]);
                acc[4 * v + 3] = fmaf(w, xv.w, acc[4 * v + 3]);
            }
        }
        if (__builtin_expect(__any(stray), 0)) {
            // cold: some stored column is not in the staged window; take those from global memory
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const bool act = it * G < rem;
                const int d16 = (ps.c[it] << 4) - cbase16;
                const int di = (int)fmaf((float)d16, inv_n16, half_inv_n);
                const int dj16 = d16 - __mul24(di, n16);
                const bool in = (unsigned)d16 < lim16 && (unsigned)dj16 < iwc16;
                if (act && !in) {
                    const float4 *src = reinterpret_cast<const float4 *>(x + (long long)ps.c[it] * g.batch + c0);
                    const float w = ps.v[it];
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        const float4 xv = src[v];
                        acc[4 * v + 0] = fmaf(w, xv.x, acc[4 * v + 0]);
                        acc[4 * v + 1] = fmaf(w, xv.y, acc[4 * v + 1]);
                        acc[4 * v + 2] = fmaf(w, xv.z, acc[4 * v + 2]);
                        acc[4 * v + 3] = fmaf(w, xv.w, acc[4 * v + 3]);
                    }
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
        } else if constexpr (G == 4) {
            combine_step<NVAL, kDppXor2>(acc, (gl & 2) != 0);
            combine_step<imax(NVAL / 2, 1), kDppXor1>(acc, (gl & 1) != 0);
        } else {
            combine_step<NVAL, kDppXor1>(acc, (gl & 1) != 0);
        }

        // lanes whose DUP low bits are clear hold CNT finished columns of their row,
        // starting at column (gl >> DUP) * CNT of this launch's column block
        const int line = pid / GPL, yy = (pid % GPL) * RW + gr;
        if (line < thc && yy < twc && (gl & ((1 << DUP) - 1)) == 0) {
            float *dst = y + ((long long)(x0 + line) * g.n_out + (y0 + yy)) * g.batch + c0 + (gl >> DUP) * CNT;
            store_row<CNT>(dst, acc, g.accum != 0);
        }
    };

    // ---- the passes of the tile (GPL per output line, line after line) are dealt to the waves
    // of the block in turn: wave w takes passes w, w + W, w + 2 W, ...  Two register sets
    // alternate so that the loads of the next pass are in flight during the arithmetic of this
    // one; the steady-state loop fetches unconditionally (fetch clamps what lies past the tile).
    const int nwaves = nthreads / kWave;
    const int total = g.th * GPL;
    if (wave >= total) return;
    const int mine = (total - wave + nwaves - 1) / nwaves;       // passes of this wave
    Pass pa, pb;
    fetch(wave, pa);
    int i = 0;
    for (; i + 2 < mine; i += 2) {
        fetch(wave + (i + 1) * nwaves, pb);
        compute(wave + i * nwaves, pa);
        fetch(wave + (i + 2) * nwaves, pa);
        compute(wave + (i + 1) * nwaves, pb);
    }
    if (mine - i == 2) {
        fetch(wave + (i + 1) * nwaves, pb);
        compute(wave + i * nwaves, pa);
        compute(wave + (i + 1) * nwaves, pb);
    } else {
        compute(wave + i * nwaves, pa);
    }
}

}  // namespace convspmv
