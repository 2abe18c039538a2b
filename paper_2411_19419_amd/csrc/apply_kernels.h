// y = T x over the stored CSR arrays (gfx950): SpMV for one vector, SpMM for a
// batch of vectors that share T (Section 3, the convolution procedure; the
// batch is the paper's "batched contexts" outlook, Section 4.2).
//
// All kernels read row_ptr, col_idx and vals as stored; nothing about the
// convolution is assumed beyond "a row has at most k*k entries".
#pragma once
#include "device_util.h"

namespace convspmv {

// ---------------------------------------------------------------------------
// Row-group kernel, x gathered straight from global memory.
//
// G consecutive lanes share one row: lane l takes entries l, l+G, l+2G, ... so
// a group reads G consecutive (col, val) pairs per step and a wave reads 64/G
// neighbouring rows, which are adjacent in the entry arrays.  Each lane
// carries C batch columns (C = 1 scalar, or 4*NV as NV float4 when the batch
// is a multiple of 4, which also makes every x and y row 16-byte aligned);
// blockIdx.y walks the batch in steps of C.  The partial sums are combined
// with DPP butterflies and lane 0 of the group stores the row.
// ---------------------------------------------------------------------------
constexpr int kGatherThreads = 256;

// Several input channels that share one index structure (the sum over channels of T_ch x_ch,
// the multi-channel context of Section 4.2): channel ch has its values at vals + ch * vals
// and its operand plane at x + ch * x, both in elements.  One channel: strides unused.
struct ChannelStrides {
    int channels;
    long long vals, x;
};

template <int G>
__global__ __launch_bounds__(kGatherThreads) void spmm_gather_scalar_kernel(
    const int *__restrict__ row_ptr, const int *__restrict__ col_idx, const float *__restrict__ vals,
    const float *__restrict__ x, float *__restrict__ y, int rows, int batch, ChannelStrides cs) {
    const long long row = ((long long)blockIdx.x * kGatherThreads + threadIdx.x) / G;
    const int lane = (int)threadIdx.x % G;
    int beg = 0, end = 0;
    if (row < rows) {
        beg = row_ptr[row];
        end = row_ptr[row + 1];
    }
    for (int c = blockIdx.y; c < batch; c += gridDim.y) {   // uniform over the block
        float acc = 0.0f;
        if (cs.channels == 1) {
            for (int e = beg + lane; e < end; e += G)
                acc = fmaf(vals[e], x[(long long)col_idx[e] * batch + c], acc);
        } else if (end > beg) {
            // the group walks the row's entries of all channels as one list: position t is
            // entry t % len of channel t / len
            const int len = end - beg;
            int ch = lane / len, eo = lane - ch * len;
            while (ch < cs.channels) {
                const int e = beg + eo;
                acc = fmaf(vals[ch * cs.vals + e], x[ch * cs.x + (long long)col_idx[e] * batch + c], acc);
                eo += G;
                while (eo >= len) { eo -= len; ++ch; }
            }
        }
        acc = group_sum<G>(acc);
        if (row < rows && lane == 0) y[row * batch + c] = acc;
    }
}

template <int G, int NV>
__global__ __launch_bounds__(kGatherThreads) void spmm_gather_vec_kernel(
    const int *__restrict__ row_ptr, const int *__restrict__ col_idx, const float *__restrict__ vals,
    const float *__restrict__ x, float *__restrict__ y, int rows, int batch, ChannelStrides cs) {
    const long long row = ((long long)blockIdx.x * kGatherThreads + threadIdx.x) / G;
    const int lane = (int)threadIdx.x % G;
    int beg = 0, end = 0;
    if (row < rows) {
        beg = row_ptr[row];
        end = row_ptr[row + 1];
    }
    for (int c0 = blockIdx.y * (4 * NV); c0 < batch; c0 += gridDim.y * (4 * NV)) {   // uniform over the block
        float4 acc[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) acc[v] = make_float4(0.f, 0.f, 0.f, 0.f);
        auto add = [&](float w, const float4 *xr) {
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const float4 xv = xr[v];
                acc[v].x = fmaf(w, xv.x, acc[v].x);
                acc[v].y = fmaf(w, xv.y, acc[v].y);
                acc[v].z = fmaf(w, xv.z, acc[v].z);
                acc[v].w = fmaf(w, xv.w, acc[v].w);
            }
        };
        if (cs.channels == 1) {
            for (int e = beg + lane; e < end; e += G)
                add(vals[e], reinterpret_cast<const float4 *>(x + (long long)col_idx[e] * batch + c0));
        } else if (end > beg) {
            // the group walks the row's entries of all channels as one list (see the scalar kernel)
            const int len = end - beg;
            int ch = lane / len, eo = lane - ch * len;
            while (ch < cs.channels) {
                const int e = beg + eo;
                add(vals[ch * cs.vals + e],
                    reinterpret_cast<const float4 *>(x + ch * cs.x + (long long)col_idx[e] * batch + c0));
                eo += G;
                while (eo >= len) { eo -= len; ++ch; }
            }
        }
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            acc[v].x = group_sum<G>(acc[v].x);
            acc[v].y = group_sum<G>(acc[v].y);
            acc[v].z = group_sum<G>(acc[v].z);
            acc[v].w = group_sum<G>(acc[v].w);
        }
        if (row < rows && lane == 0) {
            float4 *yr = reinterpret_cast<float4 *>(y + row * batch + c0);
#pragma unroll
            for (int v = 0; v < NV; ++v) yr[v] = acc[v];
        }
    }
}

// ---------------------------------------------------------------------------
// y = T x from the column-compressed arrays of T (the paper's CSC variants, Sections 3 and
// 4.1, multiply by the same T stored by columns).  By columns the product is a scatter:
// column j contributes vals[e] * x[j] to row row_idx[e].  G lanes share a column; each
// contribution is one hardware float add to y (zeroed beforehand by fill_zero_kernel), so
// the summation order, unlike everywhere else in this library, depends on timing.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kGatherThreads) void fill_zero_kernel(float *__restrict__ y, long long count) {
    const long long stride = (long long)gridDim.x * kGatherThreads;
    const long long first = (long long)blockIdx.x * kGatherThreads + threadIdx.x;
    // 16-byte stores over the aligned middle, single floats before and after it
    const long long head = min(count, (long long)((16 - (reinterpret_cast<uintptr_t>(y) & 15u)) & 15u) / 4);
    const long long quads = (count - head) / 4;
    float4 *const mid = reinterpret_cast<float4 *>(y + head);
    for (long long i = first; i < quads; i += stride) mid[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (long long i = first; i < head; i += stride) y[i] = 0.0f;
    for (long long i = head + 4 * quads + first; i < count; i += stride) y[i] = 0.0f;
}

// BL consecutive lanes take BL neighbouring batch columns of one entry, so that their adds fall
// into one 64-byte line of y and travel to the L2 as one request.
template <int G, int BL>
__global__ __launch_bounds__(kGatherThreads) void spmm_scatter_kernel(
    const int *__restrict__ col_ptr, const int *__restrict__ row_idx, const float *__restrict__ vals,
    const float *__restrict__ x, float *__restrict__ y, int cols, int batch) {
    const long long col = ((long long)blockIdx.x * kGatherThreads + threadIdx.x) / (G * BL);
    const int r = (int)threadIdx.x % (G * BL), lane = r / BL, bl = r % BL;
    if (col >= cols) return;
    const int beg = col_ptr[col], end = col_ptr[col + 1];
    for (int c = blockIdx.y * BL + bl; c < batch; c += gridDim.y * BL) {
        const float xv = x[col * batch + c];
        for (int e = beg + lane; e < end; e += G)
            unsafeAtomicAdd(y + (long long)row_idx[e] * batch + c, vals[e] * xv);
    }
}

// The same scatter with the sums kept on chip.  A workgroup takes a tile of ti x tj input
// pixels (columns of T) and a chunk of batch columns, and keeps in LDS a window of outputs
// around the ones those columns reach (Section 2: pixel i is covered by the windows x with
// 0 <= i + p - s x < k, so ti lines reach at most (ti + k - 2)/s + 1 output lines).  The
// window is wx runs of wy consecutive rows, run lx starting at row base + lx * n_out; an
// entry whose row is not in it (none is, for arrays this library built) is added to y directly.
//
// LDS float atomics run one lane at a time on this chip (about 190 clocks per wave
// instruction against 8 for a read, an add and a write), so the sums are plain
// read-add-write and the lanes are laid out so that no two of them ever meet in one slot:
//  * each wave owns VB batch columns and a window image of its own, so waves never share;
//  * the lanes of one step are entries of ONE column (each lane adds its entry's VB
//    products), and the entries of a column have pairwise different rows (the arrays come
//    from conv_csc_build, which writes every (row, column) pair once) -- or, where columns
//    are short, of several columns k pixels apart, each entry admitted only to the places
//    its own pixel's windows can have, which differ from pixel to pixel at that distance;
//  * a wave's LDS instructions execute in order, so the writes of one step are seen by the
//    reads of the next.
// The entries of one tile line are contiguous in the arrays; the workgroup copies them into
// an LDS stage one line ahead of their use, so that the waves (which all walk the same
// entries, for different batch columns) never wait for memory inside the walk.  At the end
// the workgroup adds its windows to y, which fill_zero_kernel cleared: about
// (1 + (k-1)/(s ti)) (1 + (k-1)/(s tj)) adds per output instead of one per entry.
constexpr int kCscStage = 1024;      // most entries of one tile line (tj columns)

struct CscTileGeom {
    int m, n, n_out, k, s, p, batch;
    int ti, tj, tiles_j;           // tile: ti lines of tj pixels, tj < 64; tiles per line of tiles
    int wx, wy;                    // window: runs x rows per run
    int limit;                     // (wx - 1) * n_out + wy, at most 2^21: rows base .. base + limit - 1 can be in the window
    int stage;                     // entries per stage buffer, tj * (most entries of a column) <= kCscStage
    int ptrs;                      // ints set aside for the column pointers, ti * (tj + 1) rounded up to 4
    int column_max;                // most entries of a column: ceil(k/s)^2
    int group, spacing;            // columns per step (64 / column_max, at least 1) and their distance, k pixels
    float inv_wy, inv_n_out;
};

__device__ __forceinline__ int first_window(int t0, int k, int s, int p) {   // smallest x >= 0 with t0 + p - s x < k
    const long long num = (long long)t0 + p - k + 1;
    return num <= 0 ? 0 : (int)((num + s - 1) / s);
}

template <int VB, int W>
__global__ __launch_bounds__(W *kWave) void spmm_csc_tile_kernel(
    const int *__restrict__ col_ptr, const int *__restrict__ row_idx, const float *__restrict__ vals,
    const float *__restrict__ x, float *__restrict__ y, const CscTileGeom g) {
    constexpr int NT = W * kWave, BC = W * VB;   // threads; batch columns per pass
    constexpr int PER = kCscStage / NT;          // staged entries per thread
    extern __shared__ __align__(16) int lds[];
    int2 *const stage = reinterpret_cast<int2 *>(lds);                     // [2][g.stage] (window slot or -1, value bits)
    int *const ptrs = lds + 4 * g.stage;                                   // [ti][tj + 1] column pointers
    float *const win = reinterpret_cast<float *>(ptrs + g.ptrs);           // [W][VB / 4][wx][wy][4] ([W][wx][wy][VB] for VB < 4)
    const int tile_i = (int)blockIdx.x / g.tiles_j, tile_j = (int)blockIdx.x - tile_i * g.tiles_j;
    const int i0 = tile_i * g.ti, j0 = tile_j * g.tj;
    // first row of the window; below 2^31 like every row
    const int base = first_window(i0, g.k, g.s, g.p) * g.n_out + first_window(j0, g.k, g.s, g.p);
    const int tid = (int)threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave), lane = tid % kWave;
    const int slots = g.wx * g.wy, image = slots * VB;
    float *const mine = win + wave * image;
    const int lines = min(g.ti, g.m - i0), ncols = min(g.tj, g.n - j0);
    const long long tile_col0 = (long long)i0 * g.n + j0;
    const int skip = g.n_out - g.wy;             // rows between the end of one run and the start of the next
    // several columns per step: this lane's column among them and its entry in that column; the places in
    // a run that the windows over column `lane` of the tile can have (lane l holds column l's)
    const int lane_group = lane / g.column_max, lane_entry = lane - lane_group * g.column_max;
    const int reach_col = j0 + min(lane, ncols - 1), y_lo = first_window(j0, g.k, g.s, g.p);
    const int reach_lo = first_window(reach_col, g.k, g.s, g.p) - y_lo, reach_hi = (reach_col + g.p) / g.s - y_lo;

    for (int t = tid; t < lines * (g.tj + 1); t += NT) {
        const int li = t / (g.tj + 1), cj = t - li * (g.tj + 1);
        ptrs[t] = col_ptr[tile_col0 + (long long)li * g.n + min(cj, ncols)];
    }
    for (int c0 = blockIdx.y * BC; c0 < g.batch; c0 += gridDim.y * BC) {      // uniform over the block
        for (int t = tid; t < image * W; t += NT) win[t] = 0.0f;
        __syncthreads();
        // Entry `at` of tile line li (row, value) into a stage buffer: its window slot, found here once
        // for all waves and off their chain of sums.  An entry outside the window is added to y on the
        // spot, for every batch column of this pass, and staged as slot -1.
        auto put = [&](int2 *buf, int li, int at, int row, int value) {
            const int rp = row - base;
            const bool near = (unsigned)rp < (unsigned)g.limit;
            const int lx = div_small(near ? rp : 0, g.inv_n_out), ly = rp - lx * g.n_out;
            int slot = (rp - lx * skip) | ly << 16;       // the slot, and above it the row's place in its run
            if (!near || ly >= g.wy) {
                slot = -1;
                const int *lp = ptrs + li * (g.tj + 1);
                const int e = lp[0] + at;
                int t = 0;
                while (t + 1 < ncols && e >= lp[t + 1]) ++t;
                const float *xc = x + (tile_col0 + (long long)li * g.n + t) * g.batch;
                for (int b = c0; b < min(c0 + BC, g.batch); ++b)
                    unsafeAtomicAdd(y + (long long)row * g.batch + b, __int_as_float(value) * xc[b]);
            }
            buf[at] = make_int2(slot, value);
        };
        const int cw = c0 + wave * VB;           // this wave's first batch column
        // lane l holds the wave's VB inputs of column l of a line
        auto load_x = [&](float (&xl)[VB], long long col0) {
            const float *xp = x + (col0 + min(lane, ncols - 1)) * g.batch + cw;
            if (cw + VB <= g.batch) {
#pragma unroll
                for (int v = 0; v < VB; ++v) xl[v] = xp[v];
            } else {
#pragma unroll
                for (int v = 0; v < VB; ++v) xl[v] = cw + v < g.batch ? xp[v] : 0.0f;
            }
        };
        float xl_next[VB];
        load_x(xl_next, tile_col0);
        {   // line 0 into the stage
            const int beg = ptrs[0], count = min(ptrs[ncols] - beg, g.stage);
            for (int t = tid; t < count; t += NT) put(stage, 0, t, row_idx[beg + t], __float_as_int(vals[beg + t]));
        }
        __syncthreads();
        for (int li = 0; li < lines; ++li) {
            const int2 *const cur = stage + (li & 1) * g.stage;
            const int cp = ptrs[li * (g.tj + 1) + min(lane, ncols)];       // lane l: pointer of column l
            // the next line's entries and inputs are asked for now and staged after this line's sums
            int rows_next[PER], vals_next[PER];
            int count_next = 0;
            float xl[VB];
#pragma unroll
            for (int v = 0; v < VB; ++v) xl[v] = xl_next[v];
            if (li + 1 < lines) {
                load_x(xl_next, tile_col0 + (long long)(li + 1) * g.n);
                const int beg_next = ptrs[(li + 1) * (g.tj + 1)];
                count_next = min(ptrs[(li + 1) * (g.tj + 1) + ncols] - beg_next, g.stage);
#pragma unroll
                for (int u = 0; u < PER; ++u) {
                    rows_next[u] = vals_next[u] = 0;
                    if (u * NT + tid < count_next) {
                        rows_next[u] = row_idx[beg_next + u * NT + tid];
                        vals_next[u] = __float_as_int(vals[beg_next + u * NT + tid]);
                    }
                }
            }
            const int line_beg = __builtin_amdgcn_readfirstlane(cp);
            // entries e .. of a column that ends at `end`, one per lane, from the stage
            auto fetch = [&](int e, int end) { return cur[max(min(min(e, end - 1) - line_beg, g.stage - 1), 0)]; };
            // this lane's entry into its slot of the wave's window
            auto add = [&](int slot_at, float val, const float (&xq)[VB]) {
                if (VB % 4 == 0) {
                    // planes of four batch columns: neighbouring slots are 16 bytes apart in each
                    float4 *const slot = reinterpret_cast<float4 *>(mine) + slot_at;
                    float4 q[VB / 4 + 1];
#pragma unroll
                    for (int v = 0; v < VB / 4; ++v) q[v] = slot[v * slots];
#pragma unroll
                    for (int v = 0; v < VB / 4; ++v) {
                        q[v].x = fmaf(val, xq[4 * v], q[v].x);
                        q[v].y = fmaf(val, xq[4 * v + 1], q[v].y);
                        q[v].z = fmaf(val, xq[4 * v + 2], q[v].z);
                        q[v].w = fmaf(val, xq[4 * v + 3], q[v].w);
                    }
#pragma unroll
                    for (int v = 0; v < VB / 4; ++v) slot[v * slots] = q[v];
                } else {
                    float *const slot = mine + slot_at * VB;
#pragma unroll
                    for (int v = 0; v < VB; ++v) slot[v] = fmaf(val, xq[v], slot[v]);
                }
            };
            if (g.group > 1) {
                // Short columns: a step takes up to g.group columns that lie g.spacing = k pixels apart.  No
                // window covers two such pixels (Section 2: window y covers pixels s y - p .. s y - p + k - 1),
                // so their rows lie in different places of a run; an entry is added in LDS only if its place is
                // one its pixel's windows can have (checked on the stored row), anything else goes to y directly.
                for (int first = 0; first < g.spacing; ++first)
                    for (int c_first = first; c_first < ncols; c_first += g.group * g.spacing) {
                        const int mine_col = c_first + lane_group * g.spacing;
                        const bool has = lane_group < g.group && mine_col < ncols;
                        const int cl = has ? mine_col : 0;
                        int e = __shfl(cp, cl) + lane_entry;
                        const int end = __shfl(cp, cl + 1);
                        const int lo = __shfl(reach_lo, cl), hi = __shfl(reach_hi, cl);
                        float xq[VB];
#pragma unroll
                        for (int v = 0; v < VB; ++v) xq[v] = __shfl(xl[v], cl);
                        while (__builtin_amdgcn_ballot_w64(has && e < end) != 0) {
                            const int2 ev = fetch(e, end);
                            const float val = __int_as_float(ev.y);
                            if (has && e < end && ev.x >= 0) {
                                const int slot_at = ev.x & 0xffff, place = ev.x >> 16;
                                if (place >= lo && place <= hi) {
                                    add(slot_at, val, xq);
                                } else {
                                    const long long row = (long long)base + slot_at + (long long)div_small(slot_at, g.inv_wy) * skip;
#pragma unroll
                                    for (int v = 0; v < VB; ++v)
                                        if (cw + v < g.batch) unsafeAtomicAdd(y + row * g.batch + cw + v, val * xq[v]);
                                }
                            }
                            wave_lds_order();
                            e += g.column_max;
                        }
                    }
            } else {
                int end = line_beg;
                int2 ahead = fetch(line_beg + lane, __builtin_amdgcn_readlane(cp, 1));
                for (int t = 0; t < ncols; ++t) {
                    const int beg = end;
                    end = __builtin_amdgcn_readlane(cp, t + 1);
                    int2 ev = ahead;
                    // the first 64 entries of the next column are fetched before this column's sums
                    if (t + 1 < ncols) ahead = fetch(end + lane, __builtin_amdgcn_readlane(cp, t + 2));
                    if (beg >= end) continue;
                    float xq[VB];
#pragma unroll
                    for (int v = 0; v < VB; ++v)
                        xq[v] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(xl[v]), t));
                    for (int e0 = beg; e0 < end; e0 += kWave) {      // entries e0 .. e0 + 63 of column t
                        if (e0 > beg) ev = fetch(e0 + lane, end);
                        if (e0 + lane < end && ev.x >= 0) add(ev.x & 0xffff, __int_as_float(ev.y), xq);
                        wave_lds_order();
                    }
                }
            }
            if (li + 1 < lines) {
                int2 *const nxt = stage + ((li + 1) & 1) * g.stage;
#pragma unroll
                for (int u = 0; u < PER; ++u)
                    if (u * NT + tid < count_next) put(nxt, li + 1, u * NT + tid, rows_next[u], vals_next[u]);
            }
            __syncthreads();
        }
        // consecutive threads take the batch columns of one output, so that their adds fill a line of y
        for (int t = tid; t < g.wx * g.wy * BC; t += NT) {
            const int b = t % BC, slot = t / BC;
            const int bw = b % VB;
            const float v = VB % 4 == 0 ? win[(b / VB) * image + ((bw / 4) * slots + slot) * 4 + bw % 4]
                                        : win[(b / VB) * image + slot * VB + bw];
            const int lx = div_small(slot, g.inv_wy);
            if (v != 0.0f && c0 + b < g.batch)      // a slot that received a sum stands for a row of T
                unsafeAtomicAdd(y + ((long long)base + slot + (long long)lx * skip) * g.batch + c0 + b, v);
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// Many small products in one launch.  The paper's experiment (Section 4.1)
// applies 123 small, independent transformations (the DenseNet121 layer shapes
// of Table 2, 7x7 ... 224x224 pixels); each of them is a few microseconds of
// work, far less than a kernel launch costs.  Here every product i has a
// descriptor, the grid is the concatenation of the products' row blocks, and a
// workgroup finds its product by bisection over first_block.  Inside a
// product the row-group scheme of the gather kernels is used with a per-product
// group width (1 << g_shift lanes per row).
// ---------------------------------------------------------------------------
struct MultiDesc {
    const int *row_ptr;
    const int *col_idx;
    const float *vals;
    const float *x;
    float *y;
    int rows;
    int g_shift;          // log2 of the lanes per row, 0..4
    int first_block;      // first workgroup of this product in the launch
    int pad;
};

__global__ __launch_bounds__(kGatherThreads) void spmm_multi_kernel(const MultiDesc *__restrict__ descs, int n,
                                                                    int batch) {
    int lo = 0, hi = n;                  // descs[lo].first_block <= blockIdx.x < descs[hi].first_block
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (descs[mid].first_block <= (int)blockIdx.x) lo = mid; else hi = mid;
    }
    const MultiDesc d = descs[lo];
    const int gs = d.g_shift, G = 1 << gs;
    const long long row = ((long long)(blockIdx.x - d.first_block) * kGatherThreads + threadIdx.x) >> gs;
    const int lane = (int)threadIdx.x & (G - 1);
    int beg = 0, end = 0;
    if (row < d.rows) {
        beg = d.row_ptr[row];
        end = d.row_ptr[row + 1];
    }
    for (int c = blockIdx.y; c < batch; c += gridDim.y) {   // uniform over the block
        float acc = 0.0f;
        for (int e = beg + lane; e < end; e += G)
            acc = fmaf(d.vals[e], d.x[(long long)d.col_idx[e] * batch + c], acc);
        // butterfly over the group; gs is uniform over the block, all lanes are active
        if (gs >= 1) acc += dpp_move<kDppXor1>(acc);
        if (gs >= 2) acc += dpp_move<kDppXor2>(acc);
        if (gs >= 3) acc += dpp_move<kDppXor7>(acc);
        if (gs >= 4) acc += dpp_move<kDppXor15>(acc);
        if (row < d.rows && lane == 0) d.y[row * batch + c] = acc;
    }
}

}  // namespace convspmv
