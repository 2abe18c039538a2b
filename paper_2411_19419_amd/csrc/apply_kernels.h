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
    for (long long i = (long long)blockIdx.x * kGatherThreads + threadIdx.x; i < count; i += stride) y[i] = 0.0f;
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
