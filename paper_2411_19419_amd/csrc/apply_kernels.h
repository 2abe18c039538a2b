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

template <int G>
__global__ __launch_bounds__(kGatherThreads) void spmm_gather_scalar_kernel(
    const int *__restrict__ row_ptr, const int *__restrict__ col_idx, const float *__restrict__ vals,
    const float *__restrict__ x, float *__restrict__ y, int rows, int batch) {
    const long long row = ((long long)blockIdx.x * kGatherThreads + threadIdx.x) / G;
    const int lane = (int)threadIdx.x % G;
    int beg = 0, end = 0;
    if (row < rows) {
        beg = row_ptr[row];
        end = row_ptr[row + 1];
    }
    for (int c = blockIdx.y; c < batch; c += gridDim.y) {   // uniform over the block
        float acc = 0.0f;
        for (int e = beg + lane; e < end; e += G)
            acc = fmaf(vals[e], x[(long long)col_idx[e] * batch + c], acc);
        acc = group_sum<G>(acc);
        if (row < rows && lane == 0) y[row * batch + c] = acc;
    }
}

template <int G, int NV>
__global__ __launch_bounds__(kGatherThreads) void spmm_gather_vec_kernel(
    const int *__restrict__ row_ptr, const int *__restrict__ col_idx, const float *__restrict__ vals,
    const float *__restrict__ x, float *__restrict__ y, int rows, int batch) {
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
        for (int e = beg + lane; e < end; e += G) {
            const float w = vals[e];
            const float4 *xr = reinterpret_cast<const float4 *>(x + (long long)col_idx[e] * batch + c0);
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const float4 xv = xr[v];
                acc[v].x = fmaf(w, xv.x, acc[v].x);
                acc[v].y = fmaf(w, xv.y, acc[v].y);
                acc[v].z = fmaf(w, xv.z, acc[v].z);
                acc[v].w = fmaf(w, xv.w, acc[v].w);
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

}  // namespace convspmv
