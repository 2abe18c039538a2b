// Device-side construction of T in CSR (gfx950).
//
// Theorem 2.1 gives the length of row (x, y) of T as r1(x) * r2(y) with
//   r1(x) = max(0, k - c1(x)),  c1(x) = max(0, p - s x) + max(0, s x + k - m - p)
// and r2, c2 likewise along n.  Because the length is a product of one factor
// per axis, the 2-D exclusive scan that row_ptr needs collapses to the two
// 1-D exclusive scans P1 (of r1) and P2 (of r2):
//   row_ptr[x * n_out + y] = P1[x] * S2 + r1(x) * P2[y],   S2 = P2[n_out].
// Inside a row the stored taps are the r1 x r2 rectangle of kernel positions
// that starts at (a_lo, b_lo) = (max(0, p - s x), max(0, p - s y)) (the "top"
// and "left" padding terms of c1 and c2); entry t of the row is tap
// (a_lo + t / r2, b_lo + t % r2), which lands on input pixel
// (s x + a - p, s y + b - p) (Section 2: C places K[a][b] at padded position
// (s x + a, s y + b), P maps input (i, j) to padded (i + p, j + p)).
#pragma once
#include "device_util.h"

namespace convspmv {

struct ConvShape {
    int m, n, k, s, p;
    int m_out, n_out;
};

// Row-length factor of Theorem 2.1 along one axis of extent `extent`.
__device__ __forceinline__ int axis_taps(int t, int extent, int k, int s, int p) {
    // 64-bit: s*t can reach extent + 2p
    long long st = (long long)s * t;
    long long lo = (long long)p - st;
    long long hi = st + k - extent - p;
    long long c = (lo > 0 ? lo : 0) + (hi > 0 ? hi : 0);
    long long r = (long long)k - c;
    return r > 0 ? (int)r : 0;
}

// One block per axis (blockIdx.x = 0: the m axis -> P1, 1: the n axis -> P2).
// tab holds P1[0..m_out] followed by P2[0..n_out].  The block walks its axis
// in chunks of blockDim.x with a running carry; inside a chunk an inclusive
// scan runs over LDS (Hillis-Steele).
constexpr int kAxisThreads = 1024;

__global__ __launch_bounds__(kAxisThreads) void axis_prefix_kernel(ConvShape sh, int *__restrict__ tab) {
    __shared__ int buf[2][kAxisThreads];
    const bool second = blockIdx.x == 1;
    const int extent = second ? sh.n : sh.m;
    const int count = second ? sh.n_out : sh.m_out;
    int *out = second ? tab + (sh.m_out + 1) : tab;
    int carry = 0;
    for (int base = 0; base < count; base += kAxisThreads) {
        const int t = base + (int)threadIdx.x;
        const int mine = t < count ? axis_taps(t, extent, sh.k, sh.s, sh.p) : 0;
        int cur = 0;
        buf[0][threadIdx.x] = mine;
        __syncthreads();
        for (int off = 1; off < kAxisThreads; off <<= 1) {
            int v = buf[cur][threadIdx.x];
            if ((int)threadIdx.x >= off) v += buf[cur][threadIdx.x - off];
            buf[cur ^ 1][threadIdx.x] = v;
            cur ^= 1;
            __syncthreads();
        }
        const int incl = buf[cur][threadIdx.x];
        if (t < count) out[t] = carry + incl - mine;
        carry += buf[cur][kAxisThreads - 1];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[count] = carry;
}

// row_ptr from the two axis tables; one thread per row, plus the final entry.
constexpr int kRowPtrThreads = 256;

__global__ __launch_bounds__(kRowPtrThreads) void row_ptr_kernel(ConvShape sh, const int *__restrict__ tab,
                                                                 int *__restrict__ row_ptr) {
    const int *P1 = tab, *P2 = tab + (sh.m_out + 1);
    const int blocks_per_line = (sh.n_out + kRowPtrThreads - 1) / kRowPtrThreads;
    const int x = blockIdx.x / blocks_per_line;
    const int y = (blockIdx.x - x * blocks_per_line) * kRowPtrThreads + (int)threadIdx.x;
    if (y >= sh.n_out) return;
    const long long S2 = P2[sh.n_out];
    const long long p1 = P1[x], r1 = P1[x + 1] - P1[x];
    row_ptr[(long long)x * sh.n_out + y] = (int)(p1 * S2 + r1 * P2[y]);
    if (x == sh.m_out - 1 && y == sh.n_out - 1)
        row_ptr[(long long)sh.m_out * sh.n_out] = (int)((long long)P1[sh.m_out] * S2);
}

// col_idx and vals.  G consecutive lanes share one row and write its entries
// G at a time, so a wave writes 64/G neighbouring rows, which are neighbouring
// in memory: every wave store covers one contiguous span of col_idx (vals).
// A block covers kFillThreads / G consecutive rows of one output line.
constexpr int kFillThreads = 256;

template <int G>
__global__ __launch_bounds__(kFillThreads) void csr_fill_kernel(ConvShape sh, const int *__restrict__ tab,
                                                                const float *__restrict__ kernel,
                                                                int *__restrict__ col_idx,
                                                                float *__restrict__ vals) {
    constexpr int kRowsPerBlock = kFillThreads / G;
    const int *P1 = tab, *P2 = tab + (sh.m_out + 1);
    const int blocks_per_line = (sh.n_out + kRowsPerBlock - 1) / kRowsPerBlock;
    const int x = blockIdx.x / blocks_per_line;
    const int y = (blockIdx.x - x * blocks_per_line) * kRowsPerBlock + (int)threadIdx.x / G;
    const int lane = (int)threadIdx.x % G;
    if (y >= sh.n_out) return;

    const int p1 = P1[x], r1 = P1[x + 1] - p1;
    const int p2 = P2[y], r2 = P2[y + 1] - p2;
    const int len = r1 * r2;
    if (len == 0) return;
    const long long base = (long long)p1 * P2[sh.n_out] + (long long)r1 * p2;
    const long long sx = (long long)sh.s * x, sy = (long long)sh.s * y;
    const int a_lo = sx < sh.p ? (int)(sh.p - sx) : 0;
    const int b_lo = sy < sh.p ? (int)(sh.p - sy) : 0;
    // input pixel of the row's first stored tap
    const long long i0 = sx + a_lo - sh.p, j0 = sy + b_lo - sh.p;
    const float inv_r2 = 1.0f / (float)r2;
    const bool small = len < (1 << 21);
    for (int t = lane; t < len; t += G) {
        const int da = small ? div_small(t, inv_r2) : t / r2;
        const int db = t - da * r2;
        col_idx[base + t] = (int)((i0 + da) * sh.n + j0 + db);
        vals[base + t] = kernel[(a_lo + da) * sh.k + (b_lo + db)];
    }
}

}  // namespace convspmv
