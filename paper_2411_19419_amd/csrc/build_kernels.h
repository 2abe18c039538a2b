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
//
// The transposed matrix T^T (whose CSR arrays are the CSC arrays of T, the
// other storage the paper uses, Sections 3 and 4.1) has the same product
// structure with the roles of windows and pixels exchanged: row (i, j) of T^T
// has q1(i) * q2(j) entries, q1(i) = number of window lines x in [0, m_out)
// with 0 <= i + p - s x < k, its entries are the windows (x_lo + d1, y_lo + d2)
// in ascending order with value K[i + p - s x][j + p - s y].  The kernels below
// take a flag TR and build either matrix: "line" and "position in the line"
// mean (x, y) for T and (i, j) for T^T.
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

// Number of window positions t in [0, count_out) along one axis whose window
// covers input coordinate i (0 <= i + p - s t < k), and the first of them.
__device__ __forceinline__ int axis_first_window(int i, int k, int s, int p) {
    const long long num = (long long)i + p - k + 1;          // smallest s*t allowed, may be negative
    return num > 0 ? (int)((num + s - 1) / s) : 0;
}
__device__ __forceinline__ int axis_cover(int i, int count_out, int k, int s, int p) {
    const long long lo = axis_first_window(i, k, s, p);
    long long hi = ((long long)i + p) / s;
    if (hi > count_out - 1) hi = count_out - 1;
    return hi >= lo ? (int)(hi - lo + 1) : 0;
}

// Lines of the matrix being built and rows per line.
template <bool TR> __device__ __forceinline__ int build_lines(const ConvShape &sh) { return TR ? sh.m : sh.m_out; }
template <bool TR> __device__ __forceinline__ int build_per_line(const ConvShape &sh) { return TR ? sh.n : sh.n_out; }

// One block per axis (blockIdx.x = 0: the m axis -> P1, 1: the n axis -> P2).
// tab holds P1[0..m_out] followed by P2[0..n_out].  The block walks its axis
// in chunks of blockDim.x with a running carry; inside a chunk an inclusive
// scan runs over LDS (Hillis-Steele).
constexpr int kAxisThreads = 1024;

template <bool TR>
__global__ __launch_bounds__(kAxisThreads) void axis_prefix_kernel(ConvShape sh, int *__restrict__ tab) {
    __shared__ int buf[2][kAxisThreads];
    const bool second = blockIdx.x == 1;
    const int extent = second ? sh.n : sh.m;                  // input extent along this axis
    const int count_out = second ? sh.n_out : sh.m_out;       // window positions along this axis
    const int count = TR ? extent : count_out;                // table length - 1
    int *out = second ? tab + (build_lines<TR>(sh) + 1) : tab;
    int carry = 0;
    for (int base = 0; base < count; base += kAxisThreads) {
        const int t = base + (int)threadIdx.x;
        const int mine = t >= count ? 0 : (TR ? axis_cover(t, count_out, sh.k, sh.s, sh.p)
                                                : axis_taps(t, extent, sh.k, sh.s, sh.p));
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

template <bool TR>
__global__ __launch_bounds__(kRowPtrThreads) void row_ptr_kernel(ConvShape sh, const int *__restrict__ tab,
                                                                 int *__restrict__ row_ptr) {
    const int L1 = build_lines<TR>(sh), L2 = build_per_line<TR>(sh);
    const int *P1 = tab, *P2 = tab + (L1 + 1);
    const int blocks_per_line = (L2 + kRowPtrThreads - 1) / kRowPtrThreads;
    const int x = blockIdx.x / blocks_per_line;
    const int y = (blockIdx.x - x * blocks_per_line) * kRowPtrThreads + (int)threadIdx.x;
    if (y >= L2) return;
    const long long S2 = P2[L2];
    const long long p1 = P1[x], r1 = P1[x + 1] - P1[x];
    row_ptr[(long long)x * L2 + y] = (int)(p1 * S2 + r1 * P2[y]);
    if (x == L1 - 1 && y == L2 - 1) row_ptr[(long long)L1 * L2] = (int)((long long)P1[L1] * S2);
}

// col_idx and vals.  A block takes kFillRows consecutive rows of one output
// line; their entries are one contiguous span of both arrays.  The span is cut
// into quads of four entries on 16-byte boundaries of the arrays; a thread
// takes quads t, t + 256, ..., finds the row and tap of its first entry and
// walks on from there, and stores 16 bytes per array.  Every wave store then
// covers 1 KiB of contiguous memory and whole cache lines leave the CU
// complete.  (Giving each row to a group of lanes wrote 32-byte pieces and the
// memory counters showed 1.85 bytes written per byte of output.)
//
// Entry q of the span (counted from the block's first row ya) belongs to the
// row y with r1 * (P2[y] - P2[ya]) <= q < r1 * (P2[y+1] - P2[ya]): the table
// P2 - P2[ya] sits in LDS; y is guessed as if all rows before it were full
// (r2 = k, true away from the left border) and found by bisection otherwise.
constexpr int kFillThreads = 256;
constexpr int kFillRows = 256;

// COLS = false rewrites vals only (a new kernel for the same shape; the column
// indices do not depend on K).  TR builds T^T.
template <bool COLS, bool TR>
__global__ __launch_bounds__(kFillThreads) void csr_fill_kernel(ConvShape sh, const int *__restrict__ tab,
                                                                const float *__restrict__ kernel,
                                                                int *__restrict__ col_idx,
                                                                float *__restrict__ vals) {
    typedef int ivec4 __attribute__((ext_vector_type(4)));
    typedef float fvec4 __attribute__((ext_vector_type(4)));
    __shared__ int rel[kFillRows + 1];           // P2[ya + i] - P2[ya]
    const int L1 = build_lines<TR>(sh), L2 = build_per_line<TR>(sh);
    const int *P1 = tab, *P2 = tab + (L1 + 1);
    const int blocks_per_line = (L2 + kFillRows - 1) / kFillRows;
    const int x = blockIdx.x / blocks_per_line;
    const int ya = (blockIdx.x - x * blocks_per_line) * kFillRows;
    const int nrows = min(kFillRows, L2 - ya);
    const int p1 = P1[x], r1 = P1[x + 1] - p1;
    const int p2a = P2[ya];
    for (int i = threadIdx.x; i <= nrows; i += kFillThreads) rel[i] = P2[ya + i] - p2a;
    __syncthreads();
    const long long base = (long long)p1 * P2[L2] + (long long)r1 * p2a;
    const long long total = (long long)r1 * rel[nrows];
    if (total == 0) return;                      // uniform: these rows have no entries
    // Along the line axis: first stored kernel row a_lo and its input line i0 (T), or the
    // first covering window line x_lo (T^T).  first2 does the same along the other axis.
    const long long sx = (long long)sh.s * x;
    const int a_lo = TR ? axis_first_window(x, sh.k, sh.s, sh.p) : (sx < sh.p ? (int)(sh.p - sx) : 0);
    const long long i0 = sx + a_lo - sh.p;
    auto first2 = [&](int u2) {
        if (TR) return axis_first_window(u2, sh.k, sh.s, sh.p);
        const long long sy = (long long)sh.s * u2;
        return sy < sh.p ? (int)(sh.p - sy) : 0;
    };
    // column index and kernel index of entry (da, db) of the row at position u2 with first2 = b_lo
    auto entry = [&](int u2, int b_lo, int da, int db, int &col, int &kidx) {
        if (TR) {
            const int wx = a_lo + da, wy = b_lo + db;          // window (wx, wy) covers pixel (x, u2)
            col = (int)((long long)wx * sh.n_out + wy);
            kidx = (x + sh.p - sh.s * wx) * sh.k + (u2 + sh.p - sh.s * wy);
        } else {
            col = (int)((i0 + da) * sh.n + ((long long)sh.s * u2 + b_lo - sh.p) + db);
            kidx = (a_lo + da) * sh.k + (b_lo + db);
        }
    };
    const int full2 = TR ? (sh.k + sh.s - 1) / sh.s : sh.k;   // most entries a row has along the second axis
    const float inv_r1 = 1.0f / (float)r1, inv_k = 1.0f / (float)full2;
    const bool small = total < (1 << 21);        // float-reciprocal division is exact below 2^21
    // quads are aligned in the arrays: span position q sits in quad (q + lead) / 4
    const int lead = (int)(base & 3);
    int *cdst = col_idx + (base - lead);
    float *vdst = vals + (base - lead);
    const long long nquads = (total + lead + 3) >> 2;
    const bool aligned = (((COLS ? (uintptr_t)col_idx : 0) | (uintptr_t)vals) & 15u) == 0;
    for (long long quad = threadIdx.x; quad < nquads; quad += kFillThreads) {
        const long long qbeg = max(quad * 4 - lead, 0LL), qend = min(quad * 4 - lead + 4, total);
        // row and tap of the first entry
        const int u = small ? div_small((int)qbeg, inv_r1) : (int)(qbeg / r1);   // tap columns before its row
        int yy = small ? div_small(u, inv_k) : u / full2;
        yy = min(yy, nrows - 1);
        if (!(rel[yy] <= u && u < rel[yy + 1])) {                               // rows before it were not all full
            int lo = 0, hi = nrows;                                              // rel[lo] <= u < rel[hi]
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (rel[mid] <= u) lo = mid; else hi = mid;
            }
            yy = lo;
        }
        int r2 = rel[yy + 1] - rel[yy];
        const int t = (int)(qbeg - (long long)r1 * rel[yy]);                    // 0 <= t < r1*r2
        int da = small ? div_small(t, __builtin_amdgcn_rcpf((float)r2)) : t / r2, db = t - da * r2;
        int b_lo = first2(ya + yy);
        int cval[4];
        float vval[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const long long q = quad * 4 - lead + e;
            cval[e] = 0;
            vval[e] = 0.0f;
            if (q >= qbeg && q < qend) {
                int kidx;
                entry(ya + yy, b_lo, da, db, cval[e], kidx);
                vval[e] = kernel[kidx];
                if (++db == r2) {                // next kernel row, or the next row of T that has entries
                    db = 0;
                    if (++da == r1 && q + 1 < qend) {
                        da = 0;
                        do { ++yy; } while (rel[yy + 1] == rel[yy]);
                        r2 = rel[yy + 1] - rel[yy];
                        b_lo = first2(ya + yy);
                    }
                }
            }
        }
        if (aligned && qend - qbeg == 4) {
            ivec4 cv;
            fvec4 vv;
            cv.x = cval[0]; cv.y = cval[1]; cv.z = cval[2]; cv.w = cval[3];
            vv.x = vval[0]; vv.y = vval[1]; vv.z = vval[2]; vv.w = vval[3];
            if (COLS) __builtin_nontemporal_store(cv, reinterpret_cast<ivec4 *>(cdst + quad * 4));
            __builtin_nontemporal_store(vv, reinterpret_cast<fvec4 *>(vdst + quad * 4));
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const long long q = quad * 4 - lead + e;
                if (q >= qbeg && q < qend) {
                    if (COLS) cdst[quad * 4 + e] = cval[e];
                    vdst[quad * 4 + e] = vval[e];
                }
            }
        }
    }
}

// The same fill, staged through LDS, for rows of moderate length (the usual case).
//
// The quad-walking kernel above spends about 200 vector instructions per quad on finding where
// a quad starts (64-bit offsets, two reciprocal divisions, a search) and ran at 3.5 TB/s where
// a plain fill writes 6.5 TB/s.  Here a workgroup again takes R consecutive rows of one line
// (one contiguous span of the arrays), but every row is generated by the threads that own it,
// tap line by tap line, with nothing but additions, into an LDS image of the span; the image
// is then copied out in the same aligned 16-byte quads as before, so the stores are the same
// full lines (plain stores: with nothing but writes in flight they measured 18 % faster than
// non-temporal ones, the opposite of what the apply kernels see next to their read streams).
// The image is shifted by `lead` = span start mod 4 entries, which makes LDS quads and array
// quads coincide.  R (a power of two, 1..256) is chosen by the host so that the
// image fits: LDS holds rel[R+1], the k*k kernel numbers, and `cap` entries of each array.
// With row_ptr given the kernel writes the row pointers of its rows as well (the build then
// needs no separate row_ptr launch).
constexpr int kFillStageEntries = 6400;     // entries of one span the LDS image may hold

template <bool COLS, bool TR>
__global__ __launch_bounds__(kFillThreads) void csr_fill_staged_kernel(ConvShape sh, const int *__restrict__ tab,
                                                                       const float *__restrict__ kernel,
                                                                       int *__restrict__ col_idx,
                                                                       float *__restrict__ vals, int R, int cap,
                                                                       int *__restrict__ row_ptr) {
    typedef int ivec4 __attribute__((ext_vector_type(4)));
    typedef float fvec4 __attribute__((ext_vector_type(4)));
    extern __shared__ int fill_smem[];
    const int kk = sh.k * sh.k;
    int *rel = fill_smem;                                            // P2[ya + i] - P2[ya], i <= R
    float *ks = reinterpret_cast<float *>(rel + R + 1);              // the kernel
    int *scol = fill_smem + ((R + 1 + kk + 3) & ~3);                 // 16-byte aligned image of col_idx
    float *sval = reinterpret_cast<float *>(scol + cap);             // ... and of vals (cap is a multiple of 4)
    const int L1 = build_lines<TR>(sh), L2 = build_per_line<TR>(sh);
    const int *P1 = tab, *P2 = tab + (L1 + 1);
    const int blocks_per_line = (L2 + R - 1) / R;
    const int x = blockIdx.x / blocks_per_line;
    const int ya = (blockIdx.x - x * blocks_per_line) * R;
    const int nrows = min(R, L2 - ya);
    const int tid = threadIdx.x;
    const int p1 = P1[x], r1 = P1[x + 1] - p1;
    const int p2a = P2[ya];
    for (int i = tid; i <= nrows; i += kFillThreads) rel[i] = P2[ya + i] - p2a;
    for (int t = tid; t < kk; t += kFillThreads) ks[t] = kernel[t];
    __syncthreads();
    const long long base = (long long)p1 * P2[L2] + (long long)r1 * p2a;
    const int total = r1 * rel[nrows];               // at most R * (longest row) <= kFillStageEntries
    if (row_ptr) {
        // the row pointers of these rows come for free: row_ptr[x * L2 + y] = P1[x] * S2 + r1 * P2[y]
        for (int i = tid; i < nrows; i += kFillThreads) row_ptr[(long long)x * L2 + ya + i] = (int)(base + r1 * rel[i]);
        if (blockIdx.x == gridDim.x - 1 && tid == 0) row_ptr[(long long)L1 * L2] = (int)(base + total);
    }
    if (total == 0) return;                          // uniform: these rows have no entries
    const int lead = (int)(base & 3);
    // first stored kernel row and its input line (T), or the first covering window line (T^T)
    const int a_lo = TR ? axis_first_window(x, sh.k, sh.s, sh.p) : max(sh.p - sh.s * x, 0);
    const int i0 = sh.s * x + a_lo - sh.p;           // T only: input line of tap line a_lo

    // ---- generate: thread (row, part) writes the tap lines da = part, part + parts, ... of its row
    const int row = tid & (R - 1), part = tid / R, parts = kFillThreads / R;
    if (row < nrows) {
        const int r2 = rel[row + 1] - rel[row];
        const int u2 = ya + row;
        const int b_lo = TR ? axis_first_window(u2, sh.k, sh.s, sh.p) : max(sh.p - sh.s * u2, 0);
        const int off = r1 * rel[row] + lead;
        for (int da = part; da < r1; da += parts) {
            const int e = off + da * r2;
            if (TR) {
                // window (wx, wy) = (a_lo + da, b_lo + db) covers pixel (x, u2) with tap (x+p-s wx, u2+p-s wy)
                const int wx = a_lo + da;
                const int c = wx * sh.n_out + b_lo;
                const int kidx = (x + sh.p - sh.s * wx) * sh.k + (u2 + sh.p - sh.s * b_lo);
                for (int db = 0; db < r2; ++db) {
                    if (COLS) scol[e + db] = c + db;
                    sval[e + db] = ks[kidx - sh.s * db];
                }
            } else {
                const int c = (i0 + da) * sh.n + (sh.s * u2 + b_lo - sh.p);
                const int kidx = (a_lo + da) * sh.k + b_lo;
                for (int db = 0; db < r2; ++db) {
                    if (COLS) scol[e + db] = c + db;
                    sval[e + db] = ks[kidx + db];
                }
            }
        }
    }
    __syncthreads();

    // ---- copy out in quads aligned in the arrays; image position e + lead is array position base + e
    int *cdst = col_idx + (base - lead);
    float *vdst = vals + (base - lead);
    const int nquads = (total + lead + 3) >> 2;
    const bool aligned = (((COLS ? (uintptr_t)col_idx : 0) | (uintptr_t)vals) & 15u) == 0;
    for (int quad = tid; quad < nquads; quad += kFillThreads) {
        const int lo = quad * 4;
        if (aligned && lo >= lead && lo + 4 <= lead + total) {
            if (COLS) *reinterpret_cast<ivec4 *>(cdst + lo) = *reinterpret_cast<const ivec4 *>(scol + lo);
            *reinterpret_cast<fvec4 *>(vdst + lo) = *reinterpret_cast<const fvec4 *>(sval + lo);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = lo + i;
                if (e >= lead && e < lead + total) {
                    if (COLS) cdst[e] = scol[e];
                    vdst[e] = sval[e];
                }
            }
        }
    }
}

}  // namespace convspmv
