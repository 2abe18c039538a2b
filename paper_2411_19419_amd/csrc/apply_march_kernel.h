// Marching SpMM over the stored CSR arrays: a persistent workgroup walks down a
// strip of TW output columns, keeps the input lines its rows of T can touch in
// a ring of LDS lines, and streams col_idx / vals exactly once.
//
// Why this shape.  At batch 16 the entries of T are 3/4 of all bytes and are
// used once; every x row is used by about (k/s)^2 rows of T.  Measurements of
// the tile-at-a-time variant (apply_tile_kernel.h) showed the arithmetic and
// the LDS traffic hidden behind the loads, and the time going to the start of
// every tile: load the window, barrier, only then start the entry stream.
// Here a workgroup never restarts: while the waves work on output lines
// x .. x+LS-1 the input lines needed by the next LS output lines are already
// being loaded (into registers, written to LDS just before the barrier that
// ends the step), and the entry loads of the next row group are always one
// pass ahead of the arithmetic.  Consecutive output lines share k-s input
// lines, so x is read from global memory about once, plus the column halo.
//
// Work mapping (as in the tile kernel): G consecutive lanes share one row of T,
// lane l takes entries l, l+G, ...; a wave covers 64/G neighbouring rows per
// pass, wave w of the workgroup owns columns [w*64/G, (w+1)*64/G) of the strip
// on every output line.  Each lane keeps 4*NV batch columns of partial sums,
// combined at the end of a pass by a DPP reduce-scatter so that a wave stores
// 64/G complete, contiguous y rows.
//
// The kernel is a CSR product: the LDS address of a stored column is computed
// from its value, and an entry whose column is not among the resident lines
// (possible only if the arrays were edited) is taken from global memory.
#pragma once
#include <type_traits>

#include "apply_tile_kernel.h"

namespace convspmv {

typedef float vec4 __attribute__((ext_vector_type(4)));

// The same kernel applies T^T (built by conv_csc_build): there the operand is a vector of
// output size, the result has input size, and result line i needs the operand lines
// (window lines) x with 0 <= i + p - s x < k instead of the input lines of a window.
struct MarchGeom {
    int m, n;             // operand: lines and pixels per line (the image for T, the window grid for T^T)
    int m_out, n_out;     // result: lines and pixels per line
    int s, p, k;
    int tr;               // 1: the matrix is T^T
    int batch;            // x / y row pitch, in floats
    int nnz;
    int strips;           // strips of TW output columns
    int seg;              // output lines per workgroup
    int segs;             // segments per strip
    int blocks_per_xcd;   // strips * segs split evenly over the XCDs (rounded up)
    int iw;               // operand columns a strip can touch (upper bound): (TW-1)*s + k, or (TW-2+k)/s + 2 for T^T
    int iw_pitch;         // LDS pixels per ring line (>= iw)
    float inv_n;          // 1.0f / n
    int accum;            // 1: add to y instead of storing (later channels of a multi-channel sum)
    int col_blocks;       // blocks of batch columns (4*NV each, or 1): batch / (4*NV), or batch
    int max_row;          // most entries a row of the matrix has
    int channels;         // input channels walked inside one launch (spmm_stage_march_kernel with MC), else 1
    long long x_plane;    // floats between the x planes of two channels
};

// NV: float4 column chunks per lane (NV planes in LDS, 4*NV batch columns per
// launch column block), or 0 for one scalar column per launch column block
// (SpMV: one plane of floats).  NL: ring lines (power of two, >= s*(2*LS-1) + k).
// LS: output lines per step (1 or 2).  XLD: registers (float4, or float when
// NV = 0) per thread that carry the next step's input lines.  CS: LDS pixels
// per plane (> NL*iw_pitch).
template <int G, int NIT, int NV, int TW, int NL, int LS, int XLD, int CS>
__global__ __launch_bounds__(512, 4) void spmm_march_kernel(const int *__restrict__ row_ptr,
                                                            const int *__restrict__ col_idx,
                                                            const float *__restrict__ vals,
                                                            const float *__restrict__ x, float *__restrict__ y,
                                                            MarchGeom g) {
    constexpr int RW = kWave / G;        // rows per wave pass
    constexpr bool SCALAR = NV == 0;
    constexpr int NP = SCALAR ? 1 : NV;           // LDS planes
    constexpr int NVAL = SCALAR ? 1 : 4 * NV;     // batch columns per lane
    constexpr int SH = SCALAR ? 2 : 4;            // log2 of the LDS bytes per pixel and plane
    constexpr int PIXB = 1 << SH;
    using elem_t = typename std::conditional<SCALAR, float, vec4>::type;   // one pixel of one plane
    constexpr int NTHREADS = 512;
    constexpr int SCAT = ilog2(G) < ilog2(NVAL) ? ilog2(G) : ilog2(NVAL);
    constexpr int CNT = NVAL >> SCAT;             // finished columns per storing lane
    constexpr int DUP = ilog2(G) - SCAT;          // low lane bits that end up with copies
    static_assert(G == 4 || G == 8 || G == 16, "group width");
    static_assert(NTHREADS / kWave == TW / RW, "one wave per group of RW columns");
    static_assert((NL & (NL - 1)) == 0 && (LS == 1 || LS == 2), "ring / step shape");
    extern __shared__ float4 smem[];
    elem_t *xs = reinterpret_cast<elem_t *>(smem);   // [NP planes][CS pixels]; pixel (line i, column j) at (i % NL)*pitch + (j - j0)

    // ---- which strip segment (XCD-aware: an XCD owns a band of output lines across all strips) and
    // which block of batch columns.  The column blocks of one segment are consecutive workgroups of
    // one XCD: they read the same entries at about the same time, so all but one find them in its L2.
    const int turn = blockIdx.x / kXcds;
    const int local = turn / g.col_blocks, col_block = turn - local * g.col_blocks;
    const int job = (blockIdx.x % kXcds) * g.blocks_per_xcd + local;
    if (local >= g.blocks_per_xcd || job >= g.strips * g.segs) return;      // uniform over the block
    const int sg = job / g.strips, tx = job - sg * g.strips;
    const int y0 = tx * TW, xa = sg * g.seg, xb = min(xa + g.seg, g.m_out);
    const int twc = min(TW, g.n_out - y0);
    const int c0 = col_block * NVAL;
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int gl = lane % G, gr = lane / G;

    // ---- input columns of the strip, clipped to the image
    // first window position along an axis that covers coordinate t (T^T), never negative
    auto first_window = [&](int t) {
        const int num = t + g.p - g.k + 1;
        return num > 0 ? (num + g.s - 1) / g.s : 0;
    };
    const int j_lo = g.tr ? first_window(y0) : g.s * y0 - g.p;
    const int j0 = min(max(j_lo, 0), g.n - 1);
    const int iwc = max(min(j_lo + g.iw, g.n) - j0, 0);
    const float inv_iwc = 1.0f / (float)max(iwc, 1);
    const int zslot = NL * g.iw_pitch;            // a pixel of zeros in every plane

    // first / one-past-last input line that output lines [xo, xo + cnt) can touch, clipped
    auto line_lo = [&](int xo) { return min(max(g.tr ? first_window(xo) : g.s * xo - g.p, 0), g.m); };
    auto line_hi = [&](int xo, int cnt) {
        const int last = xo + cnt - 1;
        return min(max(g.tr ? (last + g.p) / g.s + 1 : g.s * last - g.p + g.k, 0), g.m);
    };

    // ---- per-lane row of T on output line xo: bounds, clamped so that every lane holds
    // valid, ascending entry indices (a lane without a row gets an empty range)
    struct Bounds { int beg, end; };
    auto load_bounds = [&](int xo) {
        const int yy = wave * RW + gr;
        const bool valid = xo < xb && yy < twc;
        const long long r = (long long)min(xo, xb - 1) * g.n_out + y0 + min(yy, twc - 1);
        Bounds b;
        b.beg = row_ptr[r];
        b.end = row_ptr[r + 1];
        if (!valid) b.beg = b.end;
        return b;
    };

    struct Pass {
        int c[NIT];
        float v[NIT];
        int beg, end;
    };
    auto fetch = [&](const Bounds &b, Pass &ps) {
        ps.beg = b.beg;
        ps.end = b.end;
        const int span_base = __builtin_amdgcn_readfirstlane(b.beg);
        const int span_end = __builtin_amdgcn_readlane(b.end, kWave - 1);
        const int *cb = col_idx + span_base;
        const float *vb = vals + span_base;
        const unsigned off = (unsigned)(b.beg - span_base + gl) * 4u;
        // Both branches issue exactly 2*NIT loads and contain no lane-dependent
        // control flow, so the number of loads in flight is the same on every
        // path and later waits can leave the newest pass outstanding.
        if ((long long)span_end + NIT * G <= g.nnz) {
            // every slot of every lane lies inside the arrays: slots past the end of
            // a row fetch entries of later rows, which the arithmetic ignores
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                ps.c[it] = stream_load_i(cb, off + it * G * 4);
                ps.v[it] = stream_load_f(vb, off + it * G * 4);
            }
        } else {
            // the last rows of T: clamp to the last entry
            const unsigned last = (unsigned)(g.nnz - 1 - span_base) * 4u;
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const unsigned o = min(off + it * G * 4, last);
                ps.c[it] = stream_load_i(cb, o);
                ps.v[it] = stream_load_f(vb, o);
            }
        }
    };

    // Window state of the current step (wave-uniform).  Offsets are in bytes of LDS
    // (PIXB per pixel, the suffix B below): dB = PIXB * (col - cbase) = PIXB * (di * n + dj)
    // for a column on line ibase + di at strip pixel dj; ibase is a multiple of NL, so the
    // ring slot of the line is di % NL.  The host guarantees m*n <= 2^27 (col*16 fits an
    // int) and 2*NL*n*16 <= 2^25, which keeps dB (a multiple of PIXB below 2^25) exact in
    // fp32 and the quotient by n exact after one fused multiply-add and a truncation.
    const int nB = g.n * PIXB, pitchB = g.iw_pitch * PIXB, zslotB = zslot * PIXB;
    const unsigned iwcB = (unsigned)iwc * PIXB;
    const float inv_nB = g.inv_n / (float)PIXB, half_inv_n = 0.5f * g.inv_n;
    int cbaseB = 0, loB = 0;
    unsigned spanB = 0;
    auto set_window = [&](int xo) {
        const int lo = line_lo(xo), hi = line_hi(xo, LS);
        const int ibase = lo & ~(NL - 1);
        cbaseB = (ibase * g.n + j0) * PIXB;
        loB = (lo - ibase) * nB;
        spanB = (unsigned)(hi - lo) * (unsigned)nB;
    };
    auto fma_elem = [](float *a, float wt, const elem_t &e) {
        if constexpr (SCALAR) {
            a[0] = fmaf(wt, e, a[0]);
        } else {
            a[0] = fmaf(wt, e.x, a[0]);
            a[1] = fmaf(wt, e.y, a[1]);
            a[2] = fmaf(wt, e.z, a[2]);
            a[3] = fmaf(wt, e.w, a[3]);
        }
    };

    auto compute = [&](int xo, const Pass &ps) {
        float acc[NVAL];
#pragma unroll
        for (int i = 0; i < NVAL; ++i) acc[i] = 0.0f;
        bool stray = false;              // an in-row entry whose column is not on a resident line
        const int rem = ps.end - ps.beg - gl;     // slot it belongs to the row iff it*G < rem
        int addr[NIT];
        float w[NIT];
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const bool act = it * G < rem;
            const int dB = (ps.c[it] << SH) - cbaseB;
            const int di = (int)fmaf((float)dB, inv_nB, half_inv_n);
            const int djB = dB - __mul24(di, nB);
            const bool in = (unsigned)(dB - loB) < spanB && (unsigned)djB < iwcB;
            stray |= act && !in;
            addr[it] = (act && in) ? __mul24(di & (NL - 1), pitchB) + djB : zslotB;
            w[it] = (act && in) ? ps.v[it] : 0.0f;
        }
        // LDS reads run one entry ahead of the multiply-adds, and no further: the
        // scheduler is kept from hoisting all reads of a pass to its start, which
        // would cost 16 registers per entry.
        elem_t xv[2][NP];
        auto read_x = [&](int it, elem_t (&dst)[NP]) {
            const elem_t *src = reinterpret_cast<const elem_t *>(reinterpret_cast<const char *>(xs) + addr[it]);
#pragma unroll
            for (int v = 0; v < NP; ++v) dst[v] = src[v * CS];
        };
        read_x(0, xv[0]);
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            if (it + 1 < NIT) read_x(it + 1, xv[(it + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int v = 0; v < NP; ++v) fma_elem(acc + 4 * v, w[it], xv[it & 1][v]);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (__builtin_expect(__any(stray), 0)) {
            // cold: some stored column is not on a resident line; take those from global memory
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const bool act = it * G < rem;
                const int dB = (ps.c[it] << SH) - cbaseB;
                const int di = (int)fmaf((float)dB, inv_nB, half_inv_n);
                const int djB = dB - __mul24(di, nB);
                const bool in = (unsigned)(dB - loB) < spanB && (unsigned)djB < iwcB;
                if (act && !in) {
                    const elem_t *src = reinterpret_cast<const elem_t *>(x + (long long)ps.c[it] * g.batch + c0);
#pragma unroll
                    for (int v = 0; v < NP; ++v) fma_elem(acc + 4 * v, ps.v[it], src[v]);
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

        // lanes whose DUP low bits are clear hold CNT finished columns of their row,
        // starting at column (gl >> DUP) * CNT of this launch's column block
        const int yy = wave * RW + gr;
        if (xo < xb && yy < twc && (gl & ((1 << DUP) - 1)) == 0) {
            float *dst = y + ((long long)xo * g.n_out + (y0 + yy)) * g.batch + c0 + (gl >> DUP) * CNT;
            store_row<CNT>(dst, acc, g.accum != 0);
        }
    };

    // ---- input lines of the next step: global -> registers now, registers -> LDS at the
    // end of the step.  Always XLD loads per thread (clamped addresses) so that the
    // number of loads in flight does not depend on the position in the image.
    elem_t xr[XLD];
    int xdst[XLD];                       // LDS pixel index, or -1
    auto load_next_lines = [&](int xo_next) {
        const int lo = line_hi(xo_next - LS, LS), hi = line_hi(xo_next, LS);   // new lines [lo, hi)
        const int items = xo_next < xb ? (hi - lo) * iwc * NP : 0;
#pragma unroll
        for (int r = 0; r < XLD; ++r) {
            const int item = tid + r * NTHREADS;
            const int q = item / NP, v = item % NP;
            const int dl = div_small(q, inv_iwc), dj = min(q - dl * iwc, max(iwc - 1, 0));
            const int i = min(lo + dl, g.m - 1);
            const elem_t *src = reinterpret_cast<const elem_t *>(x + ((long long)i * g.n + (j0 + dj)) * g.batch + c0);
            xr[r] = src[v];
            xdst[r] = item < items ? v * CS + (i & (NL - 1)) * g.iw_pitch + dj : -1;
        }
    };
    auto store_next_lines = [&]() {
#pragma unroll
        for (int r = 0; r < XLD; ++r)
            if (xdst[r] >= 0) xs[xdst[r]] = xr[r];
    };

    // ---- the march.  Output line xa + i is pass i of every wave; passes come in pairs
    // (two entry register sets), LS passes form a step.
    const int npass = (xb - xa + 1) & ~1;
    // The first bounds and entries are requested before the first input lines, so that the
    // two round trips of the entry stream (row_ptr, then entries) overlap the window load.
    Bounds b_next = load_bounds(xa), b_next2 = load_bounds(xa + 1);
    Pass pa, pb;
    fetch(b_next, pa);
    {   // lines of the first step -> LDS
        const int lo = line_lo(xa), hi = line_hi(xa, LS);
        const int items = (hi - lo) * iwc * NP;
        for (int item = tid; item < items; item += NTHREADS) {
            const int q = item / NP, v = item % NP;
            const int dl = div_small(q, inv_iwc), dj = q - dl * iwc;
            const int i = lo + dl;
            const elem_t *src = reinterpret_cast<const elem_t *>(x + ((long long)i * g.n + (j0 + dj)) * g.batch + c0);
            xs[v * CS + (i & (NL - 1)) * g.iw_pitch + dj] = src[v];
        }
        if (tid < NP) xs[tid * CS + zslot] = elem_t(0.0f);
    }
    __syncthreads();

    for (int i = 0; i < npass; i += 2) {
        const int xo = xa + i;
        // -- pass i (entries in pa)
        set_window(xo);
        load_next_lines(xo + LS);
        b_next = b_next2;
        b_next2 = load_bounds(xo + 2);
        fetch(b_next, pb);
        __builtin_amdgcn_sched_barrier(0);       // keep the loads of the next pass ahead of this pass's arithmetic
        compute(xo, pa);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (LS == 1) {
            store_next_lines();
            __syncthreads();
            set_window(xo + 1);
            load_next_lines(xo + 2);
        }
        // -- pass i + 1 (entries in pb)
        b_next = b_next2;
        b_next2 = load_bounds(xo + 3);
        fetch(b_next, pa);
        __builtin_amdgcn_sched_barrier(0);
        compute(xo + 1, pb);
        __builtin_amdgcn_sched_barrier(0);
        store_next_lines();
        __syncthreads();
    }
}

}  // namespace convspmv
