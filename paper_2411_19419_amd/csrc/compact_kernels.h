// Structure-aware storage of T and its product (gfx950).
//
// The paper closes (Sections 4.2 and 5) by pointing at sparse formats that use the
// block structure of C.  That structure, spelled out by Section 2 and Theorem 2.1:
// every value of T is one of the k*k kernel numbers, and the entries of row (x, y)
// are the r1(x) x r2(y) rectangle of taps that starts at (a_lo, b_lo) =
// (max(0, p - s x), max(0, p - s y)), at columns base + da*n + db, base being the
// column of the first one.  So T is stored as
//   desc[r] = { base, a_lo | r1 << 8 | b_lo << 16 | r2 << 24 }   (8 bytes per row;
//             {0, 0} for a row without entries)
//   ktab[a*k + b] = K[a][b]                                       (k*k floats)
// and entry (da, db) of row r is column base + da*n + db with value
// ktab[(a_lo + da)*k + b_lo + db].  Per stored entry this is 8/(r1 r2) bytes
// instead of 8.
//
// The product kernel keeps the marching layout of the CSR kernel (a workgroup
// walks down a strip of output columns with the input lines it needs in a ring of
// LDS lines) but has no entry stream to wait for, so the arithmetic decides its
// speed.  Two paths:
//   - the described path: every lane decodes the descriptor of its row and walks
//     the rectangle it describes, whatever it is (borders, any k and s, edited
//     descriptors; a tap whose column is not on a resident line is read from
//     global memory);
//   - the rectangle path, compiled in for common (k, s) at strides 1 and 2: the ring
//     holds the zero-padded plane, so when every row a wave holds is described
//     exactly as Theorem 2.1 says the window at its position must be (checked on
//     the descriptors read, not assumed), the full k x k sum over the padded plane
//     is the row's sum.  A lane then computes RV vertically adjacent outputs at
//     once: a pixel read from LDS feeds the taps of up to RV rows, the kernel
//     numbers sit in registers and the LDS offsets of a line's pixels are
//     immediates.
#pragma once
#include <type_traits>

#include "apply_march_kernel.h"
#include "build_kernels.h"

namespace convspmv {

// ---------------------------------------------------------------------------
// Build: one thread per row
// ---------------------------------------------------------------------------
constexpr int kCompactBuildThreads = 256;

__global__ __launch_bounds__(kCompactBuildThreads) void compact_rows_kernel(ConvShape sh, int2 *__restrict__ desc) {
    const int blocks_per_line = (sh.n_out + kCompactBuildThreads - 1) / kCompactBuildThreads;
    const int x = blockIdx.x / blocks_per_line;
    const int y = (blockIdx.x - x * blocks_per_line) * kCompactBuildThreads + (int)threadIdx.x;
    if (y >= sh.n_out) return;
    const int r1 = axis_taps(x, sh.m, sh.k, sh.s, sh.p), r2 = axis_taps(y, sh.n, sh.k, sh.s, sh.p);
    int2 d = make_int2(0, 0);
    if (r1 > 0 && r2 > 0) {
        // with r > 0 the first in-image tap is max(0, p - s t) < k
        const long long sx = (long long)sh.s * x, sy = (long long)sh.s * y;
        const int a_lo = sh.p > sx ? (int)(sh.p - sx) : 0, b_lo = sh.p > sy ? (int)(sh.p - sy) : 0;
        d.x = (int)((sx + a_lo - sh.p) * sh.n + (sy + b_lo - sh.p));
        d.y = (int)((unsigned)a_lo | (unsigned)r1 << 8 | (unsigned)b_lo << 16 | (unsigned)r2 << 24);
    }
    desc[(long long)x * sh.n_out + y] = d;
}

__global__ void compact_table_kernel(const float *__restrict__ kernel, float *__restrict__ ktab, int count) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < count) ktab[t] = kernel[t];
}

// ---------------------------------------------------------------------------
// Product
// ---------------------------------------------------------------------------
struct CompactGeom {
    int m, n, m_out, n_out, s, p, k;
    int batch;            // x / y row pitch, in floats
    int tw;               // output columns per strip (rectangle kernels: 256 / lanes per row)
    int strips;           // strips of tw output columns
    int seg;              // output lines per workgroup (a multiple of rv)
    int segs;             // segments per strip
    int blocks_per_xcd;
    int iw;               // input pixels a strip can touch: (TW-1)*s + k; also the LDS pixels per ring line
    int rv;               // output lines per step
    int nl;               // ring lines (power of two); 0: no ring, every tap is read from global memory
    int ktab_lds;         // 1: the table is copied to LDS behind the ring
    int c_base;           // first batch column of this launch (wide batches take several launches)
    int accum;            // 1: y += T x (second and later channels of a multi-channel sum)
};

constexpr int kCompactThreads = 256;

// KK, SS: kernel size and stride the rectangle path is compiled for (0, 0: described
// path only, k, s, rv, nl from the geometry).  LPR lanes share a row, each with 4
// batch columns (SCALAR: one lane, one column).  RV output lines per lane and step,
// NL ring lines, XLD registers per thread that carry the next step's input lines
// (0: the lines are copied after the step instead, behind a barrier; on the described path,
// whose ring holds the lines of one step only, the registers are written to LDS between two
// barriers after the step).  ACC: the rectangle
// path adds to y (a later channel of a multi-channel sum); a compile-time switch there, so that
// the single-channel kernel carries none of it; the described path looks at g.accum.
template <int KK, int SS, int LPR, bool SCALAR, int RV, int NL, int XLD, bool ACC>
__global__ __launch_bounds__(kCompactThreads, (KK == 0 && XLD > 0) ? 1 : 2) void spmm_compact_kernel(const int2 *__restrict__ desc,
                                                                          const float *__restrict__ ktab,
                                                                          const float *__restrict__ x,
                                                                          float *__restrict__ y, CompactGeom g) {
    using elem_t = typename std::conditional<SCALAR, float, vec4>::type;
    constexpr int NT = kCompactThreads, TW = NT / LPR;
    constexpr int NCOL = SCALAR ? 1 : 4 * LPR;
    constexpr bool FAST = KK > 0;
    static_assert(!SCALAR || LPR == 1, "scalar mode has one lane per row");
    static_assert(FAST ? (SS > 0 && RV > 0 && NL > 0 && SS * (2 * RV - 1) + KK <= NL) : (SS == 0 && RV == 0 && NL == 0),
                  "rectangle path needs compile-time geometry");
    static_assert(NL == 0 || (NL & (NL - 1)) == 0, "ring lines");
    extern __shared__ float4 smem[];
    elem_t *xs = reinterpret_cast<elem_t *>(smem);

    const int s = FAST ? SS : g.s, k = FAST ? KK : g.k;
    const int rv = FAST ? RV : g.rv;
    const bool ring = FAST || g.nl > 0;
    const int nlm = FAST ? NL - 1 : g.nl - 1;
    // elements per ring line; the host sets g.iw = (TW-1)*s + k, a constant of the rectangle kernels
    const int pitchE = FAST ? ((TW - 1) * SS + KK) * LPR : g.iw * LPR;
    const float *ks = reinterpret_cast<const float *>(xs + (nlm + 1) * pitchE);

    // ---- which strip segment (an XCD owns a band of output lines across all strips)
    const int local = blockIdx.x / kXcds;
    const int job = (blockIdx.x % kXcds) * g.blocks_per_xcd + local;
    if (local >= g.blocks_per_xcd || job >= g.strips * g.segs) return;      // uniform over the block
    const int sg = job / g.strips, tx = job - sg * g.strips;
    // Strip width: the rectangle kernels give every row of an output line to its own lanes; the
    // described path may take narrower strips (the ring then fits LDS at large strides) and
    // hands the lines of a step to the NT / (tw * LPR) groups of lanes in turn.
    const int tw = FAST ? TW : g.tw;
    const int y0 = tx * tw, xa = sg * g.seg, xb = min(xa + g.seg, g.m_out);
    const int twc = min(tw, g.n_out - y0);
    const int c0 = g.c_base + blockIdx.y * NCOL;
    const int tid = threadIdx.x, v = tid % LPR;
    const int line_lanes = tw * LPR, line_group = FAST ? 0 : tid / line_lanes, line_groups = FAST ? 1 : NT / line_lanes;
    const int yy = (FAST ? tid : tid - line_group * line_lanes) / LPR;

    // ---- the ring holds the zero-padded plane: line i (any sign) in slot i mod NL, pixels
    // j_lo .. j_lo + iw - 1 of it, zeros wherever (i, j) is not a pixel of the image
    const int j_lo = s * y0 - g.p;
    const float inv_pitchE = 1.0f / (float)pitchE;

    auto first_line = [&](int xo) { return s * xo - g.p; };
    auto end_line = [&](int xo) { return s * (xo + min(rv, xb - xo) - 1) - g.p + k; };   // of the step at xo

    auto fetch = [&](int i, int q) {               // element q of ring line i
        const int j = j_lo + q / LPR, vv = q % LPR;
        elem_t e = elem_t(0.0f);
        if (i >= 0 && i < g.m && j >= 0 && j < g.n)
            e = *(reinterpret_cast<const elem_t *>(x + ((long long)i * g.n + j) * g.batch + c0) + vv);
        return e;
    };
    // CU loads in flight per thread before the first is written to LDS; the rectangle kernels
    // take the lines of their first step in one round
    constexpr int CU = FAST ? (((RV - 1) * SS + KK) * ((TW - 1) * SS + KK) * LPR + NT - 1) / NT : 4;
    auto copy_lines = [&](int lo, int hi) {
        const int items = (hi - lo) * pitchE;
        for (int first = tid; first < items; first += CU * NT) {
            elem_t e[CU];
            int dst[CU];
#pragma unroll
            for (int u = 0; u < CU; ++u) {
                const int item = first + u * NT;
                dst[u] = -1;
                if (item < items) {
                    const int dl = div_small(item, inv_pitchE), q = item - dl * pitchE;
                    e[u] = fetch(lo + dl, q);
                    dst[u] = ((lo + dl) & nlm) * pitchE + q;
                }
            }
#pragma unroll
            for (int u = 0; u < CU; ++u)
                if (dst[u] >= 0) xs[dst[u]] = e[u];
        }
    };

    // ---- next step's lines: global -> registers during the step, registers -> LDS at its end.
    // Every thread always issues XLD loads (clamped addresses): with a fixed number of loads
    // in flight the waits on older loads (the descriptors of the current step) can leave
    // these outstanding; a load inside a branch would make every such wait a wait for all.
    constexpr int NX = XLD > 0 ? XLD : 1;
    elem_t xr[NX];
    int xdst[NX];                        // LDS element, -1: nothing to write, -2 - element: write zeros
    // Addresses are a wave-uniform 64-bit base (first line of the batch of lines) plus a 32-bit
    // byte offset per lane, built from per-thread constants with 24-bit multiplies; the host
    // admits this kernel only when a line of x is shorter than 2^24 bytes.
    const int row_bytes = g.n * g.batch * 4;
    int x_q[NX], x_dl[NX], x_coloff[NX];
    bool x_colok[NX];
#pragma unroll
    for (int r = 0; r < NX; ++r) {
        const int item = tid + r * NT;
        x_dl[r] = div_small(item, inv_pitchE);
        x_q[r] = item - x_dl[r] * pitchE;
        const int j = j_lo + x_q[r] / LPR, vv = x_q[r] % LPR, jc = min(max(j, 0), g.n - 1);
        x_colok[r] = j == jc;
        x_coloff[r] = jc * g.batch * 4 + vv * (int)sizeof(elem_t);
    }
    auto load_next = [&](int xo_next) {
        int items = 0, lo = 0;
        if (xo_next < xb) {
            lo = max(first_line(xo_next - 1) + k, first_line(xo_next));      // the step before was a full one
            items = max(end_line(xo_next) - lo, 0) * pitchE;
        }
        const int base_line = min(max(lo, 0), g.m - 1);
        const char *base = reinterpret_cast<const char *>(x) + ((long long)base_line * g.n * g.batch + c0) * 4;
#pragma unroll
        for (int r = 0; r < NX; ++r) {
            const int i = lo + x_dl[r], ic = min(max(i, 0), g.m - 1);
            const unsigned off = __umul24(ic - base_line, row_bytes) + x_coloff[r];
            xr[r] = *reinterpret_cast<const elem_t *>(base + off);
            const int slot = __umul24(i & nlm, pitchE) + x_q[r];
            xdst[r] = tid + r * NT >= items ? -1 : ((i == ic && x_colok[r]) ? slot : -2 - slot);
        }
    };
    auto store_next = [&]() {
#pragma unroll
        for (int r = 0; r < NX; ++r) {
            if (xdst[r] >= 0) xs[xdst[r]] = xr[r];
            else if (xdst[r] < -1) xs[-2 - xdst[r]] = elem_t(0.0f);
        }
    };

    auto fma_elem = [](elem_t &a, float wt, const elem_t &e) {
        if constexpr (SCALAR) {
            a = fmaf(wt, e, a);
        } else {
            a.x = fmaf(wt, e.x, a.x);
            a.y = fmaf(wt, e.y, a.y);
            a.z = fmaf(wt, e.z, a.z);
            a.w = fmaf(wt, e.w, a.w);
        }
    };
    const unsigned y_lane_off = (unsigned)yy * g.batch * 4 + v * (unsigned)sizeof(elem_t);
    auto y_row = [&](int xr_) {
        char *base = reinterpret_cast<char *>(y) + (((long long)xr_ * g.n_out + y0) * g.batch + c0) * 4;
        return reinterpret_cast<elem_t *>(base + y_lane_off);
    };
    auto store_y = [&](int xr_, const elem_t &a) { __builtin_nontemporal_store(a, y_row(xr_)); };

    // ---- described path: one row, whatever its descriptor says
    auto row_described = [&](int xr_, int2 d, int lo_step, int hi_step) {
        const unsigned w = (unsigned)d.y;
        const int a_lo = w & 255u, r1 = (w >> 8) & 255u, b_lo = (w >> 16) & 255u, r2 = w >> 24;
        const int i_first = d.x / g.n, j_first = d.x - i_first * g.n;
        elem_t acc = elem_t(0.0f);
        if (ring && g.ktab_lds && i_first >= lo_step && i_first + r1 <= hi_step && j_first >= j_lo &&
            j_first + r2 <= min(j_lo + g.iw, g.n)) {
            // the whole rectangle is on resident lines and inside one image line: no per-tap tests
            const float *kp = ks + a_lo * k + b_lo;
            const int lcol = (j_first - j_lo) * LPR + v;
            for (int da = 0; da < r1; ++da) {
                const elem_t *lp = xs + __umul24((i_first + da) & nlm, pitchE) + lcol;
                int db = 0;
                for (; db + 4 <= r2; db += 4) {      // four independent LDS reads in flight per trip
                    const elem_t e0 = lp[db * LPR], e1 = lp[(db + 1) * LPR], e2 = lp[(db + 2) * LPR], e3 = lp[(db + 3) * LPR];
                    const float k0 = kp[db], k1 = kp[db + 1], k2 = kp[db + 2], k3 = kp[db + 3];
                    fma_elem(acc, k0, e0);
                    fma_elem(acc, k1, e1);
                    fma_elem(acc, k2, e2);
                    fma_elem(acc, k3, e3);
                }
                for (; db < r2; ++db) fma_elem(acc, kp[db], lp[db * LPR]);
                kp += k;
            }
        } else {
            for (int da = 0; da < r1; ++da) {
                const int i = i_first + da;
                const bool line_in = ring && i >= lo_step && i < hi_step;
                const int kbase = (a_lo + da) * k + b_lo;
                const int lbase = (i & nlm) * pitchE + (j_first - j_lo) * LPR + v;
                for (int db = 0; db < r2; ++db) {
                    const float kv = g.ktab_lds ? ks[kbase + db] : ktab[kbase + db];
                    const int j = j_first + db;
                    elem_t e;
                    if (line_in && j >= j_lo && j < j_lo + g.iw && j < g.n)
                        e = xs[lbase + db * LPR];
                    else   // not on a resident line, or past the end of its line (the column then belongs to the next one)
                        e = *(reinterpret_cast<const elem_t *>(x + ((long long)d.x + (long long)da * g.n + db) * g.batch + c0) + v);
                    fma_elem(acc, kv, e);
                }
            }
        }
        if (g.accum) acc += *y_row(xr_);      // later channel of a multi-channel sum: y already holds the earlier ones
        store_y(xr_, acc);
    };

    // ---- rectangle path state
    constexpr int NK = FAST ? KK * KK : 1;
    constexpr int NR = FAST ? RV : 1;
    float kk[NK];
    int2 d_cur[NR], d_nxt[NR];
    const unsigned d_lane_off = (unsigned)min(yy, twc - 1) * 8u;
    auto load_desc = [&](int xo, int2 (&d)[NR]) {
#pragma unroll
        for (int j = 0; j < NR; ++j) {
            const int xr_ = min(xo + j, g.m_out - 1);
            const char *base = reinterpret_cast<const char *>(desc) + ((long long)xr_ * g.n_out + y0) * 8;
            d[j] = *reinterpret_cast<const int2 *>(base + d_lane_off);
        }
    };

    // What Theorem 2.1 says the descriptor of this lane's rows must be, split into the part that
    // depends on the output column (fixed for the lane) and the part that depends on the line.
    const int yl = y0 + yy;
    const int b_lo_e = max(g.p - s * yl, 0), r2_e = k - b_lo_e - max(s * yl + k - g.n - g.p, 0);
    const int lane_word = b_lo_e << 16 | r2_e << 24, lane_col = s * yl + b_lo_e - g.p;
    bool kfinite = true;

    auto compute = [&](int xo) {
        const int lo_step = first_line(xo), hi_step = end_line(xo);
        if constexpr (FAST) {
            constexpr int FULL = KK << 8 | KK << 24;
            bool ok = true;
#pragma unroll
            for (int j = 0; j < RV; ++j) {
                const int xr_ = xo + j;
                const bool present = xr_ < xb && yy < twc;
                const int a_lo_e = max(g.p - SS * xr_, 0), r1_e = KK - a_lo_e - max(SS * xr_ + KK - g.m - g.p, 0);
                const bool live = r1_e > 0 && r2_e > 0;
                const int word_e = live ? (a_lo_e | r1_e << 8 | lane_word) : 0;
                const int base_e = live ? (SS * xr_ + a_lo_e - g.p) * g.n + lane_col : 0;
                ok = ok && (!present || (d_cur[j].y == word_e && d_cur[j].x == base_e && (kfinite || word_e == FULL)));
            }
            if (__all(ok)) {
                // Every row the wave holds is described exactly as the window at its position: the
                // taps it stores are those that land on the image, and the ring holds zeros where
                // the others would land, so the full k x k sum over the padded plane is the row's
                // sum (all kernel numbers are finite, or no tap is missing).  Lanes without a row
                // compute on in-bounds LDS addresses and store nothing.
                const int i0 = SS * xo - g.p;
                const elem_t *lane_base = xs + SS * yy * LPR + v;
                constexpr int LINES = (RV - 1) * SS + KK;
                elem_t e[2][KK];
                elem_t acc[RV];
#pragma unroll
                for (int j = 0; j < RV; ++j) acc[j] = elem_t(0.0f);
                // A later channel of a multi-channel sum adds to what the earlier launches left in
                // y: requested here, used after the multiply-adds.
                elem_t yprev[ACC ? RV : 1];
                if constexpr (ACC) {
#pragma unroll
                    for (int j = 0; j < RV; ++j) {
                        yprev[j] = elem_t(0.0f);
                        if (xo + j < xb && yy < twc) yprev[j] = *y_row(xo + j);
                    }
                }
                auto read_line = [&](int di, elem_t (&dst)[KK]) {
                    const elem_t *src = lane_base + ((i0 + di) & (NL - 1)) * pitchE;
#pragma unroll
                    for (int b = 0; b < KK; ++b) dst[b] = src[b * LPR];
                };
                read_line(0, e[0]);
#pragma unroll
                for (int di = 0; di < LINES; ++di) {
                    if (di + 1 < LINES) read_line(di + 1, e[(di + 1) & 1]);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int j = 0; j < RV; ++j) {
                        const int a = di - j * SS;
                        if (a >= 0 && a < KK) {
#pragma unroll
                            for (int b = 0; b < KK; ++b) fma_elem(acc[j], kk[a * KK + b], e[di & 1][b]);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                // the stores below are conditional; without this the compiler sinks each row's
                // multiply-adds into its branch, behind all the LDS reads
#pragma unroll
                for (int j = 0; j < RV; ++j) {
                    if constexpr (SCALAR) asm volatile("" : "+v"(acc[j]));
                    else asm volatile("" : "+v"(acc[j].x), "+v"(acc[j].y), "+v"(acc[j].z), "+v"(acc[j].w));
                }
#pragma unroll
                for (int j = 0; j < RV; ++j)
                    if (xo + j < xb && yy < twc) store_y(xo + j, ACC ? acc[j] + yprev[j] : acc[j]);
            } else {
#pragma unroll
                for (int j = 0; j < RV; ++j)
                    if (xo + j < xb && yy < twc) row_described(xo + j, d_cur[j], lo_step, hi_step);
            }
        } else {
            if (yy < twc)
                for (int j = line_group; j < rv && xo + j < xb; j += line_groups)
                    row_described(xo + j, desc[(long long)(xo + j) * g.n_out + (y0 + yy)], lo_step, hi_step);
        }
    };

    // ---- the march
    if (ring) copy_lines(first_line(xa), end_line(xa));
    if (g.ktab_lds)
        for (int t = tid; t < k * k; t += NT) const_cast<float *>(ks)[t] = ktab[t];
    if constexpr (FAST) {
#pragma unroll
        for (int t = 0; t < NK; ++t)
            kk[t] = ktab[t];
#pragma unroll
        for (int t = 0; t < NK; ++t) kfinite = kfinite && __builtin_isfinite(kk[t]);
        // the k*k numbers stay in vector registers (there is room for them); as scalars they
        // crowd out the loop's addresses and bounds, which then travel through lane spills
#pragma unroll
        for (int t = 0; t < NK; ++t) asm volatile("" : "+v"(kk[t]));
        load_desc(xa, d_nxt);
    }
    __syncthreads();
    for (int xo = xa; xo < xb; xo += rv) {
        if constexpr (XLD > 0) load_next(xo + rv);
        if constexpr (FAST) {
#pragma unroll
            for (int j = 0; j < NR; ++j) d_cur[j] = d_nxt[j];
            load_desc(xo + rv, d_nxt);
        }
        compute(xo);
        if constexpr (XLD > 0 && FAST) {
            store_next();
            __syncthreads();
        } else if constexpr (XLD > 0) {
            __syncthreads();          // the ring holds this step's lines only: everyone has to be done with them
            store_next();
            __syncthreads();
        } else if (ring) {
            __syncthreads();
            if (xo + rv < xb) copy_lines(max(end_line(xo), first_line(xo + rv)), end_line(xo + rv));
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------
// Small products: G lanes per row, x from global memory
// ---------------------------------------------------------------------------
// A plane of a few ten thousand outputs gives the marching kernel fewer workgroups than the
// chip has compute units, and one lane per row leaves most of them idle.  Here G lanes share a
// row: lane l takes taps l, l + G, ... of the rectangle its descriptor describes (tap t is
// (da, db) = (t / r2, t mod r2), column base + da*n + db, value ktab[(a_lo + da)*k + b_lo + db]),
// the partial sums meet in a DPP butterfly, lane 0 of the group stores.  Whatever the descriptor
// says is what is summed.  blockIdx.y walks the batch columns (4 at a time, or one).
template <int G, bool SCALAR>
__global__ __launch_bounds__(kCompactThreads) void spmm_compact_gather_kernel(const int2 *__restrict__ desc,
                                                                             const float *__restrict__ ktab,
                                                                             const float *__restrict__ x,
                                                                             float *__restrict__ y, int rows, int n, int k,
                                                                             int batch, int accum) {
    using elem_t = typename std::conditional<SCALAR, float, vec4>::type;
    constexpr int NCOL = SCALAR ? 1 : 4;
    const long long row = ((long long)blockIdx.x * kCompactThreads + threadIdx.x) / G;
    const int lane = (int)threadIdx.x % G;
    int2 d = make_int2(0, 0);
    if (row < rows) d = desc[row];
    const unsigned w = (unsigned)d.y;
    const int a_lo = w & 255u, r1 = (w >> 8) & 255u, b_lo = (w >> 16) & 255u, r2 = w >> 24;
    const int cnt = r1 * r2;                               // at most 255 * 255: div_small is exact
    const float inv_r2 = 1.0f / (float)max(r2, 1);
    for (int c0 = blockIdx.y * NCOL; c0 < batch; c0 += gridDim.y * NCOL) {      // uniform over the block
        elem_t acc = elem_t(0.0f);
        for (int t = lane; t < cnt; t += G) {
            const int da = div_small(t, inv_r2), db = t - da * r2;
            const float kv = ktab[(a_lo + da) * k + b_lo + db];
            const elem_t e = *reinterpret_cast<const elem_t *>(x + ((long long)d.x + (long long)da * n + db) * batch + c0);
            if constexpr (SCALAR) {
                acc = fmaf(kv, e, acc);
            } else {
                acc.x = fmaf(kv, e.x, acc.x);
                acc.y = fmaf(kv, e.y, acc.y);
                acc.z = fmaf(kv, e.z, acc.z);
                acc.w = fmaf(kv, e.w, acc.w);
            }
        }
        // every lane of the wave is here (rows past the end have no taps)
        if constexpr (SCALAR) {
            acc = group_sum<G>(acc);
        } else {
            acc.x = group_sum<G>(acc.x);
            acc.y = group_sum<G>(acc.y);
            acc.z = group_sum<G>(acc.z);
            acc.w = group_sum<G>(acc.w);
        }
        if (row < rows && lane == 0) {
            elem_t *dst = reinterpret_cast<elem_t *>(y + row * batch + c0);
            if (accum) acc += *dst;       // later channel of a multi-channel sum
            *dst = acc;
        }
    }
}

}  // namespace convspmv
