/*
 * conv_oracle.c -- CPU oracle for zero-padded, strided 2-D convolution and for
 * the sparse transformation matrix T = C P that represents it.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the
 * smoke check and the benchmark's CPU-baseline leg may call it.  It shares no
 * code, header, table or helper with the GPU library and must never be used
 * as a fallback for it.
 *
 * Everything here is the plain definition written out, slow and obvious:
 *
 *   - the convolution result is "surround A with p zeros on every side, then
 *     slide the k x k kernel with stride s" (paper, Section 1 and the opening
 *     of Section 2).  Kernel row j acts on input row j of the window and
 *     kernel column b on window column b: no flip (Section 2, the first row
 *     of C places K_11..K_1k on the first k columns of the padded input).
 *   - vec() is row-major (Section 2, the definition of vec(A)); output pixel
 *     (x, y) is row x*n_out + y of T (rows of R are horizontal slides, block
 *     rows of C are vertical slides).
 *   - m_out, n_out follow Theorem 2.1; so does the closed-form count, which
 *     is evaluated here as the literal double sum.
 *
 * Floating point: products and sums are carried in double and rounded to
 * float once per output.  A float*float product is exact in double, so the
 * only rounding before the final one is in the at most k*k additions.
 *
 * Batch layout (not in the paper, which treats one vector): B vectors that
 * share T are stored batch-minor, element (pixel q, column c) at q*B + c.
 * With B = 1 this is the paper's vec(A).
 *
 * Pins (tests/test_oracle_pins.py): hand-worked examples, closed forms for
 * "same" and unpadded convolutions, brute-force counting against Theorem 2.1,
 * the paper's dense P and C multiplied out, scipy's correlate2d on the padded
 * plane, linearity / delta-kernel / stride-subsampling invariants.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

static int64_t imax64(int64_t a, int64_t b) { return a > b ? a : b; }

/* Theorem 2.1: output extent along one axis, or 0 when the precondition
 * k <= extent + 2p fails (or an argument is out of range). */
static int64_t out_extent(int64_t extent, int64_t k, int64_t s, int64_t p)
{
    if (extent < 1 || k < 1 || s < 1 || p < 0) return 0;
    if (k > extent + 2 * p) return 0;
    return (extent + 2 * p - k) / s + 1;
}

int oracle_out_shape(int m, int n, int k, int s, int p, int64_t *m_out, int64_t *n_out)
{
    int64_t mo = out_extent(m, k, s, p), no = out_extent(n, k, s, p);
    if (mo == 0 || no == 0) return -1;
    *m_out = mo;
    *n_out = no;
    return 0;
}

/* Theorem 2.1, c_1(x) (pass extent = m) or c_2(y) (extent = n): number of
 * kernel rows (columns) that fall on padding at slide position t. */
static int64_t c_pad(int64_t t, int64_t extent, int64_t k, int64_t s, int64_t p)
{
    return imax64(0, p - s * t) + imax64(0, s * t + k - extent - p);
}

/* Theorem 2.1 as printed: the double sum over all window positions. */
int64_t oracle_nnz_closed(int m, int n, int k, int s, int p)
{
    int64_t mo, no;
    if (oracle_out_shape(m, n, k, s, p, &mo, &no) != 0) return -1;
    int64_t total = 0;
    for (int64_t x = 0; x < mo; ++x)
        for (int64_t y = 0; y < no; ++y)
            total += imax64(0, k - c_pad(x, m, k, s, p)) * imax64(0, k - c_pad(y, n, k, s, p));
    return total;
}

/* Brute force, sharing nothing with the formula: paint a 0/1 plane that is 1
 * exactly where the padded input holds an entry of A, slide the window over
 * it and count the ones it sees. */
int64_t oracle_nnz_brute(int m, int n, int k, int s, int p)
{
    int64_t mo, no;
    if (oracle_out_shape(m, n, k, s, p, &mo, &no) != 0) return -1;
    int64_t H = (int64_t)m + 2 * p, W = (int64_t)n + 2 * p;
    unsigned char *inside = (unsigned char *)calloc((size_t)(H * W), 1);
    if (!inside) return -2;
    for (int64_t i = 0; i < m; ++i)
        for (int64_t j = 0; j < n; ++j)
            inside[(i + p) * W + (j + p)] = 1;
    int64_t total = 0;
    for (int64_t x = 0; x < mo; ++x)
        for (int64_t y = 0; y < no; ++y)
            for (int64_t a = 0; a < k; ++a)
                for (int64_t b = 0; b < k; ++b)
                    total += inside[(s * x + a) * W + (s * y + b)];
    free(inside);
    return total;
}

/* One row of T = C P.  Row x*n_out + y of C holds K[a][b] at padded position
 * (s x + a, s y + b); P sends input pixel (i, j) to padded position
 * (i + p, j + p) and nothing to the border.  So the row keeps the taps whose
 * padded position is inside the copy of A, at column i*n + j.  Taps are
 * visited in (a, b) raster order, which is ascending column order.  Every such
 * tap is stored, whatever the value of K[a][b] (T is structural).
 * Returns the number of entries written to cols[] / vals[] (each k*k long). */
int64_t oracle_csr_row(int m, int n, int k, int s, int p, const float *K,
                       int64_t row, int64_t *cols, float *vals)
{
    int64_t mo, no;
    if (oracle_out_shape(m, n, k, s, p, &mo, &no) != 0) return -1;
    if (row < 0 || row >= mo * no) return -1;
    int64_t x = row / no, y = row % no, cnt = 0;
    for (int64_t a = 0; a < k; ++a) {
        for (int64_t b = 0; b < k; ++b) {
            int64_t ip = s * x + a, jp = s * y + b;       /* padded coordinates */
            if (ip < p || ip >= p + m || jp < p || jp >= p + n) continue;
            cols[cnt] = (ip - p) * n + (jp - p);
            vals[cnt] = K[a * k + b];
            ++cnt;
        }
    }
    return cnt;
}

/* All of T in CSR.  row_ptr has m_out*n_out + 1 entries; col_idx and vals
 * must have room for cap entries.  Returns nnz, or -3 if cap is too small. */
int64_t oracle_csr(int m, int n, int k, int s, int p, const float *K,
                   int64_t *row_ptr, int64_t *col_idx, float *vals, int64_t cap)
{
    int64_t mo, no;
    if (oracle_out_shape(m, n, k, s, p, &mo, &no) != 0) return -1;
    int64_t *cbuf = (int64_t *)malloc(sizeof(int64_t) * (size_t)k * k);
    float *vbuf = (float *)malloc(sizeof(float) * (size_t)k * k);
    if (!cbuf || !vbuf) { free(cbuf); free(vbuf); return -2; }
    int64_t at = 0;
    for (int64_t r = 0; r < mo * no; ++r) {
        row_ptr[r] = at;
        int64_t c = oracle_csr_row(m, n, k, s, p, K, r, cbuf, vbuf);
        if (at + c > cap) { free(cbuf); free(vbuf); return -3; }
        memcpy(col_idx + at, cbuf, sizeof(int64_t) * (size_t)c);
        memcpy(vals + at, vbuf, sizeof(float) * (size_t)c);
        at += c;
    }
    row_ptr[mo * no] = at;
    free(cbuf);
    free(vbuf);
    return at;
}

/* The convolution itself, by definition: explicit zero-padded copy, then the
 * direct strided sliding-window sum.
 *   A     : m*n*B floats, batch-minor.
 *   K     : k*k floats, row-major.
 *   out   : m_out*n_out*B floats, batch-minor.
 *   scale : optional (may be NULL), m_out*n_out*B doubles: sum of |K||A_pad|
 *           over the window, the natural error scale of the dot product.
 * Parallel over output lines when built with OpenMP; each output is computed
 * by one thread in a fixed order, so results do not depend on thread count. */
int oracle_conv(int m, int n, int k, int s, int p, int B,
                const float *A, const float *K, float *out, double *scale)
{
    int64_t mo, no;
    if (B < 1 || oracle_out_shape(m, n, k, s, p, &mo, &no) != 0) return -1;
    int64_t H = (int64_t)m + 2 * p, W = (int64_t)n + 2 * p;
    float *Apad = (float *)calloc((size_t)(H * W * B), sizeof(float));
    if (!Apad) return -2;
    for (int64_t i = 0; i < m; ++i)
        memcpy(Apad + ((i + p) * W + p) * B, A + i * n * B, sizeof(float) * (size_t)n * B);

#pragma omp parallel for schedule(static)
    for (int64_t x = 0; x < mo; ++x) {
        for (int64_t y = 0; y < no; ++y) {
            for (int64_t c = 0; c < B; ++c) {
                double acc = 0.0, mag = 0.0;
                for (int64_t a = 0; a < k; ++a) {
                    for (int64_t b = 0; b < k; ++b) {
                        double kv = (double)K[a * k + b];
                        double av = (double)Apad[((s * x + a) * W + (s * y + b)) * B + c];
                        acc += kv * av;
                        mag += fabs(kv) * fabs(av);
                    }
                }
                out[(x * no + y) * B + c] = (float)acc;
                if (scale) scale[(x * no + y) * B + c] = mag;
            }
        }
    }
    free(Apad);
    return 0;
}

/* ------------------------------------------------------------------------
 * The transposed transformation.  The paper's experiments also store T
 * column-compressed (CSC, Section 3 and Section 4.1); the CSC arrays of T are
 * the CSR arrays of T^T, and T^T = P^T C^T applied to a vector u of output
 * size is the adjoint of the convolution: C^T scatters K[a][b] * u[x][y] onto
 * padded position (s x + a, s y + b), P^T keeps the part of the padded plane
 * that holds A (drops the border).
 * ------------------------------------------------------------------------ */

/* CSC of T = CSR of T^T, by transposing the enumerated CSR with a stable
 * counting sort: entries are visited in row-major order of T, so inside a
 * column they come out in ascending row order.  col_ptr has m*n + 1 entries,
 * row_idx and vals need nnz entries.  Returns nnz or a negative status. */
int64_t oracle_csc(int m, int n, int k, int s, int p, const float *K,
                   int64_t *col_ptr, int64_t *row_idx, float *vals, int64_t cap)
{
    int64_t mo, no;
    if (oracle_out_shape(m, n, k, s, p, &mo, &no) != 0) return -1;
    int64_t rows = mo * no, cols = (int64_t)m * n;
    int64_t *cbuf = (int64_t *)malloc(sizeof(int64_t) * (size_t)k * k);
    float *vbuf = (float *)malloc(sizeof(float) * (size_t)k * k);
    int64_t *next = (int64_t *)calloc((size_t)cols + 1, sizeof(int64_t));
    if (!cbuf || !vbuf || !next) { free(cbuf); free(vbuf); free(next); return -2; }
    for (int64_t r = 0; r < rows; ++r) {                  /* count per column */
        int64_t c = oracle_csr_row(m, n, k, s, p, K, r, cbuf, vbuf);
        for (int64_t e = 0; e < c; ++e) next[cbuf[e] + 1] += 1;
    }
    col_ptr[0] = 0;
    for (int64_t j = 0; j < cols; ++j) col_ptr[j + 1] = col_ptr[j] + next[j + 1];
    int64_t nnz = col_ptr[cols];
    if (nnz > cap) { free(cbuf); free(vbuf); free(next); return -3; }
    for (int64_t j = 0; j < cols; ++j) next[j] = col_ptr[j];
    for (int64_t r = 0; r < rows; ++r) {                  /* place, rows ascending */
        int64_t c = oracle_csr_row(m, n, k, s, p, K, r, cbuf, vbuf);
        for (int64_t e = 0; e < c; ++e) {
            int64_t at = next[cbuf[e]]++;
            row_idx[at] = r;
            vals[at] = vbuf[e];
        }
    }
    free(cbuf); free(vbuf); free(next);
    return nnz;
}

/* z = T^T u by definition: scatter every tap of every window onto a padded
 * plane of doubles, then crop the border.
 *   U     : m_out*n_out*B floats, batch-minor.
 *   out   : m*n*B floats, batch-minor.
 *   scale : optional, m*n*B doubles: the same sums with absolute values.
 * Parallel over batch columns only (each column has its own plane); every
 * output is summed in a fixed order. */
int oracle_conv_t(int m, int n, int k, int s, int p, int B,
                  const float *U, const float *K, float *out, double *scale)
{
    int64_t mo, no;
    if (B < 1 || oracle_out_shape(m, n, k, s, p, &mo, &no) != 0) return -1;
    int64_t H = (int64_t)m + 2 * p, W = (int64_t)n + 2 * p;
    int fail = 0;
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < B; ++c) {
        double *plane = (double *)calloc((size_t)(H * W), sizeof(double));
        double *mag = (double *)calloc((size_t)(H * W), sizeof(double));
        if (!plane || !mag) { fail = 1; free(plane); free(mag); continue; }
        for (int64_t x = 0; x < mo; ++x)
            for (int64_t y = 0; y < no; ++y) {
                double uv = (double)U[(x * no + y) * B + c];
                for (int64_t a = 0; a < k; ++a)
                    for (int64_t b = 0; b < k; ++b) {
                        double kv = (double)K[a * k + b];
                        plane[(s * x + a) * W + (s * y + b)] += kv * uv;
                        mag[(s * x + a) * W + (s * y + b)] += fabs(kv) * fabs(uv);
                    }
            }
        for (int64_t i = 0; i < m; ++i)
            for (int64_t j = 0; j < n; ++j) {
                out[(i * n + j) * B + c] = (float)plane[(i + p) * W + (j + p)];
                if (scale) scale[(i * n + j) * B + c] = mag[(i + p) * W + (j + p)];
            }
        free(plane);
        free(mag);
    }
    return fail ? -2 : 0;
}

/* ---- structure-aware storage of T (the "more efficient sparse representation"
 * the paper leaves to future work, Sections 4.2 and 5) ------------------------
 *
 * Every value of T is one of the k*k kernel numbers, and the entries of row
 * (x, y) are the taps a in [a_lo, a_lo + r1), b in [b_lo, b_lo + r2) that land
 * on A (Theorem 2.1: r1 = k - c1(x), r2 = k - c2(y)), at columns
 * base + da*n + db with base the column of the first one.  The compact storage
 * keeps, per row, the pair
 *     desc[2r]     = base                     (0 for a row without entries)
 *     desc[2r + 1] = a_lo | r1 << 8 | b_lo << 16 | r2 << 24   (0 likewise)
 * and once the table ktab[a*k + b] = K[a][b].  It needs k <= 255.
 *
 * oracle_compact_rows finds the ranges by testing every tap against the border,
 * the same test oracle_csr_row makes.  Returns the number of rows, < 0 on error. */
int64_t oracle_compact_rows(int m, int n, int k, int s, int p, int32_t *desc)
{
    int64_t mo, no;
    if (oracle_out_shape(m, n, k, s, p, &mo, &no) != 0) return -1;
    if (k > 255) return -1;
    for (int64_t x = 0; x < mo; ++x)
        for (int64_t y = 0; y < no; ++y) {
            int64_t a_lo = -1, r1 = 0, b_lo = -1, r2 = 0;
            for (int64_t a = 0; a < k; ++a) {
                int64_t ip = s * x + a;
                if (ip < p || ip >= p + m) continue;
                if (a_lo < 0) a_lo = a;
                ++r1;
            }
            for (int64_t b = 0; b < k; ++b) {
                int64_t jp = s * y + b;
                if (jp < p || jp >= p + n) continue;
                if (b_lo < 0) b_lo = b;
                ++r2;
            }
            int64_t r = x * no + y;
            if (r1 == 0 || r2 == 0) {
                desc[2 * r] = 0;
                desc[2 * r + 1] = 0;
            } else {
                uint32_t w = (uint32_t)a_lo | (uint32_t)r1 << 8 | (uint32_t)b_lo << 16 | (uint32_t)r2 << 24;
                desc[2 * r] = (int32_t)((s * x + a_lo - p) * n + (s * y + b_lo - p));
                memcpy(&desc[2 * r + 1], &w, sizeof w);
            }
        }
    return mo * no;
}

/* The matrix a compact storage stands for, in CSR: row r holds, for da < r1 and
 * db < r2 in that order, column base + da*n + db with value
 * ktab[(a_lo + da)*k + b_lo + db].  Works on whatever desc holds (it need not come
 * from oracle_compact_rows).  Returns nnz, -3 if cap is too small, -4 if a tap
 * index leaves the table. */
int64_t oracle_compact_decode(int n, int k, int64_t rows, const int32_t *desc, const float *ktab,
                              int64_t *row_ptr, int64_t *col_idx, float *vals, int64_t cap)
{
    int64_t at = 0;
    for (int64_t r = 0; r < rows; ++r) {
        uint32_t w;
        memcpy(&w, &desc[2 * r + 1], sizeof w);
        int64_t a_lo = w & 255u, r1 = (w >> 8) & 255u, b_lo = (w >> 16) & 255u, r2 = w >> 24;
        row_ptr[r] = at;
        if (a_lo + r1 > k || b_lo + r2 > k) return -4;
        for (int64_t da = 0; da < r1; ++da)
            for (int64_t db = 0; db < r2; ++db) {
                if (at >= cap) return -3;
                col_idx[at] = (int64_t)desc[2 * r] + da * n + db;
                vals[at] = ktab[(a_lo + da) * k + (b_lo + db)];
                ++at;
            }
    }
    row_ptr[rows] = at;
    return at;
}

/* ---- several input channels, one output (the "multi-channel context" the paper
 * names as future work, Section 4.2) -----------------------------------------
 * out = sum over channels ch of the padded, strided convolution of plane A_ch
 * with kernel K_ch, i.e. [T_1 | ... | T_C] applied to the stacked vectors.
 *   A   : C planes one after the other, each m*n*B floats, batch-minor.
 *   K   : C kernels one after the other, each k*k floats, row-major.
 * By definition: every plane is padded with zeros, then each output is the sum,
 * over channels and over the window, of kernel number times padded value, carried
 * in double and rounded once. */
int oracle_conv_channels(int m, int n, int k, int s, int p, int B, int C,
                         const float *A, const float *K, float *out, double *scale)
{
    int64_t mo, no;
    if (B < 1 || C < 1 || oracle_out_shape(m, n, k, s, p, &mo, &no) != 0) return -1;
    int64_t H = (int64_t)m + 2 * p, W = (int64_t)n + 2 * p;
    float *Apad = (float *)calloc((size_t)(C * H * W * B), sizeof(float));
    if (!Apad) return -2;
    for (int64_t ch = 0; ch < C; ++ch)
        for (int64_t i = 0; i < m; ++i)
            memcpy(Apad + ((ch * H + i + p) * W + p) * B, A + (ch * m + i) * n * B, sizeof(float) * (size_t)n * B);

#pragma omp parallel for schedule(static)
    for (int64_t x = 0; x < mo; ++x) {
        for (int64_t y = 0; y < no; ++y) {
            for (int64_t c = 0; c < B; ++c) {
                double acc = 0.0, mag = 0.0;
                for (int64_t ch = 0; ch < C; ++ch)
                    for (int64_t a = 0; a < k; ++a)
                        for (int64_t b = 0; b < k; ++b) {
                            double kv = (double)K[(ch * k + a) * k + b];
                            double av = (double)Apad[(((ch * H) + s * x + a) * W + (s * y + b)) * B + c];
                            acc += kv * av;
                            mag += fabs(kv) * fabs(av);
                        }
                out[(x * no + y) * B + c] = (float)acc;
                if (scale) scale[(x * no + y) * B + c] = mag;
            }
        }
    }
    free(Apad);
    return 0;
}
