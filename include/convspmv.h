/*
 * convspmv.h -- C ABI of the padded-convolution-as-sparse-matrix library.
 *
 * A zero-padded, strided k x k convolution of an m x n input is one sparse
 * matrix T of shape (m_out*n_out) x (m*n) applied to the row-major vectorised
 * input (paper, Section 2: T = C P, result = vec^-1(T vec(A))).  T keeps only
 * the kernel taps that fall on entries of A; their number is the closed form
 * of Theorem 2.1.  The library builds T in CSR on the device and applies it
 * to one vector (SpMV) or to a batch of vectors that share T (SpMM).
 *
 * Conventions
 *   - Output pixel (x, y), 0 <= x < m_out, 0 <= y < n_out, is row x*n_out + y
 *     of T; input pixel (i, j) is column i*n + j (row-major vec, Section 2).
 *   - Tap (a, b) of window (x, y) touches input pixel (s*x + a - p,
 *     s*y + b - p) and carries K[a*k + b]: no kernel flip (Section 2, first
 *     row of C).  It is stored iff that pixel exists; it is stored even when
 *     K[a*k + b] == 0, so nnz always equals the closed form.
 *   - Entries of a row are in ascending column order (= (a, b) raster order).
 *   - Indices are int32, values fp32.  All pointers named *_dev are device
 *     (HIP) pointers owned by the caller; `stream` is a hipStream_t passed as
 *     void* (NULL = the default stream).  Build and apply only enqueue work on
 *     `stream`; they never synchronise it.
 *   - Batches are batch-minor: element (pixel q, column c) at q*batch + c.
 *
 * Every function returns a status (0 = CONV_OK, negative = error) except
 * conv_nnz, which returns the count or a negative status, and conv_strerror.
 * No function throws or aborts.
 */
#ifndef CONVSPMV_H
#define CONVSPMV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CONV_OK          0
#define CONV_EINVAL     (-1)  /* m,n,k,s < 1, p < 0, batch < 1, or k > m+2p / n+2p (Theorem 2.1's precondition) */
#define CONV_ENULL      (-2)  /* a required pointer is NULL */
#define CONV_EOVERFLOW  (-3)  /* nnz, m*n, rows or an element count does not fit the 32-bit indices */
#define CONV_EHIP       (-4)  /* a HIP call failed; see conv_last_hip_error */
#define CONV_ENOMEM     (-5)  /* host or device allocation for the plan failed */
#define CONV_EALIAS     (-6)  /* x and y overlap */

typedef struct conv_plan conv_plan;   /* opaque host object */

/* Theorem 2.1: m_out = floor((m+2p-k)/s)+1, n_out likewise.  Host only. */
int conv_out_shape(int m, int n, int k, int s, int p, int *m_out, int *n_out);

/* Theorem 2.1: number of stored entries of T,
 *   sum_x sum_y max(0, k - c1(x)) * max(0, k - c2(y)),
 * evaluated on the host in O(m_out + n_out) (the double sum of a product is
 * the product of the two sums).  Returns the count (>= 0) or a status < 0.
 * Counts above the int32 range are still returned exactly; conv_csr_build
 * refuses them. */
int64_t conv_nnz(int m, int n, int k, int s, int p);

/* Build T in CSR on the device (Section 2 for what T holds, Theorem 2.1 for
 * the row lengths: row (x, y) has max(0,k-c1(x)) * max(0,k-c2(y)) entries).
 *   kernel_dev  : k*k fp32, row-major K[a*k + b], device, read by the build
 *                 kernels on `stream` (must stay valid until they have run).
 *   row_ptr_dev : (m_out*n_out + 1) int32, device, written.
 *   col_idx_dev : nnz int32, device, written.   nnz = conv_nnz(m,n,k,s,p).
 *   vals_dev    : nnz fp32,  device, written.
 * The three CSR arrays are allocated by the caller and BORROWED by the plan:
 * they must outlive it and must not be modified while an apply is in flight.
 * The plan itself owns a small device table (the two per-axis prefix sums of
 * the row-length factors, (m_out + n_out + 2) int32), allocated here with
 * hipMalloc and released by conv_plan_destroy (both synchronise the device; a
 * caller that must not allocate uses conv_csr_fill_noalloc).
 * Argument errors (CONV_EINVAL, CONV_ENULL, CONV_EOVERFLOW, CONV_ENOMEM) are
 * found before anything is enqueued.  CONV_EHIP means that one of this call's
 * own launches failed: earlier launches of the call may already be enqueued.
 * An error that other code left in the runtime's last-error slot is neither
 * reported nor cleared.  On any error *plan_out is left NULL. */
int conv_csr_build(int m, int n, int k, int s, int p,
                   const float *kernel_dev,
                   int32_t *row_ptr_dev, int32_t *col_idx_dev, float *vals_dev,
                   void *stream, conv_plan **plan_out);

/* For callers that cannot allocate (code under HIP graph capture, serving loops,
 * harnesses that forbid hipMalloc): the three CSR arrays of conv_csr_build,
 * written by the same kernels, with no allocation of any kind -- no plan object
 * is made and the per-axis prefix tables live in a device array inside this
 * library (256 KiB per device, held until the process ends) instead of a table
 * owned by a plan.  Arguments as for conv_csr_build.  Limits: m_out + n_out + 2
 * <= 65536 (CONV_EOVERFLOW beyond).  Every call on one device uses that device's
 * one array: calls whose kernels may overlap on the same device (different
 * streams) race on it and must be ordered by the caller; calls on one stream
 * are safe.  The device that is current at the call is used. */
int conv_csr_fill_noalloc(int m, int n, int k, int s, int p,
                          const float *kernel_dev,
                          int32_t *row_ptr_dev, int32_t *col_idx_dev, float *vals_dev,
                          void *stream);

/* Several input channels, one output (the multi-channel context the paper
 * names as an outlook, Section 4.2): y = sum over ch of T_ch x_ch, i.e. the
 * horizontally concatenated matrix [T_1 | ... | T_C] applied to the stacked
 * input planes.  All T_ch have the same shape and therefore the same row_ptr
 * and col_idx (Section 2: the positions depend on m, n, k, s, p only); they
 * differ in their values.  Stored as one row_ptr, one col_idx and
 *   vals_dev    : channels*nnz fp32, device, written: the values of T_ch at
 *                 vals_dev + ch*nnz,
 * from
 *   kernels_dev : channels*k*k fp32, device: kernel ch at kernels_dev + ch*k*k.
 * conv_spmv on the plan takes x_dev of channels*m*n*batch elements (plane ch,
 * batch-minor, at x_dev + ch*m*n*batch) and writes y_dev of m_out*n_out*batch
 * elements; conv_update_kernel takes channels*k*k numbers.  channels = 1 is
 * conv_csr_build.  conv_multi_create does not accept a plan with more than one
 * channel.  Everything else as for conv_csr_build. */
int conv_csr_build_channels(int m, int n, int k, int s, int p, int channels,
                            const float *kernels_dev,
                            int32_t *row_ptr_dev, int32_t *col_idx_dev, float *vals_dev,
                            void *stream, conv_plan **plan_out);

/* Build T column-compressed (CSC), the other storage the paper uses
 * (Sections 3 and 4.1).  The CSC arrays of T are the CSR arrays of T^T:
 *   col_ptr_dev : (m*n + 1) int32, device, written.
 *   row_idx_dev : nnz int32, device, written: rows x*n_out + y of T, ascending
 *                 inside a column.
 *   vals_dev    : nnz fp32, device, written: K[i+p-s*x][j+p-s*y] for column
 *                 (i, j) and row (x, y).
 * Column (i, j) has q1(i)*q2(j) entries, q1(i) = number of window lines x in
 * [0, m_out) with 0 <= i+p-s*x < k (the same product structure as the rows of
 * T in Theorem 2.1, with windows and pixels exchanged).  Everything else is
 * as for conv_csr_build.  The plan returned is a plan for T^T: conv_spmv on it
 * takes x_dev of m_out*n_out*batch elements and writes y_dev of m*n*batch
 * elements, y = T^T x (the adjoint of the convolution: its input gradient);
 * conv_update_kernel and conv_multi_create accept it as well. */
int conv_csc_build(int m, int n, int k, int s, int p,
                   const float *kernel_dev,
                   int32_t *col_ptr_dev, int32_t *row_idx_dev, float *vals_dev,
                   void *stream, conv_plan **plan_out);

/* Build T in a structure-aware storage (the paper's closing remarks, Sections
 * 4.2 and 5, point at formats that use the block structure of C).  By
 * Section 2 and Theorem 2.1 the entries of row (x, y) are the r1 x r2
 * rectangle of taps a in [a_lo, a_lo + r1), b in [b_lo, b_lo + r2) with
 * a_lo = max(0, p - s x), r1 = k - c1(x) (b_lo, r2 likewise along n), and all
 * their values come from the k*k kernel.  So T is stored as
 *   row_desc_dev : 2*m_out*n_out int32, device, 8-byte aligned, written: for row
 *                  r the pair { base, a_lo | r1 << 8 | b_lo << 16 | r2 << 24 },
 *                  base = column of the row's first entry; {0, 0} for a row
 *                  without entries;
 *   ktab_dev     : k*k fp32, device, written: a copy of K, row-major.
 * Entry (da, db) of row r, da < r1, db < r2, is column base + da*n + db with
 * value ktab[(a_lo + da)*k + b_lo + db].  That is 8 bytes per row plus 4*k*k
 * instead of 8 bytes per entry.  Needs k <= 255 (CONV_EINVAL otherwise); the
 * number of entries may exceed the int32 range (only rows and columns are
 * indexed).
 * Both arrays are allocated by the caller and BORROWED by the plan.  conv_spmv
 * on the plan computes y = T x from these arrays as they are stored: the result
 * is the product with whatever matrix they describe, provided a_lo + r1 <= k,
 * b_lo + r2 <= k and every described column lies in [0, m*n).
 * conv_update_kernel rewrites ktab only (k*k numbers); conv_multi_create does
 * not accept such a plan.  On error nothing is enqueued and *plan_out is NULL. */
int conv_compact_build(int m, int n, int k, int s, int p,
                       const float *kernel_dev,
                       int32_t *row_desc_dev, float *ktab_dev,
                       void *stream, conv_plan **plan_out);

/* The same storage for several input channels (see conv_csr_build_channels for
 * the product): the descriptors depend on the shape only and are stored once,
 * ktab_dev holds channels*k*k values, the table of channel ch at ktab_dev +
 * ch*k*k, copied from kernels_dev.  conv_spmv takes the stacked planes and
 * computes y = sum over ch of T_ch x_ch, one kernel per channel on `stream`,
 * the later ones reading y and adding to it (plain loads and stores: the
 * result is reproducible).  channels = 1 is conv_compact_build. */
int conv_compact_build_channels(int m, int n, int k, int s, int p, int channels,
                                const float *kernels_dev,
                                int32_t *row_desc_dev, float *ktab_dev,
                                void *stream, conv_plan **plan_out);

/* Replace the kernel of a built T: rewrites the plan's vals array from a new
 * K of the same size (k*k fp32, row-major, device); row_ptr and col_idx do not
 * depend on K and are left alone.  The paper notes (Section 4.2) that the
 * method is at a disadvantage when the kernel changes, because the
 * transformation has to be recomputed; this call is that recomputation
 * reduced to one pass over vals.  Enqueues on `stream`; must not overlap an
 * apply of the same plan. */
int conv_update_kernel(conv_plan *plan, const float *kernel_dev, void *stream);

/* Apply: y = T x (Section 3, the convolution procedure: vec, multiply,
 * un-vec; vec and its inverse are reinterpretations and move nothing).
 *   x_dev : m*n*batch fp32, batch-minor, device, read.
 *   y_dev : m_out*n_out*batch fp32, batch-minor, device, written (every
 *           element; rows of T without entries give +0.0).
 *   batch : number of vectors sharing T (1 = SpMV).
 * The kernels read row_ptr, col_idx and vals as stored: the result is the
 * product with whatever the three arrays hold, provided row_ptr is still
 * non-decreasing, no row is longer than the longest row the build wrote (k*k
 * for T; ceil(k/s)^2 for the T^T of conv_csc_build) and every col_idx is in
 * [0, number of columns).
 * fp32 multiply-add, summation order unspecified but fixed: repeated calls
 * give bit-identical results.  (A plan with several channels runs either
 * one kernel that sums the channels in a fixed order, or one kernel per
 * channel on `stream`, the later ones adding to y once per element in launch
 * order.)  x and y must not overlap. */
int conv_spmv(const conv_plan *plan, const float *x_dev, float *y_dev, int batch, void *stream);

/* y = T x computed from the column-compressed arrays, as the paper's CSC
 * variants do (Sections 3 and 4.1: the same T stored by columns).  `plan` must
 * come from conv_csc_build (CONV_EINVAL otherwise); x_dev has m*n*batch
 * elements, y_dev m_out*n_out*batch, both batch-minor.  By columns the product
 * is a scatter: y is zeroed, then every stored entry adds vals[e]*x[column] to
 * y[row_idx[e]].  The sums of a tile of neighbouring pixels are collected on
 * chip and added to y with hardware float adds (for 2 <= ceil(k/s) <= 32, from
 * 3 at batches below 4; otherwise every entry is added to y directly).  The result is that of
 * conv_spmv on the CSR plan of the same T up to the order of the additions,
 * which here depends on timing: repeated calls agree to rounding, not bit for
 * bit.  The arrays are read as stored: every row_idx must be in
 * [0, m_out*n_out), col_ptr non-decreasing, no column longer than ceil(k/s)^2
 * entries (the longest conv_csc_build writes), and the row indices of one
 * column pairwise different, as conv_csc_build writes them (a row stored twice
 * in one column may lose one of its two contributions). */
int conv_spmv_from_csc(const conv_plan *plan, const float *x_dev, float *y_dev, int batch, void *stream);

/* Shape and size queries on a plan (host only).  conv_plan_is_transposed
 * returns 1 for a plan made by conv_csc_build, conv_plan_is_compact 1 for a
 * plan made by conv_compact_build, 0 otherwise, < 0 on error. */
int conv_plan_shape(const conv_plan *plan, int *m, int *n, int *k, int *s, int *p,
                    int *m_out, int *n_out, int64_t *nnz);
int conv_plan_is_transposed(const conv_plan *plan);
int conv_plan_is_compact(const conv_plan *plan);
int conv_plan_channels(const conv_plan *plan);      /* input channels (1 unless built by conv_csr_build_channels) */

/* Name of the apply variant conv_spmv would launch for this batch with
 * 16-byte-aligned x and y (for reports), or NULL on bad arguments.  The text
 * lives in a per-thread buffer and is valid until the next call on that
 * thread. */
const char *conv_spmv_variant(const conv_plan *plan, int batch);

/* What conv_spmv would launch for a shape, without a plan and without a GPU
 * (host only; 16-byte-aligned operands assumed): the kernel family and the
 * launch geometry the dispatch derives.  storage: 0 = CSR of T, 1 = CSC of T
 * (the plan applies T^T), 2 = structure-aware storage, 3 = CSC of T applied
 * by conv_spmv_from_csc; channels > 1 not with storage 1 or 3.  Status as for the build calls (CONV_EINVAL, CONV_EOVERFLOW,
 * CONV_ENULL).  For tests of the host logic and for reports. */
typedef struct conv_dispatch {
    int kernel;             /* 0 row-group scalar, 1 row-group float4, 2 LDS tile, 3 LDS march,
                               4 described rows (structure-aware), 5 rectangle path (structure-aware),
                               6 all channels in one launch, 4 x 16 outputs per wave (structure-aware),
                               7 scatter with the sums of a tile of pixels kept on chip, 8 direct scatter
                               (storage 3; for 7: strip x segment = pixels x lines of a tile, ring_lines_needed
                               x lines_per_step = runs x rows of its window, lanes_per_row = columns per step),
                               9 LDS march with the entry stream staged through LDS,
                               10 row groups over the structure-aware storage (small products) */
    int threads;            /* per workgroup */
    int64_t lds_bytes;      /* dynamic LDS per workgroup */
    int64_t workgroups;     /* that do work, over the whole launch (per channel for kernel 3) */
    int strip;              /* output columns per strip / tile line (kernels 2-6, 9), else 0 */
    int segment;            /* output lines per workgroup (kernels 2-6, 9), else 0 */
    int ring_lines;         /* LDS ring lines (kernels 3-5, 9; 0 = no ring) */
    int ring_lines_needed;  /* lines a step keeps resident (<= ring_lines when there is a ring) */
    int lines_per_step;     /* output lines per step (kernels 3-5, 9) */
    int lanes_per_row;      /* lanes that share a row of the matrix */
    int columns_per_lane;   /* batch columns per lane */
} conv_dispatch;
int conv_dispatch_info(int m, int n, int k, int s, int p, int batch, int storage, int channels,
                       conv_dispatch *out);

/* Release the host object and the plan-owned device table.  The caller must
 * have synchronised every stream the plan was used on.  NULL is accepted. */
int conv_plan_destroy(conv_plan *plan);

/* Static, human-readable text for a status code. */
const char *conv_strerror(int status);

/* hipError_t (as int) of the most recent failing HIP call made by this
 * library on the calling thread; 0 if none. */
int conv_last_hip_error(void);

/* Many small products in one launch.  The paper's experiment (Section 4.1,
 * Table 2) applies 123 small independent transformations, each far cheaper
 * than a kernel launch; conv_multi_create binds n plans to their operands
 *   x_dev[i] : cols_i*batch fp32, batch-minor, device, read by every apply,
 *   y_dev[i] : rows_i*batch fp32, batch-minor, device, written by every apply,
 * (the same batch for all) and conv_multi_apply computes y_i = T_i x_i for all
 * i with a single kernel launch on `stream`.  The plans, their CSR arrays and
 * the operand buffers are borrowed and must outlive the object; the object
 * owns a device array of n descriptors (hipMalloc and a blocking copy in
 * create).  All plans must live on the same device; x_i and y_i must not
 * overlap.  Results are those of conv_spmv up to summation order. */
typedef struct conv_multi conv_multi;
int conv_multi_create(int n, const conv_plan *const *plans, const float *const *x_dev,
                      float *const *y_dev, int batch, conv_multi **multi_out);
int conv_multi_apply(const conv_multi *multi, void *stream);
int conv_multi_destroy(conv_multi *multi);   /* NULL is accepted */

/* ---------------------------------------------------------------------------
 * Test hooks.  Not part of the product interface: they exist so that the tests
 * can drive the persistent "marching" kernels on shapes far smaller than the
 * ones the dispatch would give them.
 *
 * conv_spmv uses a marching kernel only when the problem splits into at least
 * `jobs` strip segments (64 or 32 output columns x 8 output lines x one block
 * of batch columns); smaller problems cannot fill the chip that way and go to
 * the row-group kernels.  The threshold is a field of the plan (default 256);
 * conv_plan_set_march_min_jobs changes it for that plan only and returns the
 * previous value (CONV_EINVAL for jobs < 1, CONV_ENULL without a plan).  Not
 * thread-safe against a concurrent conv_spmv on the same plan.  The result of
 * conv_spmv does not depend on it beyond the summation order.
 * conv_test_dispatch_info is conv_dispatch_info with that threshold given. */
int conv_plan_set_march_min_jobs(conv_plan *plan, int jobs);
int conv_test_dispatch_info(int m, int n, int k, int s, int p, int batch, int storage, int channels,
                            int march_min_jobs, conv_dispatch *out);

#ifdef __cplusplus
}
#endif
#endif /* CONVSPMV_H */
