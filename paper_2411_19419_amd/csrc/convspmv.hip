// Host side of the C ABI declared in include/convspmv.h: argument checking,
// the closed-form count of Theorem 2.1, the plan object and kernel dispatch.
#include "../../include/convspmv.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <cstdio>
#include <cstring>
#include <new>

#include "apply_kernels.h"
#include "apply_march_kernel.h"
#include "apply_stage_march_kernel.h"
#include "apply_tile_kernel.h"
#include "build_kernels.h"
#include "compact_channels_kernel.h"
#include "compact_kernels.h"

using namespace convspmv;

namespace {

thread_local int g_last_hip_error = 0;

inline bool hip_ok(hipError_t e) {
    if (e == hipSuccess) return true;
    g_last_hip_error = (int)e;
    return false;
}

constexpr int64_t kInt32Limit = 2147483647LL;   // largest int32

// Fewer strip segments than this cannot fill the chip with persistent workgroups; the row-group
// kernels take such problems.  A plan carries its own copy (conv_plan_set_march_min_jobs).
constexpr int kMarchMinJobs = 256;

// Attributes launch failures to this call only: the runtime's last-error slot may already
// hold an error of other code in the process (it is sticky until somebody reads it).  The
// slot is peeked before the first launch and after the last; an error that was there before
// is neither reported as ours nor cleared.
struct LaunchScope {
    hipError_t before;
    LaunchScope() : before(hipPeekAtLastError()) {}
    bool ok() const {
        const hipError_t after = hipPeekAtLastError();
        if (after == hipSuccess || after == before) return true;
        g_last_hip_error = (int)after;
        (void)hipGetLastError();      // ours: take it out of the slot
        return false;
    }
};

// Theorem 2.1, output extent along one axis (0 = precondition violated).
int64_t out_extent(int64_t extent, int64_t k, int64_t s, int64_t p) {
    if (k > extent + 2 * p) return 0;
    return (extent + 2 * p - k) / s + 1;
}

int check_shape(int m, int n, int k, int s, int p, int64_t *mo, int64_t *no) {
    if (m < 1 || n < 1 || k < 1 || s < 1 || p < 0) return CONV_EINVAL;
    *mo = out_extent(m, k, s, p);
    *no = out_extent(n, k, s, p);
    if (*mo < 1 || *no < 1) return CONV_EINVAL;
    return CONV_OK;
}

// Sum over one axis of max(0, k - c(t)), c(t) = max(0, p - s t) + max(0, s t + k - extent - p).
int64_t axis_tap_sum(int64_t count, int64_t extent, int64_t k, int64_t s, int64_t p) {
    int64_t total = 0;
    for (int64_t t = 0; t < count; ++t) {
        const int64_t lo = p - s * t, hi = s * t + k - extent - p;
        const int64_t r = k - (lo > 0 ? lo : 0) - (hi > 0 ? hi : 0);
        if (r > 0) total += r;
    }
    return total;
}

}  // namespace

struct conv_plan {
    ConvShape shape;
    int64_t rows, cols, nnz;
    int max_row_nnz;          // k*k
    const int *row_ptr;       // borrowed, device
    const int *col_idx;       // borrowed, device
    float *vals;              // borrowed, device (rewritten by conv_update_kernel)
    int *axis_tab;            // owned, device: the two per-axis prefix tables of the build
    int march_min_jobs;       // fewest strip segments for which the marching kernel is used
    int device;
    bool transposed;          // the arrays hold T^T (CSC of T): rows = m*n, cols = m_out*n_out
    int channels;             // input channels sharing row_ptr / col_idx; vals holds `channels` arrays of nnz
    bool compact;             // structure-aware storage: desc and ktab instead of the CSR arrays
    const int2 *desc;         // borrowed, device: one descriptor per row
    float *ktab;              // borrowed, device: k*k values (rewritten by conv_update_kernel)
};

extern "C" {

int conv_out_shape(int m, int n, int k, int s, int p, int *m_out, int *n_out) {
    if (!m_out || !n_out) return CONV_ENULL;
    int64_t mo, no;
    const int st = check_shape(m, n, k, s, p, &mo, &no);
    if (st != CONV_OK) return st;
    if (mo > kInt32Limit || no > kInt32Limit) return CONV_EOVERFLOW;
    *m_out = (int)mo;
    *n_out = (int)no;
    return CONV_OK;
}

int64_t conv_nnz(int m, int n, int k, int s, int p) {
    int64_t mo, no;
    const int st = check_shape(m, n, k, s, p, &mo, &no);
    if (st != CONV_OK) return st;
    const int64_t s1 = axis_tap_sum(mo, m, k, s, p);
    const int64_t s2 = axis_tap_sum(no, n, k, s, p);
    int64_t total;
    if (__builtin_mul_overflow(s1, s2, &total)) return CONV_EOVERFLOW;
    return total;
}

}  // extern "C"

namespace {

// col_idx / vals fill of a built plan's matrix: through an LDS image of R rows' entries (R = 256
// down to 1) when at least one row and the kernel fit, else the quad-walking kernel.
// Returns true when the launch also wrote row_ptr (staged kernel with row_ptr_dev given).
template <bool COLS, bool TR>
bool launch_fill(const conv_plan *plan, const float *kernel_dev, int *idx_dev, float *vals_dev, hipStream_t q,
                 int *row_ptr_dev = nullptr) {
    const ConvShape &sh = plan->shape;
    const int64_t l1 = TR ? sh.m : sh.m_out, l2 = TR ? sh.n : sh.n_out;
    int R = 256;
    while (R > 1 && (int64_t)R * plan->max_row_nnz > kFillStageEntries) R >>= 1;
    const int64_t cap = ((int64_t)R * plan->max_row_nnz + 4 + 3) & ~3LL;
    const int64_t lds = ((((int64_t)R + 1 + (int64_t)sh.k * sh.k + 3) & ~3LL) + 2 * cap) * 4;
    const int64_t blocks = l1 * ((l2 + R - 1) / R);
    if ((int64_t)R * plan->max_row_nnz <= kFillStageEntries && lds <= 64 * 1024 && blocks <= kInt32Limit) {
        csr_fill_staged_kernel<COLS, TR><<<(unsigned)blocks, kFillThreads, (size_t)lds, q>>>(
            sh, plan->axis_tab, kernel_dev, idx_dev, vals_dev, R, (int)cap, row_ptr_dev);
        return row_ptr_dev != nullptr;
    }
    const unsigned quad_blocks = (unsigned)(l1 * ((l2 + kFillRows - 1) / kFillRows));
    csr_fill_kernel<COLS, TR><<<quad_blocks, kFillThreads, 0, q>>>(sh, plan->axis_tab, kernel_dev, idx_dev, vals_dev);
    return false;
}

// Argument and size checks shared by the CSR / CSC builds; fills the size fields of *plan.
template <bool TR>
int build_check(int m, int n, int k, int s, int p, int channels, const float *kernel_dev, const int32_t *ptr_dev,
                const int32_t *idx_dev, const float *vals_dev, conv_plan *plan, int64_t *rp_blocks_out) {
    int64_t mo, no;
    int st = check_shape(m, n, k, s, p, &mo, &no);
    if (st != CONV_OK) return st;
    if (channels < 1) return CONV_EINVAL;
    const int64_t nnz = conv_nnz(m, n, k, s, p);
    if (nnz < 0) return (int)nnz;
    const int64_t out_pixels = mo * no, in_pixels = (int64_t)m * n;
    const int64_t rows = TR ? in_pixels : out_pixels, cols = (TR ? out_pixels : in_pixels) * channels;
    if (cols >= kInt32Limit) return CONV_EOVERFLOW;
    const int64_t l1 = TR ? m : mo, l2 = TR ? n : no;        // lines of the matrix, rows per line
    // 32-bit indices: entries, columns, rows (+1 for the pointer array), the per-axis
    // prefix sums, and the grids of the build kernels.
    if (nnz > kInt32Limit || in_pixels >= kInt32Limit || out_pixels >= kInt32Limit || (int64_t)k * k > kInt32Limit ||
        mo * (int64_t)k > kInt32Limit || no * (int64_t)k > kInt32Limit || (int64_t)m * k > kInt32Limit ||
        (int64_t)n * k > kInt32Limit)
        return CONV_EOVERFLOW;
    const int64_t fill_blocks = l1 * ((l2 + kFillRows - 1) / kFillRows);
    const int64_t rp_blocks = l1 * ((l2 + kRowPtrThreads - 1) / kRowPtrThreads);
    if (fill_blocks > kInt32Limit || rp_blocks > kInt32Limit) return CONV_EOVERFLOW;
    if (!ptr_dev || !kernel_dev || (nnz > 0 && (!idx_dev || !vals_dev))) return CONV_ENULL;
    *plan = conv_plan{};
    plan->shape = ConvShape{m, n, k, s, p, (int)mo, (int)no};
    plan->rows = rows;
    plan->cols = cols;
    plan->nnz = nnz;
    const int per_axis = TR ? (k + s - 1) / s : k;
    plan->max_row_nnz = per_axis * per_axis;
    plan->march_min_jobs = kMarchMinJobs;
    plan->transposed = TR;
    plan->channels = channels;
    *rp_blocks_out = rp_blocks;
    return CONV_OK;
}

// The build kernels of a checked plan whose axis_tab points at (lines + rows per line + 2) ints.
template <bool TR>
void build_enqueue(const conv_plan *plan, const float *kernel_dev, int32_t *ptr_dev, int32_t *idx_dev,
                   float *vals_dev, int64_t rp_blocks, hipStream_t q) {
    const int k = plan->shape.k;
    axis_prefix_kernel<TR><<<2, kAxisThreads, 0, q>>>(plan->shape, plan->axis_tab);
    // the staged fill writes row_ptr on its way; otherwise (no entries, or rows too long for it) its own kernel does
    bool have_row_ptr = false;
    if (plan->nnz > 0) have_row_ptr = launch_fill<true, TR>(plan, kernel_dev, idx_dev, vals_dev, q, ptr_dev);
    if (!have_row_ptr)
        row_ptr_kernel<TR><<<(unsigned)rp_blocks, kRowPtrThreads, 0, q>>>(plan->shape, plan->axis_tab, ptr_dev);
    if (plan->nnz > 0) {
        for (int ch = 1; ch < plan->channels; ++ch)      // the other channels share the indices: values only
            launch_fill<false, TR>(plan, kernel_dev + (size_t)ch * k * k, nullptr, vals_dev + (size_t)ch * plan->nnz, q);
    }
}

template <bool TR>
int build_impl(int m, int n, int k, int s, int p, int channels, const float *kernel_dev, int32_t *ptr_dev,
               int32_t *idx_dev, float *vals_dev, void *stream, conv_plan **plan_out) {
    if (!plan_out) return CONV_ENULL;
    *plan_out = nullptr;
    conv_plan checked;
    int64_t rp_blocks = 0;
    const int st = build_check<TR>(m, n, k, s, p, channels, kernel_dev, ptr_dev, idx_dev, vals_dev, &checked, &rp_blocks);
    if (st != CONV_OK) return st;
    conv_plan *plan = new (std::nothrow) conv_plan(checked);
    if (!plan) return CONV_ENOMEM;
    plan->row_ptr = ptr_dev;
    plan->col_idx = idx_dev;
    plan->vals = vals_dev;
    if (!hip_ok(hipGetDevice(&plan->device))) {
        delete plan;
        return CONV_EHIP;
    }
    const int64_t l1 = TR ? m : plan->shape.m_out, l2 = TR ? n : plan->shape.n_out;
    if (!hip_ok(hipMalloc((void **)&plan->axis_tab, sizeof(int) * (size_t)(l1 + l2 + 2)))) {
        delete plan;
        return CONV_ENOMEM;
    }
    const LaunchScope scope;
    build_enqueue<TR>(plan, kernel_dev, ptr_dev, idx_dev, vals_dev, rp_blocks, (hipStream_t)stream);
    if (!scope.ok()) {
        (void)hipFree(plan->axis_tab);
        delete plan;
        return CONV_EHIP;
    }
    *plan_out = plan;
    return CONV_OK;
}

}  // namespace

// ---------------------------------------------------------------------------
// The CSR arrays without any allocation: the per-axis prefix tables live in a
// device array of this library instead of a hipMalloc'ed table of the plan.
// ---------------------------------------------------------------------------
constexpr int kNoAllocAxisInts = 1 << 16;        // 256 KiB per device, held until the process ends
static __device__ __align__(256) int scratch[kNoAllocAxisInts];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
int *g_scratch_ptr[kMaxDevices];                 // device address of `scratch` on each device, once known

// Device address of this device's copy of `scratch` (the array's name is a host-side stand-in
// and must never be passed to a kernel).  Looked up once per device, with that device current.
int *scratch_address(int device) {
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        int *ptr = nullptr;
        if (!hip_ok(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)))) return nullptr;
        g_scratch_ptr[device] = ptr;
    }
    return g_scratch_ptr[device];
}
}  // namespace

extern "C" {

int conv_csr_fill_noalloc(int m, int n, int k, int s, int p, const float *kernel_dev, int32_t *row_ptr_dev,
                          int32_t *col_idx_dev, float *vals_dev, void *stream) {
    conv_plan plan;
    int64_t rp_blocks = 0;
    const int st = build_check<false>(m, n, k, s, p, 1, kernel_dev, row_ptr_dev, col_idx_dev, vals_dev, &plan, &rp_blocks);
    if (st != CONV_OK) return st;
    if ((int64_t)plan.shape.m_out + plan.shape.n_out + 2 > kNoAllocAxisInts) return CONV_EOVERFLOW;
    if (!hip_ok(hipGetDevice(&plan.device))) return CONV_EHIP;
    plan.axis_tab = scratch_address(plan.device);
    if (!plan.axis_tab) return CONV_EHIP;
    const LaunchScope scope;
    build_enqueue<false>(&plan, kernel_dev, row_ptr_dev, col_idx_dev, vals_dev, rp_blocks, (hipStream_t)stream);
    return scope.ok() ? CONV_OK : CONV_EHIP;
}

int conv_csr_build(int m, int n, int k, int s, int p, const float *kernel_dev, int32_t *row_ptr_dev,
                   int32_t *col_idx_dev, float *vals_dev, void *stream, conv_plan **plan_out) {
    return build_impl<false>(m, n, k, s, p, 1, kernel_dev, row_ptr_dev, col_idx_dev, vals_dev, stream, plan_out);
}

int conv_csr_build_channels(int m, int n, int k, int s, int p, int channels, const float *kernels_dev,
                            int32_t *row_ptr_dev, int32_t *col_idx_dev, float *vals_dev, void *stream,
                            conv_plan **plan_out) {
    return build_impl<false>(m, n, k, s, p, channels, kernels_dev, row_ptr_dev, col_idx_dev, vals_dev, stream,
                             plan_out);
}

int conv_csc_build(int m, int n, int k, int s, int p, const float *kernel_dev, int32_t *col_ptr_dev,
                   int32_t *row_idx_dev, float *vals_dev, void *stream, conv_plan **plan_out) {
    return build_impl<true>(m, n, k, s, p, 1, kernel_dev, col_ptr_dev, row_idx_dev, vals_dev, stream, plan_out);
}

int conv_compact_build(int m, int n, int k, int s, int p, const float *kernel_dev, int32_t *row_desc_dev,
                       float *ktab_dev, void *stream, conv_plan **plan_out) {
    return conv_compact_build_channels(m, n, k, s, p, 1, kernel_dev, row_desc_dev, ktab_dev, stream, plan_out);
}

int conv_compact_build_channels(int m, int n, int k, int s, int p, int channels, const float *kernel_dev,
                                int32_t *row_desc_dev, float *ktab_dev, void *stream, conv_plan **plan_out) {
    if (!plan_out) return CONV_ENULL;
    *plan_out = nullptr;
    int64_t mo, no;
    int st = check_shape(m, n, k, s, p, &mo, &no);
    if (st != CONV_OK) return st;
    if (channels < 1) return CONV_EINVAL;
    if (k > 255) return CONV_EINVAL;                       // tap ranges are stored in 8 bits
    const int64_t nnz = conv_nnz(m, n, k, s, p);
    if (nnz < 0) return (int)nnz;
    const int64_t rows = mo * no, cols = (int64_t)m * n * channels;
    if (rows >= kInt32Limit || cols >= kInt32Limit || mo * (int64_t)k > kInt32Limit || no * (int64_t)k > kInt32Limit ||
        (int64_t)channels * k * k > kInt32Limit)
        return CONV_EOVERFLOW;
    const int64_t blocks = mo * ((no + kCompactBuildThreads - 1) / kCompactBuildThreads);
    if (blocks > kInt32Limit) return CONV_EOVERFLOW;
    if (!kernel_dev || !row_desc_dev || !ktab_dev) return CONV_ENULL;
    if (((uintptr_t)row_desc_dev & 7u) != 0) return CONV_EINVAL;      // descriptors are read as 8-byte pairs

    conv_plan *plan = new (std::nothrow) conv_plan;
    if (!plan) return CONV_ENOMEM;
    plan->shape = ConvShape{m, n, k, s, p, (int)mo, (int)no};
    plan->rows = rows;
    plan->cols = cols;
    plan->nnz = nnz;
    plan->max_row_nnz = k * k;
    plan->row_ptr = nullptr;
    plan->col_idx = nullptr;
    plan->vals = nullptr;
    plan->axis_tab = nullptr;
    plan->device = 0;
    plan->transposed = false;
    plan->channels = channels;
    plan->compact = true;
    plan->march_min_jobs = kMarchMinJobs;
    plan->desc = reinterpret_cast<const int2 *>(row_desc_dev);
    plan->ktab = ktab_dev;
    if (!hip_ok(hipGetDevice(&plan->device))) {
        delete plan;
        return CONV_EHIP;
    }
    hipStream_t q = (hipStream_t)stream;
    const LaunchScope scope;
    compact_rows_kernel<<<(unsigned)blocks, kCompactBuildThreads, 0, q>>>(plan->shape, reinterpret_cast<int2 *>(row_desc_dev));
    compact_table_kernel<<<(channels * k * k + 255) / 256, 256, 0, q>>>(kernel_dev, ktab_dev, channels * k * k);
    if (!scope.ok()) {
        delete plan;
        return CONV_EHIP;
    }
    *plan_out = plan;
    return CONV_OK;
}

int conv_update_kernel(conv_plan *plan, const float *kernel_dev, void *stream) {
    if (!plan || !kernel_dev) return CONV_ENULL;
    const LaunchScope scope;
    if (plan->compact) {
        const int kk = plan->shape.k * plan->shape.k * plan->channels;
        compact_table_kernel<<<(kk + 255) / 256, 256, 0, (hipStream_t)stream>>>(kernel_dev, plan->ktab, kk);
        return scope.ok() ? CONV_OK : CONV_EHIP;
    }
    if (plan->nnz == 0) return CONV_OK;
    const size_t kk = (size_t)plan->shape.k * plan->shape.k;
    for (int ch = 0; ch < plan->channels; ++ch) {
        if (plan->transposed)
            launch_fill<false, true>(plan, kernel_dev + ch * kk, nullptr, plan->vals + (size_t)ch * plan->nnz,
                                     (hipStream_t)stream);
        else
            launch_fill<false, false>(plan, kernel_dev + ch * kk, nullptr, plan->vals + (size_t)ch * plan->nnz,
                                      (hipStream_t)stream);
    }
    if (!scope.ok()) return CONV_EHIP;
    return CONV_OK;
}

}  // extern "C"

namespace {

// ---------------------------------------------------------------------------
// Apply dispatch
// ---------------------------------------------------------------------------
enum class Kind { GatherScalar, GatherVec, Tile, March, StageMarch };

struct ApplyChoice {
    Kind kind;
    int g;          // lanes per row
    int nit;        // entries per lane (tile kernel: compile-time trip count)
    int nv;         // float4 column chunks per lane (0 = scalar columns)
    int tw;         // tile kernel: output pixels per tile line
    int threads;
    size_t lds;
    TileGeom geom;
    int ls;         // march kernels: output lines per step
    int nl;         // march kernels: ring lines
    int xld;        // staged march: 16-byte loads per lane, array and pass
    MarchGeom march;
};

// Lanes per row for the gather kernels: the narrowest power of two that keeps
// the trip count at or below 8 (rows have at most k*k entries).
int group_width(int max_row_nnz) {
    int g = 1;
    while (g < 16 && (max_row_nnz + g - 1) / g > 8) g <<= 1;
    return g;
}

constexpr size_t kLdsPerCu = 160 * 1024;
constexpr int kTileG = 8;
constexpr int kTileShortRow = 10, kTileShortNit = 5;      // rows this short: 2 lanes per row, 5 slots per lane
const int kTileNit[] = {2, 4, 7};       // trip counts the tile kernel is built for (8 lanes per row)

// Tile kernel instantiations: output pixels per tile line (threads = 8 * TW)
// and LDS pixels per column-chunk plane.  The plane size is 4 mod 16 so that
// the four planes start 16 banks apart.
constexpr int kTileWide = 64, kPlaneWide = 1028;
constexpr int kTileNarrow = 32, kPlaneNarrow = 516;

int round_up_mod(int v, int mod, int rem) {      // smallest r >= v with r % mod == rem
    int r = v - (v % mod) + rem;
    return r < v ? r + mod : r;
}

// Geometry of a tile kernel launch: the widest line pitch rule and the most
// output lines per tile whose input window still fits one LDS plane.
bool tile_geometry(const conv_plan *plan, int batch, int tw, int plane, TileGeom *out) {
    const ConvShape &sh = plan->shape;
    TileGeom g{};
    g.m = sh.m; g.n = sh.n; g.m_out = sh.m_out; g.n_out = sh.n_out; g.s = sh.s; g.p = sh.p;
    g.batch = batch;
    g.nnz = (int)plan->nnz;
    const int64_t iw = (int64_t)(tw - 1) * sh.s + sh.k;
    if (iw + 16 > plane) return false;
    g.iw = (int)iw;
    g.iw_pitch = round_up_mod((int)iw, 16, 8);
    // lines of input that fit: ih * iw_pitch + 1 <= plane (one pixel of zeros follows the window)
    const int64_t ih_max = (plane - 1) / g.iw_pitch;
    if (ih_max < sh.k) return false;
    int64_t th = (ih_max - sh.k) / sh.s + 1;
    if (th > 8) th = 8;
    if (th > sh.m_out) th = sh.m_out;
    const int64_t ih = (th - 1) * sh.s + sh.k;
    g.th = (int)th;
    g.ih = (int)ih;
    g.tiles_x = (sh.n_out + tw - 1) / tw;
    g.tiles_y = (int)((sh.m_out + th - 1) / th);
    const int64_t n_tiles = (int64_t)g.tiles_x * g.tiles_y;
    // int arithmetic in the kernel: s*x0 - p, i_lo + ih, ihc * n (float-reciprocal division needs < 2^21)
    if ((int64_t)sh.m + 2LL * sh.p + ih >= (1LL << 30) || (int64_t)sh.n + 2LL * sh.p + iw >= (1LL << 30)) return false;
    if (ih * sh.n >= (1LL << 21) || sh.n >= (1 << 20) || plan->cols > (1LL << 27)) return false;
    if (n_tiles + kXcds >= (1LL << 31) / kXcds) return false;
    g.n_tiles = (int)n_tiles;
    g.tiles_per_xcd = (int)((n_tiles + kXcds - 1) / kXcds);
    g.inv_n = 1.0f / (float)sh.n;
    *out = g;
    return true;
}

// Marching kernel: strips of tw output columns, a ring of 16 or 8 input lines in
// LDS.  Rows of up to 56 entries are shared by 8 lanes (strips of 64 columns),
// rows of up to 128 entries by 16 lanes (strips of 32 columns); the workgroup
// is 512 threads either way.
constexpr int kMarchThreads = 512;

struct MarchShape { int g, nit, tw; };
bool march_shape(int max_row_nnz, MarchShape *out) {
    // rows of fewer than 16 entries leave most of a group's lanes idle and the fixed cost
    // of a pass (bounds, combine, store) unpaid: measured slower than the row-group kernels
    if (max_row_nnz < 16) return false;
    if (max_row_nnz <= 16) *out = MarchShape{8, 2, 64};
    else if (max_row_nnz <= 32) *out = MarchShape{8, 4, 64};
    else if (max_row_nnz <= 56) *out = MarchShape{8, 7, 64};
    else if (max_row_nnz <= 96) *out = MarchShape{16, 6, 32};
    else if (max_row_nnz <= 128) *out = MarchShape{16, 8, 32};
    else return false;
    return true;
}
constexpr int march_plane(int nv) { return nv == 4 ? 1156 : (nv == 2 ? 2308 : 4612); }   // 4 mod 16 each; nv 0 = one plane of floats
constexpr int kMarchTargetBlocks = 512;      // two resident workgroups on each of 256 CUs

bool march_geometry(const conv_plan *plan, int batch, int nv, int tw, MarchGeom *out, int *ls_out, int *nl_out) {
    const ConvShape &sh = plan->shape;
    const bool tr = plan->transposed;
    MarchGeom g{};
    // operand and result grids: the image and the window grid for T, exchanged for T^T
    g.m = tr ? sh.m_out : sh.m;
    g.n = tr ? sh.n_out : sh.n;
    g.m_out = tr ? sh.m : sh.m_out;
    g.n_out = tr ? sh.n : sh.n_out;
    g.s = sh.s; g.p = sh.p; g.k = sh.k;
    g.tr = tr ? 1 : 0;
    g.batch = batch;
    g.nnz = (int)plan->nnz;
    // operand columns a strip of tw result columns can touch, operand lines in use or arriving
    // during a step of 2 (1) result lines, and new operand lines per step -- upper bounds
    const int64_t iw = tr ? (int64_t)(tw - 2 + sh.k) / sh.s + 2 : (int64_t)(tw - 1) * sh.s + sh.k;
    const int64_t need2 = tr ? (int64_t)(sh.k + 2) / sh.s + 2 : (int64_t)sh.s * 3 + sh.k;
    const int64_t need1 = tr ? (int64_t)sh.k / sh.s + 2 : (int64_t)sh.s + sh.k;
    const int64_t new2 = tr ? 2 / sh.s + 1 : 2LL * sh.s, new1 = tr ? 1 / sh.s + 1 : sh.s;
    const int plane = march_plane(nv);
    if (iw + 16 > plane) return false;
    g.iw = (int)iw;
    g.iw_pitch = round_up_mod((int)iw, 16, 8);
    // Ring of 16 lines with steps of two result lines when the ring, the LDS plane and the
    // per-thread line registers (2 per thread) allow it; else steps of one line with 16 or 8
    // ring lines.
    const int threads = kMarchThreads, planes = nv ? nv : 1;
    auto regs = [&](int64_t lines) { return lines * iw * planes <= 2LL * threads; };
    auto fits = [&](int nl) { return (int64_t)nl * g.iw_pitch + 1 <= plane; };
    int ls = 0, nl = 0;
    if (need2 <= 16 && regs(new2) && fits(16)) { ls = 2; nl = 16; }
    else if (need1 <= 16 && regs(new1) && fits(16)) { ls = 1; nl = 16; }
    else if (need1 <= 8 && regs(new1) && fits(8)) { ls = 1; nl = 8; }
    if (ls == 0) return false;
    // int arithmetic in the kernel: s*x - p + k, col*16, d16 < 2^25 (see the kernel)
    if ((int64_t)sh.m + 2LL * sh.p + sh.k >= (1LL << 30) || (int64_t)sh.n + 2LL * sh.p + iw >= (1LL << 30)) return false;
    if ((int64_t)g.m * g.n > (1LL << 27) || 2LL * 16 * g.n * 16 > (1LL << 25)) return false;
    if (g.n_out < tw / 2) return false;                 // a strip would be mostly empty
    g.strips = (g.n_out + tw - 1) / tw;
    const int col_blocks = nv ? batch / (4 * nv) : batch;
    if ((int64_t)g.strips * ((g.m_out + 7) / 8) * col_blocks < plan->march_min_jobs) return false;
    int64_t segs = kMarchTargetBlocks / ((int64_t)g.strips * col_blocks);
    if (segs < 1) segs = 1;
    int64_t seg = (g.m_out + segs - 1) / segs;
    if (seg < 8) seg = 8;
    seg = (seg + 1) & ~1LL;
    g.seg = (int)seg;
    g.segs = (int)((g.m_out + seg - 1) / seg);
    const int64_t jobs = (int64_t)g.strips * g.segs;
    if (jobs + kXcds >= (1LL << 31) / kXcds) return false;
    g.blocks_per_xcd = (int)((jobs + kXcds - 1) / kXcds);
    g.inv_n = 1.0f / (float)g.n;
    *out = g;
    *ls_out = ls;
    *nl_out = nl;
    return true;
}

// Marching kernel with the entry stream staged through LDS (apply_stage_march_kernel.h): strips of
// 32 result columns, 8 waves, one workgroup per CU.  Lanes per row by the longest row, so that the
// entries of a wave's 64 / G rows fit its LDS image; result lines per step WL = G (G = 2: 8 ...).
constexpr int kStageNl = 16;
constexpr int kStageTargetBlocks = 256;
constexpr int kStageXld = 3;
constexpr int kStageXldChannels = 5;    // several channels in one launch: every step loads its whole window
struct StageShape { int g, nit, nld; };
bool stage_shape(int max_row_nnz, StageShape *out) {
    // Rows of 3 x 3 taps: the fixed cost of a pass is not paid back (224^2, k 3, batch 256: 37 us
    // with either this or the tile kernel).  Rows of 101 to 128 entries take 8 lanes per row and
    // two result lines per step (4096^2, k 11, s 4, batch 4: 205 us against 246 us from the other
    // marching kernel, which keeps the still longer rows it can hold -- none at present, its limit
    // is 128 too -- and the shapes whose lines per step this one's registers do not hold).
    if (max_row_nnz < 16) return false;
    if (max_row_nnz <= 26) *out = StageShape{2, 13, 4};
    else if (max_row_nnz <= 50) *out = StageShape{2, 25, 7};
    else if (max_row_nnz <= 100) *out = StageShape{4, 25, 7};
    else if (max_row_nnz <= 128) *out = StageShape{8, 16, 4};
    else return false;
    return true;
}
constexpr size_t stage_lds(int nv, int nld) {
    return (nv ? (size_t)nv * stage_plane(nv, nld) * 16 : (size_t)stage_plane(0, nld) * 4) +
           (size_t)kStageWaves * stage_wave_bytes(nld);
}

// channels > 1: the geometry of one launch that walks the channels of every block of lines
bool stage_march_geometry(const conv_plan *plan, int batch, int nv, int channels, const StageShape &ss, MarchGeom *out,
                          int *wl_out) {
    const ConvShape &sh = plan->shape;
    const bool tr = plan->transposed;
    MarchGeom g{};
    g.m = tr ? sh.m_out : sh.m;
    g.n = tr ? sh.n_out : sh.n;
    g.m_out = tr ? sh.m : sh.m_out;
    g.n_out = tr ? sh.n : sh.n_out;
    g.s = sh.s; g.p = sh.p; g.k = sh.k;
    g.tr = tr ? 1 : 0;
    g.batch = batch;
    g.nnz = (int)plan->nnz;
    g.max_row = plan->max_row_nnz;
    g.channels = channels;
    g.x_plane = (long long)plan->cols * batch;
    if (channels > 1 && (tr || nv == 2)) return false;
    const int tw = kStageTw, rw = kWave / ss.g, wl = kStageWaves / (tw / rw);
    // the image must hold the rows of a wave: (rw - 1) full rows, the slots of the last one, 3 entries of alignment
    if ((int64_t)(rw - 1) * plan->max_row_nnz + (int64_t)ss.nit * ss.g + 3 > (int64_t)ss.nld * 256) return false;
    // operand columns a strip can touch, operand lines WL result lines can touch, new lines per step -- upper bounds
    const int64_t iw = tr ? (int64_t)(tw - 2 + sh.k) / sh.s + 2 : (int64_t)(tw - 1) * sh.s + sh.k;
    const int64_t need = tr ? (int64_t)(wl - 2 + sh.k) / sh.s + 2 : (int64_t)sh.s * (wl - 1) + sh.k;
    const int64_t fresh = tr ? (int64_t)wl / sh.s + 1 : (int64_t)sh.s * wl;
    const int plane = stage_plane(nv, ss.nld), planes = nv ? nv : 1;
    if (need > kStageNl || iw + 16 > plane) return false;
    g.iw = (int)iw;
    g.iw_pitch = round_up_mod((int)iw, 16, 8);
    if ((int64_t)kStageNl * g.iw_pitch + 1 > plane) return false;
    // line registers per thread
    if ((channels > 1 ? need * iw * planes > (int64_t)kStageXldChannels * kWave * kStageWaves
                      : fresh * iw * planes > (int64_t)kStageXld * kWave * kStageWaves))
        return false;
    // int arithmetic in the kernel, as for the other marching kernel
    if ((int64_t)sh.m + 2LL * sh.p + sh.k >= (1LL << 30) || (int64_t)sh.n + 2LL * sh.p + iw >= (1LL << 30)) return false;
    if ((int64_t)g.m * g.n > (1LL << 27) || 2LL * kStageNl * g.n * 16 > (1LL << 25)) return false;
    if (g.n_out < tw / 2) return false;                 // a strip would be mostly empty
    g.strips = (g.n_out + tw - 1) / tw;
    const int col_blocks = nv ? batch / (4 * nv) : batch;
    if ((int64_t)((g.n_out + 63) / 64) * ((g.m_out + 7) / 8) * col_blocks < plan->march_min_jobs) return false;   // jobs of 64 columns x 8 lines, as for the other kernel
    // Segment length.  A workgroup fills a CU, so the launch runs in rounds of 256 workgroups, and a
    // segment costs its lines plus about two steps for the window and entries it loads before its
    // first step: the number of segments per strip that minimises rounds x (lines + 2 steps).  (Three
    // column blocks of 32 strips: 8 segments = 768 workgroups = 3 full rounds, not 2 segments = 192.)
    int64_t seg = 0, best_cost = -1;
    for (int64_t segs = 1; segs <= 512 && (segs - 1) * wl < g.m_out; ++segs) {
        int64_t len = (g.m_out + segs - 1) / segs;
        len = (len + wl - 1) / wl * wl;
        const int64_t real = (g.m_out + len - 1) / len;
        const int64_t rounds = ((int64_t)g.strips * col_blocks * real + kStageTargetBlocks - 1) / kStageTargetBlocks;
        const int64_t cost = rounds * (len + 2 * wl);
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; seg = len; }
    }
    g.seg = (int)seg;
    g.segs = (int)((g.m_out + seg - 1) / seg);
    const int64_t jobs = (int64_t)g.strips * g.segs;
    if (jobs + kXcds >= (1LL << 31) / kXcds) return false;
    g.blocks_per_xcd = (int)((jobs + kXcds - 1) / kXcds);
    g.inv_n = 1.0f / (float)g.n;
    *out = g;
    *wl_out = wl;
    return true;
}

ApplyChoice choose_apply(const conv_plan *full, const float *x, const float *y, int batch) {
    // geometry of one channel; a multi-channel plan applies it once per channel (LDS kernels)
    // or walks the channels inside the row-group kernels
    conv_plan one = *full;
    one.cols = full->cols / full->channels;
    one.channels = 1;
    const conv_plan *plan = &one;
    ApplyChoice c{};
    const bool aligned = ((((uintptr_t)x) | ((uintptr_t)y)) & 15u) == 0;
    // (a multi-channel row is walked as one list of channels * entries by the row-group kernels)
    c.g = group_width((int)std::min<int64_t>((int64_t)plan->max_row_nnz * full->channels, 1 << 20));
    c.threads = kGatherThreads;
    const bool vec = aligned && batch % 4 == 0;
    c.nv = !vec ? 0 : (batch % 16 == 0 ? 4 : (batch % 8 == 0 ? 2 : 1));
    c.kind = vec ? Kind::GatherVec : Kind::GatherScalar;
    if (plan->nnz == 0 || (!vec && batch != 1) || (vec && batch / (4 * c.nv) > 65535)) return c;

    // marching kernel: float4 column chunks, or one scalar column for a single vector (SpMV)
    MarchShape ms;
    MarchGeom mg;
    int ls, nl;
    StageShape ss;
    int wl;
    if (full->channels > 1 && stage_shape(plan->max_row_nnz, &ss)) {
        // all channels in one launch (batches of 8, 24, ... columns as float4 chunks of 4)
        const int nv = c.nv == 2 ? 1 : c.nv;
        if (stage_march_geometry(plan, batch, nv, full->channels, ss, &mg, &wl)) {
            c.kind = Kind::StageMarch;
            c.nv = nv;
            c.g = ss.g;
            c.nit = ss.nit;
            c.tw = kStageTw;
            c.threads = kStageWaves * kWave;
            c.lds = stage_lds(c.nv, ss.nld);
            c.ls = wl;
            c.nl = kStageNl;
            c.xld = ss.nld;
            c.march = mg;
            return c;
        }
    }
    if (stage_shape(plan->max_row_nnz, &ss) && stage_march_geometry(plan, batch, c.nv, 1, ss, &mg, &wl)) {
        c.kind = Kind::StageMarch;
        c.g = ss.g;
        c.nit = ss.nit;
        c.tw = kStageTw;
        c.threads = kStageWaves * kWave;
        c.lds = stage_lds(c.nv, ss.nld);
        c.ls = wl;
        c.nl = kStageNl;
        c.xld = ss.nld;          // (16-byte loads per lane, array and pass)
        c.march = mg;
        return c;
    }
    if (march_shape(plan->max_row_nnz, &ms) && march_geometry(plan, batch, c.nv, ms.tw, &mg, &ls, &nl)) {
        c.kind = Kind::March;
        c.g = ms.g;
        c.nit = ms.nit;
        c.tw = ms.tw;
        c.threads = kMarchThreads;
        c.lds = c.nv ? (size_t)c.nv * march_plane(c.nv) * 16 : (size_t)march_plane(0) * 4;
        c.ls = ls;
        c.nl = nl;
        c.march = mg;
        return c;
    }
    if (!vec || plan->transposed) return c;     // the tile kernel is laid out for T only
    // A multi-channel sum through the LDS kernels is one launch per channel.  That pays for the
    // marching kernel (large problems); the problems the tile kernel takes are small, and the
    // row-group kernels, which walk the channels inside one launch, measured 3x faster there.
    if (full->channels > 1) return c;

    // one LDS tile per workgroup when the rows fit its unrolled trip count and the
    // input window of at least one output line fits the LDS planes
    // Rows of at most 10 entries (k = 3): two lanes per row and 5 slots each.  With 8 lanes per
    // row the kernel is bound by its instructions there (224^2, k 3, batch 256: 18.5 M vector
    // instructions for 1.8 M multiply-adds, VALU 0.70 busy): 16 slots for 9 entries and a
    // three-level combine per row.
    const bool narrow = plan->max_row_nnz <= kTileShortRow;
    const int tile_g = narrow ? 2 : kTileG;
    const int need = (plan->max_row_nnz + tile_g - 1) / tile_g;
    int nit = narrow ? kTileShortNit : 0;
    if (!narrow)
        for (int cand : kTileNit)
            if (cand >= need) { nit = cand; break; }
    if (nit == 0) return c;
    const int tws[2] = {kTileWide, kTileNarrow}, planes[2] = {kPlaneWide, kPlaneNarrow};
    for (int i = 0; i < 2; ++i) {
        TileGeom g;
        if (plan->shape.n_out <= kTileNarrow && tws[i] == kTileWide) continue;
        if (!tile_geometry(plan, batch, tws[i], planes[i], &g)) continue;
        c.kind = Kind::Tile;
        c.g = tile_g;
        c.nit = nit;
        c.tw = tws[i];
        c.threads = tws[i] * 8;
        c.lds = (size_t)c.nv * planes[i] * 16 + (size_t)g.th * (tws[i] + 1) * 4;
        c.geom = g;
        break;
    }
    return c;
}

template <int G>
void launch_gather(const ApplyChoice &c, const conv_plan *plan, const float *x, float *y, int batch, hipStream_t q) {
    const int rows = (int)plan->rows;
    const unsigned bx = (unsigned)(((int64_t)rows * G + kGatherThreads - 1) / kGatherThreads);
    auto by = [&](int per) { int b = batch / per; return (unsigned)(b > 65535 ? 65535 : b); };
    const ChannelStrides cs{plan->channels, (long long)plan->nnz, (long long)(plan->cols / plan->channels) * batch};
    switch (c.nv) {
        case 0:
            spmm_gather_scalar_kernel<G><<<dim3(bx, by(1)), kGatherThreads, 0, q>>>(
                plan->row_ptr, plan->col_idx, plan->vals, x, y, rows, batch, cs);
            break;
        case 1:
            spmm_gather_vec_kernel<G, 1><<<dim3(bx, by(4)), kGatherThreads, 0, q>>>(
                plan->row_ptr, plan->col_idx, plan->vals, x, y, rows, batch, cs);
            break;
        case 2:
            spmm_gather_vec_kernel<G, 2><<<dim3(bx, by(8)), kGatherThreads, 0, q>>>(
                plan->row_ptr, plan->col_idx, plan->vals, x, y, rows, batch, cs);
            break;
        default:
            spmm_gather_vec_kernel<G, 4><<<dim3(bx, by(16)), kGatherThreads, 0, q>>>(
                plan->row_ptr, plan->col_idx, plan->vals, x, y, rows, batch, cs);
            break;
    }
}

template <int NIT, int NV, int TW, int CS>
bool launch_tile_inst(const ApplyChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    auto kern = spmm_tile_kernel<(NIT == kTileShortNit ? 2 : kTileG), NIT, NV, TW, CS>;
    // more than 64 KiB of dynamic LDS has to be allowed once per kernel and device
    static thread_local bool allowed[64];
    const int dev = plan->device;
    if (c.lds > 64 * 1024 && (dev < 0 || dev >= 64 || !allowed[dev])) {
        if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsPerCu)))
            return false;
        if (dev >= 0 && dev < 64) allowed[dev] = true;
    }
    const dim3 grid((unsigned)(c.geom.tiles_per_xcd * kXcds), (unsigned)(c.geom.batch / (4 * NV)));
    kern<<<grid, c.threads, c.lds, q>>>(plan->row_ptr, plan->col_idx, plan->vals, x, y, c.geom);
    return true;
}

template <int NIT, int NV>
bool launch_tile_tw(const ApplyChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    if (c.tw == kTileWide) return launch_tile_inst<NIT, NV, kTileWide, kPlaneWide>(c, plan, x, y, q);
    return launch_tile_inst<NIT, NV, kTileNarrow, kPlaneNarrow>(c, plan, x, y, q);
}

template <int NV>
bool launch_tile_nv(const ApplyChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    switch (c.nit) {
        case 2: return launch_tile_tw<2, NV>(c, plan, x, y, q);
        case 4: return launch_tile_tw<4, NV>(c, plan, x, y, q);
        case kTileShortNit: return launch_tile_tw<kTileShortNit, NV>(c, plan, x, y, q);
        default: return launch_tile_tw<7, NV>(c, plan, x, y, q);
    }
}

bool launch_tile(const ApplyChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    switch (c.nv) {
        case 1: return launch_tile_nv<1>(c, plan, x, y, q);
        case 2: return launch_tile_nv<2>(c, plan, x, y, q);
        default: return launch_tile_nv<4>(c, plan, x, y, q);
    }
}

template <typename Kern>
bool allow_large_lds(Kern kern, size_t lds, int dev, bool (&allowed)[64]) {
    // more than 64 KiB of dynamic LDS has to be allowed once per kernel and device
    if (lds <= 64 * 1024 || (dev >= 0 && dev < 64 && allowed[dev])) return true;
    if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)kLdsPerCu)))
        return false;
    if (dev >= 0 && dev < 64) allowed[dev] = true;
    return true;
}

template <int G, int NIT, int NV, int TW, int NL, int LS, int XLD>
bool launch_march_inst(const ApplyChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    auto kern = spmm_march_kernel<G, NIT, NV, TW, NL, LS, XLD, march_plane(NV)>;
    static thread_local bool allowed[64];
    if (!allow_large_lds(kern, c.lds, plan->device, allowed)) return false;
    MarchGeom g = c.march;
    g.col_blocks = g.batch / (NV ? 4 * NV : 1);
    const int64_t blocks = (int64_t)g.blocks_per_xcd * kXcds * g.col_blocks;
    if (blocks > kInt32Limit) return false;
    kern<<<dim3((unsigned)blocks), c.threads, c.lds, q>>>(plan->row_ptr, plan->col_idx, plan->vals, x, y, g);
    return true;
}

template <int G, int NIT, int NV, int TW>
bool launch_march_ls(const ApplyChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    if (c.ls == 2) return launch_march_inst<G, NIT, NV, TW, 16, 2, 2>(c, plan, x, y, q);
    if (c.nl == 16) return launch_march_inst<G, NIT, NV, TW, 16, 1, 2>(c, plan, x, y, q);
    return launch_march_inst<G, NIT, NV, TW, 8, 1, 2>(c, plan, x, y, q);
}

template <int NV>
bool launch_march_nv(const ApplyChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    if (c.g == 8) {
        switch (c.nit) {
            case 2: return launch_march_ls<8, 2, NV, 64>(c, plan, x, y, q);
            case 4: return launch_march_ls<8, 4, NV, 64>(c, plan, x, y, q);
            default: return launch_march_ls<8, 7, NV, 64>(c, plan, x, y, q);
        }
    }
    if (c.nit == 6) return launch_march_ls<16, 6, NV, 32>(c, plan, x, y, q);
    return launch_march_ls<16, 8, NV, 32>(c, plan, x, y, q);
}

bool launch_march(const ApplyChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    switch (c.nv) {
        case 0: return launch_march_nv<0>(c, plan, x, y, q);
        case 1: return launch_march_nv<1>(c, plan, x, y, q);
        case 2: return launch_march_nv<2>(c, plan, x, y, q);
        default: return launch_march_nv<4>(c, plan, x, y, q);
    }
}

template <int G, int NIT, int NLD, int NV, bool MC>
bool launch_stage_march_inst(const ApplyChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    auto kern = spmm_stage_march_kernel<G, NIT, NV, kStageNl, MC ? kStageXldChannels : kStageXld, NLD, stage_plane(NV, NLD), MC>;
    static thread_local bool allowed[64];
    if (!allow_large_lds(kern, c.lds, plan->device, allowed)) return false;
    MarchGeom g = c.march;
    g.col_blocks = g.batch / (NV ? 4 * NV : 1);
    const int64_t blocks = (int64_t)g.blocks_per_xcd * kXcds * g.col_blocks;
    if (blocks > kInt32Limit) return false;
    kern<<<dim3((unsigned)blocks), c.threads, c.lds, q>>>(plan->row_ptr, plan->col_idx, plan->vals, x, y, g);
    return true;
}

template <int NV, bool MC>
bool launch_stage_march_nv(const ApplyChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    if (c.g == 2) {
        if (c.nit == 13) return launch_stage_march_inst<2, 13, 4, NV, MC>(c, plan, x, y, q);
        return launch_stage_march_inst<2, 25, 7, NV, MC>(c, plan, x, y, q);
    }
    if (c.g == 8) return launch_stage_march_inst<8, 16, 4, NV, MC>(c, plan, x, y, q);
    return launch_stage_march_inst<4, 25, 7, NV, MC>(c, plan, x, y, q);
}

bool launch_stage_march(const ApplyChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    if (c.march.channels > 1) {      // plan: all channels (vals of channel ch at vals + ch * nnz)
        switch (c.nv) {
            case 0: return launch_stage_march_nv<0, true>(c, plan, x, y, q);
            case 1: return launch_stage_march_nv<1, true>(c, plan, x, y, q);
            default: return launch_stage_march_nv<4, true>(c, plan, x, y, q);
        }
    }
    switch (c.nv) {
        case 0: return launch_stage_march_nv<0, false>(c, plan, x, y, q);
        case 1: return launch_stage_march_nv<1, false>(c, plan, x, y, q);
        case 2: return launch_stage_march_nv<2, false>(c, plan, x, y, q);
        default: return launch_stage_march_nv<4, false>(c, plan, x, y, q);
    }
}

// ---------------------------------------------------------------------------
// Structure-aware storage: dispatch
// ---------------------------------------------------------------------------
struct CompactChoice {
    bool ok;
    int kk, ss;           // rectangle path compiled for this (k, s); 0, 0: described path only
    int lpr;              // lanes per row (4 batch columns each); scalar: 1 lane, 1 column
    bool scalar;
    size_t lds;
    unsigned col_blocks;
    CompactGeom geom;
    int xld;              // described path: registers per thread that carry the next step's lines (0: copied after the step)
    int gather_g;         // > 0: the row-group kernel with this many lanes per row instead (small products)
};

// rectangle path instantiations: s = 1 and these k, RV = 4 lines per lane, ring of 16
// ring of 16 lines; 4 output lines per lane and step at stride 1, 2 at stride 2 (the ring must
// hold s*(2*RV-1) + k lines); registers per thread for the next step's RV*s lines
constexpr int kRectNl = 16;
constexpr int rect_rv(int s) { return s == 1 ? 4 : 2; }
constexpr int rect_xld(int k, int s, int lpr) {
    return (rect_rv(s) * s * ((kCompactThreads / lpr - 1) * s + k) * lpr + kCompactThreads - 1) / kCompactThreads;
}
constexpr int kCompactTargetBlocks = 512;
constexpr int kDescXld = 18;                    // described path with the next step's lines prefetched into registers
constexpr int64_t kCompactMinBlocks = 256;      // below this many workgroups the row-group kernel takes the product

bool rect_compiled(int k, int s) {
    return (s == 1 && (k == 1 || k == 3 || k == 5 || k == 7 || k == 9)) || (s == 2 && (k == 2 || k == 3 || k == 5 || k == 7));
}

CompactChoice choose_compact(const conv_plan *plan, const float *x, const float *y, int batch) {
    const ConvShape &sh = plan->shape;
    CompactChoice c{};
    const bool aligned = ((((uintptr_t)x) | ((uintptr_t)y)) & 15u) == 0;
    c.scalar = !(aligned && batch % 4 == 0);
    c.lpr = c.scalar ? 1 : (batch % 16 == 0 ? 4 : (batch % 8 == 0 ? 2 : 1));
    const int ncol = c.scalar ? 1 : 4 * c.lpr, eb = c.scalar ? 4 : 16;
    c.col_blocks = (unsigned)(batch / ncol);
    int tw = kCompactThreads / c.lpr;
    CompactGeom g{};
    g.m = sh.m; g.n = sh.n; g.m_out = sh.m_out; g.n_out = sh.n_out; g.s = sh.s; g.p = sh.p; g.k = sh.k;
    g.batch = batch;
    // int arithmetic in the kernel: s*x - p + k, s*y0 - p + iw
    int64_t iw = (int64_t)(tw - 1) * sh.s + sh.k;
    if ((int64_t)sh.m + 2LL * sh.p + sh.k >= (1LL << 30) || (int64_t)sh.n + 2LL * sh.p + iw >= (1LL << 30)) return c;
    const int kk_bytes = sh.k * sh.k * 4;
    // the rectangle path compares descriptors with (s*x - p)*n + s*y - p in int, for x up to m_out + RV
    // ... and addresses lanes by 32-bit offsets from a line's start: n*batch*4 < 2^24, TW*batch*4 < 2^32
    if (rect_compiled(sh.k, sh.s) && ((int64_t)sh.m + sh.p + sh.k + (rect_rv(sh.s) + 1) * (int64_t)sh.s) * sh.n < kInt32Limit &&
        (int64_t)sh.n * batch * 4 < (1LL << 24) && (int64_t)batch * 4 * (kCompactThreads + 1) < (1LL << 31)) {
        c.kk = sh.k;
        c.ss = sh.s;
        g.rv = rect_rv(sh.s);
        g.nl = kRectNl;
        g.ktab_lds = 1;
        c.lds = (size_t)kRectNl * iw * c.lpr * eb + kk_bytes;
    } else {
        // Described path.  A strip of tw columns is served by 256 / (tw * lpr) groups of lanes that
        // take the rv lines of a step in turn (rv = 4, 2 or 1 lines per group); two barriers per
        // step, so the ring holds one step's s*(rv-1) + k lines of (tw-1)*s + k pixels.  Widest
        // strip (not wider than the image needs) and most lines whose ring fits 64 KiB, else
        // 144 KiB (one workgroup per CU); none fits: every tap from global memory.
        g.ktab_lds = kk_bytes <= 16 * 1024;
        g.rv = 1;
        g.nl = 0;
        c.lds = g.ktab_lds ? kk_bytes : 0;
        const int64_t limits[2] = {64 * 1024, 144 * 1024};
        bool found = false;
        for (int li = 0; li < 2 && !found; ++li) {
            for (int cand = kCompactThreads / c.lpr; cand >= 16 && !found; cand >>= 1) {
                if (cand > 16 && cand / 2 >= sh.n_out) continue;      // half as wide still covers the image
                for (int mult = 4; mult >= 1 && !found; mult >>= 1) {
                    const int rv = kCompactThreads / (cand * c.lpr) * mult;
                    const int64_t cw = (int64_t)(cand - 1) * sh.s + sh.k;
                    const int64_t need = (int64_t)sh.s * (rv - 1) + sh.k;
                    int nl = 16;
                    while (nl < need && nl < 256) nl <<= 1;
                    const int64_t bytes = (int64_t)nl * cw * c.lpr * eb + (g.ktab_lds ? kk_bytes : 0);
                    if (nl < need || bytes > limits[li] || (int64_t)nl * cw * c.lpr >= (1LL << 21)) continue;
                    tw = cand;
                    iw = cw;
                    g.rv = rv;
                    g.nl = nl;
                    c.lds = (size_t)bytes;
                    found = true;
                    // the lines a step adds, in registers during the step before: when they fit, and when the
                    // ring is large enough that the workgroup is alone on its CU anyway (the registers cost
                    // the second workgroup); a line of x shorter than 2^24 bytes as for the rectangle path
                    const int64_t fresh = std::min<int64_t>((int64_t)rv * sh.s, need);
                    c.xld = (bytes > 64 * 1024 && fresh * cw * c.lpr <= (int64_t)kDescXld * kCompactThreads &&
                             (int64_t)sh.n * batch * 4 < (1LL << 24) && (int64_t)batch * 4 * (kCompactThreads + 1) < (1LL << 31))
                                ? kDescXld : 0;
                }
            }
        }
    }
    g.tw = tw;
    g.iw = (int)iw;
    g.strips = (sh.n_out + tw - 1) / tw;
    // two workgroups per CU, or one where the ring leaves room for one only (a segment starts by
    // loading the whole window of its first step: fewer, longer segments then)
    const int64_t target = c.lds > kLdsPerCu / 2 ? kCompactTargetBlocks / 2 : kCompactTargetBlocks;
    int64_t segs = target / ((int64_t)g.strips * c.col_blocks);
    if (segs < 1) segs = 1;
    int64_t seg = (sh.m_out + segs - 1) / segs;
    if (seg < 2 * g.rv) seg = 2 * g.rv;
    seg = (seg + g.rv - 1) / g.rv * g.rv;
    g.seg = (int)seg;
    g.segs = (int)((sh.m_out + seg - 1) / seg);
    const int64_t jobs = (int64_t)g.strips * g.segs;
    if (jobs + kXcds >= (1LL << 31) / kXcds) return c;
    g.blocks_per_xcd = (int)((jobs + kXcds - 1) / kXcds);
    c.geom = g;
    c.ok = true;
    // Fewer workgroups than compute units: the marching layout cannot fill the chip.  The
    // row-group kernel gives such a product rows * G lanes instead (x from global memory, which
    // for a plane this small means from the L2).
    // (the plan's marching threshold, a test hook, lowers the bound so that small test shapes march too)
    if (jobs * c.col_blocks < std::min<int64_t>(kCompactMinBlocks, plan->march_min_jobs) &&
        plan->rows * 16 / kCompactThreads + 1 < kInt32Limit) {
        c.gather_g = group_width(sh.k * sh.k);
        if (!c.scalar) { c.lpr = 1; c.col_blocks = (unsigned)(batch / 4); }
    }
    return c;
}

// Several channels in one launch (compact_channels_kernel.h): when the channels are many and a
// channel's product is short, so that one launch per channel would be bound by launches and by
// re-reading y.  VB batch columns per lane (16, 8 or 4, dividing the batch) and W = 4, 8 or 16
// waves per workgroup that split the channels: the widest VB whose launch has kChanFusedWaves
// waves with the most ways that fit LDS and the channel count, else the shape with most waves.
constexpr double kChanFusedWork = 1e8;        // multiply-adds per channel below which the launches are fused
constexpr int64_t kChanFusedWaves = 2048;     // waves that fill the chip (8 per CU)

struct ChannelsChoice {
    bool ok;
    int vb, ways;
    size_t lds;
    dim3 grid;
    CompactChannelsGeom geom;
};

ChannelsChoice choose_compact_channels(const conv_plan *plan, const float *x, const float *y, int batch) {
    const ConvShape &sh = plan->shape;
    ChannelsChoice c{};
    if (!plan->compact || plan->channels < 2 || batch % 4) return c;
    if (((((uintptr_t)x) | ((uintptr_t)y)) & 15u) != 0) return c;
    if ((double)plan->nnz * batch > kChanFusedWork) return c;
    // int arithmetic in the kernel: s*x - p + k over the padded plane, float offsets within a channel's plane
    if ((int64_t)sh.m + 2LL * sh.p + sh.k + 16LL * sh.s >= (1LL << 30) || (int64_t)sh.n + 2LL * sh.p + sh.k + 16LL * sh.s >= (1LL << 30) ||
        (int64_t)sh.m * sh.n * batch >= kInt32Limit)
        return c;
    const int64_t phx = (int64_t)(kChanTileX - 1) * sh.s + sh.k, phy = (int64_t)(kChanTileY - 1) * sh.s + sh.k;
    const int64_t npix = phx * phy;
    const int64_t tiles_x = (sh.m_out + kChanTileX - 1) / kChanTileX, tiles_y = (sh.n_out + kChanTileY - 1) / kChanTileY;
    if (tiles_x * tiles_y + kXcds > kInt32Limit) return c;
    int64_t best_waves = 0;
    for (int vb = batch % 16 == 0 ? 16 : (batch % 8 == 0 ? 8 : 4); vb >= 4; vb /= 2) {
        if (npix * (vb / 4) > (int64_t)kChanItems * kWave || batch / vb > 65535) continue;
        const int64_t vec4 = std::max<int64_t>(npix, kWave) * (vb / 4) + ((int64_t)sh.k * sh.k + 3) / 4;
        const int per_lane = (int)((npix * (vb / 4) + kWave - 1) / kWave);
        int ways = kChanMinWaves;
        while (ways < chan_max_waves(per_lane) && 2 * ways <= plan->channels && vec4 * 16 * 2 * ways <= 64 * 1024) ways *= 2;
        if (vec4 * 16 * ways > 64 * 1024) continue;
        const int64_t blocks = tiles_x * tiles_y * (batch / vb);
        while (ways > kChanMinWaves && blocks * (ways / 2) >= kChanFusedWaves) ways /= 2;     // no more ways than the chip needs
        const int64_t waves = blocks * ways;
        if (c.ok && waves <= best_waves) continue;
        best_waves = waves;
        c.ok = true;
        c.vb = vb;
        c.ways = ways;
        c.lds = (size_t)(vec4 * 16 * ways);
        const int64_t per_xcd = (tiles_x * tiles_y + kXcds - 1) / kXcds;
        c.grid = dim3((unsigned)(per_xcd * kXcds), (unsigned)(batch / vb));
        CompactChannelsGeom g{};
        g.tiles = (int)(tiles_x * tiles_y);
        g.tiles_per_xcd = (int)per_xcd;
        g.m = sh.m; g.n = sh.n; g.m_out = sh.m_out; g.n_out = sh.n_out; g.s = sh.s; g.p = sh.p; g.k = sh.k;
        g.batch = batch; g.channels = plan->channels;
        g.tiles_y = (int)tiles_y;
        g.phx = (int)phx;
        g.phy = (int)phy;
        g.wave_vec4 = (int)vec4;
        g.inv_phy = 1.0f / (float)phy;
        g.plane = (long long)sh.m * sh.n * batch;
        c.geom = g;
        if (waves >= kChanFusedWaves) break;
    }
    return c;
}

template <int VB, int KK>
void launch_compact_channels_k(const ChannelsChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    const int threads = c.ways * kWave;
    const int per_lane = (c.geom.phx * c.geom.phy * (VB / 4) + kWave - 1) / kWave;     // patch items a lane carries
    if (per_lane <= 4)
        spmm_compact_channels_kernel<VB, 4, KK><<<c.grid, threads, c.lds, q>>>(plan->desc, plan->ktab, x, y, c.geom);
    else if (per_lane <= 8)
        spmm_compact_channels_kernel<VB, 8, KK><<<c.grid, threads, c.lds, q>>>(plan->desc, plan->ktab, x, y, c.geom);
    else
        spmm_compact_channels_kernel<VB, kChanItems, KK><<<c.grid, threads, c.lds, q>>>(plan->desc, plan->ktab, x, y, c.geom);
}

template <int VB>
void launch_compact_channels_vb(const ChannelsChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    switch (c.geom.k) {       // the kernel sizes of the paper's layer table (Table 2) have unrolled tap loops
        case 1: launch_compact_channels_k<VB, 1>(c, plan, x, y, q); break;
        case 3: launch_compact_channels_k<VB, 3>(c, plan, x, y, q); break;
        case 7: launch_compact_channels_k<VB, 7>(c, plan, x, y, q); break;
        default: launch_compact_channels_k<VB, 0>(c, plan, x, y, q); break;
    }
}

void launch_compact_channels(const ChannelsChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    switch (c.vb) {
        case 16: launch_compact_channels_vb<16>(c, plan, x, y, q); break;
        case 8: launch_compact_channels_vb<8>(c, plan, x, y, q); break;
        default: launch_compact_channels_vb<4>(c, plan, x, y, q); break;
    }
}

template <int KK, int SS, int LPR, bool SCALAR, bool ACC, int XD = 0>
bool launch_compact_one(const CompactChoice &c, const CompactGeom &g, const conv_plan *plan, const float *ktab,
                        const float *x, float *y, dim3 grid, hipStream_t q) {
    constexpr bool FAST = KK > 0;
    auto kern = spmm_compact_kernel<KK, SS, LPR, SCALAR, FAST ? rect_rv(SS) : 0, FAST ? kRectNl : 0,
                                    FAST ? rect_xld(KK, SS, LPR) : XD, ACC>;
    static thread_local bool allowed[64];
    if (!allow_large_lds(kern, c.lds, plan->device, allowed)) return false;
    kern<<<grid, kCompactThreads, c.lds, q>>>(plan->desc, ktab, x, y, g);
    return true;
}

template <int KK, int SS, int LPR, bool SCALAR>
bool launch_compact_inst(const CompactChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    constexpr unsigned kMaxGridY = 65535;
    CompactGeom g = c.geom;
    const size_t plane = (size_t)(plan->cols / plan->channels) * c.geom.batch, kk = (size_t)c.geom.k * c.geom.k;
    // one launch per channel (its table, its operand plane): the first stores y, the others add to it
    for (int ch = 0; ch < plan->channels; ++ch) {
        g.accum = ch > 0;
        for (unsigned cb = 0; cb < c.col_blocks; cb += kMaxGridY) {      // column blocks beyond the grid limit: more launches
            g.c_base = (int)(cb * (SCALAR ? 1u : 4u * LPR));
            const dim3 grid((unsigned)(c.geom.blocks_per_xcd * kXcds), std::min(kMaxGridY, c.col_blocks - cb));
            const bool ok = (KK > 0 && ch > 0)
                                ? launch_compact_one<KK, SS, LPR, SCALAR, (KK > 0)>(c, g, plan, plan->ktab + ch * kk, x + ch * plane, y, grid, q)
                            : (KK == 0 && c.xld > 0)
                                ? launch_compact_one<KK, SS, LPR, SCALAR, false, (KK == 0 ? kDescXld : 0)>(c, g, plan, plan->ktab + ch * kk, x + ch * plane, y, grid, q)
                                : launch_compact_one<KK, SS, LPR, SCALAR, false>(c, g, plan, plan->ktab + ch * kk, x + ch * plane, y, grid, q);
            if (!ok) return false;
        }
    }
    return true;
}

template <int LPR, bool SCALAR>
bool launch_compact_k(const CompactChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    if (c.ss == 2) {
        switch (c.kk) {
            case 2: return launch_compact_inst<2, 2, LPR, SCALAR>(c, plan, x, y, q);
            case 3: return launch_compact_inst<3, 2, LPR, SCALAR>(c, plan, x, y, q);
            case 5: return launch_compact_inst<5, 2, LPR, SCALAR>(c, plan, x, y, q);
            default: return launch_compact_inst<7, 2, LPR, SCALAR>(c, plan, x, y, q);
        }
    }
    switch (c.kk) {
        case 1: return launch_compact_inst<1, 1, LPR, SCALAR>(c, plan, x, y, q);
        case 3: return launch_compact_inst<3, 1, LPR, SCALAR>(c, plan, x, y, q);
        case 5: return launch_compact_inst<5, 1, LPR, SCALAR>(c, plan, x, y, q);
        case 7: return launch_compact_inst<7, 1, LPR, SCALAR>(c, plan, x, y, q);
        case 9: return launch_compact_inst<9, 1, LPR, SCALAR>(c, plan, x, y, q);
        default: return launch_compact_inst<0, 0, LPR, SCALAR>(c, plan, x, y, q);
    }
}

template <int G>
void launch_compact_gather(const CompactChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    const unsigned bx = (unsigned)((plan->rows * G + kCompactThreads - 1) / kCompactThreads);
    const dim3 grid(bx, (unsigned)std::min<unsigned>(c.col_blocks, 65535u));
    const size_t plane = (size_t)(plan->cols / plan->channels) * c.geom.batch, kk = (size_t)c.geom.k * c.geom.k;
    for (int ch = 0; ch < plan->channels; ++ch) {      // one launch per channel: the first stores y, the others add to it
        if (c.scalar)
            spmm_compact_gather_kernel<G, true><<<grid, kCompactThreads, 0, q>>>(plan->desc, plan->ktab + ch * kk, x + ch * plane, y,
                                                                             (int)plan->rows, c.geom.n, c.geom.k, c.geom.batch, ch > 0);
        else
            spmm_compact_gather_kernel<G, false><<<grid, kCompactThreads, 0, q>>>(plan->desc, plan->ktab + ch * kk, x + ch * plane, y,
                                                                              (int)plan->rows, c.geom.n, c.geom.k, c.geom.batch, ch > 0);
    }
}

bool launch_compact(const CompactChoice &c, const conv_plan *plan, const float *x, float *y, hipStream_t q) {
    if (c.gather_g) {
        switch (c.gather_g) {
            case 1: launch_compact_gather<1>(c, plan, x, y, q); break;
            case 2: launch_compact_gather<2>(c, plan, x, y, q); break;
            case 4: launch_compact_gather<4>(c, plan, x, y, q); break;
            case 8: launch_compact_gather<8>(c, plan, x, y, q); break;
            default: launch_compact_gather<16>(c, plan, x, y, q); break;
        }
        return true;
    }
    if (c.scalar) return launch_compact_k<1, true>(c, plan, x, y, q);
    switch (c.lpr) {
        case 1: return launch_compact_k<1, false>(c, plan, x, y, q);
        case 2: return launch_compact_k<2, false>(c, plan, x, y, q);
        default: return launch_compact_k<4, false>(c, plan, x, y, q);
    }
}

}  // namespace

extern "C" {

int conv_spmv(const conv_plan *plan, const float *x_dev, float *y_dev, int batch, void *stream) {
    if (!plan || !x_dev || !y_dev) return CONV_ENULL;
    if (batch < 1) return CONV_EINVAL;
    {   // x and y must not overlap
        const char *xb = (const char *)x_dev, *xe = xb + sizeof(float) * (size_t)plan->cols * batch;
        const char *yb = (const char *)y_dev, *ye = yb + sizeof(float) * (size_t)plan->rows * batch;
        if (xb < ye && yb < xe) return CONV_EALIAS;
    }
    hipStream_t q = (hipStream_t)stream;
    const LaunchScope scope;
    if (plan->compact) {
        const ChannelsChoice fused = choose_compact_channels(plan, x_dev, y_dev, batch);
        if (fused.ok) {
            launch_compact_channels(fused, plan, x_dev, y_dev, q);
            return scope.ok() ? CONV_OK : CONV_EHIP;
        }
        const CompactChoice cc = choose_compact(plan, x_dev, y_dev, batch);
        if (!cc.ok) return CONV_EOVERFLOW;
        if (!launch_compact(cc, plan, x_dev, y_dev, q)) return CONV_EHIP;
        return scope.ok() ? CONV_OK : CONV_EHIP;
    }
    const ApplyChoice c = choose_apply(plan, x_dev, y_dev, batch);
    if (c.kind == Kind::StageMarch && c.march.channels > 1) {
        // one launch walks the channels of every block of lines: y is stored once, in a fixed order of sums
        if (!launch_stage_march(c, plan, x_dev, y_dev, q)) return CONV_EHIP;
    } else if (c.kind == Kind::March || c.kind == Kind::Tile || c.kind == Kind::StageMarch) {
        // one launch per channel: the first stores y, the others add to it
        conv_plan one = *plan;
        one.cols = plan->cols / plan->channels;
        one.channels = 1;
        ApplyChoice cc = c;
        for (int ch = 0; ch < plan->channels; ++ch) {
            one.vals = plan->vals + (size_t)ch * plan->nnz;
            const float *x_ch = x_dev + (size_t)ch * one.cols * batch;
            cc.march.accum = cc.geom.accum = ch > 0;
            const bool ok = c.kind == Kind::StageMarch ? launch_stage_march(cc, &one, x_ch, y_dev, q)
                            : c.kind == Kind::March   ? launch_march(cc, &one, x_ch, y_dev, q)
                                                      : launch_tile(cc, &one, x_ch, y_dev, q);
            if (!ok) return CONV_EHIP;
        }
    } else {
        switch (c.g) {
            case 1: launch_gather<1>(c, plan, x_dev, y_dev, batch, q); break;
            case 2: launch_gather<2>(c, plan, x_dev, y_dev, batch, q); break;
            case 4: launch_gather<4>(c, plan, x_dev, y_dev, batch, q); break;
            case 8: launch_gather<8>(c, plan, x_dev, y_dev, batch, q); break;
            default: launch_gather<16>(c, plan, x_dev, y_dev, batch, q); break;
        }
    }
    if (!scope.ok()) return CONV_EHIP;
    return CONV_OK;
}

}  // extern "C"

// Launch shape of the on-chip scatter: VB batch columns per wave, W waves per workgroup (W * VB
// batch columns per pass), tj < 64 pixels per tile line (the lanes of a wave hold one line's
// column pointers) with a line's entries within the stage.  The kernel is bound by the number
// of instructions it issues and needs many resident waves, so small LDS footprints are tried
// first: among the tiles within a footprint the one with the smallest window per pixel wins; a
// launch too small to fill the chip is charged for the idle units.  Not ok when no tile fits
// (k above about 32 s) or when the columns are very short (k <= s, or k <= 2 s at batches below 4):
// the walk costs about the same per column whatever its length, and with few entries per column
// adding every entry to y directly is faster.
constexpr size_t kCscTileLds[3] = {20 * 1024, 40 * 1024, 64 * 1024};
constexpr double kCscTileWindowGoal = 6.0;     // window slots per pixel that end the search for a larger footprint
constexpr int kCscTileShortColumn = 9;         // with columns of fewer entries the direct scatter is faster at batch 1 to 3,
constexpr int kCscTileShortestColumn = 4;      // and with columns of fewer than these at any batch
constexpr int kCscGroupColumn = 16;            // columns of at most this many entries share a step (4 or more of them)

struct CscTileChoice {
    bool ok;
    CscTileGeom g;
    int vb, waves;
    size_t lds;
    dim3 grid;
};

static CscTileChoice choose_csc_tile(const conv_plan *plan, int batch) {
    const ConvShape &sh = plan->shape;
    CscTileChoice c{};
    if (batch >= 9) { c.vb = 4; c.waves = 4; }
    else if (batch >= 5) { c.vb = 4; c.waves = 2; }
    else if (batch >= 3) { c.vb = 4; c.waves = 1; }
    else { c.vb = batch; c.waves = 1; }
    const int bc = c.waves * c.vb;
    const int chunks = std::min((batch + bc - 1) / bc, 65535);
    CscTileGeom g{};
    g.m = sh.m; g.n = sh.n; g.n_out = sh.n_out; g.k = sh.k; g.s = sh.s; g.p = sh.p;
    g.batch = batch;
    g.inv_n_out = 1.0f / (float)sh.n_out;
    const int64_t per_axis = ((int64_t)sh.k + sh.s - 1) / sh.s;          // windows that can cover one pixel, per axis
    const int64_t column_max = per_axis * per_axis;
    g.column_max = (int)std::min<int64_t>(column_max, kCscStage);
    g.spacing = sh.k;
    g.group = g.column_max <= kCscGroupColumn ? kWave / g.column_max : 1;
    if (column_max > kCscStage || column_max < (batch >= 4 ? kCscTileShortestColumn : kCscTileShortColumn)) return c;
    const int tj_max = (int)std::min<int64_t>(32, kCscStage / column_max);
    double best = 0.0;
    for (size_t budget : kCscTileLds) {
        for (int tj = 1; tj <= tj_max; tj *= 2) {
            if (tj > 1 && tj / 2 >= sh.n) break;
            for (int ti = 1; ti <= 64; ti *= 2) {
                if (ti > 1 && ti / 2 >= sh.m) break;
                const int64_t wx = std::min<int64_t>(((int64_t)ti + sh.k - 2) / sh.s + 1, sh.m_out);
                const int64_t wy = std::min<int64_t>(((int64_t)tj + sh.k - 2) / sh.s + 1, sh.n_out);
                const int64_t limit = (wx - 1) * sh.n_out + wy;
                if (limit > (1 << 21)) continue;
                const int64_t stage = (tj * column_max + 1) / 2 * 2, ptrs = ((int64_t)ti * (tj + 1) + 3) / 4 * 4;
                const int64_t lds = 16 * stage + 4 * ptrs + wx * wy * bc * 4;
                if (lds > (int64_t)budget) continue;
                const int64_t tiles_i = (sh.m + ti - 1) / ti, tiles_j = (sh.n + tj - 1) / tj;
                const int64_t blocks = tiles_i * tiles_j;
                if (blocks > kInt32Limit) continue;
                double score = (double)(wx * wy) / ((double)ti * tj);
                const double work = (double)blocks * chunks * c.waves;
                if (work < 8192.0) score *= 8192.0 / work;
                if (!c.ok || score < best) {
                    c.ok = true;
                    best = score;
                    g.ti = ti; g.tj = tj; g.tiles_j = (int)tiles_j;
                    g.wx = (int)wx; g.wy = (int)wy; g.inv_wy = 1.0f / (float)wy;
                    g.limit = (int)limit; g.stage = (int)stage; g.ptrs = (int)ptrs;
                    c.lds = (size_t)lds;
                    c.grid = dim3((unsigned)blocks, (unsigned)chunks);
                }
            }
        }
        if (c.ok && best <= kCscTileWindowGoal) break;
    }
    c.g = g;
    return c;
}

template <int VB, int W>
static void launch_csc_tile(const CscTileChoice &c, const conv_plan *plan, const float *x_dev, float *y_dev,
                            hipStream_t q) {
    spmm_csc_tile_kernel<VB, W><<<c.grid, W * kWave, c.lds, q>>>(plan->row_ptr, plan->col_idx, plan->vals, x_dev, y_dev,
                                                                 c.g);
}

extern "C" {

int conv_spmv_from_csc(const conv_plan *plan, const float *x_dev, float *y_dev, int batch, void *stream) {
    if (!plan || !x_dev || !y_dev) return CONV_ENULL;
    if (batch < 1 || !plan->transposed || plan->compact) return CONV_EINVAL;
    // the plan's "rows" are the columns of T (input pixels), its "cols" the rows of T
    const int64_t in_pixels = plan->rows, out_pixels = plan->cols;
    {
        const char *xb = (const char *)x_dev, *xe = xb + sizeof(float) * (size_t)in_pixels * batch;
        const char *yb = (const char *)y_dev, *ye = yb + sizeof(float) * (size_t)out_pixels * batch;
        if (xb < ye && yb < xe) return CONV_EALIAS;
    }
    hipStream_t q = (hipStream_t)stream;
    const LaunchScope scope;
    const long long count = (long long)out_pixels * batch;
    const unsigned fill_blocks = (unsigned)std::min<long long>((count / 4 + kGatherThreads) / kGatherThreads, 1 << 16);
    fill_zero_kernel<<<fill_blocks, kGatherThreads, 0, q>>>(y_dev, count);
    CscTileChoice tc{};
    if (plan->nnz > 0) tc = choose_csc_tile(plan, batch);
    if (tc.ok) {
        if (tc.vb == 1) launch_csc_tile<1, 1>(tc, plan, x_dev, y_dev, q);
        else if (tc.vb == 2) launch_csc_tile<2, 1>(tc, plan, x_dev, y_dev, q);
        else if (tc.waves == 1) launch_csc_tile<4, 1>(tc, plan, x_dev, y_dev, q);
        else if (tc.waves == 2) launch_csc_tile<4, 2>(tc, plan, x_dev, y_dev, q);
        else launch_csc_tile<4, 4>(tc, plan, x_dev, y_dev, q);
    } else if (plan->nnz > 0) {
        const int g = group_width(plan->max_row_nnz);
        const int bl = batch >= 16 ? 16 : (batch >= 4 ? 4 : 1);      // lanes across the batch
        const int64_t blocks = (in_pixels * g * bl + kGatherThreads - 1) / kGatherThreads;
        if (blocks > kInt32Limit) return CONV_EOVERFLOW;
        const unsigned bx = (unsigned)blocks;
        const unsigned by = (unsigned)std::min((batch + bl - 1) / bl, 65535);
        const dim3 grid(bx, by);
        const int cols = (int)in_pixels;
#define CONV_SCATTER_BL(G, BL)                                                                              \
    spmm_scatter_kernel<G, BL><<<grid, kGatherThreads, 0, q>>>(plan->row_ptr, plan->col_idx, plan->vals, x_dev, \
                                                               y_dev, cols, batch)
#define CONV_SCATTER(G)                                  \
    if (bl == 16) CONV_SCATTER_BL(G, 16);                \
    else if (bl == 4) CONV_SCATTER_BL(G, 4);             \
    else CONV_SCATTER_BL(G, 1)
        switch (g) {
            case 1: CONV_SCATTER(1); break;
            case 2: CONV_SCATTER(2); break;
            case 4: CONV_SCATTER(4); break;
            case 8: CONV_SCATTER(8); break;
            default: CONV_SCATTER(16); break;
        }
#undef CONV_SCATTER_BL
#undef CONV_SCATTER
    }
    return scope.ok() ? CONV_OK : CONV_EHIP;
}

// ---------------------------------------------------------------------------
// Many small products in one launch
// ---------------------------------------------------------------------------
}  // extern "C"

struct conv_multi {
    int n, batch, device;
    unsigned blocks;
    MultiDesc *descs_dev;     // owned, device
};

extern "C" {

int conv_multi_create(int n, const conv_plan *const *plans, const float *const *x_dev, float *const *y_dev,
                      int batch, conv_multi **multi_out) {
    if (!multi_out) return CONV_ENULL;
    *multi_out = nullptr;
    if (!plans || !x_dev || !y_dev) return CONV_ENULL;
    if (n < 1 || batch < 1) return CONV_EINVAL;
    MultiDesc *host = new (std::nothrow) MultiDesc[n];
    if (!host) return CONV_ENOMEM;
    int64_t blocks = 0;
    int status = CONV_OK;
    for (int i = 0; i < n && status == CONV_OK; ++i) {
        const conv_plan *p = plans[i];
        if (!p || !x_dev[i] || !y_dev[i]) { status = CONV_ENULL; break; }
        if (p->device != plans[0]->device || p->compact || p->channels != 1) { status = CONV_EINVAL; break; }
        const char *xb = (const char *)x_dev[i], *xe = xb + sizeof(float) * (size_t)p->cols * batch;
        const char *yb = (const char *)y_dev[i], *ye = yb + sizeof(float) * (size_t)p->rows * batch;
        if (xb < ye && yb < xe) { status = CONV_EALIAS; break; }
        int gs = 0;
        while ((1 << gs) < group_width(p->max_row_nnz)) ++gs;
        host[i] = MultiDesc{p->row_ptr, p->col_idx, p->vals, x_dev[i], y_dev[i], (int)p->rows, gs, (int)blocks, 0};
        blocks += ((p->rows << gs) + kGatherThreads - 1) / kGatherThreads;
        if (blocks > kInt32Limit) status = CONV_EOVERFLOW;
    }
    if (status != CONV_OK) {
        delete[] host;
        return status;
    }
    conv_multi *mu = new (std::nothrow) conv_multi;
    if (!mu) {
        delete[] host;
        return CONV_ENOMEM;
    }
    mu->n = n;
    mu->batch = batch;
    mu->device = plans[0]->device;
    mu->blocks = (unsigned)blocks;
    mu->descs_dev = nullptr;
    if (!hip_ok(hipMalloc((void **)&mu->descs_dev, sizeof(MultiDesc) * (size_t)n))) {
        delete mu;
        delete[] host;
        return CONV_ENOMEM;
    }
    const bool copied = hip_ok(hipMemcpy(mu->descs_dev, host, sizeof(MultiDesc) * (size_t)n, hipMemcpyHostToDevice));
    delete[] host;
    if (!copied) {
        (void)hipFree(mu->descs_dev);
        delete mu;
        return CONV_EHIP;
    }
    *multi_out = mu;
    return CONV_OK;
}

int conv_multi_apply(const conv_multi *multi, void *stream) {
    if (!multi) return CONV_ENULL;
    if (multi->blocks == 0) return CONV_OK;
    const unsigned by = (unsigned)(multi->batch > 65535 ? 65535 : multi->batch);
    const LaunchScope scope;
    spmm_multi_kernel<<<dim3(multi->blocks, by), kGatherThreads, 0, (hipStream_t)stream>>>(multi->descs_dev, multi->n,
                                                                                            multi->batch);
    if (!scope.ok()) return CONV_EHIP;
    return CONV_OK;
}

int conv_multi_destroy(conv_multi *multi) {
    if (!multi) return CONV_OK;
    int st = CONV_OK;
    int cur = 0;
    const bool have = hip_ok(hipGetDevice(&cur));
    if (have && cur != multi->device) (void)hipSetDevice(multi->device);
    if (multi->descs_dev && !hip_ok(hipFree(multi->descs_dev))) st = CONV_EHIP;
    if (have && cur != multi->device) (void)hipSetDevice(cur);
    delete multi;
    return st;
}

int conv_plan_shape(const conv_plan *plan, int *m, int *n, int *k, int *s, int *p, int *m_out, int *n_out,
                    int64_t *nnz) {
    if (!plan) return CONV_ENULL;
    if (m) *m = plan->shape.m;
    if (n) *n = plan->shape.n;
    if (k) *k = plan->shape.k;
    if (s) *s = plan->shape.s;
    if (p) *p = plan->shape.p;
    if (m_out) *m_out = plan->shape.m_out;
    if (n_out) *n_out = plan->shape.n_out;
    if (nnz) *nnz = plan->nnz;
    return CONV_OK;
}

int conv_plan_is_transposed(const conv_plan *plan) { return plan ? (plan->transposed ? 1 : 0) : CONV_ENULL; }
int conv_plan_is_compact(const conv_plan *plan) { return plan ? (plan->compact ? 1 : 0) : CONV_ENULL; }
int conv_plan_channels(const conv_plan *plan) { return plan ? plan->channels : CONV_ENULL; }

int conv_dispatch_info(int m, int n, int k, int s, int p, int batch, int storage, int channels, conv_dispatch *out) {
    return conv_test_dispatch_info(m, n, k, s, p, batch, storage, channels, kMarchMinJobs, out);
}

int conv_test_dispatch_info(int m, int n, int k, int s, int p, int batch, int storage, int channels,
                            int march_min_jobs, conv_dispatch *out) {
    if (!out) return CONV_ENULL;
    if (march_min_jobs < 1) return CONV_EINVAL;
    int64_t mo, no;
    const int st = check_shape(m, n, k, s, p, &mo, &no);
    if (st != CONV_OK) return st;
    if (batch < 1 || channels < 1 || storage < 0 || storage > 3 || ((storage == 1 || storage == 3) && channels != 1))
        return CONV_EINVAL;
    if (storage == 2 && k > 255) return CONV_EINVAL;
    const int64_t nnz = conv_nnz(m, n, k, s, p);
    // the structure-aware storage has no per-entry index, so its entry count is not limited to int32
    if ((storage != 2 && nnz > kInt32Limit) || mo * no >= kInt32Limit || (int64_t)m * n * channels >= kInt32Limit)
        return CONV_EOVERFLOW;
    // a plan without arrays: the dispatch looks at the shape, the storage and operand alignment only
    conv_plan plan{};
    plan.shape = ConvShape{m, n, k, s, p, (int)mo, (int)no};
    plan.transposed = storage == 1 || storage == 3;
    plan.compact = storage == 2;
    plan.channels = channels;
    plan.rows = plan.transposed ? (int64_t)m * n : mo * no;
    plan.cols = plan.transposed ? mo * no : (int64_t)m * n * channels;
    plan.nnz = nnz;
    const int per_axis = plan.transposed ? (k + s - 1) / s : k;
    plan.max_row_nnz = per_axis * per_axis;
    plan.march_min_jobs = march_min_jobs;
    conv_dispatch d{};
    const ChannelsChoice fused = choose_compact_channels(&plan, nullptr, nullptr, batch);
    if (storage == 3) {
        // conv_spmv_from_csc: the scatter with the sums kept on chip, or every entry added to y directly
        const CscTileChoice tc = plan.nnz > 0 ? choose_csc_tile(&plan, batch) : CscTileChoice{};
        if (tc.ok) {
            d.kernel = 7;
            d.threads = tc.waves * kWave;
            d.lds_bytes = (int64_t)tc.lds;
            d.workgroups = (int64_t)tc.grid.x * tc.grid.y;
            d.strip = tc.g.tj;
            d.segment = tc.g.ti;
            d.ring_lines = 0;
            d.ring_lines_needed = tc.g.wx;          // runs of the window
            d.lines_per_step = tc.g.wy;             // rows per run
            d.lanes_per_row = tc.g.group;           // columns that share a step
            d.columns_per_lane = tc.vb;
        } else {
            d.kernel = 8;
            d.threads = kGatherThreads;
            d.lanes_per_row = group_width(plan.max_row_nnz);
            d.columns_per_lane = 1;
            const int bl = batch >= 16 ? 16 : (batch >= 4 ? 4 : 1);
            d.workgroups = (plan.rows * d.lanes_per_row * bl + kGatherThreads - 1) / kGatherThreads;
        }
    } else if (fused.ok) {
        d.kernel = 6;
        d.threads = fused.ways * kWave;
        d.lds_bytes = (int64_t)fused.lds;
        d.strip = kChanTileY;
        d.segment = kChanTileX;
        d.lanes_per_row = 1;
        d.columns_per_lane = fused.vb;
        d.workgroups = (int64_t)fused.geom.tiles * fused.grid.y;
    } else if (plan.compact) {
        const CompactChoice cc = choose_compact(&plan, nullptr, nullptr, batch);
        if (!cc.ok) return CONV_EOVERFLOW;
        d.kernel = cc.gather_g ? 10 : (cc.kk ? 5 : 4);
        d.threads = kCompactThreads;
        if (cc.gather_g) {
            d.lanes_per_row = cc.gather_g;
            d.columns_per_lane = cc.scalar ? 1 : 4;
            d.workgroups = ((plan.rows * cc.gather_g + kCompactThreads - 1) / kCompactThreads) * std::min<int64_t>(cc.col_blocks, 65535);
            *out = d;
            return CONV_OK;
        }
        d.lds_bytes = (int64_t)cc.lds;
        d.strip = cc.geom.tw;
        d.segment = cc.geom.seg;
        d.ring_lines = cc.geom.nl;
        d.lines_per_step = cc.geom.rv;
        d.lanes_per_row = cc.lpr;
        d.columns_per_lane = cc.scalar ? 1 : 4;
        d.ring_lines_needed = cc.kk ? s * (2 * cc.geom.rv - 1) + k : (cc.geom.nl ? s * (cc.geom.rv - 1) + k : 0);
        d.workgroups = (int64_t)cc.geom.strips * cc.geom.segs * cc.col_blocks;
    } else {
        const ApplyChoice c = choose_apply(&plan, nullptr, nullptr, batch);
        d.kernel = c.kind == Kind::GatherScalar ? 0 : c.kind == Kind::GatherVec ? 1 : c.kind == Kind::Tile ? 2
                   : c.kind == Kind::March ? 3 : 9;
        d.threads = c.threads;
        d.lds_bytes = (int64_t)c.lds;
        d.lanes_per_row = c.g;
        d.columns_per_lane = c.nv ? 4 * c.nv : 1;
        if (c.kind == Kind::StageMarch) {
            const bool tr = plan.transposed;
            d.strip = c.tw;
            d.segment = c.march.seg;
            d.ring_lines = c.nl;
            d.lines_per_step = c.ls;
            d.ring_lines_needed = tr ? (c.ls - 2 + k) / s + 2 : s * (c.ls - 1) + k;
            d.workgroups = (int64_t)c.march.strips * c.march.segs * (c.nv ? batch / (4 * c.nv) : batch);
        } else if (c.kind == Kind::March) {
            const bool tr = plan.transposed;
            d.strip = c.tw;
            d.segment = c.march.seg;
            d.ring_lines = c.nl;
            d.lines_per_step = c.ls;
            d.ring_lines_needed = tr ? (c.ls == 2 ? (k + 2) / s + 2 : k / s + 2) : s * (2 * c.ls - 1) + k;
            d.workgroups = (int64_t)c.march.strips * c.march.segs * (c.nv ? batch / (4 * c.nv) : batch);
        } else if (c.kind == Kind::Tile) {
            d.strip = c.tw;
            d.segment = c.geom.th;
            d.workgroups = (int64_t)c.geom.n_tiles * (batch / (4 * c.nv));
        } else {
            d.workgroups = (plan.rows * c.g + kGatherThreads - 1) / kGatherThreads;
        }
    }
    *out = d;
    return CONV_OK;
}

const char *conv_spmv_variant(const conv_plan *plan, int batch) {
    if (!plan || batch < 1) return nullptr;
    static thread_local char name[96];
    if (plan->compact) {
        const ChannelsChoice fused = choose_compact_channels(plan, nullptr, nullptr, batch);
        if (fused.ok) {
            snprintf(name, sizeof name, "compact_channels_%dx%d_float4x%d_%d_ways_%d_channels", kChanTileX, kChanTileY,
                     fused.vb / 4, fused.ways, plan->channels);
            return name;
        }
        const CompactChoice cc = choose_compact(plan, nullptr, nullptr, batch);
        if (!cc.ok) return nullptr;
        char cols[16];
        if (cc.scalar) snprintf(cols, sizeof cols, "scalar");
        else snprintf(cols, sizeof cols, "float4x%d", cc.lpr);
        if (cc.gather_g)
            snprintf(name, sizeof name, "compact_gather_g%d_%s", cc.gather_g, cc.scalar ? "scalar" : "float4x1");
        else if (cc.kk)
            snprintf(name, sizeof name, "compact_rect_k%ds%d_%dx%d_ring%d_rv%d_%s", cc.kk, cc.ss, cc.geom.seg,
                     cc.geom.tw, cc.geom.nl, cc.geom.rv, cols);
        else
            snprintf(name, sizeof name, "compact_described_%dx%d_ring%d_rv%d%s_%s", cc.geom.seg, cc.geom.tw,
                     cc.geom.nl, cc.geom.rv, cc.xld ? "_prefetch" : "", cols);
        return name;
    }
    const ApplyChoice c = choose_apply(plan, nullptr, nullptr, batch);
    switch (c.kind) {
        case Kind::GatherScalar: snprintf(name, sizeof name, "gather_g%d_scalar", c.g); break;
        case Kind::GatherVec: snprintf(name, sizeof name, "gather_g%d_float4x%d", c.g, c.nv); break;
        case Kind::March:
            if (c.nv)
                snprintf(name, sizeof name, "lds_march_%dx%d_ring%d_step%d_g%d_nit%d_float4x%d", c.march.seg, c.tw, c.nl, c.ls, c.g, c.nit, c.nv);
            else
                snprintf(name, sizeof name, "lds_march_%dx%d_ring%d_step%d_g%d_nit%d_scalar", c.march.seg, c.tw, c.nl, c.ls, c.g, c.nit);
            break;
        case Kind::StageMarch:
            if (c.nv)
                snprintf(name, sizeof name, "lds_march_staged_%dx%d_ring%d_step%d_g%d_nit%d_float4x%d", c.march.seg, c.tw, c.nl, c.ls, c.g, c.nit, c.nv);
            else
                snprintf(name, sizeof name, "lds_march_staged_%dx%d_ring%d_step%d_g%d_nit%d_scalar", c.march.seg, c.tw, c.nl, c.ls, c.g, c.nit);
            break;
        case Kind::Tile:
            snprintf(name, sizeof name, "lds_tile_%dx%d_g%d_nit%d_float4x%d", c.geom.th, c.tw, c.g, c.nit, c.nv);
            break;
    }
    if (plan->channels > 1) {
        const size_t len = strlen(name);
        const bool per_channel = c.kind == Kind::March || c.kind == Kind::Tile ||
                                 (c.kind == Kind::StageMarch && c.march.channels <= 1);
        snprintf(name + len, sizeof name - len, per_channel ? "_x%d_launches" : "_%d_channels", plan->channels);
    }
    return name;
}

int conv_plan_destroy(conv_plan *plan) {
    if (!plan) return CONV_OK;
    int st = CONV_OK;
    if (plan->axis_tab) {
        int cur = 0;
        const bool have = hip_ok(hipGetDevice(&cur));
        if (have && cur != plan->device) (void)hipSetDevice(plan->device);
        if (!hip_ok(hipFree(plan->axis_tab))) st = CONV_EHIP;
        if (have && cur != plan->device) (void)hipSetDevice(cur);
    }
    delete plan;
    return st;
}

const char *conv_strerror(int status) {
    switch (status) {
        case CONV_OK: return "ok";
        case CONV_EINVAL: return "invalid argument (need m,n,k,s >= 1, p >= 0, batch >= 1, k <= m+2p and k <= n+2p)";
        case CONV_ENULL: return "required pointer is NULL";
        case CONV_EOVERFLOW: return "size does not fit the library's 32-bit indices";
        case CONV_EHIP: return "HIP call failed (see conv_last_hip_error)";
        case CONV_ENOMEM: return "allocation failed";
        case CONV_EALIAS: return "x and y overlap";
    }
    return "unknown status";
}

int conv_last_hip_error(void) { return g_last_hip_error; }

int conv_plan_set_march_min_jobs(conv_plan *plan, int jobs) {
    if (!plan) return CONV_ENULL;
    if (jobs < 1) return CONV_EINVAL;
    const int prev = plan->march_min_jobs;
    plan->march_min_jobs = jobs;
    return prev;
}

}  // extern "C"
