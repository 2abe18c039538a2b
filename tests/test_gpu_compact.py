"""GPU parity for the structure-aware storage of T (conv_compact_build): descriptors and
value table bit-exact against the oracle, y = T x from them against the sliding-window
oracle, and, for descriptors edited after the build, against the matrix the oracle's
decoder says they stand for."""
import ctypes
import itertools

import numpy as np
import pytest
import scipy.sparse
import torch

import oracle
import paper_2411_19419_amd as cs
from paper_2411_19419_amd import binding, workloads

from gpu_util import REL_TOL, build_plan, build_plan_c, check_apply, check_compact, device

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["row_groups_where_small", "marching_everywhere"])
def compact_dispatch(request):
    """Every test of this file runs twice: with the default dispatch, which gives small products to
    the row-group kernel, and with the plan's marching threshold lowered to one job (the test
    hook), so that the small test shapes also take the marching kernel's rectangle and described
    paths, which the default keeps for large planes."""
    import gpu_util
    gpu_util.MARCH_MIN_JOBS = 1 if request.param == "marching_everywhere" else None
    yield request.param
    gpu_util.MARCH_MIN_JOBS = None


def _rand(shape, batch, seed):
    m, n, k, s, p = shape
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(m * n * batch).astype(np.float32),
            rng.standard_normal(k * k).astype(np.float32))


def test_compact_exhaustive_tiny_grid():
    batches = itertools.cycle([1, 3, 4, 8, 16])
    count = 0
    for shape in itertools.product(range(1, 6), range(1, 6), range(1, 5), range(1, 4), range(0, 5)):
        m, n, k, s, p = shape
        if k > m + 2 * p or k > n + 2 * p:
            continue
        batch = next(batches)
        x, K = _rand(shape, batch, count)
        plan = build_plan_c(shape, K)
        check_compact(plan, shape, K)
        check_apply(plan, shape, K, x, batch)
        plan.close()
        count += 1
    assert count > 1000


RECT = [   # (k, s) with a compiled rectangle path: several strips, segments, ragged tails, all lane layouts
    ((37, 53, 7, 1, 3), 16), ((130, 67, 7, 1, 3), 4), ((300, 700, 3, 1, 1), 16), ((129, 300, 5, 1, 2), 8),
    ((64, 64, 7, 1, 0), 16), ((50, 1000, 7, 1, 6), 16), ((1030, 260, 7, 1, 3), 1), ((90, 515, 5, 1, 2), 2),
    ((200, 257, 3, 1, 1), 1), ((70, 70, 7, 1, 3), 32), ((41, 600, 5, 1, 4), 4), ((9, 9, 7, 1, 3), 16),
    ((7, 300, 7, 1, 0), 8), ((300, 7, 7, 1, 0), 16), ((260, 130, 3, 1, 0), 12), ((33, 65, 7, 1, 5), 48),
    ((200, 300, 9, 1, 4), 16), ((64, 500, 9, 1, 0), 4), ((150, 150, 1, 1, 0), 16), ((33, 77, 1, 1, 2), 8),
    ((200, 1, 1, 1, 0), 6), ((90, 90, 9, 1, 8), 1), ((120, 40, 9, 1, 4), 2),
]
RECT_S2 = [   # stride 2: two output lines per lane and step
    ((100, 90, 5, 2, 2), 16), ((224, 224, 7, 2, 3), 16), ((257, 513, 3, 2, 1), 1), ((300, 301, 2, 2, 0), 8),
    ((3, 50, 7, 2, 3), 5), ((112, 112, 3, 2, 1), 4), ((131, 77, 7, 2, 0), 16), ((64, 300, 5, 2, 4), 2),
    ((56, 56, 2, 2, 0), 32), ((40, 700, 3, 2, 2), 12), ((9, 9, 7, 2, 3), 16), ((515, 66, 2, 2, 1), 1),
]
DESCRIBED = [
    ((100, 90, 5, 3, 2), 16), ((75, 75, 9, 3, 8), 4), ((90, 141, 11, 4, 5), 2), ((40, 40, 13, 1, 6), 3),
    ((3, 50, 7, 5, 3), 5), ((6, 6, 2, 1, 5), 7), ((1, 1, 1, 5, 2), 3), ((200, 1, 11, 1, 5), 6),
    ((300, 301, 2, 3, 0), 8), ((257, 513, 3, 4, 1), 1), ((64, 1000, 5, 3, 1), 4), ((224, 224, 7, 3, 3), 16),
    ((120, 120, 100, 5, 50), 4), ((260, 260, 255, 3, 0), 1), ((60, 70, 40, 1, 20), 16), ((500, 40, 4, 1, 2), 8),
    ((31, 31, 6, 1, 9), 16), ((150, 150, 1, 3, 0), 16), ((97, 400, 2, 1, 1), 4),
]


@pytest.mark.parametrize("shape,batch", RECT + RECT_S2 + DESCRIBED)
def test_compact_shapes(shape, batch):
    x, K = _rand(shape, batch, 3)
    plan = build_plan_c(shape, K)
    check_compact(plan, shape, K)
    check_apply(plan, shape, K, x, batch)
    plan.close()


def test_rectangle_path_is_dispatched_where_compiled(compact_dispatch):
    if compact_dispatch != "marching_everywhere":
        # these shapes are small: by default they go to the row groups
        for shape, batch in (((37, 53, 7, 1, 3), 16), ((75, 75, 9, 3, 8), 4), ((512, 512, 9, 3, 8), 1)):
            plan = build_plan_c(shape, np.ones(shape[2] ** 2, dtype=np.float32))
            assert plan.variant(batch).startswith("compact_gather"), (shape, plan.variant(batch))
            plan.close()
        return
    for shape, batch in RECT + RECT_S2:
        plan = build_plan_c(shape, np.ones(shape[2] ** 2, dtype=np.float32))
        assert plan.variant(batch).startswith("compact_rect_k%ds%d" % (shape[2], shape[3])), plan.variant(batch)
        plan.close()
    for shape, batch in DESCRIBED:
        plan = build_plan_c(shape, np.ones(shape[2] ** 2, dtype=np.float32))
        assert plan.variant(batch).startswith("compact_described"), (shape, plan.variant(batch))
        plan.close()


@pytest.mark.parametrize("shape", sorted(set(workloads.densenet121_layer_shapes())))
def test_compact_densenet_layer_shapes(shape):
    x, K = _rand(shape, 4, 9)
    plan = build_plan_c(shape, K)
    check_compact(plan, shape, K)
    check_apply(plan, shape, K, x, 4)
    plan.close()


@pytest.mark.parametrize("name", sorted(workloads.WORKLOADS))
def test_compact_named_workloads_full_size(name):
    w = workloads.WORKLOADS[name]
    batch = min(w.batch, 16)
    x, K = _rand(w.shape, batch, 11)
    plan = build_plan_c(w.shape, K)
    check_compact(plan, w.shape, K)
    scaled, normwise = check_apply(plan, w.shape, K, x, batch)
    print("%s compact: variant %s, max err/scale %.2e" % (name, plan.variant(batch), scaled))
    plan.close()


@pytest.mark.parametrize("batch", [1, 2, 3, 4, 5, 8, 12, 16, 20, 32, 64])
def test_compact_batch_widths(batch):
    shape = (150, 270, 7, 1, 3)
    x, K = _rand(shape, batch, batch)
    plan = build_plan_c(shape, K)
    check_apply(plan, shape, K, x, batch)
    plan.close()


def test_compact_more_column_blocks_than_one_grid_holds():
    """An odd batch takes one scalar column per workgroup row; 65 541 of them need two launches."""
    shape, batch = (3, 4, 3, 1, 1), 65541
    x, K = _rand(shape, batch, 17)
    plan = build_plan_c(shape, K)
    check_apply(plan, shape, K, x, batch)
    plan.close()


def test_compact_unaligned_operands_take_the_scalar_columns():
    shape, batch = (80, 300, 7, 1, 3), 4
    m, n, k, s, p = shape
    x, K = _rand(shape, batch, 5)
    plan = build_plan_c(shape, K)
    buf = torch.zeros(m * n * batch + 1, dtype=torch.float32, device=device())
    buf[1:] = torch.from_numpy(x).to(device())
    check_apply(plan, shape, K, x, batch, x_dev=buf[1:])
    plan.close()


def _decoded_reference(shape, desc, ktab, x, batch):
    m, n, k, s, p = shape
    rp, ci, va = oracle.compact_decode(n, k, desc, ktab)
    rows = desc.shape[0]
    M = scipy.sparse.csr_matrix((va.astype(np.float64), ci, rp), shape=(rows, m * n))
    X = x.astype(np.float64).reshape(m * n, batch)
    A = scipy.sparse.csr_matrix((np.abs(va).astype(np.float64), ci, rp), shape=(rows, m * n))
    return (M @ X).reshape(-1), (A @ np.abs(X)).reshape(-1)


def _word(a_lo, r1, b_lo, r2):
    return np.array([a_lo | r1 << 8 | b_lo << 16 | r2 << 24], dtype=np.uint32).view(np.int32)[0]


@pytest.mark.parametrize("shape,batch", [((96, 300, 7, 1, 3), 16), ((96, 300, 7, 1, 3), 1), ((120, 200, 5, 2, 2), 8),
                                         ((60, 70, 40, 1, 20), 4),
                                         # strides 3 and 4: row groups by default; with the marching threshold
                                         # lowered the described path, the second with its lines prefetched
                                         ((150, 160, 9, 3, 8), 1), ((300, 1200, 11, 4, 5), 4)])
def test_compact_apply_reads_the_stored_descriptors(shape, batch, compact_dispatch):
    """Descriptors and table edited after the build: the product follows them.  Edits:
    shortened and shifted rectangles in the interior (a wave that holds one leaves the
    rectangle path), an emptied row, a row moved to lines far from its window (taps not
    resident in LDS), a rectangle that runs over a line end, and a changed table entry."""
    m, n, k, s, p = shape
    mo, no = oracle.out_shape(*shape)
    x, K = _rand(shape, batch, 21)
    plan = build_plan_c(shape, K)
    if shape[3] >= 3:
        want = "compact_described" if compact_dispatch == "marching_everywhere" else "compact_gather"
        assert plan.variant(batch).startswith(want), plan.variant(batch)
        if shape[3] == 4 and compact_dispatch == "marching_everywhere":
            assert "_prefetch_" in plan.variant(batch), plan.variant(batch)
    desc = plan.row_desc.cpu().numpy().copy()
    ktab = plan.ktab.cpu().numpy().copy()
    rng = np.random.default_rng(8)
    mid = (mo // 2) * no + no // 2
    desc[mid, 1] = _word(1, k - 2, 0, k - 1)                       # fewer taps, table offset moved
    desc[mid + 1, 0] += n + 1                                      # shifted one line down, one pixel right
    desc[mid + 2] = (0, 0)                                         # emptied
    desc[mid + no] = (0, _word(0, min(k, 3), 0, min(k, 3)))        # moved to the top-left corner of the image
    desc[mid + no + 1, 0] = (m - k) * n                            # moved to the bottom lines
    desc[5] = (n - 2, _word(0, 2, 0, min(k, 4)))                   # runs over the end of input line 0
    for r in rng.choice(mo * no, size=40, replace=False):          # random smaller rectangles in place
        if r in (mid, mid + 1, mid + 2, mid + no, mid + no + 1, 5):
            continue
        w = int(desc[r, 1].view(np.uint32)) if False else int(np.uint32(desc[r, 1]))
        a_lo, r1, b_lo, r2 = w & 255, (w >> 8) & 255, (w >> 16) & 255, w >> 24
        if r1 > 1 and r2 > 1:
            desc[r, 1] = _word(a_lo, r1 - 1, b_lo + 1, r2 - 1)
    ktab[k + 1 if k > 1 else 0] = 3.5
    plan.row_desc.copy_(torch.from_numpy(desc).to(device()))
    plan.ktab.copy_(torch.from_numpy(ktab).to(device()))
    y = torch.full((mo * no * batch,), float("nan"), dtype=torch.float32, device=device())
    cs.conv_spmv(plan, torch.from_numpy(x).to(device()), y, batch=batch)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    ref, scale = _decoded_reference(shape, desc, ktab, x, batch)
    assert not np.any(np.isnan(got))
    live = scale > 0
    assert np.all(got[~live] == 0.0)
    assert np.max(np.abs(got - ref)[live] / scale[live]) <= REL_TOL
    plan.close()


def test_compact_taps_outside_a_row_are_never_touched():
    """Inf in the kernel's first line and column: border rows that do not hold those taps stay
    finite (the taps are not stored, so nothing multiplies them); rows that hold them are Inf/NaN
    exactly where the decoded matrix says."""
    shape, batch = (70, 140, 7, 1, 3), 16
    m, n, k, s, p = shape
    x, K = _rand(shape, batch, 4)
    x = np.abs(x) + 0.5
    K = np.abs(K) + 0.5
    K[0] = np.inf
    plan = build_plan_c(shape, K)
    y = cs.conv_spmv(plan, torch.from_numpy(x).to(device()), batch=batch)
    torch.cuda.synchronize()
    got = y.cpu().numpy().reshape(70, 140, batch)
    assert np.all(np.isfinite(got[:3, :3])), "rows at the top-left border do not contain tap (0, 0)"
    assert np.all(np.isinf(got[3:, 3:])), "rows from line 3, column 3 on contain it"
    plan.close()


def test_compact_matches_the_csr_path_closely_and_is_repeatable():
    shape, batch = (200, 330, 7, 1, 3), 16
    x, K = _rand(shape, batch, 6)
    xd = torch.from_numpy(x).to(device())
    pc, pr = build_plan_c(shape, K), build_plan(shape, K)
    y1 = cs.conv_spmv(pc, xd, batch=batch)
    y2 = cs.conv_spmv(pc, xd, batch=batch)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        y3 = cs.conv_spmv(pc, xd, batch=batch, stream=side)
    yr = cs.conv_spmv(pr, xd, batch=batch)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2) and torch.equal(y1, y3)
    assert float((y1 - yr).abs().max()) <= 1e-4 * float(yr.abs().max())
    pc.close()
    pr.close()


def test_compact_update_kernel_rewrites_the_table_only():
    shape, batch = (90, 200, 5, 1, 2), 8
    x, K = _rand(shape, batch, 12)
    K2 = np.random.default_rng(13).standard_normal(25).astype(np.float32)
    plan = build_plan_c(shape, K)
    before = plan.row_desc.clone()
    cs.conv_update_kernel(plan, torch.from_numpy(K2).to(device()))
    torch.cuda.synchronize()
    assert torch.equal(before, plan.row_desc)
    check_compact(plan, shape, K2)
    check_apply(plan, shape, K2, x, batch)
    plan.close()


def test_compact_errors():
    dev = device()
    with pytest.raises(cs.ConvError) as e:
        cs.conv_compact_build(300, 300, 256, 1, 0, torch.zeros(256 * 256, device=dev))
    assert e.value.status == -1
    lib = binding._load()
    K = torch.ones(9, device=dev)
    buf = torch.zeros(2 * 16 + 1, dtype=torch.int32, device=dev)
    tab = torch.zeros(9, device=dev)
    h = ctypes.c_void_p()
    st = lib.conv_compact_build(4, 4, 3, 1, 1, K.data_ptr(), buf.data_ptr() + 4, tab.data_ptr(), None, ctypes.byref(h))
    assert st == -1 and not h.value                 # descriptors must be 8-byte aligned
    st = lib.conv_compact_build(4, 4, 3, 1, 1, K.data_ptr(), None, tab.data_ptr(), None, ctypes.byref(h))
    assert st == -2
    plan = build_plan_c((8, 8, 3, 1, 1), np.ones(9, dtype=np.float32))
    x = torch.zeros(64, device=dev)
    y = torch.zeros(64, device=dev)
    with pytest.raises(cs.ConvError):               # the fused multi-product launch takes CSR plans only
        cs.ConvMulti([plan], [x], [y], batch=1)
    assert lib.conv_plan_is_compact(plan._handle) == 1
    plan.close()


def test_compact_beyond_the_csr_index_range():
    """8192 x 8192, k = 7: 3.3e9 entries, more than int32 column-index arrays can address, so
    conv_csr_build refuses the shape; the structure-aware storage indexes rows and columns only.
    Descriptors in full and y in full against the oracle."""
    shape, batch = (8192, 8192, 7, 1, 3), 1
    m, n, k, s, p = shape
    assert oracle.nnz_closed(*shape) > 2 ** 31
    x, K = _rand(shape, batch, 23)
    with pytest.raises(cs.ConvError) as e:
        cs.conv_csr_build(m, n, k, s, p, torch.from_numpy(K).to(device()))
    assert e.value.status == -3
    plan = build_plan_c(shape, K)
    assert plan.nnz == oracle.nnz_closed(*shape)
    assert np.array_equal(plan.row_desc.cpu().numpy(), oracle.compact_rows(*shape))
    check_apply(plan, shape, K, x, batch)
    plan.close()
