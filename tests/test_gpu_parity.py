"""GPU parity: the HIP build and apply kernels, called through the C ABI,
against the CPU oracle on the same seeded host arrays.  CSR arrays must be
bit-exact; outputs within 1e-5 of the dot-product scale (see gpu_util)."""
import itertools

import numpy as np
import pytest
import torch

import oracle
import paper_2411_19419_amd as cs
from paper_2411_19419_amd import workloads

from gpu_util import REL_TOL, build_plan, check_apply, check_csr, device

pytestmark = pytest.mark.gpu


def _rand(shape, batch, seed):
    m, n, k, s, p = shape
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(m * n * batch).astype(np.float32),
            rng.standard_normal(k * k).astype(np.float32))


def test_exhaustive_tiny_grid():
    """Every valid shape with m, n <= 5, k <= 4, s <= 3, p <= 4 (k > m, p >= k
    with empty rows, slide remainders), batch cycling through 1, 3, 4, 8."""
    batches = itertools.cycle([1, 3, 4, 8])
    count = 0
    for shape in itertools.product(range(1, 6), range(1, 6), range(1, 5), range(1, 4), range(0, 5)):
        m, n, k, s, p = shape
        if k > m + 2 * p or k > n + 2 * p:
            continue
        batch = next(batches)
        x, K = _rand(shape, batch, count)
        plan = build_plan(shape, K)
        check_csr(plan, shape, K)
        check_apply(plan, shape, K, x, batch)
        plan.close()
        count += 1
    assert count > 1000


@pytest.mark.parametrize("shape", sorted(set(workloads.densenet121_layer_shapes())))
@pytest.mark.parametrize("batch", [1, 8])
def test_densenet_layer_shapes(shape, batch):
    x, K = _rand(shape, batch, 100 + batch)
    plan = build_plan(shape, K)
    check_csr(plan, shape, K)
    check_apply(plan, shape, K, x, batch)
    plan.close()


@pytest.mark.parametrize("name", list(workloads.WORKLOADS))
def test_named_workloads_full_size(name):
    """The measured configurations at their full sizes, every output compared."""
    w = workloads.WORKLOADS[name]
    x, K = workloads.make(w)
    plan = build_plan(w.shape, K)
    check_csr(plan, w.shape, K)
    scaled, normwise = check_apply(plan, w.shape, K, x, w.batch)
    print("%s: variant %s, max err/scale %.2e, normwise %.2e" % (name, plan.variant(w.batch), scaled, normwise))
    plan.close()


@pytest.mark.parametrize("shape,batch", [
    ((37, 53, 7, 1, 3), 16),      # several tiles and a ragged tail in both directions
    ((130, 67, 7, 1, 3), 16),
    ((64, 64, 7, 1, 3), 16),
    ((100, 90, 5, 2, 2), 16),
    ((33, 200, 3, 1, 1), 32),
    ((75, 75, 9, 3, 8), 4),
    ((90, 41, 11, 4, 5), 4),
    ((40, 40, 13, 1, 6), 2),      # k*k = 169 entries per row
    ((30, 30, 17, 2, 8), 16),     # k*k = 289
    ((50, 3, 3, 1, 1), 12),
    ((3, 50, 7, 2, 3), 5),        # k > m
    ((6, 6, 2, 1, 5), 7),         # p > k: mostly empty rows
    ((1, 1, 1, 5, 2), 3),         # no entries at all
    ((1, 1, 1, 1, 0), 1),
    ((200, 1, 1, 1, 0), 6),
    # long rows: the build stages 16, 4, 2, 1 rows per workgroup, then walks quads (rows beyond its LDS image)
    ((60, 70, 20, 1, 10), 3),
    ((50, 50, 30, 2, 15), 2),
    ((64, 64, 45, 1, 22), 1),
    ((70, 70, 60, 1, 30), 1),
    ((90, 90, 80, 1, 40), 1),
])
def test_ragged_and_degenerate_shapes(shape, batch):
    x, K = _rand(shape, batch, 7)
    plan = build_plan(shape, K)
    check_csr(plan, shape, K)
    check_apply(plan, shape, K, x, batch)
    plan.close()


@pytest.mark.parametrize("batch", [1, 2, 3, 4, 5, 8, 12, 16, 20, 24, 32, 48, 64])
def test_batch_widths(batch):
    shape = (45, 38, 5, 1, 2)
    x, K = _rand(shape, batch, batch)
    plan = build_plan(shape, K)
    check_apply(plan, shape, K, x, batch)
    plan.close()


def test_unaligned_operands_take_the_scalar_path():
    shape, batch = (29, 31, 3, 1, 1), 8
    x, K = _rand(shape, batch, 3)
    plan = build_plan(shape, K)
    m, n, k, s, p = shape
    buf = torch.zeros(x.size + 1, dtype=torch.float32, device=device())
    buf[1:] = torch.from_numpy(x).to(device())
    ybuf = torch.full((plan.rows * batch + 1,), float("nan"), dtype=torch.float32, device=device())
    cs.conv_spmv(plan, buf[1:], ybuf[1:], batch=batch)
    torch.cuda.synchronize()
    ref, scale = oracle.conv(m, n, k, s, p, x, K, batch=batch, want_scale=True)
    err = np.abs(ybuf[1:].cpu().numpy().astype(np.float64) - ref)
    assert np.max(err / np.maximum(scale, 1e-30)) <= 1e-5
    plan.close()


def test_apply_reads_the_stored_arrays():
    """Doubling vals doubles y; redirecting one stored column changes exactly
    that row, by the amount a CSR product over the edited arrays gives."""
    shape, batch = (40, 36, 5, 1, 2), 4
    m, n, k, s, p = shape
    x, K = _rand(shape, batch, 11)
    plan = build_plan(shape, K)
    xd = torch.from_numpy(x).to(device())
    y0 = cs.conv_spmv(plan, xd, batch=batch).clone()
    plan.vals.mul_(2.0)
    y1 = cs.conv_spmv(plan, xd, batch=batch).clone()
    torch.cuda.synchronize()
    assert torch.equal(y1, 2.0 * y0)
    plan.vals.mul_(0.5)
    rp, ci, va = oracle.csr(m, n, k, s, p, K)
    row = 17 * plan.n_out + 9
    e = int(rp[row]) + 3
    new_col = (m - 1) * n + (n - 1)          # far away from the row's window
    plan.col_idx[e] = new_col
    y2 = cs.conv_spmv(plan, xd, batch=batch)
    torch.cuda.synchronize()
    y0h, y2h = y0.cpu().numpy().reshape(-1, batch), y2.cpu().numpy().reshape(-1, batch)
    X = x.reshape(-1, batch).astype(np.float64)
    changed = np.where(np.any(y0h != y2h, axis=1))[0]
    assert changed.tolist() == [row]
    ci2 = ci.copy()
    ci2[e] = new_col
    seg = slice(int(rp[row]), int(rp[row + 1]))
    want = (va[seg].astype(np.float64)[:, None] * X[ci2[seg]]).sum(axis=0)
    scale = (np.abs(va[seg]).astype(np.float64)[:, None] * np.abs(X[ci2[seg]])).sum(axis=0)
    assert np.all(np.abs(y2h[row] - want) <= 1e-5 * scale)
    plan.close()


def test_repeatable_bit_for_bit_and_on_a_side_stream():
    shape, batch = (96, 80, 7, 1, 3), 16
    x, K = _rand(shape, batch, 5)
    plan = build_plan(shape, K)
    xd = torch.from_numpy(x).to(device())
    y0 = cs.conv_spmv(plan, xd, batch=batch).clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        y1 = cs.conv_spmv(plan, xd, batch=batch)
    side.synchronize()
    y2 = cs.conv_spmv(plan, xd, batch=batch)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1) and torch.equal(y0, y2)
    # a plan built on the side stream is identical too
    with torch.cuda.stream(side):
        plan2 = cs.conv_csr_build(*shape, torch.from_numpy(K).to(device()), stream=side)
    side.synchronize()
    assert torch.equal(plan.row_ptr, plan2.row_ptr) and torch.equal(plan.col_idx, plan2.col_idx)
    assert torch.equal(plan.vals, plan2.vals)
    plan.close()
    plan2.close()


def test_errors_on_device_calls():
    shape = (8, 8, 3, 1, 1)
    x, K = _rand(shape, 1, 1)
    plan = build_plan(shape, K)
    buf = torch.zeros(200, dtype=torch.float32, device=device())
    with pytest.raises(cs.ConvError) as ei:
        cs.conv_spmv(plan, buf[:64], buf[32:96], batch=1)        # overlapping x and y
    assert ei.value.status == -6
    lib = cs.binding._load()
    assert lib.conv_spmv(plan._handle, buf.data_ptr(), buf.data_ptr() + 400, 0, None) == -1      # batch < 1
    assert lib.conv_spmv(plan._handle, None, buf.data_ptr(), 1, None) == -2
    plan.close()


# ---------------------------------------------------------------------------
# The same checks with the dispatch knob set so that the persistent marching
# kernel is used wherever its geometry allows, however small the shape: partial
# strips, short segments, steps that run off the image, rows of every length.
# ---------------------------------------------------------------------------

@pytest.fixture
def march_everywhere():
    import gpu_util
    gpu_util.MARCH_MIN_JOBS = 1
    yield
    gpu_util.MARCH_MIN_JOBS = None


def test_march_edge_grid(march_everywhere):
    """The smallest shapes the marching kernels accept (workloads.march_edge_grid: one to a few
    output lines, strips with ragged ends, every padding from none to beyond the kernel, so
    empty rows, k > m and slide remainders all occur), each against the sliding-window oracle.
    Four in five of them must really take a marching kernel (all of those with stride 1; the
    CPU test test_march_edge_grid_dispatch checks which ones do not)."""
    count = used = 0
    kinds = set()
    for shape, batch in workloads.march_edge_grid():
        x, K = _rand(shape, batch, 1000 + count)
        plan = build_plan(shape, K)
        variant = plan.variant(batch)
        if variant.startswith("lds_march"):
            used += 1
            kinds.add("staged" if variant.startswith("lds_march_staged") else "groups")
        check_apply(plan, shape, K, x, batch)
        plan.close()
        count += 1
    assert count > 1500 and used >= 0.8 * count, (count, used)
    assert kinds == {"staged", "groups"}


MARCH_CASES = [
    ((37, 53, 7, 1, 3), 16), ((130, 67, 7, 1, 3), 16), ((64, 64, 7, 1, 3), 16), ((65, 129, 7, 1, 3), 1),
    ((100, 90, 5, 2, 2), 16), ((100, 90, 5, 2, 2), 8), ((100, 90, 5, 2, 2), 4), ((100, 90, 5, 2, 2), 1),
    ((33, 200, 3, 1, 1), 32), ((33, 200, 3, 1, 1), 1), ((70, 70, 1, 1, 0), 16), ((70, 70, 2, 2, 0), 8),
    ((75, 75, 9, 3, 8), 4), ((75, 75, 9, 3, 8), 16), ((75, 75, 9, 3, 8), 1), ((75, 75, 9, 3, 8), 8),
    ((90, 141, 11, 4, 5), 4), ((90, 141, 11, 4, 5), 1), ((150, 150, 11, 1, 5), 8), ((150, 150, 11, 1, 5), 16),
    ((140, 40, 7, 3, 3), 16), ((40, 140, 7, 5, 0), 4), ((200, 200, 3, 2, 1), 16), ((120, 120, 9, 1, 4), 16),
    ((3, 150, 7, 2, 3), 4), ((50, 50, 2, 1, 5), 8), ((64, 64, 4, 1, 6), 1), ((97, 33, 6, 1, 2), 12),
]


def test_march_ragged_shapes(march_everywhere):
    """Ring of 16 and of 8 lines, steps of one and two lines, 8 and 16 lanes per
    row, scalar / float4 x 1, 2, 4 columns.  A few of the cases do not fit the LDS
    planes and fall back; most must take the marching kernel."""
    variants = {}
    for shape, batch in MARCH_CASES:
        x, K = _rand(shape, batch, 17)
        plan = build_plan(shape, K)
        variants[(shape, batch)] = plan.variant(batch)
        check_apply(plan, shape, K, x, batch)
        plan.close()
    marching = [v for v in variants.values() if v.startswith("lds_march")]
    print(variants)
    assert len(marching) >= 16, variants
    kinds = {v.split("_", 3)[3] for v in marching}          # ring/step/lanes/trip/columns
    assert len(kinds) >= 8, kinds


@pytest.mark.parametrize("shape", sorted(set(workloads.densenet121_layer_shapes())))
@pytest.mark.parametrize("batch", [1, 4, 16])
def test_march_densenet_layer_shapes(march_everywhere, shape, batch):
    x, K = _rand(shape, batch, 300 + batch)
    plan = build_plan(shape, K)
    check_apply(plan, shape, K, x, batch)
    plan.close()


@pytest.mark.parametrize("batch", [1, 16])
@pytest.mark.parametrize("shape", [(96, 80, 7, 1, 3), (96, 80, 9, 1, 4), (96, 80, 11, 1, 5)])   # 2, 4, 8 lanes per row
def test_march_reads_the_stored_arrays(march_everywhere, shape, batch):
    """Edited arrays under the marching kernel: a column far outside the resident
    lines must be fetched from global memory (the cold path), scaled values scale y."""
    m, n, k, s, p = shape
    x, K = _rand(shape, batch, 23)
    plan = build_plan(shape, K)
    assert plan.variant(batch).startswith("lds_march_staged") and "_g%d_" % {7: 2, 9: 4, 11: 8}[k] in plan.variant(batch)
    xd = torch.from_numpy(x).to(device())
    y0 = cs.conv_spmv(plan, xd, batch=batch).clone()
    plan.vals.mul_(2.0)
    y1 = cs.conv_spmv(plan, xd, batch=batch).clone()
    torch.cuda.synchronize()
    assert torch.equal(y1, 2.0 * y0)
    plan.vals.mul_(0.5)
    rp, ci, va = oracle.csr(m, n, k, s, p, K)
    edits = {40 * plan.n_out + 9: ((m - 1) * n + (n - 1), 3),      # far below the window
             41 * plan.n_out + 70: (0, 0),                          # far above it
             7 * plan.n_out + 33: (7 * n + 79, 10)}                 # right line, column outside the strip
    ci2 = ci.copy()
    for row, (new_col, slot) in edits.items():
        e = int(rp[row]) + slot
        plan.col_idx[e] = new_col
        ci2[e] = new_col
    y2 = cs.conv_spmv(plan, xd, batch=batch)
    torch.cuda.synchronize()
    y0h, y2h = y0.cpu().numpy().reshape(-1, batch), y2.cpu().numpy().reshape(-1, batch)
    X = x.reshape(-1, batch).astype(np.float64)
    changed = np.where(np.any(y0h != y2h, axis=1))[0]
    assert sorted(changed.tolist()) == sorted(edits)
    for row in edits:
        seg = slice(int(rp[row]), int(rp[row + 1]))
        want = (va[seg].astype(np.float64)[:, None] * X[ci2[seg]]).sum(axis=0)
        scale = (np.abs(va[seg]).astype(np.float64)[:, None] * np.abs(X[ci2[seg]])).sum(axis=0)
        assert np.all(np.abs(y2h[row] - want) <= 1e-5 * scale)
    plan.close()


def test_march_is_repeatable_bit_for_bit(march_everywhere):
    shape, batch = (130, 70, 5, 1, 2), 16
    x, K = _rand(shape, batch, 29)
    plan = build_plan(shape, K)
    xd = torch.from_numpy(x).to(device())
    ys = [cs.conv_spmv(plan, xd, batch=batch).clone() for _ in range(3)]
    torch.cuda.synchronize()
    assert torch.equal(ys[0], ys[1]) and torch.equal(ys[0], ys[2])
    plan.close()


def test_inf_and_nan_stay_in_their_rows(march_everywhere):
    """A non-finite input pixel must reach exactly the outputs whose windows contain it."""
    shape, batch = (70, 70, 3, 1, 1), 4
    m, n, k, s, p = shape
    x, K = _rand(shape, batch, 31)
    K = np.abs(K) + 0.5
    x = x.copy()
    bad = (30 * n + 40) * batch + 2
    x[bad] = np.inf
    plan = build_plan(shape, K)
    y = cs.conv_spmv(plan, torch.from_numpy(x).to(device()), batch=batch)
    torch.cuda.synchronize()
    got = y.cpu().numpy().reshape(plan.m_out, plan.n_out, batch)
    nonfinite = ~np.isfinite(got)
    want = np.zeros_like(nonfinite)
    want[29:32, 39:42, 2] = True
    assert np.array_equal(nonfinite, want)
    plan.close()


def test_update_kernel_rewrites_vals_only():
    """A new K for a built T: vals equal the oracle's enumeration with the new K
    bit for bit, indices are untouched, and the apply follows."""
    for shape, batch in [((96, 80, 7, 1, 3), 16), ((75, 75, 9, 3, 8), 4), ((33, 50, 2, 2, 0), 1), ((6, 6, 2, 1, 5), 4)]:
        m, n, k, s, p = shape
        x, K = _rand(shape, batch, 41)
        K2 = np.random.default_rng(43).standard_normal(k * k).astype(np.float32)
        plan = build_plan(shape, K)
        rp_before, ci_before = plan.row_ptr.clone(), plan.col_idx.clone()
        cs.conv_update_kernel(plan, torch.from_numpy(K2).to(device()))
        torch.cuda.synchronize()
        assert torch.equal(plan.row_ptr, rp_before) and torch.equal(plan.col_idx, ci_before)
        check_csr(plan, shape, K2)
        check_apply(plan, shape, K2, x, batch)
        plan.close()


@pytest.mark.parametrize("batch", [1, 3])
def test_fused_layer_sweep_matches_oracle_layer_by_layer(batch):
    """All 123 layer shapes of Table 2 in one launch (conv_multi_apply), each
    output against the sliding-window oracle, and against conv_spmv on the same plan."""
    layers = list(workloads.densenet121_sweep(batch=batch))
    assert len(layers) == 123
    plans = [build_plan(shape, K) for shape, _, K in layers]
    xs = [torch.from_numpy(x).to(device()) for _, x, _ in layers]
    ys = [torch.full((pl.rows * batch,), float("nan"), dtype=torch.float32, device=device()) for pl in plans]
    multi = cs.ConvMulti(plans, xs, ys, batch=batch)
    multi.apply()
    torch.cuda.synchronize()
    for (shape, x, K), pl, xd, y in zip(layers, plans, xs, ys):
        m, n, k, s, p = shape
        ref, scale = oracle.conv(m, n, k, s, p, x, K, batch=batch, want_scale=True)
        got = y.cpu().numpy()
        assert not np.any(np.isnan(got))
        err = np.abs(got.astype(np.float64) - ref)
        assert np.max(err / np.maximum(scale, 1e-30)) <= 1e-5, shape
        single = cs.conv_spmv(pl, xd, batch=batch)
        torch.cuda.synchronize()
        assert np.max(np.abs(single.cpu().numpy().astype(np.float64) - ref) / np.maximum(scale, 1e-30)) <= 1e-5
    multi.apply()                      # a second apply gives the same bits
    torch.cuda.synchronize()
    again = [y.clone() for y in ys]
    multi.apply()
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(again, ys))
    multi.close()
    for pl in plans:
        pl.close()


def test_fused_apply_mixed_shapes_and_errors():
    shapes = [(40, 36, 5, 1, 2), (6, 6, 2, 1, 5), (1, 1, 1, 5, 2), (33, 20, 11, 2, 5), (50, 50, 13, 1, 6)]
    batch = 2
    plans, xs, ys, data = [], [], [], []
    for i, shape in enumerate(shapes):
        x, K = _rand(shape, batch, 50 + i)
        plans.append(build_plan(shape, K))
        xs.append(torch.from_numpy(x).to(device()))
        ys.append(torch.full((plans[-1].rows * batch,), float("nan"), dtype=torch.float32, device=device()))
        data.append((x, K))
    multi = cs.ConvMulti(plans, xs, ys, batch=batch)
    multi.apply()
    torch.cuda.synchronize()
    for shape, (x, K), y in zip(shapes, data, ys):
        m, n, k, s, p = shape
        ref, scale = oracle.conv(m, n, k, s, p, x, K, batch=batch, want_scale=True)
        got = y.cpu().numpy()
        assert not np.any(np.isnan(got))
        empty = scale == 0
        assert np.all(got[empty] == 0.0)
        assert np.all(np.abs(got.astype(np.float64) - ref)[~empty] <= 1e-5 * scale[~empty])
    multi.close()
    with pytest.raises(cs.ConvError) as ei:       # x and y of one product overlap
        buf = torch.zeros(plans[0].cols * batch + plans[0].rows * batch, device=device())
        cs.ConvMulti([plans[0]], [buf[:plans[0].cols * batch]], [buf[8:8 + plans[0].rows * batch]], batch=batch)
    assert ei.value.status == -6
    for pl in plans:
        pl.close()


def test_largest_index_range():
    """nnz just below 2^31 (the limit of the int32 indices): 6600 x 6600, k = 7, 'same' padding
    gives 2 133 331 344 entries.  row_ptr is compared in full with the prefix sums of Theorem
    2.1's row lengths, col_idx / vals on the first, last and 3000 random rows with the oracle's
    tap enumeration, y in full with the sliding-window oracle; the structure-aware storage of
    the same T likewise (descriptors in full)."""
    shape, batch = (6600, 6600, 7, 1, 3), 1
    m, n, k, s, p = shape
    mo, no = oracle.out_shape(*shape)
    nnz = oracle.nnz_closed(*shape)
    assert 2 ** 31 - 2 ** 24 < nnz < 2 ** 31
    rng = np.random.default_rng(31)
    x = rng.standard_normal(m * n * batch).astype(np.float32)
    K = rng.standard_normal(k * k).astype(np.float32)
    plan = build_plan(shape, K)
    assert plan.nnz == nnz
    # row_ptr: exclusive prefix sums of r1(x) r2(y) (Theorem 2.1), in int64 on the host
    t1, t2 = np.arange(mo, dtype=np.int64), np.arange(no, dtype=np.int64)
    r1 = np.maximum(0, k - np.maximum(0, p - s * t1) - np.maximum(0, s * t1 + k - m - p))
    r2 = np.maximum(0, k - np.maximum(0, p - s * t2) - np.maximum(0, s * t2 + k - n - p))
    want = np.concatenate([[0], np.cumsum(np.outer(r1, r2).reshape(-1))])
    assert want[-1] == nnz
    got_rp = plan.row_ptr.cpu().numpy()
    assert np.array_equal(got_rp.astype(np.int64), want)
    del want
    rows = np.unique(np.concatenate([np.arange(200), np.arange(mo * no - 200, mo * no),
                                     rng.integers(0, mo * no, size=3000)]))
    for r in rows:
        cols, vals = oracle.csr_row(m, n, k, s, p, K, int(r))
        lo, hi = int(got_rp[r]), int(got_rp[r + 1])
        assert np.array_equal(plan.col_idx[lo:hi].cpu().numpy().astype(np.int64), cols), r
        assert np.array_equal(plan.vals[lo:hi].cpu().numpy().view(np.uint32), vals.view(np.uint32)), r
    xd = torch.from_numpy(x).to(device())
    ref, scale = oracle.conv(m, n, k, s, p, x, K, batch=batch, want_scale=True)

    def compare(pl):
        y = torch.full((mo * no * batch,), float("nan"), dtype=torch.float32, device=device())
        cs.conv_spmv(pl, xd, y, batch=batch)
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        assert not np.any(np.isnan(got))
        assert np.max(np.abs(got.astype(np.float64) - ref) / scale) <= REL_TOL

    compare(plan)
    print("largest: variant %s" % plan.variant(batch))
    plan.close()
    del plan
    torch.cuda.empty_cache()
    pc = cs.conv_compact_build(m, n, k, s, p, torch.from_numpy(K).to(device()))
    assert np.array_equal(pc.row_desc.cpu().numpy(), oracle.compact_rows(*shape))
    compare(pc)
    pc.close()


def test_graph_replays_match_eager_applies():
    """The applies only enqueue kernels, so they can be captured in a HIP graph.  Replays, with
    eager applies and synchronisations between them and a fresh x before each, are compared
    bit for bit with the eager result (CSR marching kernel, Tᵀ, structure-aware storage)."""
    shape, batch = (300, 520, 7, 1, 3), 16
    m, n, k, s, p = shape
    rng = np.random.default_rng(41)
    K = rng.standard_normal(k * k).astype(np.float32)
    Kd = torch.from_numpy(K).to(device())
    plans = [cs.conv_csr_build(m, n, k, s, p, Kd), cs.conv_csc_build(m, n, k, s, p, Kd),
             cs.conv_compact_build(m, n, k, s, p, Kd)]
    xs = [torch.empty(pl.cols * batch, dtype=torch.float32, device=device()) for pl in plans]
    ys = [torch.empty(pl.rows * batch, dtype=torch.float32, device=device()) for pl in plans]
    for pl, x, y in zip(plans, xs, ys):          # first launches outside the capture
        x.normal_()
        cs.conv_spmv(pl, x, y, batch=batch)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for pl, x, y in zip(plans, xs, ys):
            cs.conv_spmv(pl, x, y, batch=batch)
    for rep in range(4):
        for x in xs:
            x.normal_()
        eager = [cs.conv_spmv(pl, x, batch=batch) for pl, x in zip(plans, xs)]
        torch.cuda.synchronize()
        for y in ys:
            y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for pl, y, e in zip(plans, ys, eager):
            assert torch.equal(y, e), (rep, pl.variant(batch))
    for pl in plans:
        pl.close()


def test_graph_replays_of_channel_sums_and_of_the_csc_product():
    """The same for the sums over channels (one launch from the structure-aware storage, the
    row-group kernel and the per-channel launches from CSR: bit for bit) and for y = T x from the
    column-compressed arrays (a fill kernel and a scatter; its adds arrive in timing order, so
    replays are compared with the eager result to the parity tolerance)."""
    shape, channels, batch = (120, 136, 3, 1, 1), 6, 16
    m, n, k, s, p = shape
    rng = np.random.default_rng(43)
    Kd = torch.from_numpy(rng.standard_normal(channels * k * k).astype(np.float32)).to(device())
    sums = [cs.conv_compact_build(m, n, k, s, p, Kd, channels=channels), cs.conv_csr_build_channels(m, n, k, s, p, Kd, channels)]
    assert sums[0].variant(batch).startswith("compact_channels")
    tshape = (300, 520, 7, 1, 3)
    Kt = rng.standard_normal(49).astype(np.float32)
    csc = cs.conv_csc_build(*tshape, torch.from_numpy(Kt).to(device()))
    xs = [torch.empty(pl.cols * batch, dtype=torch.float32, device=device()).normal_() for pl in sums]
    ys = [torch.empty(pl.rows * batch, dtype=torch.float32, device=device()) for pl in sums]
    xt = torch.empty(csc.rows * batch, dtype=torch.float32, device=device()).normal_()
    yt = torch.empty(csc.cols * batch, dtype=torch.float32, device=device())
    for pl, x, y in zip(sums, xs, ys):           # first launches outside the capture
        cs.conv_spmv(pl, x, y, batch=batch)
    cs.conv_spmv_from_csc(csc, xt, yt, batch=batch)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for pl, x, y in zip(sums, xs, ys):
            cs.conv_spmv(pl, x, y, batch=batch)
        cs.conv_spmv_from_csc(csc, xt, yt, batch=batch)
    for rep in range(4):
        for x in xs + [xt]:
            x.normal_()
        eager = [cs.conv_spmv(pl, x, batch=batch) for pl, x in zip(sums, xs)]
        torch.cuda.synchronize()
        for y in ys + [yt]:
            y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for pl, y, e in zip(sums, ys, eager):
            assert torch.equal(y, e), (rep, pl.variant(batch))
        ref, scale = oracle.conv(*tshape, xt.cpu().numpy(), Kt, batch=batch, want_scale=True)
        err = np.abs(yt.cpu().numpy().astype(np.float64) - ref.astype(np.float64))
        assert np.all(err <= REL_TOL * scale + 1e-30), rep
    for pl in sums + [csc]:
        pl.close()
