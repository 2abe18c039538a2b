"""GPU parity for the transposed side: T column-compressed (conv_csc_build) bit-exact
against the oracle, and y = T^T x (conv_spmv on that plan) against the adjoint oracle."""
import itertools

import numpy as np
import pytest
import torch

import oracle
import paper_2411_19419_amd as cs
from paper_2411_19419_amd import workloads

from gpu_util import build_plan, build_plan_t, check_apply_t, check_csc, device

pytestmark = pytest.mark.gpu


def _rand_t(shape, batch, seed):
    m, n, k, s, p = shape
    mo, no = oracle.out_shape(*shape)
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(mo * no * batch).astype(np.float32),
            rng.standard_normal(k * k).astype(np.float32))


def test_transposed_exhaustive_tiny_grid():
    batches = itertools.cycle([1, 3, 4, 8])
    count = 0
    for shape in itertools.product(range(1, 6), range(1, 6), range(1, 5), range(1, 4), range(0, 5)):
        m, n, k, s, p = shape
        if k > m + 2 * p or k > n + 2 * p:
            continue
        batch = next(batches)
        u, K = _rand_t(shape, batch, count)
        plan = build_plan_t(shape, K)
        check_csc(plan, shape, K)
        check_apply_t(plan, shape, K, u, batch)
        plan.close()
        count += 1
    assert count > 1000


@pytest.mark.parametrize("shape,batch", [
    ((37, 53, 7, 1, 3), 16), ((130, 67, 7, 1, 3), 4), ((100, 90, 5, 2, 2), 16), ((33, 200, 3, 1, 1), 1),
    ((75, 75, 9, 3, 8), 4), ((90, 141, 11, 4, 5), 2), ((40, 40, 13, 1, 6), 3), ((3, 50, 7, 2, 3), 5),
    ((6, 6, 2, 1, 5), 7), ((1, 1, 1, 5, 2), 3), ((200, 1, 1, 1, 0), 6), ((300, 301, 2, 2, 0), 8),
    ((257, 513, 3, 2, 1), 1), ((64, 1000, 5, 3, 1), 4),
    ((60, 70, 20, 1, 10), 3), ((50, 50, 30, 2, 15), 2), ((64, 64, 45, 1, 22), 1), ((70, 70, 60, 1, 30), 1),
    ((90, 90, 80, 1, 40), 1),          # long rows: every staging width of the build, and its fallback
])
def test_transposed_ragged_and_degenerate_shapes(shape, batch):
    u, K = _rand_t(shape, batch, 7)
    plan = build_plan_t(shape, K)
    check_csc(plan, shape, K)
    check_apply_t(plan, shape, K, u, batch)
    plan.close()


@pytest.mark.parametrize("shape", sorted(set(workloads.densenet121_layer_shapes())))
def test_transposed_densenet_layer_shapes(shape):
    u, K = _rand_t(shape, 4, 9)
    plan = build_plan_t(shape, K)
    check_csc(plan, shape, K)
    check_apply_t(plan, shape, K, u, 4)
    plan.close()


@pytest.mark.parametrize("name", ["strided_256_k5_b64", "headline_1024_k7_b16", "padheavy_512_k9_s3",
                                  "padheavy_4096_k11_s4_b4"])
def test_transposed_named_workloads_full_size(name):
    w = workloads.WORKLOADS[name]
    batch = min(w.batch, 16)
    u, K = _rand_t(w.shape, batch, 11)
    plan = build_plan_t(w.shape, K)
    check_csc(plan, w.shape, K)
    scaled, normwise = check_apply_t(plan, w.shape, K, u, batch)
    print("%s transposed: variant %s, max err/scale %.2e" % (name, plan.variant(batch), scaled))
    plan.close()


@pytest.mark.parametrize("name", ["strided_256_k5_b64", "headline_1024_k7_b1", "headline_1024_k7_b16",
                                  "padheavy_512_k9_s3", "cnn_224_k3_b256"])
def test_product_from_csc_named_workloads_full_size(name):
    """y = T x from the column-compressed arrays at the sizes the benchmark times, the whole result
    against the sliding-window oracle."""
    w = workloads.WORKLOADS[name]
    batch = min(w.batch, 64)
    m, n, k, s, p = w.shape
    rng = np.random.default_rng(17)
    x = rng.standard_normal(m * n * batch).astype(np.float32)
    K = rng.standard_normal(k * k).astype(np.float32)
    plan = build_plan_t(w.shape, K)
    y = cs.conv_spmv_from_csc(plan, torch.from_numpy(x).to(device()), batch=batch)
    torch.cuda.synchronize()
    got = y.cpu().numpy()
    ref, scale = oracle.conv(m, n, k, s, p, x, K, batch=batch, want_scale=True)
    live = scale > 0
    assert np.all(got[~live] == 0.0)
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    worst = float(np.max(err[live] / scale[live]))
    print("%s from CSC: max err/scale %.2e" % (name, worst))
    assert worst <= 1e-5
    plan.close()


def test_adjoint_identity_on_the_device():
    """<T x, u> = <x, T^T u> with both products from the GPU (integers: exact in fp32)."""
    shape, batch = (60, 44, 5, 2, 2), 1
    m, n, k, s, p = shape
    mo, no = oracle.out_shape(*shape)
    rng = np.random.default_rng(3)
    K = rng.integers(-3, 4, size=k * k).astype(np.float32)
    x = rng.integers(-4, 5, size=m * n).astype(np.float32)
    u = rng.integers(-4, 5, size=mo * no).astype(np.float32)
    fwd, bwd = build_plan(shape, K), build_plan_t(shape, K)
    y = cs.conv_spmv(fwd, torch.from_numpy(x).to(device()), batch=batch)
    z = cs.conv_spmv(bwd, torch.from_numpy(u).to(device()), batch=batch)
    torch.cuda.synchronize()
    lhs = float(np.dot(y.cpu().numpy().astype(np.float64), u))
    rhs = float(np.dot(x.astype(np.float64), z.cpu().numpy().astype(np.float64)))
    assert lhs == rhs
    fwd.close()
    bwd.close()


def test_transposed_update_kernel_and_fused_apply():
    shape, batch = (50, 40, 3, 2, 1), 2
    u, K = _rand_t(shape, batch, 21)
    K2 = np.random.default_rng(22).standard_normal(9).astype(np.float32)
    plan = build_plan_t(shape, K)
    cs.conv_update_kernel(plan, torch.from_numpy(K2).to(device()))
    torch.cuda.synchronize()
    check_csc(plan, shape, K2)
    check_apply_t(plan, shape, K2, u, batch)
    ud = torch.from_numpy(u).to(device())
    z = torch.full((plan.rows * batch,), float("nan"), dtype=torch.float32, device=device())
    multi = cs.ConvMulti([plan], [ud], [z], batch=batch)
    multi.apply()
    torch.cuda.synchronize()
    ref, scale = oracle.conv_t(*shape, u, K2, batch=batch, want_scale=True)
    assert np.all(np.abs(z.cpu().numpy().astype(np.float64) - ref) <= 1e-5 * np.maximum(scale, 1e-30))
    multi.close()
    plan.close()


# ---- the same with the marching kernel forced wherever its geometry allows

@pytest.fixture
def march_everywhere():
    import gpu_util
    gpu_util.MARCH_MIN_JOBS = 1
    yield
    gpu_util.MARCH_MIN_JOBS = None


def test_transposed_march_edge_grid(march_everywhere):
    """z = T^T u on the smallest shapes the marching kernels accept for the transposed matrix
    (workloads.march_edge_grid(transposed=True): result lines are input lines here, so n >= 32
    and ceil(k/s)^2 >= 9 entries per row), each against the scatter-and-crop oracle."""
    count = used = 0
    for shape, batch in workloads.march_edge_grid(transposed=True):
        u, K = _rand_t(shape, batch, 2000 + count)
        plan = build_plan_t(shape, K)
        used += plan.variant(batch).startswith("lds_march")
        check_apply_t(plan, shape, K, u, batch)
        plan.close()
        count += 1
    assert count > 1000 and used >= 0.8 * count, (count, used)


def test_transposed_march_ragged_shapes(march_everywhere):
    cases = [((37, 53, 7, 1, 3), 16), ((130, 67, 7, 1, 3), 16), ((65, 129, 7, 1, 3), 1), ((100, 90, 5, 2, 2), 16),
             ((100, 90, 5, 2, 2), 1), ((33, 200, 3, 1, 1), 32), ((70, 70, 1, 1, 0), 16), ((70, 70, 2, 2, 0), 8),
             ((75, 75, 9, 3, 8), 4), ((75, 75, 9, 3, 8), 16), ((90, 141, 11, 4, 5), 4), ((150, 150, 11, 1, 5), 8),
             ((140, 40, 7, 3, 3), 16), ((40, 140, 7, 5, 0), 4), ((200, 200, 3, 2, 1), 16), ((120, 120, 9, 1, 4), 16),
             ((50, 50, 2, 1, 5), 8), ((64, 64, 4, 1, 6), 1), ((97, 33, 6, 1, 2), 12), ((257, 300, 3, 1, 1), 4),
             ((90, 141, 11, 2, 5), 4), ((75, 75, 9, 2, 4), 16), ((140, 40, 7, 2, 3), 16), ((120, 100, 11, 3, 5), 8),
             ((130, 130, 11, 2, 5), 1), ((66, 200, 8, 2, 3), 8)]
    variants = {}
    for shape, batch in cases:
        u, K = _rand_t(shape, batch, 19)
        plan = build_plan_t(shape, K)
        variants[(shape, batch)] = plan.variant(batch)
        check_apply_t(plan, shape, K, u, batch)
        plan.close()
    marching = [v for v in variants.values() if v.startswith("lds_march")]
    print(variants)
    assert len(marching) >= 10, variants


def test_transposed_march_reads_the_stored_arrays(march_everywhere):
    shape, batch = (96, 80, 7, 1, 3), 16
    m, n, k, s, p = shape
    u, K = _rand_t(shape, batch, 23)
    plan = build_plan_t(shape, K)
    assert plan.variant(batch).startswith("lds_march")
    ud = torch.from_numpy(u).to(device())
    z0 = cs.conv_spmv(plan, ud, batch=batch).clone()
    cp, ri, va = oracle.csc(m, n, k, s, p, K)
    row = 40 * n + 9
    e = int(cp[row]) + 5
    new_col = plan.cols - 1
    plan.col_idx[e] = new_col
    z1 = cs.conv_spmv(plan, ud, batch=batch)
    torch.cuda.synchronize()
    z0h, z1h = z0.cpu().numpy().reshape(-1, batch), z1.cpu().numpy().reshape(-1, batch)
    assert np.where(np.any(z0h != z1h, axis=1))[0].tolist() == [row]
    U = u.reshape(-1, batch).astype(np.float64)
    ri2 = ri.copy()
    ri2[e] = new_col
    seg = slice(int(cp[row]), int(cp[row + 1]))
    want = (va[seg].astype(np.float64)[:, None] * U[ri2[seg]]).sum(axis=0)
    scale = (np.abs(va[seg]).astype(np.float64)[:, None] * np.abs(U[ri2[seg]])).sum(axis=0)
    assert np.all(np.abs(z1h[row] - want) <= 1e-5 * scale)
    plan.close()


@pytest.mark.parametrize("shape,batch", [
    ((37, 53, 7, 1, 3), 16), ((130, 67, 7, 1, 3), 4), ((100, 90, 5, 2, 2), 8), ((33, 200, 3, 1, 1), 1),
    ((75, 75, 9, 3, 8), 3), ((40, 40, 13, 1, 6), 5), ((6, 6, 2, 1, 5), 7), ((1, 1, 1, 5, 2), 3),
    ((224, 224, 7, 2, 3), 16), ((5, 5, 2, 2, 0), 4), ((300, 301, 2, 2, 0), 12),
    # batch tails of the four-column lanes and of the sixteen-column pass
    ((90, 77, 7, 1, 3), 2), ((90, 77, 7, 1, 3), 9), ((90, 77, 7, 1, 3), 17), ((61, 45, 5, 1, 2), 33),
    # columns no window covers (s > k), one tile line per column (k = 31), beyond the stage (k = 40)
    ((60, 60, 3, 5, 0), 4), ((70, 70, 31, 1, 15), 3), ((50, 50, 40, 1, 20), 2), ((64, 48, 17, 2, 8), 16),
    # columns of 4 entries: on chip from batch 4 on, directly below; of 1 entry: always directly
    ((90, 77, 2, 1, 1), 4), ((90, 77, 2, 1, 1), 3), ((90, 77, 3, 2, 1), 16), ((90, 77, 4, 2, 2), 8), ((90, 77, 2, 2, 0), 16),
    # a few lines of many tiles, many lines of one tile, several full tiles with a ragged rim
    ((3, 700, 5, 1, 2), 16), ((700, 3, 5, 1, 2), 16), ((515, 509, 7, 1, 3), 16), ((259, 263, 3, 1, 1), 1),
])
def test_product_from_the_csc_arrays_is_the_convolution(shape, batch):
    """y = T x computed by scattering the column-compressed entries (the paper's CSC variant)
    against the sliding-window oracle.  The additions happen in a timing-dependent order, so two
    runs are compared with each other to the same tolerance, not bit for bit."""
    m, n, k, s, p = shape
    rng = np.random.default_rng(13)
    x = rng.standard_normal(m * n * batch).astype(np.float32)
    K = rng.standard_normal(k * k).astype(np.float32)
    plan = build_plan_t(shape, K)
    xd = torch.from_numpy(x).to(device())
    y = torch.full((plan.cols * batch,), float("nan"), dtype=torch.float32, device=device())
    cs.conv_spmv_from_csc(plan, xd, y, batch=batch)
    y2 = cs.conv_spmv_from_csc(plan, xd, batch=batch)
    torch.cuda.synchronize()
    ref, scale = oracle.conv(m, n, k, s, p, x, K, batch=batch, want_scale=True)
    for got in (y.cpu().numpy(), y2.cpu().numpy()):
        assert not np.any(np.isnan(got))
        live = scale > 0
        assert np.all(got[~live] == 0.0)
        err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
        assert (np.max(err[live] / scale[live]) if np.any(live) else 0.0) <= 1e-5
    plan.close()


def test_product_from_csc_on_random_small_shapes():
    """Three hundred random shapes (planes up to 70 x 70, k up to 12, strides up to 5, paddings up
    to 9: windows clipped on every side, pixels no window covers, tiles of one line or one
    column) at the batch widths that select every lane layout of the scatter."""
    rng = np.random.default_rng(2024)
    batches = [1, 2, 3, 4, 5, 8, 9, 16, 20]
    done = 0
    while done < 300:
        k, s, p = int(rng.integers(1, 13)), int(rng.integers(1, 6)), int(rng.integers(0, 10))
        m, n = (int(v) for v in rng.integers(1, 71, size=2))
        if k > m + 2 * p or k > n + 2 * p:
            continue
        batch = batches[done % len(batches)]
        x = rng.standard_normal(m * n * batch).astype(np.float32)
        K = rng.standard_normal(k * k).astype(np.float32)
        plan = build_plan_t((m, n, k, s, p), K)
        y = cs.conv_spmv_from_csc(plan, torch.from_numpy(x).to(device()), batch=batch)
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        ref, scale = oracle.conv(m, n, k, s, p, x, K, batch=batch, want_scale=True)
        err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
        assert np.all(got[scale == 0] == 0.0), (m, n, k, s, p, batch)
        assert np.all(err <= 1e-5 * scale), (m, n, k, s, p, batch)
        plan.close()
        done += 1


@pytest.mark.parametrize("offset,batch", [(1, 1), (3, 2), (2, 5), (1, 16)])
def test_product_from_csc_into_an_unaligned_result(offset, batch):
    """y that does not start on a 16-byte boundary (the zero fill before the scatter uses 16-byte
    stores over the aligned middle); the floats around y stay untouched."""
    shape = (45, 38, 5, 1, 2)
    m, n, k, s, p = shape
    rng = np.random.default_rng(31)
    x = rng.standard_normal(m * n * batch).astype(np.float32)
    K = rng.standard_normal(k * k).astype(np.float32)
    plan = build_plan_t(shape, K)
    count = plan.cols * batch
    buf = torch.full((count + 8,), 7.0, dtype=torch.float32, device=device())
    cs.conv_spmv_from_csc(plan, torch.from_numpy(x).to(device()), buf[offset:offset + count], batch=batch)
    torch.cuda.synchronize()
    got = buf.cpu().numpy()
    assert np.all(got[:offset] == 7.0) and np.all(got[offset + count:] == 7.0)
    ref, scale = oracle.conv(m, n, k, s, p, x, K, batch=batch, want_scale=True)
    err = np.abs(got[offset:offset + count].astype(np.float64) - ref.astype(np.float64))
    assert np.all(err <= 1e-5 * scale + 1e-30)
    plan.close()


def test_product_from_csc_reads_the_stored_arrays():
    """The scatter uses the stored row indices and values, wherever they point: one entry of a
    column is sent to a row far from the pixel's windows (outside what the workgroup keeps on
    chip) and one value is changed; the result must be the product with that edited matrix."""
    import scipy.sparse as sp
    shape, batch = (96, 80, 7, 1, 3), 16
    m, n, k, s, p = shape
    rng = np.random.default_rng(29)
    x = rng.standard_normal(m * n * batch).astype(np.float32)
    K = rng.standard_normal(k * k).astype(np.float32)
    plan = build_plan_t(shape, K)
    cp, ri, va = oracle.csc(m, n, k, s, p, K)
    col = 40 * n + 9
    e = int(cp[col]) + 5
    far = plan.cols - 1                       # the last output: not among this column's rows
    assert far not in ri[cp[col]:cp[col + 1]]
    ri2, va2 = ri.copy(), va.copy()
    ri2[e] = far
    va2[e + 1] = 3.5
    plan.col_idx[e] = far
    plan.vals[e + 1] = 3.5
    y = cs.conv_spmv_from_csc(plan, torch.from_numpy(x).to(device()), batch=batch)
    torch.cuda.synchronize()
    T = sp.csc_matrix((va2.astype(np.float64), ri2, cp), shape=(plan.cols, plan.rows))
    X = x.reshape(-1, batch).astype(np.float64)
    want = T @ X
    scale = abs(T) @ np.abs(X)
    got = y.cpu().numpy().reshape(-1, batch)
    assert np.all(np.abs(got - want) <= 1e-5 * scale + 1e-30)
    # the edit is visible: the far row and the row the entry left both differ from the unedited product
    ref = oracle.conv(m, n, k, s, p, x, K, batch=batch).reshape(-1, batch)
    changed = np.where(np.any(np.abs(got - ref) > 1e-5 * scale + 1e-30, axis=1))[0].tolist()
    assert far in changed and int(ri[e]) in changed and int(ri[e + 1]) in changed
    plan.close()


@pytest.mark.parametrize("shape", [(96, 80, 3, 1, 1), (96, 80, 5, 2, 2), (60, 70, 4, 1, 2), (96, 80, 7, 2, 3), (96, 80, 2, 1, 1)])
def test_product_from_csc_with_short_columns_reads_the_stored_arrays(shape):
    """Short columns (k = 3, 4, 5: several columns share a step of the scatter).  One entry is
    sent to the row two outputs further right, which the workgroup still keeps on chip but
    which no window over that pixel has; another to the far end of y.  The result must be the
    product with the edited matrix."""
    import scipy.sparse as sp
    batch = 16
    m, n, k, s, p = shape
    rng = np.random.default_rng(37)
    x = rng.standard_normal(m * n * batch).astype(np.float32)
    K = rng.standard_normal(k * k).astype(np.float32)
    plan = build_plan_t(shape, K)
    cp, ri, va = oracle.csc(m, n, k, s, p, K)
    ri2 = ri.copy()
    edits = []
    for col, far in ((40 * n + 9, False), (41 * n + 30, True), (12 * n + 33, False)):
        e = int(cp[col + 1]) - 1                       # the column's last entry: its largest row
        new_row = plan.cols - 1 if far else int(ri[e]) + 2
        assert new_row not in ri[cp[col]:cp[col + 1]]
        ri2[e] = new_row
        plan.col_idx[e] = new_row
        edits += [int(ri[e]), new_row]
    y = cs.conv_spmv_from_csc(plan, torch.from_numpy(x).to(device()), batch=batch)
    torch.cuda.synchronize()
    T = sp.csc_matrix((va.astype(np.float64), ri2, cp), shape=(plan.cols, plan.rows))
    X = x.reshape(-1, batch).astype(np.float64)
    want, scale = T @ X, abs(T) @ np.abs(X)
    got = y.cpu().numpy().reshape(-1, batch)
    assert np.all(np.abs(got - want) <= 1e-5 * scale + 1e-30)
    ref = oracle.conv(m, n, k, s, p, x, K, batch=batch).reshape(-1, batch)
    changed = set(np.where(np.any(np.abs(got - ref) > 1e-5 * scale + 1e-30, axis=1))[0].tolist())
    assert changed == set(edits)
    plan.close()


def test_product_from_csc_needs_a_csc_plan():
    shape = (8, 8, 3, 1, 1)
    K = np.ones(9, dtype=np.float32)
    plan = build_plan(shape, K)
    x = torch.zeros(64, device=device())
    with pytest.raises(cs.ConvError) as e:
        cs.conv_spmv_from_csc(plan, x, batch=1)
    assert e.value.status == -1
    plan.close()
    pt = build_plan_t(shape, K)
    with pytest.raises(cs.ConvError) as e:          # x and y overlap
        buf = torch.zeros(128, device=device())
        cs.conv_spmv_from_csc(pt, buf[:64], buf[32:96], batch=1)
    assert e.value.status == -6
    pt.close()


def test_largest_index_range_transposed():
    """The column-compressed build and z = T^T u with nnz just below 2^31 (6600 x 6600, k = 7,
    'same' padding): col_ptr in full against the prefix sums of the window counts, row_idx /
    vals on sampled columns against the windows that cover the pixel (Section 2: tap
    (i+p-s x, j+p-s y) of window (x, y)), z in full against the scatter-and-crop oracle."""
    shape, batch = (6600, 6600, 7, 1, 3), 1
    m, n, k, s, p = shape
    mo, no = oracle.out_shape(*shape)
    nnz = oracle.nnz_closed(*shape)
    rng = np.random.default_rng(32)
    u = rng.standard_normal(mo * no * batch).astype(np.float32)
    K = rng.standard_normal(k * k).astype(np.float32)
    plan = build_plan_t(shape, K)
    assert plan.nnz == nnz

    def cover(t, count_out):      # windows x in [0, count_out) with 0 <= t + p - s x < k
        xs = np.arange(count_out, dtype=np.int64)
        return np.array([np.count_nonzero((ti + p - s * xs >= 0) & (ti + p - s * xs < k)) for ti in t], dtype=np.int64)

    # s = 1 here: q(t) = number of x in [max(0, t+p-k+1), min(count_out-1, t+p)]
    t1, t2 = np.arange(m, dtype=np.int64), np.arange(n, dtype=np.int64)
    q1 = np.minimum(mo - 1, t1 + p) - np.maximum(0, t1 + p - k + 1) + 1
    q2 = np.minimum(no - 1, t2 + p) - np.maximum(0, t2 + p - k + 1) + 1
    assert np.array_equal(q1[:20], cover(t1[:20], mo)) and np.array_equal(q1[-20:], cover(t1[-20:], mo))
    want = np.concatenate([[0], np.cumsum(np.outer(q1, q2).reshape(-1))])
    assert want[-1] == nnz
    got_cp = plan.row_ptr.cpu().numpy()
    assert np.array_equal(got_cp.astype(np.int64), want)
    del want
    K2 = K.reshape(k, k)
    cols = np.unique(np.concatenate([np.arange(150), np.arange(m * n - 150, m * n), rng.integers(0, m * n, size=2000)]))
    for c in cols:
        i, j = divmod(int(c), n)
        rows, vals = [], []
        for x in range(max(0, i + p - k + 1), min(mo - 1, i + p) + 1):
            for y in range(max(0, j + p - k + 1), min(no - 1, j + p) + 1):
                rows.append(x * no + y)
                vals.append(K2[i + p - x, j + p - y])
        lo, hi = int(got_cp[c]), int(got_cp[c + 1])
        assert plan.col_idx[lo:hi].cpu().numpy().astype(np.int64).tolist() == rows, c
        assert np.array_equal(plan.vals[lo:hi].cpu().numpy().view(np.uint32), np.array(vals, dtype=np.float32).view(np.uint32)), c
    z = cs.conv_spmv(plan, torch.from_numpy(u).to(device()), batch=batch)
    torch.cuda.synchronize()
    ref, scale = oracle.conv_t(m, n, k, s, p, u, K, batch=batch, want_scale=True)
    got = z.cpu().numpy()
    assert np.max(np.abs(got.astype(np.float64) - ref) / scale) <= 1e-5
    print("largest transposed: variant %s" % plan.variant(batch))
    plan.close()
