"""Pins for the CPU oracle: everything here runs without a GPU and compares the
oracle with things other than itself -- hand-worked fixtures, Theorem 2.1 and
its special cases, brute-force counting, the paper's dense C and P multiplied
out, scipy's correlate2d, and exact invariants of the operation."""
import itertools
import json
import os

import numpy as np
import pytest
import scipy.signal

import oracle
from oracle import paper_matrices as pm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked.json")


def _valid(m, n, k, s, p):
    return k <= m + 2 * p and k <= n + 2 * p


def _tiny_shapes(mmax, kmax, smax, pmax):
    for m, n, k, s, p in itertools.product(range(1, mmax + 1), range(1, mmax + 1),
                                           range(1, kmax + 1), range(1, smax + 1),
                                           range(0, pmax + 1)):
        if _valid(m, n, k, s, p):
            yield m, n, k, s, p


def _dense_from_csr(row_ptr, col_idx, vals, rows, cols):
    T = np.zeros((rows, cols))
    for r in range(rows):
        for e in range(row_ptr[r], row_ptr[r + 1]):
            T[r, col_idx[e]] += vals[e]
    return T


# ---------------------------------------------------------------- fixtures

with open(GOLDEN) as fh:
    _CASES = json.load(fh)["cases"]


@pytest.mark.parametrize("case", _CASES, ids=[c["name"] for c in _CASES])
def test_hand_worked_examples(case):
    m, n, k, s, p = case["shape"]
    K = np.array(case["K"], dtype=np.float32)
    A = np.arange(1, m * n + 1, dtype=np.float32)
    assert oracle.nnz_closed(m, n, k, s, p) == case["nnz"]
    assert oracle.nnz_brute(m, n, k, s, p) == case["nnz"]
    row_ptr, col_idx, vals = oracle.csr(m, n, k, s, p, K)
    assert len(col_idx) == case["nnz"] and row_ptr[-1] == case["nnz"]
    if "out" in case:
        out = oracle.conv(m, n, k, s, p, A, K)
        assert out.tolist() == [float(v) for v in case["out"]]
    if "row_ptr" in case:
        assert row_ptr.tolist() == case["row_ptr"]
    for r, want in case.get("cols", {}).items():
        r = int(r)
        assert col_idx[row_ptr[r]:row_ptr[r + 1]].tolist() == want
        assert oracle.csr_row(m, n, k, s, p, K, r)[0].tolist() == want
    for r, want in case.get("vals", {}).items():
        r = int(r)
        assert vals[row_ptr[r]:row_ptr[r + 1]].tolist() == [float(v) for v in want]
    if "row_nnz_nonzero" in case:
        lens = np.diff(row_ptr)
        want = np.zeros_like(lens)
        for r, c in case["row_nnz_nonzero"].items():
            want[int(r)] = c
        assert lens.tolist() == want.tolist()
        out = oracle.conv(m, n, k, s, p, A, K)
        assert np.all(out[lens == 0] == 0.0) and not np.any(np.signbit(out[lens == 0]))


# ------------------------------------------------- Theorem 2.1 vs counting

def test_closed_form_equals_brute_force_on_exhaustive_tiny_grid():
    """Includes k > m (window overhangs both borders), p >= k (empty rows) and
    shapes with slide remainders."""
    count = 0
    for shp in _tiny_shapes(6, 5, 3, 6):
        closed = oracle.nnz_closed(*shp)
        assert closed == oracle.nnz_brute(*shp), shp
        count += 1
    assert count > 3000


def test_csr_length_and_row_lengths_match_theorem_factors():
    for shp in _tiny_shapes(5, 4, 3, 4):
        m, n, k, s, p = shp
        mo, no = oracle.out_shape(*shp)
        K = np.ones(k * k, dtype=np.float32)
        row_ptr, col_idx, _ = oracle.csr(m, n, k, s, p, K)
        assert row_ptr[-1] == len(col_idx) == oracle.nnz_closed(*shp)
        c1 = [max(0, p - s * x) + max(0, s * x + k - m - p) for x in range(mo)]
        c2 = [max(0, p - s * y) + max(0, s * y + k - n - p) for y in range(no)]
        want = np.array([[max(0, k - a) * max(0, k - b) for b in c2] for a in c1]).reshape(-1)
        assert np.diff(row_ptr).tolist() == want.tolist(), shp
        # sorted, duplicate-free, in range
        for r in range(mo * no):
            seg = col_idx[row_ptr[r]:row_ptr[r + 1]]
            assert np.all(np.diff(seg) > 0)
            assert seg.size == 0 or (seg[0] >= 0 and seg[-1] < m * n)


def test_out_shape_formula_and_precondition():
    assert oracle.out_shape(1024, 1024, 7, 1, 3) == (1024, 1024)
    assert oracle.out_shape(256, 256, 5, 2, 2) == (128, 128)
    assert oracle.out_shape(512, 512, 9, 3, 8) == (174, 174)
    assert oracle.out_shape(4096, 4096, 11, 4, 5) == (1024, 1024)
    assert oracle.out_shape(224, 224, 7, 2, 3) == (112, 112)
    assert oracle.out_shape(5, 7, 2, 2, 0) == (2, 3)
    with pytest.raises(ValueError):
        oracle.out_shape(3, 3, 6, 1, 1)      # k > m + 2p
    with pytest.raises(ValueError):
        oracle.out_shape(3, 9, 4, 1, 0)      # k > m + 2p on one axis only
    with pytest.raises(ValueError):
        oracle.nnz_closed(3, 3, 0, 1, 0)


def test_special_closed_forms():
    # "same" convolution, s = 1, p = (k-1)/2, m, n >= k:
    # nnz = (k m - p(p+1)) (k n - p(p+1))
    for m, n, k in [(32, 32, 3), (224, 224, 3), (1024, 1024, 7), (9, 17, 5), (40, 13, 9)]:
        p = (k - 1) // 2
        assert oracle.nnz_closed(m, n, k, 1, p) == (k * m - p * (p + 1)) * (k * n - p * (p + 1))
    assert oracle.nnz_closed(32, 32, 3, 1, 1) == 94 ** 2
    assert oracle.nnz_closed(224, 224, 3, 1, 1) == 670 ** 2
    assert oracle.nnz_closed(1024, 1024, 7, 1, 3) == 7156 ** 2
    # no padding: every tap of every window is in bounds
    for m, n, k, s in [(10, 12, 3, 1), (11, 9, 4, 2), (56, 56, 2, 2), (7, 7, 7, 3)]:
        mo, no = oracle.out_shape(m, n, k, s, 0)
        assert oracle.nnz_closed(m, n, k, s, 0) == mo * no * k * k
    # s divides k and the padding is ample: each pixel is covered (k/s)^2 times
    assert oracle.nnz_closed(512, 512, 9, 3, 8) == 512 * 512 * 9
    assert oracle.nnz_closed(2, 2, 2, 1, 3) == 16
    # first window has (k - p)^2 taps when p < k (first step of the proof)
    for m, n, k, s, p in [(9, 9, 5, 1, 2), (20, 31, 7, 2, 3), (8, 8, 3, 3, 1)]:
        K = np.ones(k * k, dtype=np.float32)
        assert len(oracle.csr_row(m, n, k, s, p, K, 0)[0]) == (k - p) ** 2


def test_densenet_table_total():
    """Sum of Theorem 2.1 over the 123 layer shapes of Table 2 and the dense
    tap count m_out n_out k^2 over the same list."""
    from paper_2411_19419_amd.workloads import densenet121_layer_shapes
    shapes = densenet121_layer_shapes()
    assert len(shapes) == 123
    for shp in set(shapes):
        assert oracle.nnz_closed(*shp) == oracle.nnz_brute(*shp)
    dense = 0
    for m, n, k, s, p in shapes:
        mo, no = oracle.out_shape(m, n, k, s, p)
        dense += mo * no * k * k
    sparse = sum(oracle.nnz_closed(*shp) for shp in shapes)
    assert sparse < dense
    # k = 1 layers: T is K11 * I, so the count is m*n
    assert oracle.nnz_closed(56, 56, 1, 1, 0) == 56 * 56


# ------------------------------------- the paper's own construction, dense

def test_CP_equals_direct_tap_enumeration_and_sliding_window():
    rng = np.random.default_rng(7)
    checked = 0
    for shp in _tiny_shapes(5, 4, 3, 4):
        m, n, k, s, p = shp
        mo, no = oracle.out_shape(*shp)
        K = rng.integers(1, 9, size=(k, k)).astype(np.float32)     # no zero entries
        A = rng.integers(-9, 10, size=m * n).astype(np.float32)
        P = pm.padding_matrix(m, n, p)
        C = pm.convolution_matrix(K, m, n, p, s)
        assert P.shape == ((m + 2 * p) * (n + 2 * p), m * n)
        assert C.shape == (mo * no, (m + 2 * p) * (n + 2 * p))
        T = C @ P
        row_ptr, col_idx, vals = oracle.csr(m, n, k, s, p, K)
        assert np.array_equal(T, _dense_from_csr(row_ptr, col_idx, vals, mo * no, m * n)), shp
        assert np.count_nonzero(T) == oracle.nnz_closed(*shp)
        out = oracle.conv(m, n, k, s, p, A, K)
        assert np.array_equal(T @ A.astype(np.float64), out.astype(np.float64)), shp   # integers: exact
        checked += 1
    assert checked > 1000


def test_padding_matrix_pads():
    m, n, p = 3, 4, 2
    A = np.arange(1, 13, dtype=np.float64)
    padded = (pm.padding_matrix(m, n, p) @ A).reshape(m + 2 * p, n + 2 * p)
    assert np.array_equal(padded, np.pad(A.reshape(m, n), p))


# ----------------------------------------------------- library special case

@pytest.mark.parametrize("shp", [(13, 17, 3, 1, 1), (16, 16, 5, 2, 2), (20, 11, 4, 3, 5),
                                 (9, 9, 9, 3, 8), (31, 29, 7, 1, 3), (6, 40, 2, 2, 0),
                                 (3, 3, 5, 1, 2), (64, 64, 11, 4, 5)])
def test_conv_matches_scipy_correlate2d_on_padded_plane(shp):
    """Stride 1 on the zero-padded plane is scipy's 'valid' cross-correlation;
    stride s keeps every s-th line and column of it."""
    m, n, k, s, p = shp
    rng = np.random.default_rng(11)
    A = rng.standard_normal((m, n)).astype(np.float32)
    K = rng.standard_normal((k, k)).astype(np.float32)
    full = scipy.signal.correlate2d(np.pad(A.astype(np.float64), p), K.astype(np.float64), mode="valid")
    want = full[::s, ::s]
    out, scale = oracle.conv(m, n, k, s, p, A, K, want_scale=True)
    mo, no = oracle.out_shape(*shp)
    assert want.shape == (mo, no)
    err = np.abs(out.astype(np.float64) - want.reshape(-1))
    assert np.all(err <= 1e-6 * np.maximum(scale, 1e-30) + 1e-30)
    # and the scale is the same sum with absolute values
    wscale = scipy.signal.correlate2d(np.pad(np.abs(A).astype(np.float64), p),
                                      np.abs(K).astype(np.float64), mode="valid")[::s, ::s]
    assert np.allclose(scale, wscale.reshape(-1), rtol=1e-12, atol=0)


def test_conv_matches_torch_conv2d_cpu():
    """Cross-check against the comparator the paper itself uses (Section 4)."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    for m, n, k, s, p in [(12, 15, 3, 1, 1), (28, 28, 2, 2, 0), (33, 20, 5, 2, 2), (10, 10, 3, 2, 4)]:
        A = rng.integers(-5, 6, size=(m, n)).astype(np.float32)
        K = rng.integers(-3, 4, size=(k, k)).astype(np.float32)
        want = torch.nn.functional.conv2d(torch.from_numpy(A)[None, None].double(),
                                          torch.from_numpy(K)[None, None].double(),
                                          stride=s, padding=p)[0, 0].numpy()
        out = oracle.conv(m, n, k, s, p, A, K)
        assert np.array_equal(out.astype(np.float64), want.reshape(-1))


# -------------------------------------------------------------- invariants

def test_ones_give_row_nnz_exactly():
    for shp in [(17, 13, 5, 2, 3), (8, 8, 3, 1, 4), (30, 30, 7, 1, 3), (5, 5, 2, 1, 3)]:
        m, n, k, s, p = shp
        K = np.ones(k * k, dtype=np.float32)
        out = oracle.conv(m, n, k, s, p, np.ones(m * n, dtype=np.float32), K)
        row_ptr, _, _ = oracle.csr(m, n, k, s, p, K)
        assert np.array_equal(out, np.diff(row_ptr).astype(np.float32))
        assert out.sum() == oracle.nnz_closed(*shp)


def test_delta_kernel_is_shifted_strided_copy():
    rng = np.random.default_rng(3)
    m, n, k, s, p = 11, 14, 4, 2, 3
    A = rng.standard_normal((m, n)).astype(np.float32)
    mo, no = oracle.out_shape(m, n, k, s, p)
    for a0, b0 in [(0, 0), (1, 3), (3, 0), (2, 2)]:
        K = np.zeros((k, k), dtype=np.float32)
        K[a0, b0] = 1.0
        out = oracle.conv(m, n, k, s, p, A, K).reshape(mo, no)
        for x in range(mo):
            for y in range(no):
                i, j = s * x + a0 - p, s * y + b0 - p
                want = A[i, j] if (0 <= i < m and 0 <= j < n) else 0.0
                assert out[x, y] == want


def test_stride_subsamples_stride_one():
    rng = np.random.default_rng(9)
    m, n, k, p = 19, 23, 5, 3
    A = rng.standard_normal(m * n).astype(np.float32)
    K = rng.standard_normal(k * k).astype(np.float32)
    mo1, no1 = oracle.out_shape(m, n, k, 1, p)
    full = oracle.conv(m, n, k, 1, p, A, K).reshape(mo1, no1)
    rp1, ci1, va1 = oracle.csr(m, n, k, 1, p, K)
    for s in (2, 3, 4):
        mo, no = oracle.out_shape(m, n, k, s, p)
        assert np.array_equal(oracle.conv(m, n, k, s, p, A, K).reshape(mo, no), full[::s, ::s][:mo, :no])
        rp, ci, va = oracle.csr(m, n, k, s, p, K)
        for x in range(mo):
            for y in range(no):
                r, r1 = x * no + y, (s * x) * no1 + s * y
                assert np.array_equal(ci[rp[r]:rp[r + 1]], ci1[rp1[r1]:rp1[r1 + 1]])
                assert np.array_equal(va[rp[r]:rp[r + 1]], va1[rp1[r1]:rp1[r1 + 1]])


def test_k1_is_scaled_identity_and_column_coverage():
    K = np.array([2.5], dtype=np.float32)
    rp, ci, va = oracle.csr(6, 5, 1, 1, 0, K)
    assert rp.tolist() == list(range(31)) and ci.tolist() == list(range(30))
    assert np.all(va == np.float32(2.5))
    # column sums of the pattern = number of windows that cover the pixel
    m, n, k, s, p = 9, 8, 4, 2, 2
    mo, no = oracle.out_shape(m, n, k, s, p)
    rp, ci, _ = oracle.csr(m, n, k, s, p, np.ones(k * k, dtype=np.float32))
    cover = np.zeros((m, n), dtype=np.int64)
    for x in range(mo):
        for y in range(no):
            i0, j0 = s * x - p, s * y - p
            cover[max(0, i0):min(m, i0 + k), max(0, j0):min(n, j0 + k)] += 1
    assert np.array_equal(np.bincount(ci, minlength=m * n), cover.reshape(-1))


def test_conv_equals_spmv_over_oracle_csr_and_is_linear_on_integers():
    rng = np.random.default_rng(21)
    m, n, k, s, p = 14, 10, 3, 2, 2
    K = rng.integers(-4, 5, size=k * k).astype(np.float32)
    A1 = rng.integers(-8, 9, size=m * n).astype(np.float32)
    A2 = rng.integers(-8, 9, size=m * n).astype(np.float32)
    rp, ci, va = oracle.csr(m, n, k, s, p, K)
    y1 = oracle.conv(m, n, k, s, p, A1, K)
    spmv = np.array([np.dot(va[rp[r]:rp[r + 1]].astype(np.float64), A1[ci[rp[r]:rp[r + 1]]].astype(np.float64))
                     for r in range(len(rp) - 1)])
    assert np.array_equal(y1.astype(np.float64), spmv)
    y2 = oracle.conv(m, n, k, s, p, A2, K)
    y12 = oracle.conv(m, n, k, s, p, 3 * A1 - 2 * A2, K)
    assert np.array_equal(y12, 3 * y1 - 2 * y2)


def test_batch_minor_layout_is_column_by_column():
    rng = np.random.default_rng(2)
    m, n, k, s, p, B = 9, 7, 3, 2, 1, 5
    X = rng.standard_normal((m * n, B)).astype(np.float32)
    K = rng.standard_normal(k * k).astype(np.float32)
    mo, no = oracle.out_shape(m, n, k, s, p)
    Y, S = oracle.conv(m, n, k, s, p, X.reshape(-1), K, batch=B, want_scale=True)
    Y, S = Y.reshape(mo * no, B), S.reshape(mo * no, B)
    for c in range(B):
        yc, sc = oracle.conv(m, n, k, s, p, np.ascontiguousarray(X[:, c]), K, want_scale=True)
        assert np.array_equal(Y[:, c], yc) and np.array_equal(S[:, c], sc)


def test_results_do_not_depend_on_thread_count(monkeypatch):
    """Each output is summed by one thread in a fixed order."""
    rng = np.random.default_rng(4)
    m, n, k, s, p = 40, 33, 5, 1, 2
    A = rng.standard_normal(m * n).astype(np.float32)
    K = rng.standard_normal(k * k).astype(np.float32)
    full = oracle.conv(m, n, k, s, p, A, K)
    # same sum, written in numpy with an explicit (a, b) raster loop in float64
    Ap = np.pad(A.reshape(m, n).astype(np.float64), p)
    acc = np.zeros(oracle.out_shape(m, n, k, s, p))
    for a in range(k):
        for b in range(k):
            acc += float(K[a * k + b]) * Ap[a:a + acc.shape[0] * s:s, b:b + acc.shape[1] * s:s]
    assert np.array_equal(full, acc.astype(np.float32).reshape(-1))
