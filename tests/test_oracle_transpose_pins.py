"""Pins for the oracle's transposed side (CPU only): the CSC arrays of T (= CSR
of T^T) and the adjoint z = T^T u, against hand-worked fixtures, the paper's
dense C and P, scipy's CSR->CSC conversion, torch's conv_transpose2d, the
adjoint identity and a direct count of the windows that cover a pixel."""
import itertools
import json
import os

import numpy as np
import pytest
import scipy.sparse

import oracle
from oracle import paper_matrices as pm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked_transpose.json")
with open(GOLDEN) as fh:
    _CASES = json.load(fh)["cases"]


def _tiny_shapes(mmax, kmax, smax, pmax):
    for m, n, k, s, p in itertools.product(range(1, mmax + 1), range(1, mmax + 1), range(1, kmax + 1),
                                           range(1, smax + 1), range(0, pmax + 1)):
        if k <= m + 2 * p and k <= n + 2 * p:
            yield m, n, k, s, p


@pytest.mark.parametrize("case", _CASES, ids=[c["name"] for c in _CASES])
def test_hand_worked_adjoint(case):
    m, n, k, s, p = case["shape"]
    K = np.array(case["K"], dtype=np.float32)
    u = np.array(case["u"], dtype=np.float32)
    z = oracle.conv_t(m, n, k, s, p, u, K)
    assert z.tolist() == [float(v) for v in case["z"]]
    col_ptr, row_idx, vals = oracle.csc(m, n, k, s, p, K)
    assert col_ptr[-1] == len(row_idx) == oracle.nnz_closed(m, n, k, s, p)
    if "col_ptr" in case:
        assert col_ptr.tolist() == case["col_ptr"]
    for c, want in case.get("rows", {}).items():
        c = int(c)
        assert row_idx[col_ptr[c]:col_ptr[c + 1]].tolist() == want
    for c, want in case.get("vals", {}).items():
        c = int(c)
        assert vals[col_ptr[c]:col_ptr[c + 1]].tolist() == [float(v) for v in want]


def test_csc_equals_scipy_conversion_and_paper_matrices():
    rng = np.random.default_rng(1)
    checked = 0
    for shp in _tiny_shapes(5, 4, 3, 4):
        m, n, k, s, p = shp
        mo, no = oracle.out_shape(*shp)
        K = rng.integers(1, 9, size=(k, k)).astype(np.float32)
        rp, ci, va = oracle.csr(m, n, k, s, p, K)
        col_ptr, row_idx, vals = oracle.csc(m, n, k, s, p, K)
        ref = scipy.sparse.csr_matrix((va, ci, rp), shape=(mo * no, m * n)).tocsc()
        ref.sort_indices()
        assert np.array_equal(ref.indptr, col_ptr) and np.array_equal(ref.indices, row_idx), shp
        assert np.array_equal(ref.data, vals), shp
        for c in range(m * n):                                   # rows ascending, no duplicates
            assert np.all(np.diff(row_idx[col_ptr[c]:col_ptr[c + 1]]) > 0)
        if checked % 7 == 0:                                     # and the paper's dense product, transposed
            T = pm.transformation_matrix(K, m, n, p, s)
            dense = np.zeros((m * n, mo * no))
            for c in range(m * n):
                dense[c, row_idx[col_ptr[c]:col_ptr[c + 1]]] = vals[col_ptr[c]:col_ptr[c + 1]]
            assert np.array_equal(dense, T.T), shp
        checked += 1
    assert checked > 1000


def test_column_lengths_are_window_counts():
    """Column (i, j) of T has one entry per window that covers the pixel: the number of x with
    0 <= i + p - s x < k times the number of such y (counted here one by one)."""
    for shp in [(9, 8, 4, 2, 2), (7, 7, 3, 1, 1), (5, 6, 2, 1, 3), (10, 6, 5, 3, 0), (6, 6, 7, 2, 3), (5, 5, 2, 2, 0)]:
        m, n, k, s, p = shp
        mo, no = oracle.out_shape(*shp)
        q1 = [sum(1 for x in range(mo) if 0 <= i + p - s * x < k) for i in range(m)]
        q2 = [sum(1 for y in range(no) if 0 <= j + p - s * y < k) for j in range(n)]
        col_ptr, _, _ = oracle.csc(m, n, k, s, p, np.ones(k * k, dtype=np.float32))
        want = np.array([[a * b for b in q2] for a in q1]).reshape(-1)
        assert np.diff(col_ptr).tolist() == want.tolist(), shp


def test_adjoint_matches_dense_transpose_and_adjoint_identity():
    rng = np.random.default_rng(5)
    checked = 0
    for shp in _tiny_shapes(5, 4, 3, 4):
        m, n, k, s, p = shp
        mo, no = oracle.out_shape(*shp)
        K = rng.integers(-4, 5, size=(k, k)).astype(np.float32)
        x = rng.integers(-6, 7, size=m * n).astype(np.float32)
        u = rng.integers(-6, 7, size=mo * no).astype(np.float32)
        z = oracle.conv_t(m, n, k, s, p, u, K)
        if checked % 5 == 0:
            T = pm.transformation_matrix(K, m, n, p, s)
            assert np.array_equal(z.astype(np.float64), T.T @ u.astype(np.float64)), shp      # integers: exact
        y = oracle.conv(m, n, k, s, p, x, K)
        assert float(np.dot(y.astype(np.float64), u)) == float(np.dot(x.astype(np.float64), z)), shp
        checked += 1
    assert checked > 1000


def test_adjoint_matches_torch_conv_transpose2d():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(8)
    for m, n, k, s, p in [(12, 15, 3, 1, 1), (28, 28, 2, 2, 0), (33, 20, 5, 2, 2), (10, 10, 3, 2, 4), (9, 9, 4, 3, 1)]:
        mo, no = oracle.out_shape(m, n, k, s, p)
        K = rng.integers(-3, 4, size=(k, k)).astype(np.float32)
        u = rng.integers(-5, 6, size=(mo, no)).astype(np.float32)
        # torch crops p lines on both sides of the (m_out-1) s + k lines the windows span; the slide
        # remainder (fewer than s lines) is asked back with output_padding, which torch computes properly
        op = (m - ((mo - 1) * s - 2 * p + k), n - ((no - 1) * s - 2 * p + k))
        want = torch.nn.functional.conv_transpose2d(torch.from_numpy(u)[None, None].double(),
                                                    torch.from_numpy(K)[None, None].double(),
                                                    stride=s, padding=p, output_padding=op)[0, 0].numpy()
        assert want.shape == (m, n)
        z = oracle.conv_t(m, n, k, s, p, u.reshape(-1), K)
        assert np.array_equal(z.astype(np.float64).reshape(m, n), want), (m, n, k, s, p)


def test_adjoint_batch_layout_scale_and_spmv_over_csc():
    rng = np.random.default_rng(12)
    m, n, k, s, p, B = 9, 7, 3, 2, 1, 4
    mo, no = oracle.out_shape(m, n, k, s, p)
    U = rng.standard_normal((mo * no, B)).astype(np.float32)
    K = rng.standard_normal(k * k).astype(np.float32)
    Z, S = oracle.conv_t(m, n, k, s, p, U.reshape(-1), K, batch=B, want_scale=True)
    Z, S = Z.reshape(m * n, B), S.reshape(m * n, B)
    col_ptr, row_idx, vals = oracle.csc(m, n, k, s, p, K)
    for c in range(B):
        zc, sc = oracle.conv_t(m, n, k, s, p, np.ascontiguousarray(U[:, c]), K, want_scale=True)
        assert np.array_equal(Z[:, c], zc) and np.array_equal(S[:, c], sc)
        for j in range(m * n):                       # the same sums over the stored column
            seg = slice(col_ptr[j], col_ptr[j + 1])
            want = np.dot(vals[seg].astype(np.float64), U[row_idx[seg], c].astype(np.float64))
            mag = np.dot(np.abs(vals[seg]).astype(np.float64), np.abs(U[row_idx[seg], c]).astype(np.float64))
            assert abs(float(Z[j, c]) - want) <= 1e-6 * max(mag, 1e-30)
            assert abs(S[j, c] - mag) <= 1e-12 * max(mag, 1e-30)
