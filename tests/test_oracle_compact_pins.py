"""Pins for the oracle's structure-aware storage of T (CPU only): the per-row
descriptors against hand-worked fixtures, against the paper's dense T = C P
(every row's non-zeros are exactly the described block of taps), against the
CSR oracle through the decoder, and against Theorem 2.1's row lengths."""
import itertools
import json
import os

import numpy as np
import pytest

import oracle
from oracle import paper_matrices as pm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked_compact.json")
with open(GOLDEN) as fh:
    _CASES = json.load(fh)["cases"]


def _tiny_shapes(mmax, kmax, smax, pmax):
    for m, n, k, s, p in itertools.product(range(1, mmax + 1), range(1, mmax + 1), range(1, kmax + 1),
                                           range(1, smax + 1), range(0, pmax + 1)):
        if k <= m + 2 * p and k <= n + 2 * p:
            yield m, n, k, s, p


def _fields(desc):
    w = desc[:, 1].view(np.uint32).astype(np.int64)
    return desc[:, 0].astype(np.int64), w & 255, (w >> 8) & 255, (w >> 16) & 255, w >> 24


@pytest.mark.parametrize("case", _CASES, ids=[c["name"] for c in _CASES])
def test_hand_worked_descriptors(case):
    m, n, k, s, p = case["shape"]
    mo, no = oracle.out_shape(m, n, k, s, p)
    desc = oracle.compact_rows(m, n, k, s, p)
    assert desc.shape == (mo * no, 2)
    base, a_lo, r1, b_lo, r2 = _fields(desc)
    for row in case["rows"]:
        r = row["x"] * no + row["y"]
        assert int(base[r]) == row["base"], row
        assert int(desc[r, 1].view(np.uint32)) == row["word"], row
        if "a_lo" in row:
            assert (int(a_lo[r]), int(r1[r]), int(b_lo[r]), int(r2[r])) == \
                (row["a_lo"], row["r1"], row["b_lo"], row["r2"]), row


def test_descriptors_describe_the_rows_of_the_papers_dense_T():
    """Row r of T = C P (built densely as the paper does) has non-zeros exactly at
    base + da n + db, da < r1, db < r2, holding K[a_lo + da][b_lo + db]."""
    checked = 0
    for shp in _tiny_shapes(5, 4, 3, 3):
        m, n, k, s, p = shp
        K = np.arange(1, k * k + 1, dtype=np.float64).reshape(k, k)      # distinct, non-zero
        T = pm.transformation_matrix(K, m, n, p, s)
        desc = oracle.compact_rows(*shp)
        base, a_lo, r1, b_lo, r2 = _fields(desc)
        assert T.shape[0] == desc.shape[0]
        for r in range(T.shape[0]):
            want = np.zeros(m * n)
            for da in range(r1[r]):
                for db in range(r2[r]):
                    want[base[r] + da * n + db] = K[a_lo[r] + da, b_lo[r] + db]
            assert np.array_equal(T[r], want), (shp, r)
            if r1[r] * r2[r] == 0:
                assert desc[r, 0] == 0 and desc[r, 1] == 0, (shp, r)
        checked += 1
    assert checked > 1000


def test_decoder_reproduces_the_csr_oracle():
    rng = np.random.default_rng(5)
    shapes = list(_tiny_shapes(6, 5, 3, 5))[::7] + [(40, 33, 7, 1, 3), (31, 50, 11, 4, 5), (64, 64, 3, 2, 1),
                                                     (17, 23, 5, 3, 7), (12, 12, 12, 1, 0), (9, 14, 2, 2, 0)]
    for shp in shapes:
        m, n, k, s, p = shp
        K = rng.standard_normal(k * k).astype(np.float32)
        rp, ci, va = oracle.csr(m, n, k, s, p, K)
        rp2, ci2, va2 = oracle.compact_decode(n, k, oracle.compact_rows(*shp), K)
        assert np.array_equal(rp, rp2) and np.array_equal(ci, ci2), shp
        assert np.array_equal(va.view(np.uint32), va2.view(np.uint32)), shp


def test_decoder_by_hand():
    """Decoder against a descriptor typed in by hand (not produced by the oracle):
    base 7, a_lo 1, r1 2, b_lo 0, r2 3 on a plane of n = 10 with a 3x3 table 1..9 gives
    columns 7,8,9,17,18,19 and values K[1][0..2], K[2][0..2] = 4,5,6,7,8,9; then an empty row."""
    word = 1 + 256 * 2 + 65536 * 0 + 16777216 * 3
    desc = np.array([[7, word], [0, 0]], dtype=np.int64).astype(np.int32)
    rp, ci, va = oracle.compact_decode(10, 3, desc, np.arange(1, 10, dtype=np.float32))
    assert rp.tolist() == [0, 6, 6]
    assert ci.tolist() == [7, 8, 9, 17, 18, 19]
    assert va.tolist() == [4.0, 5.0, 6.0, 7.0, 8.0, 9.0]
    with pytest.raises(ValueError):                      # a_lo + r1 > k
        oracle.compact_decode(10, 3, np.array([[0, 2 + 256 * 2 + 16777216]], dtype=np.int32), np.ones(9))


def test_row_lengths_follow_theorem_2_1():
    """r1(x) = max(0, k - c1(x)) with c1 the printed padding overlap; sum of r1 r2 = nnz."""
    for shp in [(1024, 1024, 7, 1, 3), (224, 224, 7, 2, 3), (4096, 4096, 11, 4, 5), (5, 9, 3, 1, 4),
                (56, 56, 1, 1, 0), (3, 3, 9, 2, 3), (200, 100, 255, 3, 130)]:
        m, n, k, s, p = shp
        mo, no = oracle.out_shape(*shp)
        base, a_lo, r1, b_lo, r2 = _fields(oracle.compact_rows(*shp))
        x = np.arange(mo)[:, None] + np.zeros((1, no), dtype=np.int64)
        y = np.zeros((mo, 1), dtype=np.int64) + np.arange(no)[None, :]
        c1 = np.maximum(0, p - s * x) + np.maximum(0, s * x + k - m - p)
        c2 = np.maximum(0, p - s * y) + np.maximum(0, s * y + k - n - p)
        want1, want2 = np.maximum(0, k - c1).reshape(-1), np.maximum(0, k - c2).reshape(-1)
        live = want1 * want2 > 0                       # rows without entries are stored as (0, 0)
        assert np.array_equal(r1, np.where(live, want1, 0)), shp
        assert np.array_equal(r2, np.where(live, want2, 0)), shp
        assert int((r1 * r2).sum()) == oracle.nnz_closed(*shp), shp
        assert np.array_equal(a_lo[live], np.maximum(0, p - s * x).reshape(-1)[live]), shp
        assert np.array_equal(b_lo[live], np.maximum(0, p - s * y).reshape(-1)[live]), shp


def test_k_above_255_is_refused():
    with pytest.raises(ValueError):
        oracle.compact_rows(300, 300, 256, 1, 0)
