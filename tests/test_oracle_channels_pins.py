"""Pins for the oracle's multi-channel sum (CPU only): hand-worked fixtures, torch's conv2d
with several input channels, the single-channel oracle, exact additivity over channels on
integer data, and the matrix form [T_1 | ... | T_C] with scipy."""
import json
import os

import numpy as np
import pytest
import scipy.sparse
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked_channels.json")
with open(GOLDEN) as fh:
    _CASES = json.load(fh)["cases"]

SHAPES = [(5, 7, 3, 1, 1), (9, 6, 3, 2, 1), (8, 8, 2, 2, 0), (6, 11, 5, 1, 2), (7, 7, 7, 1, 3), (4, 5, 3, 1, 4),
          (12, 10, 4, 3, 2), (3, 3, 1, 1, 0), (10, 9, 6, 2, 5)]


@pytest.mark.parametrize("case", _CASES, ids=[c["name"] for c in _CASES])
def test_hand_worked_channel_sums(case):
    m, n, k, s, p = case["shape"]
    out = oracle.conv_channels(m, n, k, s, p, np.array(case["A"], dtype=np.float32),
                               np.array(case["K"], dtype=np.float32), case["channels"])
    assert out.tolist() == [float(v) for v in case["out"]]


def test_one_channel_is_the_single_channel_oracle():
    rng = np.random.default_rng(2)
    for shp in SHAPES:
        m, n, k, s, p = shp
        for batch in (1, 3):
            A = rng.standard_normal(m * n * batch).astype(np.float32)
            K = rng.standard_normal(k * k).astype(np.float32)
            a, sa = oracle.conv(m, n, k, s, p, A, K, batch=batch, want_scale=True)
            b, sb = oracle.conv_channels(m, n, k, s, p, A, K, 1, batch=batch, want_scale=True)
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)) and np.array_equal(sa, sb), shp


def test_against_torch_conv2d_with_input_channels():
    """Integer data: every product and sum is exact in fp32 and fp64, so equality is bitwise."""
    rng = np.random.default_rng(3)
    for shp in SHAPES:
        m, n, k, s, p = shp
        for C, batch in ((2, 1), (3, 4), (5, 2)):
            A = rng.integers(-4, 5, size=(C, m, n, batch)).astype(np.float32)
            K = rng.integers(-3, 4, size=(C, k, k)).astype(np.float32)
            got = oracle.conv_channels(m, n, k, s, p, A, K, C, batch=batch)
            inp = torch.from_numpy(A).permute(3, 0, 1, 2).double()           # (batch, C, m, n)
            ref = torch.nn.functional.conv2d(inp, torch.from_numpy(K).double()[None], stride=s, padding=p)
            ref = ref[:, 0].permute(1, 2, 0).reshape(-1).numpy()             # batch-minor
            assert np.array_equal(got.astype(np.float64), ref), (shp, C, batch)


def test_additive_over_channels_and_matrix_form():
    """Sum of the single-channel results (exact on integers), and [T_1 | ... | T_C] x with the
    CSR oracle's arrays: shared indices, values of kernel ch."""
    rng = np.random.default_rng(4)
    for shp in SHAPES:
        m, n, k, s, p = shp
        mo, no = oracle.out_shape(*shp)
        C, batch = 3, 2
        A = rng.integers(-4, 5, size=(C, m * n * batch)).astype(np.float32)
        K = rng.integers(-3, 4, size=(C, k * k)).astype(np.float32)
        got = oracle.conv_channels(m, n, k, s, p, A, K, C, batch=batch).astype(np.float64)
        parts = sum(oracle.conv(m, n, k, s, p, A[c], K[c], batch=batch).astype(np.float64) for c in range(C))
        assert np.array_equal(got, parts), shp
        blocks = []
        for c in range(C):
            rp, ci, va = oracle.csr(m, n, k, s, p, K[c])
            blocks.append(scipy.sparse.csr_matrix((va.astype(np.float64), ci, rp), shape=(mo * no, m * n)))
        T = scipy.sparse.hstack(blocks).tocsr()
        X = A.astype(np.float64).reshape(C * m * n, batch)
        assert np.array_equal(got, (T @ X).reshape(-1)), shp


def test_scale_is_the_sum_of_magnitudes():
    rng = np.random.default_rng(5)
    m, n, k, s, p = 6, 7, 3, 1, 1
    A = rng.standard_normal(2 * m * n).astype(np.float32)
    K = rng.standard_normal(2 * 9).astype(np.float32)
    _, sc = oracle.conv_channels(m, n, k, s, p, A, K, 2, want_scale=True)
    ref = oracle.conv_channels(m, n, k, s, p, np.abs(A), np.abs(K), 2)
    assert np.allclose(sc, ref, rtol=1e-6)
