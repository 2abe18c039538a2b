"""GPU test of conv_csr_fill_noalloc, the entry point for callers that cannot allocate: its three
CSR arrays against those of conv_csr_build (bit for bit), on two calls in a row, the second with
a smaller shape, through the C ABI."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2411_19419_amd as cs

pytestmark = pytest.mark.gpu


def _arrays_from_build(shape, K):
    m, n, k, s, p = shape
    plan = cs.conv_csr_build(m, n, k, s, p, K)
    torch.cuda.synchronize()
    out = (plan.row_ptr.clone(), plan.col_idx.clone(), plan.vals.clone())
    plan.close()
    return out


def _arrays_from_noalloc(shape, K):
    """Straight through ctypes: caller-allocated outputs, pre-filled so that unwritten elements show."""
    m, n, k, s, p = shape
    lib = cs.binding._load()
    mo, no = cs.conv_out_shape(m, n, k, s, p)
    nnz = cs.conv_nnz(m, n, k, s, p)
    dev = K.device
    row_ptr = torch.full((mo * no + 1,), -7, dtype=torch.int32, device=dev)
    col_idx = torch.full((max(nnz, 1),), -7, dtype=torch.int32, device=dev)
    vals = torch.full((max(nnz, 1),), float("nan"), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    st = lib.conv_csr_fill_noalloc(m, n, k, s, p, K.data_ptr(), row_ptr.data_ptr(), col_idx.data_ptr(), vals.data_ptr(),
                                   ctypes.c_void_p(stream.cuda_stream))
    assert st == 0, cs.conv_strerror(st)
    torch.cuda.synchronize()
    return row_ptr, col_idx[:nnz], vals[:nnz]


def test_noalloc_fill_matches_the_build_on_two_calls_in_a_row():
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(77)
    # the second shape is smaller in every table the scratch array holds; the third has empty rows
    # and rows long enough for the quad-walking fill; then the first again
    shapes = [(300, 517, 7, 1, 3), (41, 37, 5, 2, 2), (6, 6, 2, 1, 5), (70, 70, 60, 1, 30), (300, 517, 7, 1, 3)]
    for shape in shapes:
        k = shape[2]
        K = torch.from_numpy(rng.standard_normal(k * k).astype(np.float32)).to(dev)
        got = _arrays_from_noalloc(shape, K)
        want = _arrays_from_build(shape, K)
        for g, w, name in zip(got, want, ("row_ptr", "col_idx", "vals")):
            assert g.dtype == w.dtype and g.shape == w.shape, (shape, name)
            assert torch.equal(g.view(torch.int32), w.view(torch.int32)), (shape, name)


def test_noalloc_fill_rejects_what_it_cannot_hold():
    dev = torch.device("cuda:0")
    K = torch.zeros(1, dtype=torch.float32, device=dev)
    buf = torch.zeros(16, dtype=torch.int32, device=dev)
    lib = cs.binding._load()
    # m_out + n_out + 2 > 65536: refused before anything is enqueued
    st = lib.conv_csr_fill_noalloc(40000, 30000, 1, 1, 0, K.data_ptr(), buf.data_ptr(), buf.data_ptr(), buf.data_ptr(), None)
    assert st == -3
    torch.cuda.synchronize()
    assert int(buf.abs().sum()) == 0
