"""Helpers for the GPU parity tests: run the HIP path through the binding and
compare with the CPU oracle on the same host arrays."""
import numpy as np
import torch

import oracle
import paper_2411_19419_amd as cs

REL_TOL = 1e-5      # max |y_gpu - y_ref| / sum_e |vals[e]| |x[col_idx[e]]| per output, and normwise


def device():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch.device("cuda:0")


# Test hook: when set, every plan built through this module gets this threshold for the
# persistent marching kernels (the default, 256 strip segments, keeps them off small shapes).
MARCH_MIN_JOBS = None


def _hooked(plan):
    if MARCH_MIN_JOBS is not None:
        cs.conv_plan_set_march_min_jobs(plan, MARCH_MIN_JOBS)
    return plan


def build_plan(shape, K):
    m, n, k, s, p = shape
    return _hooked(cs.conv_csr_build(m, n, k, s, p,
                                     torch.from_numpy(np.ascontiguousarray(K, dtype=np.float32)).to(device())))


def check_csr(plan, shape, K):
    """nnz, row_ptr, col_idx and vals bit-exact against the oracle's tap enumeration."""
    m, n, k, s, p = shape
    rp, ci, va = oracle.csr(m, n, k, s, p, K)
    assert plan.nnz == len(ci) == oracle.nnz_closed(m, n, k, s, p)
    assert (plan.m_out, plan.n_out) == oracle.out_shape(m, n, k, s, p)
    g_rp = plan.row_ptr.cpu().numpy()
    assert g_rp.dtype == np.int32 and np.array_equal(g_rp.astype(np.int64), rp), "row_ptr differs"
    g_ci = plan.col_idx.cpu().numpy()
    assert g_ci.dtype == np.int32 and np.array_equal(g_ci.astype(np.int64), ci), "col_idx differs"
    g_va = plan.vals.cpu().numpy()
    assert g_va.dtype == np.float32 and np.array_equal(g_va.view(np.uint32), va.view(np.uint32)), "vals differ"
    return rp, ci, va


def check_apply(plan, shape, K, x, batch, x_dev=None):
    """y against the sliding-window oracle; returns (max scaled error, normwise error)."""
    m, n, k, s, p = shape
    xd = torch.from_numpy(x).to(device()) if x_dev is None else x_dev
    y = torch.full((plan.rows * batch,), float("nan"), dtype=torch.float32, device=device())
    cs.conv_spmv(plan, xd, y, batch=batch)
    torch.cuda.synchronize()
    got = y.cpu().numpy()
    ref, scale = oracle.conv(m, n, k, s, p, x, K, batch=batch, want_scale=True)
    assert not np.any(np.isnan(got)), "some outputs were never written"
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    empty = scale == 0.0
    if np.any(empty):      # rows without entries (or all-zero operands): exactly +0.0
        assert np.all(got[empty] == 0.0) and not np.any(np.signbit(got[empty]))
    scaled = float(np.max(err[~empty] / scale[~empty])) if np.any(~empty) else 0.0
    denom = float(np.max(np.abs(ref))) if ref.size else 0.0
    normwise = float(np.max(err)) / denom if denom > 0 else 0.0
    assert scaled <= REL_TOL, "max err/scale %.3e" % scaled
    assert normwise <= REL_TOL, "normwise error %.3e" % normwise
    return scaled, normwise


def build_plan_t(shape, K):
    m, n, k, s, p = shape
    return _hooked(cs.conv_csc_build(m, n, k, s, p,
                                     torch.from_numpy(np.ascontiguousarray(K, dtype=np.float32)).to(device())))


def check_csc(plan, shape, K):
    """col_ptr, row_idx and vals of T column-compressed, bit-exact against the oracle."""
    m, n, k, s, p = shape
    cp, ri, va = oracle.csc(m, n, k, s, p, K)
    assert plan.transposed and plan.nnz == len(ri) == oracle.nnz_closed(m, n, k, s, p)
    assert np.array_equal(plan.row_ptr.cpu().numpy().astype(np.int64), cp), "col_ptr differs"
    assert np.array_equal(plan.col_idx.cpu().numpy().astype(np.int64), ri), "row_idx differs"
    assert np.array_equal(plan.vals.cpu().numpy().view(np.uint32), va.view(np.uint32)), "vals differ"


def check_apply_t(plan, shape, K, u, batch):
    """z = T^T u against the scatter-and-crop oracle."""
    m, n, k, s, p = shape
    z = torch.full((plan.rows * batch,), float("nan"), dtype=torch.float32, device=device())
    cs.conv_spmv(plan, torch.from_numpy(u).to(device()), z, batch=batch)
    torch.cuda.synchronize()
    got = z.cpu().numpy()
    ref, scale = oracle.conv_t(m, n, k, s, p, u, K, batch=batch, want_scale=True)
    assert not np.any(np.isnan(got)), "some outputs were never written"
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    empty = scale == 0.0
    if np.any(empty):
        assert np.all(got[empty] == 0.0) and not np.any(np.signbit(got[empty]))
    scaled = float(np.max(err[~empty] / scale[~empty])) if np.any(~empty) else 0.0
    denom = float(np.max(np.abs(ref))) if ref.size else 0.0
    normwise = float(np.max(err)) / denom if denom > 0 else 0.0
    assert scaled <= REL_TOL, "max err/scale %.3e" % scaled
    assert normwise <= REL_TOL, "normwise error %.3e" % normwise
    return scaled, normwise


def build_plan_c(shape, K):
    m, n, k, s, p = shape
    return _hooked(cs.conv_compact_build(m, n, k, s, p,
                                         torch.from_numpy(np.ascontiguousarray(K, dtype=np.float32)).to(device())))


def check_compact(plan, shape, K):
    """Row descriptors and value table of the structure-aware storage, bit-exact against the oracle."""
    m, n, k, s, p = shape
    want = oracle.compact_rows(m, n, k, s, p)
    assert plan.compact and plan.nnz == oracle.nnz_closed(m, n, k, s, p)
    got = plan.row_desc.cpu().numpy()
    assert got.dtype == np.int32 and got.shape == want.shape and np.array_equal(got, want), "descriptors differ"
    tab = plan.ktab.cpu().numpy()
    assert np.array_equal(tab.view(np.uint32), np.ascontiguousarray(K, dtype=np.float32).reshape(-1).view(np.uint32))
