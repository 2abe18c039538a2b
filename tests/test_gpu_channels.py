"""GPU parity for the multi-channel sum (conv_csr_build_channels): shared indices and the
per-channel values bit-exact against the CSR oracle, y = sum_ch T_ch x_ch against the
oracle's sum of padded convolutions."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2411_19419_amd as cs
from paper_2411_19419_amd import binding

from gpu_util import REL_TOL, build_plan, device

pytestmark = pytest.mark.gpu


def _case(shape, channels, batch, seed):
    m, n, k, s, p = shape
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(channels * m * n * batch).astype(np.float32),
            rng.standard_normal(channels * k * k).astype(np.float32))


def _check(shape, channels, batch, seed=1, x_off=0):
    m, n, k, s, p = shape
    x, K = _case(shape, channels, batch, seed)
    plan = cs.conv_csr_build_channels(m, n, k, s, p, torch.from_numpy(K).to(device()), channels)
    assert binding._load().conv_plan_channels(plan._handle) == channels
    rp, ci, _ = oracle.csr(m, n, k, s, p, K[:k * k])
    assert np.array_equal(plan.row_ptr.cpu().numpy().astype(np.int64), rp)
    assert np.array_equal(plan.col_idx.cpu().numpy().astype(np.int64), ci)
    vals = plan.vals.cpu().numpy().reshape(channels, -1)
    for ch in range(channels):
        want = oracle.csr(m, n, k, s, p, K[ch * k * k:(ch + 1) * k * k])[2]
        assert np.array_equal(vals[ch].view(np.uint32), want.view(np.uint32)), "vals of channel %d differ" % ch
    buf = torch.zeros(x.size + x_off, dtype=torch.float32, device=device())
    buf[x_off:] = torch.from_numpy(x).to(device())
    y = torch.full((plan.rows * batch,), float("nan"), dtype=torch.float32, device=device())
    cs.conv_spmv(plan, buf[x_off:], y, batch=batch)
    torch.cuda.synchronize()
    got = y.cpu().numpy()
    ref, scale = oracle.conv_channels(m, n, k, s, p, x, K, channels, batch=batch, want_scale=True)
    assert not np.any(np.isnan(got))
    live = scale > 0
    assert np.all(got[~live] == 0.0)
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    assert (np.max(err[live] / scale[live]) if np.any(live) else 0.0) <= REL_TOL
    return plan, x, K


@pytest.mark.parametrize("shape,channels,batch", [
    ((37, 53, 7, 1, 3), 3, 16), ((130, 67, 7, 1, 3), 2, 4), ((100, 90, 5, 2, 2), 4, 8), ((33, 200, 3, 1, 1), 8, 1),
    ((75, 75, 9, 3, 8), 2, 3), ((40, 40, 13, 1, 6), 3, 5), ((6, 6, 2, 1, 5), 5, 7), ((1, 1, 1, 5, 2), 4, 3),
    ((224, 224, 7, 2, 3), 3, 16), ((56, 56, 3, 1, 1), 64, 4), ((300, 301, 2, 2, 0), 2, 12), ((64, 64, 3, 1, 1), 1, 16),
])
def test_channel_sum_matches_oracle(shape, channels, batch):
    plan, _, _ = _check(shape, channels, batch)
    plan.close()


def test_channel_sum_unaligned_operand():
    plan, _, _ = _check((50, 70, 5, 1, 2), 3, 4, seed=2, x_off=1)
    plan.close()


def test_one_channel_is_the_plain_build():
    shape, batch = (90, 120, 7, 1, 3), 16
    m, n, k, s, p = shape
    x, K = _case(shape, 1, batch, 3)
    a = cs.conv_csr_build_channels(m, n, k, s, p, torch.from_numpy(K).to(device()), 1)
    b = build_plan(shape, K)
    assert torch.equal(a.row_ptr, b.row_ptr) and torch.equal(a.col_idx, b.col_idx) and torch.equal(a.vals, b.vals)
    xd = torch.from_numpy(x).to(device())
    assert a.variant(batch) == b.variant(batch)
    assert torch.equal(cs.conv_spmv(a, xd, batch=batch), cs.conv_spmv(b, xd, batch=batch))
    a.close()
    b.close()


def test_update_kernel_rewrites_every_channel():
    shape, channels, batch = (60, 80, 5, 1, 2), 3, 8
    m, n, k, s, p = shape
    plan, x, _ = _check(shape, channels, batch, seed=4)
    K2 = np.random.default_rng(5).standard_normal(channels * k * k).astype(np.float32)
    cols_before = plan.col_idx.clone()
    cs.conv_update_kernel(plan, torch.from_numpy(K2).to(device()))
    y = cs.conv_spmv(plan, torch.from_numpy(x).to(device()), batch=batch)
    torch.cuda.synchronize()
    assert torch.equal(cols_before, plan.col_idx)
    ref, scale = oracle.conv_channels(m, n, k, s, p, x, K2, channels, batch=batch, want_scale=True)
    err = np.abs(y.cpu().numpy().astype(np.float64) - ref)
    assert np.max(err / np.maximum(scale, 1e-30)) <= REL_TOL
    plan.close()


def test_channel_errors():
    lib = binding._load()
    dev = device()
    K = torch.ones(18, device=dev)
    h = ctypes.c_void_p()
    assert lib.conv_csr_build_channels(4, 4, 3, 1, 1, 0, K.data_ptr(), 16, 16, 16, None, ctypes.byref(h)) == -1
    plan = cs.conv_csr_build_channels(8, 8, 3, 1, 1, K, 2)
    x = torch.zeros(128, device=dev)
    y = torch.zeros(64, device=dev)
    with pytest.raises(cs.ConvError):               # the fused multi-product launch takes one-channel plans
        cs.ConvMulti([plan], [x], [y], batch=1)
    with pytest.raises(ValueError):                 # x must hold both planes
        cs.conv_spmv(plan, torch.zeros(64, device=dev), y, batch=1)
    plan.close()


@pytest.mark.parametrize("shape,channels,batch", [
    ((37, 53, 7, 1, 3), 3, 16), ((130, 67, 7, 1, 3), 2, 4), ((100, 90, 5, 2, 2), 4, 8), ((33, 200, 3, 1, 1), 8, 1),
    ((75, 75, 9, 3, 8), 2, 3), ((6, 6, 2, 1, 5), 5, 7), ((224, 224, 7, 2, 3), 3, 16), ((56, 56, 3, 1, 1), 64, 4),
    ((64, 64, 3, 1, 1), 1, 16), ((300, 301, 2, 2, 0), 2, 12),
    # all channels in one launch (several channels, batch a multiple of 4): channel counts that do
    # and do not divide among the four waves, 4, 8 and 16 batch columns per lane, ragged tiles, strides,
    # k = 1, a patch that only fits with 4 columns per lane, tiles that lie wholly in the padding
    ((56, 56, 3, 1, 1), 64, 16), ((61, 43, 3, 1, 1), 5, 16), ((61, 43, 5, 2, 2), 7, 8), ((37, 53, 7, 1, 3), 4, 32),
    ((28, 28, 1, 1, 0), 9, 16), ((40, 45, 7, 2, 3), 6, 16), ((30, 30, 13, 1, 6), 4, 16), ((7, 7, 3, 1, 1), 33, 4),
    ((20, 22, 3, 1, 12), 4, 16), ((33, 31, 4, 3, 5), 5, 12), ((112, 112, 3, 2, 1), 16, 16),
    # planes with enough tiles for 16 and 8 batch columns per lane; patches of 5 to 16 items per lane;
    # unrolled (k = 3, 7) and looped (k = 5) taps at those widths
    ((224, 224, 3, 1, 1), 64, 16), ((224, 224, 3, 1, 1), 6, 8), ((300, 300, 7, 1, 3), 5, 16),
    ((256, 256, 5, 1, 2), 6, 16), ((448, 448, 7, 2, 3), 4, 8),
])
def test_channel_sum_from_the_structure_aware_storage(shape, channels, batch):
    m, n, k, s, p = shape
    x, K = _case(shape, channels, batch, 6)
    plan = cs.conv_compact_build(m, n, k, s, p, torch.from_numpy(K).to(device()), channels=channels)
    assert binding._load().conv_plan_channels(plan._handle) == channels
    assert np.array_equal(plan.row_desc.cpu().numpy(), oracle.compact_rows(m, n, k, s, p))
    assert np.array_equal(plan.ktab.cpu().numpy().view(np.uint32), K.view(np.uint32))
    y = torch.full((plan.rows * batch,), float("nan"), dtype=torch.float32, device=device())
    cs.conv_spmv(plan, torch.from_numpy(x).to(device()), y, batch=batch)
    y2 = cs.conv_spmv(plan, torch.from_numpy(x).to(device()), batch=batch)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)                        # the adds arrive in launch order: reproducible
    got = y.cpu().numpy()
    ref, scale = oracle.conv_channels(m, n, k, s, p, x, K, channels, batch=batch, want_scale=True)
    live = scale > 0
    assert not np.any(np.isnan(got)) and np.all(got[~live] == 0.0)
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    assert (np.max(err[live] / scale[live]) if np.any(live) else 0.0) <= REL_TOL
    K2 = np.random.default_rng(7).standard_normal(channels * k * k).astype(np.float32)
    cs.conv_update_kernel(plan, torch.from_numpy(K2).to(device()))
    y3 = cs.conv_spmv(plan, torch.from_numpy(x).to(device()), batch=batch)
    torch.cuda.synchronize()
    ref2, scale2 = oracle.conv_channels(m, n, k, s, p, x, K2, channels, batch=batch, want_scale=True)
    err2 = np.abs(y3.cpu().numpy().astype(np.float64) - ref2.astype(np.float64))
    assert (np.max(err2[scale2 > 0] / scale2[scale2 > 0]) if np.any(scale2 > 0) else 0.0) <= REL_TOL
    plan.close()


def test_channel_sums_in_one_launch_on_random_small_shapes():
    """Two hundred random shapes (planes up to 60 x 60, k up to 9, strides up to 4, paddings up to
    8) with 2 to 9 channels at batches 4, 8, 12 and 16: ragged tiles on both sides, tiles wholly in
    the padding, channel counts that leave waves without work."""
    rng = np.random.default_rng(2025)
    done = fused = 0
    while done < 200:
        k, s, p = int(rng.integers(1, 10)), int(rng.integers(1, 5)), int(rng.integers(0, 9))
        m, n = (int(v) for v in rng.integers(1, 61, size=2))
        if k > m + 2 * p or k > n + 2 * p:
            continue
        channels, batch = int(rng.integers(2, 10)), (4, 8, 12, 16)[done % 4]
        x, K = _case((m, n, k, s, p), channels, batch, 1000 + done)
        plan = cs.conv_compact_build(m, n, k, s, p, torch.from_numpy(K).to(device()), channels=channels)
        fused += plan.variant(batch).startswith("compact_channels")       # not when (3 s + k)(15 s + k) pixels do not fit
        y = cs.conv_spmv(plan, torch.from_numpy(x).to(device()), batch=batch)
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        ref, scale = oracle.conv_channels(m, n, k, s, p, x, K, channels, batch=batch, want_scale=True)
        err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
        assert np.all(got[scale == 0] == 0.0), (m, n, k, s, p, channels, batch)
        assert np.all(err <= REL_TOL * scale), (m, n, k, s, p, channels, batch)
        plan.close()
        done += 1
    assert fused >= 150, fused


def test_channels_in_one_launch_is_what_runs():
    m, n, k, s, p = 56, 56, 3, 1, 1
    K = torch.zeros(8 * k * k, device=device())
    plan = cs.conv_compact_build(m, n, k, s, p, K, channels=8)
    # 56 tiles: every batch gets the narrowest lanes (most workgroups) and all eight ways
    assert plan.variant(16) == "compact_channels_4x16_float4x1_8_ways_8_channels"
    assert plan.variant(12) == "compact_channels_4x16_float4x1_8_ways_8_channels"
    assert plan.variant(3).startswith("compact_gather")        # batch not a multiple of 4: one launch per channel (small plane: row groups)
    plan.close()
    for shape, channels, batch, want in [((224, 224, 3, 1, 1), 64, 16, "float4x4_4_ways"), ((224, 224, 3, 1, 1), 6, 8, "float4x2_4_ways"),
                                         ((300, 300, 7, 1, 3), 5, 16, "float4x4_4_ways"), ((448, 448, 7, 2, 3), 4, 8, "float4x2_4_ways")]:
        big = cs.conv_compact_build(*shape, torch.zeros(channels * shape[2] ** 2, device=device()), channels=channels)
        assert big.variant(batch) == "compact_channels_4x16_%s_%d_channels" % (want, channels)
        big.close()
    plan = cs.conv_compact_build(m, n, k, s, p, K[:3 * k * k], channels=3)
    assert plan.variant(16) == "compact_channels_4x16_float4x1_4_ways_3_channels"      # the fourth wave idles
    plan.close()
    plan = cs.conv_compact_build(m, n, k, s, p, K[:k * k])
    assert plan.variant(16).startswith("compact_gather")       # one channel: nothing to sum
    plan.close()
    plan = cs.conv_compact_build(1024, 1024, 7, 1, 3, torch.zeros(4 * 49, device=device()), channels=4)
    assert plan.variant(16).startswith("compact_rect")         # long products: a launch per channel is no burden
    plan.close()


def test_channels_in_one_launch_follow_edited_descriptors():
    """The one-launch kernel sums full k x k windows over a zero-padded patch only where the
    descriptors are the ones Theorem 2.1 gives; a wave that reads any other descriptor walks the
    described rectangles.  Rows are edited (a rectangle made smaller, one moved to another place
    of the image, one row emptied) and the result is compared with scipy on the decoded matrices."""
    import scipy.sparse as sp
    shape, channels, batch = (40, 45, 5, 1, 2), 6, 16
    m, n, k, s, p = shape
    x, K = _case(shape, channels, batch, 41)
    plan = cs.conv_compact_build(m, n, k, s, p, torch.from_numpy(K).to(device()), channels=channels)
    assert plan.variant(batch).startswith("compact_channels")
    desc = oracle.compact_rows(m, n, k, s, p).copy()
    mo, no = oracle.out_shape(m, n, k, s, p)
    r_small, r_moved, r_empty = 10 * no + 12, 25 * no + 30, 3 * no + 3
    desc[r_small, 1] = 1 | 2 << 8 | 0 << 16 | 3 << 24          # taps (1..2, 0..2) from the same first column
    desc[r_moved, 0] = 2 * n + 1                                # the full window, read from the image's corner
    desc[r_empty] = (0, 0)
    plan.row_desc.copy_(torch.from_numpy(desc).to(device()))
    y = cs.conv_spmv(plan, torch.from_numpy(x).to(device()), batch=batch)
    torch.cuda.synchronize()
    X = x.reshape(channels, m * n, batch).astype(np.float64)
    want = np.zeros((mo * no, batch))
    scale = np.zeros((mo * no, batch))
    for ch in range(channels):
        rp, ci, va = oracle.compact_decode(n, k, desc, K[ch * k * k:(ch + 1) * k * k])
        T = sp.csr_matrix((va.astype(np.float64), ci, rp), shape=(mo * no, m * n))
        want += T @ X[ch]
        scale += abs(T) @ np.abs(X[ch])
    got = y.cpu().numpy().reshape(-1, batch)
    assert np.all(got[r_empty] == 0.0)
    assert np.all(np.abs(got - want) <= REL_TOL * scale + 1e-30)
    ref = oracle.conv_channels(m, n, k, s, p, x, K, channels, batch=batch).reshape(-1, batch)
    changed = np.where(np.any(np.abs(got - ref) > REL_TOL * scale + 1e-30, axis=1))[0].tolist()
    assert set(changed) == {r_small, r_moved, r_empty}
    plan.close()


# ---- CSR storage, marching kernel: the channels of a block of lines walked inside one launch

def _check_march_channels(shape, channels, batch, seed=3, edit=None):
    m, n, k, s, p = shape
    x, K = _case(shape, channels, batch, seed)
    plan = cs.conv_csr_build_channels(m, n, k, s, p, torch.from_numpy(K).to(device()), channels)
    cs.conv_plan_set_march_min_jobs(plan, 1)       # test hook: small problems take the marching kernel too
    variant = plan.variant(batch)
    assert variant.startswith("lds_march_staged") and variant.endswith("_%d_channels" % channels), variant
    xd = torch.from_numpy(x).to(device())
    y = torch.full((plan.rows * batch,), float("nan"), dtype=torch.float32, device=device())
    cs.conv_spmv(plan, xd, y, batch=batch)
    torch.cuda.synchronize()
    got = y.cpu().numpy()
    ref, scale = oracle.conv_channels(m, n, k, s, p, x, K, channels, batch=batch, want_scale=True)
    assert not np.any(np.isnan(got)), shape
    assert np.all(got[scale == 0] == 0.0), shape
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    assert np.all(err <= REL_TOL * scale), (shape, channels, batch, float(np.max(err / np.maximum(scale, 1e-300))))
    # the sum has a fixed order: a second launch gives the same bits
    y2 = torch.full_like(y, float("nan"))
    cs.conv_spmv(plan, xd, y2, batch=batch)
    torch.cuda.synchronize()
    assert np.array_equal(got.view(np.uint32), y2.cpu().numpy().view(np.uint32))
    return plan, x, K, got


@pytest.mark.parametrize("shape,channels,batch", [
    ((37, 53, 7, 1, 3), 3, 16),        # nnz odd: the value arrays of channels 1, 2 start off a 16-byte boundary
    ((130, 97, 7, 1, 3), 2, 4),
    ((200, 150, 7, 1, 3), 3, 16),      # several strips and segments, ragged in both directions
    ((131, 70, 5, 1, 2), 4, 8),        # batch 8: float4 chunks of 4 columns, two column blocks
    ((128, 128, 9, 1, 4), 2, 1),       # SpMV, four lanes per row
    ((90, 120, 7, 1, 0), 5, 32),       # no padding; two column blocks of 16
    ((65, 33, 4, 1, 2), 7, 12),        # even kernel, strip of one column plus a full one
    ((40, 300, 6, 1, 5), 2, 16),       # p close to k: short rows at the borders
    ((90, 100, 11, 1, 5), 3, 4),       # eight lanes per row
    ((300, 200, 11, 4, 5), 2, 4),      # ... at stride 4
])
def test_march_channel_sum_in_one_launch(shape, channels, batch):
    plan, _, _, _ = _check_march_channels(shape, channels, batch)
    plan.close()


def test_march_channel_sum_reads_the_stored_arrays():
    """Values of one channel and shared columns edited in place: the launch follows the arrays
    (checked against scipy on the edited matrices)."""
    import scipy.sparse as sp
    shape, channels, batch = (70, 90, 7, 1, 3), 3, 16
    m, n, k, s, p = shape
    plan, x, K, _ = _check_march_channels(shape, channels, batch)
    rng = np.random.default_rng(5)
    nnz = plan.nnz
    vals = plan.vals.cpu().numpy().reshape(channels, nnz).copy()
    cols = plan.col_idx.cpu().numpy().copy()
    rp = plan.row_ptr.cpu().numpy()
    hit = rng.choice(nnz, size=200, replace=False)
    vals[1, hit] = rng.standard_normal(200).astype(np.float32)
    far = rng.choice(nnz, size=20, replace=False)          # columns far from the row's window: read from global memory
    cols[far] = rng.integers(0, m * n, size=20)
    plan.vals.copy_(torch.from_numpy(vals.reshape(-1)))
    plan.col_idx.copy_(torch.from_numpy(cols))
    y = cs.conv_spmv(plan, torch.from_numpy(x).to(device()), batch=batch)
    torch.cuda.synchronize()
    X = x.reshape(channels, m * n, batch).astype(np.float64)
    ref = np.zeros((plan.rows, batch))
    scale = np.zeros((plan.rows, batch))
    for ch in range(channels):
        # (copies: scipy merges duplicate columns of a row in place when asked for abs)
        T = sp.csr_matrix((vals[ch].astype(np.float64), cols.copy(), rp.copy()), shape=(plan.rows, m * n))
        ref += T @ X[ch]
        scale += abs(T) @ np.abs(X[ch])
    err = np.abs(y.cpu().numpy().reshape(plan.rows, batch).astype(np.float64) - ref)
    assert np.all(err <= REL_TOL * scale)
    plan.close()


def test_march_channel_sum_headline_shape_sampled():
    """1024 x 1024, k = 7, three channels, batch 16 (the default dispatch, no test hook): the
    whole result against the oracle's sum of padded convolutions."""
    shape, channels, batch = (1024, 1024, 7, 1, 3), 3, 16
    m, n, k, s, p = shape
    x, K = _case(shape, channels, batch, 11)
    plan = cs.conv_csr_build_channels(m, n, k, s, p, torch.from_numpy(K).to(device()), channels)
    assert plan.variant(batch).startswith("lds_march_staged") and plan.variant(batch).endswith("_3_channels")
    y = cs.conv_spmv(plan, torch.from_numpy(x).to(device()), batch=batch)
    torch.cuda.synchronize()
    ref, scale = oracle.conv_channels(m, n, k, s, p, x, K, channels, batch=batch, want_scale=True)
    err = np.abs(y.cpu().numpy().astype(np.float64) - ref.astype(np.float64))
    assert np.all(err <= REL_TOL * scale)
    plan.close()
