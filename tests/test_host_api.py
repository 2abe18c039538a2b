"""CPU-only checks of the C-ABI library: it loads, exports what the header
declares, and its host-side logic (Theorem 2.1 count, output shape, argument
validation) agrees with the oracle.  No kernel is launched here."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

import oracle
import paper_2411_19419_amd as cs
from paper_2411_19419_amd import binding, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "convspmv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(conv_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    lib = ctypes.CDLL(cs.library_path())
    for name in names:
        assert getattr(lib, name) is not None


def test_nnz_and_out_shape_match_oracle_on_tiny_grid():
    count = 0
    for m, n, k, s, p in itertools.product(range(1, 7), range(1, 7), range(1, 6), range(1, 4), range(0, 7)):
        if k > m + 2 * p or k > n + 2 * p:
            with pytest.raises(cs.ConvError) as ei:
                cs.conv_nnz(m, n, k, s, p)
            assert ei.value.status == -1
            continue
        assert cs.conv_nnz(m, n, k, s, p) == oracle.nnz_closed(m, n, k, s, p)
        assert cs.conv_out_shape(m, n, k, s, p) == oracle.out_shape(m, n, k, s, p)
        count += 1
    assert count > 3000


def test_nnz_on_named_workloads_and_layer_table():
    want = {
        "small_32_k3": 8836, "strided_256_k5_b64": 405769, "headline_1024_k7_b16": 51208336,
        "cnn_224_k3_b256": 448900, "padheavy_512_k9_s3": 2359296, "padheavy_4096_k11_s4_b4": 126697536,
    }
    for name, nnz in want.items():
        w = workloads.WORKLOADS[name]
        assert cs.conv_nnz(*w.shape) == nnz
    for shp in set(workloads.densenet121_layer_shapes()):
        assert cs.conv_nnz(*shp) == oracle.nnz_brute(*shp)
    # rectangular, k > m, p >= k
    for shp in [(3, 50, 7, 2, 3), (2, 9, 5, 1, 2), (4, 4, 2, 3, 7), (1, 1, 1, 5, 2), (100, 3, 3, 1, 0)]:
        assert cs.conv_nnz(*shp) == oracle.nnz_brute(*shp)


def test_nnz_is_exact_beyond_int32():
    # "same" 3x3 on 40000^2: (3*40000 - 2)^2 entries
    assert cs.conv_nnz(40000, 40000, 3, 1, 1) == (3 * 40000 - 2) ** 2


def test_argument_validation_without_a_gpu():
    lib = binding._load()
    for bad in [(0, 4, 1, 1, 0), (4, 0, 1, 1, 0), (4, 4, 0, 1, 0), (4, 4, 1, 0, 0), (4, 4, 1, 1, -1),
                (4, 4, 7, 1, 1), (4, 9, 7, 1, 1)]:
        assert lib.conv_nnz(*bad) == -1
        mo, no = ctypes.c_int(), ctypes.c_int()
        assert lib.conv_out_shape(*bad, ctypes.byref(mo), ctypes.byref(no)) == -1
        h = ctypes.c_void_p()
        assert lib.conv_csr_build(*bad, 16, 16, 16, 16, None, ctypes.byref(h)) == -1
        assert h.value is None
        assert lib.conv_compact_build(*bad, 16, 16, 16, None, ctypes.byref(h)) == -1 and h.value is None
    assert lib.conv_compact_build(300, 300, 256, 1, 0, 16, 16, 16, None, ctypes.byref(h)) == -1    # k > 255
    assert lib.conv_compact_build(4, 4, 3, 1, 1, 16, 20, 16, None, ctypes.byref(h)) == -1          # descriptors not 8-byte aligned
    assert lib.conv_compact_build(4, 4, 3, 1, 1, 16, None, 16, None, ctypes.byref(h)) == -2
    assert lib.conv_compact_build(4, 4, 3, 1, 1, 16, 16, 16, None, None) == -2
    assert lib.conv_compact_build(50000, 50000, 3, 1, 1, 16, 16, 16, None, ctypes.byref(h)) == -3  # rows beyond int32
    assert lib.conv_plan_is_compact(None) == -2
    assert lib.conv_csr_build_channels(4, 4, 3, 1, 1, 0, 16, 16, 16, 16, None, ctypes.byref(h)) == -1
    assert lib.conv_csr_build_channels(4, 4, 3, 1, 1, 2, None, 16, 16, 16, None, ctypes.byref(h)) == -2
    assert lib.conv_csr_build_channels(30000, 30000, 1, 1, 0, 3, 16, 16, 16, 16, None, ctypes.byref(h)) == -3
    assert lib.conv_plan_channels(None) == -2
    assert lib.conv_compact_build_channels(4, 4, 3, 1, 1, 0, 16, 16, 16, None, ctypes.byref(h)) == -1
    assert lib.conv_spmv_from_csc(None, 16, 32, 1, None) == -2
    assert lib.conv_out_shape(4, 4, 1, 1, 0, None, None) == -2
    h = ctypes.c_void_p()
    assert lib.conv_csr_build(4, 4, 3, 1, 1, None, None, None, None, None, ctypes.byref(h)) == -2
    assert lib.conv_csr_build(4, 4, 3, 1, 1, 16, 16, 16, 16, None, None) == -2
    # more entries than int32 indices can address
    assert lib.conv_csr_build(40000, 40000, 3, 1, 1, 16, 16, 16, 16, None, ctypes.byref(h)) == -3
    assert lib.conv_spmv(None, 16, 32, 1, None) == -2
    assert lib.conv_plan_shape(None, *([None] * 8)) == -2
    assert lib.conv_spmv_variant(None, 1) is None
    assert lib.conv_plan_destroy(None) == 0
    assert lib.conv_update_kernel(None, 16, None) == -2
    m_out = ctypes.c_void_p()
    assert lib.conv_multi_create(1, None, None, None, 1, ctypes.byref(m_out)) == -2
    arr = (ctypes.c_void_p * 1)(None)
    assert lib.conv_multi_create(0, arr, arr, arr, 1, ctypes.byref(m_out)) == -1
    assert lib.conv_multi_create(1, arr, arr, arr, 0, ctypes.byref(m_out)) == -1
    assert lib.conv_multi_create(1, arr, arr, arr, 1, ctypes.byref(m_out)) == -2 and m_out.value is None
    assert lib.conv_multi_apply(None, None) == -2
    assert lib.conv_multi_destroy(None) == 0
    assert lib.conv_plan_set_march_min_jobs(None, 4) == -2
    d = binding.ConvDispatch()
    assert lib.conv_test_dispatch_info(64, 64, 3, 1, 1, 1, 0, 1, 0, ctypes.byref(d)) == -1       # threshold < 1
    # the entry point that allocates nothing checks its arguments like the build, and its size limit
    assert lib.conv_csr_fill_noalloc(0, 4, 3, 1, 1, 16, 16, 16, 16, None) == -1
    assert lib.conv_csr_fill_noalloc(8, 8, 3, 1, 1, None, 16, 16, 16, None) == -2
    assert lib.conv_csr_fill_noalloc(8, 8, 3, 1, 1, 16, None, 16, 16, None) == -2
    assert lib.conv_csr_fill_noalloc(40000, 40000, 3, 1, 1, 16, 16, 16, 16, None) == -3          # nnz beyond int32
    assert lib.conv_csr_fill_noalloc(40000, 30000, 1, 1, 0, 16, 16, 16, 16, None) == -3          # m_out + n_out + 2 > 65536


def test_strerror_texts():
    seen = set()
    for code in range(0, -7, -1):
        text = cs.conv_strerror(code)
        assert text and text != "unknown status"
        seen.add(text)
    assert len(seen) == 7
    assert cs.conv_strerror(-99) == "unknown status"


def test_small_divisor_float_trick_is_exact():
    """The device code divides small non-negative integers by multiplying
    (a + 0.5) with a float reciprocal and truncating; check the claim over the
    whole range it is used for, with the reciprocal off by one ulp either way."""
    a = np.arange(0, 1 << 21, dtype=np.int64)
    af = a.astype(np.float32) + np.float32(0.5)
    for d in [1, 2, 3, 5, 7, 9, 11, 13, 25, 49, 121, 224, 1000, 1024, 4095, 4096, 4099, 65537]:
        inv = np.float32(1.0) / np.float32(d)
        for cand in (inv, np.nextafter(inv, np.float32(0)), np.nextafter(inv, np.float32(1))):
            q = (af * cand).astype(np.int64)
            assert np.array_equal(q, a // d), d


def test_workload_generators_are_seeded_and_shaped():
    w = workloads.WORKLOADS["small_32_k3"]
    x1, k1 = workloads.make(w)
    x2, k2 = workloads.make(w)
    assert x1.dtype == np.float32 and k1.dtype == np.float32
    assert x1.shape == (32 * 32,) and k1.shape == (9,)
    assert np.array_equal(x1, x2) and np.array_equal(k1, k2)
    assert np.all(np.abs(x1) <= 1.0)
    w = workloads.WORKLOADS["headline_1024_k7_b16"]
    k = workloads.make_kernel(w.k, w.k_std, w.seed)
    assert abs(float(np.std(k)) - 1.0 / 7.0) < 0.05
    assert len(workloads.densenet121_layer_shapes()) == 123


def test_header_is_plain_c(tmp_path):
    """include/convspmv.h is a C header: it compiles as C99 with gcc, alone, and a C program that
    calls the host-only entry points through it links against the library and runs."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_header.c"
    src.write_text(
        '#include "convspmv.h"\n'
        '#include <stdio.h>\n'
        'int main(void) {\n'
        '    int mo = 0, no = 0;\n'
        '    if (conv_out_shape(1024, 1024, 7, 1, 3, &mo, &no) != CONV_OK) return 1;\n'
        '    printf("%d %d %lld %s\\n", mo, no, (long long)conv_nnz(1024, 1024, 7, 1, 3), conv_strerror(CONV_EALIAS));\n'
        '    return conv_nnz(4, 4, 9, 1, 0) == CONV_EINVAL ? 0 : 2;\n'
        '}\n')
    exe = tmp_path / "use_header"
    libdir = os.path.dirname(binding.library_path())
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-lconvspmv", "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(None, 3)
    assert out[:3] == ["1024", "1024", "51208336"] and out[3].strip() == "x and y overlap"


def _dispatch(m, n, k, s, p, batch, storage=0, channels=1):
    d = cs.conv_dispatch_info(m, n, k, s, p, batch, storage, channels)
    return {f[0]: getattr(d, f[0]) for f in d._fields_}


def test_dispatch_geometry_is_consistent_over_many_shapes():
    """The host logic that picks a kernel and its launch geometry, queried without a GPU: LDS
    within a CU's 160 KiB, rings at least as long as a step needs, strips and lanes that tile
    the workgroup, on a grid of shapes, batches and storages."""
    rng = np.random.default_rng(0)
    shapes = [(1024, 1024, 7, 1, 3), (224, 224, 7, 2, 3), (4096, 4096, 11, 4, 5), (512, 512, 9, 3, 8),
              (6600, 6600, 7, 1, 3), (20000, 300, 5, 1, 2), (300, 20000, 5, 2, 2), (64, 64, 1, 1, 0),
              (300, 300, 255, 3, 100), (700, 900, 40, 1, 20), (56, 56, 2, 2, 0), (3, 3, 9, 2, 3)]
    for _ in range(400):
        k = int(rng.integers(1, 20))
        s = int(rng.integers(1, 6))
        p = int(rng.integers(0, 12))
        m, n = (int(v) for v in rng.integers(max(1, k - 2 * p), 3000, size=2))
        shapes.append((m, n, k, s, p))
    seen = set()
    for shape in shapes:
        m, n, k, s, p = shape
        for batch in (1, 3, 4, 8, 16, 64):
            for storage in (0, 1, 2):
                d = _dispatch(*shape, batch, storage)
                seen.add(d["kernel"])
                assert 0 <= d["lds_bytes"] <= 160 * 1024, (shape, batch, storage, d)
                assert 64 <= d["threads"] <= 1024 and d["threads"] % 64 == 0, (shape, batch, storage, d)
                assert d["workgroups"] >= 1
                if d["ring_lines"]:
                    assert d["ring_lines"] & (d["ring_lines"] - 1) == 0
                    assert 0 < d["ring_lines_needed"] <= d["ring_lines"], (shape, batch, storage, d)
                if d["kernel"] == 3:        # marching kernel: rows of at least 16 and at most 128 entries
                    rows = k * k if storage == 0 else ((k + s - 1) // s) ** 2
                    assert 16 <= rows <= 128 and d["strip"] in (32, 64) and d["segment"] % 2 == 0
                    assert d["lines_per_step"] in (1, 2) and d["threads"] == 512
                if d["kernel"] == 9:        # entries staged through LDS: rows of 16 to 128 entries, 2, 4 or 8 lanes per row
                    rows = k * k if storage == 0 else ((k + s - 1) // s) ** 2
                    assert 16 <= rows <= 128 and d["strip"] == 32 and d["lanes_per_row"] in (2, 4, 8)
                    assert d["lanes_per_row"] == (2 if rows <= 50 else 4 if rows <= 100 else 8)
                    assert d["lines_per_step"] * d["lanes_per_row"] == 16 and d["threads"] == 512
                    assert d["segment"] % d["lines_per_step"] == 0 and d["ring_lines"] == 16
                if d["kernel"] == 5:        # rectangle path: only the compiled (k, s)
                    assert (s == 1 and k in (1, 3, 5, 7, 9)) or (s == 2 and k in (2, 3, 5, 7))
                    assert d["lines_per_step"] == (4 if s == 1 else 2) and d["strip"] * d["lanes_per_row"] == 256
                    assert d["segment"] % d["lines_per_step"] == 0
                if d["kernel"] == 4:        # described rows: groups of lanes share the lines of a step
                    groups = 256 // (d["strip"] * d["lanes_per_row"])
                    assert groups >= 1 and 256 % (d["strip"] * d["lanes_per_row"]) == 0
                    assert d["lines_per_step"] % groups == 0 and d["segment"] % d["lines_per_step"] == 0
                if d["kernel"] == 10:       # row groups over the descriptors: only where marching leaves CUs idle
                    assert storage == 2 and d["lanes_per_row"] in (1, 2, 4, 8, 16) and d["lds_bytes"] == 0
                    mo, no = cs.conv_out_shape(m, n, k, s, p)
                    assert d["workgroups"] >= (mo * no * d["lanes_per_row"] + 255) // 256
                if storage == 2:
                    assert d["kernel"] in (4, 5, 10)
                else:
                    assert d["kernel"] in (0, 1, 2, 3, 9)
                    if batch % 4:
                        assert d["columns_per_lane"] == 1
    assert seen == {0, 1, 2, 3, 4, 5, 9, 10}


def test_march_edge_grid_dispatch():
    """The shapes of the GPU tests' edge grids, with the test hook's threshold of one job, go to a
    marching kernel (3: entries loaded by the lane groups, 9: entries staged through LDS) -- except where the geometry
    refuses, and it refuses only at strides above 1 (or rows of fewer than 16 entries): every shape
    of the grids with stride 1 marches, and four in five overall."""
    for transposed in (False, True):
        total = marching = 0
        kinds = set()
        for (m, n, k, s, p), batch in workloads.march_edge_grid(transposed=transposed):
            d = cs.conv_dispatch_info(m, n, k, s, p, batch, 1 if transposed else 0, 1, march_min_jobs=1)
            total += 1
            if d.kernel in (3, 9):
                marching += 1
                kinds.add(d.kernel)
                assert d.ring_lines_needed <= d.ring_lines and d.lds_bytes <= 160 * 1024
            else:
                # refusals: only at strides above 1, where a step adds more operand lines than the
                # kernels' line registers hold or the ring is too short, or rows are too short
                rows = ((k + s - 1) // s) ** 2 if transposed else k * k
                assert s > 1 or rows < 16, ((m, n, k, s, p), batch, d.kernel)
        assert total > 1500 and marching >= 0.8 * total, (transposed, total, marching)
        assert kinds == {3, 9}
    # with the default threshold none of these small shapes marches
    for (m, n, k, s, p), batch in list(workloads.march_edge_grid())[::50]:
        assert cs.conv_dispatch_info(m, n, k, s, p, batch).kernel in (0, 1, 2)


def test_march_quotient_trick_is_exact():
    """The marching kernels locate a stored column in the LDS ring by di = trunc(fma(float(dB),
    inv_nB, 0.5/n)) with dB = PIXB*(di*n + dj) a multiple of PIXB below 2^25, inv_nB the rounded
    1/(n*PIXB): the quotient must come out exact for every dj in [0, n) and every line di the
    ring can hold (di < 2*NL = 32), for all n the host guard lets through (2*NL*n*16 <= 2^25,
    n <= 65536), for 16- and 4-byte pixels."""
    rng = np.random.default_rng(7)
    ns = sorted(set([1, 2, 3, 5, 7, 30, 31, 32, 33, 63, 64, 65, 224, 1000, 1023, 1024, 1025, 4096, 4099, 6600, 16384,
                     32767, 32768, 32769, 65535, 65536] + [int(v) for v in rng.integers(1, 65537, size=60)]))
    for pixb in (16, 4):
        for n in ns:
            inv_n = np.float32(1.0) / np.float32(n)
            inv_nb = inv_n / np.float32(pixb)
            half = np.float32(0.5) * inv_n
            # every line, and per line the first, last and a sample of the pixels (all of them for small n)
            dj = np.arange(n, dtype=np.int64) if n <= 4096 else np.unique(np.concatenate(
                [np.arange(0, 64), np.arange(n - 64, n), rng.integers(0, n, size=2000)]))
            di = np.arange(32, dtype=np.int64)[:, None]
            db = (di * n + dj[None, :]) * pixb
            assert db.max() < 2 ** 25 * (pixb // 4 if pixb == 4 else 1) or n > 65536 // 2
            f = db.astype(np.float32)                       # exact: below 2^25 and a multiple of pixb >= 4, or below 2^24
            assert np.array_equal(f.astype(np.int64), db)
            # one fused multiply-add, rounded once: evaluate in float64 (exact product of two floats plus
            # a float is within float64's reach here) and round to float32
            q = (f.astype(np.float64) * np.float64(inv_nb) + np.float64(half)).astype(np.float32)
            got = q.astype(np.int64)
            assert np.array_equal(got, np.broadcast_to(di, got.shape)), (pixb, n)


def test_dispatch_of_channel_sums_from_the_structure_aware_storage():
    """All channels in one launch when there are several, the batch is a multiple of 4 and a
    channel's product is short; otherwise the per-channel kernels.  LDS of the waves' patches of
    (3 s + k) x (15 s + k) pixels within 64 KiB, fewer batch columns per lane when they would not fit."""
    d = _dispatch(224, 224, 3, 1, 1, 16, 2, 64)                          # 784 tiles: full lines per lane, 4 ways
    assert d["kernel"] == 6 and d["threads"] == 256 and d["columns_per_lane"] == 16
    assert d["workgroups"] == 56 * 14 and d["strip"] == 16 and d["segment"] == 4
    assert d["lds_bytes"] == 4 * 16 * (6 * 18 * 4 + 3)
    d = _dispatch(56, 56, 3, 1, 1, 16, 2, 64)                            # 56 tiles: narrow lanes, 16 ways
    assert d["kernel"] == 6 and d["threads"] == 1024 and d["columns_per_lane"] == 4 and d["workgroups"] == 14 * 4 * 4
    assert _dispatch(224, 224, 3, 1, 1, 32, 2, 64)["workgroups"] == 56 * 14 * 2
    assert _dispatch(224, 224, 3, 1, 1, 8, 2, 64)["columns_per_lane"] == 8
    assert _dispatch(224, 224, 3, 1, 1, 20, 2, 64)["columns_per_lane"] == 4
    assert _dispatch(56, 56, 3, 1, 1, 6, 2, 64)["kernel"] == 10         # batch not a multiple of 4 (small plane: row groups)
    assert _dispatch(448, 448, 3, 1, 1, 6, 2, 64)["kernel"] == 5
    assert _dispatch(56, 56, 3, 1, 1, 16, 2, 3)["threads"] == 256       # fewer channels than waves: the fourth idles
    assert _dispatch(56, 56, 3, 1, 1, 16, 2, 1)["kernel"] == 10         # one channel: nothing to sum
    assert _dispatch(448, 448, 3, 1, 1, 16, 2, 1)["kernel"] == 5
    assert _dispatch(1024, 1024, 7, 1, 3, 16, 2, 64)["kernel"] == 5     # long products
    d = _dispatch(150, 150, 13, 1, 6, 16, 2, 8)                          # 16 x 28 patch: 16 columns per lane do not fit
    assert d["kernel"] == 6 and d["columns_per_lane"] == 8 and d["lds_bytes"] <= 64 * 1024
    assert _dispatch(100, 100, 40, 1, 20, 16, 2, 8)["kernel"] == 10     # 43 x 55 patch: no fit; a small plane, so row groups
    assert _dispatch(1000, 1000, 40, 1, 20, 16, 2, 8)["kernel"] == 4    # ... described rows on a large one
    for k, s in ((1, 1), (3, 1), (3, 2), (5, 1), (7, 2), (9, 3), (11, 1)):
        for batch in (4, 8, 12, 16, 64):
            for channels in (4, 12, 100):
                d = _dispatch(112, 96, k, s, k // 2, batch, 2, channels)
                assert d["kernel"] == 6 and d["lds_bytes"] <= 64 * 1024 and batch % d["columns_per_lane"] == 0
                assert d["threads"] in (256, 512, 1024) and d["threads"] // 64 <= max(channels, 4)
                assert d["workgroups"] * d["columns_per_lane"] >= batch
                patch = (3 * s + k) * (15 * s + k) * d["columns_per_lane"] // 4
                assert patch <= 16 * 64 and d["lds_bytes"] >= d["threads"] // 64 * 16 * patch


def test_dispatch_of_the_product_from_csc_over_many_shapes():
    """Host logic of conv_spmv_from_csc (storage 3): the on-chip scatter's tile, window and lane
    layout stay within what its kernel assumes -- a tile line's entries within the 1024-entry
    stage, the lanes of a wave enough for a line's column pointers, the window within 64 KiB of
    LDS and 2^21 rows from its first one, batch columns per wave dividing 4 -- and the direct
    scatter takes the shapes the header names."""
    rng = np.random.default_rng(5)
    shapes = [(1024, 1024, 7, 1, 3), (1024, 1024, 3, 1, 1), (224, 224, 7, 2, 3), (4096, 4096, 11, 4, 5), (56, 56, 1, 1, 0),
              (300, 300, 255, 3, 100), (700, 900, 40, 1, 20), (56, 56, 2, 2, 0), (3, 3, 9, 2, 3), (20, 200000, 3, 1, 1),
              (64, 64, 33, 1, 16), (64, 64, 32, 1, 16), (500, 500, 64, 2, 10)]
    for _ in range(400):
        k, s, p = int(rng.integers(1, 40)), int(rng.integers(1, 6)), int(rng.integers(0, 12))
        m, n = (int(v) for v in rng.integers(max(1, k - 2 * p), 3000, size=2))
        if oracle.nnz_closed(m, n, k, s, p) < 2 ** 31:
            shapes.append((m, n, k, s, p))
    seen = set()
    for m, n, k, s, p in shapes:
        per_axis = -(-k // s)
        mo, no = oracle.out_shape(m, n, k, s, p)
        for batch in (1, 2, 3, 4, 5, 8, 9, 16, 48):
            d = _dispatch(m, n, k, s, p, batch, 3)
            seen.add(d["kernel"])
            if per_axis ** 2 > 1024 or per_axis ** 2 < (4 if batch >= 4 else 9):
                assert d["kernel"] == 8, (m, n, k, s, p, batch)
            if d["kernel"] == 8:
                assert d["threads"] == 256 and d["workgroups"] >= 1
                continue
            assert d["kernel"] == 7
            ti, tj, wx, wy, vb, waves = d["segment"], d["strip"], d["ring_lines_needed"], d["lines_per_step"], d["columns_per_lane"], d["threads"] // 64
            assert 1 <= tj <= 32 and 1 <= ti <= 64 and tj * per_axis ** 2 <= 1024
            assert wx == min((ti + k - 2) // s + 1, mo) and wy == min((tj + k - 2) // s + 1, no)
            assert (wx - 1) * no + wy <= 1 << 21 and wx * wy < 1 << 16
            assert vb in (1, 2, 4) and waves in (1, 2, 4) and vb * waves <= 16
            assert (vb == batch) if batch < 3 else vb == 4
            stage = (tj * per_axis ** 2 + 1) // 2 * 2
            assert d["lds_bytes"] == 16 * stage + 4 * ((ti * (tj + 1) + 3) // 4 * 4) + wx * wy * vb * waves * 4 <= 64 * 1024
            tiles = -(-m // ti) * -(-n // tj)
            assert d["workgroups"] == tiles * min(-(-batch // (vb * waves)), 65535)
            group = d["lanes_per_row"]
            assert group == (64 // per_axis ** 2 if per_axis ** 2 <= 16 else 1) and group * min(per_axis ** 2, 64) <= 64
    assert seen == {7, 8}
    with pytest.raises(cs.ConvError):
        _dispatch(64, 64, 3, 1, 1, 16, 3, 2)          # no channels with the column-compressed arrays


def test_dispatch_of_the_named_workloads():
    want = {"small_32_k3": 0, "strided_256_k5_b64": 2, "headline_1024_k7_b1": 9, "headline_1024_k7_b16": 9,
            "cnn_224_k3_b256": 2, "padheavy_512_k9_s3": 0, "padheavy_4096_k11_s4_b4": 9}
    for name, kernel in want.items():
        w = workloads.WORKLOADS[name]
        assert _dispatch(*w.shape, w.batch)["kernel"] == kernel, name
    d = _dispatch(*workloads.WORKLOADS["headline_1024_k7_b16"].shape, 16)
    assert (d["strip"], d["segment"], d["ring_lines"], d["lines_per_step"], d["lds_bytes"], d["workgroups"]) == \
        (32, 128, 16, 8, 163072, 256)
    c = _dispatch(*workloads.WORKLOADS["headline_1024_k7_b16"].shape, 16, storage=2)
    assert (c["kernel"], c["strip"], c["segment"], c["lines_per_step"], c["workgroups"]) == (5, 64, 32, 4, 512)
    # several channels: the LDS tile kernel is not used (one launch per channel would not pay)
    assert _dispatch(224, 224, 3, 1, 1, 16, 0, 64)["kernel"] == 1
    assert _dispatch(1024, 1024, 7, 1, 3, 16, 0, 3)["kernel"] == 9
    for bad in [(4, 4, 9, 1, 0, 1, 0, 1), (8, 8, 3, 1, 1, 0, 0, 1), (8, 8, 3, 1, 1, 1, 4, 1), (8, 8, 3, 1, 1, 1, 1, 2),
                (300, 300, 256, 1, 0, 1, 2, 1)]:
        with pytest.raises(cs.ConvError):
            cs.conv_dispatch_info(*bad)
