"""Host-side tests of the C-ABI library (no GPU): exported symbols, the
offline step (a) against the oracle's vector-wise form, the round trip, and
every error path of argument validation."""
import ctypes
import re
import os

import numpy as np
import pytest

from oracle import definition
from paper_2203_05016_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "shflbw.h")).read()
    declared = set(re.findall(r"\b(shflbw_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    L = binding.lib()
    for name in declared:
        assert hasattr(L, name), name


@pytest.mark.parametrize("V", [16, 32, 64, 128])
@pytest.mark.parametrize("ragged", [False, True])
def test_compress_matches_vectorwise_form_and_round_trips(V, ragged):
    p = synth.make_spmm(4 * V, 200, 8, V, 0.7, seed=100 + V, ragged=ragged)
    A = binding.compress(p.W, p.mask, p.perm, V)
    ri, cols, _ = definition.vectorwise_form(p.W, p.mask, p.perm, V)
    assert np.array_equal(A.row_indices(), ri)
    for g in range(4):
        got = A.group_columns(g)
        assert np.array_equal(got, cols[g])
        assert np.all(np.diff(got) > 0) and (got.size == 0 or (got[0] >= 0 and got[-1] < 200))
    info = A.info()
    assert (info["M"], info["K"], info["V"], info["groups"]) == (4 * V, 200, V, 4)
    assert info["nnz"] == int(p.mask.sum()) == V * sum(len(c) for c in cols)
    assert abs(info["sparsity"] - (1 - p.mask.mean())) < 1e-12
    want = np.where(p.mask != 0, p.W, np.float16(0))
    assert np.array_equal(A.decompress().view(np.uint16), want.view(np.uint16))
    assert A.device_bytes() % 256 == 0 and A.device_bytes() > 0


def test_empty_group_and_all_empty():
    p = synth.make_spmm(64, 40, 4, 32, 0.5, seed=7)
    p.mask[p.perm[32:]] = 0
    A = binding.compress(p.W, p.mask, p.perm, 32)
    assert A.group_columns(1).size == 0 and A.group_columns(0).size == 20
    B = binding.compress(p.W, np.zeros_like(p.mask), p.perm, 32)
    assert B.info()["nnz"] == 0 and B.info()["sparsity"] == 1.0
    assert not B.decompress().any()


@pytest.mark.parametrize("V", [16, 32])
def test_distant_column_bands_round_trip(V):
    """Two bands of kept columns far apart: the windowed layout bridges them
    with empty k-steps, which must not show in the columns or the weights."""
    p = synth.make_spmm(3 * V, 2560, 8, V, 0.0, seed=23 + V)
    p.mask[:, 512:2048] = 0
    p.mask[p.perm[V:2 * V], :448] = 0
    A = binding.compress(p.W, p.mask, p.perm, V)
    band = np.concatenate([np.arange(512), np.arange(2048, 2560)])
    assert np.array_equal(A.group_columns(0), band)
    assert np.array_equal(A.group_columns(1), band[band >= 448])
    assert A.info()["nnz"] == int(p.mask.sum())
    want = np.where(p.mask != 0, p.W, np.float16(0))
    assert np.array_equal(A.decompress().view(np.uint16), want.view(np.uint16))


def test_null_mask_keeps_vectors_with_any_nonzero():
    p = synth.make_spmm(32, 24, 4, 16, 0.5, seed=8)
    Wm = np.where(p.mask != 0, p.W, np.float16(0))
    # a kept vector that is zero in all but one row stays kept; -0.0 counts as zero
    g0rows = p.perm[:16]
    c = int(p.cols[0][0])
    Wm[g0rows, c] = 0
    Wm[g0rows[3], c] = np.float16(0.5)
    c2 = int(p.cols[0][1])
    Wm[g0rows, c2] = np.float16(-0.0)
    A = binding.compress(Wm, None, p.perm, 16)
    got = A.group_columns(0)
    assert c in got and c2 not in got
    assert np.array_equal(A.decompress().view(np.uint16) & 0x7fff,
                          Wm.view(np.uint16) & 0x7fff)


def test_leading_dimension():
    p = synth.make_spmm(32, 20, 4, 16, 0.5, seed=9)
    Wp = np.full((32, 29), np.float16(7))
    Wp[:, :20] = p.W
    A = binding.compress(Wp, p.mask, p.perm, 16, K=20)
    want = np.where(p.mask != 0, p.W, np.float16(0))
    out = A.decompress(ldw=23)
    assert np.array_equal(out[:, :20], want) and not out[:, 20:].any()


def test_kept_zero_weights_are_stored():
    p = synth.make_spmm(32, 20, 4, 16, 0.5, seed=10)
    p.W[p.perm[0], p.cols[0][0]] = 0
    A = binding.compress(p.W, p.mask, p.perm, 16)
    assert A.info()["nnz"] == int(p.mask.sum())
    assert p.cols[0][0] in A.group_columns(0)


def _raw_compress(W, ldw, mask, perm, M, K, V, dtype=binding.F16, out=True):
    h = ctypes.c_void_p()
    rc = binding.lib().shflbw_compress(
        None if W is None else W.ctypes.data, ldw, None if mask is None else mask.ctypes.data,
        None if perm is None else perm.ctypes.data, M, K, V, dtype,
        ctypes.byref(h) if out else None)
    if rc == 0:
        binding.lib().shflbw_destroy(h)
    return rc


def test_error_paths():
    p = synth.make_spmm(64, 30, 4, 32, 0.5, seed=11)
    W, m, pm = p.W, p.mask, p.perm
    assert _raw_compress(W, 30, m, pm, 64, 30, 32) == 0
    assert _raw_compress(None, 30, m, pm, 64, 30, 32) == -1
    assert _raw_compress(W, 30, m, pm, 64, 30, 32, out=False) == -1
    assert _raw_compress(W, 30, m, pm, 64, 30, 24) == -2          # unsupported V
    assert _raw_compress(W, 30, m, pm, 48, 30, 32) == -2          # M % V
    assert _raw_compress(W, 29, m, pm, 64, 30, 32) == -2          # ldw < K
    assert _raw_compress(W, 30, m, pm, 64, 0, 32) == -2
    assert _raw_compress(W, 30, m, pm, 64, 30, 32, dtype=binding.F32) == -5
    bad = pm.copy()
    bad[5] = bad[6]
    assert _raw_compress(W, 30, m, bad, 64, 30, 32) == -3
    assert "perm[6]" in binding.last_error()
    bad[5] = 64
    assert _raw_compress(W, 30, m, bad, 64, 30, 32) == -3
    mb = m.copy()
    row = pm[32 + 4]
    col = int(np.nonzero(mb[row] == 0)[0][0])
    mb[row, col] = 1
    assert _raw_compress(W, 30, mb, pm, 64, 30, 32) == -4
    msg = binding.last_error()
    want = definition.check_pattern(mb, pm, 32)
    assert want == (1, 36, col)
    assert "group 1" in msg and "stored row 36" in msg and ("column %d" % col) in msg
    assert binding.status_string(-4).startswith("mask is not")
    assert binding.status_string(0) == "ok" and binding.status_string(-99) == "unknown status"


def test_device_calls_validate_before_touching_the_gpu():
    p = synth.make_spmm(32, 20, 8, 16, 0.5, seed=12)
    A = binding.compress(p.W, p.mask, p.perm, 16)
    L = binding.lib()
    one = ctypes.c_void_p(256)
    assert L.shflbw_spmm(None, one, 8, one, 8, 8, binding.F16, None) == -1
    assert L.shflbw_spmm(A._h, one, 8, one, 8, 0, binding.F16, None) == 0       # N == 0: no-op
    assert L.shflbw_spmm(A._h, one, 8, one, 8, 8, 1, None) == -5
    assert L.shflbw_spmm(A._h, one, 4, one, 8, 8, binding.F16, None) == -2      # ldx < N
    assert L.shflbw_spmm(A._h, None, 8, one, 8, 8, binding.F16, None) == -1
    assert L.shflbw_spmm(A._h, one, 8, one, 8, 8, binding.F16, None) == -6      # not bound
    conv = lambda *a: L.shflbw_conv2d(A._h, one, one, *a, None)
    assert conv(2, 5, 4, 4, 2, 2, 1, 1, 0, 0, binding.NCHW, binding.F16) == -6  # K = 5*2*2 ok
    assert conv(2, 4, 4, 4, 2, 2, 1, 1, 0, 0, binding.NCHW, binding.F16) == -2  # K mismatch
    assert conv(2, 5, 1, 4, 2, 2, 1, 1, 0, 0, binding.NCHW, binding.F16) == -2  # kernel > input
    assert conv(2, 5, 4, 4, 2, 2, 0, 1, 0, 0, binding.NCHW, binding.F16) == -2  # stride 0
    assert conv(2, 5, 4, 4, 2, 2, 1, 1, 0, 0, 7, binding.F16) == -2
    assert conv(2, 5, 4, 4, 2, 2, 1, 1, 0, 0, binding.NCHW, 1) == -5
    assert L.shflbw_bind_device(A._h, None, None) == -1
    assert L.shflbw_bind_device(A._h, ctypes.c_void_p(8), None) == -2           # misaligned
    assert L.shflbw_set_tuning(A._h, 5, 0) == -9 and L.shflbw_set_tuning(A._h, 0, 100) == -9
    assert L.shflbw_set_tuning(A._h, 1, 64) == 0
    assert L.shflbw_device_status(None, None) == -1 and L.shflbw_device_status(A._h, None) == -6
    assert L.shflbw_set_wait_limit(A._h, -1) == -9 and L.shflbw_set_wait_limit(A._h, 1000) == 0
    assert binding.lib().shflbw_status_string(-10) == b"a bounded wait of a kernel ran out"


def test_bfloat16_weights_round_trip_bitwise():
    """bfloat16 weights travel as 16-bit patterns: same packing, same test hooks."""
    p = synth.make_spmm(128, 200, 4, 32, 0.7, seed=9, fmt="bf16")
    A = binding.compress(p.W, p.mask, p.perm, 32)
    assert A.bf16
    want = np.where(p.mask != 0, p.W, np.uint16(0))
    got = A.decompress()
    assert got.dtype == np.uint16 and np.array_equal(got, want)
    # NULL mask: a vector is kept iff any weight is non-zero; -0 (0x8000) counts as zero
    W = want.copy()
    W[p.perm[:32], 5] = 0x8000
    W[p.perm[:32], 6] = 0
    B = binding.compress(W, None, p.perm, 32)
    cols = B.group_columns(0)
    assert 5 not in cols and 6 not in cols


def test_probe_library_loads_and_exports_its_entry_point():
    """The benchmark's L2 streaming probe is a library of its own (no compute call here)."""
    import ctypes
    import os
    import bench
    lib = ctypes.CDLL(bench.PROBE_LIB if os.path.exists(bench.PROBE_LIB) else bench.build_probe())
    assert hasattr(lib, "shflbw_probe_l2_stream")
