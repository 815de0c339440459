"""Seeded cases for the host-only part of the library, run by
test_host_sanitizers.py in a child process whose library was compiled with
AddressSanitizer and UndefinedBehaviorSanitizer (the sanitizer runtime is
preloaded into that process).  Usage: python host_sanitizer_cases.py LIBRARY.

Every case checks its result as well (round trip bit for bit, valid
permutation, conforming mask), so a run that ends with "ok" has both clean
memory accesses and right answers."""
import ctypes
import sys

import numpy as np


def main(path):
    L = ctypes.CDLL(path)
    vp, i32 = ctypes.c_void_p, ctypes.c_int
    L.shflbw_compress.restype = i32
    L.shflbw_compress.argtypes = [vp, i32, vp, vp, i32, i32, i32, i32, ctypes.POINTER(vp)]
    L.shflbw_destroy.argtypes = [vp]
    L.shflbw_decompress.restype = i32
    L.shflbw_decompress.argtypes = [vp, vp, i32]
    L.shflbw_group_columns.restype = i32
    L.shflbw_group_columns.argtypes = [vp, i32, vp, i32]
    L.shflbw_row_indices.restype = i32
    L.shflbw_row_indices.argtypes = [vp, vp]
    L.shflbw_device_bytes.restype = ctypes.c_size_t
    L.shflbw_device_bytes.argtypes = [vp]
    L.shflbw_pattern_search.restype = i32
    L.shflbw_pattern_search.argtypes = [vp, i32, i32, i32, i32, ctypes.c_double, ctypes.c_double, i32, i32, vp, vp]
    ptr = lambda a: None if a is None else ctypes.c_void_p(a.ctypes.data)

    def make_mask(rng, kind, M, K, V, perm):
        mask = np.zeros((M, K), dtype=np.uint8)
        for g in range(M // V):
            if kind == "banded":          # a band of consecutive columns that moves with the group
                lo = (g * 37) % K
                cols = np.arange(lo, min(K, lo + max(1, K // 5)))
            elif kind == "empty_groups" and g % 2 == 0:
                cols = np.zeros(0, dtype=np.int64)
            elif kind == "two_bands":     # far-apart bands: the windowed layout must bridge them
                cols = np.concatenate([np.arange(0, min(K, 5)), np.arange(max(0, K - 7), K)])
                cols = np.unique(cols)
            else:
                kg = int(rng.integers(0, K + 1))
                cols = np.sort(rng.choice(K, kg, replace=False)) if kg else np.zeros(0, dtype=np.int64)
            mask[np.ix_(perm[g * V:(g + 1) * V], cols)] = 1
        return mask

    rng = np.random.Generator(np.random.PCG64(20220305))
    n_round_trips = 0
    kinds = ("random", "banded", "empty_groups", "two_bands", "full")
    for case in range(320):
        V = int(rng.choice([16, 32, 64, 128]))
        G = int(rng.integers(1, 5))
        M = G * V
        K = 1 if case % 40 == 0 else int(rng.choice([2, 7, 16, 31, 64, 100, 257, 700, 2100]))
        pad = int(rng.integers(0, 3))
        bf16 = bool(case % 3 == 0)
        Wfull = rng.integers(0, 1 << 16, size=(M, K + pad)).astype(np.uint16)   # any bit pattern, NaNs included
        perm = rng.permutation(M).astype(np.int32)
        kind = kinds[case % len(kinds)]
        mask = np.ones((M, K), dtype=np.uint8) if kind == "full" else make_mask(rng, kind, M, K, V, perm)
        h = vp()
        rc = L.shflbw_compress(ptr(Wfull), K + pad, ptr(mask), ptr(perm), M, K, V, 1 if bf16 else 0, ctypes.byref(h))
        assert rc == 0, (case, rc)
        out = np.full((M, K + 1), 0xABCD, dtype=np.uint16)
        assert L.shflbw_decompress(h, ptr(out), K + 1) == 0
        assert np.array_equal(out[:, :K], np.where(mask != 0, Wfull[:, :K], 0)), case
        assert np.all(out[:, K] == 0xABCD)
        rows = np.empty(M, dtype=np.int32)
        assert L.shflbw_row_indices(h, ptr(rows)) == 0 and np.array_equal(rows, perm)
        for g in range(G):
            n = L.shflbw_group_columns(h, g, None, 0)
            cols = np.empty(max(n, 1), dtype=np.int32)
            assert L.shflbw_group_columns(h, g, ptr(cols), n) == n
            assert np.array_equal(cols[:n], np.flatnonzero(mask[perm[g * V]])), (case, g)
        assert L.shflbw_device_bytes(h) % 256 == 0
        L.shflbw_destroy(h)
        n_round_trips += 1
        # a mask that breaks the pattern in one place must be refused (and nothing leaked)
        if M > V or K > 1:
            bad = mask.copy()
            r, k = int(rng.integers(0, M)), int(rng.integers(0, K))
            bad[r, k] ^= 1
            h = vp()
            rc = L.shflbw_compress(ptr(Wfull), K + pad, ptr(bad), ptr(perm), M, K, V, 0, ctypes.byref(h))
            assert rc == -4 or V == 1, (case, rc)
    # mask == NULL: a vector is kept iff any of its weights is non-zero
    for case in range(20):
        V, M, K = 16, 48, int(rng.integers(1, 90))
        W = (rng.integers(-2, 3, size=(M, K)) * (rng.random((M, K)) < 0.1)).astype(np.float16)
        h = vp()
        assert L.shflbw_compress(ptr(W), K, None, None, M, K, V, 0, ctypes.byref(h)) == 0
        out = np.empty((M, K), dtype=np.float16)
        assert L.shflbw_decompress(h, ptr(out), K) == 0 and np.array_equal(out, W)
        L.shflbw_destroy(h)
        n_round_trips += 1

    n_search = 0
    for case in range(60):
        V = int(rng.choice([16, 32, 64]))
        G = int(rng.integers(1, 5))
        M, K = G * V, (1 if case % 15 == 0 else int(rng.integers(2, 120)))
        bf16 = bool(case % 2)
        Wf = rng.standard_normal((M, K)).astype(np.float32)
        Wf[rng.random((M, K)) < 0.1] = 0
        if bf16:
            W = (Wf.view(np.uint32) >> 16).astype(np.uint16)
        else:
            W = Wf.astype(np.float16).view(np.uint16)
        alpha = float(rng.choice([0.0, 0.1, 0.25, 0.5, 1.0]))
        its = int(rng.integers(0, 5))
        perm = np.empty(M, dtype=np.int32)
        mask = np.empty((M, K), dtype=np.uint8)
        rc = L.shflbw_pattern_search(ptr(W), K, M, K, V, alpha, -1.0, its, 1 if bf16 else 0, ptr(perm), ptr(mask))
        assert rc == 0, (case, rc)
        assert sorted(perm.tolist()) == list(range(M))
        kg = int(np.floor(alpha * K + 0.5))
        for g in range(G):
            rows = perm[g * V:(g + 1) * V]
            assert np.all(mask[rows] == mask[rows[0]]) and int(mask[rows[0]].sum()) == kg, (case, g)
        h = vp()
        assert L.shflbw_compress(ptr(W), K, ptr(mask), ptr(perm), M, K, V, 1 if bf16 else 0, ctypes.byref(h)) == 0
        L.shflbw_destroy(h)
        n_search += 1
    print("ok: %d compress/decompress round trips, %d searches" % (n_round_trips, n_search))


if __name__ == "__main__":
    main(sys.argv[1])
