"""Pattern search for the Shfl-BW pattern (Section 5), written out step by
step in numpy integer arithmetic.  TEST INFRASTRUCTURE ONLY: it shares no
code with the library's own search and is imported by tests alone.

The paper's procedure, in its order:

1. the importance score of a weight is its absolute value;
2. unstructured pruning of the score matrix to the non-zero ratio beta
   (the paper finds beta = 2 alpha to work best) gives a binary mask;
3. K-Means on the rows of that binary mask, with clusters of the fixed size
   V, decides which rows are put together (the row shuffle);
4. the rows are permuted so that each cluster is one group of V rows;
5. ordinary vector-wise pruning to the target non-zero ratio alpha on the
   permuted matrix: a V x 1 vector's score is the sum of its scores;
6. the permutation is undone: the mask is returned in the original row order
   together with the permutation.

Readings where the paper is silent (the library takes the same ones, so that
the two can be compared bit for bit):

* scores are compared as the 15 magnitude bits of the 16-bit pattern
  (monotone in |w| for binary16 and for bfloat16 alike); ties go to the lower
  flat index; step 2 keeps round(beta M K) weights, halves rounded up;
* fixed-size K-Means: clusters start as the consecutive blocks of V rows; one
  iteration computes every cluster's centre (mean of its rows of the binary
  mask) and re-assigns greedily, going through all (row, cluster) pairs by
  increasing squared distance (ties: lower row, then lower cluster) and
  taking a pair when the row is still free and the cluster not full; it
  stops after `iterations` rounds or when nothing moves.  Distances are
  compared exactly, as integers: V^2 |b_r - c|^2 = sum_k (V b_rk - n_ck)^2
  with n_ck the number of ones of cluster c in column k;
* step 5 keeps the same number round(alpha K) of vectors in every group (the
  largest sums; ties to the lower column); a vector's sum is taken exactly,
  as an integer (units of 2^-24 for binary16, of 2^-133 for bfloat16);
  the other fair reading of "vector-wise pruning to the ratio alpha" - one
  threshold over all groups' vectors, so that groups keep different numbers -
  is not taken: equal counts keep every group's work equal on the GPU;
* perm[i] is the original row of stored row i; rows of a cluster keep their
  original order.

Weights are float16 arrays, or uint16 arrays holding bfloat16 bit patterns
(numpy has no such type).

Parity status: pinned by tests/test_pattern_search.py (planted groups recovered
exactly; V = 1 and zero rounds reduce to top-k and plain vector-wise pruning
written separately; the unstructured step's count, threshold and tie rule
checked directly; a four-row K-Means case worked by hand; bfloat16 sums
against exact rational arithmetic).
"""
import math

import numpy as np


def round_half_up(x):
    """Nearest integer of a non-negative number, halves upwards."""
    return int(math.floor(x + 0.5))


def _bits(W):
    W = np.ascontiguousarray(W)
    if W.dtype == np.float16:
        return W.view(np.uint16), False
    if W.dtype == np.uint16:
        return W, True
    raise TypeError("weights must be float16, or uint16 holding bfloat16 bits")


def magnitude_key(W):
    """Sort key monotone in |w|: the 15 bits below the sign."""
    return (_bits(W)[0] & 0x7FFF).astype(np.int64)


def exact_magnitude(W):
    """|w| as exact integers: in units of 2^-24 (binary16; int64 array) or of
    2^-133 (bfloat16; array of Python integers, which do not overflow)."""
    bits, bf = _bits(W)
    if not bf:
        a = np.abs(bits.view(np.float16).astype(np.float64)) * float(1 << 24)
        if not np.all(np.isfinite(a)):
            raise ValueError("pattern search needs finite weights")
        out = a.astype(np.int64)
        assert np.array_equal(out.astype(np.float64), a)
        return out
    e = ((bits >> 7) & 255).astype(np.int64)
    f = (bits & 127).astype(np.int64)
    if np.any(e == 255):
        raise ValueError("pattern search needs finite weights")
    out = np.empty(bits.shape, dtype=object)
    for idx in np.ndindex(bits.shape):
        # subnormal: f * 2^-133; normal: (128 + f) * 2^(e - 127 - 7)
        out[idx] = int(f[idx]) if e[idx] == 0 else (128 + int(f[idx])) << (int(e[idx]) - 1)
    return out


def unstructured_mask(W, beta):
    M, K = W.shape
    keep = round_half_up(beta * (M * K))
    keep = max(0, min(M * K, keep))
    key = magnitude_key(W).reshape(-1)
    order = np.lexsort((np.arange(key.size), -key))       # key descending, index ascending
    B = np.zeros(M * K, dtype=np.int64)
    B[order[:keep]] = 1
    return B.reshape(M, K)


def balanced_kmeans(B, V, iterations):
    """Cluster id of every row; every cluster has exactly V rows."""
    M, K = B.shape
    G = M // V
    assign = np.arange(M) // V
    for _ in range(iterations):
        counts = np.zeros((G, K), dtype=np.int64)
        np.add.at(counts, assign, B)
        # V^2 |b_r - c|^2 = V^2 |b_r|^2 - 2 V b_r . n_c + |n_c|^2   (b is 0/1, so |b_r|^2 = sum b_r)
        d = (V * V) * B.sum(axis=1)[:, None] - 2 * V * (B @ counts.T) + (counts * counts).sum(axis=1)[None, :]
        rows = np.repeat(np.arange(M), G)
        clus = np.tile(np.arange(G), M)
        order = np.lexsort((clus, rows, d.reshape(-1)))
        new = np.full(M, -1, dtype=np.int64)
        room = np.full(G, V, dtype=np.int64)
        left = M
        for idx in order:
            r, c = rows[idx], clus[idx]
            if new[r] < 0 and room[c] > 0:
                new[r] = c
                room[c] -= 1
                left -= 1
                if left == 0:
                    break
        if np.array_equal(new, assign):
            break
        assign = new
    return assign


def search(W, V, alpha, beta=None, iterations=10):
    """(perm, mask) for weights W (M x K): float16, or uint16 bfloat16 bits."""
    bits, bf = _bits(W)
    W = bits if bf else bits.view(np.float16)
    M, K = W.shape
    if M % V:
        raise ValueError("M % V != 0")
    beta = min(1.0, 2.0 * alpha) if beta is None else beta
    B = unstructured_mask(W, beta)
    assign = balanced_kmeans(B, V, iterations)
    perm = np.lexsort((np.arange(M), assign)).astype(np.int32)     # by cluster, then original row
    mag = exact_magnitude(W)
    kg = round_half_up(alpha * K)
    kg = max(0, min(K, kg))
    mask = np.zeros((M, K), dtype=np.uint8)
    for g in range(M // V):
        rows = perm[g * V:(g + 1) * V]
        vs = mag[rows].sum(axis=0)
        # largest sum first, ties to the lower column (sorted() is stable and exact on integers)
        order = sorted(range(K), key=lambda k: -int(vs[k]))
        mask[np.ix_(rows, order[:kg])] = 1
    return perm, mask
