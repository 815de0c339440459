"""Pins for the pattern-search oracle (Section 5) and, below, the library's
search against it.  The procedure is a heuristic, so the pins are what the
paper and the construction fix: the result is a Shfl-BW pattern of the
requested density; rows that already share their supports are found; with
V = 1 or with no K-Means round it reduces to plain top-k / vector-wise
pruning written separately; on a matrix with planted groups it keeps more
total score than vector-wise pruning without the shuffle."""
import numpy as np
import pytest

from oracle import definition, pattern_search
from paper_2203_05016_amd import synth


def _planted(M, K, V, kg, seed, noise=0.05):
    """Weights whose large entries follow a hidden Shfl-BW pattern."""
    rng = np.random.Generator(np.random.PCG64(seed))
    perm = rng.permutation(M)
    W = (noise * rng.standard_normal((M, K))).astype(np.float32)
    truth = np.zeros((M, K), dtype=np.uint8)
    for g in range(M // V):
        cols = rng.choice(K, kg, replace=False)
        rows = perm[g * V:(g + 1) * V]
        W[np.ix_(rows, cols)] = (1.0 + rng.random((V, kg))) * rng.choice([-1.0, 1.0], (V, kg))
        truth[np.ix_(rows, cols)] = 1
    return W.astype(np.float16), truth, perm


def test_result_is_a_shflbw_pattern_of_the_requested_density():
    p = synth.make_spmm(64, 96, 4, 8, 0.0, seed=801)
    perm, mask = pattern_search.search(p.W, 8, alpha=0.25)
    assert sorted(perm.tolist()) == list(range(64))
    assert definition.check_pattern(mask, perm, 8) is None
    assert np.all(mask.sum(axis=1) == 24)


def test_planted_groups_are_recovered():
    W, truth, _ = _planted(48, 64, 4, 8, seed=802)
    perm, mask = pattern_search.search(W, 4, alpha=8 / 64, beta=8 / 64, iterations=10)
    assert np.array_equal(mask, truth)


def test_v1_is_per_row_top_k_and_zero_rounds_is_vectorwise_pruning():
    rng = np.random.default_rng(803)
    W = rng.standard_normal((12, 40)).astype(np.float16)
    perm, mask = pattern_search.search(W, 1, alpha=0.25, iterations=3)
    for i in range(12):
        top = np.argsort(-np.abs(W[i].astype(np.float64)), kind="stable")[:10]
        assert set(np.flatnonzero(mask[i])) == set(top.tolist())
    perm, mask = pattern_search.search(W, 4, alpha=0.25, iterations=0)
    assert np.array_equal(perm, np.arange(12))
    for g in range(3):
        score = np.abs(W[4 * g:4 * g + 4].astype(np.float64)).sum(axis=0)
        top = np.argsort(-score, kind="stable")[:10]
        assert all(set(np.flatnonzero(mask[4 * g + i])) == set(top.tolist()) for i in range(4))


def test_shuffle_keeps_more_score_than_plain_vectorwise_on_planted_groups():
    W, _, _ = _planted(64, 128, 8, 16, seed=804, noise=0.2)
    mag = np.abs(W.astype(np.float64))
    _, m_shuffled = pattern_search.search(W, 8, alpha=0.125, iterations=10)
    _, m_plain = pattern_search.search(W, 8, alpha=0.125, iterations=0)
    assert (mag * m_shuffled).sum() > 1.5 * (mag * m_plain).sum()


def test_kmeans_keeps_every_cluster_at_v_rows_and_is_deterministic():
    rng = np.random.default_rng(805)
    B = (rng.random((40, 30)) < 0.3).astype(np.int64)
    a = pattern_search.balanced_kmeans(B, 5, 6)
    assert np.array_equal(np.bincount(a, minlength=8), np.full(8, 5))
    assert np.array_equal(a, pattern_search.balanced_kmeans(B.copy(), 5, 6))


# ----------------------------------------------------------------- the library against the oracle
from paper_2203_05016_amd import binding


@pytest.mark.parametrize("M,K,V,alpha,beta,its", [
    (64, 96, 8, 0.25, None, 10), (48, 64, 4, 0.125, 0.125, 10), (128, 200, 32, 0.1, None, 4),
    (32, 40, 16, 0.5, 1.0, 3), (12, 40, 1, 0.25, None, 3), (12, 40, 4, 0.25, None, 0),
    (64, 72, 8, 0.0, None, 2), (64, 72, 8, 1.0, None, 2),
])
def test_library_search_equals_the_oracle_bit_for_bit(M, K, V, alpha, beta, its):
    rng = np.random.Generator(np.random.PCG64(810 + M + K + V))
    W = rng.standard_normal((M, K), dtype=np.float32).astype(np.float16)
    W[rng.random((M, K)) < 0.05] = 0            # ties among zeros
    W[0, :5] = W[1, :5]                          # ties among equal magnitudes
    perm, mask = binding.pattern_search(W, V, alpha, beta, its)
    perm_o, mask_o = pattern_search.search(W, V, alpha, beta, its)
    assert np.array_equal(perm, perm_o)
    assert np.array_equal(mask, mask_o)


def test_library_search_on_planted_groups_and_into_compress():
    W, truth, _ = _planted(96, 128, 8, 16, seed=811)
    perm, mask = binding.pattern_search(W, 8, 16 / 128, 16 / 128, 10)
    assert np.array_equal(mask, truth)
    W2, truth2, _ = _planted(128, 160, 16, 24, seed=812)
    perm2, mask2 = binding.pattern_search(W2, 16, 24 / 160, 24 / 160, 10)
    assert np.array_equal(mask2, truth2)
    A = binding.compress(W2, mask2, perm2, 16)
    assert A.info()["nnz"] == int(truth2.sum())
    assert np.array_equal(A.decompress().view(np.uint16), np.where(truth2 != 0, W2, np.float16(0)).view(np.uint16))


def test_library_search_argument_checks():
    W = np.zeros((8, 8), dtype=np.float16)
    with pytest.raises(binding.ShflbwError):
        binding.pattern_search(W, 3, 0.5)               # M % V != 0
    with pytest.raises(binding.ShflbwError):
        binding.pattern_search(W, 4, 1.5)               # alpha outside [0, 1]
    W[0, 0] = np.inf
    with pytest.raises(binding.ShflbwError):
        binding.pattern_search(W, 4, 0.5)               # non-finite weight
