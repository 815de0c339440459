"""Pins for the CPU oracle (no GPU).  Each test fixes the oracle to something
other than itself: brute force written separately, exact integer arithmetic,
a library routine on a special case, a closed form, or an invariant the
paper states (row shuffling of W equals row shuffling of the output,
Section 4.2; Shfl-BW with the identity permutation is vector-wise,
Section 3.1).  The paper prints no worked numeric example for this path
(its examples sit in figures), so none of the pins is a printed value.
"""
import itertools

import numpy as np
import pytest
import torch

from oracle import c_oracle, definition
from paper_2203_05016_amd import synth
from conftest import assert_within_scaled_tolerance


# ----------------------------------------------------------------- half decode
def test_half_decode_all_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([c_oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_half_decode_closed_forms():
    assert c_oracle.half_to_double(0x3C00) == 1.0
    assert c_oracle.half_to_double(0xC000) == -2.0
    assert c_oracle.half_to_double(0x0001) == 2.0 ** -24       # smallest subnormal
    assert c_oracle.half_to_double(0x0400) == 2.0 ** -14       # smallest normal
    assert c_oracle.half_to_double(0x7BFF) == 65504.0          # largest finite
    assert c_oracle.half_to_double(0x7C00) == float("inf")


# ----------------------------------------------------------------- SpMM value
def _brute_spmm(W, mask, X):
    """Triple loop in Python floats, written apart from the oracle."""
    M, K = W.shape
    N = X.shape[1]
    Y = [[0.0] * N for _ in range(M)]
    S = [[0.0] * N for _ in range(M)]
    for i in range(M):
        for j in range(N):
            acc, sc = 0.0, 0.0
            for k in range(K):
                if mask[i, k]:
                    acc += float(W[i, k]) * float(X[k, j])
                    sc += abs(float(W[i, k])) * abs(float(X[k, j]))
            Y[i][j], S[i][j] = acc, sc
    return np.array(Y), np.array(S)


@pytest.mark.parametrize("M,K,N,V,sp", [(4, 6, 3, 2, 0.5), (8, 5, 7, 4, 0.4), (6, 9, 1, 3, 0.0)])
def test_spmm_brute_force_tiny(M, K, N, V, sp):
    p = synth.make_spmm(M, K, N, V, sp, seed=11)
    Yb, Sb = _brute_spmm(p.W, p.mask, p.X)
    for Y, S in (c_oracle.spmm(p.W, p.mask, p.X), definition.spmm(p.W, p.mask, p.X)):
        np.testing.assert_allclose(Y, Yb, rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(S, Sb, rtol=1e-13, atol=1e-13)


def test_spmm_empty_group_gives_zero_rows():
    p = synth.make_spmm(8, 10, 5, 4, 0.5, seed=3)
    rows = p.perm[4:8]
    p.mask[rows] = 0
    Y, S = c_oracle.spmm(p.W, p.mask, p.X)
    assert np.all(Y[rows] == 0) and np.all(S[rows] == 0)
    assert np.any(Y[p.perm[0:4]] != 0)


def test_spmm_integer_inputs_are_exact():
    """Small-integer inputs make every product and sum exact: the oracle must
    equal integer arithmetic bit for bit."""
    p = synth.make_spmm(64, 96, 40, 16, 0.5, seed=5, integer=True)
    Wi = p.W.astype(np.int64) * p.mask.astype(np.int64)
    want = Wi @ p.X.astype(np.int64)
    want_s = np.abs(Wi) @ np.abs(p.X.astype(np.int64))
    for Y, S in (c_oracle.spmm(p.W, p.mask, p.X), definition.spmm(p.W, p.mask, p.X)):
        assert np.array_equal(Y, want.astype(np.float64))
        assert np.array_equal(S, want_s.astype(np.float64))


def test_spmm_dense_identity_is_matmul():
    """Sparsity 0 with the identity permutation is a dense GEMM."""
    p = synth.make_spmm(96, 80, 33, 32, 0.0, seed=7, identity_perm=True)
    assert p.mask.all()
    want = np.matmul(p.W.astype(np.float64), p.X.astype(np.float64))
    Y, S = c_oracle.spmm(p.W, p.mask, p.X)
    np.testing.assert_allclose(Y, want, rtol=0, atol=1e-12 * np.abs(S).max())


def test_spmm_c_and_definition_agree_midsize():
    p = synth.make_spmm(256, 256, 64, 32, 0.75, seed=synth.BASE_SEED)
    Yc, Sc = c_oracle.spmm(p.W, p.mask, p.X)
    Yd, Sd = definition.spmm(p.W, p.mask, p.X)
    assert_within_scaled_tolerance(Yc, Yd, Sd, tol=1e-13, what="C vs numpy definition")
    np.testing.assert_allclose(Sc, Sd, rtol=1e-13)


def test_spmm_unit_vectors_pick_masked_columns():
    """X = identity gives Y = W . mask: catches a transposed operand or a
    wrong column index."""
    p = synth.make_spmm(32, 24, 24, 8, 0.5, seed=9)
    X = np.eye(24, dtype=np.float16)
    Y, _ = c_oracle.spmm(p.W, p.mask, X)
    assert np.array_equal(Y, p.W.astype(np.float64) * p.mask)


def test_spmm_ones_weights_sum_selected_rows():
    p = synth.make_spmm(16, 20, 6, 4, 0.5, seed=10)
    W = np.ones_like(p.W)
    Y, _ = c_oracle.spmm(W, p.mask, p.X)
    for g, c in enumerate(p.cols):
        want = p.X[c].astype(np.float64).sum(axis=0)
        for r in p.perm[g * 4:(g + 1) * 4]:
            np.testing.assert_allclose(Y[r], want, rtol=1e-14, atol=1e-14)


def test_scale_equals_value_for_nonnegative_inputs():
    p = synth.make_spmm(32, 48, 10, 8, 0.5, seed=12)
    W, X = np.abs(p.W), np.abs(p.X)
    Y, S = c_oracle.spmm(W, p.mask, X)
    assert np.array_equal(Y, S)


# --------------------------------------------------------- permutation / pattern
def test_row_shuffle_of_weights_is_row_shuffle_of_output():
    p = synth.make_spmm(64, 40, 12, 16, 0.5, seed=13)
    q = np.random.Generator(np.random.PCG64(99)).permutation(64)
    Y, S = c_oracle.spmm(p.W, p.mask, p.X)
    Yq, Sq = c_oracle.spmm(p.W[q], p.mask[q], p.X)
    assert np.array_equal(Yq, Y[q]) and np.array_equal(Sq, S[q])


def test_vectorwise_form_reproduces_product_with_non_involutive_perm():
    """The stitched per-group dense product plus reordered write-back equals
    the masked product; a permutation that is not its own inverse makes a
    swapped direction fail."""
    p = synth.make_spmm(48, 30, 9, 8, 0.6, seed=14)
    inv = np.empty_like(p.perm)
    inv[p.perm] = np.arange(48)
    assert not np.array_equal(inv, p.perm)
    ri, cols, vecs = definition.vectorwise_form(p.W, p.mask, p.perm, 8)
    Y = definition.spmm_from_vectorwise(ri, cols, vecs, p.X, 48)
    Yc, Sc = c_oracle.spmm(p.W, p.mask, p.X)
    assert_within_scaled_tolerance(Y, Yc, Sc, tol=1e-13, what="vector-wise form")
    # wrong direction must NOT reproduce it
    Ybad = definition.spmm_from_vectorwise(inv, cols, vecs, p.X, 48)
    assert not np.allclose(Ybad, Yc)
    for g, c in enumerate(cols):
        assert np.array_equal(c, p.cols[g])
        assert np.all(np.diff(c) > 0)


def test_identity_perm_is_vectorwise():
    p = synth.make_spmm(32, 20, 4, 8, 0.5, seed=15, identity_perm=True)
    for g in range(4):
        blk = p.mask[g * 8:(g + 1) * 8]
        assert np.all(blk == blk[0])
    assert definition.check_pattern(p.mask, None, 8) is None


def test_check_pattern_reports_first_violation():
    p = synth.make_spmm(32, 20, 4, 8, 0.5, seed=16)
    assert definition.check_pattern(p.mask, p.perm, 8) is None
    bad = p.mask.copy()
    row = p.perm[8 + 3]
    col = int(np.nonzero(bad[row] == 0)[0][0])
    bad[row, col] = 1
    g, srow, c = definition.check_pattern(bad, p.perm, 8)
    assert (g, srow, c) == (1, 11, col)
    with pytest.raises(ValueError):
        definition.check_pattern(p.mask, np.zeros(32, dtype=np.int32), 8)


def test_scatter_rows_direction():
    tiles = np.arange(12.0).reshape(4, 3)
    out = definition.scatter_rows(tiles, [2, 0, 3, 1])
    assert np.array_equal(out[2], tiles[0]) and np.array_equal(out[1], tiles[3])


def test_generator_properties():
    p = synth.config(0)
    assert (p.M, p.K, p.N, p.V) == (256, 256, 64, 32)
    assert p.nnz == 256 * 64 and p.mask.sum() == p.nnz
    assert sorted(p.perm.tolist()) == list(range(256))
    assert not np.array_equal(p.perm, np.arange(256))
    assert np.count_nonzero(p.W) > 0.99 * p.W.size          # W left dense
    p2 = synth.config(0)
    assert np.array_equal(p.W, p2.W) and np.array_equal(p.mask, p2.mask)
    assert synth.kept_per_group(1024, 0.9) == 102 and synth.kept_per_group(8192, 0.95) == 410


# ----------------------------------------------------------------- convolution
def _brute_conv(Wt, mask, inp, R, S, stride, pad):
    B, C, H, Wd = inp.shape
    Cout = Wt.shape[0]
    sh, sw = stride
    ph, pw = pad
    Ho, Wo = (H + 2 * ph - R) // sh + 1, (Wd + 2 * pw - S) // sw + 1
    out = np.zeros((B, Cout, Ho, Wo))
    for b, o, y, x in itertools.product(range(B), range(Cout), range(Ho), range(Wo)):
        acc = 0.0
        for c, r, s in itertools.product(range(C), range(R), range(S)):
            iy, ix = y * sh + r - ph, x * sw + s - pw
            if 0 <= iy < H and 0 <= ix < Wd and mask[o, (c * R + r) * S + s]:
                acc += float(Wt[o, (c * R + r) * S + s]) * float(inp[b, c, iy, ix])
        out[b, o, y, x] = acc
    return out


@pytest.mark.parametrize("stride,pad", [((1, 1), (1, 1)), ((2, 1), (0, 2)), ((2, 2), (1, 0))])
def test_conv_brute_force_tiny(stride, pad):
    p = synth.make_conv(2, 3, 5, 6, 4, 3, 2, 2, 0.5, seed=21, stride=stride, pad=pad)
    g = p.conv
    want = _brute_conv(p.W, p.mask, g["input"], 3, 2, stride, pad)
    got, _ = c_oracle.conv2d(p.W, p.mask, g["input"], 3, 2, stride, pad)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)
    got2, _ = definition.conv2d(p.W, p.mask, g["input"], 3, 2, stride, pad)
    np.testing.assert_allclose(got2, want, rtol=1e-13, atol=1e-13)


def test_conv_matches_library_conv2d_float64():
    p = synth.make_conv(3, 8, 9, 7, 16, 3, 3, 4, 0.5, seed=22, stride=(2, 1), pad=(1, 1))
    g = p.conv
    w = torch.from_numpy((p.W.astype(np.float64) * p.mask).reshape(16, 8, 3, 3))
    x = torch.from_numpy(g["input"].astype(np.float64))
    want = torch.nn.functional.conv2d(x, w, stride=(2, 1), padding=(1, 1)).numpy()
    got, sc = c_oracle.conv2d(p.W, p.mask, g["input"], 3, 3, (2, 1), (1, 1))
    assert got.shape == want.shape == (3, 16, 5, 7)
    assert_within_scaled_tolerance(got, want, sc, tol=1e-13, what="C conv vs torch f64")


def test_conv_1x1_is_spmm_on_reshaped_input():
    p = synth.make_conv(4, 12, 5, 5, 8, 1, 1, 4, 0.5, seed=23)
    inp = p.conv["input"]
    X = np.ascontiguousarray(inp.transpose(1, 0, 2, 3).reshape(12, 4 * 25))
    Y, _ = c_oracle.spmm(p.W, p.mask, X)
    got, _ = c_oracle.conv2d(p.W, p.mask, inp, 1, 1)
    assert np.array_equal(got, Y.reshape(8, 4, 5, 5).transpose(1, 0, 2, 3))


def test_conv_delta_kernel_shifts_image_without_flip():
    """A single tap at (r, s) = (0, 2) of a 3x3 kernel with pad 1 reads the
    input one row up and one column right: out[y, x] = in[y-1, x+1]."""
    inp = np.arange(1, 21, dtype=np.float16).reshape(1, 1, 4, 5)
    Wt = np.zeros((1, 9), dtype=np.float16)
    Wt[0, 0 * 3 + 2] = 1
    mask = (Wt != 0).astype(np.uint8)
    got, _ = c_oracle.conv2d(Wt, mask, inp, 3, 3, (1, 1), (1, 1))
    want = np.zeros((4, 5))
    want[1:, :4] = inp[0, 0, :3, 1:]
    assert np.array_equal(got[0, 0], want)
    got2, _ = definition.conv2d(Wt, mask, inp, 3, 3, (1, 1), (1, 1))
    assert np.array_equal(got2[0, 0], want)


def test_conv_chwn_layout_is_a_transpose_of_nchw():
    p = synth.make_conv(3, 4, 6, 5, 8, 3, 3, 4, 0.5, seed=24, pad=(1, 1))
    inp = p.conv["input"]
    a, sa = c_oracle.conv2d(p.W, p.mask, inp, 3, 3, (1, 1), (1, 1), layout="NCHW")
    inp_t = np.ascontiguousarray(inp.transpose(1, 2, 3, 0))
    b, sb = c_oracle.conv2d(p.W, p.mask, inp_t, 3, 3, (1, 1), (1, 1), layout="CHWN")
    assert np.array_equal(b, a.transpose(1, 2, 3, 0))
    assert np.array_equal(sb, sa.transpose(1, 2, 3, 0))
    c, _ = definition.conv2d(p.W, p.mask, inp_t, 3, 3, (1, 1), (1, 1), layout="CHWN")
    np.testing.assert_allclose(c, b, rtol=1e-13, atol=1e-13)


def test_conv_integer_exact_midsize():
    p = synth.make_conv(2, 16, 7, 7, 32, 3, 3, 16, 0.75, seed=25, pad=(1, 1), integer=True)
    inp = p.conv["input"]
    got, _ = c_oracle.conv2d(p.W, p.mask, inp, 3, 3, (1, 1), (1, 1))
    w = torch.from_numpy((p.W.astype(np.int64) * p.mask).reshape(32, 16, 3, 3).astype(np.float64))
    want = torch.nn.functional.conv2d(torch.from_numpy(inp.astype(np.float64)), w, padding=1).numpy()
    assert np.array_equal(got, want)


# ----------------------------------------------------------------- bfloat16 operands
def _bf16_to_f64_by_torch(bits):
    """bfloat16 bit patterns widened by the library's own conversion."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).double().numpy()


def test_bfloat16_decode_all_patterns_match_library():
    bits = np.arange(65536, dtype=np.uint16)
    want = _bf16_to_f64_by_torch(bits)
    got = np.array([c_oracle.bfloat16_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_bfloat16_decode_closed_forms():
    assert c_oracle.bfloat16_to_double(0x3F80) == 1.0
    assert c_oracle.bfloat16_to_double(0xC000) == -2.0
    assert c_oracle.bfloat16_to_double(0x0001) == 2.0 ** -133     # smallest subnormal
    assert c_oracle.bfloat16_to_double(0x0080) == 2.0 ** -126     # smallest normal
    assert c_oracle.bfloat16_to_double(0x7F7F) == (2.0 - 2.0 ** -7) * 2.0 ** 127
    assert c_oracle.bfloat16_to_double(0x7F80) == float("inf")


def test_spmm_bfloat16_brute_force_and_definition():
    p = synth.make_spmm(8, 10, 5, 4, 0.4, seed=31, fmt="bf16")
    Wf, Xf = _bf16_to_f64_by_torch(p.W), _bf16_to_f64_by_torch(p.X)
    Y, S = c_oracle.spmm(p.W, p.mask, p.X)
    Yb, Sb = _brute_spmm(Wf, p.mask, Xf)
    assert np.allclose(Y, Yb, rtol=1e-13, atol=0) and np.allclose(S, Sb, rtol=1e-13, atol=0)
    q = synth.make_spmm(96, 80, 33, 32, 0.5, seed=32, fmt="bf16")
    Y, S = c_oracle.spmm(q.W, q.mask, q.X)
    Yd, Sd = definition.spmm(_bf16_to_f64_by_torch(q.W), q.mask, _bf16_to_f64_by_torch(q.X))
    assert np.allclose(Y, Yd, rtol=1e-12, atol=1e-12) and np.allclose(S, Sd, rtol=1e-12, atol=1e-12)


def test_spmm_bfloat16_integer_inputs_equal_the_binary16_result():
    """Small integers are exact in both formats, so the two formats' oracles
    must give the same numbers bit for bit (same seed, same draws)."""
    a = synth.make_spmm(64, 48, 20, 32, 0.5, seed=33, integer=True)
    b = synth.make_spmm(64, 48, 20, 32, 0.5, seed=33, integer=True, fmt="bf16")
    assert np.array_equal(a.mask, b.mask)
    Ya, _ = c_oracle.spmm(a.W, a.mask, a.X)
    Yb, _ = c_oracle.spmm(b.W, b.mask, b.X)
    assert np.array_equal(Ya, Yb)


def test_conv_bfloat16_matches_library_conv2d_float64():
    p = synth.make_conv(2, 6, 7, 5, 8, 3, 3, 4, 0.5, seed=34, stride=(2, 1), pad=(1, 1), fmt="bf16")
    g = p.conv
    got, _ = c_oracle.conv2d(p.W, p.mask, g["input"], 3, 3, (2, 1), (1, 1))
    Wm = torch.from_numpy(_bf16_to_f64_by_torch(p.W) * p.mask).reshape(8, 6, 3, 3)
    want = torch.nn.functional.conv2d(torch.from_numpy(_bf16_to_f64_by_torch(g["input"])), Wm,
                                      stride=(2, 1), padding=(1, 1)).numpy()
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)


def test_bfloat16_rounding_of_the_generator_matches_library():
    a = np.random.default_rng(5).standard_normal(50000).astype(np.float32)
    bits = synth.float32_to_bfloat16_bits(a)
    want = torch.from_numpy(a).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), want.view(torch.int16).numpy())


# ----------------------------------------------------------------- LayerNorm-side transposition
def test_layernorm_transpose_matches_library_layer_norm():
    rng = np.random.default_rng(41)
    x = rng.standard_normal((37, 96)).astype(np.float16)
    gamma = rng.standard_normal(96).astype(np.float16)
    beta = rng.standard_normal(96).astype(np.float16)
    got, _ = definition.layernorm_transpose(x, gamma, beta, eps=1e-5)
    want = torch.nn.functional.layer_norm(torch.from_numpy(x.astype(np.float64)), (96,),
                                          torch.from_numpy(gamma.astype(np.float64)),
                                          torch.from_numpy(beta.astype(np.float64)), 1e-5).numpy().T
    assert got.shape == (96, 37) and np.allclose(got, want, rtol=1e-12, atol=1e-12)


def test_layernorm_transpose_closed_forms_and_invariants():
    # a constant row has zero variance: the output is beta whatever the constant
    x = np.full((3, 8), 2.5)
    beta = np.arange(8.0)
    y, _ = definition.layernorm_transpose(x, np.ones(8), beta)
    assert np.allclose(y, np.tile(beta[:, None], (1, 3)))
    # two features {a, b}: x_hat = -+ 1/sqrt(1 + 4 eps/(a-b)^2)
    y, _ = definition.layernorm_transpose(np.array([[1.0, 3.0]]), eps=0.25)
    assert np.allclose(y[:, 0], [-1 / np.sqrt(1.25), 1 / np.sqrt(1.25)])
    # shifting a token by a constant changes nothing; scaling by c > 0 only through eps
    rng = np.random.default_rng(42)
    x = rng.standard_normal((5, 64))
    y0, _ = definition.layernorm_transpose(x, eps=0.0)
    y1, _ = definition.layernorm_transpose(x * 3.0 + 7.0, eps=0.0)
    assert np.allclose(y0, y1, atol=1e-12)
    # per token: zero mean and unit variance over the features when eps = 0, gamma = 1, beta = 0
    assert np.allclose(y0.mean(axis=0), 0, atol=1e-12) and np.allclose(y0.var(axis=0), 1, atol=1e-12)
    # without normalisation it is the transpose, element for element
    t, _ = definition.layernorm_transpose(x, normalize=False)
    assert np.array_equal(t, x.T)
