"""The hot path's result, written as its definition with numpy primitives in
float64 (test infrastructure only; shares nothing with the GPU path).

* ``spmm`` / ``conv2d``: the masked product the kernels reformulate
  (Section 2.1; Algorithm 1's inputs and result; Section 4.1 for the
  implicit-GEMM view of convolution).
* ``check_pattern`` / ``vectorwise_form``: the Shfl-BW pattern rule of
  Section 3.1 (after the row permutation, every group of V consecutive rows
  keeps one column set) and the offline step (a) of Section 4.1-4.2: rows
  reordered into vector-wise form, each kept V x 1 vector stored together,
  the original row indices kept in an array.
* ``scatter_rows``: the reordered write-back of Section 4.2 as an index
  assignment.

Reading of the permutation's direction (the paper says the row indices are
kept "for reversing the row order in the output"): ``perm[i]`` is the
original row of stored row ``i``; stored row ``i`` is ``W[perm[i]]`` and its
result is written to ``Y[perm[i]]``.
"""
import numpy as np


def spmm(W, mask, X):
    """Y = (W * mask) @ X and S = |W * mask| @ |X| in float64."""
    Wm = W.astype(np.float64) * (np.asarray(mask) != 0)
    Xd = X.astype(np.float64)
    return Wm @ Xd, np.abs(Wm) @ np.abs(Xd)


def unfold_nchw(inp, R, S, stride=(1, 1), pad=(0, 0)):
    """Explicit im2col of an NCHW tensor: returns U of shape
    (Cin*R*S, B*Ho*Wo) with U[(c*R+r)*S+s, (b*Ho+y)*Wo+x] =
    inp[b, c, y*sh+r-ph, x*sw+s-pw], zero outside the image."""
    B, C, H, Wd = inp.shape
    sh, sw = stride
    ph, pw = pad
    Ho = (H + 2 * ph - R) // sh + 1
    Wo = (Wd + 2 * pw - S) // sw + 1
    padded = np.zeros((B, C, H + 2 * ph, Wd + 2 * pw), dtype=inp.dtype)
    padded[:, :, ph:ph + H, pw:pw + Wd] = inp
    U = np.empty((C, R, S, B, Ho, Wo), dtype=inp.dtype)
    for r in range(R):
        for s in range(S):
            win = padded[:, :, r:r + (Ho - 1) * sh + 1:sh, s:s + (Wo - 1) * sw + 1:sw]
            U[:, r, s] = win.transpose(1, 0, 2, 3)
    return U.reshape(C * R * S, B * Ho * Wo), (B, Ho, Wo)


def conv2d(Wt, mask, inp, R, S, stride=(1, 1), pad=(0, 0), layout="NCHW"):
    """Masked conv2d as unfold followed by the masked product."""
    if layout == "CHWN":
        inp = np.ascontiguousarray(inp.transpose(3, 0, 1, 2))
    U, (B, Ho, Wo) = unfold_nchw(inp, R, S, stride, pad)
    Y, Sc = spmm(Wt, mask, U)
    Cout = Wt.shape[0]
    Y = Y.reshape(Cout, B, Ho, Wo)
    Sc = Sc.reshape(Cout, B, Ho, Wo)
    if layout == "CHWN":
        return Y.transpose(0, 2, 3, 1).copy(), Sc.transpose(0, 2, 3, 1).copy()
    return Y.transpose(1, 0, 2, 3).copy(), Sc.transpose(1, 0, 2, 3).copy()


def check_pattern(mask, perm, V):
    """None if the mask is a Shfl-BW pattern under ``perm`` with group size V,
    else (group, stored_row, column) of the first disagreement."""
    mask = np.asarray(mask) != 0
    M, K = mask.shape
    if M % V:
        raise ValueError("M must be a multiple of V")
    perm = np.arange(M) if perm is None else np.asarray(perm)
    if sorted(perm.tolist()) != list(range(M)):
        raise ValueError("perm is not a permutation")
    for g in range(M // V):
        rows = perm[g * V:(g + 1) * V]
        ref = mask[rows[0]]
        for i in range(1, V):
            diff = np.nonzero(mask[rows[i]] != ref)[0]
            if diff.size:
                return (g, g * V + i, int(diff[0]))
    return None


def vectorwise_form(W, mask, perm, V):
    """Offline step (a): (row_indices, cols, vectors) where ``cols[g]`` is the
    ascending list of kept columns of group g and ``vectors[g]`` is a
    (len(cols[g]), V) array whose row j is the kept V x 1 vector of column
    cols[g][j], in stored-row order."""
    M, K = W.shape
    perm = np.arange(M) if perm is None else np.asarray(perm)
    bad = check_pattern(mask, perm, V)
    if bad is not None:
        raise ValueError("mask is not Shfl-BW under perm: %r" % (bad,))
    mask = np.asarray(mask) != 0
    cols, vectors = [], []
    for g in range(M // V):
        rows = perm[g * V:(g + 1) * V]
        c = np.nonzero(mask[rows[0]])[0]
        cols.append(c.astype(np.int64))
        vectors.append(np.ascontiguousarray(W[np.ix_(rows, c)].T))
    return perm.astype(np.int64).copy(), cols, vectors


def spmm_from_vectorwise(row_indices, cols, vectors, X, M):
    """The product computed from the vector-wise form: per group a dense
    (V x k_g) by (k_g x N) product on the gathered rows of X (in-buffer
    stitching, Section 4.3), then the reordered write-back."""
    Xd = X.astype(np.float64)
    Y = np.zeros((M, X.shape[1]), dtype=np.float64)
    V = len(row_indices) // max(len(cols), 1)
    for g, (c, vec) in enumerate(zip(cols, vectors)):
        tile = vec.astype(np.float64).T @ Xd[c]
        Y[row_indices[g * V:(g + 1) * V]] = tile
    return Y


def scatter_rows(tiles, row_indices):
    """Reordered write-back: out[row_indices[i]] = tiles[i]."""
    out = np.empty_like(tiles)
    out[np.asarray(row_indices)] = tiles
    return out


def layernorm_transpose(x, gamma=None, beta=None, eps=1e-5, normalize=True):
    """The layout step of Section 4.3's discussion: activations that a
    LayerNorm produces feature-innermost, ``x`` of shape (N tokens, K
    features), are handed to the sparse kernels batch-innermost, i.e. as the
    (K, N) matrix.  With ``normalize`` the LayerNorm itself is applied on the
    way (per token: subtract the mean over the K features, divide by
    sqrt(biased variance + eps), times gamma plus beta); without it the result
    is the plain transpose.  float64 throughout.  Returns (Y, S) with S the
    magnitude the tolerance is stated against: |gamma| |x_hat| + |beta|."""
    xd = np.asarray(x, dtype=np.float64)
    N, K = xd.shape
    g = np.ones(K) if gamma is None else np.asarray(gamma, dtype=np.float64)
    b = np.zeros(K) if beta is None else np.asarray(beta, dtype=np.float64)
    if not normalize:
        return xd.T.copy(), np.abs(xd.T)
    mean = xd.mean(axis=1, keepdims=True)
    var = ((xd - mean) ** 2).mean(axis=1, keepdims=True)
    xhat = (xd - mean) / np.sqrt(var + eps)
    y = xhat * g[None, :] + b[None, :]
    s = np.abs(xhat) * np.abs(g)[None, :] + np.abs(b)[None, :]
    return y.T.copy(), s.T.copy()
