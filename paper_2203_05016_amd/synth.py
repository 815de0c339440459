"""Seeded synthetic inputs for the Shfl-BW hot path.

This module holds no arithmetic of the method: it only draws random weights,
activations, a row permutation and a Shfl-BW-conforming mask.  It serves the
tests, the oracle side and the benchmark alike.

Recipe.  ``numpy.random.Generator(PCG64(seed))``; draw order is fixed:
W (float32 N(0,1) rounded to float16, left DENSE so that a kernel ignoring
the mask fails parity), then the activations (same distribution), then
``perm = rng.permutation(M)`` (``perm[i]`` = original row of stored row i),
then for each group g in order a sorted uniform sample of ``k_g`` distinct
columns.  ``mask[perm[g*V + i], cols_g] = 1``.
"""
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20220305


def kept_per_group(K, sparsity):
    """Columns kept in each row group for a nominal sparsity (rounded)."""
    return int(round(K * (1.0 - float(sparsity))))


def float32_to_bfloat16_bits(a):
    """Round float32 to bfloat16 (nearest, ties to even); uint16 bit patterns.
    numpy has no bfloat16 dtype, so such tensors travel as uint16 arrays."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bfloat16_bits_to_float32(b):
    """Exact widening of bfloat16 bit patterns (uint16) to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def as_float(a):
    """float view of a host tensor of either format (float16 array, or uint16
    array of bfloat16 bits) for code that needs numbers, not bits."""
    return bfloat16_bits_to_float32(a) if a.dtype == np.uint16 else a


def _normal_f16(rng, shape, integer=False, fmt="f16"):
    """N(0,1) drawn in float32 and rounded to the 16-bit format (or small
    integers, exact in both formats).  fmt "bf16" returns uint16 bit patterns."""
    narrow = (lambda v: v.astype(np.float16)) if fmt == "f16" else float32_to_bfloat16_bits
    if integer:
        return narrow(rng.integers(-4, 5, size=shape).astype(np.float32))
    out = np.empty(shape, dtype=np.float16 if fmt == "f16" else np.uint16)
    flat = out.reshape(-1)
    step = 1 << 24
    for lo in range(0, flat.size, step):
        n = min(step, flat.size - lo)
        flat[lo:lo + n] = narrow(rng.standard_normal(n, dtype=np.float32))
    return out


@dataclass
class Problem:
    M: int
    K: int
    N: int
    V: int
    W: np.ndarray            # (M, K) float16 (or uint16 bfloat16 bits), dense (not masked)
    mask: np.ndarray         # (M, K) uint8
    perm: np.ndarray         # (M,) int32, perm[i] = original row of stored row i
    X: np.ndarray            # (K, N) same format as W, or None for conv problems
    cols: list = field(default_factory=list)   # per group, ascending kept columns
    conv: dict = None        # conv geometry and the activation tensor, if any

    @property
    def nnz(self):
        return int(self.V * sum(len(c) for c in self.cols))


def make_mask(rng, M, K, V, k_g, perm, ragged=False):
    """Mask with one random column set per permuted row group."""
    G = M // V
    mask = np.zeros((M, K), dtype=np.uint8)
    cols = []
    for g in range(G):
        kg = k_g
        if ragged:
            kg = int(rng.integers(0, k_g + 1))
        c = np.sort(rng.choice(K, size=kg, replace=False)) if kg > 0 else \
            np.zeros((0,), dtype=np.int64)
        cols.append(c.astype(np.int64))
        rows = perm[g * V:(g + 1) * V]
        mask[np.ix_(rows, c)] = 1
    return mask, cols


def make_spmm(M, K, N, V, sparsity, seed, identity_perm=False, integer=False,
              ragged=False, with_x=True, fmt="f16"):
    """A linear-layer problem Y = (W . mask) X."""
    if M % V:
        raise ValueError("M %% V != 0")
    rng = np.random.Generator(np.random.PCG64(seed))
    W = _normal_f16(rng, (M, K), integer, fmt)
    X = _normal_f16(rng, (K, N), integer, fmt) if with_x else None
    perm = rng.permutation(M).astype(np.int32)
    if identity_perm:
        perm = np.arange(M, dtype=np.int32)
    mask, cols = make_mask(rng, M, K, V, kept_per_group(K, sparsity), perm, ragged)
    return Problem(M, K, N, V, W, mask, perm, X, cols)


def make_conv(batch, Cin, H, Wd, Cout, R, S, V, sparsity, seed, stride=(1, 1),
              pad=(0, 0), layout="NCHW", integer=False, fmt="f16"):
    """A convolution problem in implicit-GEMM view: M = Cout, K = Cin*R*S
    with k = (c*R + r)*S + s, N = batch*Ho*Wo."""
    rng = np.random.Generator(np.random.PCG64(seed))
    K = Cin * R * S
    W = _normal_f16(rng, (Cout, K), integer, fmt)
    shape = (batch, Cin, H, Wd) if layout == "NCHW" else (Cin, H, Wd, batch)
    inp = _normal_f16(rng, shape, integer, fmt)
    perm = rng.permutation(Cout).astype(np.int32)
    mask, cols = make_mask(rng, Cout, K, V, kept_per_group(K, sparsity), perm)
    Ho = (H + 2 * pad[0] - R) // stride[0] + 1
    Wo = (Wd + 2 * pad[1] - S) // stride[1] + 1
    geom = dict(batch=batch, Cin=Cin, H=H, W=Wd, Cout=Cout, R=R, S=S, stride=tuple(stride),
                pad=tuple(pad), layout=layout, Ho=Ho, Wo=Wo, input=inp)
    return Problem(Cout, K, batch * Ho * Wo, V, W, mask, perm, None, cols, geom)


# The five workloads of the benchmark definition (index = config number - 1).
def config(index, variant=0, **over):
    seed = BASE_SEED + 1000 * index + variant
    if index == 0:      # tiny SpMM
        p = dict(M=256, K=256, N=64, V=32, sparsity=0.75)
    elif index == 1:    # Transformer-big FFN layer
        p = dict(M=4096, K=1024, N=8192, V=32, sparsity=0.75)
    elif index == 2:    # attention projection sweep: variant = 3*vi + si
        Vs, Ss = (16, 32, 64), (0.5, 0.75, 0.9)
        p = dict(M=1024, K=1024, N=4096, V=Vs[variant // 3], sparsity=Ss[variant % 3])
    elif index == 3:    # ResNet-50-style 3x3 conv
        c = dict(batch=32, Cin=256, H=14, Wd=14, Cout=256, R=3, S=3, V=32, sparsity=0.75,
                 stride=(1, 1), pad=(1, 1), layout="NCHW")
        c.update(over)
        return make_conv(seed=seed, **c)
    elif index == 4:    # large-layer scaling: variant indexes the sparsity
        Ss = (0.0, 0.75, 0.875, 0.95)
        p = dict(M=8192, K=8192, N=16384, V=64, sparsity=Ss[variant])
    else:
        raise ValueError("no such config")
    p.update(over)
    return make_spmm(seed=seed, **p)
