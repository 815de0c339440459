"""GPU parity with bfloat16 operands (the other 16-bit operand format of the
matrix cores), against the CPU oracle on the same bit patterns.

Bounds.  fp32 output: |Y - Y_ref| <= 2^-10 * (|W.mask| |X|), the same bound
as for binary16 operands (products are exact in fp32, only the fp32
accumulation rounds).  bfloat16 output: its rounding alone is 2^-9 * |Y|, so
the bound is 2^-8 * (|W.mask| |X|).  Small-integer inputs are exact in both
formats and must match the oracle bit for bit."""
import numpy as np
import pytest

from oracle import c_oracle
from paper_2203_05016_amd import binding, synth
from conftest import assert_within_scaled_tolerance
from gpu_util import announce, run_spmm, to_device, to_host

pytestmark = pytest.mark.gpu
TOL_BF16_OUT = 2.0 ** -8


def _parity(p, out_dtype, **kw):
    Y = run_spmm(p, out_dtype=out_dtype, **kw)
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    tol = TOL_BF16_OUT if out_dtype == "bfloat16" else 2.0 ** -10
    return assert_within_scaled_tolerance(Y, Yr, S, tol=tol, what="spmm bf16 -> " + out_dtype)


@pytest.mark.parametrize("V", [16, 32, 64, 128])
@pytest.mark.parametrize("out_dtype", ["float32", "bfloat16"])
def test_gather_kernel_ragged_shapes(V, out_dtype):
    announce("bf16 gather", V, out_dtype)
    p = synth.make_spmm(4 * V, 333, 472, V, 0.6, seed=61 + V, fmt="bf16")
    _parity(p, out_dtype, kernel=1)
    _parity(p, out_dtype, kernel=1, tile_n=64)


@pytest.mark.parametrize("V,sp", [(16, 0.5), (32, 0.75), (64, 0.5)])
@pytest.mark.parametrize("out_dtype", ["float32", "bfloat16"])
def test_slab_kernel(V, sp, out_dtype):
    announce("bf16 slab", V, sp, out_dtype)
    p = synth.make_spmm(16 * V, 700, 392, V, sp, seed=71 + V, fmt="bf16")
    _parity(p, out_dtype, kernel=2)


@pytest.mark.parametrize("V", [16, 32, 64, 128])
def test_integer_inputs_bit_exact_and_equal_to_binary16(V):
    announce("bf16 integer", V)
    p = synth.make_spmm(2 * V, 192, 200, V, 0.75, seed=31 + V, integer=True, fmt="bf16")
    q = synth.make_spmm(2 * V, 192, 200, V, 0.75, seed=31 + V, integer=True)
    Yr, _ = c_oracle.spmm(p.W, p.mask, p.X)
    for kernel in (1, 2) if V <= 64 else (1,):
        Y = run_spmm(p, out_dtype="float32", kernel=kernel)
        assert np.array_equal(Y.astype(np.float64), Yr), kernel
        assert np.array_equal(Y, run_spmm(q, out_dtype="float32", kernel=kernel)), kernel


def test_unaligned_and_tiny_n():
    announce("bf16 unaligned")
    for N in (1, 7, 130):
        p = synth.make_spmm(64, 100, N, 32, 0.5, seed=81 + N, fmt="bf16")
        _parity(p, "float32")
        _parity(p, "bfloat16")
    p = synth.make_spmm(64, 100, 136, 32, 0.5, seed=82, fmt="bf16")
    Y = run_spmm(p, out_dtype="bfloat16", pad_ld=24, offset=3)
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    assert_within_scaled_tolerance(Y, Yr, S, tol=TOL_BF16_OUT, what="padded ld, odd offset")


def test_headline_shape_sampled_columns():
    """Config 2's shape with bfloat16 operands, slab kernel, checked on 96 sampled columns."""
    announce("bf16 config2 sampled")
    import torch
    p = synth.make_spmm(4096, 1024, 8192, 32, 0.75, seed=synth.BASE_SEED + 1000, fmt="bf16")
    A = binding.compress(p.W, p.mask, p.perm, 32).bind_device("cuda:0")
    Y = to_host(A.spmm(to_device(p.X), out_dtype=torch.float32))
    cols = np.random.default_rng(7).choice(p.N, 96, replace=False)
    Yr, S = c_oracle.spmm(p.W, p.mask, np.ascontiguousarray(p.X[:, cols]))
    assert_within_scaled_tolerance(Y[:, cols], Yr, S, what="bf16 config2")


@pytest.mark.parametrize("layout", ["NCHW", "CHWN"])
@pytest.mark.parametrize("V", [32, 64])
def test_conv_both_kernels(layout, V):
    import torch
    announce("bf16 conv", layout, V)
    p = synth.make_conv(3, 24, 9, 7, 2 * V, 3, 3, V, 0.6, seed=91, stride=(1, 1), pad=(1, 1),
                        layout=layout, fmt="bf16")
    g = p.conv
    want, sc = c_oracle.conv2d(p.W, p.mask, g["input"], 3, 3, (1, 1), (1, 1), layout)
    for kernel in (1, 2):
        for dt, tol in ((torch.float32, 2.0 ** -10), (torch.bfloat16, TOL_BF16_OUT)):
            A = binding.compress(p.W, p.mask, p.perm, V)
            A.set_tuning(kernel, 0)
            A.bind_device("cuda:0")
            out = A.conv2d(to_device(g["input"]), 3, 3, (1, 1), (1, 1), layout, out_dtype=dt)
            torch.cuda.synchronize()
            assert_within_scaled_tolerance(to_host(out), want, sc, tol=tol,
                                           what="conv bf16 kernel %d" % kernel)


@pytest.mark.parametrize("layout,H,Wd", [("NCHW", 4, 6), ("NCHW", 2, 6), ("CHWN", 3, 5)])
def test_conv_1x1_shortcuts(layout, H, Wd):
    """1x1, stride 1, no padding: the linear-layer product on CHWN tensors, one
    launch over all images on NCHW tensors (H*W a multiple of 8, and of 4 only)."""
    import torch
    announce("bf16 conv 1x1", layout, H, Wd)
    V = 32
    p = synth.make_conv(7, 40, H, Wd, 2 * V, 1, 1, V, 0.5, seed=93, layout=layout, fmt="bf16")
    g = p.conv
    want, sc = c_oracle.conv2d(p.W, p.mask, g["input"], 1, 1, (1, 1), (0, 0), layout)
    for dt, tol in ((torch.float32, 2.0 ** -10), (torch.bfloat16, TOL_BF16_OUT)):
        A = binding.compress(p.W, p.mask, p.perm, V).bind_device("cuda:0")
        out = A.conv2d(to_device(g["input"]), 1, 1, (1, 1), (0, 0), layout, out_dtype=dt)
        torch.cuda.synchronize()
        assert_within_scaled_tolerance(to_host(out), want, sc, tol=tol, what="conv 1x1 bf16")


def test_output_type_must_match_operand_format():
    import torch
    announce("bf16 dtype checks")
    p = synth.make_spmm(64, 64, 64, 32, 0.5, seed=95, fmt="bf16")
    A = binding.compress(p.W, p.mask, p.perm, 32).bind_device("cuda:0")
    with pytest.raises(binding.ShflbwError):
        A.spmm(to_device(p.X), out_dtype=torch.float16)
    with pytest.raises(TypeError):
        A.spmm(to_device(p.X).to(torch.float16))
    q = synth.make_spmm(64, 64, 64, 32, 0.5, seed=95)
    B = binding.compress(q.W, q.mask, q.perm, 32).bind_device("cuda:0")
    with pytest.raises(binding.ShflbwError):
        B.spmm(to_device(q.X), out_dtype=torch.bfloat16)
