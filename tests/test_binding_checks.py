"""The binding refuses, on the host and before anything is enqueued, operands
that the C ABI could not tell from valid ones (it sees bare addresses and has
no K argument): wrong shapes, overlapping or transposed rows, host tensors,
tensors of another device.  No GPU is needed: the matrix is given a stand-in
for its device buffer, and every call must raise before it reaches the
library's launchers."""
import types

import numpy as np
import pytest
import torch

from paper_2203_05016_amd import binding, synth


@pytest.fixture()
def bound_matrix():
    p = synth.make_spmm(64, 40, 24, 32, 0.5, seed=7)
    A = binding.compress(p.W, p.mask, p.perm, p.V)
    A._dev = types.SimpleNamespace(device=torch.device("cuda:0"))   # "bound", without a GPU
    return A, p


def test_spmm_before_bind_is_refused():
    p = synth.make_spmm(64, 40, 24, 32, 0.5, seed=7)
    A = binding.compress(p.W, p.mask, p.perm, p.V)
    with pytest.raises(RuntimeError, match="bind_device"):
        A.spmm(torch.zeros((40, 24), dtype=torch.float16))


def test_spmm_refuses_host_tensors_and_wrong_shapes(bound_matrix):
    A, p = bound_matrix
    X = torch.zeros((p.K, p.N), dtype=torch.float16)
    with pytest.raises(ValueError, match="must live on"):
        A.spmm(X)                                            # host memory
    with pytest.raises(ValueError, match="K = 40"):
        A.spmm(torch.zeros((p.K - 8, p.N), dtype=torch.float16))   # short X: the ABI has no K argument
    with pytest.raises(TypeError):
        A.spmm(torch.zeros((p.K, p.N), dtype=torch.float32))
    with pytest.raises(TypeError):
        A.spmm(torch.zeros((p.N, p.K), dtype=torch.float16).t())   # column stride != 1
    with pytest.raises(ValueError, match="overlap"):
        A.spmm(torch.zeros((1, p.N), dtype=torch.float16).expand(p.K, p.N))
    for bad in (torch.zeros((p.M, p.N - 8), dtype=torch.float16),      # too narrow
                torch.zeros((p.M - 32, p.N), dtype=torch.float16),     # too short
                torch.zeros((p.N, p.M), dtype=torch.float16).t(),      # transposed view
                torch.zeros((p.M * p.N,), dtype=torch.float16)):       # not a matrix
        with pytest.raises(ValueError):
            A.spmm(X, bad)
    with pytest.raises(TypeError):
        A.spmm(X, torch.zeros((p.M, p.N), dtype=torch.float64))
    with pytest.raises(ValueError, match="must live on"):
        A.spmm(X, torch.zeros((p.M, p.N), dtype=torch.float16))    # right shape, host memory


def test_conv2d_refuses_host_tensors_and_wrong_shapes():
    q = synth.make_conv(2, 8, 6, 6, 32, 3, 3, 32, 0.5, seed=3, pad=(1, 1))
    A = binding.compress(q.W, q.mask, q.perm, q.V)
    inp = torch.from_numpy(q.conv["input"])
    with pytest.raises(RuntimeError, match="bind_device"):
        A.conv2d(inp, 3, 3, (1, 1), (1, 1))
    A._dev = types.SimpleNamespace(device=torch.device("cuda:0"))
    with pytest.raises(ValueError, match="must live on"):
        A.conv2d(inp, 3, 3, (1, 1), (1, 1))
    with pytest.raises(ValueError, match="K = 72"):
        A.conv2d(inp[:, :4].contiguous(), 3, 3, (1, 1), (1, 1))
    with pytest.raises(ValueError):
        A.conv2d(inp, 3, 3, (1, 1), (1, 1), layout="NHWC")
    with pytest.raises(TypeError):
        A.conv2d(inp.permute(0, 1, 3, 2), 3, 3, (1, 1), (1, 1))    # not contiguous
    with pytest.raises(ValueError, match="shape"):
        A.conv2d(inp, 3, 3, (1, 1), (1, 1), out=torch.zeros((2, 32, 6, 5), dtype=torch.float16))
    with pytest.raises(ValueError, match="shape"):
        A.conv2d(inp, 3, 3, (1, 1), (1, 1), out=torch.zeros((2, 32, 8, 6), dtype=torch.float16)[:, :, :6])
    with pytest.raises(ValueError):
        A.conv2d(inp, 3, 3, (0, 1), (1, 1))


def test_layernorm_transpose_refuses_mixed_devices_and_shapes():
    x = torch.zeros((16, 64), dtype=torch.float16)
    with pytest.raises(TypeError):
        binding.layernorm_transpose(x, out=torch.zeros((64, 8), dtype=torch.float16))
    with pytest.raises(TypeError):
        binding.layernorm_transpose(x.float())
    with pytest.raises(ValueError, match="one GPU"):
        binding.layernorm_transpose(x, out=torch.zeros((64, 16), dtype=torch.float16))


def test_last_kernel_is_empty_before_any_launch():
    assert binding.last_kernel() == "" or "kernel<" in binding.last_kernel()
