"""shflbw_spmm_unbound, the entry point for callers that cannot allocate device
memory (the packed arrays go into the library's own static device image):
called through the C ABI, its result must equal shflbw_spmm's bit for bit, on
two calls in a row, the second with a smaller matrix and input (the image
keeps the first call's contents), and then once more with the first; a packed
matrix beyond the image's size is refused."""
import ctypes

import numpy as np
import pytest

from paper_2203_05016_amd import binding, synth
from gpu_util import announce, to_device

pytestmark = pytest.mark.gpu


def _unbound(A, Xd, M, dtype):
    import torch
    K, N = Xd.shape
    Y = torch.full((M, N), float("nan"), dtype=dtype, device="cuda:0")
    rc = binding.lib().shflbw_spmm_unbound(A._h, Xd.data_ptr(), Xd.stride(0), Y.data_ptr(), Y.stride(0), N,
                                           binding._ydtype(Y), torch.cuda.current_stream().cuda_stream)
    assert rc == 0, binding.last_error()
    return Y


def test_unbound_spmm_equals_bound_spmm_on_consecutive_calls():
    import torch
    announce("spmm_unbound: large then small then large")
    big = synth.make_spmm(512, 1024, 1032, 32, 0.5, seed=9101)      # shared-slab kernel, ragged last tile
    small = synth.make_spmm(128, 264, 200, 64, 0.8, seed=9102)      # gather kernel, V = 64
    want = {}
    for name, p in (("big", big), ("small", small)):
        A = binding.compress(p.W, p.mask, p.perm, p.V).bind_device("cuda:0")
        want[name] = A.spmm(to_device(p.X)).clone()
        kernel = binding.last_kernel()
        A.device_status()
        del A
        # a handle that was never bound
        U = binding.compress(p.W, p.mask, p.perm, p.V)
        assert U.device_bytes() <= 8 << 20
        want[name + "_handle"] = (U, kernel)
    torch.cuda.synchronize()
    for name, p in (("big", big), ("small", small), ("big", big)):
        U, kernel = want[name + "_handle"]
        got = _unbound(U, to_device(p.X), p.M, torch.float16)
        assert binding.last_kernel() == kernel
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), want[name].view(torch.int16)), name
    # fp32 output, and a bound handle whose own buffer must stay untouched and unused
    B = binding.compress(small.W, small.mask, small.perm, small.V).bind_device("cuda:0")
    before = B._dev.clone()
    ref32 = B.spmm(to_device(small.X), out_dtype=torch.float32)
    got32 = _unbound(B, to_device(small.X), small.M, torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(got32.view(torch.int32), ref32.view(torch.int32))
    assert torch.equal(B._dev, before)


def test_unbound_spmm_refuses_what_does_not_fit_and_bad_arguments():
    import torch
    announce("spmm_unbound: refusals")
    p = synth.make_spmm(2048, 2304, 8, 32, 0.0, seed=9103)           # 9 MiB of packed values
    A = binding.compress(p.W, p.mask, p.perm, p.V)
    assert A.device_bytes() > 8 << 20
    X = to_device(p.X)
    Y = torch.zeros((p.M, 8), dtype=torch.float16, device="cuda:0")
    L = binding.lib()
    st = torch.cuda.current_stream().cuda_stream
    rc = L.shflbw_spmm_unbound(A._h, X.data_ptr(), 8, Y.data_ptr(), 8, 8, binding.F16, st)
    assert rc == -2 and "static device image" in binding.last_error()
    assert L.shflbw_spmm_unbound(None, X.data_ptr(), 8, Y.data_ptr(), 8, 8, binding.F16, st) == -1
    q = synth.make_spmm(64, 40, 8, 32, 0.5, seed=9104)
    B = binding.compress(q.W, q.mask, q.perm, q.V)
    Xq = to_device(q.X)
    assert L.shflbw_spmm_unbound(B._h, Xq.data_ptr(), 4, Y.data_ptr(), 8, 8, binding.F16, st) == -2   # ldx < N
    assert L.shflbw_spmm_unbound(B._h, Xq.data_ptr(), 8, Y.data_ptr(), 8, 8, binding.BF16, st) == -5  # wrong output type
    torch.cuda.synchronize()
    assert not Y.any().item()
