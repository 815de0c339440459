"""Helpers shared by the GPU parity tests (all of them call the library
through its C ABI via the binding)."""
import sys

import numpy as np


def announce(*what):
    """Name the case on stdout, flushed, before the GPU is touched."""
    print("[gpu-case]", *what, flush=True)
    sys.stdout.flush()


def to_device(a):
    """Host tensor (float16 array, or uint16 array of bfloat16 bits) on cuda:0."""
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to("cuda:0")
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def to_host(t):
    """Device tensor as a numpy array; bfloat16 is widened (exactly) to float32."""
    import torch
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.cpu().numpy()


def run_spmm(p, out_dtype="float16", tile_n=0, X=None, pad_ld=0, offset=0, kernel=0):
    """Compress, bind and multiply on cuda:0; returns Y as a numpy array
    (bfloat16 output widened to float32)."""
    import torch
    from paper_2203_05016_amd import binding
    A = binding.compress(p.W, p.mask, p.perm, p.V)
    A.set_tuning(kernel, tile_n)
    A.bind_device("cuda:0")
    Xh = p.X if X is None else X
    K, N = Xh.shape
    dt = getattr(torch, out_dtype)
    if pad_ld or offset:
        Xsrc = to_device(Xh)
        Xbuf = torch.zeros(K * (N + pad_ld) + offset + 8, dtype=Xsrc.dtype, device="cuda:0")
        Xd = Xbuf[offset:offset + K * (N + pad_ld)].view(K, N + pad_ld)[:, :N]
        Xd.copy_(Xsrc)
        Ybuf = torch.full((p.M * (N + pad_ld) + offset + 8,), float("nan"), dtype=dt, device="cuda:0")
        Yd = Ybuf[offset:offset + p.M * (N + pad_ld)].view(p.M, N + pad_ld)[:, :N]
        A.spmm(Xd, Yd)
        torch.cuda.synchronize()
        full = to_host(Ybuf)
        body = full[offset:offset + p.M * (N + pad_ld)].reshape(p.M, N + pad_ld)
        # nothing outside the M x N window may have been written
        assert np.isnan(body[:, N:]).all() and np.isnan(full[:offset]).all() and \
            np.isnan(full[offset + p.M * (N + pad_ld):]).all()
        return body[:, :N].copy()
    Xd = to_device(Xh)
    Yd = torch.full((p.M, N), float("nan"), dtype=dt, device="cuda:0")
    A.spmm(Xd, Yd)
    torch.cuda.synchronize()
    return to_host(Yd)
