"""GPU parity of shflbw_layernorm_transpose (the LayerNorm-side transposition
of Section 4.3's layout discussion) against the float64 definition.

Bound: statistics are taken in fp32 and the result is rounded once to the
16-bit output format, so |y - y_ref| <= tol * (|gamma| |x_hat| + |beta|) +
tol * 2^-4 with tol = 2^-10 for float16 and 2^-8 for bfloat16 (the absolute
term covers cancellation to zero inside x_hat * gamma + beta).  The plain
transposition is bit exact."""
import numpy as np
import pytest

from oracle import c_oracle, definition
from paper_2203_05016_amd import binding, synth
from conftest import assert_within_scaled_tolerance
from gpu_util import announce, to_device, to_host

pytestmark = pytest.mark.gpu


def _draw(N, K, fmt, seed, offset=0.0, scale=1.0):
    rng = np.random.Generator(np.random.PCG64(seed))
    narrow = (lambda v: v.astype(np.float16)) if fmt == "f16" else synth.float32_to_bfloat16_bits
    x = narrow((rng.standard_normal((N, K), dtype=np.float32) * scale + offset).astype(np.float32))
    gamma = narrow(1.0 + 0.25 * rng.standard_normal(K, dtype=np.float32))
    beta = narrow(0.5 * rng.standard_normal(K, dtype=np.float32))
    return x, gamma, beta


def _check(x, gamma, beta, eps, fmt):
    got = to_host(binding.layernorm_transpose(to_device(x), None if gamma is None else to_device(gamma),
                                              None if beta is None else to_device(beta), eps))
    want, S = definition.layernorm_transpose(synth.as_float(x), None if gamma is None else synth.as_float(gamma),
                                             None if beta is None else synth.as_float(beta), eps)
    tol = 2.0 ** -10 if fmt == "f16" else 2.0 ** -8
    err = np.abs(got.astype(np.float64) - want)
    bound = tol * S + tol * 2.0 ** -4
    assert np.all(np.isfinite(got)) and np.all(err <= bound), \
        "max excess %.3e at %r" % (float((err - bound).max()), np.unravel_index(int((err - bound).argmax()), err.shape))


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
@pytest.mark.parametrize("N,K", [(64, 64), (200, 1024), (1000, 328), (8, 8), (72, 4096), (16456, 72),
                                 (96, 2264), (96, 2272), (40008, 1024), (200, 3000), (72, 4104), (40, 8192), (24, 8200), (40, 16384), (16, 16392)])
def test_layernorm_transpose_parity(fmt, N, K):
    """Shapes for each code path: blocks of 32 tokens held in LDS, blocks of 64
    (input and output beyond 160 MB, ragged last block), the largest K that
    still fits, the register-resident kernel beyond it (one to four parts of
    4096 features, full and partial) and the streaming kernel beyond 16384."""
    announce("layernorm", fmt, N, K)
    x, gamma, beta = _draw(N, K, fmt, seed=700 + N + K)
    _check(x, gamma, beta, 1e-5, fmt)
    _check(x, None, None, 1e-5, fmt)


def test_layernorm_large_mean_small_spread_and_constant_rows():
    """Tokens sitting far from zero with a small spread (the case a naive
    sum-of-squares variance loses), and constant tokens (zero variance)."""
    announce("layernorm hard rows")
    x, gamma, beta = _draw(128, 512, "f16", seed=711, offset=100.0, scale=0.25)
    _check(x, gamma, beta, 1e-5, "f16")
    x[5, :] = np.float16(3.0)
    x[77, :] = np.float16(-0.5)
    got = to_host(binding.layernorm_transpose(to_device(x), to_device(gamma), to_device(beta), 1e-5))
    assert np.array_equal(got[:, 5], beta) and np.array_equal(got[:, 77], beta)


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
def test_plain_transposition_is_bit_exact_with_padded_leading_dimensions(fmt):
    import torch
    announce("transpose only", fmt)
    x, _, _ = _draw(136, 200, fmt, seed=720)
    xd = to_device(x)
    xbuf = torch.zeros((136, 216), dtype=xd.dtype, device="cuda:0")
    xbuf[:, :200].copy_(xd)
    obuf = torch.full((200, 160), float("nan"), dtype=xd.dtype, device="cuda:0")
    binding.layernorm_transpose(xbuf[:, :200], normalize=False, out=obuf[:, :136])
    torch.cuda.synchronize()
    full = obuf.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(full[:, :136], x.view(np.uint16).T)
    nan_bits = obuf[0, 159:160].view(torch.int16).cpu().numpy().view(np.uint16)[0]
    assert np.all(full[:, 136:] == nan_bits)          # nothing outside the K x N window is written


def test_layernorm_then_spmm_chain_matches_the_oracles():
    """Token-major activations -> LayerNorm-side transposition -> shflbw_spmm,
    against the float64 chain that starts from the GPU's own rounded X."""
    announce("layernorm -> spmm")
    p = synth.make_spmm(256, 512, 384, 32, 0.75, seed=730)
    x, gamma, beta = _draw(384, 512, "f16", seed=731)
    X = binding.layernorm_transpose(to_device(x), to_device(gamma), to_device(beta), 1e-5)
    A = binding.compress(p.W, p.mask, p.perm, 32).bind_device("cuda:0")
    Y = to_host(A.spmm(X))
    Xh = to_host(X)
    Yr, S = c_oracle.spmm(p.W, p.mask, Xh)
    assert_within_scaled_tolerance(Y, Yr, S, what="chain")


def test_argument_checks():
    import torch
    announce("layernorm argument checks")
    x = torch.zeros((16, 12), dtype=torch.float16, device="cuda:0")      # K not a multiple of 8
    with pytest.raises(binding.ShflbwError):
        binding.layernorm_transpose(x)
    y = torch.zeros((16, 16), dtype=torch.float32, device="cuda:0")
    with pytest.raises(TypeError):
        binding.layernorm_transpose(y)
