"""GPU parity of the shared-slab SpMM kernel (forced through the tuning
switch) against the CPU oracle; same bound as the other SpMM tests."""
import numpy as np
import pytest

from oracle import c_oracle
from paper_2203_05016_amd import binding, synth
from conftest import assert_within_scaled_tolerance
from gpu_util import announce, run_spmm

pytestmark = pytest.mark.gpu
SLAB = 2


def _parity(p, **kw):
    Y = run_spmm(p, kernel=SLAB, **kw)
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    return assert_within_scaled_tolerance(Y, Yr, S, what="slab spmm")


@pytest.mark.parametrize("out_dtype", ["float16", "float32"])
def test_slab_config1_tiny(out_dtype):
    announce("slab config1", out_dtype)
    _parity(synth.config(0), out_dtype=out_dtype)


@pytest.mark.parametrize("V", [16, 32, 64, 128])
def test_slab_integer_inputs_bit_exact(V):
    announce("slab integer", V)
    p = synth.make_spmm(20 * V, 400, 264, V, 0.6, seed=131 + V, integer=True)
    Yr, _ = c_oracle.spmm(p.W, p.mask, p.X)
    assert np.abs(Yr).max() < 2048
    for dt in ("float16", "float32"):
        Y = run_spmm(p, out_dtype=dt, kernel=SLAB)
        assert np.array_equal(Y.astype(np.float64), Yr), dt


@pytest.mark.parametrize("V,K,sp", [(16, 333, 0.5), (32, 333, 0.5), (32, 1000, 0.75),
                                    (64, 520, 0.6), (32, 128, 0.0), (64, 384, 0.0),
                                    (128, 520, 0.6), (128, 333, 0.0)])
def test_slab_multi_tile_ragged(V, K, sp):
    """Several column tiles with a ragged tail (N = 8*59), K not a multiple of
    the chunk, group counts that leave wavefronts of the last block idle."""
    announce("slab ragged", V, K, sp)
    p = synth.make_spmm(18 * V, K, 472, V, sp, seed=141 + V)
    _parity(p)
    _parity(p, out_dtype="float32")


def test_slab_variable_kept_counts_and_empty_groups():
    announce("slab ragged groups")
    p = synth.make_spmm(20 * 32, 700, 264, 32, 0.5, seed=151, ragged=True)
    rows = p.perm[32:64]
    p.mask[rows] = 0
    p.cols[1] = np.zeros((0,), dtype=np.int64)
    Y = run_spmm(p, kernel=SLAB)
    assert np.all(Y[rows] == 0)
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    assert_within_scaled_tolerance(Y, Yr, S, what="slab ragged groups")


def test_slab_v128_two_wavefronts_per_group():
    """V = 128: two compute wavefronts share a group (64 of its rows each, the same
    steps and activation rows).  An odd number of groups leaves half a workgroup idle,
    ragged kept counts and an empty group; both output types; the gather kernel on
    exact inputs must give the same bits."""
    announce("slab V=128")
    p = synth.make_spmm(5 * 128, 700, 392, 128, 0.5, seed=171, ragged=True)
    rows = p.perm[128:256]
    p.mask[rows] = 0
    p.cols[1] = np.zeros((0,), dtype=np.int64)
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    for out_dtype in ("float16", "float32"):
        Y = run_spmm(p, kernel=SLAB, out_dtype=out_dtype)
        assert np.all(Y[rows] == 0)
        assert_within_scaled_tolerance(Y, Yr, S, what="slab V=128 " + out_dtype)
    q = synth.make_spmm(3 * 128, 640, 264, 128, 0.75, seed=172, integer=True)
    assert np.array_equal(run_spmm(q, kernel=1).view(np.uint16), run_spmm(q, kernel=SLAB).view(np.uint16))
    b = synth.make_spmm(2 * 128, 384, 136, 128, 0.5, seed=173, fmt="bf16")
    Yb, Sb = c_oracle.spmm(b.W, b.mask, b.X)
    assert_within_scaled_tolerance(run_spmm(b, kernel=SLAB, out_dtype="float32"), Yb, Sb, what="slab V=128 bf16")


def test_slab_matches_gather_kernel_on_exact_inputs():
    announce("slab vs gather")
    p = synth.make_spmm(512, 640, 392, 32, 0.75, seed=152, integer=True)
    a = run_spmm(p, kernel=1)
    b = run_spmm(p, kernel=SLAB)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))


def test_slab_refused_when_layout_or_operands_do_not_allow_it():
    import torch
    announce("slab refusal")
    p = synth.make_spmm(64, 4096, 64, 32, 0.98, seed=153)      # far too sparse for the window
    A = binding.compress(p.W, p.mask, p.perm, 32).bind_device("cuda:0")
    A.set_tuning(2, 0)
    with pytest.raises(binding.ShflbwError) as e:
        A.spmm(torch.from_numpy(p.X).to("cuda:0"))
    assert e.value.status == -9
    A.set_tuning(0, 0)
    Y = A.spmm(torch.from_numpy(p.X).to("cuda:0"))
    torch.cuda.synchronize()
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    assert_within_scaled_tolerance(Y.cpu().numpy(), Yr, S, what="fallback")


def _bench_rotation(p, out_bytes=2, cache=256 << 20):
    """Number of (X, Y) pairs the benchmark rotates through for this problem."""
    per = 2 * p.K * p.N + out_bytes * p.M * p.N
    return max(2, min(8, -(-2 * cache // per)))


@pytest.mark.parametrize("sparsity", [0.75, 0.0])
def test_config2_ffn_full_size_every_element_as_the_benchmark_launches_it(sparsity):
    """Headline workload (4096 x 1024 by 1024 x 8192, V = 32) at 75 % and its own
    dense run (sparsity 0), every element against the oracle, in the launch
    configuration the benchmark times: automatic kernel choice, the same packed
    matrix launched in turn over the benchmark's rotating (X, Y) pairs; each pair's
    Y must be the same bits, and the choice must be the shared-slab kernel."""
    import torch
    from gpu_util import to_device, to_host
    announce("config2 full size", sparsity)
    p = synth.config(1, sparsity=sparsity)
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    A = binding.compress(p.W, p.mask, p.perm, p.V).bind_device("cuda:0")
    rot = _bench_rotation(p)
    x0 = to_device(p.X)
    Xs = [x0] + [x0.clone() for _ in range(rot - 1)]
    Ys = [torch.full((p.M, p.N), float("nan"), dtype=torch.float16, device="cuda:0") for _ in range(rot)]
    for step in range(2 * rot):              # every pair twice, back to back, as in the timed loop
        A.spmm(Xs[step % rot], Ys[step % rot])
    torch.cuda.synchronize()
    A.device_status()
    assert binding.last_kernel().startswith("shflbw_slab_kernel<32,"), binding.last_kernel()
    Y0 = to_host(Ys[0])
    assert_within_scaled_tolerance(Y0, Yr, S, what="config2 s=%.2f" % sparsity)
    for j in range(1, rot):
        assert torch.equal(Ys[j], Ys[0]), "pair %d differs" % j
    del Xs, Ys, A
    torch.cuda.empty_cache()


def test_slab_distant_steps_are_bridged():
    """Every group keeps two bands of columns 24 chunks apart (further than the
    table's 4-bit chunk difference reaches, so the compressor puts an empty
    step between them), and one group starts late (its first chunk is not 0)."""
    announce("slab distant steps")
    p = synth.make_spmm(12 * 32, 2560, 264, 32, 0.0, seed=157)
    p.mask[:, 512:2048] = 0
    p.mask[p.perm[32:64], :448] = 0
    for out_dtype in ("float16", "float32"):
        Y = run_spmm(p, kernel=SLAB, out_dtype=out_dtype)
        Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
        assert_within_scaled_tolerance(Y, Yr, S, what="slab distant steps")


def test_slab_reports_a_wait_that_ran_out():
    """The hand-over between loader and compute wavefronts is bounded; with the
    bound at zero every wait gives up at once (the kernel still ends normally,
    its numbers are not to be trusted) and the status call says so, once."""
    import torch
    announce("slab wait limit")
    p = synth.make_spmm(16 * 32, 1024, 1024, 32, 0.5, seed=161)
    A = binding.compress(p.W, p.mask, p.perm, 32).bind_device("cuda:0")
    A.set_tuning(SLAB, 0)
    X = torch.from_numpy(p.X).to("cuda:0")
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    Y = A.spmm(X)
    A.device_status()                      # nothing ran out
    assert_within_scaled_tolerance(Y.cpu().numpy(), Yr, S, what="before")
    A.set_wait_limit(0)
    Ybad = A.spmm(X)
    with pytest.raises(binding.ShflbwError) as e:
        A.device_status()
    assert e.value.status == -10
    # the failure is visible in the data: a tile whose wavefront gave up (or finished after a
    # wait of its workgroup ran out) is NaN, every other element is right - never a
    # plausible wrong number
    Yb = Ybad.cpu().numpy().astype(np.float64)
    bad = np.isnan(Yb)
    assert bad.any(), "no tile was poisoned although every wait gave up at once"
    assert np.all(np.abs(Yb[~bad] - Yr[~bad]) <= 2.0 ** -10 * S[~bad])
    # poisoning goes by whole 32-row x 128-column tiles
    rows_of_group0 = p.perm[:32]
    block = bad[np.ix_(rows_of_group0, np.arange(128))]
    assert block.all() or not block.any()
    A.device_status()                      # the word was cleared
    A.set_wait_limit(1 << 20)
    Y = A.spmm(X)
    A.device_status()
    assert_within_scaled_tolerance(Y.cpu().numpy(), Yr, S, what="after")
    with pytest.raises(binding.ShflbwError):
        A.set_wait_limit(-1)
