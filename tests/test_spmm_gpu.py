"""GPU parity of shflbw_spmm against the CPU oracle, element by element, on
seeded inputs.  Bound: |Y - Y_ref| <= 2^-10 * (|W.mask| |X|) per element
(fp16 inputs, fp32 accumulation); bit-exact where small-integer inputs make
the result unique."""
import numpy as np
import pytest

from oracle import c_oracle
from paper_2203_05016_amd import synth
from conftest import assert_within_scaled_tolerance
from gpu_util import announce, run_spmm

pytestmark = pytest.mark.gpu


def _parity(p, **kw):
    Y = run_spmm(p, **kw)
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    return assert_within_scaled_tolerance(Y, Yr, S, what="spmm")


@pytest.mark.parametrize("out_dtype", ["float16", "float32"])
@pytest.mark.parametrize("tile_n", [64, 128])
def test_config1_tiny(out_dtype, tile_n):
    announce("config1", out_dtype, tile_n)
    _parity(synth.config(0), out_dtype=out_dtype, tile_n=tile_n)


@pytest.mark.parametrize("V", [16, 32, 64, 128])
@pytest.mark.parametrize("tile_n", [64, 128])
def test_integer_inputs_bit_exact(V, tile_n):
    """Small integers: every product and partial sum is exact in fp32, so the
    GPU must reproduce the oracle bit for bit (also after fp16 rounding of
    the output, since |Y| stays below 2048)."""
    announce("integer", V, tile_n)
    p = synth.make_spmm(2 * V, 192, 200, V, 0.75, seed=31 + V, integer=True)
    Yr, _ = c_oracle.spmm(p.W, p.mask, p.X)
    assert np.abs(Yr).max() < 2048
    for dt in ("float16", "float32"):
        Y = run_spmm(p, out_dtype=dt, tile_n=tile_n)
        assert np.array_equal(Y.astype(np.float64), Yr), dt


@pytest.mark.parametrize("V,sp", [(16, 0.5), (16, 0.9), (32, 0.5), (32, 0.9), (64, 0.75),
                                  (64, 0.9), (128, 0.75)])
def test_multi_tile_ragged_tail(V, sp):
    """Several N tiles with a ragged tail (N = 8*59), kept counts that are not
    a multiple of the k-step, non-trivial permutation."""
    announce("ragged-tail", V, sp)
    p = synth.make_spmm(4 * V, 333, 472, V, sp, seed=41 + V)
    _parity(p)
    _parity(p, out_dtype="float32", tile_n=64)


def test_variable_kept_counts_and_empty_groups():
    announce("ragged groups")
    p = synth.make_spmm(8 * 32, 300, 264, 32, 0.6, seed=51, ragged=True)
    rows = p.perm[32:64]
    p.mask[rows] = 0
    p.cols[1] = np.zeros((0,), dtype=np.int64)
    Y = run_spmm(p)
    assert np.all(Y[rows] == 0)
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    assert_within_scaled_tolerance(Y, Yr, S, what="ragged groups")


def test_all_groups_empty_writes_zeros():
    announce("all empty")
    p = synth.make_spmm(64, 40, 72, 32, 0.5, seed=52)
    p.mask[:] = 0
    Y = run_spmm(p)
    assert Y.shape == (64, 72) and np.all(Y == 0)


@pytest.mark.parametrize("N", [1, 7, 9, 130])
def test_unaligned_n_takes_general_path(N):
    announce("unaligned N", N)
    p = synth.make_spmm(64, 100, N, 32, 0.5, seed=60 + N)
    _parity(p)
    _parity(p, out_dtype="float32")


def test_leading_dimensions_and_misaligned_bases():
    announce("ld / offset")
    p = synth.make_spmm(64, 100, 136, 32, 0.5, seed=70)
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    for pad_ld, offset in ((8, 0), (3, 0), (0, 1), (8, 8)):
        Y = run_spmm(p, pad_ld=pad_ld, offset=offset)
        assert_within_scaled_tolerance(Y, Yr, S, what="ld=%d off=%d" % (pad_ld, offset))


def test_very_long_leading_dimension_takes_plain_addressing():
    """Rows of X and Y 16 MiB apart: beyond what the gather kernel's 24-bit
    offset arithmetic covers, so the aligned path with 64-bit addresses runs
    (every smaller aligned case goes through the buffer-descriptor path)."""
    import torch
    from paper_2203_05016_amd import binding
    from gpu_util import to_device, to_host
    announce("long ld")
    p = synth.make_spmm(64, 40, 72, 32, 0.5, seed=77)
    ld = (1 << 23) + 8
    A = binding.compress(p.W, p.mask, p.perm, p.V).bind_device("cuda:0")
    Xbuf = torch.zeros(p.K * ld, dtype=torch.float16, device="cuda:0")
    Xd = Xbuf.view(p.K, ld)[:, :p.N]
    Xd.copy_(to_device(p.X))
    Ybuf = torch.full((p.M * ld,), float("nan"), dtype=torch.float16, device="cuda:0")
    Yd = Ybuf.view(p.M, ld)[:, :p.N]
    A.spmm(Xd, Yd)
    torch.cuda.synchronize()
    Y = to_host(Yd.contiguous())
    # nothing next to the window was written
    assert torch.isnan(Ybuf.view(p.M, ld)[:, p.N:p.N + 64]).all().item()
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    assert_within_scaled_tolerance(Y, Yr, S, what="long leading dimension")
    del Xbuf, Ybuf, Xd, Yd
    torch.cuda.empty_cache()


def test_dense_identity_is_gemm():
    """Sparsity 0 with the identity permutation: the kernel is a dense GEMM."""
    announce("dense identity")
    p = synth.make_spmm(128, 256, 136, 32, 0.0, seed=80, identity_perm=True)
    Y = run_spmm(p, out_dtype="float32")
    want = p.W.astype(np.float64) @ p.X.astype(np.float64)
    S = np.abs(p.W.astype(np.float64)) @ np.abs(p.X.astype(np.float64))
    assert_within_scaled_tolerance(Y, want, S, what="dense")


def test_permutation_invariant_bitwise():
    """Shuffling the rows of W (and composing the permutation) gives the
    packed arrays of the same groups, so Y[q] must match bit for bit."""
    announce("perm invariant")
    p = synth.make_spmm(128, 200, 136, 32, 0.75, seed=81)
    Y = run_spmm(p)
    q = np.random.Generator(np.random.PCG64(5)).permutation(128)
    inv = np.empty(128, dtype=np.int64)
    inv[q] = np.arange(128)
    p2 = synth.Problem(p.M, p.K, p.N, p.V, p.W[q], p.mask[q], inv[p.perm].astype(np.int32), p.X,
                       p.cols)
    Y2 = run_spmm(p2)
    assert np.array_equal(Y2.view(np.uint16), Y[q].view(np.uint16))


def test_identity_permutation_matches_shuffled_rows():
    announce("identity perm")
    p = synth.make_spmm(128, 200, 136, 32, 0.75, seed=82, identity_perm=True)
    _parity(p)


def test_repeat_runs_are_bitwise_identical():
    announce("determinism")
    p = synth.config(0)
    a = run_spmm(p)
    b = run_spmm(p)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))


def test_large_magnitudes_and_signed_zero():
    announce("magnitudes")
    p = synth.make_spmm(64, 128, 72, 32, 0.5, seed=83)
    p.W[:] = (p.W.astype(np.float32) * 30).astype(np.float16)
    X = (p.X.astype(np.float32) * 2.0 ** -12).astype(np.float16)   # subnormal-range products
    Y = run_spmm(p, X=X, out_dtype="float32")
    Yr, S = c_oracle.spmm(p.W, p.mask, X)
    assert_within_scaled_tolerance(Y, Yr, S, what="magnitudes")


@pytest.mark.parametrize("kernel", [0, 1, 2])
def test_infinite_weights_stay_in_their_group(kernel):
    """Three k-steps per group (an odd count: the kernels' batches of steps
    run past the group's end) and a middle group whose weights are all
    infinite: the steps past the end must multiply zeros, not the
    neighbour's weights, so the other groups' rows stay finite and right."""
    announce("infinite neighbour", kernel)
    V = 32
    p = synth.make_spmm(3 * V, 96, 72, V, 0.5, seed=87)
    rows_mid = p.perm[V:2 * V]
    others = np.concatenate([p.perm[:V], p.perm[2 * V:]])
    p.W[rows_mid, :] = np.float16(np.inf)
    Y = run_spmm(p, out_dtype="float32", kernel=kernel)
    assert not np.isfinite(Y[rows_mid]).any()
    Wf = p.W.copy()
    Wf[rows_mid, :] = 0
    Yr, S = c_oracle.spmm(Wf, p.mask, p.X)
    assert_within_scaled_tolerance(Y[others], Yr[others], S[others], what="rows beside an infinite group")


@pytest.mark.parametrize("kernel", [1, 2])
def test_launches_replayed_from_a_graph_match_eager(kernel):
    """shflbw_spmm only enqueues a kernel on the caller's stream (no
    allocation, no synchronisation, no memset), so its launches can be captured
    into a HIP graph; every replay, with eager launches and synchronisations
    in between, must reproduce the eager result bit for bit."""
    import torch
    from paper_2203_05016_amd import binding
    from gpu_util import to_device, to_host
    announce("graph replay", kernel)
    p = synth.make_spmm(256, 512, 384, 32, 0.75, seed=91)
    A = binding.compress(p.W, p.mask, p.perm, p.V)
    A.set_tuning(kernel, 0)
    A.bind_device("cuda:0")
    X = to_device(p.X)
    X2 = to_device(synth.make_spmm(256, 512, 384, 32, 0.75, seed=92).X)
    eager = torch.empty((p.M, p.N), dtype=torch.float16, device="cuda:0")
    A.spmm(X, eager)
    torch.cuda.synchronize()
    want = to_host(eager).view(np.uint16)
    Yg = torch.zeros((p.M, p.N), dtype=torch.float16, device="cuda:0")
    Xg = X.clone()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        A.spmm(Xg, Yg)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        A.spmm(Xg, Yg)
        A.spmm(Xg, Yg)
    for replay in range(4):
        Yg.fill_(float("nan"))
        other = torch.empty_like(eager)
        A.spmm(X2, other)               # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(to_host(Yg).view(np.uint16), want), "replay %d" % replay
    A.device_status()


@pytest.mark.parametrize("variant", range(9))
def test_config3_attention_projection_every_variant_every_element(variant):
    """Config 3 (1024 x 1024 by 1024 x 4096) in all nine variants, V in {16, 32, 64} x
    sparsity in {50, 75, 90 %}: automatic kernel choice as the benchmark launches
    it, every element against the oracle."""
    p = synth.config(2, variant=variant)
    announce("config3 variant", variant, "V", p.V, "kept", len(p.cols[0]))
    Y = run_spmm(p)
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    assert_within_scaled_tolerance(Y, Yr, S, what="config3 variant %d" % variant)


@pytest.mark.parametrize("V_index", [0, 1, 2])
def test_config3_dense_runs_every_element(V_index):
    """The sparsity-0 runs of config 3 that every quoted speedup is divided by
    (V = 16, 32, 64; same seeds as the benchmark's dense legs), every element."""
    p = synth.config(2, variant=3 * V_index, sparsity=0.0)
    announce("config3 dense run V", p.V)
    Y = run_spmm(p)
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    assert_within_scaled_tolerance(Y, Yr, S, what="config3 dense V=%d" % p.V)


@pytest.mark.parametrize("variant", [0, 1, 2, 3])
def test_config5_large_layer_sampled(variant):
    """Config 5 at full size (8192 x 8192 by 8192 x 16384, V = 64; sparsity
    0 / 75 / 87.5 / 95 %), in the launch configuration the benchmark times
    (automatic kernel choice): all rows on 256 sampled columns plus 64 sampled
    full rows."""
    import torch
    from paper_2203_05016_amd import binding
    from gpu_util import to_device, to_host
    announce("config5", variant)
    p = synth.config(4, variant=variant)
    A = binding.compress(p.W, p.mask, p.perm, p.V).bind_device("cuda:0")
    Y = to_host(A.spmm(to_device(p.X)))
    rng = np.random.default_rng(500 + variant)
    cols = np.sort(rng.choice(p.N, 256, replace=False))
    Yr, S = c_oracle.spmm(p.W, p.mask, np.ascontiguousarray(p.X[:, cols]))
    assert_within_scaled_tolerance(Y[:, cols], Yr, S, what="config5 columns")
    rows = np.sort(rng.choice(p.M, 64, replace=False))
    Yr, S = c_oracle.spmm(np.ascontiguousarray(p.W[rows]), np.ascontiguousarray(p.mask[rows]), p.X)
    assert_within_scaled_tolerance(Y[rows], Yr, S, what="config5 rows")
    del A, Y
    torch.cuda.empty_cache()


# ---------------------------------------------------------------- split k-steps (skinny N)
@pytest.mark.parametrize("V", [16, 32, 64, 128])
@pytest.mark.parametrize("N", [1, 16, 64, 130])
def test_split_k_gather_kernel(V, N):
    """The wavefronts of a workgroup share one column tile and a share of the k-steps each."""
    announce("split-k", V, N)
    p = synth.make_spmm(3 * V, 777, N, V, 0.5, seed=601 + V + N)
    Y = run_spmm(p, kernel=3)
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    assert_within_scaled_tolerance(Y, Yr, S, what="split-k")
    assert_within_scaled_tolerance(run_spmm(p, kernel=3, out_dtype="float32"), Yr, S, what="split-k f32")


def test_split_k_few_steps_empty_groups_and_integers():
    announce("split-k edge cases")
    # fewer k-steps than wavefronts, ragged and empty groups
    p = synth.make_spmm(8 * 32, 40, 48, 32, 0.0, seed=611, ragged=True)
    rows = p.perm[32:64]
    p.mask[rows] = 0
    p.cols[1] = np.zeros((0,), dtype=np.int64)
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    Y = run_spmm(p, kernel=3)
    assert_within_scaled_tolerance(Y, Yr, S, what="split-k ragged")
    assert not Y[rows].any()
    # exact integers: the split changes the order of the sums, not the result
    q = synth.make_spmm(128, 384, 40, 64, 0.5, seed=612, integer=True)
    Yq, _ = c_oracle.spmm(q.W, q.mask, q.X)
    assert np.array_equal(run_spmm(q, kernel=3, out_dtype="float32").astype(np.float64), Yq)
    assert np.array_equal(run_spmm(q, kernel=3, out_dtype="float32"), run_spmm(q, kernel=1, out_dtype="float32"))
    # bfloat16 operands
    b = synth.make_spmm(128, 384, 40, 32, 0.5, seed=613, fmt="bf16")
    Yb, Sb = c_oracle.spmm(b.W, b.mask, b.X)
    assert_within_scaled_tolerance(run_spmm(b, kernel=3, out_dtype="float32"), Yb, Sb, what="split-k bf16")


def test_skinny_shape_is_routed_to_split_k_and_matches():
    """A recurrent-layer-like shape (4096 x 4096 weights, 64 columns): the
    automatic choice, the split kernel and the plain gather kernel agree with
    the oracle on all elements."""
    announce("skinny auto")
    p = synth.make_spmm(4096, 4096, 64, 32, 0.75, seed=614)
    Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
    for kernel in (0, 3, 1):
        assert_within_scaled_tolerance(run_spmm(p, kernel=kernel), Yr, S, what="skinny kernel %d" % kernel)


def test_searched_pattern_end_to_end():
    """Pattern search (Section 5) -> compress -> product, on weights whose large entries
    follow hidden groups: the mask comes from the library's search, the product is
    checked against the oracle with that mask."""
    from paper_2203_05016_amd import binding
    from gpu_util import to_device, to_host
    announce("search -> compress -> spmm")
    rng = np.random.Generator(np.random.PCG64(901))
    M, K, N, V = 512, 640, 264, 32
    W = (0.1 * rng.standard_normal((M, K), dtype=np.float32))
    hidden = rng.permutation(M)
    for g in range(M // V):
        cols = rng.choice(K, 160, replace=False)
        W[np.ix_(hidden[g * V:(g + 1) * V], cols)] += rng.standard_normal((V, 160), dtype=np.float32)
    W = W.astype(np.float16)
    X = rng.standard_normal((K, N), dtype=np.float32).astype(np.float16)
    perm, mask = binding.pattern_search(W, V, 0.25, None, 8)
    A = binding.compress(W, mask, perm, V).bind_device("cuda:0")
    assert A.info()["nnz"] == M * 160
    Y = to_host(A.spmm(to_device(X)))
    Yr, S = c_oracle.spmm(W, mask, X)
    assert_within_scaled_tolerance(Y, Yr, S, what="searched pattern")


def test_seeded_sweep_of_shapes_kernels_and_sparsities():
    """Thirty seeded draws of V, group count, K, N (aligned and not), sparsity,
    ragged kept counts, output type and kernel choice (automatic, gather,
    split k-steps), each against the oracle."""
    rng = np.random.default_rng(2024)
    for it in range(30):
        V = int(rng.choice([16, 32, 64, 128]))
        G = int(rng.integers(1, 14))
        K = int(rng.integers(1, 160)) * 8 if rng.random() < 0.8 else int(rng.integers(8, 900))
        N = int(rng.integers(1, 60)) * 8 if rng.random() < 0.7 else int(rng.integers(1, 500))
        sp = float(rng.choice([0.0, 0.3, 0.5, 0.75, 0.9, 0.97]))
        kernel = int(rng.choice([0, 0, 1, 3]))
        ragged = bool(rng.random() < 0.3)
        out_dtype = str(rng.choice(["float16", "float32"]))
        announce("sweep", it, V, G, K, N, sp, kernel, ragged, out_dtype)
        p = synth.make_spmm(G * V, K, N, V, sp, seed=5000 + it, ragged=ragged)
        Y = run_spmm(p, out_dtype=out_dtype, kernel=kernel)
        Yr, S = c_oracle.spmm(p.W, p.mask, p.X)
        assert_within_scaled_tolerance(Y, Yr, S, what="sweep case %d" % it)
