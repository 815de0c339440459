"""GPU parity of shflbw_conv2d (implicit GEMM) against the CPU oracle."""
import numpy as np
import pytest

from oracle import c_oracle
from paper_2203_05016_amd import binding, synth
from conftest import assert_within_scaled_tolerance
from gpu_util import announce

pytestmark = pytest.mark.gpu


def _run_conv(p, out_dtype="float16", tile_n=0, kernel=0):
    """kernel: 0 automatic (the staged kernel where it applies), 1 gather
    kernel, 2 staged kernel or an error."""
    import torch
    g = p.conv
    A = binding.compress(p.W, p.mask, p.perm, p.V)
    A.set_tuning(kernel, tile_n)
    A.bind_device("cuda:0")
    x = torch.from_numpy(g["input"]).to("cuda:0")
    shape = (g["batch"], g["Cout"], g["Ho"], g["Wo"]) if g["layout"] == "NCHW" else \
        (g["Cout"], g["Ho"], g["Wo"], g["batch"])
    out = torch.full(shape, float("nan"), dtype=getattr(torch, out_dtype), device="cuda:0")
    A.conv2d(x, g["R"], g["S"], g["stride"], g["pad"], g["layout"], out=out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _parity(p, **kw):
    g = p.conv
    got = _run_conv(p, **kw)
    want, sc = c_oracle.conv2d(p.W, p.mask, g["input"], g["R"], g["S"], g["stride"], g["pad"],
                               g["layout"])
    assert got.shape == want.shape
    return assert_within_scaled_tolerance(got, want, sc, what="conv2d")


@pytest.mark.parametrize("layout", ["NCHW", "CHWN"])
@pytest.mark.parametrize("stride,pad,R,S", [((1, 1), (1, 1), 3, 3), ((2, 2), (1, 1), 3, 3),
                                            ((1, 1), (0, 0), 1, 1), ((2, 1), (0, 2), 3, 2)])
def test_conv_small_shapes(layout, stride, pad, R, S):
    announce("conv small", layout, stride, pad, R, S)
    p = synth.make_conv(3, 24, 9, 7, 64, R, S, 32, 0.6, seed=201, stride=stride, pad=pad,
                        layout=layout)
    _parity(p, kernel=2)
    _parity(p, kernel=1)
    _parity(p, out_dtype="float32", kernel=2)
    _parity(p, out_dtype="float32", tile_n=64, kernel=1)


@pytest.mark.parametrize("V", [16, 64, 128])
def test_conv_other_group_sizes_integer_exact(V):
    announce("conv integer", V)
    p = synth.make_conv(2, 16, 7, 7, 2 * V, 3, 3, V, 0.75, seed=202, pad=(1, 1), integer=True)
    g = p.conv
    got = _run_conv(p, out_dtype="float32")
    if V >= 64:  # the staged kernel covers V = 32, 64 and 128; both kernels must agree bit for bit
        assert np.array_equal(got, _run_conv(p, out_dtype="float32", kernel=1))
        assert np.array_equal(got, _run_conv(p, out_dtype="float32", kernel=2))
    want, _ = c_oracle.conv2d(p.W, p.mask, g["input"], 3, 3, (1, 1), (1, 1))
    assert np.array_equal(got.astype(np.float64), want)


def test_conv_1x1_equals_spmm_path_bitwise():
    """1x1, stride 1, no padding, CHWN: the implicit GEMM is exactly the
    linear-layer product on the reshaped input."""
    import torch
    announce("conv 1x1 vs spmm")
    p = synth.make_conv(8, 48, 5, 5, 64, 1, 1, 32, 0.5, seed=203, layout="CHWN")
    got = _run_conv(p)
    A = binding.compress(p.W, p.mask, p.perm, 32).bind_device("cuda:0")
    X = torch.from_numpy(p.conv["input"].reshape(48, 5 * 5 * 8)).to("cuda:0")
    Y = A.spmm(X)
    torch.cuda.synchronize()
    assert np.array_equal(got.reshape(64, 200).view(np.uint16), Y.cpu().numpy().view(np.uint16))


@pytest.mark.parametrize("V,out_dtype", [(16, "float16"), (32, "float32"), (64, "float16"), (128, "float16")])
def test_conv_1x1_nchw_one_launch_for_all_images(V, out_dtype):
    """1x1, stride 1, no padding, NCHW with H*W a multiple of 8: one product per
    image, all in one launch of the gather kernel (tiles of 64 columns span
    several images of 24 positions here); against the oracle, and bit for
    bit against the staged kernel on integers."""
    announce("conv 1x1 nchw", V, out_dtype)
    p = synth.make_conv(7, 40, 4, 6, 2 * V, 1, 1, V, 0.5, seed=241)
    _parity(p, out_dtype=out_dtype)
    q = synth.make_conv(7, 40, 4, 6, 2 * V, 1, 1, V, 0.5, seed=242, integer=True)
    got = _run_conv(q, out_dtype="float32")
    want, _ = c_oracle.conv2d(q.W, q.mask, q.conv["input"], 1, 1, (1, 1), (0, 0))
    assert np.array_equal(got.astype(np.float64), want)
    if V in (32, 64, 128):
        assert np.array_equal(got, _run_conv(q, out_dtype="float32", kernel=2))
    # H*W a multiple of 4 only (images of 14 x 14 and the like): loads and stores in halves
    r = synth.make_conv(5, 40, 2, 6, 2 * V, 1, 1, V, 0.5, seed=243, integer=True)
    for dt in ("float16", "float32"):
        got = _run_conv(r, out_dtype=dt)
        want, _ = c_oracle.conv2d(r.W, r.mask, r.conv["input"], 1, 1, (1, 1), (0, 0))
        assert np.array_equal(got.astype(np.float64), want)
    _parity(synth.make_conv(5, 40, 2, 6, 2 * V, 1, 1, V, 0.5, seed=244), out_dtype=out_dtype)


@pytest.mark.parametrize("layout,batch,Cin,H,Wd,Cout,V", [
    ("NCHW", 2, 8, 6, 150, 32, 32),     # rows wider than a box: several boxes along x
    ("CHWN", 40, 8, 6, 50, 32, 32),     # batch innermost, boxes of a few positions x all images
    ("NCHW", 5, 300, 12, 12, 32, 32),   # many channels: the staged box shrinks to fit the LDS
    ("NCHW", 3, 16, 10, 10, 640, 64),   # V = 64, ten groups: two blocks of groups per box
    ("CHWN", 130, 4, 3, 3, 32, 32),     # more images than one box holds
    ("NCHW", 4, 8, 96, 96, 32, 32),     # enough positions for boxes of 128 (four instruction tiles)
    ("NCHW", 4, 8, 72, 72, 32, 32),     # boxes of 64 (two instruction tiles)
    ("CHWN", 16, 8, 48, 48, 64, 64),    # batch innermost, boxes of 128, V = 64
    ("NCHW", 4, 8, 72, 72, 256, 128),   # V = 128: four row blocks, boxes of 64 at most
    ("CHWN", 24, 12, 9, 9, 128, 128),   # V = 128, batch innermost, one group
    ("NCHW", 4, 8, 96, 96, 48, 16),     # V = 16 (16-position instruction tiles), boxes of 128, three groups share wavefronts
    ("NCHW", 3, 24, 10, 10, 160, 16),   # V = 16, ten groups: two blocks of groups per box
    ("CHWN", 40, 8, 6, 50, 16, 16),     # V = 16, batch innermost, one group
    ("NCHW", 2, 150, 9, 9, 32, 16),     # V = 16, 1350 reduction indices: the koff list is refilled in bulks of 32 steps
])
def test_conv_staged_kernel_box_shapes(layout, batch, Cin, H, Wd, Cout, V):
    announce("conv boxes", layout, batch, Cin, H, Wd, Cout, V)
    p = synth.make_conv(batch, Cin, H, Wd, Cout, 3, 3, V, 0.5, seed=204, pad=(1, 1), layout=layout)
    _parity(p, kernel=2)
    _parity(p, kernel=1)


@pytest.mark.parametrize("kernel", [1, 2])
def test_conv_infinite_weights_stay_in_their_group(kernel):
    """Groups of 5 k-steps (the step loops run whole batches and so reach
    past a group's end) beside a group whose weights are all infinite: the
    steps past the end must multiply zeros, not the neighbour's weights."""
    announce("conv infinite neighbour", kernel)
    V = 32
    p = synth.make_conv(2, 16, 9, 9, 3 * V, 3, 3, V, 0.45, seed=231, pad=(1, 1))   # 79 kept columns
    g = p.conv
    rows_mid = p.perm[V:2 * V]
    others = np.concatenate([p.perm[:V], p.perm[2 * V:]])
    p.W[rows_mid, :] = np.float16(np.inf)
    got = _run_conv(p, out_dtype="float32", kernel=kernel)
    assert not np.isfinite(got[:, rows_mid]).any()
    Wf = p.W.copy()
    Wf[rows_mid, :] = 0
    want, sc = c_oracle.conv2d(Wf, p.mask, g["input"], g["R"], g["S"], g["stride"], g["pad"], g["layout"])
    assert_within_scaled_tolerance(got[:, others], want[:, others], sc[:, others],
                                   what="channels beside an infinite group")


def test_conv_staged_kernel_refuses_what_it_cannot_hold():
    """Forcing the staged kernel on an input whose channels do not fit the LDS even for
    the smallest box is an error, not a silent switch; the automatic choice takes the
    gather kernel there."""
    announce("conv staged refusal")
    p = synth.make_conv(1, 4000, 5, 5, 32, 3, 3, 32, 0.9, seed=205, pad=(1, 1))
    with pytest.raises(binding.ShflbwError):
        _run_conv(p, kernel=2)
    _parity(p)


def test_conv_v16_staged_kernel_on_config4_shape():
    """Config 4's tensor with groups of 16 output channels, every element, staged kernel
    (automatic choice) and gather kernel."""
    announce("config4 shape, V=16")
    p = synth.config(3, V=16)
    got = _parity(p)
    assert binding.last_kernel().startswith("shflbw_conv_kernel<16,"), binding.last_kernel()
    _parity(p, kernel=1)


@pytest.mark.parametrize("layout,batch,Cin,H,Wd,Cout,V,stride,pad,wide", [
    ("NCHW", 8, 16, 56, 56, 64, 32, 1, 1, True),    # odd padding: the staged box starts one column further left
    ("NCHW", 2, 16, 40, 40, 64, 64, 1, 0, True),    # no padding, V = 64
    ("NCHW", 2, 16, 48, 48, 32, 32, 2, 1, True),    # stride 2
    ("NCHW", 16, 8, 40, 40, 32, 16, 1, 1, True),    # V = 16
    ("CHWN", 16, 8, 20, 20, 32, 32, 1, 1, True),    # pairs along the batch
    ("NCHW", 2, 16, 39, 39, 32, 32, 1, 1, False),   # odd image width: pairs would straddle the border
    ("CHWN", 15, 8, 20, 20, 32, 32, 1, 1, False),   # odd batch
])
def test_conv_staging_with_4_byte_loads(layout, batch, Cin, H, Wd, Cout, V, stride, pad, wide):
    """Boxes staged two elements per load where the tensor allows it: the kernel the library
    reports, and parity either way."""
    announce("conv 4-byte staging", layout, batch, Cin, H, Wd, Cout, V, stride, pad)
    p = synth.make_conv(batch, Cin, H, Wd, Cout, 3, 3, V, 0.5, seed=206, stride=(stride, stride),
                        pad=(pad, pad), layout=layout)
    _parity(p, kernel=2)
    assert ("4-byte staging" in binding.last_kernel()) == wide, binding.last_kernel()
    _parity(p, out_dtype="float32", kernel=2)


def test_conv_staging_falls_back_to_2_byte_loads_for_an_input_that_is_not_4_byte_aligned():
    import torch
    announce("conv staging, misaligned input")
    p = synth.make_conv(2, 64, 56, 56, 64, 3, 3, 32, 0.5, seed=207, pad=(1, 1))
    g = p.conv
    A = binding.compress(p.W, p.mask, p.perm, p.V)
    A.set_tuning(2, 0)
    A.bind_device("cuda:0")
    flat = torch.zeros(g["input"].size + 1, dtype=torch.float16, device="cuda:0")
    x = flat[1:].view(g["input"].shape)          # two bytes past a 4-byte boundary
    x.copy_(torch.from_numpy(g["input"]))
    assert x.data_ptr() % 4 == 2
    out = torch.full((g["batch"], g["Cout"], g["Ho"], g["Wo"]), float("nan"), dtype=torch.float16, device="cuda:0")
    A.conv2d(x, g["R"], g["S"], g["stride"], g["pad"], g["layout"], out=out)
    torch.cuda.synchronize()
    assert "shflbw_conv_kernel" in binding.last_kernel() and "4-byte staging" not in binding.last_kernel()
    want, sc = c_oracle.conv2d(p.W, p.mask, g["input"], g["R"], g["S"], g["stride"], g["pad"], g["layout"])
    assert_within_scaled_tolerance(out.cpu().numpy(), want, sc, what="conv2d, misaligned input")


def test_config4_resnet_conv_full():
    """Config 4 at full size (32x256x14x14, 3x3, pad 1, V=32, 75 %), both kernels."""
    announce("config4")
    p = synth.config(3)
    _parity(p, kernel=2)
    _parity(p, kernel=1)


def test_seeded_sweep_of_conv_geometries():
    """Sixteen seeded draws of V, group count, batch, channels, image size,
    1x1 / 3x3, stride, padding and layout, each against the oracle (few row
    groups, so the shared-tile mapping and the 1x1 shortcuts are all hit)."""
    rng = np.random.default_rng(2025)
    for it in range(16):
        V = int(rng.choice([32, 64, 128, 16]))
        G = int(rng.integers(1, 6))
        B = int(rng.integers(1, 6)); C = int(rng.integers(1, 40))
        H = int(rng.integers(3, 20)); Wd = int(rng.integers(3, 20))
        R = int(rng.choice([1, 3])); st = int(rng.choice([1, 2])); pad = int(rng.choice([0, 1]))
        layout = str(rng.choice(["NCHW", "CHWN"]))
        sp = float(rng.choice([0.0, 0.5, 0.75]))
        announce("conv sweep", it, V, G, B, C, H, Wd, R, st, pad, layout, sp)
        p = synth.make_conv(B, C, H, Wd, G * V, R, R, V, sp, seed=7000 + it, stride=(st, st),
                            pad=(pad, pad), layout=layout)
        _parity(p, out_dtype="float32")
