#!/usr/bin/env python3
"""Benchmark of the Shfl-BW hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--all] [--no-cpu]

A step is one pass of the whole hot path (metadata prefetch, stitched tile
loads, matrix-core product, reordered write-back: one shflbw_spmm launch)
over one batch of synthetic input.  Headline workload: the Transformer-big
FFN layer, W 4096x1024 fp16, V=32, 75 % sparsity, X 1024x8192 fp16, with all
operands resident in HBM before the timed region.  Successive steps rotate
through enough (X, Y) buffer pairs that no activation or output byte
survives in the 256 MB last-level cache between two uses ("cold"); the packed
weights (2 MB) are the same every step, as in inference.

Prints ONE JSON line.  value = useful TFLOP/s = 2*nnz*N / t.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_F16_PEAK = 2.5166e15      # 256 CU x 4096 FLOP/clk x 2.4 GHz
HBM_PEAK = 8.0e12
# Counter readings of the headline kernel, copied from the rocprofv3 --pmc summary named in
# COUNTER_SOURCE (they are not measured by this run: counters are collected in runs of their
# own).  They are reported only when the run launches what that summary profiled: automatic
# kernel choice, no tile override, and the kernel named in COUNTER_KERNEL.
COUNTER_SOURCE = "profiles/slab_kernel_ffn_config2_pmc.md"
COUNTER_KERNEL = "shflbw_slab_kernel<32,12,f16,f16 out>"
L2_TO_CU_BYTES = 330.0e6        # TCP_TCC_READ_REQ x 128 B per launch
MEASURED_TRAFFIC_BYTES = 107.2e6  # FETCH_SIZE + WRITE_SIZE per launch, scaled by the same counters on a 64 MiB copy
PAPER_CONTEXT = "paper: up to 1.81x/4.18x/1.90x over cuBLAS dense at 75% on V100/T4/A100 (context only)"


def algorithmic_bytes(M, K, N, nnz, V, out_bytes=2):
    """Bytes the method itself must move once: packed values, column and row
    indices, X, Y."""
    kept_cols = nnz // V
    return 2 * nnz + 4 * kept_cols + 4 * M + 2 * K * N + out_bytes * M * N


class Case:
    """One packed matrix on the device plus rotating activation/output pairs."""

    def __init__(self, p, rotate, out_dtype="float16", tile_n=0, kernel=0):
        import torch
        from paper_2203_05016_amd import binding
        self.p = p
        self.A = binding.compress(p.W, p.mask, p.perm, p.V)
        self.A.set_tuning(kernel, tile_n)
        self.A.bind_device("cuda:0")
        self.info = self.A.info()
        if p.X.dtype == np.uint16:   # bfloat16 bit patterns
            x0 = torch.from_numpy(p.X.view(np.int16)).view(torch.bfloat16).to("cuda:0")
            if out_dtype == "float16":
                out_dtype = "bfloat16"
        else:
            x0 = torch.from_numpy(p.X).to("cuda:0")
        self.X = [x0] + [x0.clone() for _ in range(rotate - 1)]
        dt = getattr(torch, out_dtype)
        self.Y = [torch.empty((p.M, p.N), dtype=dt, device="cuda:0") for _ in range(rotate)]
        self.out_bytes = 4 if out_dtype == "float32" else 2
        self.i = 0

    def step(self):
        j = self.i % len(self.X)
        self.A.spmm(self.X[j], self.Y[j])
        self.i += 1

    def flop(self):
        return 2.0 * self.info["nnz"] * self.p.N

    def bytes(self):
        return algorithmic_bytes(self.p.M, self.p.K, self.p.N, self.info["nnz"], self.p.V,
                                 self.out_bytes)


SETTLE_MS = 30.0   # untimed load before every timed leg, see time_steps


def time_steps(fn, steps, warmup):
    """Average milliseconds per call of fn over `steps` calls, HIP events on
    the stream the kernels are launched on (torch's current stream).

    The GPU raises its clocks over the first ~10 ms of load: back-to-back batches of
    100 launches of the headline product measured 44, 40 and 38 us per launch.  So
    that a 20-step run and a 200-step run time the same machine state, every leg first
    runs its own workload untimed for SETTLE_MS of GPU time, then the `warmup`
    steps, then the timed steps."""
    import torch
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    spent = 0.0
    while spent < SETTLE_MS:
        e0.record()
        for _ in range(50):
            fn()
        e1.record()
        torch.cuda.synchronize()
        spent += e0.elapsed_time(e1)
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def time_graph(fn, per_graph, replays):
    """Average milliseconds per call of fn when `per_graph` calls are captured into one HIP
    graph and the graph is replayed: what a launch costs once the host's issue rate is out
    of the way (a product of a few microseconds is otherwise bound by it)."""
    import torch
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for _ in range(per_graph):
            fn()
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for _ in range(per_graph):
            fn()
    graph.replay()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (replays * per_graph)


def rotation_for(p, out_bytes=2, cache=256 << 20):
    per = 2 * p.K * p.N + out_bytes * p.M * p.N
    return max(2, min(8, -(-2 * cache // per)))


def measure_spmm(p, steps, warmup, cold=True, graph=False, sample_rows=None, **kw):
    """Times `steps` launches.  sample_rows: row indices whose results, as the timed launches
    left them in every rotating output buffer, are returned for the check against the oracle."""
    import torch
    from paper_2203_05016_amd import binding
    rot = rotation_for(p) if cold else 1
    c = Case(p, rot, **kw)
    ms = time_steps(c.step, steps, warmup)
    c.A.device_status()   # raises if a bounded hand-over wait ran out in any of these launches
    r = dict(ms=ms, tflops=c.flop() / (ms * 1e-3) / 1e12, gbps=c.bytes() / (ms * 1e-3) / 1e9,
             nnz=c.info["nnz"], sparsity=c.info["sparsity"], bytes=c.bytes(), flop=c.flop(),
             rotate=rot, kernel=binding.last_kernel())
    if sample_rows is not None:
        idx = torch.as_tensor(np.asarray(sample_rows), device="cuda:0")
        r["sample"] = [y.index_select(0, idx).float().cpu().numpy() for y in c.Y[:min(rot, steps + warmup)]]
    if graph:
        # the same launches, rotating operands included, replayed from a HIP graph
        r["graph_ms"] = time_graph(c.step, 4 * rot, max(1, steps // (4 * rot)))
        c.A.device_status()
    del c
    torch.cuda.empty_cache()
    return r


def measure_conv(p, steps, warmup, pairs=8):
    """conv2d on rotating input/output pairs (cold operands)."""
    import torch
    from paper_2203_05016_amd import binding
    g = p.conv
    A = binding.compress(p.W, p.mask, p.perm, p.V).bind_device("cuda:0")
    shape = (g["batch"], g["Cout"], g["Ho"], g["Wo"]) if g["layout"] == "NCHW" else \
        (g["Cout"], g["Ho"], g["Wo"], g["batch"])
    xs = [torch.from_numpy(g["input"]).to("cuda:0") for _ in range(pairs)]
    outs = [torch.empty(shape, dtype=torch.float16, device="cuda:0") for _ in range(pairs)]
    state = {"i": 0}

    def fn():
        j = state["i"] % pairs
        A.conv2d(xs[j], g["R"], g["S"], g["stride"], g["pad"], g["layout"], out=outs[j])
        state["i"] += 1
    ms = time_steps(fn, steps, warmup)
    flop = 2.0 * A.info()["nnz"] * p.N
    return dict(ms=ms, tflops=flop / (ms * 1e-3) / 1e12, flop=flop)


def binding_last_kernel():
    from paper_2203_05016_amd import binding
    return binding.last_kernel()


def measure_conv_shapes(steps, warmup):
    """ResNet-50-like layer shapes at batch 32, V = 32, 75 % sparsity, NCHW: this library's
    conv2d on rotating input/output pairs, and the vendor's dense convolution as context."""
    import torch
    from paper_2203_05016_amd import binding, synth
    shapes = [(64, 56, 64, 3, 1, 1), (128, 28, 128, 3, 1, 1), (256, 14, 256, 3, 1, 1), (512, 7, 512, 3, 1, 1),
              (128, 56, 128, 3, 2, 1), (256, 56, 64, 1, 1, 0), (1024, 14, 256, 1, 1, 0), (2048, 7, 512, 1, 1, 0)]
    res = {}
    for (C, H, Co, R, st, pad) in shapes:
        p = synth.make_conv(32, C, H, H, Co, R, R, 32, 0.75, seed=synth.BASE_SEED + 9000 + C + R,
                            stride=(st, st), pad=(pad, pad))
        g = p.conv
        A = binding.compress(p.W, p.mask, p.perm, p.V).bind_device("cuda:0")
        pairs = 4
        xs = [torch.from_numpy(g["input"]).to("cuda:0") for _ in range(pairs)]
        outs = [torch.empty((32, Co, g["Ho"], g["Wo"]), dtype=torch.float16, device="cuda:0") for _ in range(pairs)]
        state = {"i": 0}

        def fn():
            j = state["i"] % pairs
            A.conv2d(xs[j], R, R, (st, st), (pad, pad), "NCHW", out=outs[j])
            state["i"] += 1
        ms = time_steps(fn, steps, warmup)
        wt = torch.from_numpy(p.W.reshape(Co, C, R, R)).to("cuda:0")

        def dense():
            j = state["i"] % pairs
            torch.nn.functional.conv2d(xs[j], wt, stride=st, padding=pad)
            state["i"] += 1
        dense_ms = time_steps(dense, max(5, steps // 4), 3)
        flop = 2.0 * A.info()["nnz"] * p.N
        res["%dch_%dx%d_to_%dch_%dx%d_s%d" % (C, H, H, Co, R, R, st)] = dict(
            ms=ms, tflops=flop / (ms * 1e-3) / 1e12, vendor_dense_conv_ms=dense_ms)
        del xs, outs, wt
        torch.cuda.empty_cache()
    return res


def measure_library_gemm(p, steps, warmup):
    """The vendor library's dense fp16 GEMM (torch.matmul) on the same shape,
    unpruned W, rotating operands: context for the speedup, not part of the path."""
    import torch
    rot = rotation_for(p)
    Wd = torch.from_numpy(p.W).to("cuda:0")
    Xs = [torch.from_numpy(p.X).to("cuda:0") for _ in range(rot)]
    Ys = [torch.empty((p.M, p.N), dtype=torch.float16, device="cuda:0") for _ in range(rot)]
    state = {"i": 0}

    def fn():
        j = state["i"] % rot
        torch.matmul(Wd, Xs[j], out=Ys[j])
        state["i"] += 1
    ms = time_steps(fn, steps, warmup)
    return dict(ms=ms, dense_tflops=2.0 * p.M * p.K * p.N / (ms * 1e-3) / 1e12)


def measure_layernorm_transpose(p, steps, warmup):
    """The LayerNorm-side transposition that hands token-major activations (N x K) to the
    headline product as X (K x N); HBM-bound: 2*N*K bytes read, 2*N*K written."""
    import torch
    from paper_2203_05016_amd import binding
    rot = rotation_for(p)
    rng = np.random.Generator(np.random.PCG64(12))
    xs = [torch.from_numpy(rng.standard_normal((p.N, p.K), dtype=np.float32).astype(np.float16)).to("cuda:0")
          for _ in range(rot)]
    outs = [torch.empty((p.K, p.N), dtype=torch.float16, device="cuda:0") for _ in range(rot)]
    gamma = torch.ones(p.K, dtype=torch.float16, device="cuda:0")
    beta = torch.zeros(p.K, dtype=torch.float16, device="cuda:0")
    state = {"i": 0}

    def fn():
        j = state["i"] % rot
        binding.layernorm_transpose(xs[j], gamma, beta, 1e-5, out=outs[j])
        state["i"] += 1
    ms = time_steps(fn, steps, warmup)
    nbytes = 4.0 * p.N * p.K
    return dict(ms=ms, bytes=nbytes, GBps=nbytes / (ms * 1e-3) / 1e9, hbm_frac=nbytes / (ms * 1e-3) / HBM_PEAK)


PROBE_SRC = os.path.join(ROOT, "bench_l2_probe.hip")
PROBE_LIB = os.path.join(ROOT, "bench_l2_probe.so")


def build_probe():
    """Compile the L2 streaming probe (measurement aid, not part of the product)."""
    import subprocess
    from paper_2203_05016_amd import build as lib_build
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = PROBE_LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([hipcc, "-x", "hip", PROBE_SRC, "-shared", "-o", tmp] + lib_build.FLAGS,
                          stderr=subprocess.DEVNULL)
    os.replace(tmp, PROBE_LIB)
    return PROBE_LIB


def measure_l2_stream(p):
    """The probe library's two streaming runs on the headline's X: the rate at which the
    L2s can feed LDS with this access pattern when nothing else runs (hot), and with the
    slab kernel's grid and sharing on cold operands."""
    import ctypes
    import torch
    lib = ctypes.CDLL(PROBE_LIB if os.path.exists(PROBE_LIB) else build_probe())
    fn = lib.shflbw_probe_l2_stream
    fn.restype = ctypes.c_longlong
    fn.argtypes = [ctypes.c_void_p, ctypes.c_longlong, ctypes.c_int, ctypes.c_longlong, ctypes.c_int,
                   ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    rot = rotation_for(p)
    Xs = [torch.from_numpy(p.X).to("cuda:0") for _ in range(rot)]
    sink = torch.zeros(4, dtype=torch.float32, device="cuda:0")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    out = {}
    for name, mode, passes, steps in (("hot", 0, 16, 20), ("kernel_pattern_cold", 1, 1, 100)):
        state = {"i": 0, "bytes": 0}

        def step():
            x = Xs[state["i"] % rot]
            state["bytes"] = fn(ctypes.c_void_p(x.data_ptr()), p.N, p.K, p.N, mode, 11, passes,
                                ctypes.c_void_p(sink.data_ptr()), stream)
            assert state["bytes"] > 0, "probe refused its arguments"
            state["i"] += 1
        ms = time_steps(step, steps, 5)
        out[name] = {"ms": ms, "bytes": state["bytes"], "GBps": state["bytes"] / (ms * 1e-3) / 1e9}
    return out


def measure_lds_read():
    """The probe library's LDS read rates over the chip: the transposing 16-bit read the slab
    kernel's matrix instructions are fed with, and a plain read of the same width, twelve
    wavefronts per CU (the slab kernel's compute wavefronts)."""
    import ctypes
    import torch
    lib = ctypes.CDLL(PROBE_LIB if os.path.exists(PROBE_LIB) else build_probe())
    fn = lib.shflbw_probe_lds_read
    fn.restype = ctypes.c_longlong
    fn.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    sink = torch.zeros(4, dtype=torch.float32, device="cuda:0")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    out = {}
    for name, tr in (("transposing_ds_read_b64_tr_b16", 1), ("plain_ds_read_b64", 0)):
        state = {"bytes": 0}

        def step():
            state["bytes"] = fn(tr, 12, 500, ctypes.c_void_p(sink.data_ptr()), stream)
            assert state["bytes"] > 0
        ms = time_steps(step, 10, 2)
        out[name] = {"ms": ms, "TBps": state["bytes"] / (ms * 1e-3) / 1e12,
                     "bytes_per_clock_per_cu_at_2.4GHz": state["bytes"] / (ms * 1e-3) / 256 / 2.4e9}
    return out


def measure_stream_store():
    """The probe library's loads and stores through one CU's memory path: 256 workgroups stream
    201 MB of L2-resident X into LDS, write 75 MB of Y in the slab kernel's write-back pattern, or do
    both at once - how far a launch's loads and stores can overlap."""
    import ctypes
    import torch
    lib = ctypes.CDLL(PROBE_LIB if os.path.exists(PROBE_LIB) else build_probe())
    fn = lib.shflbw_probe_stream_store
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_void_p, ctypes.c_longlong, ctypes.c_void_p, ctypes.c_longlong, ctypes.c_int,
                   ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_longlong),
                   ctypes.POINTER(ctypes.c_longlong), ctypes.c_void_p, ctypes.c_void_p]
    X = torch.ones((1024, 8192), dtype=torch.float16, device="cuda:0")
    Y = torch.zeros((4096, 8192), dtype=torch.float16, device="cuda:0")
    sink = torch.zeros(4, dtype=torch.float32, device="cuda:0")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    out = {}
    for name, ld, st in (("stream_only", 1, 0), ("store_only", 0, 1), ("both", 1, 1)):
        lb, sb = ctypes.c_longlong(0), ctypes.c_longlong(0)

        def step():
            rc = fn(ctypes.c_void_p(X.data_ptr()), 8192, ctypes.c_void_p(Y.data_ptr()), 8192, ld, st, 3, 3,
                    ctypes.byref(lb), ctypes.byref(sb), ctypes.c_void_p(sink.data_ptr()), stream)
            assert rc == 0
        ms = time_steps(step, 20, 5)
        out[name] = {"ms": ms, "load_bytes": lb.value, "store_bytes": sb.value,
                     "TBps": (lb.value + sb.value) / (ms * 1e-3) / 1e12}
    out["both_over_sum_of_parts"] = out["both"]["ms"] / (out["stream_only"]["ms"] + out["store_only"]["ms"])
    return out


def check_sample(p, rows, samples):
    """The rows `rows` of every output buffer the timed launches wrote, against the oracle
    (element-wise, the parity tests' bound)."""
    from oracle import c_oracle
    Yr, S = c_oracle.spmm(np.ascontiguousarray(p.W[rows]), np.ascontiguousarray(p.mask[rows]), p.X)
    worst = 0.0
    for y in samples:
        err = np.abs(y.astype(np.float64) - Yr)
        ok_zero = bool(np.all(y[S == 0] == 0))
        # a binary16 result may sit 2^-25 from the exact one whatever S is (subnormal spacing)
        ratio = float(np.max(np.where(S > 0, np.maximum(err - 2.0 ** -25, 0.0) / np.where(S > 0, S, 1.0), 0.0)))
        worst = max(worst, ratio if ok_zero and np.all(np.isfinite(y)) else float("inf"))
    return {"rows_checked": int(len(rows)), "buffers_checked": len(samples), "max_scaled_error": worst,
            "bound": 2.0 ** -10, "ok": bool(worst <= 2.0 ** -10)}


def cpu_baseline(p):
    """The oracle as it stands, on the host cores, on the full headline
    workload (values only, no tolerance scale), best of two runs."""
    from oracle import c_oracle
    best = None
    for _ in range(2):
        t = time.perf_counter()
        c_oracle.spmm(p.W, p.mask, p.X, want_scale=False)
        dt = time.perf_counter() - t
        best = dt if best is None else min(best, dt)
    flop = 2.0 * p.nnz * p.N
    return dict(value=flop / best / 1e12, unit="TFLOP/s", cores=c_oracle.num_threads(),
                kind="oracle", sample="full workload (4096x1024 by 1024x8192, 75%% sparse), "
                "best of 2 runs, %.2f s each" % best, seconds=best)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--all", action="store_true", help="also run the other configs (extra JSON file)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-baseline leg")
    ap.add_argument("--tile-n", type=int, default=0)
    ap.add_argument("--kernel", type=int, default=0, help="0 auto, 1 gather, 2 slab")
    ap.add_argument("--headline-only", action="store_true",
                    help="time only the headline workload (for a kernel trace whose average is that workload's)")
    ap.add_argument("--pmc", action="store_true",
                    help="counter-collection run: one 64 MiB device copy (calibration) and three "
                         "launches of the headline workload, nothing else")
    ap.add_argument("--pmc-workload", default="headline", choices=["headline", "conv", "layernorm", "config5"],
                    help="what --pmc launches three times after the calibration copy")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); with more, the product would "
              "shard over the columns of X without any exchange between GPUs", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2203_05016_amd import synth
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    p = synth.config(1)
    if args.pmc:
        # FETCH_SIZE / WRITE_SIZE of the copy (64 MiB read, 64 MiB written) give the
        # factor that turns the counters' units into bytes for the kernel's rows
        src = torch.zeros(32 << 20, dtype=torch.float16, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        if args.pmc_workload == "conv":
            measure_conv(synth.config(3), 3, 0, pairs=3)
        elif args.pmc_workload == "layernorm":
            measure_layernorm_transpose(p, 3, 0)
        elif args.pmc_workload == "config5":
            q = Case(synth.config(4, variant=1), 2)
            for _ in range(3):
                q.step()
        else:
            c = Case(p, 3, tile_n=args.tile_n, kernel=args.kernel)
            for _ in range(3):
                c.step()
        torch.cuda.synchronize()
        print(json.dumps({"pmc_run": True, "workload": args.pmc_workload,
                          "copy_bytes_each_way": 64 << 20, "launches": 3}))
        return
    check_rows = np.sort(np.random.Generator(np.random.PCG64(77)).choice(p.M, 24, replace=False))
    main_r = measure_spmm(p, args.steps, args.warmup, cold=True, tile_n=args.tile_n, kernel=args.kernel,
                          sample_rows=check_rows)
    main_sample = main_r.pop("sample")
    if args.headline_only:
        achieved = main_r["bytes"] / (main_r["ms"] * 1e-3)
        print(json.dumps({"metric": "useful TFLOP/s (2*nnz*N/s), Shfl-BW SpMM at 75% sparsity, V=32",
                          "value": main_r["tflops"], "unit": "TFLOP/s", "ms_per_step": main_r["ms"],
                          "steps": args.steps, "warmup": args.warmup,
                          "roofline": {"bound": "hbm", "achieved": achieved / 1e9, "peak": HBM_PEAK / 1e9,
                                       "unit": "GB/s", "frac": achieved / HBM_PEAK}}))
        return
    warm_r = measure_spmm(p, args.steps, args.warmup, cold=False, tile_n=args.tile_n, kernel=args.kernel)
    dense_p = synth.config(1, sparsity=0.0)
    # the two legs of the speedup are timed alike: same steps, same warm-up, same rotation rule
    dense_r = measure_spmm(dense_p, args.steps, args.warmup, cold=True,
                           tile_n=args.tile_n, kernel=args.kernel, sample_rows=check_rows)
    dense_sample = dense_r.pop("sample")
    ident_p = synth.config(1, identity_perm=True)
    ident_r = measure_spmm(ident_p, args.steps, args.warmup, cold=True, tile_n=args.tile_n, kernel=args.kernel)
    conv_r = measure_conv(synth.config(3), args.steps, args.warmup)
    conv_dense = measure_conv(synth.config(3, sparsity=0.0), args.steps, args.warmup)
    conv_r["speedup_vs_own_dense"] = conv_dense["ms"] / conv_r["ms"]
    conv_r["dense_ms"] = conv_dense["ms"]
    bf16_r = measure_spmm(synth.config(1, fmt="bf16"), args.steps, args.warmup, cold=True,
                          tile_n=args.tile_n, kernel=args.kernel)
    ln_r = measure_layernorm_transpose(p, args.steps, args.warmup)
    ln_r["fraction_of_headline_time"] = ln_r["ms"] / main_r["ms"]
    l2_r = measure_l2_stream(p)
    # bytes the headline kernel pulls from the L2s into its CUs per launch (TCP_TCC_READ_REQ x 128 B,
    # profiles/slab_kernel_ffn_config2_pmc.md) over its launch time, against the probe's rates
    counters_apply = args.kernel == 0 and args.tile_n == 0 and main_r["kernel"] == COUNTER_KERNEL
    if counters_apply:
        l2_r["kernel_l2_bytes_per_launch"] = L2_TO_CU_BYTES
        l2_r["kernel_l2_bytes_source"] = COUNTER_SOURCE
        l2_r["kernel_l2_GBps"] = L2_TO_CU_BYTES / (main_r["ms"] * 1e-3) / 1e9
        l2_r["frac_of_hot_stream"] = l2_r["kernel_l2_GBps"] / l2_r["hot"]["GBps"]
    lds_r = measure_lds_read()
    path_r = measure_stream_store()
    lib_r = measure_library_gemm(p, args.steps, args.warmup)
    lib_r["sparse_speedup_over_library_dense"] = lib_r["ms"] / main_r["ms"]

    # every GPU leg is timed before the CPU leg: the oracle's worker threads keep the host's
    # cores busy for a while after it returns, which slows the issue of small launches
    extra_file = None
    if args.all:
        extra = {}
        for variant in range(9):
            q = synth.config(2, variant=variant)
            r = measure_spmm(q, args.steps, args.warmup, cold=True, graph=True)
            d = measure_spmm(synth.config(2, variant=variant, sparsity=0.0), args.steps, args.warmup, cold=True)
            extra["config3_V%d_s%.2f" % (q.V, r["sparsity"])] = dict(r, dense_ms=d["ms"], dense_kernel=d["kernel"],
                                                                    speedup=d["ms"] / r["ms"])
        for variant in (3, 2, 1, 0):
            q = synth.config(4, variant=variant)
            r = measure_spmm(q, 10, 2, cold=True)
            extra["config5_s%.3f" % r["sparsity"]] = r
            del q
        # matrix-vector-like regime (recurrent layers): few output columns
        for (M, K, N, V, sp) in ((4096, 4096, 64, 32, 0.75), (4096, 1024, 128, 32, 0.75)):
            q = synth.make_spmm(M, K, N, V, sp, seed=synth.BASE_SEED + 7000 + N)
            r = measure_spmm(q, args.steps, args.warmup, cold=True, graph=True)
            r1 = measure_spmm(q, args.steps, args.warmup, cold=True, kernel=1)
            extra["skinny_%dx%dx%d_s%.2f" % (M, K, N, sp)] = dict(r, whole_tile_gather_ms=r1["ms"])
        extra["conv_shapes_batch32_V32_s0.75"] = measure_conv_shapes(50, 5)
        # config 4's tensor with the other group sizes (all through the staged kernel), and V = 128
        # on a large layer through the shared-slab kernel
        for V in (16, 64, 128):
            r = measure_conv(synth.config(3, V=V), args.steps, args.warmup)
            r["kernel"] = binding_last_kernel()
            extra["conv_config4_shape_V%d_s0.75" % V] = r
        for sp in (0.0, 0.75):
            q = synth.make_spmm(4096, 4096, 8192, 128, sp, seed=synth.BASE_SEED + 7128)
            extra["V128_4096x4096x8192_s%.2f" % sp] = measure_spmm(q, 30, 5, cold=True)
        os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
        with open(os.path.join(ROOT, "gpurun_out", "bench_all.json"), "w") as f:
            json.dump(extra, f, indent=1)
        extra_file = "gpurun_out/bench_all.json"
    cpu = None if args.no_cpu else cpu_baseline(p)
    # result check of what the timed launches left behind (oracle: part of the CPU leg)
    checks = None
    if not args.no_cpu:
        checks = {"headline": check_sample(p, check_rows, main_sample),
                  "dense_run": check_sample(dense_p, check_rows, dense_sample)}

    achieved = main_r["bytes"] / (main_r["ms"] * 1e-3)
    out = {
        "metric": "useful TFLOP/s (2*nnz*N/s), Shfl-BW SpMM at 75% sparsity, V=32",
        "value": main_r["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": main_r["ms"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "configs[1]: Transformer-big FFN SpMM, W 4096x1024 fp16, V=32, "
                               "75% sparsity, X 1024x8192 fp16, Y fp16, cold operands",
                   "M": p.M, "K": p.K, "N": p.N, "V": p.V, "nnz": main_r["nnz"],
                   "rotating_buffer_pairs": main_r["rotate"]},
        "roofline": {"bound": "hbm", "achieved": achieved / 1e9, "peak": HBM_PEAK / 1e9,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK,
                     "traffic": MEASURED_TRAFFIC_BYTES if counters_apply else None,
                     "traffic_source": COUNTER_SOURCE if counters_apply else None,
                     "algorithmic_bytes_per_launch": main_r["bytes"],
                     "kernel": main_r["kernel"]},
        "mfma_peak_frac_useful": main_r["tflops"] * 1e12 / MFMA_F16_PEAK,
        "speedup_vs_own_dense": dense_r["ms"] / main_r["ms"],
        "dense_run": {"ms": dense_r["ms"], "tflops": dense_r["tflops"], "kernel": dense_r["kernel"],
                      "steps": args.steps, "warmup": args.warmup,
                      "mfma_peak_frac": dense_r["tflops"] * 1e12 / MFMA_F16_PEAK},
        "result_check": checks,
        "warm_cache": {"ms": warm_r["ms"], "tflops": warm_r["tflops"]},
        "identity_perm": {"ms": ident_r["ms"], "shuffled_over_identity": main_r["ms"] / ident_r["ms"]},
        "conv2d_config4": conv_r,
        "bf16_operands": {"ms": bf16_r["ms"], "tflops": bf16_r["tflops"]},
        "layernorm_transpose": ln_r,
        "l2_stream_probe": l2_r,
        "lds_read_probe": lds_r,
        "cu_memory_path_probe": path_r,
        "library_dense_gemm": lib_r,
        "cpu_baseline": cpu,
        "context": PAPER_CONTEXT,
    }
    if extra_file:
        out["extra_file"] = extra_file
    print(json.dumps(out))
    if checks and not all(c["ok"] for c in checks.values()):
        print("bench.py: the timed launches left results outside the parity bound: %r" % checks, file=sys.stderr)
        sys.exit(3)


if __name__ == "__main__":
    main()
