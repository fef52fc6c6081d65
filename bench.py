#!/usr/bin/env python3
"""Bench of the RMM linear layer (Algorithm 1 forward + backward) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--kind gaussian|rademacher]

A step is one forward + one backward of a single layer on a synthetic batch that
is already resident in HBM.  The default workload is the headline shape
(N = 4096 tokens, 768 -> 3072, bf16, k = 410 = 10 % of N, Gaussian sketch).
Prints ONE JSON line: whole-step throughput in TFLOP/s of the flops Algorithm 1
executes, the roofline of the slowest stage (timed with HIP events inside the
timed region), and the fp64 oracle timed on the host cores as a plain baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3       # MI355X fp32 vector
PEAK_HBM_GBS = 8000.0
CLOCK_WARMUP_S = 0.05          # untimed steps before the warm-up steps (GPU back from idle clocks)

STAGES = ["fwd_Y", "fwd_Xproj", "bwd_dX", "bwd_G", "bwd_dW"]
STAGE_ID = {"fwd_Y": 0, "fwd_Xproj": 1, "bwd_dX": 2, "bwd_G": 3, "bwd_dW": 4}
# One kernel per stage carries its flops; for the two sketch stages that is the product kernel,
# timed without the small kernel that sums the token-slice partials.
KERNEL_STAGE_ID = {"fwd_Y": 0, "fwd_Xproj": 6, "bwd_dX": 2, "bwd_G": 7, "bwd_dW": 4}
# Where the library issues Y with the sketch of X (dX with the sketch of dY) as ONE launch, that
# paired kernel is what a step really runs; the per-product stages above are then timed on the
# separate-launch path (same kernels, one after the other).
PAIR_STAGE_ID = {"fwd_pair": 8, "bwd_pair": 9}
PAIR_PARTS = {"fwd_pair": ("fwd_Y", "fwd_Xproj"), "bwd_pair": ("bwd_dX", "bwd_G")}
KERNEL_NAME = {"fwd_Y": "gemm_mfma_kernel (X, W^T operands)", "fwd_Xproj": "sketch product kernel on X",
               "bwd_dX": "gemm_mfma_kernel (dY, W operands)", "bwd_G": "sketch product kernel on dY",
               "bwd_dW": "gemm_mfma_kernel (G^T, X_proj operands)",
               "fwd_pair": "gemm_pair_kernel (Y = X W^T with the sketch product of X, one launch)",
               "bwd_pair": "gemm_pair_kernel (dX = dY W with the sketch product of dY, one launch)"}


def stage_flops(n, d_in, d_out, k):
    return {"fwd_Y": 2 * n * d_in * d_out, "fwd_Xproj": 2 * n * k * d_in, "bwd_dX": 2 * n * d_in * d_out,
            "bwd_G": 2 * n * k * d_out, "bwd_dW": 2 * k * d_in * d_out}


def stage_bytes(n, d_in, d_out, k, e):
    """Algorithmic HBM bytes of each stage: every operand read once, every result written once, none for S."""
    return {"fwd_Y": e * (n * d_in + d_in * d_out + n * d_out), "fwd_Xproj": e * (n * d_in + k * d_in),
            "bwd_dX": e * (n * d_out + d_in * d_out + n * d_in), "bwd_G": e * (n * d_out + k * d_out),
            "bwd_dW": e * (k * d_out + k * d_in + d_in * d_out)}


def with_pairs(per_stage, shared):
    """Adds the paired kernels to a per-stage dict: the sum of their two products, less what the
    pair shares (the one read of X, of dY)."""
    out = dict(per_stage)
    for pair, (a, b) in PAIR_PARTS.items():
        out[pair] = per_stage[a] + per_stage[b] - shared.get(pair, 0)
    return out


def read_traffic(workload, stage, kernels_version):
    """HBM bytes per launch of `stage` from the committed counter summary (line
    `traffic_bytes_per_launch <workload> <stage> <bytes>` in profiles/hbm_traffic.txt), or None when
    there is none or when it was measured on another version of the kernels (line
    `kernels_version <rmm_version()>`): a stale figure is worse than none."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    found, version = None, None
    for line in open(path):
        t = line.split()
        if len(t) == 2 and t[0] == "kernels_version":
            version = int(t[1])
        if len(t) == 4 and t[0] == "traffic_bytes_per_launch" and t[1] == workload and t[2] == stage:
            found = float(t[3])
    return found if version == kernels_version else None


def cpu_baseline(cfg, kind, budget_s=10.0):
    """fp64 oracle forward + backward of the same layer on the host cores."""
    import numpy as np
    from oracle import rmm as o_rmm
    from paper_2201_13195_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    X, W, dY = synth.layer_inputs(cfg["n"], cfg["d_in"], cfg["d_out"], cfg["dtype"], cfg["seeds"])
    X, W, dY = synth.to_f64(X), synth.to_f64(W), synth.to_f64(dY)
    fl = sum(stage_flops(cfg["n"], cfg["d_in"], cfg["d_out"], cfg["k"]).values())

    def step():
        _, Xp = o_rmm.forward(X, W, None, cfg["k"], kind, cfg["seed"], 0)
        o_rmm.backward(dY, W, Xp, kind, cfg["seed"], 0)

    step()
    t0 = time.perf_counter()
    reps = 0
    while True:
        step()
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or reps >= 500:
            break
    return {"value": fl * reps / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": "%d full forward+backward step(s) of the same workload in fp64 numpy, %.1f s" % (reps, dt),
            "ms_per_step": dt / reps * 1e3}


def sketch_roofline(torch, rmm, binding, dev, kind, kind_name, version, n=16384, d=4096, k=32, reps=30):
    """rmm_sketch (S^T A) at small k on a RoBERTa-large sized operand: bound by one read of A.
    Three operands are rotated (402 MB) so that no call finds its input in the last-level cache.
    `achieved` is that of the streaming product kernel alone (events recorded by the library
    around it); the whole call, with the small kernel that sums the token-slice partials, is
    reported beside it."""
    bufs = [torch.randn((n, d), device=dev).bfloat16() for _ in range(3)]
    out = torch.empty((k, d), dtype=torch.bfloat16, device=dev)
    ws = torch.empty(max(rmm.rmm_workspace_bytes(n, d, d, k, torch.bfloat16, kind, binding.OP_SKETCH), 16),
                     dtype=torch.uint8, device=dev)
    for i in range(3):
        rmm.rmm_sketch(bufs[i], k, kind, 1, i, out=out, ws=ws)
    torch.cuda.synchronize()

    def events():
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in evs:
            a.record()
            b.record()
        torch.cuda.synchronize()
        return evs

    kev, cev = events(), events()
    for i in range(reps):
        cev[i][0].record()
        rmm.rmm_sketch(bufs[i % 3], k, kind, 1, i, out=out, ws=ws, events=kev[i])
        cev[i][1].record()
    torch.cuda.synchronize()
    kms = sum(a.elapsed_time(b) for a, b in kev) / reps
    cms = sum(a.elapsed_time(b) for a, b in cev) / reps
    nbytes = 2 * (n * d + k * d)
    return {"workload": "rmm_sketch N=%d d=%d k=%d (%s), bf16" % (n, d, k, kind_name), "bound": "hbm",
            "kernel": "sketch_smallk_kernel", "achieved": nbytes / (kms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
            "unit": "GB/s", "frac": nbytes / (kms * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "traffic": read_traffic("sketch_n%d_d%d_k%d" % (n, d, k), "product", version), "avg_launch_ms": kms,
            "avg_call_ms": cms, "algorithmic_bytes_per_launch": nbytes}


def variance_monitor(torch, rmm, X, dY, k, kind, reps=30):
    """rmm_variance_stats (Section 2.3 monitors) on the workload's X and dY: one HBM pass for the
    row norms, the X^T dY product with a squared-norm epilogue, a one-wave finalize."""
    n, d_in = X.shape
    d_out = dY.shape[1]
    out = torch.empty((8,), dtype=torch.float64, device=X.device)
    ws = torch.empty(rmm.rmm_workspace_bytes(n, d_in, d_out, k, X.dtype, kind, 3), dtype=torch.uint8, device=X.device)
    for _ in range(3):
        rmm.rmm_variance_stats(X, dY, k, kind, out=out, ws=ws)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record()
        rmm.rmm_variance_stats(X, dY, k, kind, out=out, ws=ws)
        b.record()
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in evs)[reps // 2]
    fl = 2 * n * d_in * d_out
    return {"avg_call_ms": ms, "flops_per_call": fl, "tflops": fl / (ms * 1e-3) / 1e12,
            "alpha": float(out[6]), "d2_rmm_over_d2_sgd": float(out[5] / out[4])}


def bench_stack(args, torch, rmm, synth, dev, kind):
    """The 24-block stack of RoBERTa-large-shaped layers (144 layers, N = 16384, k = 1638): a step
    is the forward sweep that keeps only X_proj + state per layer, then the backward sweep in
    reverse order.  Inputs of one shape are shared by all layers of that shape (device draws);
    every layer has its own sketch state and its own resident X_proj."""
    S, layers = synth.STACK, synth.stack_layers()
    n, k = S["n"], S["k"]
    g = torch.Generator(device=dev)
    g.manual_seed(S["pool_seed_base"])
    pool, ws_bytes = {}, 16
    for L in layers:
        if L["shape"] not in pool:
            pool[L["shape"]] = dict(
                X=torch.randn((n, L["d_in"]), device=dev, generator=g).bfloat16(),
                W=(0.02 * torch.randn((L["d_out"], L["d_in"]), device=dev, generator=g)).bfloat16(),
                dY=torch.randn((n, L["d_out"]), device=dev, generator=g).bfloat16(),
                Y=torch.empty((n, L["d_out"]), dtype=torch.bfloat16, device=dev),
                dX=torch.empty((n, L["d_in"]), dtype=torch.bfloat16, device=dev),
                dW=torch.empty((L["d_out"], L["d_in"]), dtype=torch.bfloat16, device=dev))
        for op in (0, 1):
            ws_bytes = max(ws_bytes, rmm.rmm_workspace_bytes(n, L["d_in"], L["d_out"], k, torch.bfloat16, kind, op))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    xproj = [torch.empty((k, L["d_in"]), dtype=torch.bfloat16, device=dev) for L in layers]

    def step():
        for L in layers:
            b = pool[L["shape"]]
            rmm.rmm_forward(b["X"], b["W"], None, k, kind, L["seed"], L["offset"], Y=b["Y"], X_proj=xproj[L["layer"]], ws=ws)
        for L in reversed(layers):
            b = pool[L["shape"]]
            rmm.rmm_backward(b["dY"], b["W"], xproj[L["layer"]], kind, L["seed"], L["offset"], dX=b["dX"], dW=b["dW"], ws=ws)

    steps, warmup = min(args.steps, 20), min(args.warmup, 3)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    flops = sum(sum(stage_flops(n, L["d_in"], L["d_out"], k).values()) for L in layers)
    saved = sum(k * L["d_in"] * 2 + 16 for L in layers)
    plain = sum(n * L["d_in"] * 2 for L in layers)
    print(json.dumps({
        "metric": "RMM 24-block stack fwd+bwd TFLOP/s (executed flops of Algorithm 1), N=16384, d=1024/4096, k=1638",
        "value": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "c5_stack: 24 x (4 x 1024->1024, 1024->4096, 4096->1024), N=16384 tokens, k=1638 (%s), "
                               "bf16, all 144 X_proj resident" % args.kind,
                   "flops_per_step": flops, "saved_activation_bytes": saved, "plain_layer_saved_bytes": plain,
                   "saved_fraction": saved / plain}}))
    return 0


class LayerRun:
    """One layer workload resident in HBM (rotating buffer sets) and the calls that make a step."""

    def __init__(self, torch, rmm, binding, synth, dev, cfg, kind, nsets):
        self.torch, self.rmm, self.kind, self.cfg = torch, rmm, kind, cfg
        n, d_in, d_out, k = cfg["n"], cfg["d_in"], cfg["d_out"], cfg["k"]
        tdtype = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
        Xc, Wc, dYc = synth.layer_inputs(n, d_in, d_out, cfg["dtype"], cfg["seeds"])
        self.sets = []
        for _ in range(max(1, nsets)):
            # every set holds the same values (so results are comparable) at its own addresses
            self.sets.append(dict(X=Xc.to(dev).clone(), W=Wc.to(dev).clone(), dY=dYc.to(dev).clone(),
                                  Y=torch.empty((n, d_out), dtype=tdtype, device=dev),
                                  Xp=torch.empty((k, d_in), dtype=tdtype, device=dev),
                                  dX=torch.empty((n, d_in), dtype=tdtype, device=dev),
                                  dW=torch.empty((d_out, d_in), dtype=tdtype, device=dev)))
        ws_bytes = max(rmm.rmm_workspace_bytes(n, d_in, d_out, k, tdtype, kind, binding.OP_FORWARD),
                       rmm.rmm_workspace_bytes(n, d_in, d_out, k, tdtype, kind, binding.OP_BACKWARD), 16)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.bias = self.dbias = None
        self.paired = {"fwd_pair": rmm.rmm_uses_paired_launch(n, d_in, d_out, k, tdtype, kind, binding.OP_FORWARD),
                       "bwd_pair": rmm.rmm_uses_paired_launch(n, d_in, d_out, k, tdtype, kind, binding.OP_BACKWARD)}

    def step(self, i, profile=None):
        b, k, c = self.sets[i % len(self.sets)], self.cfg["k"], self.cfg
        # each pass records the events only if the stage id is one of its own
        self.rmm.rmm_forward(b["X"], b["W"], self.bias, k, self.kind, c["seed"], i, Y=b["Y"], X_proj=b["Xp"], ws=self.ws,
                             profile=profile)
        self.rmm.rmm_backward(b["dY"], b["W"], b["Xp"], self.kind, c["seed"], i, dX=b["dX"], dW=b["dW"], ws=self.ws,
                              profile=profile, dbias=self.dbias, need_dbias=self.dbias is not None)

    def with_bias(self, on):
        """Switch the bias add of the forward pass and the bias gradient of the backward pass on or off."""
        d_out, t = self.cfg["d_out"], self.sets[0]["X"]
        self.bias = self.torch.zeros((d_out,), dtype=t.dtype, device=t.device) if on else None
        self.dbias = self.torch.empty((d_out,), dtype=t.dtype, device=t.device) if on else None

    def new_events(self, count):
        evs = []
        for _ in range(count):
            a, b = self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)
            a.record()
            b.record()          # recording once creates the handles the library re-records
            evs.append((a, b))
        self.torch.cuda.synchronize()
        return evs

    def median_ms(self, stage_id, reps):
        evs = self.new_events(reps)
        for r in range(reps):
            self.step(r, (stage_id, evs[r][0], evs[r][1]))
        self.torch.cuda.synchronize()
        return sorted(a.elapsed_time(b) for a, b in evs)[reps // 2]

    def stage_table(self, reps):
        """(stage ms, ms of the kernel that carries the stage's flops, ms of the paired kernels in use)."""
        stage_ms, kernel_ms, pair_ms = {}, {}, {}
        for name in STAGES:
            stage_ms[name] = self.median_ms(STAGE_ID[name], reps)
            kernel_ms[name] = stage_ms[name] if KERNEL_STAGE_ID[name] == STAGE_ID[name] else \
                self.median_ms(KERNEL_STAGE_ID[name], reps)
        for name, sid in PAIR_STAGE_ID.items():
            if self.paired[name]:
                pair_ms[name] = self.median_ms(sid, reps)
        return stage_ms, kernel_ms, pair_ms

    def step_ms(self, steps, warm_s=0.05):
        # warm up for a twentieth of a second (the inputs were just made on the host: the GPU has been idle
        # and needs some milliseconds of work to come back to its clocks)
        t0, i = time.perf_counter(), 0
        while i < 3 or time.perf_counter() - t0 < warm_s:
            self.step(i)
            i += 1
            if i % 8 == 0:
                self.torch.cuda.synchronize()
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(i)
        self.torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3


def layer_report(run, cfg, kind_name, steps, peaks):
    """Step time and per-kernel TFLOP/s (fraction of the published bf16 peak, and of the measured
    MFMA ceiling when given) of one more workload, for the bench line's side objects."""
    n, d_in, d_out, k = cfg["n"], cfg["d_in"], cfg["d_out"], cfg["k"]
    ms = run.step_ms(steps)
    stage_ms, kernel_ms, pair_ms = run.stage_table(reps=5)
    fl = with_pairs(stage_flops(n, d_in, d_out, k), {})
    kernels = {}
    for name, t in list(kernel_ms.items()) + list(pair_ms.items()):
        tf = fl[name] / (t * 1e-3) / 1e12
        kernels[name] = {"ms": t, "tflops": tf, "frac": tf / PEAK_BF16_TFLOPS}
        if peaks:
            kernels[name]["frac_of_measured_mfma"] = tf / peaks["mfma_bf16_tflops"]
            kernels[name]["frac_of_sustained_mfma"] = tf / peaks["mfma_bf16_tflops_sustained"]
    total = sum(stage_flops(n, d_in, d_out, k).values())
    return {"workload": "N=%d tokens, d_in=%d, d_out=%d, k=%d (%s sketch), bf16" % (n, d_in, d_out, k, kind_name),
            "ms_per_step": ms, "tflops": total / (ms * 1e-3) / 1e12, "steps": steps, "stages_ms": stage_ms,
            "kernels": kernels}


def sors_report(run, cfg, steps, dense_ms):
    """The structured sketch kind (SORS: signs, Walsh-Hadamard transform along the tokens, row
    selection) on the same layer: step time, and its two sketch stages against the HBM roofline
    (algorithmic bytes = one read of the operand + one write of the k selected rows)."""
    n, d_in, d_out, k = cfg["n"], cfg["d_in"], cfg["d_out"], cfg["k"]
    ms = run.step_ms(steps)
    stage_ms, kernel_ms, pair_ms = run.stage_table(reps=5)
    stages = {}
    for name, d in (("fwd_Xproj", d_in), ("bwd_G", d_out)):
        nbytes = 2 * (n * d + k * d)
        gbs = nbytes / (kernel_ms[name] * 1e-3) / 1e9
        stages[name] = {"ms": kernel_ms[name], "algorithmic_bytes": nbytes, "bound": "hbm", "achieved": gbs,
                        "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS}
    return {"workload": "N=%d tokens, d_in=%d, d_out=%d, k=%d (SORS sketch), bf16" % (n, d_in, d_out, k),
            "ms_per_step": ms, "steps": steps, "stages_ms": stage_ms, "paired_kernel_ms": pair_ms, "sketch_stages": stages,
            "step_time_vs_dense_sketch": ms / dense_ms if dense_ms else None}


def library_gemm(torch, run, cfg, kernel_ms, reps=30):
    """The vendor's GEMM library (torch.matmul, bf16) on the three plain products of the layer, same
    shapes and the same rotating buffers: a yardstick beside the hand-written kernels' own times
    (`this_build_ms`, event-bracketed the same way), not a part of the path."""
    k, d_out = cfg["k"], cfg["d_out"]
    dev = run.sets[0]["X"].device
    G = torch.randn((k, d_out), device=dev).bfloat16()
    fl = stage_flops(cfg["n"], cfg["d_in"], d_out, k)
    products = {
        "fwd_Y": lambda b: torch.matmul(b["X"], b["W"].t(), out=b["Y"]),
        "bwd_dX": lambda b: torch.matmul(b["dY"], b["W"], out=b["dX"]),
        "bwd_dW": lambda b: torch.matmul(G.t(), b["Xp"], out=b["dW"]),
    }
    res = {}
    for name, fn in products.items():
        for i in range(10):
            fn(run.sets[i % len(run.sets)])
        evs = run.new_events(reps)
        for i, (a, b) in enumerate(evs):
            a.record()
            fn(run.sets[i % len(run.sets)])
            b.record()
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in evs)[reps // 2]
        res[name] = {"ms": ms, "tflops": fl[name] / (ms * 1e-3) / 1e12, "this_build_ms": kernel_ms[name]}
    return res


def measured_peaks(torch, rmm, dev, reps=5):
    """What a kernel that only issues MFMAs, and one that only reads memory, reach on this machine
    (rmm_probe_mfma on one work-group per compute unit; rmm_probe_read over three rotating 512 MiB
    buffers, larger together than the last-level cache)."""
    sink = torch.zeros(1024, dtype=torch.uint8, device=dev)
    cus = torch.cuda.get_device_properties(dev).multi_processor_count

    def timed(fn):
        best = None
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            work = fn()
            b.record()
            torch.cuda.synchronize()
            rate = work / (a.elapsed_time(b) * 1e-3)
            best = rate if best is None or rate > best else best
        return best

    rmm.rmm_probe_mfma(cus, 200, sink)
    mfma = timed(lambda: rmm.rmm_probe_mfma(cus, 20000, sink)) / 1e12
    # the same loop held for about a quarter of a second: what the matrix pipes sustain once the
    # power management has settled (the layer's kernels run in that regime)
    for _ in range(30):
        rmm.rmm_probe_mfma(cus, 20000, sink)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    work = sum(rmm.rmm_probe_mfma(cus, 20000, sink) for _ in range(30))
    b.record()
    torch.cuda.synchronize()
    mfma_sustained = work / (a.elapsed_time(b) * 1e-3) / 1e12
    bufs = [torch.ones(512 << 20, dtype=torch.uint8, device=dev) for _ in range(3)]
    turn = [0]

    def read():
        turn[0] += 1
        return rmm.rmm_probe_read(bufs[turn[0] % 3], cus * 8, sink)

    read()
    hbm = timed(read) / 1e9
    # the same read at the size of the small-k sketch's operand (one launch of about 25 us: ramp-up and
    # drain weigh more than in the 512 MiB read)
    del bufs
    small = [torch.ones(16384 * 4096 * 2, dtype=torch.uint8, device=dev) for _ in range(3)]

    def read_small():
        turn[0] += 1
        return rmm.rmm_probe_read(small[turn[0] % 3], cus * 8, sink)

    for _ in range(3):
        read_small()
    hbm_small = timed(read_small) / 1e9
    return {"mfma_bf16_tflops": mfma, "mfma_bf16_tflops_sustained": mfma_sustained, "hbm_read_gbs": hbm,
            "hbm_read_gbs_128MiB": hbm_small, "compute_units": cus,
            "how": "best of %d launches: 32x32x16 bf16 MFMAs on pseudo-random operands held in registers, one 4-wave work-group per compute unit; "
                   "sustained = launches 31-60 of 60 back to back (about 0.13 s); "
                   "one streaming read of 512 MiB, and one of 128 MiB (three buffers in turn each)" % reps}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c3_base_ffn_up",
                    help="a single-layer config of paper_2201_13195_amd.synth.CONFIGS (default: the headline shape) "
                         "or c5_stack (the 144-layer stack; reports end-to-end time and stored-activation bytes only)")
    ap.add_argument("--kind", default="gaussian", choices=["gaussian", "rademacher"])
    ap.add_argument("--k", type=int, default=0, help="override the sketch size")
    ap.add_argument("--sets", type=int, default=4, help="rotating input/output sets (keeps the working set above the 256 MB last-level cache)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sketch-roofline", action="store_true",
                    help="skip the small-k rmm_sketch measurement against the HBM roofline")
    ap.add_argument("--no-variance-monitor", action="store_true",
                    help="skip timing rmm_variance_stats on the workload's X and dY")
    ap.add_argument("--no-measured-peaks", action="store_true",
                    help="skip the pure-MFMA and streaming-read probes (fractions of measured ceilings)")
    ap.add_argument("--no-extra-workloads", action="store_true",
                    help="skip the RoBERTa-large FFN shape and the other sketch kind (side objects of the line)")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="only run a plain copy of this many MiB (counter calibration) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (no collective or sharded path exists)",
              file=sys.stderr)
        return 2

    import torch
    import paper_2201_13195_amd as rmm
    from paper_2201_13195_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    if args.calibrate_copy:
        # Plain device-to-device copy of a known size, for scaling the FETCH_SIZE / WRITE_SIZE counters.
        nbytes = args.calibrate_copy << 20
        src = torch.ones(nbytes, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": nbytes, "copy_bytes_written": nbytes, "copies": 5}))
        return 0
    if args.workload == "c5_stack":
        return bench_stack(args, torch, rmm, synth, dev, 0 if args.kind == "gaussian" else 1)
    cfg = dict(synth.CONFIGS[args.workload])
    if args.k:
        cfg["k"] = args.k
    kind = rmm.GAUSSIAN if args.kind == "gaussian" else rmm.RADEMACHER
    n, d_in, d_out, k = cfg["n"], cfg["d_in"], cfg["d_out"], cfg["k"]
    esize = 2 if cfg["dtype"] == "bf16" else 4
    version = rmm.rmm_version()

    run = LayerRun(torch, rmm, binding, synth, dev, cfg, kind, args.sets)
    # The inputs were made on the host, which takes seconds: the GPU has been idle and sits at its idle
    # clocks.  A twentieth of a second of the same steps, untimed, brings it back before the W warm-up
    # steps and the timed region (the stated throughput is a steady-state figure).
    run.step_ms(1, warm_s=CLOCK_WARMUP_S)
    for i in range(args.warmup):
        run.step(i)
    torch.cuda.synchronize()
    # the last warm-up steps time every stage once (separate launches) and the paired kernels, to
    # find the slowest kernel of the path a step really takes
    stage_ms, kernel_ms, pair_ms = run.stage_table(reps=5)
    real = dict(pair_ms)
    for pair, parts in PAIR_PARTS.items():
        if pair not in pair_ms:
            for part in parts:
                real[part] = kernel_ms[part]
    real["bwd_dW"] = kernel_ms["bwd_dW"]
    dominant = max(real, key=real.get)
    dom_idx = PAIR_STAGE_ID.get(dominant, KERNEL_STAGE_ID.get(dominant))

    # ---- timed region: exactly `steps` steps, events around the dominant kernel of every step
    # (an event pair costs the stream about 5 us, 5 % of a step at the headline shape: every tenth step
    # carries one, which still samples the dominant kernel all over the timed region)
    EVERY = 10
    evs = run.new_events((args.steps + EVERY - 1) // EVERY)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % EVERY == 0:
            run.step(i, (dom_idx, evs[i // EVERY][0], evs[i // EVERY][1]))
        else:
            run.step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    dom_ms = sum(a.elapsed_time(b) for a, b in evs) / len(evs)
    # what an event pair with nothing between it measures on this stream (for comparing the
    # event-bracketed duration with the profiler's kernel duration; not subtracted anywhere)
    cal = run.new_events(50)
    for a, b in cal:
        a.record()
        b.record()
    torch.cuda.synchronize()
    empty_pair_ms = sorted(a.elapsed_time(b) for a, b in cal)[len(cal) // 2]

    shared = {"fwd_pair": esize * n * d_in, "bwd_pair": esize * n * d_out}     # X / dY is read once by a pair
    fl = with_pairs(stage_flops(n, d_in, d_out, k), {})
    by = with_pairs(stage_bytes(n, d_in, d_out, k, esize), shared)
    total_flops = sum(stage_flops(n, d_in, d_out, k).values())
    ms_per_step = dt / args.steps * 1e3
    value = total_flops / (ms_per_step * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if cfg["dtype"] == "bf16" else PEAK_F32_TFLOPS
    achieved = fl[dominant] / (dom_ms * 1e-3) / 1e12
    saved = k * d_in * esize + 16
    out = {
        "metric": "RMM layer fwd+bwd TFLOP/s (executed flops of Algorithm 1) at N=%d, %d->%d" % (n, d_in, d_out),
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": "%s: N=%d tokens, d_in=%d, d_out=%d, k=%d (%s sketch), %s, X,dY~N(0,1), "
                               "W~N(0,%s), %d rotating buffer sets"
                               % (args.workload, n, d_in, d_out, k, args.kind, cfg["dtype"],
                                  "0.02^2" if cfg["dtype"] == "bf16" else "1/d_in", len(run.sets)),
                   "flops_per_step": total_flops,
                   "saved_activation_bytes": saved, "plain_layer_saved_bytes": n * d_in * esize,
                   "saved_fraction": saved / (n * d_in * esize), "kernels_version": version,
                   "clock_warmup_ms": CLOCK_WARMUP_S * 1e3},
        "roofline": {"bound": "mfma" if cfg["dtype"] == "bf16" else "alu",
                     "kernel": KERNEL_NAME[dominant] if cfg["dtype"] == "bf16" else "gemm_plain_kernel (%s)" % dominant,
                     "stage": dominant, "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": read_traffic(args.workload, dominant, version),
                     "avg_launch_ms": dom_ms, "launches_timed": len(evs), "empty_event_pair_ms": empty_pair_ms,
                     "flops_per_launch": fl[dominant],
                     "algorithmic_bytes_per_launch": by[dominant]},
        "stages_ms": stage_ms, "stage_kernel_ms": kernel_ms, "paired_kernel_ms": pair_ms,
        "stages_tflops": {s: fl[s] / (stage_ms[s] * 1e-3) / 1e12 for s in STAGES},
    }
    bf16 = cfg["dtype"] == "bf16"
    if not args.no_extra_workloads and bf16:
        # the shape the MFMA targets are quoted on, and the other sketch kind at the headline shape
        big = dict(synth.CONFIGS["c4_large_ffn_up"])
        big_run = LayerRun(torch, rmm, binding, synth, dev, big, kind, 2)
        out["large_shape"] = layer_report(big_run, big, args.kind, 20, None)
        out["library_gemm"] = {
            "what": "torch.matmul (the vendor GEMM library) on the plain products, median of 30 event-bracketed calls",
            "headline_shape": library_gemm(torch, run, cfg, kernel_ms),
            "large_shape": library_gemm(torch, big_run, big, {s: v["ms"] for s, v in out["large_shape"]["kernels"].items()})}
        # the same steps with the optional bias (Eq. 1) and its gradient db = dY^T 1 (Eq. 3): one more pass over dY
        bias_ms = {}
        for name, r in (("headline_shape", run), ("large_shape", big_run)):
            steps_b = 50 if r is run else 20
            r.with_bias(True)
            on = r.step_ms(steps_b)
            r.with_bias(False)
            off = r.step_ms(steps_b)  # right after, in the same clock and thermal state
            bias_ms[name] = {"ms_per_step": on, "ms_per_step_without": off, "extra_ms": on - off, "steps": steps_b}
        out["with_bias"] = {
            "what": "ms per step with the bias add in Y and the bias gradient (column sums of dY, HBM-bound) switched on, "
                    "and the same steps without them timed right after",
            "headline_shape": dict(bias_ms["headline_shape"], dY_bytes=esize * n * d_out),
            "large_shape": dict(bias_ms["large_shape"], dY_bytes=esize * big["n"] * big["d_out"])}
        del big_run
        other = rmm.RADEMACHER if kind == rmm.GAUSSIAN else rmm.GAUSSIAN
        out["other_kind"] = layer_report(LayerRun(torch, rmm, binding, synth, dev, cfg, other, args.sets), cfg,
                                         "rademacher" if other == rmm.RADEMACHER else "gaussian", 50, None)
        # the structured sketch kind on both shapes (dense sketch of the main line for comparison)
        out["sors_kind"] = {
            "headline_shape": sors_report(LayerRun(torch, rmm, binding, synth, dev, cfg, rmm.SORS, args.sets), cfg, 50,
                                          ms_per_step),
            "large_shape": sors_report(LayerRun(torch, rmm, binding, synth, dev, big, rmm.SORS, 2), big, 20,
                                       out["large_shape"]["ms_per_step"])}
        # the fp32 data path (plain FMA kernels, full-precision generator) on the headline shape
        f32 = dict(cfg, dtype="f32")
        run32 = LayerRun(torch, rmm, binding, synth, dev, f32, kind, 2)
        ms32 = run32.step_ms(5)
        out["fp32_path"] = {"workload": "N=%d tokens, d_in=%d, d_out=%d, k=%d (%s sketch), f32" % (n, d_in, d_out, k, args.kind),
                            "ms_per_step": ms32, "tflops": total_flops / (ms32 * 1e-3) / 1e12, "bound": "alu",
                            "peak": PEAK_F32_TFLOPS, "frac": total_flops / (ms32 * 1e-3) / 1e12 / PEAK_F32_TFLOPS, "steps": 5}
        del run32
    if not args.no_sketch_roofline:
        out["sketch_hbm_roofline"] = sketch_roofline(torch, rmm, binding, dev, kind, args.kind, version)
    if not args.no_variance_monitor and bf16:
        out["variance_monitor"] = variance_monitor(torch, rmm, run.sets[0]["X"], run.sets[0]["dY"], k, kind)
    if not args.no_measured_peaks:
        # last of the GPU work: a quarter of a second of MFMAs at full power leaves the chip warm, which the
        # workloads above should not pay for
        out["measured_peaks"] = mp = measured_peaks(torch, rmm, dev)
        if bf16:
            out["roofline"]["frac_of_measured_mfma"] = achieved / mp["mfma_bf16_tflops"]
            out["roofline"]["frac_of_sustained_mfma"] = achieved / mp["mfma_bf16_tflops_sustained"]
            for side in ("large_shape", "other_kind"):
                for kern in out.get(side, {}).get("kernels", {}).values():
                    kern["frac_of_measured_mfma"] = kern["tflops"] / mp["mfma_bf16_tflops"]
                    kern["frac_of_sustained_mfma"] = kern["tflops"] / mp["mfma_bf16_tflops_sustained"]
        if "sketch_hbm_roofline" in out:
            out["sketch_hbm_roofline"]["frac_of_measured_read"] = out["sketch_hbm_roofline"]["achieved"] / mp["hbm_read_gbs"]
            out["sketch_hbm_roofline"]["frac_of_measured_read_same_size"] = (
                out["sketch_hbm_roofline"]["achieved"] / mp["hbm_read_gbs_128MiB"])
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, kind)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
