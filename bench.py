#!/usr/bin/env python3
"""Benchmark: shifted-window attention forward+backward on one MI355X.

A step is one pass of the whole hot path over one synthetic batch: for every
layer of the workload (an unshifted and a half-window-shifted attention layer
alternate in the AERIS Swin stack) the forward kernel, then the delta, dK/dV
and dQ kernels.  Inputs are generated on the device before the clock starts.

Prints ONE JSON line.  `value` is model TFLOP/s: 4*d*U forward + 8*d*U backward
per layer, U = unmasked (query, key) pairs; recomputation inside the backward
kernels (18*d*U are executed in total) is not credited.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0

WORKLOADS = {
    # diffusion-ensemble batch on the 0.25-degree grid: the headline workload
    "c5": dict(shape=(4, 720, 1440, 16, 128), win=(60, 60), layers=[(0, 0), (30, 30)],
               mask=2, kind="blend", sigmas=[0.1, 0.5, 1.0, 2.0], bwd=True, seed=5000,
               name="B=4 x 720x1440 grid, 16 heads x 128, 60x60 windows, shift 0/30, SWIN mask"),
    # one GPU's share of a large-model layer
    "c4": dict(shape=(1, 120, 1440, 24, 128), win=(60, 60), layers=[(30, 30)], mask=2,
               kind="blend", sigmas=None, bwd=True, seed=4000,
               name="48 windows 60x60 (2x24 band), 24 heads x 128, shift 30, SWIN mask"),
    # small parity-test configurations (HBM/latency-bound: judge them on GB/s)
    "c1": dict(shape=(1, 64, 128, 4, 32), win=(8, 8), layers=[(0, 0), (4, 4)], mask=2,
               kind="normal", sigmas=None, bwd=False, seed=1000,
               name="64x128 grid, 4 heads x 32, 8x8 windows, shift 0/4, forward only"),
    "c2": dict(shape=(1, 180, 360, 8, 64), win=(12, 12), layers=[(0, 0), (6, 6)], mask=2,
               kind="normal", sigmas=None, bwd=True, seed=2000,
               name="180x360 grid, 8 heads x 64, 12x12 windows, shift 0/6"),
    "c3": dict(shape=(1, 720, 1440, 16, 64), win=(60, 60), layers=[(30, 30)], mask=2,
               kind="normal", sigmas=None, bwd=False, seed=3000,
               name="720x1440 grid, 16 heads x 64, 60x60 windows, shift 30, forward only"),
    # the headline workload through the rotary-embedding entry points (Model Architecture
    # section: queries and keys are rotated before the attention): forward = rotation pass over
    # K + attention kernel (which rotates Q as it loads it and keeps the rotated rows), backward
    # from the rotated operands the forward call kept
    "c5_rope": dict(shape=(4, 720, 1440, 16, 128), win=(60, 60), layers=[(0, 0), (30, 30)],
                    mask=2, kind="blend", sigmas=[0.1, 0.5, 1.0, 2.0], bwd=True, seed=5000,
                    rope=(100.0, 0),
                    name="c5 with axial 2-D RoPE (base 100, window positions) on Q and K"),
    # one of eight window-parallel ranks of the headline workload (SWiPe section: round-robin
    # subsets of the windows): every eighth window of the 12 x 24 grid, full-grid tensor layout
    "c5_share36": dict(shape=(4, 720, 1440, 16, 128), win=(60, 60), layers=[(0, 0), (30, 30)],
                       mask=2, kind="blend", sigmas=[0.1, 0.5, 1.0, 2.0], bwd=True, seed=5000,
                       share=(8, 3),
                       name="c5, windows w = 3 (mod 8) only: 36 of 288 windows (one of 8 ranks)"),
    # the 6-hourly model's windows (Model Architecture section): T = 900, ragged tiles on both sides
    "w30": dict(shape=(1, 720, 1440, 16, 128), win=(30, 30), layers=[(0, 0), (15, 15)], mask=2,
                kind="blend", sigmas=None, bwd=True, seed=6000,
                name="720x1440 grid, 16 heads x 128, 30x30 windows, shift 0/15, SWIN mask"),
}

# rocprofv3 FETCH_SIZE + WRITE_SIZE of one launch at 4 x 1,036,800 rows x 2048 channels
# (profiles/layer_ops_kernel_trace.txt; from that profiling session, not from this run)
LAYER_OPS_TRAFFIC = {"rmsnorm_adaln_fwd": 34.09e9, "rmsnorm_adaln_bwd": 51.04e9,
                     "gate_residual_fwd": 50.97e9, "gate_residual_bwd": 50.98e9,
                     "swiglu_fwd": 25.48e9, "swiglu_bwd": 42.47e9}


class PowerSampler:
    """Board power while a region runs: a thread reads the amdgpu hwmon power file of the first
    card every 50 ms.  summary() is None if the file is not there (nothing else depends on it)."""

    def __init__(self):
        import glob
        self.path = self.cap = None
        for h in sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*")):
            for name in ("power1_input", "power1_average"):
                if os.path.exists(os.path.join(h, name)):
                    self.path = os.path.join(h, name)
                    self.cap = os.path.join(h, "power1_cap")
                    break
            if self.path:
                break
        self.samples, self._stop, self._thread = [], False, None

    def _run(self):
        while not self._stop:
            try:
                self.samples.append(float(open(self.path).read()) / 1e6)
            except (OSError, ValueError):
                pass
            time.sleep(0.05)

    def start(self):
        if self.path:
            import threading
            self.samples, self._stop = [], False
            self._thread = threading.Thread(target=self._run, daemon=True)
            self._thread.start()
        return self

    def summary(self):
        if not self._thread:
            return None
        self._stop = True
        self._thread.join()
        xs = sorted(self.samples)
        if not xs:
            return None
        out = {"median_w": round(xs[len(xs) // 2], 0), "max_w": round(xs[-1], 0), "samples": len(xs),
               "source": "amdgpu hwmon %s, every 50 ms during the timed steps" % os.path.basename(self.path)}
        try:
            out["cap_w"] = round(float(open(self.cap).read()) / 1e6, 0)
        except (OSError, ValueError):
            pass
        return out


def kernel_symbol(stage, head_dim):
    """Name of the kernel the library launches for a stage (its dispatch rule: the dK/dV stage
    has a software-pipelined kernel of its own at head_dim 128)."""
    if stage == "dkdv" and head_dim == 128:
        return "winattn_dkdv_pipe_kernel"
    return "winattn_%s_kernel" % stage


def profiled_traffic(workload, stage, summary="c5_kernels_and_counters.txt"):
    """HBM bytes per launch of a kernel as the committed rocprofv3 counter summary records them
    (lines `TRAFFIC <workload> <stage> <bytes>` in profiles/): measured in that profiling
    session, not in this run, and labelled so.  None when no summary covers the kernel."""
    path = os.path.join(ROOT, "profiles", summary)
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 4 and f[0] == "TRAFFIC" and f[1] == workload and f[2] == stage:
                return {"traffic": float(f[3]),
                        "traffic_source": "profiles/%s (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE "
                                          "of an earlier run of this file)" % summary}
    except OSError:
        pass
    return {"traffic": None}


def unmasked_pairs(H, W, win, shift, mask):
    """Closed form of the oracle's pair count (per batch member and head)."""
    def axis(L, ws, s, masked):
        n = L // ws
        if not masked or s == 0:
            return float(n)
        return (n - 1) + ((ws - s) ** 2 + s ** 2) / ws ** 2
    fy = axis(H, win[0], shift[0], mask in (1, 2))
    fx = axis(W, win[1], shift[1], mask == 2)
    return fy * fx * (win[0] * win[1]) ** 2


def window_pairs(H, W, win, shift, mask, wy, wx):
    """Unmasked (query, key) pairs of one window (seam windows see fewer)."""
    def axis(L, ws, s, masked, idx):
        if not masked or s == 0 or idx != L // ws - 1:
            return 1.0
        return ((ws - s) ** 2 + s ** 2) / ws ** 2
    return (axis(H, win[0], shift[0], mask in (1, 2), wy) * axis(W, win[1], shift[1], mask == 2, wx)
            * (win[0] * win[1]) ** 2)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c5", choices=sorted(WORKLOADS) + ["layer_ops", "qkv_proj", "qkv_proj_bwd", "layer"],
                    help="layer_ops: the element-wise kernels of include/aeris_layer_ops.h on the "
                         "headline grid's tokens (a bandwidth figure, not the headline metric); "
                         "qkv_proj: the fused RMSNorm + modulation + QKV projection and the fused "
                         "SwiGLU up-projection on the same tokens (bf16 MFMA TFLOP/s); "
                         "qkv_proj_bwd: the two gradient GEMMs of the QKV projection; "
                         "layer: one whole transformer layer, forward and backward, on one "
                         "sample of the headline grid, every step by this library")
    ap.add_argument("--channels", type=int, default=2048, help="row width for --workload layer_ops")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-pairs", type=int, default=64)
    ap.add_argument("--no-mfma-loop", action="store_true",
                    help="skip the register-operand MFMA loop that measures the MFMA rate this "
                         "machine sustains under its power limit (about one second)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="end with three 1 GiB read + 1 GiB write elementwise kernels "
                         "(the last three dispatches), to scale rocprofv3 FETCH_SIZE/WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (pairs of (batch, window, head) are "
                 "independent, so more GPUs would each run this same kernel on their share); "
                 "--gpus %d is not supported" % args.gpus)

    import numpy as np
    import torch
    from paper_2509_13523_amd import binding as B
    from paper_2509_13523_amd import synth

    B.load()   # fails loudly if the HIP library is not built
    if args.workload == "layer_ops":
        return bench_layer_ops(args)
    if args.workload == "qkv_proj":
        return bench_projections(args)
    if args.workload == "qkv_proj_bwd":
        return bench_projection_bwd(args)
    if args.workload == "layer":
        return bench_layer(args)
    wl = WORKLOADS[args.workload]
    shape, win, mask = wl["shape"], wl["win"], wl["mask"]
    Bn, H, W, nh, d = shape
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    n_in = 4 if wl["bwd"] else 3
    tensors = synth.make_inputs_device(wl["kind"], wl["seed"], shape, n_in, sigmas=wl["sigmas"],
                                       device=dev)
    tq, tk, tv = tensors[:3]
    tdo = tensors[3] if wl["bwd"] else None
    o = torch.empty_like(tq)
    lse = torch.empty((Bn, nh, H, W), dtype=torch.float32, device=dev)
    if wl["bwd"]:
        dq, dk, dv = torch.empty_like(tq), torch.empty_like(tq), torch.empty_like(tq)
        p0 = B.make_params(shape, win, (0, 0), mask)
        ws = torch.empty(B.aeris_winattn_bwd_workspace_bytes(p0), dtype=torch.uint8, device=dev)
    rope, share = wl.get("rope"), wl.get("share")
    nwx = W // win[1]
    picks = None
    if share:
        picks = [w for w in range((H // win[0]) * nwx) if w % share[0] == share[1]]
        lst = torch.tensor(picks, dtype=torch.int32, device=dev)
    if rope:
        fws = torch.empty(B.aeris_winattn_rope_fwd_workspace_bytes(p0), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    if picks is None:
        U = {s: Bn * nh * unmasked_pairs(H, W, win, s, mask) for s in wl["layers"]}
    else:
        U = {s: Bn * nh * sum(window_pairs(H, W, win, s, mask, w // nwx, w % nwx) for w in picks)
             for s in wl["layers"]}
    model_flops = sum((12 if wl["bwd"] else 4) * d * U[s] for s in wl["layers"])
    kernel_flops = {"fwd": 4, "dq": 6, "dkdv": 8, "bwd": 14}
    events = {k: [] for k in kernel_flops}

    def timed(name, fn, record):
        if not record:
            fn()
            return
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        events[name].append((e0, e1))

    def step_calls(record):
        """Workloads that go through entry points without a per-kernel split: one event pair
        per call (forward call, backward call)."""
        for s in wl["layers"]:
            if rope:
                timed("fwd", lambda: B.aeris_winattn_rope_fwd(
                    tq, tk, tv, win, s, rope[0], rope[1], mask, o=o, lse=lse, workspace=fws), record)
                timed("bwd", lambda: B.aeris_winattn_rope_bwd(
                    tq, tk, tv, o, lse, tdo, win, s, rope[0], rope[1], mask, workspace=ws,
                    saved=fws, dq=dq, dk=dk, dv=dv), record)
            else:
                timed("fwd", lambda: B.aeris_winattn_fwd_windows(tq, tk, tv, win, s, lst, o, lse,
                                                                 mask), record)
                timed("bwd", lambda: B.aeris_winattn_bwd_windows(
                    tq, tk, tv, o, lse, tdo, win, s, lst, dq, dk, dv, mask=mask, workspace=ws),
                    record)

    def step_plain(record):
        for s in wl["layers"]:
            timed("fwd", lambda: B.aeris_winattn_fwd(tq, tk, tv, win, s, mask, o=o, lse=lse),
                  record)
            if wl["bwd"]:
                # the backward pass as aeris_winattn_bwd runs it, one event pair per kernel: the
                # dQ kernel (which also produces delta and LSE*log2e), then the dK/dV kernel
                for name, st in (("dq", B.AERIS_BWD_DELTA | B.AERIS_BWD_DQ),
                                 ("dkdv", B.AERIS_BWD_DKDV)):
                    timed(name, lambda: B.aeris_winattn_bwd_stages(
                        tq, tk, tv, o, lse, tdo, win, s, mask, dq=dq, dk=dk, dv=dv,
                        workspace=ws, stages=st), record)

    step = step_calls if (rope or share) else step_plain
    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    step_marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    power = PowerSampler().start()
    t0 = time.perf_counter()
    step_marks[0].record()
    for i in range(args.steps):
        step(True)
        step_marks[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    board_power = power.summary()
    ms_per_step = elapsed * 1e3 / args.steps
    value = model_flops / (ms_per_step * 1e-3) / 1e12
    step_ms = sorted(a.elapsed_time(b) for a, b in zip(step_marks, step_marks[1:]))

    def median(xs):
        xs = sorted(xs)
        n = len(xs)
        return xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])

    kern = {}
    layers = len(wl["layers"])
    for name, evs in events.items():
        if evs:
            times = [a.elapsed_time(b) for a, b in evs]
            ms = sum(times) / len(times)
            kern[name] = {"avg_ms": round(ms, 4), "launches": len(evs)}
            # median and minimum per layer kind (the masked layer does less work)
            for li, s in enumerate(wl["layers"]):
                ts = times[li::layers]
                kern[name]["shift%d" % s[0]] = {"median_ms": round(median(ts), 4),
                                                "min_ms": round(min(ts), 4)}
            if kernel_flops[name]:
                fl = kernel_flops[name] * d * sum(U.values()) / len(U)
                kern[name]["tflops_executed"] = round(fl / (ms * 1e-3) / 1e12, 2)
    dom = max((k for k in kern if kernel_flops[k]), key=lambda k: kern[k]["avg_ms"] * len(events[k]))
    dom_flops = kernel_flops[dom] * d * sum(U.values()) / len(U)
    achieved = dom_flops / (kern[dom]["avg_ms"] * 1e-3) / 1e12
    dom_name = (kernel_symbol("dq", d) + " + " + kernel_symbol("dkdv", d) if dom == "bwd"
                else kernel_symbol(dom, d))
    roofline = {"kernel": dom_name, "bound": "mfma", "achieved": round(achieved, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_BF16_TFLOPS, 4)}
    roofline.update(profiled_traffic(args.workload, dom))
    extra = {}
    if rope or share:
        # the same layers through the plain full-grid entry points, timed in this run, so that the
        # cost of the rotation / the efficiency of a share is a figure of this run
        step_plain(False)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            step_plain(False)
        e1.record()
        torch.cuda.synchronize()
        plain_ms = e0.elapsed_time(e1) / 3
        extra["plain_full_grid_ms_per_step"] = round(plain_ms, 3)
        if rope:
            extra["rope_overhead_pct"] = round(100 * (ms_per_step / plain_ms - 1), 2)
        else:
            extra["share_rate_vs_full_grid"] = round(plain_ms * len(picks) /
                                                    ((H // win[0]) * nwx) / ms_per_step, 4)

    out = {"metric": "window-attn fwd+bwd TFLOP/s (model FLOPs) and % bf16 MFMA peak, "
                     "720x1440 grid, 60x60 win",
           "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
           "ms_per_step_median": round(median(step_ms), 3), "ms_per_step_min": round(step_ms[0], 3),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic", "pct_bf16_mfma_peak": round(100 * value / PEAK_BF16_TFLOPS, 2),
           "config": {"workload": "%s: %s" % (args.workload, wl["name"]),
                      "passes": "fwd+bwd" if wl["bwd"] else "fwd",
                      "layers_per_step": len(wl["layers"]),
                      "model_tflop_per_step": round(model_flops / 1e12, 2)},
           "kernels": kern, "roofline": roofline}
    out.update(extra)
    out["board_power"] = board_power
    # algorithmic HBM bytes per step: fwd reads Q,K,V and writes O, LSE; bwd reads Q,K,V,O,dO
    # twice over its three kernels (O,dO; Q,K,V,dO; Q,K,V,dO) and writes dQ,dK,dV
    tensor = 2.0 * Bn * H * W * nh * d
    if picks is not None:
        tensor *= len(picks) / ((H // win[0]) * nwx)
    step_bytes = len(wl["layers"]) * ((4 + (13 if wl["bwd"] else 0)) * tensor)
    out["algorithmic_gbs"] = round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1)

    if not args.no_mfma_loop:
        # the MFMA rate the machine sustains on random operands (power-limited clock), measured
        # right after the timed steps: context for roofline.frac, which stays against the
        # published peak
        sink = torch.empty(512 * 256, dtype=torch.float32, device=dev)
        B.aeris_mfma_loop_probe(512, 20000, True, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        loop_power = PowerSampler().start()
        e0.record()
        flop = B.aeris_mfma_loop_probe(512, 600000, True, sink)
        e1.record()
        torch.cuda.synchronize()
        loop_tflops = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
        loop_power = loop_power.summary()
        out["roofline"]["measured_mfma_loop_tflops"] = round(loop_tflops, 1)
        out["roofline"]["measured_mfma_loop_board_power_w"] = loop_power and loop_power["median_w"]
        out["roofline"]["frac_of_measured_loop"] = round(achieved / loop_tflops, 4)
        del sink

    if args.calibrate_copy:
        a = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            torch.add(a, 1.0, out=b)
        torch.cuda.synchronize()
        del a, b

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, tq, tk, tv, tdo, args.cpu_pairs)
    print(json.dumps(out))


def cpu_baseline(wl, tq, tk, tv, tdo, n_pairs):
    """The fp64 oracle, untouched, timed on a bounded sample of (batch, window, head)
    pairs of this workload; reported in the metric's unit (model TFLOP/s)."""
    import numpy as np
    from oracle import winattn_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([t.get("num_threads", 1) for t in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    Bn, H, W, nh, d = wl["shape"]
    win, mask = wl["win"], wl["mask"]
    shift = wl["layers"][-1]
    scale = 1.0 / np.sqrt(d)
    nwy, nwx = H // win[0], W // win[1]
    rng = np.random.default_rng(0)
    flops, secs = 0.0, 0.0
    picks = [(0, 0, 0, 0), (Bn - 1, nwy - 1, nwx - 1, nh - 1), (0, nwy - 1, 1, 1), (0, 0, nwx - 1, 2)]
    while len(picks) < n_pairs:
        picks.append((int(rng.integers(Bn)), int(rng.integers(nwy)), int(rng.integers(nwx)),
                      int(rng.integers(nh))))
    for (b, wy, wx, h) in picks[:n_pairs]:
        y, x, yh, xh = orc.window_tokens(H, W, win, shift, wy, wx)
        reg = orc.token_regions(H, W, win, shift, mask, yh, xh)
        g = lambda t: t[b, :, :, h, :][y, x].float().cpu().numpy().astype(np.float64)
        qw, kw, vw = g(tq), g(tk), g(tv)
        dow = g(tdo) if tdo is not None else None
        t0 = time.perf_counter()
        orc.window_pair_fwd(qw, kw, vw, reg, scale)
        if dow is not None:
            orc.window_pair_bwd(qw, kw, vw, dow, reg, scale)
        secs += time.perf_counter() - t0
        pairs = float((reg[:, None] == reg[None, :]).sum())
        flops += (12 if dow is not None else 4) * d * pairs
    return {"value": round(flops / secs / 1e12, 5), "unit": "TFLOP/s", "cores": int(threads),
            "kind": "oracle",
            "sample": "%d (batch, window, head) pairs of the workload (interior, seam and corner "
                      "windows), fwd%s, %.1f s of CPU time" %
                      (n_pairs, "+bwd" if tdo is not None else "", secs)}


def bench_projections(args):
    """One step = the fused QKV projection (2048 -> 6144) and the fused SwiGLU up-projection
    (2048 -> 2 x 5504, gate in the epilogue) of one layer on 4 x 720 x 1440 token rows.  FLOPs =
    2 * rows * channels * features per GEMM; torch's bf16 matmul (the vendor GEMM) on the same
    shape is timed beside them as context."""
    import numpy as np
    import torch
    from paper_2509_13523_amd import binding as B
    nb, rps, C = 4, 720 * 1440, args.channels
    n, F, hidden = nb * rps, 3 * args.channels, 5504
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    gen = torch.Generator(device=dev).manual_seed(7100)
    x = torch.randn(n, C, device=dev, dtype=torch.bfloat16, generator=gen)
    wqkv = (torch.randn(F, C, device=dev, generator=gen) / C ** 0.5).to(torch.bfloat16)
    wup = (torch.randn(2 * hidden, C, device=dev, generator=gen) / C ** 0.5).to(torch.bfloat16)
    w = 1.0 + 0.1 * torch.randn(C, device=dev, generator=gen)
    gamma = 0.3 * torch.randn(nb, C, device=dev, generator=gen)
    beta = 0.5 * torch.randn(nb, C, device=dev, generator=gen)
    y = torch.empty(n, F, dtype=torch.bfloat16, device=dev)
    g = torch.empty(n, hidden, dtype=torch.bfloat16, device=dev)
    ws = torch.empty(B.aeris_norm_linear_workspace_bytes(n, rps, C, 2 * hidden), dtype=torch.uint8,
                     device=dev)
    ops = [("norm_qkv_projection", lambda: B.aeris_norm_linear_fwd(x, w, gamma, beta, 1e-6, wqkv, rps,
                                                                  y=y, workspace=ws), 2.0 * n * C * F),
           ("norm_swiglu_up_projection", lambda: B.aeris_norm_linear_swiglu_fwd(
               x, w, gamma, beta, 1e-6, wup, rps, g=g, want_uv=False, workspace=ws),
            2.0 * n * C * 2 * hidden)]
    for _ in range(args.warmup):
        for _, fn, _ in ops:
            fn()
    torch.cuda.synchronize()
    ev = {name: [] for name, _, _ in ops}
    power = PowerSampler().start()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        for name, fn, _ in ops:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            ev[name].append((e0, e1))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    board_power = power.summary()
    step_ms = wall * 1e3 / args.steps
    per = {}
    for name, _, fl in ops:
        ts = sorted(a.elapsed_time(b) for a, b in ev[name])
        per[name] = {"median_ms": round(ts[len(ts) // 2], 3), "min_ms": round(ts[0], 3),
                     "tflops": round(fl / (ts[len(ts) // 2] * 1e-3) / 1e12, 1)}
    # context: the vendor GEMM on the QKV shape (no normalisation, no epilogue)
    torch.matmul(x, wqkv.t(), out=y)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(3):
        torch.matmul(x, wqkv.t(), out=y)
    e1.record()
    torch.cuda.synchronize()
    vendor_ms = e0.elapsed_time(e1) / 3
    total = sum(fl for _, _, fl in ops)
    slow = max(ops, key=lambda o: per[o[0]]["median_ms"])
    achieved = per[slow[0]]["tflops"]
    print(json.dumps({
        "metric": "fused_projection_tflops", "value": round(total / (step_ms * 1e-3) / 1e12, 1),
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(step_ms, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic", "board_power": board_power,
        "config": {"workload": "qkv_proj: %d x %d token rows, %d channels -> %d (QKV) and 2 x %d "
                               "(SwiGLU up, gated)" % (nb, rps, C, F, hidden), "kernels": per,
                   "vendor_gemm_qkv_shape_ms": round(vendor_ms, 3),
                   "vendor_gemm_qkv_shape_tflops": round(2.0 * n * C * F / (vendor_ms * 1e-3) / 1e12, 1)},
        "roofline": {"kernel": "norm_linear_gemm_kernel (%s)" % slow[0], "bound": "mfma",
                     "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     **profiled_traffic("qkv_proj", slow[0],
                                        "projection_gemm_kernel_trace_and_counters.txt")}}))


def bench_projection_bwd(args):
    """One step = the two gradient GEMMs of the QKV projection (dx = dy W, dW = dy^T x) on
    4 x 720 x 1440 token rows, 2048 channels, 6144 features.  FLOPs = 2 * rows * channels *
    features each; torch's bf16 matmul (the vendor GEMM) on the same two products beside them."""
    import torch
    from paper_2509_13523_amd import binding as B
    n, C = 4 * 720 * 1440, args.channels
    F = 3 * C
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    gen = torch.Generator(device=dev).manual_seed(7200)
    x = torch.randn(n, C, device=dev, dtype=torch.bfloat16, generator=gen)
    wqkv = (torch.randn(F, C, device=dev, generator=gen) / C ** 0.5).to(torch.bfloat16)
    dy = torch.empty(n, F, device=dev, dtype=torch.bfloat16)
    for i in range(0, n, n // 8):
        dy[i:i + n // 8] = torch.randn(n // 8, F, device=dev, dtype=torch.bfloat16, generator=gen)
    dx = torch.empty_like(x)
    dw = torch.empty(F, C, device=dev, dtype=torch.float32)
    ws = torch.empty(B.aeris_linear_bwd_workspace_bytes(n, C, F), dtype=torch.uint8, device=dev)
    fl = 2.0 * n * C * F
    ops = [("dx", lambda: B.aeris_linear_bwd(None, wqkv, dy, want_dweight=False, dx=dx, workspace=ws)),
           ("dweight", lambda: B.aeris_linear_bwd(x, wqkv, dy, want_dx=False, dweight=dw, workspace=ws))]
    dw16 = torch.empty(F, C, device=dev, dtype=torch.bfloat16)
    vendor = [("dx", lambda: torch.matmul(dy, wqkv, out=dx)),
              ("dweight", lambda: torch.matmul(dy.t(), x, out=dw16))]

    def timed(fn, reps):
        evs = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        return sorted(a.elapsed_time(b) for a, b in evs)

    for _ in range(args.warmup):
        for _, fn in ops:
            fn()
    torch.cuda.synchronize()
    power = PowerSampler().start()
    t0 = time.perf_counter()
    ev = {name: [] for name, _ in ops}
    for _ in range(args.steps):
        for name, fn in ops:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            ev[name].append((e0, e1))
    torch.cuda.synchronize()
    step_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    board_power = power.summary()
    per = {}
    for name, _ in ops:
        ts = sorted(a.elapsed_time(b) for a, b in ev[name])
        per[name] = {"median_ms": round(ts[len(ts) // 2], 3), "min_ms": round(ts[0], 3),
                     "tflops": round(fl / (ts[len(ts) // 2] * 1e-3) / 1e12, 1)}
    ven = {}
    for name, fn in vendor:
        fn()
        ts = timed(fn, 3)
        ven[name] = {"median_ms": round(ts[1], 3), "tflops": round(fl / (ts[1] * 1e-3) / 1e12, 1)}
    slow = min(per, key=lambda k: per[k]["tflops"])
    achieved = per[slow]["tflops"]
    print(json.dumps({
        "metric": "projection_backward_tflops", "value": round(2 * fl / (step_ms * 1e-3) / 1e12, 1),
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(step_ms, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic", "board_power": board_power,
        "config": {"workload": "qkv_proj_bwd: %d token rows, %d channels, %d features: dx = dy W "
                               "(bf16) and dW = dy^T x (fp32)" % (n, C, F), "kernels": per,
                   "vendor_gemm_same_products": ven},
        "roofline": {"kernel": "%s (%s)" % ("linear_wgrad_kernel" if slow == "dweight"
                                            else "norm_linear_gemm_kernel", slow), "bound": "mfma",
                     "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     **profiled_traffic("qkv_proj_bwd", slow,
                                        "projection_gemm_kernel_trace_and_counters.txt")}}))


def bench_layer(args):
    """One step = one AERIS transformer layer (Model Architecture section: adaptive RMSNorm ->
    QKV projection -> rotary shifted-window attention -> output projection -> gated residual;
    adaptive RMSNorm -> SwiGLU feed-forward -> gated residual), forward and backward, on ONE
    sample of the headline grid (720 x 1440 tokens, 2048 channels = 16 heads x 128, 60 x 60
    windows shifted by 30, SWIN mask, hidden width 5504), every step an entry point of this
    library (the residual sums of the backward pass are taken inside the RMSNorm backward
    kernel).  FLOPs: the GEMMs
    (2 N C F each forward, twice that backward) plus the attention's model FLOPs."""
    import ctypes
    import torch
    from paper_2509_13523_amd import binding as B
    H, W, nh, d, hidden = 720, 1440, 16, 128, 5504
    C, N, rps = nh * d, H * W, H * W
    win, shift, mask, base, eps = (60, 60), (30, 30), B.AERIS_MASK_SWIN, 100.0, 1e-6
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    gen = torch.Generator(device=dev).manual_seed(7300)
    bf = lambda *sh, scale=1.0: (torch.randn(*sh, device=dev, generator=gen) * scale).to(torch.bfloat16)
    f32 = lambda *sh, scale=1.0, shift_=0.0: shift_ + scale * torch.randn(*sh, device=dev, generator=gen)
    x, dout = bf(N, C), bf(N, C)
    wqkv, wo = bf(3 * C, C, scale=C ** -0.5), bf(C, C, scale=C ** -0.5)
    wup, wdown = bf(2 * hidden, C, scale=C ** -0.5), bf(C, hidden, scale=hidden ** -0.5)
    w1, w2 = f32(C, scale=0.1, shift_=1.0), f32(C, scale=0.1, shift_=1.0)
    g1, b1, a1 = f32(1, C, scale=0.3), f32(1, C, scale=0.5), f32(1, C, scale=0.8)
    g2, b2, a2 = f32(1, C, scale=0.3), f32(1, C, scale=0.5), f32(1, C, scale=0.8)
    lib = B.load()
    p = B.make_params((1, H, W, nh, d), win, shift, mask, qkv_strides=(3 * C, d))
    rp = B.aeris_rope_params(base, B.AERIS_ROPE_POS_WINDOW)
    u8 = lambda nbytes: torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=dev)
    ws_proj = u8(B.aeris_norm_linear_workspace_bytes(N, rps, C, 2 * hidden))
    ws_attn_f = u8(B.aeris_winattn_rope_fwd_workspace_bytes(p))
    ws_attn_b = u8(B.aeris_winattn_bwd_workspace_bytes(p))
    ws_lin = u8(max(B.aeris_linear_bwd_workspace_bytes(N, C, 2 * hidden),
                    B.aeris_linear_bwd_workspace_bytes(N, hidden, C),
                    B.aeris_linear_bwd_workspace_bytes(N, C, 3 * C)))
    ws_el = u8(max(B.aeris_rmsnorm_adaln_bwd_workspace_bytes(N, rps, C),
                   B.aeris_gate_residual_bwd_workspace_bytes(N, rps, C)))
    lse = torch.empty(1, nh, H, W, dtype=torch.float32, device=dev)
    a = torch.empty(N, C, dtype=torch.bfloat16, device=dev)
    dqkv = torch.empty(N, 3 * C, dtype=torch.bfloat16, device=dev)
    part = lambda t, i: t.data_ptr() + i * C * 2
    log = []

    def op(name, fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        out = fn()
        e1.record()
        log.append((name, e0, e1))
        return out

    def attn_fwd(qkv):
        rc = lib.aeris_winattn_rope_fwd(ctypes.byref(p), ctypes.byref(rp), part(qkv, 0), part(qkv, 1),
                                        part(qkv, 2), a.data_ptr(), lse.data_ptr(), ws_attn_f.data_ptr(),
                                        ws_attn_f.numel(), torch.cuda.current_stream().cuda_stream)
        assert rc == 0, rc

    def attn_bwd(qkv, da):
        rc = lib.aeris_winattn_rope_bwd(ctypes.byref(p), ctypes.byref(rp), part(qkv, 0), part(qkv, 1),
                                        part(qkv, 2), a.data_ptr(), lse.data_ptr(), da.data_ptr(),
                                        part(dqkv, 0), part(dqkv, 1), part(dqkv, 2), ws_attn_f.data_ptr(),
                                        ws_attn_b.data_ptr(), ws_attn_b.numel(),
                                        torch.cuda.current_stream().cuda_stream)
        assert rc == 0, rc

    def step():
        # ---- forward
        qkv = op("norm_qkv_projection", lambda: B.aeris_norm_linear_fwd(x, w1, g1, b1, eps, wqkv, rps, workspace=ws_proj))
        op("attention_fwd", lambda: attn_fwd(qkv))
        y = op("out_projection", lambda: B.aeris_linear_fwd(a, wo))
        x1 = op("gate_residual_fwd", lambda: B.aeris_gate_residual_fwd(x, y, a1, rps))
        g, uv = op("norm_swiglu_up_projection", lambda: B.aeris_norm_linear_swiglu_fwd(
            x1, w2, g2, b2, eps, wup, rps, workspace=ws_proj))
        y2 = op("down_projection", lambda: B.aeris_linear_fwd(g, wdown))
        out = op("gate_residual_fwd", lambda: B.aeris_gate_residual_fwd(x1, y2, a2, rps))
        # ---- backward
        dy2, _ = op("gate_residual_bwd", lambda: B.aeris_gate_residual_bwd(y2, a2, dout, rps, workspace=ws_el))
        dg, dwdown = op("down_projection_bwd", lambda: B.aeris_linear_bwd(g, wdown, dy2, workspace=ws_lin))
        duv = op("swiglu_bwd", lambda: B.aeris_swiglu_bwd(uv, dg))
        h2, r2 = op("rmsnorm_adaln_fwd (recomputed)", lambda: B.aeris_rmsnorm_adaln_fwd(x1, w2, g2, b2, eps, rps))
        dh2, dwup = op("up_projection_bwd", lambda: B.aeris_linear_bwd(h2, wup, duv, workspace=ws_lin))
        dx1 = op("rmsnorm_adaln_bwd", lambda: B.aeris_rmsnorm_adaln_bwd(x1, w2, g2, r2, dh2, rps, workspace=ws_el,
                                                                        dres=dout))[0]
        dy, _ = op("gate_residual_bwd", lambda: B.aeris_gate_residual_bwd(y, a1, dx1, rps, workspace=ws_el))
        da, dwo = op("out_projection_bwd", lambda: B.aeris_linear_bwd(a, wo, dy, workspace=ws_lin))
        op("attention_bwd", lambda: attn_bwd(qkv, da))
        h1, r1 = op("rmsnorm_adaln_fwd (recomputed)", lambda: B.aeris_rmsnorm_adaln_fwd(x, w1, g1, b1, eps, rps))
        dh1, dwqkv = op("qkv_projection_bwd", lambda: B.aeris_linear_bwd(h1, wqkv, dqkv, workspace=ws_lin))
        dx = op("rmsnorm_adaln_bwd", lambda: B.aeris_rmsnorm_adaln_bwd(x, w1, g1, r1, dh1, rps, workspace=ws_el,
                                                                       dres=dx1))[0]
        return out, dx

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    log.clear()
    power = PowerSampler().start()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out, dx = step()
    torch.cuda.synchronize()
    step_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    board_power = power.summary()
    assert bool(torch.isfinite(out.float()).all()) and bool(torch.isfinite(dx.float()).all())
    per = {}
    for name, e0, e1 in log:
        per[name] = per.get(name, 0.0) + e0.elapsed_time(e1) / args.steps
    gemm_fl = 3 * 2.0 * N * C * (3 * C + C + 2 * hidden + hidden)
    attn_fl = 12.0 * d * nh * unmasked_pairs(H, W, win, shift, mask)
    groups = {"attention": ("attention_fwd", "attention_bwd"),
              "projections": tuple(k for k in per if "projection" in k),
              "element-wise": tuple(k for k in per if "projection" not in k and "attention" not in k)}
    print(json.dumps({
        "metric": "layer_fwd_bwd_tflops", "value": round((gemm_fl + attn_fl) / (step_ms * 1e-3) / 1e12, 1),
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(step_ms, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic", "board_power": board_power,
        "config": {"workload": "layer: one transformer layer forward+backward, 1 x %d x %d tokens, %d channels "
                               "(%d heads x %d), windows %dx%d shifted by %d, SWIN mask, rotary, SwiGLU hidden %d"
                               % (H, W, C, nh, d, win[0], win[1], shift[0], hidden),
                   "gemm_tflop": round(gemm_fl / 1e12, 2), "attention_model_tflop": round(attn_fl / 1e12, 2),
                   "ms": {k: round(v, 3) for k, v in per.items()},
                   "ms_by_kind": {k: round(sum(per[n] for n in names), 3) for k, names in groups.items()}},
        "roofline": {"kernel": "whole layer (GEMMs and attention products)", "bound": "mfma",
                     "achieved": round((gemm_fl + attn_fl) / (step_ms * 1e-3) / 1e12, 1),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round((gemm_fl + attn_fl) / (step_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                     "traffic": None}}))


def bench_layer_ops(args):
    """One step = the six element-wise kernels around the attention of one transformer layer
    (RMSNorm + modulation forward and backward, gated residual forward and backward, SwiGLU gate
    forward and backward) on 4 x 720 x 1440 token rows.  Bound by HBM: algorithmic bytes = every
    activation read once and every result written once."""
    import numpy as np
    import torch
    from paper_2509_13523_amd import binding as B
    nb, rps, C = 4, 720 * 1440, args.channels
    n = nb * rps
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    gen = torch.Generator(device=dev).manual_seed(7000)
    x = torch.randn(n, C, device=dev, dtype=torch.bfloat16, generator=gen)
    dh = torch.randn(n, C, device=dev, dtype=torch.bfloat16, generator=gen)
    w = 1.0 + 0.1 * torch.randn(C, device=dev, generator=gen)
    gamma = 0.3 * torch.randn(nb, C, device=dev, generator=gen)
    beta = 0.5 * torch.randn(nb, C, device=dev, generator=gen)
    h, out = torch.empty_like(x), torch.empty_like(x)
    r = torch.empty(n, dtype=torch.float32, device=dev)
    g = torch.empty(n, C // 2, dtype=torch.bfloat16, device=dev)
    ws = torch.empty(B.aeris_rmsnorm_adaln_bwd_workspace_bytes(n, rps, C), dtype=torch.uint8,
                     device=dev)
    ops = [   # name, call, algorithmic bytes
        ("rmsnorm_adaln_fwd", lambda: B.aeris_rmsnorm_adaln_fwd(x, w, gamma, beta, 1e-6, rps, h=h, r=r),
         4 * n * C + 4 * n),
        ("rmsnorm_adaln_bwd", lambda: B.aeris_rmsnorm_adaln_bwd(x, w, gamma, r, dh, rps, workspace=ws),
         6 * n * C + 4 * n),
        ("gate_residual_fwd", lambda: B.aeris_gate_residual_fwd(x, dh, beta, rps, out=out), 6 * n * C),
        ("gate_residual_bwd", lambda: B.aeris_gate_residual_bwd(x, beta, dh, rps, dy=out, workspace=ws),
         6 * n * C),
        ("swiglu_fwd", lambda: B.aeris_swiglu_fwd(x, g=g), 3 * n * C),
        ("swiglu_bwd", lambda: B.aeris_swiglu_bwd(x, g, duv=out), 5 * n * C),
    ]
    for _ in range(args.warmup):
        for _, fn, _ in ops:
            fn()
    torch.cuda.synchronize()
    ev = {name: [] for name, _, _ in ops}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        for name, fn, _ in ops:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            ev[name].append((e0, e1))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = {name: sum(a.elapsed_time(b) for a, b in ev[name]) / args.steps for name in ev}
    ms_min = {name: min(a.elapsed_time(b) for a, b in ev[name]) for name in ev}
    total_bytes = sum(b for _, _, b in ops)
    step_ms = wall * 1e3 / args.steps
    per_kernel = {name: {"ms": round(ms[name], 3), "min_ms": round(ms_min[name], 3),
                         "GBps": round(b / ms[name] / 1e6, 1)}
                  for name, _, b in ops}
    slow = max(ops, key=lambda o: ms[o[0]])
    achieved = slow[2] / ms[slow[0]] / 1e6
    result = {"metric": "layer_ops_algorithmic_bandwidth", "value": round(total_bytes / step_ms / 1e6, 1),
              "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
              "ms_per_step": round(step_ms, 3), "higher_is_better": True, "scaling": "weak",
              "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
              "config": {"workload": "layer_ops: %d x %d token rows x %d channels (bf16), SwiGLU "
                                     "hidden %d" % (nb, rps, C, C // 2), "kernels": per_kernel},
              "roofline": {"bound": "hbm", "kernel": slow[0], "achieved": round(achieved, 1),
                           "peak": 8000.0, "unit": "GB/s", "frac": round(achieved / 8000.0, 4),
                           "traffic": LAYER_OPS_TRAFFIC.get(slow[0]) if C == 2048 else None,
                           "traffic_source": "profiles/layer_ops_kernel_trace.txt (rocprofv3 --pmc, "
                                             "an earlier run of this file)"}}
    if not args.no_cpu_baseline:
        from oracle import block_oracle as bo
        rows = 4096
        x64 = x[:rows].float().cpu().numpy().astype(np.float64)
        g64 = dh[:rows].float().cpu().numpy().astype(np.float64)
        w64 = w.cpu().numpy().astype(np.float64)
        gm, bt = gamma[:1].cpu().numpy().astype(np.float64), beta[:1].cpu().numpy().astype(np.float64)
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 10.0:
            bo.rmsnorm_adaln_fwd(x64, w64, gm, bt, 1e-6, rows)
            bo.rmsnorm_adaln_bwd(x64, w64, gm, bt, 1e-6, rows, g64)
            bo.gate_residual_fwd(x64, g64, bt, rows)
            bo.gate_residual_bwd(x64, bt, g64, rows)
            bo.swiglu_fwd(x64)
            bo.swiglu_bwd(x64, g64[:, :C // 2])
            reps += 1
        secs = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": round(total_bytes * (rows / n) * reps / secs / 1e9, 3),
                                  "unit": "GB/s", "cores": 1, "kind": "oracle",
                                  "sample": "%d rows, %d passes of the six operations, %.1f s; counted "
                                            "in the kernels' algorithmic (bf16) bytes" % (rows, reps, secs)}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
