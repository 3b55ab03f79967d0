#!/usr/bin/env python3
"""Throughput of one ragged, batch-size-weighted SGD step on one MI355X.

A "step" is the whole hot path on one synthetic batch already resident in HBM:
controller (throughputs -> b_k, offsets) + forward + loss + backward with
per-worker gradients + weighted aggregation + SGD update.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet18]

The headline is the largest benchmark configuration (the ResNet-18-shaped net, B = 2048, K = 8,
bf16 operands with fp32 accumulation); the other four configurations are timed in the same run and
reported in the `configs` array of the same line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# dense MFMA peaks and HBM peak of one MI355X (published figures)
PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}
PEAK_HBM_GBS = 8000.0

# contraction kernel classes of a step, per dtype (names of the library's timing classes)
CLASSES = {"f32": ("linear_fwd", "linear_dgrad", "linear_wgrad"), "bf16": ("conv_fwd", "conv_dgrad", "conv_wgrad")}
PREWARM_S = 2.0     # steps are repeated for at least this long before anything is timed (clocks settle)


def layer_flops(layers, in_shape, li, rows):
    """Algorithmic flop of one forward / dgrad / wgrad launch of layer li over `rows` samples."""
    import synth.nets as nets
    L = layers[li]
    if L["op"] == "linear":
        return 2.0 * rows * L["cin"] * L["cout"]
    ho, wo, _ = nets.layer_shapes(layers, in_shape)[li]
    return 2.0 * rows * ho * wo * L["cout"] * L["k"] * L["k"] * L["cin"]


def class_flops(w, cls):
    """Algorithmic flop per step of all launches the timing class `cls` covers.

    bf16 networks: the class covers the convolutions (the classifier head is its own class).
    fp32 networks: the fully connected layers before the classifier head; their input gradients
    exist for every layer but the first."""
    op = "conv" if cls.startswith("conv") else "linear"
    idx = [i for i, L in enumerate(w.layers) if L["op"] == op]
    if op == "linear":
        idx = idx[:-1]                         # the head runs in fused kernels of the loss class
    if cls.endswith("dgrad"):
        idx = [i for i in idx if w.layers[i]["src"] >= 0]
    return sum(layer_flops(w.layers, w.in_shape, i, w.B) for i in idx), idx


def step_tensor_bytes(w):
    """Bytes of activation and gradient tensors one step has to move if every layer reads its operands and
    writes its result exactly once (nothing fused, nothing re-read): a convolution or fully connected layer
    reads its input and writes its output (forward), reads dY and writes dX (input gradient, where one is
    needed), reads dY and X (weight gradient); a batch norm reads its input twice and writes once (forward)
    and reads x and dy and writes dx (backward); pooling and residual adds read and write once each way;
    plus the update's (K + 2) * 4 * P.  ReLUs are folded into their producers."""
    import numpy as np

    import synth.nets as nets
    el = 2 if w.dtype == "bf16" else 4
    shapes = nets.layer_shapes(w.layers, w.in_shape)
    size = lambda i: float(np.prod(w.in_shape if i < 0 else shapes[i]))
    total = 0.0
    for i, L in enumerate(w.layers):
        a, o = size(L["src"]), size(i)
        if L["op"] in ("conv", "linear"):
            total += (a + o) + (a + o) + ((a + o) if L["src"] >= 0 else 0.0)
        elif L["op"] == "bn":
            total += 3 * o + 3 * o
        elif L["op"] == "add":
            total += 3 * o + 3 * o
        elif L["op"] in ("maxpool2", "gap"):
            total += (a + o) + (a + o)
    return total * el * w.B + (w.K + 2) * 4.0 * w.P


def cpu_baseline(w, rows, budget_s=12.0):
    """The CPU oracle timed on the host cores on a sub-batch of the same workload: `rows` rows split
    over the same K workers in the same proportions (the controller run on the same throughputs).
    The K workers' passes run on a thread pool (the oracle's own `pmap` hook), one BLAS thread each."""
    from concurrent.futures import ThreadPoolExecutor

    from threadpoolctl import threadpool_limits

    from oracle import step as oracle_step
    from oracle.controller import controller_run
    rows = min(rows, w.B)
    b, off = controller_run(w.T, rows)
    store = None
    if w.dtype == "bf16":
        from oracle import layers as oracle_layers
        store = oracle_layers.round_bf16
    x = w.x[:rows].reshape((rows,) + tuple(w.in_shape))
    threads = max(1, min(w.K, os.cpu_count() or 1))
    n = 0
    with ThreadPoolExecutor(threads) as ex, threadpool_limits(limits=1):
        t0 = time.perf_counter()
        while True:
            oracle_step.sgd_step(w.layers, w.params, x, w.labels[:rows], off, w.lr, store=store, pmap=ex.map)
            n += 1
            el = time.perf_counter() - t0
            if el >= budget_s:
                break
    what = "full steps of the same workload" if rows == w.B else f"steps on a {rows}-row sub-batch of the same workload"
    return {"value": rows * n / el, "unit": "samples/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n} {what} (b={b}), fp64 numpy, one thread per worker, {el:.1f} s"}


def measured_traffic(workload, key):
    """HBM bytes (per launch, or per step for a kernel class) from the committed counter summary of this
    workload, or None.

    The summary carries the hash of every source file the kernels live in, taken when the counters were;
    a figure for kernels that have changed since is not reported."""
    import hashlib
    import re
    path = os.path.join(ROOT, "profiles", f"step_{workload}_hbm_traffic.md")
    if not os.path.exists(path):
        return None

    def unchanged(src, sha):
        full = os.path.join(ROOT, src)
        return os.path.exists(full) and hashlib.sha256(open(full, "rb").read()).hexdigest() == sha

    for line in open(path):
        m = re.match(r"\s*traffic (.+?) bytes=(\S+) ((?:source=\S+ sha256=[0-9a-f]{64}\s*)+)$", line)
        if not m or m.group(1) != key:
            continue
        pairs = re.findall(r"source=(\S+) sha256=([0-9a-f]{64})", m.group(3))
        if pairs and all(unchanged(src, sha) for src, sha in pairs):
            return float(m.group(2))
    return None


class Job:
    """One workload on the GPU: network, buffers, controller; `step()` is one pass of the hot path."""

    def __init__(self, name, lr=1e-3):
        import torch

        import paper_2503_17469_amd as omni
        import synth
        self.omni, self.torch = omni, torch
        self.w = w = synth.workload(synth.CONFIG_NAMES.index(name))
        self.ctl = omni.ctl_create(w.K, w.B)
        # the dynamic configuration walks the workers' throughputs: a new split of the batch every step
        self.walk = synth.throughput_walk(w.seed, w.K, 200) if name == "cnn3_dynamic" else [w.T]
        self.i = 0
        omni.ctl_set_throughputs(self.ctl, w.T)
        self.b, self.off = omni.ctl_run(self.ctl, w.K)
        self.net = omni.net_create(w.layers, w.in_shape, w.dtype, w.K, w.B)
        self.ws = torch.zeros(omni.net_workspace_bytes(self.net), dtype=torch.uint8, device="cuda")
        self.params = torch.from_numpy(w.params).cuda()
        x = torch.from_numpy(w.x.reshape(w.B, -1)).cuda()
        self.x = x.to(torch.bfloat16) if w.dtype == "bf16" else x
        self.y = torch.from_numpy(w.labels).cuda()
        self.lpw = torch.zeros(w.K, device="cuda")
        self.loss = torch.zeros(1, device="cuda")
        self.lr = lr      # a small learning rate keeps the synthetic problem finite over thousands of steps

    def step(self, params=None):
        omni, w = self.omni, self.w
        omni.ctl_set_throughputs(self.ctl, self.walk[self.i % len(self.walk)])
        self.i += 1
        bb, oo = omni.ctl_run(self.ctl, w.K)
        omni.step(self.net, self.params if params is None else params, self.x, self.y, oo, bb, self.lr, self.ws,
                  self.lpw, self.loss)

    def prewarm(self, min_steps, min_s):
        n, t0 = 0, time.perf_counter()
        while n < min_steps or time.perf_counter() - t0 < min_s:
            self.step()
            n += 1
            if n % 16 == 0:
                self.torch.cuda.synchronize()
        self.torch.cuda.synchronize()
        return n, time.perf_counter() - t0

    def timed(self, steps):
        """(wall seconds, device milliseconds) of `steps` steps, nothing else on the stream in between."""
        torch = self.torch
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        for _ in range(steps):
            self.step()
        ev1.record()
        torch.cuda.synchronize()
        return time.perf_counter() - t0, ev0.elapsed_time(ev1)

    def class_time(self, cls, steps, params=None):
        """Summed device time and number of launches of one kernel class over `steps` steps, every launch
        between HIP events of its own on the stream it runs on (a separate loop: never inside `timed`)."""
        omni = self.omni
        omni.net_timing_sample(self.net, 1)
        omni.net_timing_enable(self.net, cls, -1, 4096)
        for _ in range(steps):
            self.step(params)
        self.torch.cuda.synchronize()
        ms, n = omni.net_timing_read(self.net)
        omni.net_timing_enable(self.net, -1, -1, 1)
        return ms, n

    def rooflines(self, steps):
        """Per contraction class: algorithmic flop of all its launches in a step / their summed duration."""
        w = self.w
        out = []
        for cls in CLASSES[w.dtype]:
            flops, idx = class_flops(w, cls)
            if not idx:
                continue
            ms, n = self.class_time(cls, steps)
            if n == 0:
                continue
            per_step_s = ms * 1e-3 / steps
            ach = flops / per_step_s / 1e12
            label = f"{cls}: all {n // steps} launches of a step, layers {idx[0]}..{idx[-1]}, time-weighted"
            out.append({"bound": "mfma", "kernel": label, "achieved": ach, "peak": PEAK_TFLOPS[w.dtype],
                        "unit": "TFLOP/s", "frac": ach / PEAK_TFLOPS[w.dtype],
                        "traffic": measured_traffic(w.name, cls),
                        "traffic_note": "HBM bytes of all the class's launches in a step, by counters",
                        "flop_per_step": flops,
                        "us_per_step": per_step_s * 1e6, "avg_launch_us": ms * 1e3 / n, "launches": int(n),
                        "steps": steps})
        return out

    def update_roofline(self, steps, momentum=False):
        omni, torch, w = self.omni, self.torch, self.w
        params = None
        if momentum:
            params = self.params.clone()
            vel = torch.zeros_like(params)
            omni.net_set_momentum(self.net, vel, 0.9, 5e-4)
        ms, n = self.class_time("update", steps, params)
        if momentum:
            omni.net_set_momentum(self.net, None, 0.0, 0.0)
        nbytes = (w.K + (4 if momentum else 2)) * 4.0 * w.P
        gbs = nbytes / (ms / max(n, 1) * 1e-3) / 1e9
        r = {"bound": "hbm", "kernel": "weighted reduce + momentum SGD with weight decay" if momentum
             else "weighted reduce + SGD", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
             "frac": gbs / PEAK_HBM_GBS, "traffic": measured_traffic(w.name, "update_momentum" if momentum else "update"),
             "bytes_per_launch": nbytes, "avg_launch_us": ms / max(n, 1) * 1e3, "launches": int(n)}
        if nbytes < 256e6:
            r["note"] = "working set below 256 MB may be served from the Infinity Cache"
        return r

    def close(self):
        self.omni.net_destroy(self.net)
        self.omni.ctl_destroy(self.ctl)
        del self.ws


def copy_ceiling(torch):
    """What a plain device-to-device copy reaches (256 MiB read + 256 MiB written per copy, more than the
    Infinity Cache holds): the practical ceiling beside the 8 TB/s the HBM fractions divide by."""
    src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n = 20
    c0.record()
    for _ in range(n):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    gbs = 2.0 * src.numel() * n / (c0.elapsed_time(c1) * 1e-3) / 1e9
    return {"achieved": gbs, "unit": "GB/s", "bytes_per_copy": 2.0 * (256 << 20),
            "note": "plain device-to-device copy, read + write counted"}


def read_ceiling(torch, omni, K=8, P=11220132):
    """A read-dominated stream of the update kernel's own shape: K + 1 fp32 arrays read, 1 written, far more
    than the Infinity Cache holds (the library's own update kernel on buffers of its own, back to back)."""
    stride = (P + 63) // 64 * 64
    G = torch.ones(K, stride, device="cuda")
    th = torch.zeros(P, device="cuda")
    b = [1] * K
    for _ in range(3):
        omni.weighted_sgd(th, G, b, 1e-6, P=P)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n = 20
    c0.record()
    for _ in range(n):
        omni.weighted_sgd(th, G, b, 1e-6, P=P)
    c1.record()
    torch.cuda.synchronize()
    nbytes = (K + 2) * 4.0 * P
    return {"achieved": nbytes * n / (c0.elapsed_time(c1) * 1e-3) / 1e9, "unit": "GB/s", "bytes_per_launch": nbytes,
            "note": f"update kernel alone, back to back: {K}+1 arrays read, 1 written"}


def asp_variant(job, rounds=50):
    """The asynchronous variant (Algorithm 2) on the same network, data and batch split: simulated
    workers whose speed matches their batch size push in turn; every push is one launch of the push
    kernel followed by that worker's next gradient (forward + backward over its own rows, one worker,
    no update) at the model it has just pulled.  Reports samples/s over all pushes and the push kernel
    against the HBM roofline (model read, gradient read, model written: 12 bytes per parameter)."""
    omni, torch, w, net = job.omni, job.torch, job.w, job.net
    K, B, b, off, lr = w.K, w.B, job.b, job.off, job.lr
    server = job.params.clone()
    nbytes = omni.net_workspace_bytes(net)
    wss = [torch.zeros(nbytes, dtype=torch.uint8, device="cuda") for _ in range(K)]
    lpw = torch.zeros(1, device="cuda")
    loss = torch.zeros(1, device="cuda")
    xs = [job.x[off[k]:off[k + 1]] for k in range(K)]
    ys = [job.y[off[k]:off[k + 1]] for k in range(K)]
    grads = [omni.net_worker_grads(net, wss[k], 1)[0] for k in range(K)]
    n_events = rounds * K
    worker, version = omni.asp_schedule(w.T, b, n_events)

    def compute(k):
        omni.step(net, server, xs[k], ys[k], [0, b[k]], [b[k]], 0.0, wss[k], lpw, loss, 1)

    def run(events):
        for k in events:
            omni.asp_update(server, server, grads[k], lr, b[k], B, True)
            compute(k)

    for k in range(K):
        compute(k)
    run(worker[:2 * K])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(worker)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    samples = sum(b[k] for k in worker)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_push = 200
    e0.record()
    for i in range(n_push):
        omni.asp_update(server, server, grads[i % K], lr, b[i % K], B, True)
    e1.record()
    torch.cuda.synchronize()
    push_s = e0.elapsed_time(e1) * 1e-3 / n_push
    push_bytes = 12.0 * w.P
    gbs = push_bytes / push_s / 1e9
    stale = [e - v for e, v in enumerate(version)][K:]
    return {"value": samples / dt, "unit": "samples/s", "pushes": n_events, "us_per_push": dt / n_events * 1e6,
            "mean_staleness": sum(stale) / max(len(stale), 1), "final_loss": float(loss.item()),
            "roofline_push": {"bound": "hbm", "kernel": "push (server model -= eta_k * g_k)", "achieved": gbs,
                              "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "traffic": None,
                              "bytes_per_launch": push_bytes, "avg_launch_us": push_s * 1e6,
                              "note": "back-to-back launches; working set below 256 MB may be served from the "
                                      "Infinity Cache"}}


def side_config(name, budget_s=1.0):
    """A short measurement of another benchmark configuration for the `configs` array."""
    job = Job(name)
    try:
        n_warm, _ = job.prewarm(5, 0.5)
        wall, _ = job.timed(8)
        steps = max(8, min(4000, int(budget_s / (wall / 8))))
        wall, dev_ms = job.timed(steps)
        roofs = job.rooflines(max(2, min(20, steps)))
        dom = max(roofs, key=lambda r: r["us_per_step"]) if roofs else None
        w = job.w
        out = {"workload": name, "dtype": w.dtype, "K": w.K, "B": w.B, "params": int(w.P), "steps": steps,
               "ms_per_step": wall / steps * 1e3, "device_ms_per_step": dev_ms / steps,
               "value": w.B * steps / wall, "unit": "samples/s", "roofline": dom,
               "roofline_update": job.update_roofline(max(2, min(50, steps)))}
        if name == "mlp3072":
            out["asp_variant"] = asp_variant(job)     # (one workspace per simulated worker: on this workload only)
        return out
    finally:
        job.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100, help="timed steps of the headline workload")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet18")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-side-configs", action="store_true", help="skip the other configurations' short runs")
    ap.add_argument("--no-rooflines", action="store_true", help="headline loop only (for profiling runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on ONE GPU; --gpus must be 1 (no collectives or sharding exist here)")

    import numpy as np
    import torch

    import paper_2503_17469_amd as omni
    import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    job = Job(args.workload)
    w = job.w

    # One plain device-to-device copy of known size (256 MiB read + 256 MiB written): under
    # `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` its counters calibrate the traffic figures.
    cal_src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    # W untimed steps as asked, then more of the same until the GPU has been busy for PREWARM_S seconds:
    # a handful of steps does not bring the clocks up, and a short timed loop would report the ramp
    prewarm_steps, prewarm_s = job.prewarm(args.warmup, PREWARM_S)

    # ---- the headline: exactly K steps, nothing but the steps on the stream
    dt, dev_ms = job.timed(args.steps)
    final_loss = float(job.loss.item())
    assert np.isfinite(final_loss), "loss diverged"
    ms_per_step = dt / args.steps * 1e3
    value = w.B * args.steps / dt

    out = {
        "metric": "samples/sec per ragged weighted SGD step (fwd+bwd+reduce+update)",
        "value": value,
        "unit": "samples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "device_ms_per_step": dev_ms / args.steps,
        "prewarm": {"steps": prewarm_steps, "seconds": prewarm_s,
                    "note": "untimed steps before the timed loop: --warmup of them, then until the time is up"},
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "dtype_note": ("bf16 operands and stored activations, fp32 accumulation, fp32 parameters, gradients, loss "
                       "and update" if w.dtype == "bf16" else "fp32 throughout"),
        "data": "synthetic",
        "config": {"workload": w.name, "K": w.K, "B": w.B, "b": job.b, "params": int(w.P),
                   "includes": "controller+offsets+fwd+loss+bwd+weighted reduce+SGD"},
        "final_loss": final_loss,
    }

    if not args.no_rooflines:
        # spread of single steps: every step of a second loop between two events of its own
        n_each = max(10, min(200, args.steps))
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_each)]
        for e0, e1 in evs:
            e0.record()
            job.step()
            e1.record()
        torch.cuda.synchronize()
        each_us = np.sort(np.array([e0.elapsed_time(e1) * 1e3 for e0, e1 in evs]))
        out["step_spread"] = {"unit": "us", "n": n_each, "median": float(np.percentile(each_us, 50)),
                              "p10": float(np.percentile(each_us, 10)), "p90": float(np.percentile(each_us, 90)),
                              "note": "device time of single steps, each between two events of its own"}
        # contraction classes, each in a loop of its own (event pairs around every launch of the class)
        n_cls = max(5, min(50, args.steps))
        roofs = job.rooflines(n_cls)
        out["roofline"] = max(roofs, key=lambda r: r["us_per_step"])     # the class the step spends most time in
        out["roofline_classes"] = roofs
        total_flop = sum(r["flop_per_step"] for r in roofs)
        out["step_mfma_frac"] = total_flop / (dev_ms / args.steps * 1e-3) / 1e12 / PEAK_TFLOPS[w.dtype]
        nbytes = step_tensor_bytes(w)
        out["step_hbm"] = {"bytes_per_step": nbytes, "achieved": nbytes / (dev_ms / args.steps * 1e-3) / 1e9,
                           "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": nbytes / (dev_ms / args.steps * 1e-3) / 1e9 / PEAK_HBM_GBS,
                           "note": "every layer's operands read once and its result written once, per pass, "
                                   "nothing fused: the unfused method's own traffic, not a counter reading"}
        n_upd = max(10, min(200, args.steps))
        out["roofline_update"] = job.update_roofline(n_upd)
        out["roofline_update_momentum"] = job.update_roofline(n_upd, momentum=True)
        out["hbm_copy_ceiling"] = copy_ceiling(torch)
        out["hbm_read_ceiling"] = read_ceiling(torch, omni)
    job.close()

    if not args.no_side_configs:
        out["configs"] = [side_config(n) for n in synth.CONFIG_NAMES if n != w.name]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, 256 if w.name == "resnet18" else w.B)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
