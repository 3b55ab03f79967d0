#!/usr/bin/env python3
"""Throughput of one ragged, batch-size-weighted SGD step on one MI355X.

A "step" is the whole hot path on one synthetic batch already resident in HBM:
controller (throughputs -> b_k, offsets) + forward + loss + backward with
per-worker gradients + weighted aggregation + SGD update.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mlp3072]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# fp32 dense MFMA peak and HBM peak of one MI355X (published figures)
PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}
PEAK_HBM_GBS = 8000.0

# kernel whose roofline is reported, per workload: (timing class, layer index)
# dominant kernel of every workload: (timing class, layer, roofline that bounds it)
DOMINANT = {
    "tiny_mlp": ("linear_wgrad", 0, "mfma"),
    "mlp3072": ("linear_wgrad", 0, "mfma"),
    # weight gradient of the second conv layer (32 -> 64 channels on 16 x 16 maps): 2 x 9 x 32 x 64 flop per
    # (64 + 32) x 2 bytes of activations = 192 flop per byte, below the chip's ridge point of 312
    "cnn3": ("conv_wgrad", 3, "hbm"),
    "cnn3_dynamic": ("conv_wgrad", 3, "hbm"),
    "resnet18": ("conv_fwd", 3, "mfma"),
}


def layer_flops(layers, in_shape, li, rows):
    """Algorithmic flop of one forward / dgrad / wgrad launch of layer li over `rows` samples."""
    import synth.nets as nets
    L = layers[li]
    if L["op"] == "linear":
        return 2.0 * rows * L["cin"] * L["cout"]
    ho, wo, _ = nets.layer_shapes(layers, in_shape)[li]
    return 2.0 * rows * ho * wo * L["cout"] * L["k"] * L["k"] * L["cin"]


def wgrad_bytes(layers, in_shape, li, rows, K):
    """Algorithmic HBM bytes of one conv weight-gradient launch of layer li: the output gradient and
    the (channel-padded, bf16) layer input read once, K per-worker fp32 gradients written."""
    import synth.nets as nets
    L = layers[li]
    shapes = nets.layer_shapes(layers, in_shape)
    ho, wo, _ = shapes[li]
    hi, wi, ci = in_shape if L["src"] < 0 else shapes[L["src"]]
    ci_pad = (ci + 7) // 8 * 8
    return 2.0 * rows * (ho * wo * L["cout"] + hi * wi * ci_pad) + 4.0 * K * L["cout"] * L["k"] * L["k"] * L["cin"]


def dgrad_bytes(layers, in_shape, li, rows):
    """Algorithmic HBM bytes of one conv data-gradient launch of layer li (bf16): the output gradient read
    once, the input gradient written once, and the layer input read once for the folded ReLU mask."""
    import synth.nets as nets
    L = layers[li]
    shapes = nets.layer_shapes(layers, in_shape)
    ho, wo, _ = shapes[li]
    hi, wi, ci = in_shape if L["src"] < 0 else shapes[L["src"]]
    ci_pad = (ci + 7) // 8 * 8
    return 2.0 * rows * (ho * wo * L["cout"] + 2 * hi * wi * ci_pad)


def cpu_baseline(w, off, budget_s=12.0):
    """The CPU oracle, as it stands, timed on the host cores on the same workload."""
    from oracle import step as oracle_step
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    x = w.x
    store = None
    if w.dtype == "bf16":
        from oracle import layers as oracle_layers
        store = oracle_layers.round_bf16
    n = 0
    t0 = time.perf_counter()
    while True:
        oracle_step.sgd_step(w.layers, w.params, x, w.labels, off, w.lr, store=store)
        n += 1
        el = time.perf_counter() - t0
        if el >= budget_s:
            break
    return {"value": w.B * n / el, "unit": "samples/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n} full steps of the same workload (B={w.B}), fp64 numpy, {el:.1f} s"}


def measured_traffic(workload, key):
    """HBM bytes per launch from the committed counter summary of this workload, or None.

    The summary carries the hash of the kernel's source file at the time the counters were
    taken; a figure for a kernel that has changed since is not reported."""
    import hashlib
    import re
    root = os.path.dirname(os.path.abspath(__file__))
    path = os.path.join(root, "profiles", f"step_{workload}_hbm_traffic.md")
    if not os.path.exists(path):
        return None
    for line in open(path):
        m = re.match(r"\s*traffic (.+?) bytes=(\S+) source=(\S+) sha256=([0-9a-f]{64})\s*$", line)
        if not m or m.group(1) != key:
            continue
        src = os.path.join(root, m.group(3))
        if os.path.exists(src) and hashlib.sha256(open(src, "rb").read()).hexdigest() == m.group(4):
            return float(m.group(2))
    return None


def asp_variant(omni, torch, net, w, b, off, params, x, y, lr, rounds=50):
    """The asynchronous variant (Algorithm 2) on the same network, data and batch split: simulated
    workers whose speed matches their batch size push in turn; every push is one launch of the push
    kernel followed by that worker's next gradient (forward + backward over its own rows, one worker,
    no update) at the model it has just pulled.  Reports samples/s over all pushes and the push kernel
    against the HBM roofline (model read, gradient read, model written: 12 bytes per parameter)."""
    K, B = w.K, w.B
    server = params.clone()
    nbytes = omni.net_workspace_bytes(net)
    wss = [torch.zeros(nbytes, dtype=torch.uint8, device="cuda") for _ in range(K)]
    lpw = torch.zeros(1, device="cuda")
    loss = torch.zeros(1, device="cuda")
    xs = [x[off[k]:off[k + 1]] for k in range(K)]
    ys = [y[off[k]:off[k + 1]] for k in range(K)]
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
    # the push kernel alone, bracketed by events on the stream it is launched on
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000, help="timed steps (use ~50 for resnet18)")
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="mlp3072")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-asp", action="store_true", help="skip the asynchronous-variant measurement")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on ONE GPU; --gpus must be 1 (no collectives or sharding exist here)")

    import numpy as np
    import torch

    import paper_2503_17469_amd as omni
    import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    idx = synth.CONFIG_NAMES.index(args.workload)
    w = synth.workload(idx)

    ctl = omni.ctl_create(w.K, w.B)
    omni.ctl_set_throughputs(ctl, w.T)
    b, off = omni.ctl_run(ctl, w.K)

    net = omni.net_create(w.layers, w.in_shape, w.dtype, w.K, w.B)
    ws = torch.zeros(omni.net_workspace_bytes(net), dtype=torch.uint8, device="cuda")
    params = torch.from_numpy(w.params).cuda()
    x = torch.from_numpy(w.x.reshape(w.B, -1)).cuda()
    if w.dtype == "bf16":
        x = x.to(torch.bfloat16)
    y = torch.from_numpy(w.labels).cuda()
    lpw = torch.zeros(w.K, device="cuda")
    loss = torch.zeros(1, device="cuda")
    # a small learning rate keeps the synthetic problem finite over thousands of steps
    lr = 1e-3

    def one_step():
        omni.ctl_set_throughputs(ctl, w.T)
        bb, oo = omni.ctl_run(ctl, w.K)
        omni.step(net, params, x, y, oo, bb, lr, ws, lpw, loss)

    # One plain device-to-device copy of known size (256 MiB read + 256 MiB written): under
    # `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` its counters calibrate the traffic figures.
    cal_src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()

    # the dominant kernel is bracketed by HIP events on every 8th step of the timed loop (a pair of
    # event packets costs about 3 us on the stream; on every step that is 2 % of this workload's step)
    kcls, klayer, kbound = DOMINANT[w.name]
    sample_every = 8 if args.steps >= 64 else 1
    omni.net_timing_sample(net, sample_every)
    omni.net_timing_enable(net, kcls, klayer, args.steps)
    torch.cuda.synchronize()
    # device-only time of the same loop: two events on the stream the steps are enqueued on
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        one_step()
    ev1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    device_ms_per_step = ev0.elapsed_time(ev1) / args.steps
    k_ms, k_n = omni.net_timing_read(net)
    omni.net_timing_enable(net, -1, -1, 1)
    omni.net_timing_sample(net, 1)
    final_loss = float(loss.item())
    assert np.isfinite(final_loss), "loss diverged"

    ms_per_step = dt / args.steps * 1e3
    value = w.B * args.steps / dt

    # spread of single steps: every step of a second, shorter loop between two events of its own
    # (the event packets add about 3 us to each, which is why the headline loop above has none inside)
    n_each = min(200, args.steps)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_each)]
    for e0, e1 in evs:
        e0.record()
        one_step()
        e1.record()
    torch.cuda.synchronize()
    each_us = np.sort(np.array([e0.elapsed_time(e1) * 1e3 for e0, e1 in evs]))
    step_spread = {"unit": "us", "n": n_each, "median": float(np.percentile(each_us, 50)),
                   "p10": float(np.percentile(each_us, 10)), "p90": float(np.percentile(each_us, 90)),
                   "note": "device time of single steps, each between two events of its own"}

    # the fused weighted-reduce + SGD kernel against the HBM roofline (separate short loop, same buffers)
    n_upd = min(200, args.steps)
    omni.net_timing_enable(net, "update", -1, n_upd)
    for _ in range(n_upd):
        one_step()
    torch.cuda.synchronize()
    u_ms, u_n = omni.net_timing_read(net)
    omni.net_timing_enable(net, -1, -1, 1)
    upd_bytes = (w.K + 2) * 4.0 * w.P
    upd_gbs = upd_bytes / (u_ms / max(u_n, 1) * 1e-3) / 1e9

    # the same kernel with the momentum / weight-decay update of the paper's experiments selected
    # (velocity read and written beside the parameters); on a copy of the parameters, after everything else
    params_m = params.clone()
    vel = torch.zeros_like(params_m)
    omni.net_set_momentum(net, vel, 0.9, 5e-4)
    omni.net_timing_enable(net, "update", -1, n_upd)
    for _ in range(n_upd):
        omni.ctl_set_throughputs(ctl, w.T)
        bb, oo = omni.ctl_run(ctl, w.K)
        omni.step(net, params_m, x, y, oo, bb, lr, ws, lpw, loss)
    torch.cuda.synchronize()
    m_ms, m_n = omni.net_timing_read(net)
    omni.net_timing_enable(net, -1, -1, 1)
    omni.net_set_momentum(net, None, 0.0, 0.0)
    mom_bytes = (w.K + 4) * 4.0 * w.P
    mom_gbs = mom_bytes / (m_ms / max(m_n, 1) * 1e-3) / 1e9

    # the asynchronous variant keeps one workspace per worker; it is measured on the default workload only
    asp = None if (args.no_asp or w.name != "mlp3072") else asp_variant(omni, torch, net, w, b, off, params, x, y, lr)

    # what a plain device-to-device copy reaches on this GPU (256 MiB read + 256 MiB written per copy, more
    # than the Infinity Cache holds): the practical ceiling beside the 8 TB/s the rooflines divide by
    cp_src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
    cp_dst = torch.empty_like(cp_src)
    for _ in range(3):
        cp_dst.copy_(cp_src)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_copy = 20
    c0.record()
    for _ in range(n_copy):
        cp_dst.copy_(cp_src)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 2.0 * cp_src.numel() * n_copy / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del cp_src, cp_dst

    kernel_s = k_ms / max(k_n, 1) * 1e-3
    klabel = f"{kcls}[layer {klayer}]"
    if kbound == "mfma":
        covered = [klayer]
        if kcls == "linear_wgrad":
            # an fp32 network computes the weight gradients of all fully connected layers before the
            # classifier head in one launch, timed as layer 0: its flop are those of all of them
            covered = [i for i, L in enumerate(w.layers) if L["op"] == "linear"][:-1]
            if len(covered) > 1:
                klabel = f"{kcls}[layers {', '.join(str(i) for i in covered)}: one launch]"
        flops = sum(layer_flops(w.layers, w.in_shape, i, w.B) for i in covered)
        achieved = flops / kernel_s / 1e12
        peak, unit = PEAK_TFLOPS[w.dtype], "TFLOP/s"
    else:
        nbytes = (dgrad_bytes(w.layers, w.in_shape, klayer, w.B) if kcls == "conv_dgrad"
                  else wgrad_bytes(w.layers, w.in_shape, klayer, w.B, w.K))
        achieved = nbytes / kernel_s / 1e9
        peak, unit = PEAK_HBM_GBS, "GB/s"
    roofline = {"bound": kbound, "kernel": klabel, "achieved": achieved, "peak": peak,
                "unit": unit, "frac": achieved / peak,
                "traffic": measured_traffic(w.name, klabel),
                "avg_launch_us": kernel_s * 1e6, "launches": int(k_n),
                "sampled": f"every {sample_every} steps of the timed loop"}

    out = {
        "metric": "samples/sec per ragged weighted SGD step (fwd+bwd+reduce+update)",
        "value": value,
        "unit": "samples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "device_ms_per_step": device_ms_per_step,
        "step_spread": step_spread,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.dtype == "f32" else "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "K": w.K, "B": w.B, "b": b, "params": int(w.P),
                   "net": "MLP 3072-1024-1024-10 fp32" if w.name == "mlp3072" else w.name,
                   "includes": "controller+offsets+fwd+loss+bwd+weighted reduce+SGD"},
        "roofline": roofline,
        "roofline_update": {"bound": "hbm", "kernel": "weighted reduce + SGD", "achieved": upd_gbs,
                            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": upd_gbs / PEAK_HBM_GBS,
                            "traffic": measured_traffic(w.name, "update"),
                            "bytes_per_launch": upd_bytes, "avg_launch_us": u_ms / max(u_n, 1) * 1e3,
                            "note": "working set below 256 MB may be served from the Infinity Cache"},
        "roofline_update_momentum": {"bound": "hbm", "kernel": "weighted reduce + momentum SGD with weight decay",
                                     "achieved": mom_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                     "frac": mom_gbs / PEAK_HBM_GBS,
                                     "traffic": measured_traffic(w.name, "update_momentum"), "bytes_per_launch": mom_bytes,
                                     "avg_launch_us": m_ms / max(m_n, 1) * 1e3},
        "hbm_copy_ceiling": {"achieved": copy_gbs, "unit": "GB/s", "bytes_per_copy": 2.0 * (256 << 20),
                             "note": "plain device-to-device copy, read + write counted"},
        "final_loss": final_loss,
    }
    if asp is not None:
        out["asp_variant"] = asp
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, off)
    omni.net_destroy(net)
    omni.ctl_destroy(ctl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
