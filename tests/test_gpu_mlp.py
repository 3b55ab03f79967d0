"""GPU parity: fp32 fully connected path against the fp64 oracle (through the C-ABI)."""
import numpy as np
import pytest

import synth
from oracle import step as OS
from oracle.controller import controller_run

from gpu_util import GpuRun, assert_close, away_from_kinks, param_tensor_slices, rel_err
from layerwise import Layerwise

pytestmark = pytest.mark.gpu

TOL = 1e-4      # relative, fp32 path (max-norm and l2, per tensor)


def _check_step(layers, in_shape, params, x, labels, off, lr, tol=TOL, tag=""):
    K = len(off) - 1
    x, redrawn = away_from_kinks(layers, in_shape, params, x, seed=K + off[-1])
    print(f"case {tag}: K={K} off={off} rows re-drawn away from ReLU kinks: {redrawn}", flush=True)
    run = GpuRun(layers, in_shape, "f32", K, off[-1])
    try:
        got = run.step(params, x, labels, off, lr)
        ref = OS.sgd_step(layers, params, x.reshape((x.shape[0],) + tuple(in_shape)), labels, off, lr, keep_acts=True)
        assert got["status"] == 0
        # layer outputs (concatenate the oracle's per-worker activations)
        for li, lay in enumerate(layers):
            if lay["op"] == "linear" and li + 1 < len(layers) and layers[li + 1]["op"] == "relu":
                continue   # stored after the folded ReLU; compared at the ReLU layer
            ref_act = np.concatenate([ref.acts[k][li].reshape(off[k + 1] - off[k], -1) for k in range(K)])
            assert_close(run.activation(li, off[-1]), ref_act, tol, f"{tag} act[{li}]")
        assert_close(got["loss_per_worker"], ref.loss_per_worker, tol, f"{tag} L_k")
        assert abs(got["loss"] - ref.loss) <= tol * abs(ref.loss)
        for name, s, e in param_tensor_slices(layers):
            for k in range(K):
                assert_close(got["worker_grads"][k, s:e], ref.worker_grads[k, s:e], tol, f"{tag} g_{k} {name}")
            assert_close(got["params"][s:e], ref.params[s:e], tol, f"{tag} theta' {name}")
            # the aggregated gradient itself (kept by the step on request), not hidden behind theta's magnitude
            assert_close(got["grad"][s:e], ref.grad[s:e], tol, f"{tag} g {name}")
    finally:
        run.close()


def test_config0_tiny_mlp():
    w = synth.workload(0)
    b, off = controller_run(w.T, w.B)
    assert b == [8, 24]
    _check_step(w.layers, w.in_shape, w.params, w.x, w.labels, off, w.lr, tag="tiny_mlp")


def test_config1_mlp3072():
    w = synth.workload(1)
    b, off = controller_run(w.T, w.B)
    assert b == [32, 64, 128, 256]
    _check_step(w.layers, w.in_shape, w.params, w.x, w.labels, off, w.lr, tag="mlp3072")


@pytest.mark.parametrize("dims,off", [
    ([70, 45, 13], [0, 1, 2, 67]),                 # odd widths: unaligned rows, scalar load path, b_k = 1
    ([132, 200, 96, 7], [0, 33, 34, 133, 197]),    # several tiles with ragged tails
    ([64, 64, 64], [0, 64, 128]),                  # exact tile multiples
    ([260, 10], [0, 5, 300]),                      # single layer, no ReLU
    # reductions that are multiples of 32 with few output tiles take the small-batch kernels:
    # ragged row tile (77 = 2*32 + 13), ragged column tile (200 = 3*64 + 8), uneven steps per wavefront (320/32 = 10)
    ([256, 320, 200, 10], [0, 3, 40, 41, 77]),
    ([288, 256, 30, 5], [0, 31, 32, 33]),          # one row tile, 30-column tile, 9 steps
    # enough 32 x 64 tiles (7 x 16) for the small-batch kernels, with a ragged last row tile (201 rows) and
    # a half-full last column tile (992 columns): forward of layer 0 and data gradient of layer 1
    ([256, 992, 512, 10], [0, 3, 90, 91, 201]),
    # the same with 7 x 15 tiles: not a multiple of the 8 XCDs, so the tiles keep their launch order; in both
    # cases the classifier's parameter gradients ride in the launch of layer 1's data gradient
    ([256, 960, 512, 10], [0, 3, 90, 91, 201]),
])
def test_ragged_shapes(dims, off):
    layers = synth.mlp(dims)
    rng = np.random.default_rng(sum(dims))
    params = synth.he_normal_params(layers, 5, False)
    params += (rng.standard_normal(params.size) * 0.05).astype(np.float32)     # non-zero biases
    B = off[-1]
    x = rng.standard_normal((B, dims[0])).astype(np.float32)
    labels = rng.integers(0, dims[-1], B).astype(np.int32)
    _check_step(layers, (1, 1, dims[0]), params, x, labels, off, 0.05, tag=f"mlp{dims}")


def test_shared_launch_with_many_classes_and_no_head_bias():
    """40 classes (three 16-class rows of classifier workgroups behind the input-gradient tiles of the
    shared launch), a classifier without bias, eight ragged workers."""
    dims = [256, 960, 512, 40]
    off = [0, 1, 30, 31, 90, 140, 141, 200, 230]
    layers = synth.mlp(dims)
    layers[-1]["bias"] = False
    layers[0]["bias"] = False
    rng = np.random.default_rng(4040)
    params = synth.he_normal_params(layers, 11, False)
    params += (rng.standard_normal(params.size) * 0.05).astype(np.float32)
    B = off[-1]
    x = rng.standard_normal((B, dims[0])).astype(np.float32)
    labels = rng.integers(0, dims[-1], B).astype(np.int32)
    _check_step(layers, (1, 1, dims[0]), params, x, labels, off, 0.05, tag="mlp-40-classes")


def test_deep_stack_batched_weight_gradients():
    """Twelve fully connected layers: their weight gradients share launches of at most eight problems
    (8 + 2 + the odd-width layer and its neighbour, which cannot take the shared launch, alone)."""
    dims = [96, 64, 80, 64, 72, 64, 45, 64, 96, 64, 128, 64, 10]
    off = [0, 7, 40, 41, 120]
    layers = synth.mlp(dims)
    rng = np.random.default_rng(77)
    params = synth.he_normal_params(layers, 9, False)
    params += (rng.standard_normal(params.size) * 0.05).astype(np.float32)
    B = off[-1]
    x = rng.standard_normal((B, dims[0])).astype(np.float32)
    labels = rng.integers(0, dims[-1], B).astype(np.int32)
    _check_step(layers, (1, 1, dims[0]), params, x, labels, off, 0.05, tag="deep-mlp")


def test_config1_unfiltered_batch():
    """Config 2's batch as generated, WITHOUT re-drawing the rows that sit on a ReLU kink.  An fp32
    forward pass may land on the other side of zero than the fp64 oracle for a pre-activation of
    order 1e-7; both gradients are then right for their own forward pass, but differ by a rank-one
    term.  Shown here: (1) every entry whose ReLU mask differs between the two is such a near-zero
    entry (|pre-activation| < 2e-5 of the layer's rms, by the oracle's own forward pass), so the
    excess error sits in the rows the filter would have re-drawn and nowhere else; (2) layer by layer,
    with each layer fed the GPU's own stored tensors, everything agrees at the fp32 tolerance on ALL
    rows, kinks included."""
    w = synth.workload(1)
    b, off = controller_run(w.T, w.B)
    x = w.x.reshape(w.B, -1)
    run = GpuRun(w.layers, w.in_shape, "f32", w.K, w.B)
    try:
        got = run.step(w.params, x, w.labels, off, w.lr)
        ref = OS.sgd_step(w.layers, w.params, x.reshape((w.B,) + tuple(w.in_shape)), w.labels, off, w.lr, keep_acts=True)
        flagged_rows = np.zeros(w.B, dtype=bool)
        flips = 0
        for li, L in enumerate(w.layers):
            if L["op"] != "relu":
                continue
            pre = np.concatenate([ref.acts[k][L["src"]].reshape(off[k + 1] - off[k], -1) for k in range(w.K)])
            near = np.abs(pre) < 2e-5 * np.sqrt((pre ** 2).mean())
            flagged_rows |= near.any(axis=1)
            mask_gpu = run.activation(li, w.B) > 0
            differ = mask_gpu != (pre > 0)
            flips += int(differ.sum())
            assert not (differ & ~near).any(), f"ReLU layer {li}: a mask differs away from zero"
        print(f"   unfiltered config 2: {int(flagged_rows.sum())} of {w.B} rows have a pre-activation within 2e-5 rms of "
              f"zero; {flips} ReLU masks differ between fp32 and fp64, all of them among those", flush=True)
        over = [name for name, s, e in param_tensor_slices(w.layers) for k in range(w.K)
                if max(rel_err(got["worker_grads"][k, s:e], ref.worker_grads[k, s:e])) > TOL]
        print(f"   per-worker gradient tensors beyond {TOL} against the whole-network oracle: {len(over)}", flush=True)
        if flips == 0:
            assert not over
        lw = Layerwise(run, w.layers, w.in_shape, w.params, x, w.labels, off, got, TOL, dtype="f32")
        try:
            lw.run_all()
        finally:
            lw.close()
    finally:
        run.close()


def test_split_reduction_is_reproducible_and_robust_to_a_dirty_workspace():
    """Shapes whose products split their reduction across workgroups (a few output tiles, a long
    reduction: partial tiles parked in the workspace, the last workgroup to arrive adds them up in
    split order).  Twenty runs must agree bit for bit -- a partial tile read before it had arrived
    would show as a different sum -- also when the caller's workspace is overwritten with 0xFF
    between the steps (the arrival counters live there), and the result must match the oracle."""
    dims = [512, 1024, 128, 2048, 10]      # forward of layers 0 and 1 and the input gradient of layer 2 split 4, 8 and 16 ways
    off = [0, 5, 40, 41, 96]
    layers = synth.mlp(dims)
    rng = np.random.default_rng(5150)
    params = synth.he_normal_params(layers, 13, False)
    params += (rng.standard_normal(params.size) * 0.05).astype(np.float32)
    B = off[-1]
    x = rng.standard_normal((B, dims[0])).astype(np.float32)
    labels = rng.integers(0, dims[-1], B).astype(np.int32)
    _check_step(layers, (1, 1, dims[0]), params, x, labels, off, 0.05, tag=f"mlp{dims} split")
    x, _ = away_from_kinks(layers, (1, 1, dims[0]), params, x, seed=len(off) - 1 + off[-1])
    run = GpuRun(layers, (1, 1, dims[0]), "f32", len(off) - 1, B)
    try:
        first = run.step(params, x, labels, off, 0.05)
        for i in range(20):
            if i % 2:
                run.ws.fill_(0xFF)
            again = run.step(params, x, labels, off, 0.05)
            assert np.array_equal(again["params"], first["params"]), i
            assert np.array_equal(again["worker_grads"], first["worker_grads"]), i
            assert again["loss"] == first["loss"]
    finally:
        run.close()


def test_step_flags_and_determinism():
    w = synth.workload(0)
    b, off = controller_run(w.T, w.B)
    run = GpuRun(w.layers, w.in_shape, "f32", 2, 32)
    try:
        a = run.step(w.params, w.x, w.labels, off, 0.1)
        c = run.step(w.params, w.x, w.labels, off, 0.1)
        assert np.array_equal(a["params"], c["params"]) and np.array_equal(a["worker_grads"], c["worker_grads"])
        z = run.step(w.params, w.x, w.labels, off, 0.0)
        assert np.array_equal(z["params"], w.params)                 # lr = 0: theta bit-identical
        n = run.step(w.params, w.x, w.labels, off, 0.1, flags=1)     # NO_UPDATE
        assert np.array_equal(n["params"], w.params)
        assert np.array_equal(n["worker_grads"], a["worker_grads"])
        assert np.array_equal(n["grad"], a["grad"])                  # the aggregated gradient is stored either way
        p = run.step(w.params, w.x, w.labels, off, 0.1, keep_g=False)   # ... and asking for it changes nothing else
        assert np.array_equal(p["params"], a["params"]) and np.array_equal(p["worker_grads"], a["worker_grads"])
    finally:
        run.close()


def test_step_rejects_bad_arguments():
    import torch
    import paper_2503_17469_amd as omni
    w = synth.workload(0)
    run = GpuRun(w.layers, w.in_shape, "f32", 2, 32)
    try:
        params = torch.from_numpy(w.params).cuda()
        x = torch.from_numpy(w.x.reshape(32, -1)).cuda()
        y = torch.from_numpy(w.labels).cuda()
        before = params.clone()
        for off, b, code in [
            ([0, 8, 32], [8, 23], -1),        # off and b disagree
            ([0, 0, 32], [0, 32], -1),        # empty worker
            ([1, 9, 33], [8, 24], -1),        # off[0] != 0
            ([0, 8, 40], [8, 32], -4),        # more rows than B_max
            ([0, 8, 16, 32], [8, 8, 16], -4), # more workers than K_max
        ]:
            with pytest.raises(omni.OmniError) as e:
                omni.step(run.net, params, x, y, off, b, 0.1, run.ws, run.lpw, run.loss)
            assert e.value.code == code, (off, b)
        with pytest.raises(omni.OmniError):
            omni.step(run.net, params, x, y, [0, 8, 32], [8, 24], float("nan"), run.ws, run.lpw, run.loss)
        torch.cuda.synchronize()
        assert torch.equal(params, before)      # nothing was launched
    finally:
        run.close()


def test_bad_label_sets_status():
    w = synth.workload(0)
    b, off = controller_run(w.T, w.B)
    labels = w.labels.copy()
    labels[5] = 10
    labels[20] = -1
    run = GpuRun(w.layers, w.in_shape, "f32", 2, 32)
    try:
        got = run.step(w.params, w.x, labels, off, 0.1)
        assert got["status"] & 1
        assert np.all(np.isfinite(got["params"]))
    finally:
        run.close()


def test_step_with_momentum_and_weight_decay():
    """Three steps of omni_step with the momentum update selected, against the oracle chain
    (per-step fp64 gradients from the oracle's own parameters, then the momentum oracle)."""
    import torch
    import paper_2503_17469_amd as omni
    from oracle import optim as OO
    dims, off = [96, 64, 32, 10], [0, 5, 6, 29, 40]
    layers = synth.mlp(dims)
    rng = np.random.default_rng(17)
    params = synth.he_normal_params(layers, 9, False)
    B, K = off[-1], len(off) - 1
    b = [off[k + 1] - off[k] for k in range(K)]
    lr, mu, wd = 0.05, 0.9, 5e-4
    run = GpuRun(layers, (1, 1, dims[0]), "f32", K, B)
    try:
        th = torch.from_numpy(params).cuda()
        vel = torch.zeros_like(th)
        omni.net_set_momentum(run.net, vel, mu, wd)
        lpw, loss = torch.zeros(K, device="cuda"), torch.zeros(1, device="cuda")
        ref_t, ref_v = params.astype(np.float64), np.zeros(params.size)
        for s in range(3):
            x = rng.standard_normal((B, dims[0])).astype(np.float32)
            y = rng.integers(0, dims[-1], B).astype(np.int32)
            omni.step(run.net, th, torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda(), off, b, lr, run.ws, lpw, loss)
            ref = OS.sgd_step(layers, ref_t, x, y, off, lr)
            ref_t, ref_v, _ = OO.weighted_momentum_step(ref_t, ref_v, ref.worker_grads, b, lr, mu, wd)
            torch.cuda.synchronize()
            assert abs(float(loss.item()) - ref.loss) <= 1e-4 * abs(ref.loss), f"step {s} loss"
        assert_close(th.cpu().numpy(), ref_t, 1e-4, "theta after 3 momentum steps")
        assert_close(vel.cpu().numpy(), ref_v, 1e-4, "velocity after 3 momentum steps")
        # back to plain SGD: one more step changes theta by exactly -lr * g (velocity untouched)
        omni.net_set_momentum(run.net, None, 0.0, 0.0)
        v_before = vel.clone()
        x = rng.standard_normal((B, dims[0])).astype(np.float32)
        y = rng.integers(0, dims[-1], B).astype(np.int32)
        omni.step(run.net, th, torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda(), off, b, lr, run.ws, lpw, loss)
        torch.cuda.synchronize()
        assert torch.equal(vel, v_before)
        ref = OS.sgd_step(layers, ref_t, x, y, off, lr)
        assert_close(th.cpu().numpy(), ref.params, 1e-4, "theta after returning to plain SGD")
    finally:
        run.close()


def test_max_workers():
    """K = 64, the largest worker count the library takes, with batches of 1 to 5 rows."""
    rng = np.random.default_rng(64)
    b = [int(v) for v in rng.integers(1, 6, size=64)]
    off = [0] + list(np.cumsum(b))
    off = [int(v) for v in off]
    dims = [96, 64, 10]
    layers = synth.mlp(dims)
    params = synth.he_normal_params(layers, 64, False)
    x, labels = synth.make_batch(640, off[-1], (1, 1, dims[0]), dims[-1], False)
    _check_step(layers, (1, 1, dims[0]), params, x, labels, off, 0.05, tag="mlp-64-workers")


def test_head_gradients_share_the_launch_of_the_input_gradient_below():
    """At the benchmark's size the classifier's parameter gradients and losses run in the launch of the
    data gradient of the layer below: that launch is timed as the layer's data gradient, the loss class
    keeps one launch per step, and the step's results do not depend on what is timed."""
    import paper_2503_17469_amd as omni
    w = synth.workload(1)
    b, off = controller_run(w.T, w.B)
    run = GpuRun(w.layers, w.in_shape, "f32", w.K, w.B)
    try:
        base = run.step(w.params, w.x, w.labels, off, w.lr)
        for cls, layer in (("linear_dgrad", 2), ("loss", -1)):
            omni.net_timing_enable(run.net, cls, layer, 8)
            for _ in range(3):
                timed = run.step(w.params, w.x, w.labels, off, w.lr)
            ms, n = omni.net_timing_read(run.net)
            assert n == 3 and 0.0 < ms / n < 1.0, (cls, ms, n)
            assert np.array_equal(timed["params"], base["params"])
            assert np.array_equal(timed["worker_grads"], base["worker_grads"])
            assert np.array_equal(timed["loss_per_worker"], base["loss_per_worker"]) and timed["status"] == 0
        omni.net_timing_enable(run.net, -1, -1, 1)
    finally:
        run.close()


def test_kernel_timing_counts_and_sampling():
    """The event brackets the benchmark reads: every matching launch, or every n-th; a class that
    does not occur in the network records nothing; timing off leaves the step's results unchanged."""
    import paper_2503_17469_amd as omni
    w = synth.workload(0)
    b, off = controller_run(w.T, w.B)
    run = GpuRun(w.layers, w.in_shape, "f32", w.K, w.B)
    try:
        base = run.step(w.params, w.x, w.labels, off, 0.1)
        omni.net_timing_enable(run.net, "linear_wgrad", 0, 16)
        for _ in range(5):
            timed = run.step(w.params, w.x, w.labels, off, 0.1)
        ms, n = omni.net_timing_read(run.net)
        assert n == 5 and 0.0 < ms < 50.0
        assert np.array_equal(timed["params"], base["params"])
        omni.net_timing_sample(run.net, 3)
        omni.net_timing_enable(run.net, "linear_wgrad", 0, 16)
        for _ in range(7):
            run.step(w.params, w.x, w.labels, off, 0.1)
        ms, n = omni.net_timing_read(run.net)
        assert n == 3                                      # launches 0, 3 and 6
        omni.net_timing_sample(run.net, 1)
        omni.net_timing_enable(run.net, "conv_fwd", -1, 4)
        run.step(w.params, w.x, w.labels, off, 0.1)
        assert omni.net_timing_read(run.net)[1] == 0
        omni.net_timing_enable(run.net, -1, -1, 1)
        with pytest.raises(omni.OmniError):
            omni.net_timing_sample(run.net, 0)
    finally:
        run.close()
