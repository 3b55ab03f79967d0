"""GPU parity: bf16 convolutional path (bf16 operands and activations, fp32 accumulate) against
the fp64 oracle evaluated on the same bf16-representable inputs and weights."""
import numpy as np
import pytest

import synth
from oracle import layers as OL
from oracle import step as OS
from oracle.controller import controller_run

from gpu_util import GpuRun, OraclePool, assert_close, param_tensor_slices, rel_err

pytestmark = pytest.mark.gpu

TOL = 2e-2      # relative (max-norm and l2 per tensor), bf16 storage with fp32 accumulation


def _check_step(layers, in_shape, params, x, labels, off, lr, tag, tol=TOL, check_acts=True):
    K = len(off) - 1
    print(f"case {tag}: K={K} off={off}", flush=True)
    run = GpuRun(layers, in_shape, "bf16", K, off[-1])
    try:
        got = run.step(params, x, labels, off, lr)
        # Discrete decisions (ReLU masks, pooling arg-maxima) are taken on the values a bf16
        # pipeline actually stores: the oracle rounds every stored activation to bf16, then
        # works in fp64.  Without that, a sign flip of a near-zero pre-activation moves a
        # whole gradient term and parity would measure luck, not arithmetic.
        with OraclePool() as pmap:
            ref = OS.sgd_step(layers, params, x[:off[-1]], labels[:off[-1]], off, lr, store=OL.round_bf16,
                              keep_acts=check_acts, pmap=pmap)
            # graded against the storage model; the distance to exact fp64 arithmetic on the same inputs is
            # printed beside it, so that what the model of the stored values absorbs can be seen
            exact = OS.sgd_step(layers, params, x[:off[-1]], labels[:off[-1]], off, lr, pmap=pmap)
        assert got["status"] == 0
        worst = 0.0
        if check_acts:
            for li, lay in enumerate(layers):
                if li + 1 < len(layers) and layers[li + 1]["op"] == "relu" and layers[li + 1]["src"] == li:
                    continue   # stored after the folded ReLU; compared at the ReLU layer
                ref_act = np.concatenate([ref.acts[k][li].reshape(off[k + 1] - off[k], -1) for k in range(K)])
                dt = "f32" if li == len(layers) - 1 else "bf16"
                a = run.omni.net_activation(run.net, run.ws, li, off[-1], dt).float().cpu().numpy()
                e = assert_close(a, ref_act, tol, f"{tag} act[{li}] {lay['op']}")
                worst = max(worst, e[0])
        assert_close(got["loss_per_worker"], ref.loss_per_worker, tol, f"{tag} L_k")
        assert abs(got["loss"] - ref.loss) <= tol * abs(ref.loss)
        for name, s, e in param_tensor_slices(layers):
            for k in range(K):
                er = assert_close(got["worker_grads"][k, s:e], ref.worker_grads[k, s:e], tol, f"{tag} g_{k} {name}")
                worst = max(worst, er[0])
            upd = params[s:e].astype(np.float64) - got["params"][s:e].astype(np.float64)
            if np.abs(ref.grad[s:e]).max() > 0:
                assert_close(upd, lr * ref.grad[s:e], tol, f"{tag} update {name}")
            assert_close(got["params"][s:e], ref.params[s:e], tol, f"{tag} theta' {name}")
        w_store = max(rel_err(got["worker_grads"][k, s:e], ref.worker_grads[k, s:e])[1]
                      for _, s, e in param_tensor_slices(layers) for k in range(K))
        w_exact = max(rel_err(got["worker_grads"][k, s:e], exact.worker_grads[k, s:e])[1]
                      for _, s, e in param_tensor_slices(layers) for k in range(K))
        print(f"   worst max-norm relative error {worst:.2e}; worst g_k l2: {w_store:.2e} against the bf16 storage "
              f"model (graded), {w_exact:.2e} against exact fp64 arithmetic (not graded)", flush=True)
    finally:
        run.close()


def test_small_cnn():
    layers = synth.cnn3(num_classes=10, hw=16, chans=(3, 16, 32, 64))
    rng = np.random.default_rng(7)
    params = synth.he_normal_params(layers, 3, True)
    x, y = synth.make_batch(11, 37, (16, 16, 3), 10, True)
    _check_step(layers, (16, 16, 3), params, x, y, [0, 5, 6, 37], 0.1, "cnn3-16px")


def test_cnn_with_biases_and_odd_batches():
    layers = synth.cnn3(num_classes=10, hw=8, chans=(3, 8, 24, 40))
    rng = np.random.default_rng(9)
    params = synth.he_normal_params(layers, 4, True)
    for sl in synth.param_slices(layers):
        if "b" in sl:
            s, e = sl["b"]
            params[s:e] = synth.to_bf16_grid(rng.standard_normal(e - s).astype(np.float32) * 0.2)
    x, y = synth.make_batch(12, 131, (8, 8, 3), 10, True)
    _check_step(layers, (8, 8, 3), params, x, y, [0, 1, 2, 66, 131], 0.05, "cnn3-8px-bias")


@pytest.mark.parametrize("hw,chans,B,cuts", [
    # 3x3 patch kernels with biases, channel tiles that are not full, units that are not full:
    # conv2 64->96 on 8x8 maps (two-image / four-image units, second channel tile half empty),
    # conv3 96->64 on 4x4 maps (96 stored channels: two input-channel tiles, the second half empty)
    (16, (3, 64, 96, 64), 21, [0, 1, 8, 21]),
    # conv2 64->64 on 16x16 maps (one image per forward unit, two units per image for wgrad), conv3 on 8x8
    (32, (3, 64, 64, 128), 9, [0, 2, 9]),
    # the 32-channel output tile of the forward / data-gradient patch kernel: conv2 64->24 (forward: a tile
    # three quarters full; its data gradient reduces over 24, another kernel), conv3 24->64 (data gradient:
    # 24 outputs from a reduction over 64)
    (16, (3, 64, 24, 64), 21, [0, 5, 6, 21]),
    (32, (3, 64, 32, 64), 10, [0, 3, 10]),
])
def test_cnn_patch_kernels(hw, chans, B, cuts):
    layers = synth.cnn3(num_classes=10, hw=hw, chans=chans)
    rng = np.random.default_rng(hw + B)
    params = synth.he_normal_params(layers, 6, True)
    for sl in synth.param_slices(layers):
        if "b" in sl:
            s, e = sl["b"]
            params[s:e] = synth.to_bf16_grid(rng.standard_normal(e - s).astype(np.float32) * 0.2)
    x, y = synth.make_batch(13 + hw, B, (hw, hw, 3), 10, True)
    _check_step(layers, (hw, hw, 3), params, x, y, cuts, 0.05, f"cnn3-{hw}px-{chans}")


def test_config2_cnn3():
    w = synth.workload(2)
    b, off = controller_run(w.T, w.B)
    assert sum(b) == 1024 and len(b) == 8
    _check_step(w.layers, w.in_shape, w.params, w.x, w.labels, off, w.lr, "cnn3")


def test_bf16_mlp_hidden_linear():
    # fully connected layers through the same implicit-GEMM kernels (1x1 "convolution")
    layers = synth.mlp([64, 96, 40, 10])
    params = synth.he_normal_params(layers, 2, True)
    x, y = synth.make_batch(5, 77, (1, 1, 64), 10, True)
    _check_step(layers, (1, 1, 64), params, x, y, [0, 30, 31, 77], 0.1, "bf16-mlp")


def test_cnn_determinism():
    layers = synth.cnn3(num_classes=10, hw=16, chans=(3, 16, 32, 64))
    params = synth.he_normal_params(layers, 3, True)
    x, y = synth.make_batch(11, 200, (16, 16, 3), 10, True)
    run = GpuRun(layers, (16, 16, 3), "bf16", 3, 200)
    try:
        a = run.step(params, x, y, [0, 50, 90, 200], 0.1)
        c = run.step(params, x, y, [0, 50, 90, 200], 0.1)
        assert np.array_equal(a["params"], c["params"]) and np.array_equal(a["worker_grads"], c["worker_grads"])
    finally:
        run.close()


def test_cnn_max_workers():
    """K = 64 workers of 1 to 3 images each through every bf16 kernel family of the small CNN."""
    rng = np.random.default_rng(65)
    b = [int(v) for v in rng.integers(1, 4, size=64)]
    off = [int(v) for v in [0] + list(np.cumsum(b))]
    layers = synth.cnn3(num_classes=10, hw=8, chans=(3, 8, 16, 32))
    params = synth.he_normal_params(layers, 6, True)
    x, y = synth.make_batch(650, off[-1], (8, 8, 3), 10, True)
    _check_step(layers, (8, 8, 3), params, x, y, off, 0.05, "cnn3-64-workers")


@pytest.mark.parametrize("c1,B,cuts", [
    (8, 21, [0, 1, 8, 21]),        # one block of output channels, mostly empty
    (24, 21, [0, 5, 6, 21]),
    (32, 40, [0, 13, 40]),
    (40, 21, [0, 1, 8, 21]),       # two blocks, the second a quarter full
    (64, 300, [0, 7, 150, 300]),   # two full blocks; enough strips that workers are cut into chunks
])
def test_first_layer_weight_gradient_kernel(c1, B, cuts):
    """32 x 32 inputs with 3 channels: the first layer's weight gradient takes its own kernel
    (positions as the reduction, (tap, channel) pairs as columns, bias gradient as a column of ones)."""
    layers = synth.cnn3(num_classes=10, hw=32, chans=(3, c1, 16, 32))
    rng = np.random.default_rng(c1)
    params = synth.he_normal_params(layers, 10 + c1, True)
    for sl in synth.param_slices(layers):
        if "b" in sl:
            s, e = sl["b"]
            params[s:e] = synth.to_bf16_grid(rng.standard_normal(e - s).astype(np.float32) * 0.2)
    x, y = synth.make_batch(900 + c1, B, (32, 32, 3), 10, True)
    _check_step(layers, (32, 32, 3), params, x, y, cuts, 0.05, f"cnn3-32px-c{c1}", check_acts=(B <= 64))


def test_first_layer_weight_gradient_kernel_many_workers():
    """The same kernel with 64 workers of 1 to 3 images each (8 to 24 strips per worker)."""
    rng = np.random.default_rng(66)
    b = [int(v) for v in rng.integers(1, 4, size=64)]
    off = [int(v) for v in [0] + list(np.cumsum(b))]
    layers = synth.cnn3(num_classes=10, hw=32, chans=(3, 16, 16, 32))
    params = synth.he_normal_params(layers, 77, True)
    x, y = synth.make_batch(977, off[-1], (32, 32, 3), 10, True)
    _check_step(layers, (32, 32, 3), params, x, y, off, 0.05, "cnn3-32px-64-workers", check_acts=False)


def test_workspace_overwritten_between_steps():
    """The workspace is the caller's memory: a step must not rely on anything an earlier step left there.
    The bytes that loads of absent pieces (padding, ragged edges) are pointed at live in it; with the whole
    workspace set to 0xFF (bf16 NaN patterns) between two steps, the second step's results must still be
    bit-identical to the first's.  A CNN with pooling and a residual batch-norm block."""
    cases = [
        (synth.cnn3(num_classes=10, hw=16, chans=(3, 16, 32, 64)), (16, 16, 3), [0, 5, 6, 37]),
        (synth.resnet18(num_classes=10, widths=(8, 16), blocks=(1, 1), cin=3), (8, 8, 3), [0, 6, 19, 40]),
    ]
    for layers, shp, off in cases:
        params = synth.he_normal_params(layers, 3, True)
        x, y = synth.make_batch(11, off[-1], shp, 10, True)
        run = GpuRun(layers, shp, "bf16", len(off) - 1, off[-1])
        try:
            run.ws.fill_(0xFF)
            first = run.step(params, x, y, off, 0.1)
            assert first["status"] == 0 and np.all(np.isfinite(first["worker_grads"]))
            for _ in range(3):
                run.ws.fill_(0xFF)
                again = run.step(params, x, y, off, 0.1)
                assert np.array_equal(again["params"], first["params"])
                assert np.array_equal(again["worker_grads"], first["worker_grads"])
                assert again["loss"] == first["loss"] and again["status"] == 0
        finally:
            run.close()
