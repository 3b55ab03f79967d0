"""Helpers for the GPU parity tests: run the library on a workload, compare tensors."""
import numpy as np


def rel_err(got, ref):
    """(max-norm error / max-norm of ref, l2 error / l2 of ref)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    d = got - ref
    mx = np.abs(ref).max()
    l2 = np.sqrt((ref ** 2).sum())
    return (np.abs(d).max() / mx if mx > 0 else np.abs(d).max(),
            np.sqrt((d ** 2).sum()) / l2 if l2 > 0 else np.sqrt((d ** 2).sum()))


def assert_close(got, ref, tol, what="", tol_max=None):
    """Per-tensor relative error: l2 within `tol`, max-norm within `tol_max` (default: `tol`)."""
    tol_max = tol if tol_max is None else tol_max
    e_max, e_l2 = rel_err(got, ref)
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), what
    assert e_max <= tol_max and e_l2 <= tol, \
        f"{what}: max-norm rel {e_max:.3e} (limit {tol_max}), l2 rel {e_l2:.3e} (limit {tol})"
    return e_max, e_l2


def param_tensor_slices(layers):
    import synth
    out = []
    for i, d in enumerate(synth.param_slices(layers)):
        for name, (s, e) in d.items():
            out.append((f"layer{i}.{name}", s, e))
    return out


def fused_bn_layers(layers):
    """Batch norms whose only consumer is the residual add right after them: normalisation and add are
    one kernel, and the normalised tensor is never stored."""
    out = set()
    for li, L in enumerate(layers[:-1]):
        nxt = layers[li + 1]
        if L["op"] == "bn" and nxt["op"] == "add" and (nxt["src"] == li) != (nxt.get("src2") == li):
            users = sum(1 for M in layers if M.get("src") == li or M.get("src2") == li)
            if users == 1:
                out.add(li)
    return out


def unstored_layers(layers):
    """Layers whose output the library does not keep under their own index: a layer whose ReLU was
    folded into it (compared at the ReLU layer), and a batch norm fused into the add after it
    (compared at the add)."""
    return {L["src"] for L in layers if L["op"] == "relu"} | fused_bn_layers(layers)


class OraclePool:
    """`with OraclePool() as pmap:` gives a map for `oracle.step.sgd_step(..., pmap=pmap)` that runs the
    workers' passes on a thread pool (numpy releases the interpreter lock), one BLAS thread each."""

    def __init__(self, threads=16):
        from concurrent.futures import ThreadPoolExecutor
        from threadpoolctl import threadpool_limits
        self.ex, self.limits = ThreadPoolExecutor(threads), threadpool_limits(limits=1)

    def __enter__(self):
        return self.ex.map

    def __exit__(self, *exc):
        self.ex.shutdown()
        self.limits.restore_original_limits()
        return False


class GpuRun:
    """One network instance on the GPU with its buffers."""

    def __init__(self, layers, in_shape, dtype, K_max, B_max):
        import torch
        import paper_2503_17469_amd as omni
        self.omni, self.torch = omni, torch
        self.layers, self.in_shape, self.dtype = layers, in_shape, dtype
        self.net = omni.net_create(layers, in_shape, dtype, K_max, B_max)
        self.P = omni.net_param_count(self.net)
        self.ws = torch.zeros(omni.net_workspace_bytes(self.net), dtype=torch.uint8, device="cuda")
        self.K_max = K_max
        self.lpw = torch.zeros(K_max, dtype=torch.float32, device="cuda")
        self.loss = torch.zeros(1, dtype=torch.float32, device="cuda")

    def close(self):
        self.omni.net_destroy(self.net)

    def step(self, params_np, x_np, labels_np, off, lr, flags=0, keep_g=True):
        torch = self.torch
        B = off[-1]
        b = [off[k + 1] - off[k] for k in range(len(off) - 1)]
        params = torch.from_numpy(np.ascontiguousarray(params_np, dtype=np.float32)).cuda()
        x = torch.from_numpy(np.ascontiguousarray(x_np[:B], dtype=np.float32).reshape(B, -1)).cuda()
        if self.dtype == "bf16":
            x = x.to(torch.bfloat16)          # exact: the generator put x on the bf16 grid
        labels = torch.from_numpy(np.ascontiguousarray(labels_np[:B], dtype=np.int32)).cuda()
        if keep_g:
            flags |= self.omni.STEP_KEEP_REDUCED_GRAD
        self.omni.step(self.net, params, x, labels, off, b, lr, self.ws, self.lpw, self.loss, flags)
        torch.cuda.synchronize()
        K = len(b)
        return dict(
            grad=self.omni.net_reduced_grad(self.net, self.ws).cpu().numpy() if keep_g else None,
            params=params.cpu().numpy(),
            loss=float(self.loss.item()),
            loss_per_worker=self.lpw[:K].cpu().numpy(),
            worker_grads=self.omni.net_worker_grads(self.net, self.ws, K).cpu().numpy(),
            status=self.omni.net_status(self.net, self.ws),
        )

    def activation(self, layer, rows):
        return self.omni.net_activation(self.net, self.ws, layer, rows, self.dtype).float().cpu().numpy()


def away_from_kinks(layers, in_shape, params, x, seed, margin=2e-5):
    """Re-draw (seeded, N(0,1)) every input row that puts some ReLU argument within
    `margin` (relative to that layer's rms pre-activation) of zero.

    A ReLU's derivative jumps at zero: an fp32 forward pass and the fp64 oracle can
    land on different sides for an argument of order 1e-7, and the two gradients then
    differ by a whole rank-one term although both are right for their own forward
    pass.  The fp32 parity cases therefore use inputs on which the decision is not
    in doubt.  Only the oracle's forward pass is consulted; rows are independent
    (no batch norm in these nets), so re-drawing one row does not disturb the others.
    Returns (x, number of rows re-drawn)."""
    from oracle import step as OS
    assert not any(L["op"] in ("bn", "maxpool2") for L in layers)
    x = np.array(x, dtype=np.float32, copy=True)
    rng = np.random.default_rng(seed)
    n = x.shape[0]
    todo = np.arange(n)
    redrawn = 0
    for _ in range(50):
        xs = x[todo].reshape((len(todo),) + tuple(in_shape))
        _, _, acts = OS.forward_backward(layers, params, xs, np.zeros(len(todo), dtype=np.int64), 0.0,
                                         keep_acts=True)
        bad = np.zeros(len(todo), dtype=bool)
        for li, L in enumerate(layers):
            if L["op"] == "relu":
                pre = acts[L["src"]].reshape(len(todo), -1)
                scale = np.sqrt((pre ** 2).mean())
                bad |= (np.abs(pre) < margin * scale).any(axis=1)
        if not bad.any():
            return x, redrawn
        todo = todo[bad]
        redrawn += len(todo)
        x[todo] = rng.standard_normal((len(todo),) + x.shape[1:]).astype(np.float32)
    raise RuntimeError("could not move inputs away from ReLU kinks")
