"""Teacher-forced, layer-by-layer comparison of one GPU step with the oracle's single-layer functions.

A deep ReLU + batch-norm network at initialisation amplifies a rounding-sized difference between two
correct bf16 pipelines into tens of percent in the deep gradients, so comparing whole-network
gradients says little about arithmetic.  One layer at a time is well-posed: after a step the GPU
holds every layer's stored input, stored output and the gradient with respect to that output.
For every layer the oracle's definition of that ONE operation (`oracle.layers`) is applied to the
GPU's own stored input (and, backwards, to the GPU's own stored output gradient), per worker, and
the result is compared with what the GPU stored next: the layer's output, the gradient of every
tensor (the sum of its consumers' contributions, masked by a folded ReLU), and every worker's
parameter gradients.  Nothing is amplified, so the plain tolerance applies to every tensor.

Oracle calls run on row chunks in a thread pool (rows of different samples are independent in every
layer but batch norm, which is called once per worker); parameter gradients of a worker are the
fp64 sum of its chunks' contributions in row order.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
from threadpoolctl import threadpool_limits

import synth
from oracle import layers as OL

from gpu_util import fused_bn_layers, rel_err

CHUNK_ROWS = 32


class Layerwise:
    def __init__(self, run, layers, in_shape, params, x, labels, off, got, tol, threads=16, log=print, dtype="bf16"):
        self.run, self.layers, self.in_shape = run, layers, tuple(in_shape)
        self.theta = np.asarray(params, dtype=np.float64)
        self.off, self.K, self.B = list(off), len(off) - 1, off[-1]
        self.x = np.asarray(x[:self.B], dtype=np.float32).reshape((self.B,) + self.in_shape)
        self.labels = np.asarray(labels[:self.B])
        self.got, self.tol, self.log = got, tol, log
        self.shapes = synth.layer_shapes(layers, in_shape)
        self.slices = synth.param_slices(layers)
        self.unstored = fused_bn_layers(layers)        # batch norms fused into the add after them: never stored
        self.pool = ThreadPoolExecutor(threads)
        self.worst = {}                                # what -> (max-norm rel, l2 rel)
        self.n = len(layers)
        # how the pipeline stores a layer output or a gradient: rounded to bf16, or (fp32 networks) as computed
        self.dtype = dtype
        self.store = OL.round_bf16 if dtype == "bf16" else (lambda a: a)

    # ---------------------------------------------------------------- plumbing
    def root(self, i):
        """The layer whose stored tensor layer i's output is (a ReLU is folded into its producer)."""
        while i >= 0 and self.layers[i]["op"] == "relu":
            i = self.layers[i]["src"]
        return i

    def has_relu(self, r):
        return any(L["op"] == "relu" and L["src"] == r for L in self.layers)

    def shape(self, i):
        return self.in_shape if i < 0 else self.shapes[i]

    def act(self, i):
        """What a consumer of layer i reads: the GPU's stored tensor, [B, h, w, c] fp32."""
        if i < 0:
            return self.x
        dt = "f32" if self.root(i) == self.n - 1 else self.dtype
        a = self.run.omni.net_activation(self.run.net, self.run.ws, i, self.B, dt).float().cpu().numpy()
        return a.reshape((self.B,) + self.shape(i))

    def grad(self, i):
        """The GPU's stored gradient with respect to layer i's output (before a folded ReLU).  The one
        gradient a step may not store (the first convolution's when a pooling follows: the library says
        so with an error) is replaced by what the oracle derives for it from the stored tensors after it."""
        dt = "f32" if self.root(i) == self.n - 1 else self.dtype
        try:
            g = self.run.omni.net_activation_grad(self.run.net, self.run.ws, i, self.B, dt).float().cpu().numpy()
        except self.run.omni.OmniError:
            self.log(f"   gradient of layer {i}'s output is not stored: derived from its consumers")
            return self.store(self._consumer_total(self.root(i))).astype(np.float32)
        return g.reshape((self.B,) + self.shape(i))

    def p(self, li, name):
        s, e = self.slices[li][name]
        L = self.layers[li]
        if name == "w":
            shp = (L["cout"], L["cin"]) if L["op"] == "linear" else (L["cout"], L["k"], L["k"], L["cin"])
            return self.theta[s:e].reshape(shp)
        return self.theta[s:e]

    def chunks(self):
        """(worker, row0, row1) pieces that never straddle a worker."""
        out = []
        for k in range(self.K):
            for r0 in range(self.off[k], self.off[k + 1], CHUNK_ROWS):
                out.append((k, r0, min(r0 + CHUNK_ROWS, self.off[k + 1])))
        return out

    def workers(self):
        return [(k, self.off[k], self.off[k + 1]) for k in range(self.K)]

    def pmap(self, fn, items):
        with threadpool_limits(limits=1):
            return list(self.pool.map(fn, items))

    def compare(self, what, got, ref):
        e = rel_err(got, ref)
        self.worst[what] = e
        assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), what
        assert e[0] <= self.tol and e[1] <= self.tol, \
            f"{what}: max-norm rel {e[0]:.3e}, l2 rel {e[1]:.3e} (limit {self.tol})"

    # ---------------------------------------------------------------- one layer forward, from stored inputs
    def _bn_out(self, li, rows=None):
        """Oracle batch norm of layer li from its stored input, per worker, as stored (rounded)."""
        X = self.act(self.layers[li]["src"])
        gamma, beta = self.p(li, "gamma"), self.p(li, "beta")
        out = np.empty(X.shape, dtype=np.float64)

        def job(w):
            k, r0, r1 = w
            out[r0:r1] = self.store(OL.bn_fwd(X[r0:r1].astype(np.float64), gamma, beta)[0])
        self.pmap(job, self.workers())
        return out

    def _operand(self, i):
        """Input i of an add as the add sees it: stored, or a batch norm output that was never stored."""
        if i >= 0 and self.layers[i]["op"] == "bn" and i in self.unstored:
            return self._bn_out(i)
        return self.act(i)

    def check_forward(self, li):
        L = self.layers[li]
        op = L["op"]
        last = li == self.n - 1
        if op == "relu" or li in self.unstored and op == "bn":
            return
        if op == "bn":
            ref = self._bn_out(li)
        elif op == "add":
            a, b = self._operand(L["src"]), self._operand(L["src2"])
            ref = self.store(a.astype(np.float64) + b)
        else:
            X = self.act(L["src"])
            ref = np.empty((self.B,) + self.shapes[li], dtype=np.float64)

            def job(c):
                k, r0, r1 = c
                xs = X[r0:r1].astype(np.float64)
                if op == "conv":
                    y = OL.conv_fwd(xs, self.p(li, "w"), self.p(li, "b") if L["bias"] else None, L["stride"], L["pad"])
                elif op == "linear":
                    y = OL.linear_fwd(xs.reshape(r1 - r0, -1), self.p(li, "w"), self.p(li, "b") if L["bias"] else None)
                    y = y.reshape((r1 - r0,) + self.shapes[li])
                elif op == "maxpool2":
                    y = OL.maxpool2_fwd(xs)
                elif op == "gap":
                    y = OL.gap_fwd(xs)
                else:
                    raise ValueError(op)
                ref[r0:r1] = y if last else self.store(y)
            self.pmap(job, self.chunks())
        if self.has_relu(li):
            ref = OL.relu_fwd(ref)          # decided on the stored (rounded) value; a stored value stays one
        self.compare(f"layer {li} {op} output", self.act(li), ref)

    # ---------------------------------------------------------------- loss and logits gradient
    def check_loss(self):
        z = self.act(self.n - 1).reshape(self.B, -1).astype(np.float64)
        loss_rows, p = OL.softmax_xent(z, self.labels)
        dz = np.empty_like(p)
        Lk = np.zeros(self.K)
        for k, r0, r1 in self.workers():
            dz[r0:r1] = p[r0:r1] / (r1 - r0)
            Lk[k] = loss_rows[r0:r1].sum() / (r1 - r0)
        lam = np.diff(self.off) / self.B
        self.compare("L_k", self.got["loss_per_worker"], Lk)
        assert abs(self.got["loss"] - float(lam @ Lk)) <= self.tol * abs(float(lam @ Lk))
        self.compare("logits gradient", self.grad(self.n - 1).reshape(self.B, -1), dz)

    # ---------------------------------------------------------------- backward, tensor by tensor
    def consumers(self, r):
        """Layers that read tensor r (r = -1: the network input), each once per operand that is r."""
        out = []
        for li, L in enumerate(self.layers):
            if L["op"] == "relu":
                continue
            for key in ("src", "src2"):
                if key in L and (self.root(L[key]) if L[key] >= 0 else -1) == r:
                    out.append(li)
        return out

    def tensors(self):
        """Roots of all stored tensors that have a consumer, plus -1 for the network input."""
        return [-1] + [i for i, L in enumerate(self.layers) if L["op"] != "relu" and self.consumers(i)]

    def _layer_backward(self, li, need_dx):
        """Oracle backward of layer li from the GPU's stored input and stored output gradient: compares
        every worker's parameter gradients of that layer, returns the input gradient (fp64) if asked."""
        L = self.layers[li]
        op = L["op"]
        G = self.got["worker_grads"]
        dY = self.grad(li)
        if op == "add":
            return dY.astype(np.float64)
        X = self.act(L["src"])
        dX = np.empty(X.shape, dtype=np.float64) if need_dx else None
        if op == "bn":
            gamma = self.p(li, "gamma")
            dgam = np.zeros((self.K, L["c"]))
            dbet = np.zeros((self.K, L["c"]))

            def job(w):
                k, r0, r1 = w
                _, cache = OL.bn_fwd(X[r0:r1].astype(np.float64), gamma, self.p(li, "beta"))
                dx, dgam[k], dbet[k] = OL.bn_bwd(cache, gamma, dY[r0:r1].astype(np.float64))
                if need_dx:
                    dX[r0:r1] = dx
            self.pmap(job, self.workers())
            for name, ref in (("gamma", dgam), ("beta", dbet)):
                s, e = self.slices[li][name]
                for k in range(self.K):
                    self.compare(f"g_{k} layer {li} bn {name}", G[k, s:e], ref[k])
            return dX
        pieces = self.chunks()
        dW = [None] * len(pieces)
        dB = [None] * len(pieces)

        def job(idx):
            k, r0, r1 = pieces[idx]
            xs = X[r0:r1].astype(np.float64)
            dy = dY[r0:r1].astype(np.float64)
            if op == "conv":
                dx, dW[idx], dB[idx] = OL.conv_bwd(xs, self.p(li, "w"), dy, L["stride"], L["pad"])
            elif op == "linear":
                dx, dW[idx], dB[idx] = OL.linear_bwd(xs.reshape(r1 - r0, -1), self.p(li, "w"), dy.reshape(r1 - r0, -1))
                dx = dx.reshape(xs.shape)
            elif op == "maxpool2":
                dx = OL.maxpool2_bwd(xs, dy)
            elif op == "gap":
                dx = OL.gap_bwd(xs, dy)
            else:
                raise ValueError(op)
            if need_dx:
                dX[r0:r1] = dx
        self.pmap(job, range(len(pieces)))
        if op in ("conv", "linear"):
            s, e = self.slices[li]["w"]
            for k in range(self.K):
                mine = [i for i, c in enumerate(pieces) if c[0] == k]
                ref = np.zeros(e - s)
                for i in mine:
                    ref += dW[i].reshape(-1)
                self.compare(f"g_{k} layer {li} {op} weight", G[k, s:e], ref)
                if L["bias"]:
                    sb, eb = self.slices[li]["b"]
                    refb = np.zeros(eb - sb)
                    for i in mine:
                        refb += dB[i]
                    self.compare(f"g_{k} layer {li} {op} bias", G[k, sb:eb], refb)
        return dX

    def check_tensor_gradient(self, r):
        """The stored gradient of tensor r against the sum of its consumers' oracle backward passes
        (each fed the GPU's stored tensors), masked where a folded ReLU closed; on the way, the
        parameter gradients of those consumers.  r = -1: the layers that read the network input
        (parameter gradients only)."""
        if r < 0:
            for li in self.consumers(r):
                self._layer_backward(li, need_dx=False)
            return
        total = self._consumer_total(r)
        try:
            dt = "f32" if r == self.n - 1 else self.dtype
            self.run.omni.net_activation_grad(self.run.net, self.run.ws, r, self.B, dt)
        except self.run.omni.OmniError:
            return                      # not stored by the step: nothing to compare (its consumers were checked)
        self.compare(f"gradient of layer {r} {self.layers[r]['op']} output", self.grad(r), self.store(total))

    def _consumer_total(self, r):
        total = None
        for li in self.consumers(r):
            dx = self._layer_backward(li, need_dx=True)
            total = dx if total is None else total + dx
        if self.has_relu(r):
            total = total * (self.act(r) > 0)
        return total

    def run_all(self):
        for li in range(self.n):
            self.check_forward(li)
        self.check_loss()
        for r in self.tensors():
            self.check_tensor_gradient(r)
        return self.summary()

    def summary(self):
        worst = max(self.worst.items(), key=lambda kv: max(kv[1]))
        self.log(f"   layer by layer: {len(self.worst)} tensors compared, worst {worst[0]}: "
                 f"max-norm {worst[1][0]:.2e}, l2 {worst[1][1]:.2e}")
        return worst

    def close(self):
        self.pool.shutdown()
