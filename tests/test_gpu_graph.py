"""GPU: repeated steps replayed as a HIP graph give, bit for bit, what the same steps give launched
one by one -- on every replay, with other work and synchronisations in between, after a change of
the batch split, with kernel timing sampled in between, and for the fp32 and the bf16 path."""
import numpy as np
import pytest

import synth
from oracle.controller import controller_run

pytestmark = pytest.mark.gpu


class _Net:
    def __init__(self, w, graph):
        import torch
        import paper_2503_17469_amd as omni
        self.omni, self.torch, self.w = omni, torch, w
        self.net = omni.net_create(w.layers, w.in_shape, w.dtype, w.K, w.B)
        self.ws = torch.zeros(omni.net_workspace_bytes(self.net), dtype=torch.uint8, device="cuda")
        self.params = torch.from_numpy(w.params.copy()).cuda()
        x = torch.from_numpy(w.x.reshape(w.B, -1)).cuda()
        self.x = x.to(torch.bfloat16) if w.dtype == "bf16" else x
        self.y = torch.from_numpy(w.labels).cuda()
        self.lpw = torch.zeros(w.K, dtype=torch.float32, device="cuda")
        self.loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        if graph:
            omni.net_graph_enable(self.net, True)

    def step(self, off, lr, flags=0):
        b = [off[k + 1] - off[k] for k in range(len(off) - 1)]
        self.omni.step(self.net, self.params, self.x, self.y, off, b, lr, self.ws, self.lpw, self.loss, flags)

    def state(self):
        self.torch.cuda.synchronize()
        K = self.w.K
        return (self.params.cpu().numpy().copy(), float(self.loss.item()), self.lpw.cpu().numpy().copy(),
                self.omni.net_worker_grads(self.net, self.ws, K).cpu().numpy().copy())

    def close(self):
        self.omni.net_destroy(self.net)


def _same(a, b, what):
    assert np.array_equal(a[0], b[0]), f"{what}: parameters differ"
    assert a[1] == b[1], f"{what}: loss differs"
    assert np.array_equal(a[2], b[2]), f"{what}: worker losses differ"
    assert np.array_equal(a[3], b[3]), f"{what}: worker gradients differ"


@pytest.mark.parametrize("cfg", [0, 2])
def test_graph_replays_match_eager_steps(cfg):
    import torch
    import paper_2503_17469_amd as omni
    w = synth.workload(cfg) if cfg == 0 else synth.workload(cfg, B=96, K=4)
    _, off = controller_run(w.T, w.B)
    T2 = list(reversed(w.T))
    _, off2 = controller_run(T2, w.B)
    assert off2 != off
    lr = 0.01
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        g, e = _Net(w, True), _Net(w, False)
        try:
            scratch = torch.zeros(1 << 20, device="cuda")
            for i in range(12):
                print(f"case graph cfg={cfg} step {i}", flush=True)
                cur = off if i < 8 else off2            # the split changes at step 8: launch by launch again, then a new graph
                g.step(cur, lr)
                e.step(cur, lr)
                scratch.add_(1.0)                        # other work between the replays
                if i % 2 == 0:
                    _same(g.state(), e.state(), f"step {i}")
            _same(g.state(), e.state(), "end")
            # steps 0 and 1 and 8 and 9 are enqueued or captured, the other eight replayed
            assert omni.net_graph_replays(g.net) == 8, omni.net_graph_replays(g.net)
            assert omni.net_graph_replays(e.net) == 0
            # with timing sampled every third launch, the sampled steps are enqueued launch by launch
            omni.net_timing_sample(g.net, 3)
            omni.net_timing_enable(g.net, "update", -1, 64)
            before = omni.net_graph_replays(g.net)
            for i in range(9):
                g.step(off2, lr)
                e.step(off2, lr)
            _same(g.state(), e.state(), "timed")
            ms, n = omni.net_timing_read(g.net)
            assert n == 3 and ms > 0.0                   # launches 0, 3 and 6
            assert omni.net_graph_replays(g.net) > before
            omni.net_timing_enable(g.net, -1, -1, 1)
            omni.net_timing_sample(g.net, 1)
            # the flag that skips the update is part of the key
            g.step(off2, lr, flags=1)
            e.step(off2, lr, flags=1)
            _same(g.state(), e.state(), "no update")
            omni.net_graph_enable(g.net, False)
            g.step(off2, lr)
            e.step(off2, lr)
            _same(g.state(), e.state(), "graph off")
        finally:
            g.close()
            e.close()
    torch.cuda.synchronize()
