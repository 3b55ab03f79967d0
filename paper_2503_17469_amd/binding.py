"""ctypes binding of libomnistep.so: argument marshalling only.

Every function maps one to one onto an `omni_*` entry point of
include/omnistep.h.  Device buffers are torch tensors used purely as owners of
HBM; their `data_ptr()` and the current stream's handle are what crosses the
boundary.  Nothing here computes: if the shared library is missing the import
fails loudly, there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libomnistep.so")

OK, EINVAL, EINFEASIBLE, EOVERFLOW, ECAPACITY, EHIP = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1
MAX_WORKERS = 64
STEP_NO_UPDATE = 1
OPS = {"linear": 0, "conv": 1, "relu": 2, "maxpool2": 3, "bn": 4, "add": 5, "gap": 6}

EXPORTS = [
    "omni_last_error", "omni_version",
    "omni_ctl_create", "omni_ctl_set_throughputs", "omni_ctl_run", "omni_ctl_destroy",
    "omni_net_create", "omni_net_param_count", "omni_net_workspace_bytes", "omni_net_grad_stride",
    "omni_step", "omni_net_worker_grads", "omni_net_status", "omni_net_activation", "omni_net_destroy",
    "omni_net_activation_grad", "omni_net_reduced_grad", "omni_step_static",
    "omni_weighted_sgd", "omni_softmax_xent", "omni_net_timing_enable", "omni_net_timing_read",
    "omni_net_timing_sample", "omni_net_graph_enable", "omni_net_graph_replays",
    "omni_weighted_sgd_momentum", "omni_net_set_momentum", "omni_lr_step_decay",
    "omni_dyn_create", "omni_dyn_observe", "omni_dyn_adjust", "omni_dyn_get", "omni_dyn_destroy",
    "omni_asp_schedule", "omni_asp_update",
    "omni_asp_ps_create", "omni_asp_ps_eval_bsz", "omni_asp_ps_sizes", "omni_asp_ps_destroy",
    "omni_static_batches", "omni_heterogeneity_level", "omni_mem_fit_linear", "omni_mem_total",
    "omni_mem_max_batch", "omni_net_max_batch",
]
RULES = {"none": 0, "multiplicative": 1, "additive": 2}
KERNEL_CLASSES = {"linear_fwd": 0, "linear_dgrad": 1, "linear_wgrad": 2, "loss": 3, "update": 4,
                  "conv_fwd": 5, "conv_dgrad": 6, "conv_wgrad": 7}


class OmniError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"omnistep error {code}: {msg}")
        self.code = code


class LayerDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("op", "src", "src2", "cin", "cout", "ksize", "stride", "pad", "bias")]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    # The process must hold ONE HIP runtime.  torch brings its own copy of
    # libamdhip64; importing torch first makes the loader resolve this library's
    # dependency on the HIP runtime (same soname) to that already-loaded copy.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32, u64, sz, f32, u32 = C.c_void_p, C.c_int32, C.c_uint64, C.c_size_t, C.c_float, C.c_uint32
    P = C.POINTER
    lib.omni_last_error.restype = C.c_char_p
    lib.omni_version.restype = C.c_char_p
    lib.omni_ctl_create.argtypes = [i32, i32, i32, i32, P(vp)]
    lib.omni_ctl_set_throughputs.argtypes = [vp, P(u64)]
    lib.omni_ctl_run.argtypes = [vp, P(i32), P(i32)]
    lib.omni_ctl_destroy.argtypes = [vp]
    lib.omni_ctl_destroy.restype = None
    lib.omni_net_create.argtypes = [P(LayerDesc), i32, i32, i32, i32, i32, i32, i32, P(vp)]
    lib.omni_net_param_count.argtypes = [vp]
    lib.omni_net_param_count.restype = sz
    lib.omni_net_workspace_bytes.argtypes = [vp]
    lib.omni_net_workspace_bytes.restype = sz
    lib.omni_net_grad_stride.argtypes = [vp]
    lib.omni_net_grad_stride.restype = sz
    lib.omni_step.argtypes = [vp, vp, vp, vp, vp, P(i32), P(i32), i32, f32, vp, vp, vp, u32]
    lib.omni_step_static.argtypes = [vp, vp, vp, vp, vp, P(i32), P(i32), i32, f32, vp, vp, u32]
    lib.omni_net_worker_grads.argtypes = [vp, vp]
    lib.omni_net_worker_grads.restype = vp
    lib.omni_net_status.argtypes = [vp, vp]
    lib.omni_net_status.restype = vp
    lib.omni_net_activation.argtypes = [vp, vp, i32, P(vp), P(sz)]
    lib.omni_net_activation_grad.argtypes = [vp, vp, i32, P(vp), P(sz)]
    lib.omni_net_reduced_grad.argtypes = [vp, vp]
    lib.omni_net_reduced_grad.restype = vp
    lib.omni_net_destroy.argtypes = [vp]
    lib.omni_net_destroy.restype = None
    lib.omni_net_timing_enable.argtypes = [vp, i32, i32, i32]
    lib.omni_net_timing_read.argtypes = [vp, P(C.c_double), P(C.c_int64)]
    lib.omni_net_timing_sample.argtypes = [vp, i32]
    lib.omni_net_graph_enable.argtypes = [vp, i32]
    lib.omni_net_graph_replays.argtypes = [vp]
    lib.omni_net_graph_replays.restype = C.c_int64
    lib.omni_weighted_sgd.argtypes = [vp, vp, vp, sz, sz, P(i32), i32, f32, vp]
    lib.omni_softmax_xent.argtypes = [vp, vp, vp, i32, P(i32), i32, vp, vp, vp, vp, vp]
    lib.omni_weighted_sgd_momentum.argtypes = [vp, vp, vp, vp, sz, sz, P(i32), i32, f32, f32, f32, vp]
    lib.omni_net_set_momentum.argtypes = [vp, vp, f32, f32]
    lib.omni_lr_step_decay.argtypes = [C.c_double, C.c_double, P(i32), i32, i32, P(C.c_double)]
    lib.omni_dyn_create.argtypes = [i32, i32, i32, i32, C.c_double, C.c_double, i32, P(i32), P(vp)]
    lib.omni_dyn_observe.argtypes = [vp, P(C.c_double)]
    lib.omni_dyn_adjust.argtypes = [vp, P(i32), P(i32), P(i32)]
    lib.omni_dyn_get.argtypes = [vp, P(i32), P(i32)]
    lib.omni_dyn_destroy.argtypes = [vp]
    lib.omni_dyn_destroy.restype = None
    lib.omni_asp_schedule.argtypes = [i32, P(u64), P(i32), i32, P(i32), P(i32)]
    lib.omni_asp_update.argtypes = [vp, vp, vp, vp, sz, f32, i32, i32, i32]
    lib.omni_asp_ps_create.argtypes = [i32, i32, i32, C.c_double, P(vp)]
    lib.omni_asp_ps_eval_bsz.argtypes = [vp, i32, i32, C.c_double, P(i32)]
    lib.omni_asp_ps_sizes.argtypes = [vp, P(i32)]
    lib.omni_asp_ps_destroy.argtypes = [vp]
    lib.omni_asp_ps_destroy.restype = None
    f64, i64 = C.c_double, C.c_int64
    lib.omni_static_batches.argtypes = [i32, P(u64), i32, i32, i32, P(i32), P(i32)]
    lib.omni_heterogeneity_level.argtypes = [i32, P(u64), P(u64), P(u64), P(f64)]
    lib.omni_mem_fit_linear.argtypes = [i32, P(i64), P(i64), P(f64), P(f64)]
    lib.omni_mem_total.argtypes = [i64, i64, i32, i32, f64, f64, f64, P(f64)]
    lib.omni_mem_max_batch.argtypes = [f64, i64, i32, i32, f64, f64, f64, i64, P(i64)]
    lib.omni_net_max_batch.argtypes = [P(LayerDesc), i32, i32, i32, i32, i32, i32, i32, u64, P(i32), P(u64)]
    return lib


lib = _load()


def last_error() -> str:
    return lib.omni_last_error().decode()


def _check(rc):
    if rc != OK:
        raise OmniError(rc, last_error())


def _i32(seq: Sequence[int]):
    return (C.c_int32 * len(seq))(*[int(v) for v in seq])


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


# ------------------------------------------------------------------ controller
def ctl_create(K: int, B: int, b_min: int = 1, b_max: int = 0):
    h = C.c_void_p()
    _check(lib.omni_ctl_create(K, B, b_min, b_max, C.byref(h)))
    return h


def ctl_set_throughputs(ctl, T: Sequence[int]):
    arr = (C.c_uint64 * len(T))(*[int(t) for t in T])
    _check(lib.omni_ctl_set_throughputs(ctl, arr))


def ctl_run(ctl, K: int):
    b = (C.c_int32 * K)()
    off = (C.c_int32 * (K + 1))()
    _check(lib.omni_ctl_run(ctl, b, off))
    return list(b), list(off)


def ctl_destroy(ctl):
    lib.omni_ctl_destroy(ctl)


# ------------------------------------------------------------------ network
def _layer_descs(layers):
    descs = (LayerDesc * len(layers))()
    for d, L in zip(descs, layers):
        d.op = OPS[L["op"]]
        d.src = L.get("src", -1)
        d.src2 = L.get("src2", -1)
        d.cin = L.get("cin", L.get("c", 0))
        d.cout = L.get("cout", L.get("c", 0))
        d.ksize = L.get("k", 0)
        d.stride = L.get("stride", 1)
        d.pad = L.get("pad", 0)
        d.bias = 1 if L.get("bias", False) else 0
    return descs


def net_create(layers, in_shape, dtype: str, K_max: int, B_max: int):
    descs = _layer_descs(layers)
    h = C.c_void_p()
    _check(lib.omni_net_create(descs, len(layers), in_shape[0], in_shape[1], in_shape[2],
                               {"f32": F32, "bf16": BF16}[dtype], K_max, B_max, C.byref(h)))
    return h


def net_param_count(net) -> int:
    return lib.omni_net_param_count(net)


def net_workspace_bytes(net) -> int:
    return lib.omni_net_workspace_bytes(net)


def net_grad_stride(net) -> int:
    return lib.omni_net_grad_stride(net)


def net_destroy(net):
    lib.omni_net_destroy(net)


STEP_NO_UPDATE, STEP_KEEP_REDUCED_GRAD = 1, 2


def step(net, params, x, labels, off, b, lr, workspace, loss_per_worker, loss, flags: int = 0, stream=None):
    K = len(b)
    _check(lib.omni_step(net, stream if stream is not None else _stream(), _ptr(params), _ptr(x), _ptr(labels),
                         _i32(off), _i32(b), K, float(lr), _ptr(workspace), _ptr(loss_per_worker), _ptr(loss),
                         flags))


STATIC_WORKSPACE_BYTES = 32 << 20


def step_static(net, params, x, labels, off, b, lr, loss_per_worker, loss, flags: int = 0, stream=None):
    """omni_step on the library's own fixed workspace (nothing is allocated or created by the call)."""
    K = len(b)
    _check(lib.omni_step_static(net, stream if stream is not None else _stream(), _ptr(params), _ptr(x), _ptr(labels),
                                _i32(off), _i32(b), K, float(lr), _ptr(loss_per_worker), _ptr(loss), flags))


def net_worker_grads(net, workspace, K: int):
    """[K, P] view (a torch tensor aliasing the workspace)."""
    import torch
    P, stride = net_param_count(net), net_grad_stride(net)
    base = lib.omni_net_worker_grads(net, _ptr(workspace))
    byte_off = base - workspace.data_ptr()
    flat = workspace.view(torch.uint8)[byte_off:byte_off + K * stride * 4].view(torch.float32)
    return flat.view(K, stride)[:, :P]


def net_status(net, workspace) -> int:
    import torch
    base = lib.omni_net_status(net, _ptr(workspace))
    byte_off = base - workspace.data_ptr()
    return int(workspace.view(torch.uint8)[byte_off:byte_off + 4].view(torch.int32).item()) & 0xFFFFFFFF


def net_activation(net, workspace, layer: int, rows: int, dtype: str = "f32"):
    import torch
    p = C.c_void_p()
    n = C.c_size_t()
    _check(lib.omni_net_activation(net, _ptr(workspace), layer, C.byref(p), C.byref(n)))
    byte_off = p.value - workspace.data_ptr()
    if dtype == "f32":
        return workspace.view(torch.uint8)[byte_off:byte_off + rows * n.value * 4].view(torch.float32).view(rows, n.value)
    return workspace.view(torch.uint8)[byte_off:byte_off + rows * n.value * 2].view(torch.bfloat16).view(rows, n.value)


def net_activation_grad(net, workspace, layer: int, rows: int, dtype: str = "f32"):
    import torch
    p = C.c_void_p()
    n = C.c_size_t()
    _check(lib.omni_net_activation_grad(net, _ptr(workspace), layer, C.byref(p), C.byref(n)))
    byte_off = p.value - workspace.data_ptr()
    if dtype == "f32":
        return workspace.view(torch.uint8)[byte_off:byte_off + rows * n.value * 4].view(torch.float32).view(rows, n.value)
    return workspace.view(torch.uint8)[byte_off:byte_off + rows * n.value * 2].view(torch.bfloat16).view(rows, n.value)


def net_reduced_grad(net, workspace):
    """[P] view of the aggregated gradient a step with STEP_KEEP_REDUCED_GRAD stored."""
    import torch
    P = net_param_count(net)
    base = lib.omni_net_reduced_grad(net, _ptr(workspace))
    byte_off = base - workspace.data_ptr()
    return workspace.view(torch.uint8)[byte_off:byte_off + P * 4].view(torch.float32)


def net_timing_enable(net, kernel_class, layer: int = -1, max_launches: int = 4096):
    cls = KERNEL_CLASSES[kernel_class] if isinstance(kernel_class, str) else int(kernel_class)
    _check(lib.omni_net_timing_enable(net, cls, layer, max_launches))


def net_timing_sample(net, every: int):
    _check(lib.omni_net_timing_sample(net, int(every)))


def net_graph_enable(net, on: bool = True):
    _check(lib.omni_net_graph_enable(net, 1 if on else 0))


def net_graph_replays(net) -> int:
    return int(lib.omni_net_graph_replays(net))


def net_timing_read(net):
    """(total milliseconds, launches) of the timed kernel class since the last read."""
    ms = C.c_double()
    n = C.c_int64()
    _check(lib.omni_net_timing_read(net, C.byref(ms), C.byref(n)))
    return ms.value, n.value


# ------------------------------------------------------------------ single kernels
def weighted_sgd(params, grads, b, lr, shadow_bf16=None, P=None, stream=None):
    K = len(b)
    stride = grads.stride(0)
    P = params.numel() if P is None else P
    _check(lib.omni_weighted_sgd(stream if stream is not None else _stream(), _ptr(params), _ptr(grads), stride, P,
                                 _i32(b), K, float(lr), _ptr(shadow_bf16)))


def weighted_sgd_momentum(params, velocity, grads, b, lr, momentum, weight_decay, shadow_bf16=None, P=None,
                          stream=None):
    K = len(b)
    stride = grads.stride(0)
    P = params.numel() if P is None else P
    _check(lib.omni_weighted_sgd_momentum(stream if stream is not None else _stream(), _ptr(params), _ptr(velocity),
                                          _ptr(grads), stride, P, _i32(b), K, float(lr), float(momentum),
                                          float(weight_decay), _ptr(shadow_bf16)))


def net_set_momentum(net, velocity, momentum, weight_decay):
    _check(lib.omni_net_set_momentum(net, _ptr(velocity), float(momentum), float(weight_decay)))


def lr_step_decay(lr0, gamma, milestones, epoch):
    out = C.c_double(0.0)
    n = len(milestones)
    arr = _i32(milestones) if n else None
    _check(lib.omni_lr_step_decay(float(lr0), float(gamma), arr, n, int(epoch), C.byref(out)))
    return out.value


def dyn_create(K, B, b_min=1, b_max=0, deadband=0.0, alpha=1.0, rule="multiplicative", b_init=None):
    h = C.c_void_p()
    init = _i32(b_init) if b_init is not None else None
    _check(lib.omni_dyn_create(K, B, b_min, b_max, float(deadband), float(alpha), RULES[rule], init, C.byref(h)))
    return h


def dyn_observe(ctl, t):
    arr = (C.c_double * len(t))(*[float(x) for x in t])
    _check(lib.omni_dyn_observe(ctl, arr))


def dyn_adjust(ctl, K):
    b = (C.c_int32 * K)()
    off = (C.c_int32 * (K + 1))()
    changed = C.c_int32(0)
    _check(lib.omni_dyn_adjust(ctl, b, off, C.byref(changed)))
    return list(b), list(off), bool(changed.value)


def dyn_get(ctl, K):
    b = (C.c_int32 * K)()
    off = (C.c_int32 * (K + 1))()
    _check(lib.omni_dyn_get(ctl, b, off))
    return list(b), list(off)


def dyn_destroy(ctl):
    lib.omni_dyn_destroy(ctl)


def static_batches(c, B, b_min=1, b_max=0):
    K = len(c)
    b = (C.c_int32 * K)()
    off = (C.c_int32 * (K + 1))()
    _check(lib.omni_static_batches(K, (C.c_uint64 * K)(*[int(v) for v in c]), B, b_min, b_max, b, off))
    return list(b), list(off)


def heterogeneity_level(c):
    K = len(c)
    hi, lo, hl = C.c_uint64(0), C.c_uint64(0), C.c_double(0.0)
    _check(lib.omni_heterogeneity_level(K, (C.c_uint64 * K)(*[int(v) for v in c]), C.byref(hi), C.byref(lo),
                                        C.byref(hl)))
    return hi.value, lo.value, hl.value


def mem_fit_linear(b, nbytes):
    n = len(b)
    slope, icpt = C.c_double(0.0), C.c_double(0.0)
    _check(lib.omni_mem_fit_linear(n, (C.c_int64 * n)(*[int(v) for v in b]), (C.c_int64 * n)(*[int(v) for v in nbytes]),
                                   C.byref(slope), C.byref(icpt)))
    return slope.value, icpt.value


def mem_total(b, P, bytes_per_param, opt_copies, act_per_sample, batch_slope, batch_intercept):
    out = C.c_double(0.0)
    _check(lib.omni_mem_total(int(b), int(P), bytes_per_param, opt_copies, float(act_per_sample), float(batch_slope),
                              float(batch_intercept), C.byref(out)))
    return out.value


def mem_max_batch(mem_avail, P, bytes_per_param, opt_copies, act_per_sample, batch_slope, batch_intercept,
                  limit=1 << 30):
    out = C.c_int64(0)
    _check(lib.omni_mem_max_batch(float(mem_avail), int(P), bytes_per_param, opt_copies, float(act_per_sample),
                                  float(batch_slope), float(batch_intercept), int(limit), C.byref(out)))
    return out.value


def net_max_batch(layers, in_shape, dtype: str, K_max: int, opt_copies: int, budget_bytes: int):
    descs = _layer_descs(layers)
    B, total = C.c_int32(0), C.c_uint64(0)
    _check(lib.omni_net_max_batch(descs, len(layers), in_shape[0], in_shape[1], in_shape[2],
                                  {"f32": F32, "bf16": BF16}[dtype], K_max, opt_copies, int(budget_bytes),
                                  C.byref(B), C.byref(total)))
    return B.value, total.value


def asp_schedule(T, b, n_events):
    K = len(T)
    worker = (C.c_int32 * max(n_events, 1))()
    version = (C.c_int32 * max(n_events, 1))()
    _check(lib.omni_asp_schedule(K, (C.c_uint64 * K)(*[int(v) for v in T]), _i32(b), n_events, worker, version))
    return list(worker)[:n_events], list(version)[:n_events]


def asp_update(dst, base, grad, lr, b_k, B, lr_scaling=True, P=None, stream=None):
    """grad: a device tensor, or a raw device address (int) such as net_worker_grads returns."""
    P = dst.numel() if P is None else P
    g = C.c_void_p(grad) if isinstance(grad, int) else _ptr(grad)
    _check(lib.omni_asp_update(stream if stream is not None else _stream(), _ptr(dst), _ptr(base), g, P, float(lr),
                               int(b_k), int(B), 1 if lr_scaling else 0))


def asp_ps_create(K, b_min, b_max, deadband):
    h = C.c_void_p()
    _check(lib.omni_asp_ps_create(K, b_min, b_max, float(deadband), C.byref(h)))
    return h


def asp_ps_eval_bsz(ps, k, b, t):
    out = C.c_int32(0)
    _check(lib.omni_asp_ps_eval_bsz(ps, int(k), int(b), float(t), C.byref(out)))
    return out.value


def asp_ps_sizes(ps, K):
    out = (C.c_int32 * K)()
    _check(lib.omni_asp_ps_sizes(ps, out))
    return list(out)


def asp_ps_destroy(ps):
    lib.omni_asp_ps_destroy(ps)


def softmax_xent(z, labels, off, dz, loss_rows, loss_per_worker, loss, status, stream=None):
    K = len(off) - 1
    _check(lib.omni_softmax_xent(stream if stream is not None else _stream(), _ptr(z), _ptr(labels), z.shape[1],
                                 _i32(off), K, _ptr(dz), _ptr(loss_rows), _ptr(loss_per_worker), _ptr(loss),
                                 _ptr(status)))
