"""MI355X-native ragged, batch-size-weighted SGD step (OmniLearn dynamic batching).

Thin Python face of libomnistep.so; see include/omnistep.h for the contract.
"""
from . import binding
from .binding import (  # noqa: F401
    OmniError, ctl_create, ctl_destroy, ctl_run, ctl_set_throughputs, last_error, net_activation, net_activation_grad,
    net_reduced_grad, STEP_NO_UPDATE, STEP_KEEP_REDUCED_GRAD, step_static, STATIC_WORKSPACE_BYTES,
    net_create, net_destroy, net_grad_stride, net_param_count, net_status, net_worker_grads,
    net_timing_enable, net_timing_read, net_timing_sample, net_graph_enable, net_graph_replays, net_workspace_bytes, softmax_xent, step, weighted_sgd, weighted_sgd_momentum, net_set_momentum, lr_step_decay,
    dyn_create, dyn_observe, dyn_adjust, dyn_get, dyn_destroy,
    static_batches, heterogeneity_level, mem_fit_linear, mem_total, mem_max_batch, net_max_batch,
    asp_schedule, asp_update, asp_ps_create, asp_ps_eval_bsz, asp_ps_sizes, asp_ps_destroy,
)
