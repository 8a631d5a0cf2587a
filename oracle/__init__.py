"""CPU oracle for the GPU A-SGD hot path (arXiv 1312.6186).

TEST INFRASTRUCTURE ONLY: a slow, plain, double-precision statement of what the
hot path computes.  Nothing under ``paper_1312_6186_amd`` may import this
package; only ``tests/``, the smoke check and the benchmark's ``cpu_baseline``
leg do.  It shares no code with the HIP library.
"""
from .ops import (  # noqa: F401
    build, num_threads, conv_fwd, conv_bwd_data, conv_bwd_weight, relu_fwd, relu_bwd,
    maxpool_fwd, maxpool_bwd, maxpool_gather, fc_fwd, fc_bwd, dropout_threshold, dropout_mask,
    dropout_apply, softmax_ce, apply_update, snapshot_bf16, bf16_to_f64, schedule, round_bf16,
)
from .net import OracleNet  # noqa: F401
from .asgd import replay, sgd_loop  # noqa: F401
