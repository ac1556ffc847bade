"""CPU fp64 oracle of the preemptible MoE layer.  Test infrastructure only: nothing on the
product path may import this package (only tests/, the smoke check and the benchmark's
cpu_baseline leg do)."""
from .oracle import (  # noqa: F401
    OracleLayer,
    build,
    combine,
    dequant_mxfp4,
    expert_rows,
    mxfp4_weights_as_bf16,
    gate_logits,
    queues,
    route,
    silu,
    softmax,
    threads,
    set_threads,
    topk,
    topk_margin,
    units,
)
