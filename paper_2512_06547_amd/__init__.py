"""MI355X (gfx950) library for the per-token policy-probability path of A-3PO training.

The compute lives in ``liba3po.so`` (HIP kernels behind the C ABI of ``include/a3po.h``);
this package only marshals arguments.  PyTorch is used for device memory and streams.
"""
from .binding import (  # noqa: F401
    A3PO_BF16,
    A3PO_F32,
    A3PO_PROX_BEHAV,
    A3PO_PROX_GIVEN,
    A3PO_PROX_INTERP,
    A3poError,
    count_tokens,
    plan_microbatches,
    fused_lmhead_logprob,
    fused_lmhead_loss_fwd_bwd,
    STATS_DTYPE,
    grpo_advantages,
    histogram,
    lib,
    lib_path,
    loss_fwd_bwd,
    loss_fwd_bwd_noalloc,
    NOALLOC_MAX_TOKENS,
    proximal_interp,
    shard_combine,
    shard_loss_bwd,
    shard_partials,
    stats_to_dict,
    strerror,
    token_logprobs,
    workspace_bytes,
)
