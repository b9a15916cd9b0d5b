"""Glue between the synthetic workloads and the binding: upload of the seeded host arrays in
their storage dtype and the `Params` of a workload.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np

from . import binding as B
from . import synth


def to_device(a: np.ndarray, dtype: str):
    """float32 host array (already rounded to `dtype`) -> device tensor of that dtype."""
    import torch
    if dtype == "bf16":
        bits = synth.bf16_bits(a).view(np.int16)
        return torch.from_numpy(bits).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def params_for(w: synth.Workload, *, window=None, scale_mode=B.AHA_SCALE_ADAPTIVE,
               fixed_scale=0.0, lambda_floor=-1.0, value_prior=True, pool=7,
               score_pool=0, **extra) -> B.Params:
    """`Params` of workload `w` with the score switches given (strides still to be filled in
    with `Params.with_strides`)."""
    return B.Params(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
                    head_dim=w.head_dim, seq_len=w.seq_len, window=window or w.window,
                    budget=w.budget, recent=w.recent,
                    dtype=B.AHA_BF16 if w.dtype == "bf16" else B.AHA_F32,
                    scale_mode=scale_mode, fixed_scale=fixed_scale, lambda_floor=lambda_floor,
                    value_prior=1 if value_prior else 0, pool_kernel=pool, score_pool=score_pool,
                    **extra)
