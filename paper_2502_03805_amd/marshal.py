"""Argument marshalling shared by the benchmark and the tests: a layer descriptor from a workload configuration,
and the host tensors of a layer as device tensors in the descriptor's dtype.  No arithmetic of the method."""
from __future__ import annotations

from typing import Dict

import numpy as np

from . import binding as B


def cfg_desc(cfg, *, flags=0, window_reduce=None, softmax_scale=0.0, norm=B.CKV_NORM_L1, **over) -> "B.LayerDesc":
    """cfg: any object with the shape fields of workload.LayerConfig."""
    kw = dict(batch=cfg.batch, n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
              d_model=cfg.d_model, n_ctx=cfg.n_ctx, window=cfg.window, pool_kernel=cfg.pool_kernel,
              dtype=B.CKV_BF16 if cfg.dtype == "bf16" else B.CKV_F32, flags=flags, eps=cfg.eps,
              window_reduce=B.CKV_MEAN if window_reduce is None else window_reduce, softmax_scale=softmax_scale,
              norm=norm)
    kw.update(over)
    return B.make_desc(**kw)


def to_device(cfg, tensors: Dict[str, np.ndarray], wo_out_in: bool, device="cuda"):
    """Host float32 arrays -> device tensors (bf16 values are exact in float32, so the cast loses nothing);
    with wo_out_in the projection is handed over in [d_model, H*d_h] layout."""
    import torch
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    out = {}
    for name, a in tensors.items():
        if name == "w_o" and wo_out_in:
            a = np.ascontiguousarray(a.T)
        out[name] = torch.from_numpy(a).to(device=device, dtype=dt).contiguous()
    return out
