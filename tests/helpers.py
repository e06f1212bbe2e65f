"""Shared test plumbing: device marshalling for the GPU path and the parity rules.

The comparison rules are the acceptance criteria of the build:
  * scores within 2e-3 relative of the float64 oracle (bf16 inputs, fp32 accumulation);
  * selected index sets identical, except for swaps between entries whose oracle key lies
    within 2e-3 relative of the stage threshold; every swap is counted.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

from oracle.parity_rules import REL_TOL, assert_scores_close, compare_selection, score_errors  # noqa: F401


def cfg_desc(P, cfg, **kw):
    """Layer descriptor of a workload configuration (the package's own marshalling helper)."""
    from paper_2502_03805_amd.marshal import cfg_desc as impl
    return impl(cfg, **kw)


def to_device(cfg, tensors: Dict[str, np.ndarray], wo_out_in: bool, device="cuda"):
    from paper_2502_03805_amd.marshal import to_device as impl
    return impl(cfg, tensors, wo_out_in, device)


@dataclass
class GpuResult:
    attn: np.ndarray
    crit: np.ndarray
    vnorm: Optional[np.ndarray]
    idx: np.ndarray
    count: np.ndarray
    k_out: np.ndarray
    v_out: np.ndarray


def run_gpu_pass(P, cfg, tensors, budget, alpha, *, flags=0, wo_out_in=False, max_budget=None, want_vnorm=True,
                 window_reduce=None, softmax_scale=0.0, dev=None, norm=1) -> GpuResult:  # flags may carry CKV_CAUSAL_TAIL etc.
    """score -> select -> compact through the C ABI on cuda:0; returns host copies."""
    import torch
    if wo_out_in:
        flags |= P.CKV_WO_OUT_IN
    desc = cfg_desc(P, cfg, flags=flags, window_reduce=window_reduce, softmax_scale=softmax_scale, norm=norm)
    dev = dev or to_device(cfg, tensors, wo_out_in)
    b, H, Hkv, n, dh = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.n_ctx, cfg.head_dim
    budget = np.broadcast_to(np.asarray(budget, dtype=np.int32), (b, Hkv)).copy()
    if max_budget is None:
        max_budget = max(1, int(budget.max()))
    ws = torch.empty(P.workspace_bytes(desc, max_budget), dtype=torch.uint8, device="cuda")
    attn = torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda")
    crit = torch.empty_like(attn)
    vnorm = torch.empty((b, H, n), dtype=torch.float32, device="cuda") if want_vnorm else None
    idx = torch.full((b, Hkv, max_budget), -7, dtype=torch.int32, device="cuda")
    count = torch.full((b, Hkv), -7, dtype=torch.int32, device="cuda")
    k_out = torch.zeros((b, Hkv, max_budget, dh), dtype=dev["k"].dtype, device="cuda")
    v_out = torch.zeros_like(k_out)
    bud = torch.from_numpy(budget).cuda()
    P.criticalkv_score(desc, dev["q_win"], dev["k"], dev["v"], dev["w_o"], attn, crit, vnorm, workspace=ws)
    P.criticalkv_select(desc, attn, crit, bud, alpha, max_budget, idx, count, workspace=ws)
    P.criticalkv_compact(desc, dev["k"], dev["v"], idx, count, max_budget, k_out, v_out)
    torch.cuda.synchronize()
    return GpuResult(attn.cpu().numpy(), crit.cpu().numpy(), None if vnorm is None else vnorm.cpu().numpy(),
                     idx.cpu().numpy(), count.cpu().numpy(), k_out.float().cpu().numpy(), v_out.float().cpu().numpy())


def assert_compaction_exact(res: GpuResult, tensors, budget):
    """k_out / v_out rows are bit-exact copies of the rows idx names (checked against the GPU's own idx)."""
    b, Hkv, mb = res.idx.shape
    budget = np.broadcast_to(np.asarray(budget, dtype=np.int64), (b, Hkv))
    for bi in range(b):
        for g in range(Hkv):
            B = int(budget[bi, g])
            sel = res.idx[bi, g, :B]
            assert np.array_equal(res.k_out[bi, g, :B], tensors["k"][bi, g, sel])
            assert np.array_equal(res.v_out[bi, g, :B], tensors["v"][bi, g, sel])
            assert not res.k_out[bi, g, B:].any() and not res.v_out[bi, g, B:].any(), "rows past count must be untouched"
