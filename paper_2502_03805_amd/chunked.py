"""Chunked prefill with eviction between chunks: a host loop over the three C-ABI calls.

After each chunk of the prompt the cache kept so far, followed by the chunk's new K/V rows, is scored with
the chunk's last W queries (causal inside the window, the window's own tokens protected), cut down to the
budget and compacted; the compacted cache is what the next chunk sees.  Only orchestration and buffer
concatenation happen here; every step of each pass runs in the library's kernels.
"""
from __future__ import annotations

from typing import Callable, List, Sequence, Tuple

from . import binding as B


def chunked_prefill_evict(make_desc: Callable[[int], "B.LayerDesc"], q_windows: Sequence, k_chunks: Sequence,
                          v_chunks: Sequence, w_o, budget: int, alpha: float, stream=None) -> Tuple[object, object, List]:
    """q_windows[c]: [b,H,W,d_h] last W queries of chunk c; k_chunks[c], v_chunks[c]: [b,Hkv,len_c,d_h].
    make_desc(n) builds the layer descriptor for n cached entries (flags should include CKV_CAUSAL_TAIL and
    CKV_PROTECT_WINDOW).  Returns (k_cache, v_cache, kept) where kept[c] is the idx tensor of chunk c's pass
    (positions in that pass's concatenated cache) or None when everything fitted the budget."""
    import torch
    k_cache = v_cache = None
    kept = []
    for q_win, k_new, v_new in zip(q_windows, k_chunks, v_chunks):
        k_all = k_new if k_cache is None else torch.cat([k_cache, k_new], dim=2).contiguous()
        v_all = v_new if v_cache is None else torch.cat([v_cache, v_new], dim=2).contiguous()
        b, Hkv, n, dh = k_all.shape
        if n <= budget:
            k_cache, v_cache = k_all, v_all
            kept.append(None)
            continue
        desc = make_desc(n)
        ws = torch.empty(B.workspace_bytes(desc, budget), dtype=torch.uint8, device=k_all.device)
        attn = torch.empty((b, Hkv, n), dtype=torch.float32, device=k_all.device)
        crit = torch.empty_like(attn)
        idx = torch.empty((b, Hkv, budget), dtype=torch.int32, device=k_all.device)
        count = torch.empty((b, Hkv), dtype=torch.int32, device=k_all.device)
        bud = torch.full((b, Hkv), budget, dtype=torch.int32, device=k_all.device)
        k_out = torch.empty((b, Hkv, budget, dh), dtype=k_all.dtype, device=k_all.device)
        v_out = torch.empty_like(k_out)
        B.criticalkv_score(desc, q_win, k_all, v_all, w_o, attn, crit, None, workspace=ws, stream=stream)
        B.criticalkv_select(desc, attn, crit, bud, alpha, budget, idx, count, workspace=ws, stream=stream)
        B.criticalkv_compact(desc, k_all, v_all, idx, count, budget, k_out, v_out, stream=stream)
        k_cache, v_cache = k_out, v_out
        kept.append(idx)
    return k_cache, v_cache, kept
