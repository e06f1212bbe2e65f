"""ctypes front end of the float64 CPU oracle (test infrastructure, not product code).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this.
It never imports the GPU package.  Steps are called in the paper's order:
Algorithm 2 lines 2-4 (window attention, mean, max-pool), Algorithm 1 lines 2-3
(projected-value L1 norm, criticality), lines 4-9 (two-stage Top-k), line 10
(compacted cache).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "criticalkv_oracle.c")
_LIB = os.path.join(_HERE, "libckv_oracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math: float64 sums keep their order)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O3", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int))


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def num_threads() -> int:
    return int(lib().ckvo_num_threads())


def window_attention(q_win, k, scale: Optional[float] = None, window_sum: bool = False,
                     causal_tail: bool = False) -> np.ndarray:
    """a[b,H,n]: softmax over all n keys per window row, mean (or sum) over the window."""
    q_win, qp = _f32(q_win)
    k, kp = _f32(k)
    b, H, W, dh = q_win.shape
    b2, Hkv, n, dh2 = k.shape
    assert b == b2 and dh == dh2
    if scale is None:
        scale = 1.0 / np.sqrt(dh)
    a = np.empty((b, H, n), dtype=np.float64)
    rc = lib().ckvo_window_attention(b, H, Hkv, dh, n, W, ctypes.c_double(scale), int(window_sum), int(causal_tail), qp, kp,
                                     a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    _check(rc, "window_attention")
    return a


def maxpool1d(x, kernel: int) -> np.ndarray:
    x, xp = _f64(x)
    n = x.shape[-1]
    rows = x.size // n
    y = np.empty_like(x)
    rc = lib().ckvo_maxpool1d(rows, n, kernel, xp, y.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    _check(rc, "maxpool1d")
    return y


def projected_value_norm(v, w_o, n_q_heads: int, norm: int = 1) -> np.ndarray:
    """N[b,H,n] = norm of row i of V^g W_O^h, w_o canonical [H*d_h, d_model]."""
    v, vp = _f32(v)
    w_o, wp = _f32(w_o)
    b, Hkv, n, dh = v.shape
    assert w_o.shape[0] == n_q_heads * dh
    dm = w_o.shape[1]
    N = np.empty((b, n_q_heads, n), dtype=np.float64)
    rc = lib().ckvo_projected_value_norm(b, n_q_heads, Hkv, dh, dm, n, norm, vp, wp,
                                         N.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    _check(rc, "projected_value_norm")
    return N


def group_keys(abar, N, n_kv_heads: int, eps: float = 1e-4):
    abar, ap = _f64(abar)
    N, Np = _f64(N)
    b, H, n = abar.shape
    attn = np.empty((b, n_kv_heads, n), dtype=np.float64)
    crit = np.empty((b, n_kv_heads, n), dtype=np.float64)
    rc = lib().ckvo_group_keys(b, H, n_kv_heads, n, ctypes.c_double(eps), ap, Np,
                               attn.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                               crit.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    _check(rc, "group_keys")
    return attn, crit


def select(attn, crit, budget, alpha: float, max_budget: Optional[int] = None, with_stage1: bool = False,
           protect_last: int = 0):
    """Two-stage selection per (batch, kv head).  Returns idx [b,Hkv,max_budget] (tail -1),
    count [b,Hkv], tau [b,Hkv,2] (smallest key taken in stage 1 / stage 2) and, with with_stage1,
    the uint8 flags [b,Hkv,max_budget] of the entries fixed before stage 2 (stage 1, kept window).
    protect_last = W: the last W entries are kept as they are and the algorithm runs on the entries
    before them with what is left of the budget."""
    attn, ap = _f64(attn)
    crit, cp = _f64(crit)
    b, Hkv, n = attn.shape
    budget = np.broadcast_to(np.asarray(budget, dtype=np.int32), (b, Hkv))
    budget, bp = _i32(budget)
    if max_budget is None:
        max_budget = int(budget.max()) if budget.size else 0
    idx = np.empty((b, Hkv, max(max_budget, 1)), dtype=np.int32)[:, :, :max_budget]
    idx = np.ascontiguousarray(idx)
    count = np.zeros((b, Hkv), dtype=np.int32)
    tau = np.empty((b, Hkv, 2), dtype=np.float64)
    stage1 = np.zeros((b, Hkv, max_budget), dtype=np.uint8)
    rc = lib().ckvo_select(b * Hkv, n, ap, cp, bp, ctypes.c_double(float(alpha)), int(protect_last), max_budget,
                           idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int)),
                           count.ctypes.data_as(ctypes.POINTER(ctypes.c_int)),
                           tau.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                           stage1.ctypes.data_as(ctypes.POINTER(ctypes.c_ubyte)))
    _check(rc, "select")
    return (idx, count, tau, stage1) if with_stage1 else (idx, count, tau)


DIAG_FIELDS = ("sigma", "s", "C", "theta", "theta_hat", "theta_relax", "L", "M")


def diagnostics(a_head, v, w_o, idx, count, stage1, norm: int = 1) -> np.ndarray:
    """out[b,H,8] (DIAG_FIELDS) for the distribution a_head [b,H,n] and the selection (idx, count, stage1)."""
    a_head, ap = _f64(a_head)
    v, vp = _f32(v)
    w_o, wp = _f32(w_o)
    idx, ip = _i32(idx)
    count, cp = _i32(count)
    stage1 = np.ascontiguousarray(stage1, dtype=np.uint8)
    b, H, n = a_head.shape
    _, Hkv, _, dh = v.shape
    assert w_o.shape[0] == H * dh and idx.shape == stage1.shape
    out = np.empty((b, H, 8), dtype=np.float64)
    rc = lib().ckvo_diagnostics(b, H, Hkv, dh, w_o.shape[1], n, norm, ap, vp, wp, idx.shape[-1], ip, cp,
                                stage1.ctypes.data_as(ctypes.POINTER(ctypes.c_ubyte)),
                                out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    _check(rc, "diagnostics")
    return out


def select_head(attn, crit, B: int, alpha: float, protect_last: int = 0):
    """One head; returns (idx ascending [B], fixed-before-stage-2 flag [B], tau[2])."""
    attn, ap = _f64(attn)
    crit, cp = _f64(crit)
    n = attn.shape[0]
    idx = np.empty(max(B, 1), dtype=np.int32)
    flag = np.zeros(max(B, 1), dtype=np.uint8)
    tau = np.empty(2, dtype=np.float64)
    rc = lib().ckvo_select_head(n, ap, cp, int(B), ctypes.c_double(float(alpha)), int(protect_last),
                                idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int)),
                                flag.ctypes.data_as(ctypes.POINTER(ctypes.c_ubyte)),
                                tau.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    _check(rc, "select_head")
    return idx[:B], flag[:B].astype(bool), tau


def allocate(attn, total: int, floor_frac: float) -> np.ndarray:
    """Per-head budgets [b,Hkv] from a per-batch-item total (this build's definition of Algorithm 2 line 1)."""
    attn, ap = _f64(attn)
    b, Hkv, n = attn.shape
    budget = np.zeros((b, Hkv), dtype=np.int32)
    rc = lib().ckvo_allocate(b, Hkv, n, ap, int(total), ctypes.c_double(float(floor_frac)),
                             budget.ctypes.data_as(ctypes.POINTER(ctypes.c_int)))
    _check(rc, "allocate")
    return budget


def compact(src, idx, count) -> np.ndarray:
    """out[b,Hkv,max_budget,d_h]; rows j >= count are zero-filled here (the C routine leaves them)."""
    src, sp = _f32(src)
    idx, ip = _i32(idx)
    count, cp = _i32(count)
    b, Hkv, n, dh = src.shape
    mb = idx.shape[-1]
    out = np.zeros((b, Hkv, mb, dh), dtype=np.float32)
    rc = lib().ckvo_compact(b * Hkv, n, dh, mb, sp, ip, cp, out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    _check(rc, "compact")
    return out


@dataclass
class OracleResult:
    a_head: np.ndarray      # [b,H,n] window score per query head, before pooling
    abar_head: np.ndarray   # [b,H,n] pooled
    vnorm: np.ndarray       # [b,H,n]
    attn: np.ndarray        # [b,Hkv,n] stage-1 key
    crit: np.ndarray        # [b,Hkv,n] stage-2 key
    idx: Optional[np.ndarray] = None
    count: Optional[np.ndarray] = None
    tau: Optional[np.ndarray] = None
    k_out: Optional[np.ndarray] = None
    v_out: Optional[np.ndarray] = None


def score(q_win, k, v, w_o, *, pool_kernel: int, eps: float = 1e-4, scale: Optional[float] = None,
          window_sum: bool = False, norm: int = 1, causal_tail: bool = False) -> OracleResult:
    H = q_win.shape[1]
    Hkv = k.shape[1]
    a = window_attention(q_win, k, scale, window_sum, causal_tail)
    abar = maxpool1d(a, pool_kernel)
    N = projected_value_norm(v, w_o, H, norm)
    attn, crit = group_keys(abar, N, Hkv, eps)
    return OracleResult(a, abar, N, attn, crit)


def full_pass(q_win, k, v, w_o, budget, alpha: float, *, pool_kernel: int, eps: float = 1e-4,
              scale: Optional[float] = None, window_sum: bool = False, norm: int = 1,
              max_budget: Optional[int] = None, causal_tail: bool = False,
              protect_window: bool = False) -> OracleResult:
    r = score(q_win, k, v, w_o, pool_kernel=pool_kernel, eps=eps, scale=scale, window_sum=window_sum, norm=norm,
              causal_tail=causal_tail)
    r.idx, r.count, r.tau = select(r.attn, r.crit, budget, alpha, max_budget,
                                   protect_last=q_win.shape[2] if protect_window else 0)
    r.k_out = compact(k, r.idx, r.count)
    r.v_out = compact(v, r.idx, r.count)
    return r
