"""Seeded synthetic inputs for one layer of the KV-cache selection pass.

This module only draws random tensors and rounds them to the storage dtype.
It holds none of the method's arithmetic (no softmax, no projection, no
selection): both the CPU oracle's tests and the GPU path's tests/benchmark
take their inputs from here so that they consume identical bytes.

Shapes follow the paper's notation: `n` cached entries per head, observation
window of `W` queries (Algorithm 2, input line), per-head slice of the output
projection `W^O` of shape d_h x d (Section 3.1).

Recipe (all draws with numpy.random.Generator(PCG64(seed)), float32):
  * Qwin, K, V ~ N(0, 1) i.i.d.
  * heavy hitters: per (batch, kv head) a fraction p_hh of token indices drawn
    without replacement; their key rows are shifted along the mean window
    query of the head's group so that the mean-query logit rises by `delta_hh`
    (in units of the logit's standard deviation).  Optional sink tokens 0..3
    get the same shift with `delta_sink`.
  * value rows are scaled per (batch, kv head, token) by LogNormal(0, sigma_v).
  * W_O ~ N(0, wo_std), canonical layout [H*d_h, d_model].
  * for bf16 workloads every tensor is rounded to nearest-even bf16 and
    returned as float32 holding exactly those values.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

TENSOR_IDS = {"q_win": 0, "k": 1, "v": 2, "w_o": 3, "hh_idx": 4, "v_scale": 5}


@dataclass(frozen=True)
class LayerConfig:
    name: str
    config_id: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_model: int
    n_ctx: int
    window: int
    pool_kernel: int
    budget: int            # per kv head
    alpha: float
    dtype: str             # "bf16" | "f32"
    p_hh: float
    delta_hh: float
    n_sinks: int
    delta_sink: float
    sigma_v: float
    wo_std: float
    eps: float = 1e-4
    n_layers: int = 1

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def entries(self) -> int:
        """KV entries of one layer: one per (batch item, kv head, token)."""
        return self.batch * self.n_kv_heads * self.n_ctx

    def with_(self, **kw) -> "LayerConfig":
        return dataclasses.replace(self, **kw)


def budget_from_fraction(frac: float, n: int) -> int:
    """Per-head budget for a cache-size fraction: round half up."""
    return int(np.floor(frac * n + 0.5))


def _cfg(name, cid, batch, H, Hkv, dh, dm, n, W, k, frac, alpha, dtype, p_hh, d_hh,
         sinks, d_sink, sigma_v, wo_std, n_layers=1, budget=None) -> LayerConfig:
    B = budget if budget is not None else budget_from_fraction(frac, n)
    return LayerConfig(name, cid, batch, H, Hkv, dh, dm, n, W, k, B, alpha, dtype, p_hh, d_hh,
                       sinks, d_sink, sigma_v, wo_std, 1e-4, n_layers)


CONFIGS: Dict[str, LayerConfig] = {
    # tiny MHA layer, fp32
    "tiny": _cfg("tiny", 0, 1, 4, 4, 64, 256, 1024, 8, 5, None, 0.5, "f32",
                 0.02, 3.0, 0, 0.0, 0.75, 1.0 / 16.0, budget=128),
    # Llama-3-8B-shaped layer, 32K context, 20 % budget
    "llama32k": _cfg("llama32k", 1, 1, 32, 8, 128, 4096, 32768, 32, 7, 0.20, 0.5, "bf16",
                     0.01, 3.0, 4, 4.0, 0.75, 0.02),
    # same layer at 128K context, 40 % budget
    "llama128k": _cfg("llama128k", 2, 1, 32, 8, 128, 4096, 131072, 32, 7, 0.40, 0.5, "bf16",
                      0.01, 3.0, 4, 4.0, 0.75, 0.02),
    # Mistral-7B-shaped prefill: 32 layers, batch 4, 32K
    "mistral_prefill": _cfg("mistral_prefill", 3, 4, 32, 8, 128, 4096, 32768, 32, 7, 0.20, 0.5, "bf16",
                            0.01, 3.0, 4, 4.0, 0.75, 0.02, n_layers=32),
    # Qwen-32B-shaped layer, 128K, W = 64 (budget / alpha are swept by the caller)
    "qwen128k": _cfg("qwen128k", 4, 1, 40, 8, 128, 5120, 131072, 64, 7, 0.20, 0.5, "bf16",
                     0.005, 3.0, 4, 4.0, 1.0, 0.02),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already exact bf16."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    assert not np.any(bits & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (bits >> np.uint32(16)).astype(np.uint16)


def seed_for(cfg: LayerConfig, layer: int, tensor: str) -> int:
    return 1000 * cfg.config_id + 10 * layer + TENSOR_IDS[tensor]


def make_layer(cfg: LayerConfig, layer: int = 0, seed_offset: int = 0) -> Dict[str, np.ndarray]:
    """Return {'q_win','k','v','w_o'} as float32 arrays in the canonical layouts
    q_win [b,H,W,d_h], k/v [b,Hkv,n,d_h], w_o [H*d_h, d_model]."""
    b, H, Hkv, dh, dm, n, W = (cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                               cfg.d_model, cfg.n_ctx, cfg.window)
    G = cfg.group

    def rng(t):
        return np.random.Generator(np.random.PCG64(seed_for(cfg, layer, t) + 100000 * seed_offset))

    q = rng("q_win").standard_normal((b, H, W, dh), dtype=np.float32)
    k = rng("k").standard_normal((b, Hkv, n, dh), dtype=np.float32)
    v = rng("v").standard_normal((b, Hkv, n, dh), dtype=np.float32)
    w_o = (rng("w_o").standard_normal((H * dh, dm), dtype=np.float32) * np.float32(cfg.wo_std))

    r_hh = rng("hh_idx")
    m_hh = int(round(cfg.p_hh * n))
    for bi in range(b):
        for g in range(Hkv):
            qbar = q[bi, g * G:(g + 1) * G].reshape(G * W, dh).mean(axis=0, dtype=np.float64)
            direction = (np.sqrt(dh) * qbar / float(qbar @ qbar)).astype(np.float32)
            if m_hh > 0:
                hh = r_hh.permutation(n)[:m_hh]
                k[bi, g, hh] += np.float32(cfg.delta_hh) * direction
            if cfg.n_sinks > 0:
                k[bi, g, :cfg.n_sinks] += np.float32(cfg.delta_sink) * direction

    if cfg.sigma_v > 0:
        s = rng("v_scale").lognormal(0.0, cfg.sigma_v, size=(b, Hkv, n, 1)).astype(np.float32)
        v *= s

    out = {"q_win": q, "k": k, "v": v, "w_o": w_o}
    if cfg.dtype == "bf16":
        out = {name: round_to_bf16(a) for name, a in out.items()}
    return out


def reduced(cfg: LayerConfig, n_ctx: int, budget: Optional[int] = None, **kw) -> LayerConfig:
    """Same generators at a smaller context (parity-test sizes)."""
    if budget is None:
        budget = max(1, int(round(cfg.budget / cfg.n_ctx * n_ctx)))
    return cfg.with_(n_ctx=n_ctx, budget=budget, **kw)
