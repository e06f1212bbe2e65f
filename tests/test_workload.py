"""The seeded generators: determinism, storage rounding, and the structure the recipe promises."""
import hashlib

import numpy as np
import torch

from workload import CONFIGS, bf16_bits, make_layer, reduced, round_to_bf16
from workload.gen import budget_from_fraction


def test_bf16_rounding_matches_library_conversion():
    r = np.random.Generator(np.random.PCG64(7))
    x = np.concatenate([r.standard_normal(10000).astype(np.float32) * 10,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40], dtype=np.float32)])
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = round_to_bf16(x)
    assert got.tobytes() == ref.tobytes()
    bits = bf16_bits(got)
    assert bits.dtype == np.uint16
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert back.tobytes() == got.tobytes()


def test_budgets_of_the_named_configs():
    assert CONFIGS["llama32k"].budget == 6554
    assert CONFIGS["llama128k"].budget == 52429
    assert [budget_from_fraction(f, 131072) for f in (0.1, 0.2, 0.4)] == [13107, 26214, 52429]
    assert CONFIGS["tiny"].budget == 128 and CONFIGS["tiny"].dtype == "f32"
    assert CONFIGS["qwen128k"].group == 5 and CONFIGS["mistral_prefill"].n_layers == 32


def test_generation_is_deterministic_and_layer_dependent():
    cfg = reduced(CONFIGS["llama32k"], 512)
    a = make_layer(cfg, layer=0)
    b = make_layer(cfg, layer=0)
    c = make_layer(cfg, layer=1)
    for name in a:
        assert a[name].tobytes() == b[name].tobytes()
        assert a[name].tobytes() != c[name].tobytes()
        assert a[name].dtype == np.float32
        bf16_bits(a[name])  # asserts exact bf16 values
    h = hashlib.sha256(b"".join(a[n].tobytes() for n in ("q_win", "k", "v", "w_o"))).hexdigest()
    assert h == hashlib.sha256(b"".join(b[n].tobytes() for n in ("q_win", "k", "v", "w_o"))).hexdigest()


def test_heavy_hitters_and_value_scales_have_the_stated_structure():
    cfg = reduced(CONFIGS["llama32k"], 4096)
    t = make_layer(cfg)
    G, W, dh = cfg.group, cfg.window, cfg.head_dim
    q = t["q_win"][0, :G].reshape(G * W, dh).astype(np.float64)
    k = t["k"][0, 0].astype(np.float64)
    logits_mean_query = (k @ q.mean(0)) / np.sqrt(dh)
    # sinks (first 4 tokens) carry +4 on the mean-query logit, about 1 % of the others carry +3
    assert np.all(logits_mean_query[:4] > 3.0)
    shifted = (logits_mean_query[4:] > 2.0).mean()
    assert 0.005 < shifted < 0.03
    # value rows are scaled per token: row norms are far more spread than chi(d_h) alone
    vn = np.linalg.norm(t["v"][0, 0].astype(np.float64), axis=1)
    assert vn.std() / vn.mean() > 0.5
    assert abs(t["w_o"].std() - cfg.wo_std) / cfg.wo_std < 0.05
