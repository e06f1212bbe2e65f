"""Seeded synthetic workloads (input generation only; no method arithmetic)."""
from .gen import CONFIGS, LayerConfig, make_layer, reduced, round_to_bf16, bf16_bits, budget_from_fraction  # noqa: F401
