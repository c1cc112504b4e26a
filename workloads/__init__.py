"""Seeded synthetic workloads (input generators only; no method arithmetic)."""
from .generate import (  # noqa: F401
    WORKLOADS, Workload, LayerInputs, make_layer, hub_positions, hub_active, to_oracle_array,
    C1_TINY, C2_32K, C3_128K, C4_1M, C5_RAGGED,
    S_BF16, S_BF16_W64, S_BF16_D64, S_BF16_RAGGED, S_F32_W8, S_F32_RAGGED,
)
