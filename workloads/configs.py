"""Shapes of the synthetic workloads.

Each entry stands in for a LLaVA model processing one 336x336 image
(576 visual tokens) or a high-resolution tiled image (5 x 576 tokens), with a
system prompt before the image and an instruction after it (layout
[S, V, I, O] of the paper's Eq. 1).  No dataset item and no trained weight is
used: only the token counts, layer/head counts and value distributions.

A workload names its retention schedule by *parameters only*; turning those
parameters into a table of kept-token counts is part of the method and is
done separately by the oracle and by the library's host helpers.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Tuple


@dataclass(frozen=True)
class Workload:
    name: str
    layers: int
    heads: int
    head_dim: int
    dtype: str                 # "f32" or "bf16": storage type of Q/K/V
    n_sys: int                 # |S|
    n_vis: int                 # |V| before any pruning
    n_txt: int                 # |I|
    steps: int                 # decode steps T
    batches: Tuple[int, ...]
    sigma: float               # std-dev of Q/K/V entries
    seed: int
    # retention over layers at prefill (t = 0)
    layer_schedule: Dict[str, object] = field(default_factory=dict)
    # retention over decode steps (t > 0)
    step_schedule: Dict[str, object] = field(default_factory=dict)
    planted: bool = False      # skewed-attention structure in the visual keys

    @property
    def n_prompt(self) -> int:
        return self.n_sys + self.n_vis + self.n_txt


def _sigma_proj(heads: int, head_dim: int) -> float:
    # Entry std-dev of x @ W for x ~ N(0, 1), W ~ N(0, 0.02^2), hidden = H*d.
    return 0.02 * float(heads * head_dim) ** 0.5


WORKLOADS: Dict[str, Workload] = {
    # 2 layers; half of the visual tokens dropped after layer 0; then 4 more
    # dropped per decode step until layer 1 has none left at t = 8.
    "tiny": Workload(
        name="tiny", layers=2, heads=4, head_dim=64, dtype="f32",
        n_sys=8, n_vis=64, n_txt=16, steps=8, batches=(1,),
        sigma=1.0, seed=0x5713_0001,
        layer_schedule={"kind": "table", "keep": (64, 32)},
        step_schedule={"kind": "drop", "per_step": 4},
    ),
    "llava15_7b": Workload(
        name="llava15_7b", layers=32, heads=32, head_dim=128, dtype="bf16",
        n_sys=35, n_vis=576, n_txt=64, steps=256, batches=(1, 16),
        sigma=_sigma_proj(32, 128), seed=0x5713_0007,
        layer_schedule={"kind": "linear", "last_full_layer": 2, "end_ratio_bp": 1000},
        step_schedule={"kind": "cos", "tau": 256},
    ),
    "llava15_13b": Workload(
        name="llava15_13b", layers=40, heads=40, head_dim=128, dtype="bf16",
        n_sys=35, n_vis=576, n_txt=128, steps=512, batches=(1, 8, 32),
        sigma=_sigma_proj(40, 128), seed=0x5713_0013,
        layer_schedule={"kind": "linear", "last_full_layer": 2, "end_ratio_bp": 1000},
        step_schedule={"kind": "cos", "tau": 512},
    ),
    "llava_next_hr": Workload(
        name="llava_next_hr", layers=32, heads=32, head_dim=128, dtype="bf16",
        n_sys=0, n_vis=2880, n_txt=256, steps=256, batches=(8,),
        sigma=_sigma_proj(32, 128), seed=0x5713_0016,
        layer_schedule={"kind": "linear", "last_full_layer": 2, "end_ratio_bp": 500},
        step_schedule={"kind": "cos", "tau": 256},
    ),
    "skewed_13b": Workload(
        name="skewed_13b", layers=40, heads=40, head_dim=128, dtype="bf16",
        n_sys=35, n_vis=576, n_txt=128, steps=128, batches=(64,),
        sigma=_sigma_proj(40, 128), seed=0x5713_0064,
        layer_schedule={"kind": "linear", "last_full_layer": 2, "end_ratio_bp": 1000},
        step_schedule={"kind": "cos", "tau": 128},
        planted=True,
    ),
}


def get_workload(name: str) -> Workload:
    try:
        return WORKLOADS[name]
    except KeyError:
        raise KeyError(f"unknown workload {name!r}; have {sorted(WORKLOADS)}") from None
