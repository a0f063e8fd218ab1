"""Shape tables of the five synthetic workloads.

Each stands in for a model of the paper's evaluation (Table of benchmark
models: fully-connected heads of VGG19, Transformer / BERT layers, ViT layers)
with N(0, sigma) tensors instead of Cifar-10 / WikiText-2 data and trained
weights: operation counts depend on shapes only.  Device speeds are relative
flops-per-second of the virtual devices; shard sizes are NOT stored here -
each side (oracle, library) derives them itself.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Tuple


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                      # "f32" or "bf16"
    speeds: Tuple[float, ...]       # relative device speeds
    dims: Dict[str, int] = field(default_factory=dict)
    sigma_act: float = 1.0
    sigma_w: float = 0.02
    seed: int = 0
    note: str = ""


WORKLOADS = {
    "cfg1_fc_f32": Workload(
        "cfg1_fc_f32", "f32", (1.0, 0.67),
        dict(tokens=64, in_features=1024, out_features=1024),
        note="single fully-connected layer, batch rows sharded"),
    "cfg2_mlp_bf16": Workload(
        "cfg2_mlp_bf16", "bf16", (1.0, 0.6, 0.35),
        dict(tokens=8192, hidden=4096, ffn=16384),
        note="GPT-style MLP block, ffn dimension sharded"),
    "cfg3_sfb_bf16": Workload(
        "cfg3_sfb_bf16", "bf16", (1.0,) * 8,
        dict(in_features=4096, out_features=16384, capacity=512,
             rows=(512, 512, 384, 384, 256, 256, 128, 128)),
        note="sufficient-factor gradient rebuild from 8 devices' gathered factors"),
    "cfg4_encoder_bf16": Workload(
        "cfg4_encoder_bf16", "bf16", (1.0, 1.0, 0.5, 0.5),
        dict(batch=16, seq=1024, hidden=2048, heads=16, head_dim=128, ffn=8192),
        note="pre-LayerNorm Transformer encoder layer, heads and ffn sharded"),
    "cfg5_vit_bf16": Workload(
        "cfg5_vit_bf16", "bf16", (1.0, 0.8, 0.8, 0.4, 0.25),
        dict(batch=256, seq=197, hidden=1024, heads=16, head_dim=64, ffn=4096),
        note="ViT-L-style layer, batch sharded for attention block, ffn sharded for MLP"),
    "moe_experts_bf16": Workload(
        "moe_experts_bf16", "bf16", (1.0, 1.0, 0.5, 0.5),
        dict(experts=30, capacity=2048, hidden=768, ffn=3072),
        note="BERT-Base-sized MoE feed-forward layer, 30 experts (not a multiple of the 4 devices) placed by the LP + rounding; "
             "every expert buffer holds `capacity` tokens (tokens proportional to experts)"),
}
