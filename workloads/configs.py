"""Workload shapes: the five benchmark configurations and small stand-ins.

These stand in for the paper's production traces and released checkpoints
(Section 5.1: Qwen2.5-32B on the GRPO/DAPO/PPO-32B-20K traces, per-worker batch
128-256; Section 5.3: Qwen3-235B MoE), none of which is available offline:
Qwen2.5-7B/32B-like dense and Qwen3-30B-A3B-like MoE geometry, random weights,
seeded random prefixes.
"""
from __future__ import annotations

from dataclasses import dataclass, replace


@dataclass(frozen=True)
class Shape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    n_experts: int = 0
    top_k: int = 0
    d_expert: int = 0
    dtype: str = "bf16"
    rope_theta: float = 1.0e6
    rms_eps: float = 1.0e-6
    # workload
    batch: int = 1
    k: int = 4
    n_chains: int = 1
    prefix_lo: int = 128
    prefix_hi: int = 128
    draft_sigma: tuple = (0.5,)
    verify_mode: int = 1          # 0 greedy, 1 stochastic
    seed: int = 0

    def model_fields(self) -> dict:
        return dict(n_layers=self.n_layers, d_model=self.d_model, n_q_heads=self.n_q_heads,
                    n_kv_heads=self.n_kv_heads, head_dim=self.head_dim, d_ff=self.d_ff,
                    vocab=self.vocab, n_experts=self.n_experts, top_k=self.top_k,
                    d_expert=self.d_expert, dtype=self.dtype, rope_theta=self.rope_theta,
                    rms_eps=self.rms_eps)


CONFIGS = {
    # tiny decoder, fp32, greedy verification, drafts = argmax(target logits + N(0,1))
    "cfg1": Shape("cfg1-tiny-fp32", 2, 256, 4, 4, 64, 1024, 2048, dtype="fp32", rope_theta=1.0e4,
                  batch=4, k=4, prefix_lo=128, prefix_hi=128, draft_sigma=(1.0,), verify_mode=0, seed=1000),
    # dense 7B-shaped decoder, B=64, prefixes 1k-8k, stochastic verification
    "cfg2": Shape("cfg2-7b-b64-k4", 28, 3584, 28, 4, 128, 18944, 152064,
                  batch=64, k=4, prefix_lo=1024, prefix_hi=8192, draft_sigma=(0.5,), seed=2000),
    # same shape, large per-worker batch; k and sigma are swept by the caller
    "cfg3": Shape("cfg3-7b-b256", 28, 3584, 28, 4, 128, 18944, 152064,
                  batch=256, k=4, prefix_lo=2048, prefix_hi=8192, draft_sigma=(0.25,), seed=3000),
    # MoE decoder
    "cfg4": Shape("cfg4-moe-b128-k4", 48, 2048, 32, 4, 128, 0, 151936, n_experts=128, top_k=8, d_expert=768,
                  batch=128, k=4, prefix_lo=1024, prefix_hi=8192, draft_sigma=(0.5,), seed=4000),
    # long-tail rollout, 32B shape, three chains of eight drafts
    "cfg5": Shape("cfg5-32b-b32-n3-k8", 64, 5120, 40, 8, 128, 27648, 152064,
                  batch=32, k=8, n_chains=3, prefix_lo=16384, prefix_hi=32768,
                  draft_sigma=(0.25, 0.5, 1.0), seed=5000),
}


def scaled_down(shape: Shape, **overrides) -> Shape:
    """Same structure, smaller numbers: for parity cases the oracle finishes in seconds."""
    return replace(shape, **overrides)
