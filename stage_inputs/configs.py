"""Workload descriptions: the stage shapes, pipeline positions and budgets of the
benchmark configurations, plus shrunken twins for tests.

This module holds plain data only (no arithmetic of the method).  It is the one
place shared by the oracle-side tests and the HIP-side binding.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

GPT = 0     # LayerNorm, GELU, no rotary
LLAMA = 1   # RMSNorm, rotary, SwiGLU
FP32 = 0
BF16 = 1


@dataclass(frozen=True)
class StageConfig:
    name: str
    family: int
    dtype: int
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    seq: int
    micro_batch: int
    stage_index: int
    n_stages: int
    n_microbatches: int
    norm_eps: float = 1e-5
    rope_base: float = 10000.0
    seed: int = 0
    # schedule family: "1f1b", "zb" (split B/W), "zb_offload"
    schedule: str = "1f1b"
    # activation budget: absolute bytes, or a fraction of the no-offload peak, or None
    budget_bytes: int | None = None
    budget_frac_of_peak: float | None = None
    offload_kinds: tuple = ()

    @property
    def qkv_width(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def up_width(self) -> int:
        return 2 * self.ffn if self.family == LLAMA else self.ffn

    @property
    def elem_size(self) -> int:
        return 4 if self.dtype == FP32 else 2


CFG1 = StageConfig("cfg1_tiny_fp32", GPT, FP32, 2, 256, 4, 4, 64, 1024, 128, 1, 0, 4, 4,
                   schedule="1f1b")
CFG2 = StageConfig("cfg2_llama_bf16", LLAMA, BF16, 4, 4096, 32, 32, 128, 11008, 4096, 1, 1, 8, 16,
                   schedule="zb")
CFG3 = replace(CFG2, name="cfg3_llama_bf16_offload", schedule="zb_offload",
               budget_frac_of_peak=0.4, offload_kinds=("X_IN", "QKV", "X_MID"))
CFG4 = StageConfig("cfg4_gqa_bf16", LLAMA, BF16, 5, 8192, 64, 8, 128, 28672, 4096, 1, 3, 16, 32,
                   schedule="zb_offload", budget_bytes=120 * 10**9,
                   offload_kinds=("X_IN", "QKV", "X_MID"))
CFG5 = StageConfig("cfg5_longseq_bf16", LLAMA, BF16, 4, 5120, 40, 40, 128, 13824, 16384, 1, 0, 8, 8,
                   schedule="zb_offload", budget_bytes=64 * 10**9,
                   offload_kinds=("X_IN", "QKV", "X_MID"))

# second workload: a GPT-style stage at sequence length 1024 with grouped-query attention (hidden 2048, 16 heads in
# 8 groups, MLP 4096), 8 of 128 layers on stage 2 of p = 16, micro-batch size 8
CFG6 = StageConfig("cfg6_gpt_seq1024_bf16", GPT, BF16, 8, 2048, 16, 8, 128, 4096, 1024, 8, 2, 16, 16,
                   schedule="zb")

CONFIGS = {c.name: c for c in (CFG1, CFG2, CFG3, CFG4, CFG5, CFG6)}


def shrunken(cfg: StageConfig, hidden: int, n_q: int, n_kv: int, ffn: int, seq: int,
             n_layers: int | None = None, n_microbatches: int | None = None,
             dtype: int | None = None, name: str | None = None) -> StageConfig:
    """Same structure (family, head_dim, pipeline position, schedule kind) at a size
    the fp64 oracle finishes in seconds."""
    return replace(cfg, name=name or (cfg.name + "_small"), hidden=hidden, n_q_heads=n_q,
                   n_kv_heads=n_kv, ffn=ffn, seq=seq,
                   n_layers=cfg.n_layers if n_layers is None else n_layers,
                   n_microbatches=cfg.n_microbatches if n_microbatches is None else n_microbatches,
                   dtype=cfg.dtype if dtype is None else dtype,
                   budget_bytes=None if cfg.budget_bytes is not None else cfg.budget_bytes)
