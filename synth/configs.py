"""Workload table: the draft-model-shaped configurations.

Shapes follow small draft models of the kind the paper uses (a 16-layer
32-query/8-kv-head model with head_dim 64, and a 28-layer 16/8-head model with
head_dim 128; Table 1 of the paper names drafts of these families), with the
paper's hyper-parameters (lookahead 8, pool 13, chunk 32, and chunk 128 for the
code-debugging setting; Appendix A.3).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple


@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_q: int                      # lookahead query rows
    L: int                        # prompt length (0 for the ragged batch)
    pool: int = 13
    chunk: int = 32
    keep_num: int = 20            # keep rate = keep_num / keep_den
    keep_den: int = 100
    hh_frac_num: int = 1          # heavy-hitter fraction = num / den of positions
    hh_frac_den: int = 100
    hh_bands: int = 0             # >0: heavy hitters confined to this many bands
    hh_band_len: int = 512
    char_model: str = "geometric"  # "uniform" or "geometric"
    draft_chars: Tuple[int, float] = (8, 4.0)    # (uniform max, geometric mean)
    target_chars: Tuple[int, float] = (7, 3.5)
    batch: int = 0                # >0: ragged batch of this many prompts
    batch_len_range: Tuple[int, int] = (2048, 65536)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def scale(self) -> float:
        return 1.0 / float(self.head_dim) ** 0.5

    @property
    def k_bytes_per_token(self) -> int:
        """Algorithmic bytes of K read per prompt token over all layers (bf16)."""
        return self.n_layers * self.n_kv_heads * self.head_dim * 2


CONFIGS = {
    "tiny": Workload("tiny", 1, 2, 4, 2, 64, 8, 1024, keep_num=25,
                     char_model="uniform"),
    "llama1b-8k": Workload("llama1b-8k", 2, 16, 32, 8, 64, 8, 8192, keep_num=20),
    "qwen06b-32k": Workload("qwen06b-32k", 3, 28, 16, 8, 128, 8, 32768, keep_num=15),
    "long-128k": Workload("long-128k", 4, 16, 32, 8, 64, 16, 131072, chunk=64,
                          keep_num=10, hh_frac_num=1, hh_frac_den=1000,
                          hh_bands=8, hh_band_len=512),
    # the longest prompts of the paper's suites (a quarter of a million tokens) with the chunk size of
    # its code-debugging setting
    "long-256k": Workload("long-256k", 6, 16, 32, 8, 64, 8, 262144, chunk=128,
                          keep_num=10, hh_frac_num=1, hh_frac_den=1000,
                          hh_bands=8, hh_band_len=512),
    "ragged-16": Workload("ragged-16", 5, 16, 32, 8, 64, 8, 0, keep_num=20, batch=16),
}


def get_config(name: str) -> Workload:
    return CONFIGS[name]
