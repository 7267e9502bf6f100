"""Shard shapes of the synthetic workloads (shapes only, no arithmetic).

The 70B and 8B shapes are those of the paper's model table (appendix
"Configurations of the used models": Llama 2-70B 80 layers / hidden 8192 /
64 heads / 8 KV heads; Llama 3.1-8B 32 layers / 4096 / 32 / 8) with the FFN
widths of those models; the tiny shape is a hand-sized stand-in.
"""
from __future__ import annotations

from dataclasses import dataclass


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    hidden: int        # h
    n_heads: int       # a
    n_kv_heads: int    # b
    head_dim: int      # d
    ffn: int           # s
    n_shards: int      # N devices, equal shares p_i = 1/N
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def nq_local(self) -> int:
        return self.n_heads // self.n_shards

    @property
    def nkv_local(self) -> int:
        return self.n_kv_heads // self.n_shards

    @property
    def ffn_local(self) -> int:
        return self.ffn // self.n_shards

    def layer_shard_params(self) -> int:
        """Parameters of one layer of one shard: attention block + FFN block."""
        h, d = self.hidden, self.head_dim
        dq, dkv = self.nq_local * d, self.nkv_local * d
        return 2 * h * dq + 2 * h * dkv + 3 * h * self.ffn_local + 2 * h


TINY = ModelShape("tiny", 2, 256, 4, 4, 64, 688, 2)
LLAMA31_8B_TP4 = ModelShape("llama3.1-8b-shaped-tp4", 32, 4096, 32, 8, 128, 14336, 4)
LLAMA2_70B_TP8 = ModelShape("llama2-70b-shaped-tp8", 80, 8192, 64, 8, 128, 28672, 8)

BY_NAME = {m.name: m for m in (TINY, LLAMA31_8B_TP4, LLAMA2_70B_TP8)}
