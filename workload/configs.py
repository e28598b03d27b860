"""The five synthetic workload shapes (OLMoE-, Mixtral-, Phi-3.5-MoE- and
DeepSeekMoE-like layer stacks plus a tiny fp32 case).

Layer counts / expert counts / top-k follow the paper's model table (Table 6);
hidden and intermediate widths are those of the public model families.  The
per-sequence logit bias on a small preferred set stands in for the routing
concentration the paper's fine-tuning produces (Section 3.1, Fig. 1b).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

BASE_SEED = 260211192


@dataclass(frozen=True)
class MoEConfig:
    name: str
    cfg_id: int            # seed = BASE_SEED + cfg_id
    dtype: str             # "fp32" | "bf16": storage type of weights, x and y
    n_layers: int
    d_model: int
    d_ff: int
    n_experts: int
    n_shared: int
    top_k: int
    capacity: int          # resident experts per layer
    n_seqs: int
    n_steps: int           # decode steps per sequence
    prefill_len: int       # prompt tokens per sequence (0 = none)
    beta: float            # logit bias on preferred experts
    pref_lo: int           # preferred-set size is uniform in [pref_lo, pref_hi]
    pref_hi: int
    delta: float           # minimum gap between the K-th and (K+1)-th logit
    norm_topk: int = 1

    @property
    def seed(self) -> int:
        return BASE_SEED + self.cfg_id

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "fp32" else 2

    @property
    def expert_bytes(self) -> int:
        return 3 * self.d_model * self.d_ff * self.elem_bytes

    def with_(self, **kw) -> "MoEConfig":
        return replace(self, **kw)


CONFIGS = {
    "tiny_fp32": MoEConfig("tiny_fp32", 1, "fp32", 1, 64, 128, 8, 0, 2, 2, 4, 16, 0,
                           3.0, 2, 2, 1e-5),
    "olmoe_like": MoEConfig("olmoe_like", 2, "bf16", 1, 2048, 1024, 64, 0, 8, 16, 16, 128, 0,
                            2.5, 8, 8, 1e-3),
    "mixtral_like": MoEConfig("mixtral_like", 3, "bf16", 32, 4096, 14336, 8, 0, 2, 4, 8, 256, 0,
                              2.0, 2, 3, 1e-3),
    "phi35_like_concentrated": MoEConfig("phi35_like_concentrated", 4, "bf16", 32, 4096, 6400, 16,
                                         0, 2, 6, 32, 128, 0, 2.5, 3, 3, 1e-3),
    "phi35_like_diverse": MoEConfig("phi35_like_diverse", 4, "bf16", 32, 4096, 6400, 16,
                                    0, 2, 6, 32, 128, 0, 0.0, 0, 0, 1e-3),
    "deepseek_like": MoEConfig("deepseek_like", 5, "bf16", 28, 2048, 1408, 64, 2, 6, 12, 64, 64,
                               512, 2.0, 6, 6, 1e-3),
}


def get_config(name: str) -> MoEConfig:
    return CONFIGS[name]
