"""Named synthetic workloads: shapes and routing statistics of the layers the paper evaluates.

Shapes follow Table 1 of the paper (Mixtral-8x7B: hidden 4096, expert FFN 14336, 8 experts,
top-2; DeepSeek-MoE-16B: 64 routed + 2 shared experts, top-6) plus a Qwen3-30B-A3B-shaped layer.
Compensation settings follow Section 4.2 (top-1 restored for Mixtral, a few for the fine-grained
models).  This module holds shapes and seeds only: none of the method's arithmetic lives here.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional


@dataclass(frozen=True)
class LayerConfig:
    name: str
    hidden: int            # H
    ffn: int               # F (per-expert SwiGLU width)
    n_experts: int         # E routed experts
    top_k: int             # k
    top_n: int             # n <= k, pairs that receive the low-rank correction
    bits: int              # routed-expert code width
    group: int             # quantization group along the input dimension
    rank: int              # compensator rank r (uniform per layer)
    tokens: int            # T
    n_shared: int = 0      # S always-on shared experts
    shared_bits: int = 4
    renormalize: int = 0   # 0: weights are softmax-over-all scores (Section 2.1); 1: divide by sum over top-k
    gate_kind: str = "normal"   # "normal": Wg ~ N(0, gate_std); "unit": Wg ~ N(0,1)/sqrt(H) * gate_std
    gate_std: float = 0.5
    zipf_s: float = 0.0    # > 0: add log p_e, p_e ~ rank^-s over a seeded expert permutation, to the logits
    seed: int = 1234

    def with_(self, **kw) -> "LayerConfig":
        return replace(self, **kw)

    @property
    def params_per_expert(self) -> int:
        return 3 * self.hidden * self.ffn


TINY = LayerConfig("tiny", hidden=256, ffn=512, n_experts=8, top_k=2, top_n=1, bits=3, group=64,
                   rank=8, tokens=16, gate_std=0.5, seed=1234)

MIXTRAL_DECODE = LayerConfig("mixtral_decode", hidden=4096, ffn=14336, n_experts=8, top_k=2, top_n=1,
                             bits=2, group=64, rank=32, tokens=64, gate_std=0.5, seed=1235)

# gate_std here is the logit standard deviation: 2.2 puts ~0.60 of the score mass on the top-1
# expert and ~0.20 on the second for 8 experts, the skew Section 2.2 reports for Mixtral.
MIXTRAL_PREFILL = LayerConfig("mixtral_prefill", hidden=4096, ffn=14336, n_experts=8, top_k=2, top_n=1,
                              bits=3, group=64, rank=64, tokens=2048, gate_kind="unit", gate_std=2.2,
                              seed=1236)

DEEPSEEK = LayerConfig("deepseek", hidden=2048, ffn=1408, n_experts=64, n_shared=2, top_k=6, top_n=2,
                       bits=2, shared_bits=4, group=64, rank=16, tokens=512, gate_std=0.3, seed=1237)

QWEN3 = LayerConfig("qwen3", hidden=2048, ffn=768, n_experts=128, top_k=8, top_n=2, bits=3, group=128,
                    rank=16, tokens=64, gate_kind="unit", gate_std=1.0, zipf_s=1.1, seed=1238)


def get(name: str) -> LayerConfig:
    """Look up a workload by name, e.g. 'mixtral_decode_T8_b3', 'qwen3_T4096', 'tiny'."""
    base = {"tiny": TINY, "mixtral_decode": MIXTRAL_DECODE, "mixtral_prefill": MIXTRAL_PREFILL,
            "deepseek": DEEPSEEK, "qwen3": QWEN3}
    parts = name.split("_")
    # longest prefix that names a base config
    for cut in range(len(parts), 0, -1):
        key = "_".join(parts[:cut])
        if key in base:
            cfg = base[key]
            for opt in parts[cut:]:
                if opt.startswith("T") and opt[1:].isdigit():
                    cfg = cfg.with_(tokens=int(opt[1:]))
                elif opt.startswith("b") and opt[1:].isdigit():
                    cfg = cfg.with_(bits=int(opt[1:]))
                elif opt.startswith("r") and opt[1:].isdigit():
                    cfg = cfg.with_(rank=int(opt[1:]))
                elif opt.startswith("n") and opt[1:].isdigit():
                    cfg = cfg.with_(top_n=int(opt[1:]))
                else:
                    raise KeyError(f"unknown workload option {opt!r} in {name!r}")
            return cfg.with_(name=name)
    raise KeyError(f"unknown workload {name!r}")


def small_variant(cfg: LayerConfig, hidden: int, ffn: int, tokens: Optional[int] = None) -> LayerConfig:
    """Same routing structure, smaller matrices: for cases the oracle must finish in seconds."""
    return cfg.with_(hidden=hidden, ffn=ffn, tokens=cfg.tokens if tokens is None else tokens,
                     name=f"{cfg.name}_small")
