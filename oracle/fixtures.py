"""TEST INFRASTRUCTURE — builds the stored artefacts of a whole synthetic layer by running the
oracle-side compressor on the seeded raw weights.  Used by tests, the smoke check and the
benchmark's CPU-baseline leg; the product path never imports it.
"""
from __future__ import annotations

import sys
import time

import numpy as np

from workload import synth
from workload.configs import LayerConfig

from . import compress
from . import moe_lrc_oracle as orc


def build_layer(cfg: LayerConfig, method: str = "exact", keep_weights: bool = False,
                keep_fp64_factors: bool = False, progress: bool = False) -> dict:
    """Quantize-then-compensate every expert of `cfg` (Section 3.1 step 2, uniform rank).

    Returns {"wg", "bias", "experts": [ {mat: artefacts} ... routed then shared ]}.
    Shared experts use cfg.shared_bits and carry no factors.
    """
    wg, bias = synth.make_gate(cfg)
    experts = []
    t0 = time.time()
    for e in range(cfg.n_experts + cfg.n_shared):
        shared = e >= cfg.n_experts
        ex = {}
        for mat in (synth.MAT_W1, synth.MAT_W3, synth.MAT_W2):
            W = synth.make_expert_weight(cfg, e, mat)
            art = compress.compress_matrix(W, synth.expert_bits(cfg, e), cfg.group,
                                           0 if shared else cfg.rank, method=method,
                                           seed=cfg.seed + 31 * e + mat,
                                           keep_fp64_factors=keep_fp64_factors)
            if keep_weights:
                art["W"] = W
            ex[mat] = art
        experts.append(ex)
        if progress:
            print(f"[fixture {cfg.name}] expert {e + 1}/{cfg.n_experts + cfg.n_shared} "
                  f"compressed ({time.time() - t0:.0f}s)", flush=True, file=sys.stderr)
    return {"wg": wg, "bias": bias, "experts": experts}


def sample_layer(cfg: LayerConfig) -> dict:
    """A layer whose artefacts are drawn directly (workload.synth.sample_artifacts): for timing."""
    wg, bias = synth.make_gate(cfg)
    experts = [{mat: synth.sample_artifacts(cfg, e, mat) for mat in (0, 1, 2)}
               for e in range(cfg.n_experts + cfg.n_shared)]
    return {"wg": wg, "bias": bias, "experts": experts}


def oracle_forward(cfg: LayerConfig, layer: dict, x_bits: np.ndarray, token_mask=None) -> dict:
    return orc.forward(x_bits, layer["wg"], layer["experts"], n_experts=cfg.n_experts,
                       top_k=cfg.top_k, top_n=cfg.top_n, group=cfg.group,
                       renormalize=cfg.renormalize, bias=layer["bias"], n_shared=cfg.n_shared,
                       token_mask=token_mask)


def covering_token_mask(cfg: LayerConfig, route_idx: np.ndarray, min_tokens: int = 64) -> np.ndarray:
    """A deterministic token subset that touches every active expert in both flag classes
    (compensated / not) where such a pair exists, padded to `min_tokens` with the lowest ids."""
    T, k = route_idx.shape
    mask = np.zeros(T, bool)
    seen = set()
    for t in range(T):
        for j in range(k):
            key = (int(route_idx[t, j]), j < cfg.top_n)
            if key not in seen:
                seen.add(key)
                mask[t] = True
    for t in range(T):
        if mask.sum() >= min(min_tokens, T):
            break
        mask[t] = True
    return mask
