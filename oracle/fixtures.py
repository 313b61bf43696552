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


def _compress_one(args):
    cfg, e, mat, method, keep_weights, keep_fp64_factors = args
    return _compress_job(cfg, e, mat, method, keep_weights, keep_fp64_factors)


def _compress_one_single_thread(args):
    # worker processes: one BLAS thread each, the pool provides the parallelism
    try:
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):
            return _compress_one(args)
    except ImportError:
        return _compress_one(args)


def _compress_job(cfg, e, mat, method, keep_weights, keep_fp64_factors):
    shared = e >= cfg.n_experts
    W = synth.make_expert_weight(cfg, e, mat)
    art = compress.compress_matrix(W, synth.expert_bits(cfg, e), cfg.group, 0 if shared else cfg.rank,
                                   method=method, seed=cfg.seed + 31 * e + mat,
                                   keep_fp64_factors=keep_fp64_factors)
    art.pop("sigma", None)
    if keep_weights:
        art["W"] = W
    return e, mat, art


def build_layer(cfg: LayerConfig, method: str = "exact", keep_weights: bool = False,
                keep_fp64_factors: bool = False, progress: bool = False, workers: int = 0) -> dict:
    """Quantize-then-compensate every expert of `cfg` (Section 3.1 step 2, uniform rank).

    Returns {"wg", "bias", "experts": [ {mat: artefacts} ... routed then shared ]}.
    Shared experts use cfg.shared_bits and carry no factors.  `workers` > 1 compresses the
    projections in that many processes (each one is independent and seeded on its own).
    """
    wg, bias = synth.make_gate(cfg)
    n_all = cfg.n_experts + cfg.n_shared
    jobs = [(cfg, e, mat, method, keep_weights, keep_fp64_factors)
            for e in range(n_all) for mat in (synth.MAT_W1, synth.MAT_W3, synth.MAT_W2)]
    experts = [dict() for _ in range(n_all)]
    t0 = time.time()
    done = 0

    def note():
        if progress and (done % max(1, len(jobs) // 8) == 0 or done == len(jobs)):
            print(f"[fixture {cfg.name}] {done}/{len(jobs)} projections compressed "
                  f"({time.time() - t0:.0f}s)", flush=True, file=sys.stderr)

    if workers > 1:
        import multiprocessing as mp
        with mp.get_context("fork").Pool(workers) as pool:
            for e, mat, art in pool.imap_unordered(_compress_one_single_thread, jobs):
                experts[e][mat] = art
                done += 1
                note()
    else:
        for job in jobs:
            e, mat, art = _compress_one(job)
            experts[e][mat] = art
            done += 1
            note()
    return {"wg": wg, "bias": bias, "experts": experts}


def default_workers() -> int:
    """Process count for full-size fixtures: the host's cores, at most 16."""
    import os
    return max(1, min(16, os.cpu_count() or 1))


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
