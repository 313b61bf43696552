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
    cfg, e, mat, method, keep_weights, keep_fp64_factors, rank, int3 = args
    return _compress_job(cfg, e, mat, method, keep_weights, keep_fp64_factors, rank, int3)


def _compress_one_single_thread(args):
    # worker processes: one BLAS thread each, the pool provides the parallelism
    try:
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):
            return _compress_one(args)
    except ImportError:
        return _compress_one(args)


def _compress_job(cfg, e, mat, method, keep_weights, keep_fp64_factors, rank=None, int3=False):
    shared = e >= cfg.n_experts
    W = synth.make_expert_weight(cfg, e, mat)
    r = 0 if shared else (cfg.rank if rank is None else int(rank))
    art = compress.compress_matrix(W, synth.expert_bits(cfg, e), cfg.group, r,
                                   method=method, seed=cfg.seed + 31 * e + mat,
                                   keep_fp64_factors=keep_fp64_factors, int3_factors=int3)
    art.pop("sigma", None)
    if rank is not None and not shared:
        art["rank"] = r            # this projection's own rank (Section 3.1)
    if keep_weights:
        art["W"] = W
    return e, mat, art


def kurtosis_ranks(cfg: LayerConfig, r_avg: int, buckets) -> np.ndarray:
    """Ranks [n_experts][3] of the routed experts' projections by the kurtosis-guided greedy
    allocation of Section 3.1 (step 1) on the seeded raw weights."""
    kappas = [compress.kurtosis(synth.make_expert_weight(cfg, e, mat))
              for e in range(cfg.n_experts) for mat in (synth.MAT_W1, synth.MAT_W3, synth.MAT_W2)]
    return compress.allocate_ranks(kappas, r_avg, buckets).reshape(cfg.n_experts, 3)


def build_layer(cfg: LayerConfig, method: str = "exact", keep_weights: bool = False,
                keep_fp64_factors: bool = False, progress: bool = False, workers: int = 0,
                ranks=None, int3_factors: bool = False) -> dict:
    """Quantize-then-compensate every expert of `cfg` (Section 3.1 step 2).  Uniform rank cfg.rank,
    or `ranks` [n_experts][3] (columns in the order W1, W3, W2) for a rank per projection.
    int3_factors: the factor pairs are stored at 3 bits ("Aq", "Bq") instead of bf16.

    Returns {"wg", "bias", "experts": [ {mat: artefacts} ... routed then shared ]}.
    Shared experts use cfg.shared_bits and carry no factors.  `workers` > 1 compresses the
    projections in that many processes (each one is independent and seeded on its own).
    """
    wg, bias = synth.make_gate(cfg)
    n_all = cfg.n_experts + cfg.n_shared
    order = (synth.MAT_W1, synth.MAT_W3, synth.MAT_W2)
    jobs = [(cfg, e, mat, method, keep_weights, keep_fp64_factors,
             None if ranks is None or e >= cfg.n_experts else int(ranks[e][order.index(mat)]), int3_factors)
            for e in range(n_all) for mat in order]
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


def stratified_rows(cnt: int) -> list:
    """Positions (0-based, within one expert's `cnt` grouped rows) that a full-size check must look
    at: the first and last row of the first and of the last 16-row tile of the first, a middle and
    the last (ragged) 128-row chunk; the same for the second 32-row pass when there is one (rows 32,
    47, 48, 63); and row 16 (the first row of a second row tile) whenever the expert has one."""
    pos = set()
    if cnt <= 0:
        return []
    chunks = (cnt + 127) // 128
    for c in sorted({0, chunks // 2, chunks - 1}):
        base = 128 * c
        n = min(128, cnt - base)
        last_tile = base + 16 * ((n - 1) // 16)
        for r in (base, min(base + 15, base + n - 1), last_tile, base + n - 1):
            pos.add(r)
    for r in (16, 31, 32, 47, 48, 63):
        if r < cnt:
            pos.add(r)
    return sorted(pos)


def stratified_token_mask(cfg: LayerConfig, route_idx: np.ndarray, perm: dict, min_tokens: int = 64) -> np.ndarray:
    """Tokens for a full-size output check: for every expert the tokens that hold its rows at
    stratified_rows(count), plus covering_token_mask (both flag classes of every active expert),
    padded to `min_tokens` with tokens spread evenly over the batch."""
    T, k = route_idx.shape
    mask = covering_token_mask(cfg, route_idx, min_tokens=0)
    off = perm["offsets"]
    for e in range(len(off) - 1):
        for r in stratified_rows(int(off[e + 1] - off[e])):
            mask[perm["row_pair"][off[e] + r] // k] = True
    want = min(min_tokens, T)
    if mask.sum() < want:
        for t in np.linspace(0, T - 1, num=T, dtype=np.int64)[:: max(1, T // want)]:
            if mask.sum() >= want:
                break
            mask[t] = True
        for t in range(T):
            if mask.sum() >= want:
                break
            mask[t] = True
    return mask
