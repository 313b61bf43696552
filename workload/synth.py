"""Seeded synthetic inputs for one MoE layer: tokens, gate, raw expert weights, and (for timing
runs) directly sampled stored artefacts.

Everything here is a random draw or a storage-format conversion (bf16 / fp16 bit patterns).
None of the method's arithmetic (routing, quantization, SVD, dequantization, FFN) lives in this
module: it serves both the CPU oracle and the HIP library, which share no other code.

Value recipe (stands in for the trained checkpoints and calibration text the paper measures on):
  tokens   x  ~ N(0,1), rounded to bf16
  gate     Wg ~ N(0, gate_std) per entry ("normal"), or N(0,1)/sqrt(H)*gate_std ("unit", so the
           logits have standard deviation gate_std); optional Zipf bias log p_e
  experts  W  ~ N(0, 0.02) fp32, a Bernoulli(0.001) subset of entries multiplied by 10
"""
from __future__ import annotations

from math import comb

import numpy as np

from .configs import LayerConfig

# tags that separate the random streams of one layer
_TAG_X, _TAG_GATE, _TAG_W, _TAG_ZIPF, _TAG_ART = 11, 12, 13, 14, 15

MAT_W1, MAT_W3, MAT_W2 = 0, 1, 2   # gate projection, up projection, down projection


# --------------------------------------------------------------------------- storage formats
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def f16_bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float16).view(np.uint16)


# --------------------------------------------------------------------------- shapes
def mat_shape(cfg: LayerConfig, mat: int) -> tuple[int, int]:
    """(K_in, N_out) of projection `mat`; weights are stored input-dim-major, y = x @ W."""
    return (cfg.ffn, cfg.hidden) if mat == MAT_W2 else (cfg.hidden, cfg.ffn)


def expert_bits(cfg: LayerConfig, expert: int) -> int:
    return cfg.shared_bits if expert >= cfg.n_experts else cfg.bits


# --------------------------------------------------------------------------- raw tensors
def make_tokens(cfg: LayerConfig, tokens: int | None = None) -> np.ndarray:
    """x[T][H] as bf16 bit patterns."""
    T = cfg.tokens if tokens is None else tokens
    rng = np.random.default_rng([cfg.seed, _TAG_X])
    return f32_to_bf16_bits(rng.standard_normal((T, cfg.hidden), dtype=np.float32))


def make_gate(cfg: LayerConfig) -> tuple[np.ndarray, np.ndarray | None]:
    """(Wg[E][H] bf16 bits, bias[E] float32 or None)."""
    rng = np.random.default_rng([cfg.seed, _TAG_GATE])
    wg = rng.standard_normal((cfg.n_experts, cfg.hidden), dtype=np.float32)
    if cfg.gate_kind == "unit":
        wg *= np.float32(cfg.gate_std / np.sqrt(cfg.hidden))
    elif cfg.gate_kind == "normal":
        wg *= np.float32(cfg.gate_std)
    else:
        raise ValueError(cfg.gate_kind)
    bias = None
    if cfg.zipf_s > 0:
        zr = np.random.default_rng([cfg.seed, _TAG_ZIPF])
        order = zr.permutation(cfg.n_experts)
        p = np.empty(cfg.n_experts, dtype=np.float64)
        p[order] = 1.0 / np.arange(1, cfg.n_experts + 1, dtype=np.float64) ** cfg.zipf_s
        p /= p.sum()
        bias = np.log(p).astype(np.float32)
    return f32_to_bf16_bits(wg), bias


def make_expert_weight(cfg: LayerConfig, expert: int, mat: int) -> np.ndarray:
    """Raw fp32 weight W[K][N] of one projection of one expert (routed: 0..E-1, shared: E..E+S-1)."""
    K, N = mat_shape(cfg, mat)
    rng = np.random.default_rng([cfg.seed, _TAG_W, expert, mat])
    w = rng.standard_normal((K, N), dtype=np.float32)
    w *= np.float32(0.02)
    mask = rng.random((K, N), dtype=np.float32) < np.float32(0.001)
    w[mask] *= np.float32(10.0)
    return w


# --------------------------------------------------------------------------- timing artefacts
def sample_artifacts(cfg: LayerConfig, expert: int, mat: int, with_factors: bool = True) -> dict:
    """Stored artefacts of one projection drawn directly (no weights, no quantizer, no SVD).

    For timing runs only: the kernels' work does not depend on the values, so codes come from a
    bell-shaped categorical over [0, 2^b), scale/zero from the ranges a min/max quantizer produces
    on N(0,0.02) weights, and factors are Gaussian with the magnitude of a residual's factors.
    Returns codes uint8 [K][N], scale/zero fp16 bits [K/g][N], A bf16 bits [K][r], B bf16 bits [r][N].
    """
    K, N = mat_shape(cfg, mat)
    b = expert_bits(cfg, expert)
    g, r = cfg.group, cfg.rank
    levels = (1 << b) - 1
    rng = np.random.default_rng([cfg.seed, _TAG_ART, expert, mat])
    # 256-entry table: byte -> code with binomial(levels, 1/2) frequencies
    pmf = np.array([comb(levels, i) for i in range(levels + 1)], dtype=np.float64)
    edges = np.floor(np.cumsum(pmf) / pmf.sum() * 256 + 0.5).astype(np.int64)
    table = np.zeros(256, dtype=np.uint8)
    lo = 0
    for code, hi in enumerate(edges):
        table[lo:hi] = code
        lo = hi
    codes = table[rng.integers(0, 256, size=(K, N), dtype=np.uint8)]
    scale = (0.096 / levels) * np.exp(0.15 * rng.standard_normal((K // g, N), dtype=np.float32))
    zero = 0.5 * levels + 0.15 * rng.standard_normal((K // g, N), dtype=np.float32)
    out = {"codes": codes, "scale": f16_bits(scale), "zero": f16_bits(zero), "A": None, "B": None}
    if with_factors and r > 0 and expert < cfg.n_experts:
        amp = np.float32(np.sqrt(0.028 * (np.sqrt(K) + np.sqrt(N)) / levels))
        out["A"] = f32_to_bf16_bits(amp / np.float32(np.sqrt(K)) * rng.standard_normal((K, r), dtype=np.float32))
        out["B"] = f32_to_bf16_bits(amp / np.float32(np.sqrt(N)) * rng.standard_normal((r, N), dtype=np.float32))
    return out


def sample_factor_codes(cfg: LayerConfig, expert: int, mat: int) -> tuple:
    """A factor pair held at 3 bits, drawn directly (for timing runs only): uniform codes, scale and
    zero of the magnitude a min/max quantizer gives on the factors of sample_artifacts.
    Returns (Aq, Bq): {"codes" uint8 [K][r] / [N][r], "scale", "zero" fp16 bits [K/64][r] / [N/64][r]}."""
    K, N = mat_shape(cfg, mat)
    r = cfg.rank
    rng = np.random.default_rng([cfg.seed, _TAG_ART, expert, mat, 3])
    out = []
    for rows in (K, N):
        codes = rng.integers(0, 8, size=(rows, r), dtype=np.uint8)
        scale = 0.004 * np.exp(0.15 * rng.standard_normal((rows // 64, r), dtype=np.float32))
        zero = 3.5 + 0.15 * rng.standard_normal((rows // 64, r), dtype=np.float32)
        out.append({"codes": codes, "scale": f16_bits(scale), "zero": f16_bits(zero)})
    return out[0], out[1]
