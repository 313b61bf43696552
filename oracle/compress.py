"""TEST INFRASTRUCTURE — the offline half of the method, in plain numpy fp64: group-wise uniform
quantization, the quantization residual and its rank-r factors, kurtosis, the greedy bucketed
rank allocation, and the transfer-size accounting.  It builds the stored artefacts that both the
oracle's forward pass and the HIP library consume; the product path never imports it.

  residual      E = W - Qinv(Q(W))                                   (Section 2.3)
  factors       U, S, Vt = SVD_r(E);  U <- U sqrt(S),  V <- sqrt(S) Vt   (Section 3.1, step 2)
  kurtosis      kappa = (1/d) sum_j (w_j - mu)^4 / sigma^4           (Section 3.1, step 1)
  allocation    sort by kappa descending, give each matrix the largest bucket value that keeps
                sum r_i <= N * R_avg                                  (Section 3.1, step 1)
  sizes         the per-expert transfer sizes of Section 4.4

Readings: the quantizer is plain asymmetric min/max round-to-nearest per group of `group` input-dim
entries of one output column (the paper's HQQ-style refinement is a third-party method with no
stated hyper-parameters; the forward pass is agnostic to how codes were chosen).  scale and zero
are rounded to fp16 *before* the codes are chosen, so the codes are optimal for the stored values.
A constant group (max == min, or a scale that rounds to 0 in fp16) gets scale 1, zero = -min, codes 0.
Factors are rounded to bf16 for storage (INT3 factors, as the paper stores them, are a later row).
"""
from __future__ import annotations

import numpy as np

RANK_BUCKETS = (0, 16, 32, 128, 256, 512, 1024)   # Section 3.1


# ----------------------------------------------------------------------------- storage rounding
def round_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float -> bf16 bit patterns, round to nearest even (via float32, exact for the magnitudes here)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


# ----------------------------------------------------------------------------- quantizer
def quantize_groupwise(W: np.ndarray, bits: int, group: int) -> dict:
    """Q(W): codes uint8 [K][N] in [0, 2^bits), scale/zero as fp16 bit patterns [K/group][N]."""
    K, N = W.shape
    if K % group:
        raise ValueError("K must be a multiple of the group size")
    levels = (1 << bits) - 1
    Wg = np.asarray(W, dtype=np.float64).reshape(K // group, group, N)
    lo, hi = Wg.min(axis=1), Wg.max(axis=1)
    with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
        s = ((hi - lo) / levels).astype(np.float16)
        degenerate = ~(s.astype(np.float64) > 0) | ~np.isfinite(s.astype(np.float64))
        s = np.where(degenerate, np.float16(1.0), s)
        z = (-lo / s.astype(np.float64))
        z = np.where(degenerate, -lo, z).astype(np.float16)
        q = np.rint(Wg / s.astype(np.float64)[:, None, :] + z.astype(np.float64)[:, None, :])
    q = np.where(degenerate[:, None, :], 0.0, q)
    codes = np.clip(q, 0, levels).astype(np.uint8).reshape(K, N)
    return {"codes": codes, "scale": s.view(np.uint16), "zero": z.view(np.uint16)}


def shrink_lp(x: np.ndarray, beta: float, p: float) -> np.ndarray:
    """Generalised soft threshold of the half-quadratic solver: sign(x) max(|x| - |x|^(p-1) / beta, 0)
    (0 at x = 0).  For p = 1 this is the ordinary soft threshold with width 1 / beta."""
    ax = np.abs(x)
    with np.errstate(divide="ignore", invalid="ignore"):
        t = np.where(ax > 0, ax - ax ** (p - 1.0) / beta, 0.0)
    return np.sign(x) * np.maximum(t, 0.0)


def quantize_refined(W: np.ndarray, bits: int, group: int, iters: int = 20, p: float = 0.7, beta: float = 10.0,
                     kappa: float = 1.01) -> dict:
    """Q(W) with the zero points refined by a half-quadratic solver (Section 3.1 step 2 names an
    "HQQ-style weight optimization" without parameters; this is the published half-quadratic scheme
    with its customary settings: l_p error with p = 0.7, penalty 10 growing by 1 % per step, 20 steps).
    Per group, with the min/max scale s (rounded to fp16) kept fixed and the zero point z real-valued:
        q  = clamp(round(w / s + z), 0, 2^bits - 1)
        e  = shrink_lp(w - (q - z) s, beta, p)          (the part of the error the l_p term keeps)
        z  = mean over the group of (q - (w - e) / s)   (least squares for what is left)
        beta <- kappa beta
    then z is rounded to fp16 and the codes are chosen once more for the stored values.  iters = 0 is
    quantize_groupwise.  Degenerate groups are handled as there."""
    K, N = W.shape
    if K % group:
        raise ValueError("K must be a multiple of the group size")
    levels = (1 << bits) - 1
    Wg = np.asarray(W, dtype=np.float64).reshape(K // group, group, N)
    lo, hi = Wg.min(axis=1), Wg.max(axis=1)
    with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
        s16 = ((hi - lo) / levels).astype(np.float16)
        degenerate = ~(s16.astype(np.float64) > 0) | ~np.isfinite(s16.astype(np.float64))
        s16 = np.where(degenerate, np.float16(1.0), s16)
        s = s16.astype(np.float64)
        z = np.where(degenerate, -lo, -lo / s)
        b = float(beta)
        for _ in range(iters):
            q = np.clip(np.rint(Wg / s[:, None, :] + z[:, None, :]), 0, levels)
            e = shrink_lp(Wg - (q - z[:, None, :]) * s[:, None, :], b, p)
            z_new = (q - (Wg - e) / s[:, None, :]).mean(axis=1)
            z = np.where(degenerate, z, z_new)
            b *= kappa
        z16 = z.astype(np.float16)
        q = np.rint(Wg / s[:, None, :] + z16.astype(np.float64)[:, None, :])
    q = np.where(degenerate[:, None, :], 0.0, q)
    codes = np.clip(q, 0, levels).astype(np.uint8).reshape(K, N)
    return {"codes": codes, "scale": s16.view(np.uint16), "zero": z16.view(np.uint16)}


def dequantize(q: dict, group: int) -> np.ndarray:
    """Qinv(Q(W)) in fp64 from the stored values."""
    s = np.repeat(q["scale"].view(np.float16).astype(np.float64), group, axis=0)
    z = np.repeat(q["zero"].view(np.float16).astype(np.float64), group, axis=0)
    return (q["codes"].astype(np.float64) - z) * s


# ----------------------------------------------------------------------------- low-rank factors
def residual_factors(E: np.ndarray, r: int, method: str = "exact", seed: int = 0, power_iters: int = 2):
    """(A = U_r sqrt(S_r), B = sqrt(S_r) Vt_r, singular values used) in fp64.

    method "exact": LAPACK SVD of E.  "gram": eigen-decomposition of the smaller Gram matrix (same
    factors up to rounding, for matrices where the full SVD is too slow).  "randomized": subspace
    iteration (Halko-Martinsson-Tropp) — an approximation of SVD_r used only to build full-size
    fixtures quickly; the forward pass is checked on whatever factors are stored.
    """
    E = np.asarray(E, dtype=np.float64)
    K, N = E.shape
    if r == 0:
        return np.zeros((K, 0)), np.zeros((0, N)), np.zeros(0)
    if method == "exact":
        U, S, Vt = np.linalg.svd(E, full_matrices=False)
        U, S, Vt = U[:, :r], S[:r], Vt[:r]
    elif method == "gram":
        if K <= N:
            lam, Q = np.linalg.eigh(E @ E.T)
            U = Q[:, ::-1][:, :r]
            S = np.sqrt(np.maximum(lam[::-1][:r], 0))
            Vt = (U.T @ E) / S[:, None]
        else:
            lam, Q = np.linalg.eigh(E.T @ E)
            V = Q[:, ::-1][:, :r]
            S = np.sqrt(np.maximum(lam[::-1][:r], 0))
            U = (E @ V) / S[None, :]
            Vt = V.T
    elif method == "randomized":
        rng = np.random.default_rng(seed)
        Y = E @ rng.standard_normal((N, r + 8))
        for _ in range(power_iters):
            Y, _ = np.linalg.qr(Y)
            Y = E @ (E.T @ Y)
        Qm, _ = np.linalg.qr(Y)
        Ub, S, Vt = np.linalg.svd(Qm.T @ E, full_matrices=False)
        U, S, Vt = (Qm @ Ub)[:, :r], S[:r], Vt[:r]
    else:
        raise ValueError(method)
    root = np.sqrt(S)
    return U * root[None, :], root[:, None] * Vt, S


FACTOR_BITS, FACTOR_GROUP = 3, 64


def quantize_factors(A: np.ndarray, B: np.ndarray) -> tuple:
    """(Aq, Bq): the factor pair at FACTOR_BITS bits (Section 3.1 step 2 stores the factors at INT3).
    The paper gives no group format; here both factors are quantized like the weights (asymmetric,
    fp16 scale/zero) in groups of FACTOR_GROUP along their long dimension, one rank index per
    column: A [K][r] along K, B as its transpose [N][r] along N."""
    return (quantize_groupwise(np.asarray(A, np.float64), FACTOR_BITS, FACTOR_GROUP),
            quantize_groupwise(np.asarray(B, np.float64).T.copy(), FACTOR_BITS, FACTOR_GROUP))


def compress_matrix(W: np.ndarray, bits: int, group: int, rank: int, method: str = "exact",
                    seed: int = 0, keep_fp64_factors: bool = False, int3_factors: bool = False) -> dict:
    """Quantize-then-compensate for one matrix: stored artefacts in the layout the C ABI takes.
    int3_factors: the factor pair is stored quantized ("Aq", "Bq") instead of as bf16 ("A", "B")."""
    q = quantize_groupwise(W, bits, group)
    art = {"codes": q["codes"], "scale": q["scale"], "zero": q["zero"], "A": None, "B": None}
    if rank > 0:
        E = np.asarray(W, dtype=np.float64) - dequantize(q, group)
        A, B, S = residual_factors(E, rank, method, seed)
        art["sigma"] = S
        if int3_factors:
            art["Aq"], art["Bq"] = quantize_factors(A, B)
        elif keep_fp64_factors:
            art["A"], art["B"] = A, B
        else:
            art["A"], art["B"] = round_to_bf16_bits(A), round_to_bf16_bits(B)
    return art


# ----------------------------------------------------------------------------- rank allocation
def kurtosis(W: np.ndarray) -> float:
    """Non-excess kurtosis over all entries of a matrix (a Gaussian gives 3)."""
    w = np.asarray(W, dtype=np.float64).ravel()
    mu = w.mean()
    var = ((w - mu) ** 2).mean()
    return float((((w - mu) ** 4).mean()) / (var * var))


def allocate_ranks(kappas, r_avg: int, buckets=RANK_BUCKETS) -> np.ndarray:
    """Greedy bucketed allocation: in descending kurtosis order, each matrix takes the largest
    bucket value that keeps the running total within N * r_avg."""
    kappas = np.asarray(kappas, dtype=np.float64)
    budget = len(kappas) * r_avg
    ranks = np.zeros(len(kappas), dtype=np.int64)
    used = 0
    for i in np.argsort(-kappas, kind="stable"):
        fit = [b for b in buckets if used + b <= budget]
        ranks[i] = max(fit) if fit else 0
        used += ranks[i]
    return ranks


# ----------------------------------------------------------------------------- transfer sizes
def expert_code_bytes(hidden: int, ffn: int, bits: int) -> int:
    """Bytes of one expert's three packed projections at a dense `bits` per weight."""
    return 3 * hidden * ffn * bits // 8


def expert_meta_bytes(hidden: int, ffn: int, group: int) -> int:
    """fp16 scale + fp16 zero per group of one expert's three projections."""
    return 3 * hidden * ffn // group * 4


def factor_meta_bytes(hidden: int, ffn: int, rank: int) -> int:
    """fp16 scale + fp16 zero per group of FACTOR_GROUP of one expert's three quantized factor pairs:
    every pair has r (K + N) values."""
    return 3 * rank * (hidden + ffn) // FACTOR_GROUP * 4


def compensator_bytes(hidden: int, ffn: int, rank: int, factor_bits: int) -> int:
    """Bytes of one expert's three factor pairs: 3 * r * (H + F) values of `factor_bits` each."""
    return 3 * rank * (hidden + ffn) * factor_bits // 8


def staged_bytes(counts, comp_counts, hidden: int, ffn: int, bits: int, group: int, rank: int,
                 factor_bits: int = 16) -> dict:
    """What the router-guided transfer of Section 3.2 moves for one batch: packed codes and
    scale/zero of every expert with a routed pair, factors only of experts with a Top-n pair."""
    active = int((np.asarray(counts) > 0).sum())
    comp = int((np.asarray(comp_counts) > 0).sum())
    return {"active_experts": active, "comp_experts": comp,
            "bytes_codes": active * expert_code_bytes(hidden, ffn, bits),
            "bytes_meta": active * expert_meta_bytes(hidden, ffn, group),
            "bytes_factors": comp * compensator_bytes(hidden, ffn, rank, factor_bits)}
