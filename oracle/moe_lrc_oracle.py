"""TEST INFRASTRUCTURE — plain fp64 CPU oracle of one router-guided, low-rank-compensated MoE layer.

This file is the definition the HIP library is checked against.  It is slow on purpose, shares no
code with the library, and must never be imported by the product path (only by tests, the smoke
check and the benchmark's CPU-baseline leg).

What it computes, on the *stored artefacts* (bf16 tokens and gate, b-bit codes, fp16 scale/zero,
bf16 factors), every stored value widened exactly to fp64 and no intermediate rounded:

  routing      w = softmax(G(x)) over all experts, the k highest form TopK        (Section 2.1)
  Top-n        the n < k highest-scored of those k, read off the sorted scores    (Section 3.2)
  weights      W_hat_e = Qinv(Q(W_e)) + U_e V_e for a Top-n (token, expert) pair,
               Qinv(Q(W_e)) otherwise                                             (Section 3.2)
  output       y = sum_{i in TopK} w_i E_i(x)  (+ always-on shared experts)      (Section 2.1, Table 1 note)

Readings where the paper is silent (each is listed with its reason in the design notes):
  * ties in Top-k / Top-n go to the lower expert index; the selection is made on the logits
    (softmax is monotone, so the order is the same and immune to rounding collisions);
  * routing weights are the softmax-over-all-experts scores, not renormalised over the k
    (Section 2.1's formula); `renormalize=1` divides by their sum;
  * compensation is per (token, expert) pair: slot j < n of a token's sorted list is compensated;
  * E_i(x) = (silu(x W1) * (x W3)) W2 with weights stored input-dim-major, y = x W;
  * Qinv(q) = (q - zero) * scale with one fp16 (scale, zero) per group of `group` consecutive
    input-dim entries of one output column;
  * shared experts: all tokens, weight 1, never compensated, outside the softmax.

Pinned by tests/test_oracle_*.py against brute-force sorting, a dense textbook MoE, closed forms,
Eckart-Young and the byte counts the paper prints in Section 4.4.
"""
from __future__ import annotations

import numpy as np

MAT_W1, MAT_W3, MAT_W2 = 0, 1, 2


# ----------------------------------------------------------------------------- exact widening
def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    with np.errstate(invalid="ignore"):          # signalling-NaN patterns widen to NaN quietly
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f16_to_f64(bits: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


# ----------------------------------------------------------------------------- routing
def gate_logits(x_bits: np.ndarray, wg_bits: np.ndarray, bias: np.ndarray | None = None) -> np.ndarray:
    """logit[t][e] = sum_h x[t][h] * Wg[e][h] (+ bias[e]); G(x) of Section 2.1 as a linear gate."""
    logits = bf16_to_f64(x_bits) @ bf16_to_f64(wg_bits).T
    if bias is not None:
        logits = logits + np.asarray(bias, dtype=np.float32).astype(np.float64)[None, :]
    return logits


def softmax(logits: np.ndarray) -> np.ndarray:
    z = logits - logits.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def route(x_bits, wg_bits, top_k: int, renormalize: int = 0, bias=None) -> dict:
    """Top-k routing of Section 2.1 with the sorted order Section 3.2 relies on.

    Returns idx[T][k] (descending score, ties to the lower index), w[T][k] fp64 routing weights,
    the logits, the scores, and `margin[T]`: the smallest gap between adjacent logits among sorted
    ranks 1..k+1 (how far the token is from a different selection or order).
    Slots 0..n-1 of a token's row are its Top-n experts.
    """
    logits = gate_logits(x_bits, wg_bits, bias)
    T, E = logits.shape
    scores = softmax(logits)
    # stable sort of -logit keeps the lower index first among equals
    order = np.argsort(-logits, axis=1, kind="stable")
    idx = order[:, :top_k].astype(np.int32)
    w = np.take_along_axis(scores, idx.astype(np.int64), axis=1)
    if renormalize:
        w = w / w.sum(axis=1, keepdims=True)
    upto = min(top_k + 1, E)
    srt = np.take_along_axis(logits, order[:, :upto], axis=1)
    margin = np.min(srt[:, :-1] - srt[:, 1:], axis=1) if upto > 1 else np.full(T, np.inf)
    return {"idx": idx, "w": w, "logits": logits, "scores": scores, "margin": margin}


# ----------------------------------------------------------------------------- grouping
def permute(topk_idx: np.ndarray, n_experts: int, top_n: int) -> dict:
    """Group the T*k (token, slot) pairs by expert: rows sorted by (expert asc, token asc).

    counts[e]       pairs routed to expert e
    offsets[e]      exclusive prefix sum of counts (offsets[E] = T*k)
    row_pair[p]     pair id t*k+j held by row p
    pair_row[t*k+j] row of that pair (inverse map)
    comp_counts[e]  pairs of expert e with slot j < top_n (those that take the low-rank term)
    """
    T, k = topk_idx.shape
    flat = topk_idx.reshape(-1).astype(np.int64)
    counts = np.bincount(flat, minlength=n_experts).astype(np.int32)
    offsets = np.zeros(n_experts + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    # pair ids ascend with the token, so a stable sort by expert gives (expert asc, token asc)
    row_pair = np.argsort(flat, kind="stable").astype(np.int32)
    pair_row = np.empty(T * k, dtype=np.int32)
    pair_row[row_pair] = np.arange(T * k, dtype=np.int32)
    slot = np.arange(T * k) % k
    comp_counts = np.bincount(flat[slot < top_n], minlength=n_experts).astype(np.int32)
    return {"counts": counts, "offsets": offsets, "row_pair": row_pair, "pair_row": pair_row,
            "comp_counts": comp_counts}


# ----------------------------------------------------------------------------- experts
FACTOR_GROUP = 64     # group size of the quantized factors along their long dimension (our choice: the paper gives none)


def dequant(codes: np.ndarray, scale_bits: np.ndarray, zero_bits: np.ndarray, group: int) -> np.ndarray:
    """Qinv(Q(W)) of Section 2.3: D[k][o] = (code[k][o] - zero[k/group][o]) * scale[k/group][o]."""
    K, N = codes.shape
    s = np.repeat(f16_to_f64(scale_bits), group, axis=0)[:K]
    z = np.repeat(f16_to_f64(zero_bits), group, axis=0)[:K]
    return (codes.astype(np.float64) - z) * s


def silu(g: np.ndarray) -> np.ndarray:
    return g / (1.0 + np.exp(-g))


def _project(X: np.ndarray, flags: np.ndarray, art: dict, group: int) -> np.ndarray:
    """X @ W_hat row by row: D for every row, plus (X A) B for rows whose flag is set (Section 3.2)."""
    out = X @ dequant(art["codes"], art["scale"], art["zero"], group)
    if art.get("Aq") is not None and flags.any():
        # INT3-quantized factors (Section 3.1 stores the factors at 3 bits): A [K][r] in groups of
        # FACTOR_GROUP along K, B kept transposed [N][r] in groups of FACTOR_GROUP along N
        A = dequant(art["Aq"]["codes"], art["Aq"]["scale"], art["Aq"]["zero"], FACTOR_GROUP)
        B = dequant(art["Bq"]["codes"], art["Bq"]["scale"], art["Bq"]["zero"], FACTOR_GROUP).T
        out[flags] += (X[flags] @ A) @ B
    elif art.get("A") is not None and flags.any():
        A = art["A"] if art["A"].dtype == np.float64 else bf16_to_f64(art["A"])
        B = art["B"] if art["B"].dtype == np.float64 else bf16_to_f64(art["B"])
        out[flags] += (X[flags] @ A) @ B
    return out


def expert_apply(X: np.ndarray, flags: np.ndarray, expert: dict, group: int) -> np.ndarray:
    """E_i(x) for a block of rows of one expert; `expert` maps MAT_W1/W3/W2 to stored artefacts."""
    g = _project(X, flags, expert[MAT_W1], group)
    u = _project(X, flags, expert[MAT_W3], group)
    h = silu(g) * u
    return _project(h, flags, expert[MAT_W2], group)


def expert_ffn(x_bits, perm: dict, experts, top_k: int, top_n: int, group: int,
               token_mask: np.ndarray | None = None) -> np.ndarray:
    """y_rows[T*k][H]: row p holds E_e(x_t) for the pair at row p.  Rows of tokens outside
    `token_mask` (if given) are left as NaN so that a partial evaluation cannot be misread."""
    X = bf16_to_f64(x_bits)
    T, H = X.shape
    y = np.full((T * top_k, H), np.nan)
    off = perm["offsets"]
    for e in range(len(off) - 1):
        rows = np.arange(off[e], off[e + 1])
        if rows.size == 0:
            continue
        pairs = perm["row_pair"][rows]
        tok, slot = pairs // top_k, pairs % top_k
        if token_mask is not None:
            keep = token_mask[tok]
            rows, tok, slot = rows[keep], tok[keep], slot[keep]
            if rows.size == 0:
                continue
        y[rows] = expert_apply(X[tok], slot < top_n, experts[e], group)
    return y


def combine(y_rows: np.ndarray, topk_w: np.ndarray, pair_row: np.ndarray,
            shared_out: np.ndarray | None = None) -> np.ndarray:
    """out[t] = sum_j w[t][j] * y_rows[pair_row[t*k+j]]  (+ shared experts with weight 1)."""
    T, k = topk_w.shape
    rows = pair_row.reshape(T, k)
    out = np.einsum("tj,tjh->th", topk_w, y_rows[rows])
    if shared_out is not None:
        out = out + shared_out
    return out


def forward(x_bits, wg_bits, experts, *, n_experts: int, top_k: int, top_n: int, group: int,
            renormalize: int = 0, bias=None, n_shared: int = 0, shared_group: int | None = None,
            token_mask: np.ndarray | None = None) -> dict:
    """The whole layer.  `experts` lists the routed experts then the shared ones.
    With `token_mask`, routing and grouping cover all tokens but expert outputs and `out` are
    evaluated for the masked tokens only (other rows NaN)."""
    r = route(x_bits, wg_bits, top_k, renormalize, bias)
    p = permute(r["idx"], n_experts, top_n)
    y_rows = expert_ffn(x_bits, p, experts, top_k, top_n, group, token_mask)
    shared = None
    if n_shared:
        X = bf16_to_f64(x_bits)
        sel = np.ones(X.shape[0], bool) if token_mask is None else token_mask
        shared = np.full(X.shape, np.nan)
        acc = np.zeros((int(sel.sum()), X.shape[1]))
        none = np.zeros(int(sel.sum()), bool)
        for s in range(n_shared):
            acc += expert_apply(X[sel], none, experts[n_experts + s], shared_group or group)
        shared[sel] = acc
    out = combine(y_rows, r["w"], p["pair_row"], shared)
    return {"route": r, "perm": p, "y_rows": y_rows, "out": out}


def rel_frobenius(got: np.ndarray, ref: np.ndarray) -> float:
    """|| got - ref ||_F / || ref ||_F over the entries where ref is defined (not NaN)."""
    m = ~np.isnan(ref)
    d = np.asarray(got, dtype=np.float64)[m] - ref[m]
    return float(np.sqrt((d * d).sum() / (ref[m] * ref[m]).sum()))
