"""Pins for the oracle's expert computation and the whole layer: special cases that reduce to a
textbook dense MoE written with a different library (torch, per-token loops), the two
algebraic forms of the compensation, and pair-level flags."""
import numpy as np
import pytest
import torch

from oracle import compress, fixtures
from oracle import moe_lrc_oracle as orc
from workload import configs, synth

torch.set_num_threads(4)


def dense_moe_torch(x_bits, wg_bits, weights, k, shared=(), bias=None, renorm=False):
    """Textbook MoE (Section 2.1): y = sum_{i in TopK} w_i E_i(x), E_i a SwiGLU FFN with dense
    fp64 weights, evaluated token by token with torch primitives.  `weights[e] = (W1, W3, W2)`,
    each [in][out]."""
    X = torch.from_numpy(synth.bf16_bits_to_f32(x_bits)).double()
    Wg = torch.from_numpy(synth.bf16_bits_to_f32(wg_bits)).double()
    out = torch.zeros_like(X)
    for t in range(X.shape[0]):
        logits = torch.nn.functional.linear(X[t], Wg)
        if bias is not None:
            logits = logits + torch.from_numpy(bias).double()
        scores = torch.softmax(logits, dim=0)
        top_w, top_i = torch.topk(scores, k)
        if renorm:
            top_w = top_w / top_w.sum()
        for w, e in zip(top_w, top_i):
            W1, W3, W2 = (torch.from_numpy(np.asarray(m, dtype=np.float64)) for m in weights[int(e)])
            h = torch.nn.functional.silu(X[t] @ W1) * (X[t] @ W3)
            out[t] += w * (h @ W2)
        for (W1, W3, W2) in shared:
            W1, W3, W2 = (torch.from_numpy(np.asarray(m, dtype=np.float64)) for m in (W1, W3, W2))
            out[t] += (torch.nn.functional.silu(X[t] @ W1) * (X[t] @ W3)) @ W2
    return out.numpy()


def _deq(ex, group):
    return tuple(orc.dequant(ex[m]["codes"], ex[m]["scale"], ex[m]["zero"], group) for m in (0, 1, 2))


def test_silu_matches_library():
    g = np.linspace(-30, 30, 1001)
    np.testing.assert_allclose(orc.silu(g), torch.nn.functional.silu(torch.from_numpy(g)).numpy(), rtol=1e-13, atol=1e-300)


def test_dequant_by_hand():
    # 1 output column, two groups of 2: D = (q - z) * s with per-group fp16 (s, z)
    codes = np.array([[0], [3], [1], [2]], dtype=np.uint8)
    scale = np.array([[0.5], [0.25]], dtype=np.float16).view(np.uint16)
    zero = np.array([[1.5], [1.0]], dtype=np.float16).view(np.uint16)
    np.testing.assert_array_equal(orc.dequant(codes, scale, zero, 2)[:, 0], [-0.75, 0.75, 0.0, 0.25])


def test_n0_is_the_pure_quantized_layer():
    cfg = configs.TINY.with_(top_n=0)
    layer = fixtures.build_layer(cfg)
    x = synth.make_tokens(cfg)
    got = fixtures.oracle_forward(cfg, layer, x)["out"]
    ref = dense_moe_torch(x, layer["wg"], [_deq(ex, cfg.group) for ex in layer["experts"]], cfg.top_k)
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)
    # and rank 0 with n > 0 is the same layer
    cfg_r0 = configs.TINY.with_(rank=0)
    got_r0 = fixtures.oracle_forward(cfg_r0, fixtures.build_layer(cfg_r0), x)["out"]
    np.testing.assert_array_equal(got, got_r0)


@pytest.mark.parametrize("renorm", [0, 1])
def test_full_rank_all_compensated_restores_the_fp_layer(renorm):
    # n = k and exact full-rank factors of the residual (kept in fp64): W_hat = W, so the layer
    # equals a dense floating-point MoE on the original weights
    cfg = configs.TINY.with_(hidden=64, ffn=128, top_n=2, rank=64, renormalize=renorm, tokens=12, group=32)
    layer = fixtures.build_layer(cfg, keep_weights=True, keep_fp64_factors=True)
    for ex in layer["experts"]:
        for m in (0, 1, 2):
            W_hat = orc.dequant(ex[m]["codes"], ex[m]["scale"], ex[m]["zero"], cfg.group) + ex[m]["A"] @ ex[m]["B"]
            np.testing.assert_allclose(W_hat, ex[m]["W"].astype(np.float64), atol=1e-12)
    x = synth.make_tokens(cfg)
    got = fixtures.oracle_forward(cfg, layer, x)["out"]
    ref = dense_moe_torch(x, layer["wg"], [tuple(ex[m]["W"] for m in (0, 1, 2)) for ex in layer["experts"]],
                          cfg.top_k, renorm=bool(renorm))
    np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-11)


def test_factored_and_materialised_forms_agree():
    # (x A) B on top of x D   ==   x (D + A B)   (Section 3.2's reconstruction)
    cfg = configs.TINY.with_(top_n=2)     # every pair compensated
    layer = fixtures.build_layer(cfg)
    x = synth.make_tokens(cfg)
    got = fixtures.oracle_forward(cfg, layer, x)["out"]
    W_hat = []
    for ex in layer["experts"]:
        W_hat.append(tuple(orc.dequant(ex[m]["codes"], ex[m]["scale"], ex[m]["zero"], cfg.group)
                           + orc.bf16_to_f64(ex[m]["A"]) @ orc.bf16_to_f64(ex[m]["B"]) for m in (0, 1, 2)))
    ref = dense_moe_torch(x, layer["wg"], W_hat, cfg.top_k)
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)


def test_pair_level_flags_brute_force():
    # n = 1 of k = 2: a token's first expert uses D + AB, its second uses D, even when the same
    # expert serves both kinds of pair in one batch
    cfg = configs.TINY.with_(tokens=24)
    layer = fixtures.build_layer(cfg)
    x = synth.make_tokens(cfg)
    res = fixtures.oracle_forward(cfg, layer, x)
    idx, w = res["route"]["idx"], res["route"]["w"]
    both = set(idx[:, 0]) & set(idx[:, 1])
    assert both, "fixture should have an expert that is Top-1 for one token and second for another"
    X = orc.bf16_to_f64(x)
    out = np.zeros_like(X)
    for t in range(cfg.tokens):
        for j in range(cfg.top_k):
            ex = layer["experts"][idx[t, j]]
            Ws = []
            for m in (0, 1, 2):
                Wm = orc.dequant(ex[m]["codes"], ex[m]["scale"], ex[m]["zero"], cfg.group)
                if j < cfg.top_n:
                    Wm = Wm + orc.bf16_to_f64(ex[m]["A"]) @ orc.bf16_to_f64(ex[m]["B"])
                Ws.append(Wm)
            g, u = X[t] @ Ws[0], X[t] @ Ws[1]
            out[t] += w[t, j] * ((g / (1 + np.exp(-g)) * u) @ Ws[2])
    np.testing.assert_allclose(res["out"], out, rtol=1e-10, atol=1e-12)
    # compensation moves the output towards the uncompressed layer
    assert orc.rel_frobenius(res["out"], fixtures.oracle_forward(cfg.with_(top_n=0), layer, x)["out"]) > 1e-3


def test_shared_experts_and_bias():
    cfg = configs.DEEPSEEK.with_(hidden=128, ffn=192, n_experts=8, tokens=10, top_k=3, top_n=0, rank=0, zipf_s=1.1)
    layer = fixtures.build_layer(cfg)
    x = synth.make_tokens(cfg)
    got = fixtures.oracle_forward(cfg, layer, x)["out"]
    E = cfg.n_experts
    ref = dense_moe_torch(x, layer["wg"], [_deq(ex, cfg.group) for ex in layer["experts"][:E]], cfg.top_k,
                          shared=[_deq(ex, cfg.group) for ex in layer["experts"][E:]], bias=layer["bias"])
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)


def test_token_mask_evaluates_subset_only():
    cfg = configs.TINY
    layer = fixtures.build_layer(cfg)
    x = synth.make_tokens(cfg)
    full = fixtures.oracle_forward(cfg, layer, x)
    mask = fixtures.covering_token_mask(cfg, full["route"]["idx"], min_tokens=4)
    part = fixtures.oracle_forward(cfg, layer, x, token_mask=mask)
    np.testing.assert_allclose(part["out"][mask], full["out"][mask], rtol=1e-10, atol=1e-14)
    assert np.isnan(part["out"][~mask]).all()
    seen = {(int(full["route"]["idx"][t, j]), j < cfg.top_n) for t in np.nonzero(mask)[0] for j in range(cfg.top_k)}
    allp = {(int(full["route"]["idx"][t, j]), j < cfg.top_n) for t in range(cfg.tokens) for j in range(cfg.top_k)}
    assert seen == allp


def test_compensation_reduces_layer_error():
    # the point of the method: Top-n compensation brings the quantized layer closer to the fp layer
    cfg = configs.TINY.with_(rank=32)
    layer = fixtures.build_layer(cfg, keep_weights=True)
    x = synth.make_tokens(cfg)
    fp = dense_moe_torch(x, layer["wg"], [tuple(ex[m]["W"] for m in (0, 1, 2)) for ex in layer["experts"]], cfg.top_k)
    errs = [orc.rel_frobenius(fixtures.oracle_forward(cfg.with_(top_n=n), layer, x)["out"], fp) for n in (0, 1, 2)]
    assert errs[0] > errs[1] > errs[2]


def test_rank_per_projection_from_kurtosis():
    # Section 3.1: the rank budget goes to the matrices in descending kurtosis order, so every
    # projection has a rank of its own (0 included).  The layer with such factors equals the
    # materialised form built from each projection's own factor pair.
    cfg = configs.TINY.with_(rank=32, top_n=2)
    ranks = fixtures.kurtosis_ranks(cfg, 10, (0, 8, 16, 32))
    assert ranks.shape == (cfg.n_experts, 3) and ranks.sum() <= cfg.n_experts * 3 * 10
    assert len(set(ranks.ravel().tolist())) >= 3 and (ranks[:, 0] != ranks[:, 1]).any()
    layer = fixtures.build_layer(cfg, ranks=ranks)
    for e, ex in enumerate(layer["experts"]):
        for j, m in enumerate((0, 1, 2)):
            r = int(ranks[e][j])
            assert ex[m]["rank"] == r
            assert (ex[m]["A"] is None) == (r == 0)
            if r:
                assert ex[m]["A"].shape[1] == r and ex[m]["B"].shape[0] == r
    x = synth.make_tokens(cfg)
    got = fixtures.oracle_forward(cfg, layer, x)["out"]
    W_hat = []
    for ex in layer["experts"]:
        mats = []
        for m in (0, 1, 2):
            Wm = orc.dequant(ex[m]["codes"], ex[m]["scale"], ex[m]["zero"], cfg.group)
            if ex[m]["A"] is not None:
                Wm = Wm + orc.bf16_to_f64(ex[m]["A"]) @ orc.bf16_to_f64(ex[m]["B"])
            mats.append(Wm)
        W_hat.append(tuple(mats))
    ref = dense_moe_torch(x, layer["wg"], W_hat, cfg.top_k)
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-12)


def test_int3_factors_layer_equals_materialised_form_and_still_compensates():
    # Section 3.1 step 2 stores the factors at INT3.  The layer with quantized factors equals the
    # materialised form D + Qinv(Aq) Qinv(Bq)^T, and the quantized compensator still removes most of
    # what the bf16 one removes of the quantization error.
    cfg = configs.TINY.with_(top_n=2, rank=16, bits=2)
    x = synth.make_tokens(cfg)
    layer_q = fixtures.build_layer(cfg, int3_factors=True, keep_weights=True)
    got = fixtures.oracle_forward(cfg, layer_q, x)["out"]
    W_hat = []
    for ex in layer_q["experts"]:
        mats = []
        for m in (0, 1, 2):
            a = ex[m]
            assert a["A"] is None and a["Aq"]["codes"].max() <= 7 and a["Bq"]["codes"].shape == (a["codes"].shape[1], cfg.rank)
            A = orc.dequant(a["Aq"]["codes"], a["Aq"]["scale"], a["Aq"]["zero"], orc.FACTOR_GROUP)
            B = orc.dequant(a["Bq"]["codes"], a["Bq"]["scale"], a["Bq"]["zero"], orc.FACTOR_GROUP).T
            mats.append(orc.dequant(a["codes"], a["scale"], a["zero"], cfg.group) + A @ B)
        W_hat.append(tuple(mats))
    np.testing.assert_allclose(got, dense_moe_torch(x, layer_q["wg"], W_hat, cfg.top_k), rtol=1e-10, atol=1e-12)
    dense = dense_moe_torch(x, layer_q["wg"], [tuple(ex[m]["W"] for m in (0, 1, 2)) for ex in layer_q["experts"]], cfg.top_k)
    layer_b = fixtures.build_layer(cfg)
    e_none = orc.rel_frobenius(fixtures.oracle_forward(cfg.with_(top_n=0), layer_b, x)["out"], dense)
    e_bf16 = orc.rel_frobenius(fixtures.oracle_forward(cfg, layer_b, x)["out"], dense)
    e_int3 = orc.rel_frobenius(got, dense)
    assert e_bf16 < e_int3 < e_none
    assert (e_none - e_int3) > 0.5 * (e_none - e_bf16)


def test_factor_byte_accounting_at_int3():
    from oracle import compress
    # one expert's factor pairs at rank 32 of a Mixtral-sized layer: 3 bits per value + scale/zero per 64
    H, F, r = 4096, 14336, 32
    vals = 3 * r * (H + F)
    assert compress.compensator_bytes(H, F, r, 3) == vals * 3 // 8
    assert compress.factor_meta_bytes(H, F, r) == vals // 64 * 4
