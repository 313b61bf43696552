"""Pins for the oracle's routing and grouping: brute force, closed forms, invariants,
constructed ties, and the router-score skew the paper reports (Section 2.2)."""
import itertools
import os

import numpy as np
import pytest

from oracle import moe_lrc_oracle as orc
from workload import configs, synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _bits(a):
    return synth.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def test_widening_is_exact():
    # every bf16 / fp16 bit pattern widens to the value numpy/torch assign to it
    import torch
    allbits = np.arange(65536, dtype=np.uint16)
    ref16 = torch.from_numpy(allbits.view(np.int16)).view(torch.float16).double().numpy()
    refb = torch.from_numpy(allbits.view(np.int16)).view(torch.bfloat16).double().numpy()
    np.testing.assert_array_equal(orc.f16_to_f64(allbits), ref16)
    np.testing.assert_array_equal(orc.bf16_to_f64(allbits), refb)


def test_softmax_closed_forms():
    rng = np.random.default_rng(0)
    z = rng.normal(size=(50, 9)) * 5
    s = orc.softmax(z)
    np.testing.assert_allclose(s.sum(axis=1), 1.0, atol=1e-15)
    np.testing.assert_allclose(orc.softmax(z + 123.456), s, rtol=1e-12)      # shift invariance
    np.testing.assert_array_equal(orc.softmax(np.array([[7.0]])), [[1.0]])    # one expert
    np.testing.assert_allclose(orc.softmax(np.zeros((1, 4))), 0.25)
    # two experts: logistic function of the logit difference
    d = 1.7
    np.testing.assert_allclose(orc.softmax(np.array([[d, 0.0]]))[0, 0], 1 / (1 + np.exp(-d)), rtol=1e-15)
    # overflow safety
    assert np.isfinite(orc.softmax(np.array([[1e4, 0.0, -1e4]]))).all()


def test_gate_logits_match_python_sum():
    rng = np.random.default_rng(1)
    x = _bits(rng.normal(size=(3, 40)))
    wg = _bits(rng.normal(size=(5, 40)))
    bias = rng.normal(size=5).astype(np.float32)
    got = orc.gate_logits(x, wg, bias)
    xf, wf = synth.bf16_bits_to_f32(x).astype(float), synth.bf16_bits_to_f32(wg).astype(float)
    for t in range(3):
        for e in range(5):
            ref = sum(float(xf[t, h]) * float(wf[e, h]) for h in range(40)) + float(bias[e])
            assert abs(got[t, e] - ref) < 1e-12


def _one_hot_tokens(logit_rows, E):
    """Tokens/gate such that logits are exactly `logit_rows`: x = one-hot rows, Wg[e][t] = logit."""
    T = len(logit_rows)
    x = np.eye(T, dtype=np.float32)
    wg = np.asarray(logit_rows, dtype=np.float32).T.copy()      # [E][T]
    return _bits(x), _bits(wg)


@pytest.mark.parametrize("E,k", [(3, 1), (4, 2), (5, 3), (6, 6)])
def test_topk_equals_brute_force_with_ties(E, k):
    # small-integer logits: ties are everywhere; brute force is the sorted() definition
    rows = list(itertools.product([-1, 0, 2], repeat=E))
    rng = np.random.default_rng(E * 10 + k)
    if len(rows) > 400:
        rows = [rows[i] for i in rng.choice(len(rows), 400, replace=False)]
    x, wg = _one_hot_tokens(rows, E)
    r = orc.route(x, wg, k)
    for t, row in enumerate(rows):
        brute = sorted(range(E), key=lambda e: (-row[e], e))[:k]
        assert list(r["idx"][t]) == brute, (row, r["idx"][t])
        sc = np.exp(np.array(row, float) - max(row))
        sc /= sc.sum()
        np.testing.assert_allclose(r["w"][t], sc[brute], rtol=1e-14)


def test_topk_random_vs_brute_force():
    rng = np.random.default_rng(7)
    for _ in range(20):
        E = int(rng.integers(2, 12)); k = int(rng.integers(1, E + 1)); T = 9; H = 16
        x = _bits(rng.normal(size=(T, H))); wg = _bits(rng.normal(size=(E, H)))
        r = orc.route(x, wg, k)
        for t in range(T):
            brute = sorted(range(E), key=lambda e: (-r["logits"][t, e], e))[:k]
            assert list(r["idx"][t]) == brute
        # sorted order: weights descend
        assert (np.diff(r["w"], axis=1) <= 0).all()


def test_constructed_ties_go_to_lower_index():
    rng = np.random.default_rng(3)
    H, E, k = 32, 8, 3
    wg = rng.normal(size=(E, H)).astype(np.float32)
    wg[5] = wg[2]                      # duplicated gate rows: experts 2 and 5 always tie
    wg[7] = wg[2]
    x = rng.normal(size=(20, H)).astype(np.float32)
    x[0] = 0.0                         # all-zero token: every score is 1/E
    r = orc.route(_bits(x), _bits(wg), k)
    assert list(r["idx"][0]) == [0, 1, 2]
    np.testing.assert_allclose(r["w"][0], 1.0 / E)
    for t in range(20):
        row = list(r["idx"][t])
        for hi in (5, 7):
            if hi in row:
                assert 2 in row and row.index(2) < row.index(hi)
        if 7 in row:
            assert 5 in row and row.index(5) < row.index(7)
    assert (r["margin"] >= 0).all() and r["margin"][0] == 0.0


def test_routing_weight_mass():
    cfg = configs.TINY
    x = synth.make_tokens(cfg); wg, _ = synth.make_gate(cfg)
    r0 = orc.route(x, wg, cfg.top_k, 0)
    r1 = orc.route(x, wg, cfg.top_k, 1)
    np.testing.assert_array_equal(r0["idx"], r1["idx"])
    np.testing.assert_allclose(r1["w"].sum(axis=1), 1.0, atol=1e-15)
    mass = np.sort(r0["scores"], axis=1)[:, -cfg.top_k:].sum(axis=1)
    np.testing.assert_allclose(r0["w"].sum(axis=1), mass, rtol=1e-14)
    assert (r0["w"].sum(axis=1) <= 1 + 1e-15).all()


def test_zipf_bias_shifts_load():
    cfg = configs.get("qwen3_T4096")
    x = synth.make_tokens(cfg); wg, bias = synth.make_gate(cfg)
    assert bias is not None
    r = orc.route(x, wg, cfg.top_k, 0, bias)
    load = np.bincount(r["idx"].ravel(), minlength=cfg.n_experts)
    # the expert with the largest prior gets far more than a uniform share, the smallest far less
    uniform = cfg.tokens * cfg.top_k / cfg.n_experts
    assert load[np.argmax(bias)] > 4 * uniform
    assert load[np.argmin(bias)] < 0.5 * uniform
    assert (r["margin"] > 1e-9).all()


def test_prefill_gate_reproduces_reported_skew():
    # synthetic stand-in for the calibration-set statistics: mean top-1 / top-2 scores fall in or
    # next to the bands the paper reports for the Mixtral models
    bands = {}
    for line in open(os.path.join(GOLDEN, "router_skew.txt")):
        if line.strip() and not line.startswith("#"):
            name, *v = line.split()
            bands[name] = [float(s) for s in v]
    cfg = configs.MIXTRAL_PREFILL
    x = synth.make_tokens(cfg); wg, _ = synth.make_gate(cfg)
    r = orc.route(x, wg, 2)
    top1, top2 = r["w"][:, 0].mean(), r["w"][:, 1].mean()
    lo1 = min(b[0] for b in bands.values()); hi1 = max(b[1] for b in bands.values())
    lo2 = min(b[2] for b in bands.values()); hi2 = max(b[3] for b in bands.values())
    assert lo1 <= top1 <= hi1 + 0.03, top1
    assert lo2 - 0.02 <= top2 <= hi2 + 0.02, top2
    assert (r["margin"] > 1e-9).all()


# ----------------------------------------------------------------------------- grouping
def _perm_brute(idx, E, n):
    T, k = idx.shape
    rows = []
    for e in range(E):
        for t in range(T):
            for j in range(k):
                if idx[t, j] == e:
                    rows.append((e, t, j))
    return rows


@pytest.mark.parametrize("T,E,k,n", [(1, 8, 2, 1), (16, 8, 2, 1), (33, 5, 3, 2), (64, 128, 8, 2), (7, 4, 4, 0)])
def test_permute_invariants_and_brute_force(T, E, k, n):
    rng = np.random.default_rng(T * 100 + E)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    p = orc.permute(idx, E, n)
    assert p["counts"].sum() == T * k
    np.testing.assert_array_equal(p["offsets"], np.concatenate([[0], np.cumsum(p["counts"])]))
    assert sorted(p["row_pair"]) == list(range(T * k))                 # bijection
    np.testing.assert_array_equal(p["pair_row"][p["row_pair"]], np.arange(T * k))
    assert p["comp_counts"].sum() == T * n
    brute = _perm_brute(idx, E, n)
    for row, (e, t, j) in enumerate(brute):
        assert p["row_pair"][row] == t * k + j
        assert p["offsets"][e] <= row < p["offsets"][e + 1]
    for e in range(E):
        toks = p["row_pair"][p["offsets"][e]:p["offsets"][e + 1]] // k
        assert (np.diff(toks) > 0).all()                               # strictly increasing tokens
        assert p["comp_counts"][e] == sum(1 for (ee, t, j) in brute if ee == e and j < n)
