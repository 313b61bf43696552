"""Pins of the comparison metric and of the token subset the full-size GPU checks use (CPU only).

Every GPU tolerance assertion goes through oracle.rel_frobenius, so it is pinned against values
worked out by hand: a slip in it (a missing square root, a wrong mask, a norm of the wrong operand)
would let every parity test pass vacuously.
"""
import math

import numpy as np

from oracle import fixtures
from oracle import moe_lrc_oracle as orc
from workload import configs


def test_rel_frobenius_by_hand():
    ref = np.array([[3.0, 4.0], [0.0, 12.0]])           # ||ref||_F = 13
    got = np.array([[3.0, 4.5], [1.0, 12.0]])           # difference (0, .5, 1, 0): norm sqrt(1.25)
    assert math.isclose(orc.rel_frobenius(got, ref), math.sqrt(1.25) / 13.0, rel_tol=1e-15)
    assert orc.rel_frobenius(ref, ref) == 0.0
    # scale invariance and the square root: doubling the difference doubles the metric
    got2 = ref + 2.0 * (got - ref)
    assert math.isclose(orc.rel_frobenius(got2, ref), 2.0 * math.sqrt(1.25) / 13.0, rel_tol=1e-15)
    assert math.isclose(orc.rel_frobenius(10.0 * got, 10.0 * ref), math.sqrt(1.25) / 13.0, rel_tol=1e-15)
    # a relative perturbation eps of every entry gives exactly eps
    assert math.isclose(orc.rel_frobenius(ref * (1 + 2.4e-3), ref), 2.4e-3, rel_tol=1e-12)


def test_rel_frobenius_nan_mask():
    # entries where the reference is undefined (rows the oracle did not evaluate) do not count,
    # whatever the other side holds there; entries where it is defined always count
    ref = np.array([[3.0, 4.0], [np.nan, np.nan], [0.0, 12.0]])
    got = np.array([[3.0, 4.5], [1e30, -7.0], [1.0, 12.0]])
    assert math.isclose(orc.rel_frobenius(got, ref), math.sqrt(1.25) / 13.0, rel_tol=1e-15)
    got_bad = got.copy()
    got_bad[0, 0] = np.nan                                 # a NaN where the reference is defined must show
    assert math.isnan(orc.rel_frobenius(got_bad, ref))


def test_stratified_rows_cover_every_class():
    for cnt in list(range(0, 70)) + [100, 127, 128, 129, 255, 256, 257, 519, 520, 640, 1000]:
        pos = fixtures.stratified_rows(cnt)
        assert pos == sorted(set(pos)) and all(0 <= r < cnt for r in pos)
        if cnt == 0:
            assert pos == []
            continue
        assert 0 in pos and cnt - 1 in pos
        if cnt > 16:
            assert 16 in pos and 15 in pos                 # both row tiles of a 32-row pass
        if cnt > 32:
            assert 32 in pos                               # a second 32-row pass
        chunks = (cnt + 127) // 128
        for c in {0, chunks // 2, chunks - 1}:             # first, middle and last 128-row chunk
            base, n = 128 * c, min(128, cnt - 128 * c)
            assert base in pos and base + n - 1 in pos
            assert base + 16 * ((n - 1) // 16) in pos      # first row of the chunk's last row tile


def test_stratified_token_mask_reaches_high_rows():
    # Mixtral-shaped routing statistics at small hidden size: the mask must reach, for every
    # expert, its last row and a row of its second row tile, and hold at least 64 tokens
    for name, T in (("mixtral_decode", 64), ("mixtral_prefill", 2048), ("deepseek", 512), ("qwen3", 4096)):
        cfg = configs.get(name).with_(hidden=256, tokens=T)
        from workload import synth
        wg, bias = synth.make_gate(cfg)
        r = orc.route(synth.make_tokens(cfg), wg, cfg.top_k, cfg.renormalize, bias)
        p = orc.permute(r["idx"], cfg.n_experts, cfg.top_n)
        mask = fixtures.stratified_token_mask(cfg, r["idx"], p, min_tokens=64)
        assert mask.sum() >= min(64, T)
        assert fixtures.covering_token_mask(cfg, r["idx"], 0)[~mask].sum() == 0
        for e in range(cfg.n_experts):
            lo, hi = p["offsets"][e], p["offsets"][e + 1]
            tok = p["row_pair"][lo:hi] // cfg.top_k
            hit = np.flatnonzero(mask[tok])
            for rpos in fixtures.stratified_rows(int(hi - lo)):
                assert rpos in hit
