"""Pins for the offline side: quantizer bounds, Eckart-Young for the truncated factors, the
reparameterisation invariant, kurtosis closed forms, the greedy rank allocation and the transfer
sizes the paper prints (Section 4.4)."""
import os

import numpy as np
import pytest

from oracle import compress
from oracle import moe_lrc_oracle as orc
from workload import configs, synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_quantizer_bounds(bits):
    cfg = configs.TINY
    W = synth.make_expert_weight(cfg, 0, 0)
    q = compress.quantize_groupwise(W, bits, 64)
    assert q["codes"].max() <= (1 << bits) - 1 and q["codes"].dtype == np.uint8
    D = compress.dequantize(q, 64)
    s = np.repeat(q["scale"].view(np.float16).astype(np.float64), 64, axis=0)
    inner = (q["codes"] > 0) & (q["codes"] < (1 << bits) - 1)           # not clipped
    assert (np.abs(W - D)[inner] <= 0.5 * s[inner] * (1 + 1e-9)).all()
    # clipped entries are off by at most one step more than fp16 rounding of (scale, zero) explains
    assert (np.abs(W - D) <= 1.01 * s).all()
    # codes are the best choice for the stored (scale, zero): no neighbour code is closer
    z = np.repeat(q["zero"].view(np.float16).astype(np.float64), 64, axis=0)
    for d in (-1, 1):
        alt = np.clip(q["codes"].astype(np.int64) + d, 0, (1 << bits) - 1)
        assert (np.abs(W - D) <= np.abs(W - (alt - z) * s) + 1e-12).all()


def test_quantizer_constant_and_two_level_groups():
    W = np.full((64, 3), 0.125, dtype=np.float32)
    W[:, 1] = -0.5
    W[:32, 2] = 1.0; W[32:, 2] = 3.0
    q = compress.quantize_groupwise(W, 2, 64)
    D = compress.dequantize(q, 64)
    np.testing.assert_array_equal(D[:, :2], W[:, :2].astype(np.float64))     # constant groups exact
    assert (q["codes"][:, :2] == 0).all()
    np.testing.assert_allclose(D[:, 2], W[:, 2], rtol=2e-3)                  # endpoints of the range
    assert set(q["codes"][:, 2]) == {0, 3}


def test_quantizer_uses_rounded_metadata():
    # the code must be chosen against the *stored* fp16 scale/zero: re-deriving codes from the
    # stored values reproduces them exactly
    W = synth.make_expert_weight(configs.TINY, 1, 2)
    q = compress.quantize_groupwise(W, 3, 64)
    s = np.repeat(q["scale"].view(np.float16).astype(np.float64), 64, axis=0)
    z = np.repeat(q["zero"].view(np.float16).astype(np.float64), 64, axis=0)
    np.testing.assert_array_equal(np.clip(np.rint(W / s + z), 0, 7).astype(np.uint8), q["codes"])


@pytest.mark.parametrize("shape", [(48, 80), (80, 48)])
def test_truncated_factors_eckart_young(shape):
    rng = np.random.default_rng(5)
    E = rng.normal(size=shape) * np.geomspace(1, 0.01, shape[1])[None, :]
    sig = np.linalg.svd(E, compute_uv=False)
    for r in (1, 4, 16, min(shape)):
        A, B, S = compress.residual_factors(E, r)
        np.testing.assert_allclose(S, sig[:r], rtol=1e-12)
        R = E - A @ B
        np.testing.assert_allclose((R * R).sum(), (sig[r:] ** 2).sum(), rtol=1e-9, atol=1e-20)
        if r < min(shape):
            np.testing.assert_allclose(np.linalg.norm(R, 2), sig[r], rtol=1e-9)
        # reparameterisation of Section 3.1: both factors carry sqrt(S)
        np.testing.assert_allclose(A.T @ A, np.diag(sig[:r]), atol=1e-10)
        np.testing.assert_allclose(B @ B.T, np.diag(sig[:r]), atol=1e-10)


def test_gram_and_randomized_factors():
    rng = np.random.default_rng(6)
    for shape in [(40, 120), (120, 40)]:
        E = rng.normal(size=shape) @ np.diag(np.geomspace(1, 1e-3, shape[1]))
        A, B, S = compress.residual_factors(E, 8, "exact")
        Ag, Bg, Sg = compress.residual_factors(E, 8, "gram")
        np.testing.assert_allclose(Sg, S, rtol=1e-9)
        np.testing.assert_allclose(Ag @ Bg, A @ B, atol=1e-9)
        Ar, Br, Sr = compress.residual_factors(E, 8, "randomized", seed=1, power_iters=3)
        # an approximation: within a few percent of the optimal rank-8 error
        opt = np.linalg.norm(E - A @ B)
        assert np.linalg.norm(E - Ar @ Br) <= 1.05 * opt


def test_error_decreases_with_rank():
    cfg = configs.TINY
    W = synth.make_expert_weight(cfg, 2, 0)
    prev = None
    for r in (0, 8, 32, 128, 256):
        art = compress.compress_matrix(W, 2, 64, r, keep_fp64_factors=True)
        D = compress.dequantize(art, 64)
        What = D + (art["A"] @ art["B"] if r else 0)
        err = np.linalg.norm(W - What) / np.linalg.norm(W)
        assert prev is None or err < prev
        prev = err
    assert prev < 1e-12      # r = min(K, N): exact restoration


def test_bf16_rounding_helper():
    import torch
    rng = np.random.default_rng(8)
    a = (rng.normal(size=4096) * np.exp(rng.normal(size=4096) * 5)).astype(np.float32)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(compress.round_to_bf16_bits(a), ref)
    np.testing.assert_array_equal(synth.f32_to_bf16_bits(a), ref)


def test_kurtosis_closed_forms():
    rng = np.random.default_rng(9)
    n = 2_000_000
    assert abs(compress.kurtosis(rng.normal(size=n)) - 3.0) < 0.02           # Gaussian
    assert abs(compress.kurtosis(rng.uniform(size=n)) - 1.8) < 0.01          # uniform
    assert abs(compress.kurtosis(rng.laplace(size=n)) - 6.0) < 0.15          # Laplace
    np.testing.assert_allclose(compress.kurtosis(np.array([-1.0, 1.0, -1.0, 1.0])), 1.0)  # two-point
    # shift and scale invariant
    w = rng.normal(size=1000)
    np.testing.assert_allclose(compress.kurtosis(5 - 3 * w), compress.kurtosis(w), rtol=1e-12)
    # outliers raise it: the workload's 0.1 % x10 entries
    assert compress.kurtosis(synth.make_expert_weight(configs.TINY, 0, 0)) > 10


def test_rank_allocation_greedy():
    k = np.array([3.0, 9.0, 4.0, 3.5, 8.0, 3.1, 3.2, 3.3])
    # literal greedy, N = 8, R_avg = 32: the highest-kurtosis matrix takes the whole 256 budget
    np.testing.assert_array_equal(compress.allocate_ranks(k, 32), [0, 256, 0, 0, 0, 0, 0, 0])
    r = compress.allocate_ranks(k, 100)           # budget 800: 512 + 256 + 32 + 0 ...
    np.testing.assert_array_equal(r, [0, 512, 32, 0, 256, 0, 0, 0])
    for r_avg in (0, 16, 40, 64, 1024, 5000):
        r = compress.allocate_ranks(k, r_avg)
        assert r.sum() <= len(k) * r_avg and set(r) <= set(compress.RANK_BUCKETS)
        order = np.argsort(-k, kind="stable")
        assert (np.diff(r[order]) <= 0).all()     # rank never increases as kurtosis decreases
    np.testing.assert_array_equal(compress.allocate_ranks(k, 1024), np.full(8, 1024))


def test_transfer_sizes_match_the_paper():
    H, F = 4096, 14336
    int2 = compress.expert_code_bytes(H, F, 2)
    assert int2 == 44_040_192
    for line in open(os.path.join(GOLDEN, "compensator_bytes.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        rank, mb, pct = line.split()
        b = compress.compensator_bytes(H, F, int(rank), factor_bits=3)
        assert abs(b / 2**20 - float(mb)) < 0.006, (rank, b)
        assert abs(100 * b / int2 - float(pct)) < 0.006, (rank, b)
    assert compress.compensator_bytes(H, F, 16, 3) == 331_776
    assert compress.compensator_bytes(H, F, 128, 3) == 2_654_208


def test_staged_bytes_only_selected_experts():
    counts = np.array([3, 0, 1, 0]); comp = np.array([2, 0, 0, 0])
    s = compress.staged_bytes(counts, comp, 256, 512, 3, 64, 8)
    assert s["active_experts"] == 2 and s["comp_experts"] == 1
    assert s["bytes_codes"] == 2 * 3 * 256 * 512 * 3 // 8
    assert s["bytes_meta"] == 2 * 3 * 256 * 512 // 64 * 4
    assert s["bytes_factors"] == 3 * 8 * (256 + 512) * 2


def test_shrink_operator_closed_forms():
    x = np.array([-3.0, -0.05, 0.0, 0.05, 0.2, 3.0])
    # p = 1: the ordinary soft threshold of width 1 / beta
    np.testing.assert_allclose(compress.shrink_lp(x, 10.0, 1.0), np.sign(x) * np.maximum(np.abs(x) - 0.1, 0.0), atol=1e-15)
    # p = 0.5, beta = 4 at x = 1: 1 - 1^(-0.5) / 4 = 0.75; at x = 0.25: 0.25 - 2 / 4 < 0 -> 0; odd; zero at zero
    got = compress.shrink_lp(np.array([1.0, 0.25, -1.0, 0.0]), 4.0, 0.5)
    np.testing.assert_allclose(got, [0.75, 0.0, -0.75, 0.0], atol=1e-15)
    # never grows a value, never flips its sign
    r = np.random.default_rng(0).standard_normal(1000)
    y = compress.shrink_lp(r, 10.0, 0.7)
    assert (np.abs(y) <= np.abs(r)).all() and (y * r >= 0).all()


def test_refined_quantizer_reduces_to_minmax_and_lowers_the_lp_error():
    rng = np.random.default_rng(4)
    W = rng.standard_normal((256, 48)) * 0.02
    W *= 1.0 + 9.0 * (rng.random(W.shape) < 0.01)          # outliers stretch the min/max grid
    W[:64, 0] = 0.5                                         # a constant group
    for bits in (2, 3, 4):
        base = compress.quantize_groupwise(W, bits, 64)
        same = compress.quantize_refined(W, bits, 64, iters=0)
        for k in ("codes", "scale", "zero"):
            np.testing.assert_array_equal(same[k], base[k])
        ref = compress.quantize_refined(W, bits, 64)
        np.testing.assert_array_equal(ref["scale"], base["scale"])            # the scale is kept
        assert ref["codes"].max() < (1 << bits)
        lp = lambda q: (np.abs(W - compress.dequantize(q, 64)) ** 0.7).sum()
        assert lp(ref) < lp(base)                                              # what the solver minimises
        # the stored codes are the nearest ones for the stored zero and scale
        s = np.repeat(orc.f16_to_f64(ref["scale"]), 64, axis=0)
        z = np.repeat(orc.f16_to_f64(ref["zero"]), 64, axis=0)
        want = np.clip(np.rint(W / s + z), 0, (1 << bits) - 1)
        want[:64, 0] = 0
        np.testing.assert_array_equal(ref["codes"], want.astype(np.uint8))
    # a group whose bulk sits on a grid shifted against min/max's: one outlier pins the min/max zero
    # point; the refinement moves the zero point to where the bulk is represented exactly
    g = np.concatenate([[0.0], 0.26 + 0.5 * rng.integers(0, 2, 63)])[:, None]      # outlier 0; bulk at 0.26, 0.76
    g[-1, 0] = 1.5                                                                   # max: scale = 0.5 at 2 bits
    base, ref = compress.quantize_groupwise(g, 2, 64), compress.quantize_refined(g, 2, 64)
    e0, e1 = np.abs(g - compress.dequantize(base, 64)), np.abs(g - compress.dequantize(ref, 64))
    assert np.median(e1) < 0.02 < np.median(e0)
