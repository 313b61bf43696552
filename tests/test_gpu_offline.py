"""GPU tests of the offline pipeline (moe_lrc_offline_*) against oracle/compress.py.

Quantizer: codes, scales, zeros and the residual bit for bit (both sides work in fp64 and round the
scale and zero to fp16 before choosing codes).  Factors: what is unique about them — the singular
values, the product A B, the factors up to the sign of each pair — against the oracle's subspace
iteration on the same test matrix, and the approximation error against the exact SVD's optimum
(Eckart-Young).  Kurtosis to 1e-12.  End to end: a layer compressed on the device, loaded through the
C ABI and run, against the forward oracle on the same artefacts.
"""
import numpy as np
import pytest

from oracle import compress, fixtures
from oracle import moe_lrc_oracle as orc
from workload import configs, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def amd():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2512_17073_amd as amd
    amd.lib()
    return amd


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _bits(t):
    return t.cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("bits,group,K,N", [(2, 64, 512, 384), (3, 64, 256, 528), (4, 128, 512, 272), (3, 256, 768, 100)])
def test_quantizer_bit_exact(amd, bits, group, K, N):
    rng = np.random.default_rng(bits * 1000 + group)
    W = rng.standard_normal((K, N)) * 0.02
    W *= 1.0 + 4.0 * (rng.random((K, N)) < 0.01)            # heavy tails
    W[:group, 0] = 0.0                                      # a group of zeros
    W[:group, 1] = 0.3125                                   # a constant group
    W[group:2 * group, 2] *= 1e-9                           # a scale that rounds to zero in fp16
    W[:group, 3] *= 1e7                                     # a scale beyond fp16
    W[:group, 4] = np.linspace(-1.0, 1.0, group)            # exact ties between codes
    want = compress.quantize_groupwise(W, bits, group)
    codes, scale, zero, resid = amd.offline_quantize(_dev(W), bits, group)
    np.testing.assert_array_equal(codes.cpu().numpy(), want["codes"])
    np.testing.assert_array_equal(_bits(scale), want["scale"])
    np.testing.assert_array_equal(_bits(zero), want["zero"])
    E = W - compress.dequantize(want, group)
    np.testing.assert_array_equal(resid.cpu().numpy(), E)
    # what the quantizer promises: no code of a regular group is more than half a step off
    s = np.repeat(orc.f16_to_f64(want["scale"]), group, axis=0)
    regular = np.repeat(np.ptp(W.reshape(K // group, group, N), axis=1) < 6e4, group, axis=0)
    assert (np.abs(E)[regular] <= 0.5 * s[regular] * (1 + 2e-3) + 1e-12).all()


@pytest.mark.parametrize("bits,group", [(2, 64), (3, 64), (4, 128)])
def test_refined_quantizer_against_the_oracle(amd, bits, group):
    rng = np.random.default_rng(40 + bits)
    K, N = 512, 320
    W = rng.standard_normal((K, N)) * 0.02
    W *= 1.0 + 9.0 * (rng.random((K, N)) < 0.01)
    W[:group, 0] = 0.25                                     # a constant group
    want = compress.quantize_refined(W, bits, group)
    codes, scale, zero, resid = amd.offline_quantize(_dev(W), bits, group, refine={})
    codes, scale, zero = codes.cpu().numpy(), _bits(scale), _bits(zero)
    np.testing.assert_array_equal(scale, want["scale"])
    # The zero point comes out of twenty steps that call pow(); the two libraries' pow may differ in
    # the last bit, which can move a zero point that sits on a rounding boundary: allow one group in
    # ten thousand to differ by one fp16 step (and its codes by one), nothing else.
    dz = zero.astype(np.int64) - want["zero"].astype(np.int64)
    assert (np.abs(dz) <= 1).all() and (dz != 0).mean() <= 1e-4
    dc = codes.astype(np.int64) - want["codes"].astype(np.int64)
    assert (np.abs(dc) <= 1).all() and (dc != 0).mean() <= 1e-4
    got = {"codes": codes, "scale": scale, "zero": zero}
    lp = lambda q: (np.abs(W - compress.dequantize(q, group)) ** 0.7).sum()
    assert abs(lp(got) - lp(want)) <= 1e-6 * lp(want)
    assert lp(got) < lp(compress.quantize_groupwise(W, bits, group))
    np.testing.assert_array_equal(resid.cpu().numpy(), W - compress.dequantize(got, group))
    # no steps: the plain quantizer, bit for bit
    c0, s0, z0, _ = amd.offline_quantize(_dev(W), bits, group, refine={"iters": 0})
    base = compress.quantize_groupwise(W, bits, group)
    np.testing.assert_array_equal(c0.cpu().numpy(), base["codes"])
    np.testing.assert_array_equal(_bits(z0), base["zero"])


def test_kurtosis(amd):
    rng = np.random.default_rng(3)
    for W in (rng.standard_normal((700, 513)), rng.laplace(size=(300, 1001)) * 0.05 + 0.01, rng.random((257, 129))):
        want = compress.kurtosis(W)
        got = amd.offline_kurtosis(_dev(W))
        assert abs(got - want) <= 1e-12 * want, (got, want)


def _aligned(A, B, A0, B0):
    sign = np.sign(np.sum(A * A0, axis=0))
    return A * sign[None, :], B * sign[:, None]


@pytest.mark.parametrize("K,N,r,bits", [(256, 512, 8, 3), (512, 768, 40, 2), (1024, 640, 16, 2), (384, 384, 128, 4)])
def test_residual_factors(amd, K, N, r, bits):
    rng = np.random.default_rng(K + N + r)
    W = rng.standard_normal((K, N)) * 0.02
    W *= 1.0 + 4.0 * (rng.random((K, N)) < 0.01)
    q = compress.quantize_groupwise(W, bits, 64)
    E = W - compress.dequantize(q, 64)
    seed, l = 11, r + 8
    omega = np.random.default_rng(seed).standard_normal((N, l))    # what the oracle's "randomized" method draws
    A0, B0, S0 = compress.residual_factors(E, r, method="randomized", seed=seed, power_iters=2)
    A, B, sigma, Ab, Bb = amd.offline_factors(_dev(E), r, _dev(omega), power_iters=2)
    A, B = A.cpu().numpy(), B.cpu().numpy()
    np.testing.assert_allclose(sigma, S0, rtol=1e-9)
    assert (np.diff(sigma) <= 0).all()
    assert orc.rel_frobenius(A @ B, A0 @ B0) <= 1e-8
    # Section 3.1 step 2's reparameterisation: A^T A = B B^T = diag(sigma)
    np.testing.assert_allclose(A.T @ A, np.diag(sigma), atol=1e-9 * sigma[0])
    np.testing.assert_allclose(B @ B.T, np.diag(sigma), atol=1e-9 * sigma[0])
    # the factors themselves, up to the sign of each pair (the singular values of a quantizer's
    # residual are close together, so single vectors are less well determined than the product)
    As, Bs = _aligned(A, B, A0, B0)
    assert orc.rel_frobenius(As, A0) <= 1e-5 and orc.rel_frobenius(Bs, B0) <= 1e-5
    # against the exact SVD: never better than the optimum, and as close to it as the oracle's iteration
    Sx = np.linalg.svd(E, compute_uv=False)
    best = np.sqrt((Sx[r:] ** 2).sum())
    err, err0 = np.linalg.norm(E - A @ B), np.linalg.norm(E - A0 @ B0)
    assert best * (1 - 1e-12) <= err <= err0 * (1 + 1e-9) and err <= best * 1.05
    # stored form: the same rounding to bf16 as the oracle's
    np.testing.assert_array_equal(_bits(Ab), compress.round_to_bf16_bits(A))
    np.testing.assert_array_equal(_bits(Bb), compress.round_to_bf16_bits(B))


def test_low_rank_matrix_is_recovered(amd):
    # E of exact rank 6 plus nothing: the factors of rank 6 reproduce it (l = rank: no room to spare)
    rng = np.random.default_rng(8)
    E = rng.standard_normal((300, 6)) @ rng.standard_normal((6, 200))
    omega = rng.standard_normal((200, 6))
    A, B, sigma, _, _ = amd.offline_factors(_dev(E), 6, _dev(omega), power_iters=1)
    np.testing.assert_allclose(sigma, np.linalg.svd(E, compute_uv=False)[:6], rtol=1e-10)
    assert orc.rel_frobenius(A.cpu().numpy() @ B.cpu().numpy(), E) <= 1e-12
    # a sketch wider than the matrix's rank cannot be orthonormalised: reported, not computed
    with pytest.raises(amd.MoeLrcError) as ei:
        amd.offline_factors(_dev(E), 6, _dev(rng.standard_normal((200, 14))), power_iters=1)
    assert ei.value.code == -2


def test_layer_compressed_on_the_device_runs_through_the_hot_path(amd):
    cfg = configs.TINY.with_(tokens=40, name="offline_e2e")
    wg, bias = synth.make_gate(cfg)
    experts = []
    for e in range(cfg.n_experts):
        ex = {}
        for mat in (0, 1, 2):
            W = np.asarray(synth.make_expert_weight(cfg, e, mat), dtype=np.float64)
            codes, scale, zero, resid = amd.offline_quantize(_dev(W), cfg.bits, cfg.group)
            omega = np.random.default_rng(100 * e + mat).standard_normal((W.shape[1], cfg.rank + 8))
            A, B, sigma, Ab, Bb = amd.offline_factors(resid, cfg.rank, _dev(omega), power_iters=2)
            ex[mat] = {"codes": codes.cpu().numpy(), "scale": _bits(scale), "zero": _bits(zero), "A": _bits(Ab), "B": _bits(Bb)}
            # the compensated weights are closer to W than the quantized ones, by what Eckart-Young allows
            D = compress.dequantize(ex[mat], cfg.group)
            Sx = np.linalg.svd(W - D, compute_uv=False)
            gain = np.linalg.norm(W - D - A.cpu().numpy() @ B.cpu().numpy()) / np.linalg.norm(W - D)
            assert gain <= np.sqrt((Sx[cfg.rank:] ** 2).sum() / (Sx ** 2).sum()) * 1.05
        experts.append(ex)
    layer = {"wg": wg, "bias": bias, "experts": experts}
    L = amd.Layer.from_config(cfg)
    L.load(layer)
    x_bits = synth.make_tokens(cfg)
    ref = fixtures.oracle_forward(cfg, layer, x_bits)
    out = L.forward(amd.bf16_tensor(x_bits)).float().cpu().numpy().astype(np.float64)
    assert orc.rel_frobenius(out, ref["out"]) <= 5e-3
    L.close()
