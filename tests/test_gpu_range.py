"""GPU tests of the activation range.  Activations cross the boundary as bf16 (8 exponent bits),
the matrix cores take fp16 (5): the library scales every input row by a power of two into fp16's
range, undoes it on the fp32 results and carries the square of the scale through the SwiGLU output.
Here the same layer is run on inputs scaled by 2^8, 2^-12 (and much further out), on tokens of mixed
magnitudes, and with weights scaled up until the SwiGLU output h reaches the top of the fp16 range;
every output is compared with the fp64 oracle on the same bits, to the 5e-3 bar.
"""
import copy

import numpy as np
import pytest

from oracle import fixtures
from oracle import moe_lrc_oracle as orc
from workload import configs, synth

pytestmark = pytest.mark.gpu
TOL = 5e-3


@pytest.fixture(scope="module")
def amd():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2512_17073_amd as amd
    amd.lib()
    return amd


def _scale_bf16(bits: np.ndarray, k) -> np.ndarray:
    """bf16 bit patterns times 2^k (k an int or one per row): exponent field arithmetic, zeros kept."""
    b = bits.astype(np.int64)
    k = np.broadcast_to(np.asarray(k, dtype=np.int64).reshape(-1, 1) if np.ndim(k) else np.int64(k), b.shape)
    e = (b >> 7) & 0xFF
    out = np.where(e == 0, b, b + (k << 7))
    assert (((out >> 7) & 0xFF)[e != 0] > 0).all() and (((out >> 7) & 0xFF) < 255).all()
    return out.astype(np.uint16)


def _scale_f16(bits: np.ndarray, k: int) -> np.ndarray:
    b = bits.astype(np.int64)
    e = (b >> 10) & 0x1F
    out = np.where(e == 0, b, b + (k << 10))
    assert (((out >> 10) & 0x1F)[e != 0] > 0).all() and (((out >> 10) & 0x1F) < 31).all()
    return out.astype(np.uint16)


def _run(amd, cfg, layer, L, x_bits):
    ref = fixtures.oracle_forward(cfg, layer, x_bits)
    out = L.forward(amd.bf16_tensor(x_bits)).float().cpu().numpy().astype(np.float64)
    assert np.isfinite(out).all()
    return orc.rel_frobenius(out, ref["out"]), ref


@pytest.mark.parametrize("name,cfg", [
    ("decode", configs.TINY.with_(tokens=24, name="range_decode")),            # skinny kernels
    ("many_rows", configs.TINY.with_(tokens=300, bits=2, name="range_rows")),   # grouped GEMM
    ("shared", configs.DEEPSEEK.with_(hidden=512, n_experts=16, tokens=40, name="range_shared")),
])
def test_inputs_scaled_by_powers_of_two(amd, name, cfg):
    layer = fixtures.build_layer(cfg)
    L = amd.Layer.from_config(cfg)
    L.load(layer)
    x_bits = synth.make_tokens(cfg)
    base, _ = _run(amd, cfg, layer, L, x_bits)
    assert base <= TOL
    for k in (8, -12, 30, -40):
        err, ref = _run(amd, cfg, layer, L, _scale_bf16(x_bits, k))
        assert (ref["route"]["margin"] > 0).all()
        print(f"[{cfg.name}] x * 2^{k}: {err:.2e} (unscaled {base:.2e})")
        assert err <= TOL, f"x * 2^{k}: {err:.2e}"
    # tokens of very different magnitudes in one batch: every row has a scale of its own
    ks = np.array([(-1) ** t * (3 * t % 37) for t in range(cfg.tokens)])
    err, _ = _run(amd, cfg, layer, L, _scale_bf16(x_bits, ks))
    print(f"[{cfg.name}] mixed row scales: {err:.2e}")
    assert err <= TOL
    # a token of zeros among the others
    xz = x_bits.copy()
    xz[1] = 0
    err, _ = _run(amd, cfg, layer, L, xz)
    assert err <= TOL
    L.close()


def test_swiglu_output_near_the_top_of_fp16(amd):
    cfg = configs.TINY.with_(tokens=24, name="range_h")
    layer = fixtures.build_layer(cfg)
    x_bits = synth.make_tokens(cfg)
    x = orc.bf16_to_f64(x_bits)

    # rows are scaled so that max |x| lands in [1, 2); h is carried times the square of that scale
    row_scale = 2.0 ** -np.floor(np.log2(np.abs(x).max(axis=1)))

    def max_h(lay):
        m = 0.0
        for ex in lay["experts"][:cfg.n_experts]:
            g = x @ orc.dequant(ex[0]["codes"], ex[0]["scale"], ex[0]["zero"], cfg.group)
            u = x @ orc.dequant(ex[1]["codes"], ex[1]["scale"], ex[1]["zero"], cfg.group)
            m = max(m, (np.abs(orc.silu(g) * u) * row_scale[:, None] ** 2).max())
        return m

    # scale W1 and W3 (the codes' scales and the B factors) by 2^k until the largest stored |h| is
    # within a factor of four below fp16's largest finite value
    k, m0 = 0, max_h(layer)
    while m0 * 4.0 ** k < 2.0 ** 13.5:
        k += 1
    big = copy.deepcopy(layer)
    for ex in big["experts"][:cfg.n_experts]:
        for mat in (0, 1):
            ex[mat]["scale"] = _scale_f16(ex[mat]["scale"], k)
            ex[mat]["B"] = _scale_bf16(ex[mat]["B"], k)
    top = max_h(big)
    assert 2.0 ** 13.5 <= top < 2.0 ** 15.6, top
    L = amd.Layer.from_config(cfg)
    L.load(big)
    err, _ = _run(amd, cfg, big, L, x_bits)
    print(f"[range_h] W1, W3 * 2^{k}: max |h| {top:.3g}, error {err:.2e}")
    assert err <= TOL
    L.close()
