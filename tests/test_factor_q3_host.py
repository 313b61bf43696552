"""CPU check of the 3-bit factor format (Section 3.1 step 2 stores the factor pairs at INT3): the
library's host model of how the kernels read a packed pair (unit and metadata indices, field
extraction, one fp16 FMA per element) against the oracle's dequantized factors."""
import numpy as np
import pytest

import paper_2512_17073_amd as amd
from oracle import compress


def _pair(K, N, rank, seed, spread=1.0):
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((K, rank)) * 0.02 * spread
    B = rng.standard_normal((rank, N)) * 0.01 * spread
    # columns of very different size, as the singular values make them
    A *= np.geomspace(1.0, 0.05, rank)[None, :]
    B *= np.geomspace(1.0, 0.05, rank)[:, None]
    return compress.quantize_factors(A, B)


@pytest.mark.parametrize("K,N,rank", [(256, 512, 32), (512, 256, 16), (128, 192, 24), (256, 128, 72), (64, 64, 8)])
def test_packed_pair_reads_back_as_the_oracles_dequantized_factors(K, N, rank):
    Aq, Bq = _pair(K, N, rank, seed=K + N + rank)
    A, B = amd.selftest_factor_pair(Aq, Bq)
    A_ref = compress.dequantize(Aq, compress.FACTOR_GROUP)                 # [K][rank]
    B_ref = compress.dequantize(Bq, compress.FACTOR_GROUP).T               # [rank][N]
    # one fp16 rounding of the element and one of the group's offset zero * scale
    for got, ref, q in ((A, A_ref, Aq), (B, B_ref.T, Bq)):
        got = got if q is Aq else got.T
        s = np.repeat(q["scale"].view(np.float16).astype(np.float64), compress.FACTOR_GROUP, axis=0)
        z = np.repeat(q["zero"].view(np.float16).astype(np.float64), compress.FACTOR_GROUP, axis=0)
        tol = 2.0 ** -11 * (np.abs(ref) + np.abs(z * s)) + 1e-12
        assert (np.abs(got - ref) <= tol).all(), np.abs(got - ref).max()
    # and the error is not hiding a wrong code: distinct codes are a whole scale apart
    s_min = Aq["scale"].view(np.float16).astype(np.float64)
    assert np.abs(A - A_ref).max() < 0.01 * s_min[s_min > 0].min() * 8


def test_large_scales_are_folded_into_a_power_of_two():
    # scale * 2^17 would overflow fp16 for scales above 0.25: the packer folds a power of two out
    Aq, Bq = _pair(128, 128, 16, seed=3, spread=400.0)
    assert Aq["scale"].view(np.float16).astype(np.float64).max() > 0.5
    A, B = amd.selftest_factor_pair(Aq, Bq)
    A_ref = compress.dequantize(Aq, compress.FACTOR_GROUP)
    assert np.isfinite(A).all() and np.abs(A - A_ref).max() <= 2.0 ** -9 * np.abs(A_ref).max()


def test_out_of_range_codes_are_rejected():
    Aq, Bq = _pair(64, 64, 8, seed=4)
    bad = dict(Aq, codes=Aq["codes"].copy())
    bad["codes"][5, 3] = 8
    with pytest.raises(amd.MoeLrcError):
        amd.selftest_factor_pair(bad, Bq)
