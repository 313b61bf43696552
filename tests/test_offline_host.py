"""CPU pins of the offline pipeline's host-testable pieces: the quantizer's fp64 -> fp16 rounding
(the one place where floating point decides stored bits) against numpy's correctly rounded
conversion."""
import numpy as np

import paper_2512_17073_amd as amd


def test_f64_to_f16_rounding_matches_numpy():
    rng = np.random.default_rng(5)
    parts = [
        rng.standard_normal(200000) * 10.0 ** rng.integers(-9, 6, 200000),
        # every fp16 value, its neighbours' midpoints (ties) and points just beside the ties
        np.arange(0, 0x7c00, dtype=np.uint16).view(np.float16).astype(np.float64),
    ]
    h = parts[1]
    mid = (h[:-1] + h[1:]) / 2
    parts += [mid, np.nextafter(mid, np.inf), np.nextafter(mid, -np.inf), -mid,
              np.array([0.0, -0.0, 65504.0, 65519.999, 65520.0, 65536.0, 1e300, -1e300, np.inf, -np.inf,
                        2.0 ** -24, 2.0 ** -25, np.nextafter(2.0 ** -25, 1), 2.0 ** -26, 5e-324, 2.0 ** -14,
                        np.nextafter(2.0 ** -14, 0)])]
    a = np.concatenate(parts)
    with np.errstate(over="ignore"):
        want = a.astype(np.float16).view(np.uint16)
    got = amd.f64_to_f16_bits(a)
    bad = np.flatnonzero(got != want)
    assert bad.size == 0, (a[bad[:5]], got[bad[:5]], want[bad[:5]])
    assert amd.f64_to_f16_bits(np.array([np.nan]))[0] & 0x7c00 == 0x7c00


def test_rank_allocation_matches_the_oracle_and_the_literal_example():
    from oracle import compress
    # Section 3.1 step 1, taken literally: N = 8 matrices, R_avg = 32, the paper's bucket -> the matrix
    # with the largest kurtosis takes 256 = the whole budget, the others nothing
    kap = np.array([3.1, 9.0, 3.0, 4.5, 3.3, 2.9, 5.0, 3.2])
    got = amd.allocate_ranks(kap, 32)
    assert got.tolist() == [0, 256, 0, 0, 0, 0, 0, 0]
    assert got.tolist() == compress.allocate_ranks(kap, 32).tolist()
    rng = np.random.default_rng(0)
    for n, r_avg, buckets in ((24, 32, compress.RANK_BUCKETS), (24, 100, compress.RANK_BUCKETS), (7, 16, (0, 8, 16, 32)),
                              (192, 40, compress.RANK_BUCKETS), (5, 0, compress.RANK_BUCKETS)):
        kap = rng.gamma(2.0, 2.0, n) + 1.8
        kap[rng.integers(0, n, 3)] = kap[0]                  # ties: index order
        want = compress.allocate_ranks(kap, r_avg, buckets)
        got = amd.allocate_ranks(kap, r_avg, buckets)
        assert got.tolist() == want.tolist()
        assert got.sum() <= n * r_avg and set(got.tolist()) <= set(buckets)
