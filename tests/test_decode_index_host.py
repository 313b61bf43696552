"""Host-side model of the skinny (decode) FFN kernels' index arithmetic: the kernels and this check
share the same integer functions (csrc/decode_index.h).  Swept over shapes, bit widths, groups, a
rank per projection (0 .. 1024, Section 3.1), row counts, block shares and K-blocks, it asserts that
every buffer offset stays inside its resource, every LDS address inside its region, and that each
packed tile and each rank step is read exactly once.  No GPU needed."""
import itertools

import pytest

import paper_2512_17073_amd as amd


def _kblocks(ffn):
    ks = (ffn + 255) // 256
    return min(8, (ks + 15) // 16)


# (the last two: the longest K of either projection that a layer accepts: several staging phases per K-block)
@pytest.mark.parametrize("hidden,ffn", [(256, 512), (512, 768), (2048, 1408), (2048, 768), (4096, 14336), (256, 65536), (16384, 512)])
def test_index_model_over_ranks_and_shares(hidden, ffn):
    big = hidden >= 4096 or ffn >= 65536
    layer_ranks = (0, 8, 32, 40, 256, 1024) if not big else (32, 1024)
    for bits, group, layer_rank in itertools.product((2, 3, 4) if not big else (2, 3), (64, 128) if not big else (64,), layer_ranks):
        if hidden % group or ffn % group:
            continue
        rank_sets = {(layer_rank,) * 3, (0, layer_rank, layer_rank // 2 // 8 * 8), (layer_rank, 0, 0),
                     (min(layer_rank, 16), min(layer_rank, 128), layer_rank)}
        for ranks in sorted(rank_sets):
            for rows, first in ((1, 0), (16, 5), (17, 0), (33, 2)) if not big else ((19, 3),):
                nt13, nt2 = ffn // 16, hidden // 16
                per = 32                                       # n-tiles a block can own
                for g13, g2 in (((nt13 + per - 1) // per, (nt2 + per - 1) // per), (nt13, nt2), (max(2, nt13 // 5), max(2, nt2 // 3))):
                    amd.selftest_decode_index(hidden, ffn, bits, group, layer_rank, ranks, first, rows, first + rows + 7,
                                              g13, g2, _kblocks(ffn))


def test_index_model_rejects_a_share_that_is_too_large():
    # one block for 896 n-tiles: more than the 32 a block can take; the check must say so
    with pytest.raises(amd.MoeLrcError):
        amd.selftest_decode_index(4096, 14336, 2, 64, 32, (32, 32, 32), 0, 8, 8, 1, 8, 4)
