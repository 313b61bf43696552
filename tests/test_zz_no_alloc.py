"""GPU test of moe_lrc_forward_noalloc, the entry point that allocates nothing: its workspace is a
fixed device array inside the library.  Called through the C ABI on two batches in a row, the second
smaller than the first (whatever the first left in the array must not matter); each output is
compared with moe_lrc_forward on a caller workspace, bit for bit (same kernels, same bar as the
other parity tests: the reference side is itself within 5e-3 of the oracle), and with the oracle.
"""
import numpy as np
import pytest

from oracle import fixtures
from oracle import moe_lrc_oracle as orc
from workload import configs, synth

pytestmark = pytest.mark.gpu
TOL = 5e-3


def test_forward_noalloc_matches_forward_twice_in_a_row():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    import paper_2512_17073_amd as amd
    amd.lib()
    cfg = configs.TINY.with_(tokens=40, name="noalloc")
    layer = fixtures.build_layer(cfg)
    L = amd.Layer.from_config(cfg)
    L.load(layer)
    for T in (40, 7):                                        # the second call is the smaller one
        x_bits = synth.make_tokens(cfg.with_(seed=cfg.seed + T), T)
        x = amd.bf16_tensor(x_bits)
        want = L.forward(x).clone()
        out = torch.full((T, cfg.hidden), float("nan"), dtype=torch.bfloat16, device="cuda")
        L.forward_noalloc(x, out)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want.view(torch.int16)), f"T={T}: differs from moe_lrc_forward"
        ref = fixtures.oracle_forward(cfg, layer, x_bits)
        err = orc.rel_frobenius(out.float().cpu().numpy().astype(np.float64), ref["out"])
        assert err <= TOL, f"T={T}: {err:.2e}"
    # a batch whose workspace exceeds the built-in array is refused before any device work
    big = amd.Layer(hidden=4096, ffn=14336, n_experts=8, top_k=2, top_n=1, bits=2, group=64, rank=32,
                    max_tokens=4096)
    assert big.workspace_bytes(4096) > (32 << 20)
    xb = torch.zeros((4096, 4096), dtype=torch.bfloat16, device="cuda")
    ob = torch.empty_like(xb)
    with pytest.raises(amd.MoeLrcError) as ei:
        big.forward_noalloc(xb, ob)
    assert ei.value.code == -4
    big.close()
    L.close()
