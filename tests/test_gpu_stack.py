"""GPU tests of the layer stack (moe_lrc_stack_*): decoding through several MoE layers whose experts
live in host memory and share one device slot pool (Section 4.3, case study 1).

Arithmetic: every layer's output against the single-layer oracle applied to that layer's own input
(read back from the device, so that a near-tie in a later layer's routing cannot mask or fake an
error), to the same 5e-3 bar as the single layer; bit-equal to a chain of device-resident layers.
Transfers: the library's counters against the slot-cache model of oracle/stack_model.py driven by
the oracle's routing (exact: routing indices are bit-exact).
"""
import numpy as np
import pytest

from oracle import compress, fixtures
from oracle import moe_lrc_oracle as orc
from oracle.stack_model import SlotCache
from workload import configs, synth

pytestmark = pytest.mark.gpu
TOL = 5e-3
N_LAYERS = 3


@pytest.fixture(scope="module")
def amd():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2512_17073_amd as amd
    amd.lib()
    return amd


@pytest.fixture(scope="module")
def stack_layers():
    # three layers with weights of their own; the middle one has a shared expert (always on, never staged)
    cfgs = [configs.TINY.with_(seed=1234 + 100 * l, tokens=5, name=f"stack{l}",
                               n_shared=1 if l == 1 else 0, shared_bits=4) for l in range(N_LAYERS)]
    return cfgs, [fixtures.build_layer(c) for c in cfgs]


def _bits(t):
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def _make(amd, cfgs, layers, residency):
    Ls = [amd.Layer.from_config(c, max_tokens=16, residency=residency) for c in cfgs]
    for L, layer in zip(Ls, layers):
        L.load(layer)
    return Ls


@pytest.mark.parametrize("residual,prefetch,slots", [(True, True, 8), (False, True, 9), (True, False, 8), (False, False, 24)])
def test_stack_against_oracle_and_cache_model(amd, stack_layers, residual, prefetch, slots):
    import torch
    cfgs, layers = stack_layers
    Ls = _make(amd, cfgs, layers, amd.POOLED)
    st = amd.Stack(Ls, slots=slots, prefetch=prefetch, residual=residual)
    model = SlotCache(slots)
    H = cfgs[0].hidden
    for step, T in enumerate((5, 3, 5, 1)):                     # decode steps with batches of their own
        x_bits = synth.make_tokens(cfgs[0].with_(seed=500 + step), T)
        x = amd.bf16_tensor(x_bits)
        li = torch.empty((N_LAYERS, T, H), dtype=torch.bfloat16, device="cuda")
        out = st.step(x, layer_inputs=li)
        torch.cuda.synchronize()
        assert np.array_equal(_bits(li[0]), x_bits)
        for l, (cfg, layer) in enumerate(zip(cfgs, layers)):
            xl_bits = _bits(li[l])
            nxt = li[l + 1] if l + 1 < N_LAYERS else out
            ref = fixtures.oracle_forward(cfg, layer, xl_bits)
            want = ref["out"] + (orc.bf16_to_f64(xl_bits) if residual else 0.0)
            err = orc.rel_frobenius(_f64(nxt), want)
            assert err <= TOL, f"step {step} layer {l}: {err:.2e}"
            if residual:      # the layer's own contribution, beside the (larger) residual: looser by the sum's bf16 rounding
                got_delta = _f64(nxt) - orc.bf16_to_f64(xl_bits)
                scale = np.linalg.norm(want) / max(np.linalg.norm(ref["out"]), 1e-30)
                assert orc.rel_frobenius(got_delta, ref["out"]) <= TOL + 2.0 ** -8 * scale, f"step {step} layer {l}"
            # the cache model, driven by the oracle's routing of the same inputs
            fu = cfg.rank > 0 and cfg.top_n > 0
            model.layer(l, ref["perm"]["counts"], ref["perm"]["comp_counts"], fu)
            if prefetch and l + 1 < N_LAYERS:
                nc = cfgs[l + 1]
                g = orc.route(xl_bits, layers[l + 1]["wg"], nc.top_k, nc.renormalize, layers[l + 1]["bias"])
                model.prefetch(l + 1, g["idx"], nc.n_experts, nc.top_n, nc.rank > 0 and nc.top_n > 0)
        s = st.stats()
        for k in ("expert_uses", "hits", "misses", "prefetched", "prefetch_hits", "factor_copies"):
            assert s[k] == model.c[k], (step, k, s, model.c)
        assert s["steps"] == step + 1
    # bytes: every copy moves at least the expert's packed codes, scales and zeros / its factor pair
    c0 = cfgs[0]
    w_alg = compress.expert_code_bytes(c0.hidden, c0.ffn, c0.bits) + compress.expert_meta_bytes(c0.hidden, c0.ffn, c0.group)
    f_alg = compress.compensator_bytes(c0.hidden, c0.ffn, c0.rank, 16)
    wc, fc = model.c["weight_copies"], model.c["factor_copies"]
    assert wc * w_alg + fc * f_alg <= s["bytes_h2d"] <= wc * w_alg * 1.05 + fc * f_alg * 4.5
    assert s["last_step_ms"] > 0
    if slots >= N_LAYERS * c0.n_experts:
        assert s["misses"] + s["prefetched"] <= N_LAYERS * c0.n_experts       # nothing is copied twice
    st.close()
    for L in Ls:
        L.close()


def test_stack_is_bit_equal_to_resident_layers_and_reuses_slots(amd, stack_layers):
    import torch
    cfgs, layers = stack_layers
    Lp = _make(amd, cfgs, layers, amd.POOLED)
    Lr = _make(amd, cfgs, layers, amd.RESIDENT)
    st = amd.Stack(Lp, slots=N_LAYERS * cfgs[0].n_experts, prefetch=False, residual=False)
    x = amd.bf16_tensor(synth.make_tokens(cfgs[0].with_(seed=77), 6))
    want = x
    for L in Lr:
        want = L.forward(want).clone()
    got = st.step(x).clone()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    cold = st.stats()
    assert cold["hits"] == 0 and cold["misses"] == cold["expert_uses"] > 0 and cold["bytes_h2d"] > 0
    # the same batch again: every expert is found in its slot, nothing crosses the bus, same bits
    got2 = st.step(x).clone()
    warm = st.stats()
    assert torch.equal(got2.view(torch.int16), want.view(torch.int16))
    assert warm["misses"] == cold["misses"] and warm["bytes_h2d"] == cold["bytes_h2d"]
    assert warm["hits"] == cold["expert_uses"] and warm["last_copy_ms"] == 0.0
    # after a reset the pool is cold again
    st.reset()
    got3 = st.step(x).clone()
    assert torch.equal(got3.view(torch.int16), want.view(torch.int16))
    assert st.stats()["misses"] == cold["misses"]
    # an eviction-heavy pool (one layer's worth of slots) still gives the same bits
    st.close()
    st2 = amd.Stack(Lp, slots=cfgs[0].n_experts, prefetch=True, residual=False)
    for _ in range(2):
        assert torch.equal(st2.step(x).view(torch.int16), want.view(torch.int16))
    st2.close()
    for L in Lp + Lr:
        L.close()


def test_stack_with_factor_pairs_held_at_3_bits(amd):
    """Pooled layers whose factor pairs are stored at INT3 (Section 3.1 step 2): the pairs cross the
    bus and sit in the slots at 3 bits and are dequantized inside the kernels; the stack gives the
    bits of the resident layers, matches the oracle on the quantized factors, and moves fewer factor
    bytes than with fp16 pairs."""
    import torch
    cfgs = [configs.TINY.with_(seed=4321 + 100 * l, tokens=6, rank=32, bits=2, name=f"stackq{l}") for l in range(2)]
    layers = [fixtures.build_layer(c, int3_factors=True) for c in cfgs]
    Lp = _make(amd, cfgs, layers, amd.POOLED)
    Lr = _make(amd, cfgs, layers, amd.RESIDENT)
    st = amd.Stack(Lp, slots=2 * cfgs[0].n_experts, prefetch=False, residual=False)
    x_bits = synth.make_tokens(cfgs[0].with_(seed=78), 6)
    x = amd.bf16_tensor(x_bits)
    H = cfgs[0].hidden
    li = torch.empty((2, 6, H), dtype=torch.bfloat16, device="cuda")
    got = st.step(x, layer_inputs=li).clone()
    want = x
    for L in Lr:
        want = L.forward(want).clone()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    ref = fixtures.oracle_forward(cfgs[1], layers[1], _bits(li[1]))
    assert orc.rel_frobenius(_f64(got), ref["out"]) <= TOL
    s = st.stats()
    c0 = cfgs[0]
    w_alg = compress.expert_code_bytes(c0.hidden, c0.ffn, c0.bits) + compress.expert_meta_bytes(c0.hidden, c0.ffn, c0.group)
    vals = 3 * c0.rank * (c0.hidden + c0.ffn)
    f_q3 = vals * 4 // 8 + vals // 64 * 4                     # a 4-bit cell per code, fp16 scale and zero per 64
    assert s["factor_copies"] > 0
    assert s["bytes_h2d"] <= s["misses"] * w_alg * 1.05 + s["factor_copies"] * f_q3 * 1.05
    st.close()
    for L in Lp + Lr:
        L.close()


def test_stack_argument_errors(amd, stack_layers):
    cfgs, layers = stack_layers
    Lp = _make(amd, cfgs[:1], layers[:1], amd.POOLED)
    Lr = _make(amd, cfgs[:1], layers[:1], amd.RESIDENT)
    x = amd.bf16_tensor(synth.make_tokens(cfgs[0], 4))
    with pytest.raises(amd.MoeLrcError) as ei:
        Lp[0].forward(x)                                   # a pooled layer has no slots of its own
    assert ei.value.code == -3
    with pytest.raises(amd.MoeLrcError) as ei:
        amd.Stack(Lr, slots=8)                             # not a pooled layer
    assert ei.value.code == -1
    with pytest.raises(amd.MoeLrcError) as ei:
        amd.Stack(Lp, slots=7)                             # fewer slots than one layer can need
    assert ei.value.code == -1
    st = amd.Stack(Lp, slots=8)
    with pytest.raises(amd.MoeLrcError) as ei:
        amd.Stack(Lp, slots=8)                             # the layer already belongs to a stack
    assert ei.value.code == -3
    import torch
    big = torch.zeros((17, cfgs[0].hidden), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(amd.MoeLrcError) as ei:
        st.step(big)
    assert ei.value.code == -3
    st.close()
    for L in Lp + Lr:
        L.close()
