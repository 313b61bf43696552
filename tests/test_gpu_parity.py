"""GPU parity: the HIP library against the fp64 CPU oracle, element by element, through the C ABI.

Bars (written here, from the benchmark spec): routing indices, counts, permutation and unpacked
codes bit-exact; layer outputs within 5e-3 relative Frobenius error.
"""
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
    amd.lib()          # raises if the HIP library is not built: no fallback
    return amd


def _to_np(t):
    import torch
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy().astype(np.float64)
    return t.cpu().numpy()


def _build(amd, cfg, method="exact", residency=0, **kw):
    layer = fixtures.build_layer(cfg, method=method, **kw)
    L = amd.Layer.from_config(cfg, residency=residency)
    L.load(layer)
    return layer, L


SMALL = {
    "tiny": configs.TINY,
    "tiny_b2": configs.TINY.with_(bits=2, name="tiny_b2"),
    "tiny_b4_n2": configs.TINY.with_(bits=4, top_n=2, rank=16, name="tiny_b4_n2"),
    # > 32 rows per expert: exercises two row tiles and the row-chunk loop, ragged tails
    "tiny_T200": configs.TINY.with_(tokens=200, name="tiny_T200"),
    # several 128-row chunks per expert with a ragged last one; a rank that is no multiple of 16 or 32
    # (padding columns of the factors) at 4 bit
    "tiny_T700_r40": configs.TINY.with_(tokens=700, rank=40, bits=4, name="tiny_T700_r40"),
    # heavily skewed routing at decode size: some experts get more than 32 rows (several passes of
    # the decode kernel), others none
    "tiny_skew": configs.TINY.with_(tokens=44, gate_kind="unit", gate_std=1.0, zipf_s=3.0, name="tiny_skew"),
    # the largest quantization group (one scale/zero per 256 inputs = one per k-step of a lane row)
    "tiny_g256": configs.TINY.with_(group=256, bits=2, tokens=20, name="tiny_g256"),
    # a single expert: every token routes to it with weight 1, k = n = 1
    "tiny_e1": configs.TINY.with_(n_experts=1, top_k=1, top_n=1, tokens=40, name="tiny_e1"),
    "tiny_T1": configs.TINY.with_(tokens=1, name="tiny_T1"),
    # the limits of the configuration: 256 experts, k = 16 (n = 15), some experts without rows
    "tiny_e256_k16": configs.TINY.with_(n_experts=256, top_k=16, top_n=15, tokens=40, ffn=256, rank=8, name="tiny_e256_k16"),
    "tiny_renorm": configs.TINY.with_(renormalize=1, tokens=33, name="tiny_renorm"),
    # DeepSeek-shaped: shared experts at 4 bit, FFN 1408 (not a multiple of the 256-row k-step), k=6
    "deepseek_small": configs.DEEPSEEK.with_(hidden=512, n_experts=16, tokens=70, name="deepseek_small"),
    # Qwen3-shaped: group 128, many experts, k=8, Zipf-skewed routing
    "qwen3_small": configs.QWEN3.with_(hidden=512, ffn=768, tokens=48, name="qwen3_small"),
}


@pytest.fixture(scope="module", params=list(SMALL))
def case(request, amd):
    cfg = SMALL[request.param]
    print(f"\n[case {cfg.name}] building fixture", flush=True)
    layer, L = _build(amd, cfg)
    x_bits = synth.make_tokens(cfg)
    ref = fixtures.oracle_forward(cfg, layer, x_bits)
    assert (ref["route"]["margin"] > 1e-9).all(), "fixture has a near-tie; routing would be undecidable"
    x = amd.bf16_tensor(x_bits)
    yield cfg, layer, L, x_bits, x, ref
    L.close()


def test_unpacked_codes_bit_exact(case, amd):
    cfg, layer, L, *_ = case
    for e in range(cfg.n_experts + cfg.n_shared):
        for mat in (0, 1, 2):
            got = _to_np(L.debug_unpack(e, mat))
            np.testing.assert_array_equal(got, layer["experts"][e][mat]["codes"], err_msg=f"expert {e} mat {mat}")


def test_route_bit_exact(case):
    cfg, layer, L, x_bits, x, ref = case
    idx, w = L.route(x)
    np.testing.assert_array_equal(_to_np(idx), ref["route"]["idx"])
    np.testing.assert_allclose(_to_np(w), ref["route"]["w"], rtol=2e-6, atol=1e-30)


def test_permute_bit_exact(case):
    cfg, layer, L, x_bits, x, ref = case
    idx, _ = L.route(x)
    counts, offsets, row_pair, pair_row, comp = L.permute(idx)
    p = ref["perm"]
    np.testing.assert_array_equal(_to_np(counts), p["counts"])
    np.testing.assert_array_equal(_to_np(offsets), p["offsets"])
    np.testing.assert_array_equal(_to_np(row_pair), p["row_pair"])
    np.testing.assert_array_equal(_to_np(pair_row), p["pair_row"])
    np.testing.assert_array_equal(_to_np(comp), p["comp_counts"])


@pytest.mark.parametrize("experts,top_k,top_n,tokens", [(8, 2, 1, 4097), (8, 2, 1, 20000), (128, 8, 2, 1025), (128, 8, 3, 7777),
                                                         (61, 6, 2, 3000)])
def test_permute_by_several_blocks(amd, experts, top_k, top_n, tokens):
    """Above 8192 pairs the grouping runs as two launches of several blocks: bit-exact against the
    oracle for ragged sizes, skewed expert loads and experts without rows, twice in a row, then once
    more with a smaller batch (another number of blocks)."""
    import torch
    cfg = configs.TINY.with_(n_experts=experts, top_k=top_k, top_n=top_n, tokens=tokens, rank=0, name="perm_blocks")
    L = amd.Layer.from_config(cfg, max_tokens=tokens)
    rng = np.random.default_rng(experts * 1000 + tokens)
    for T in (tokens, tokens, max(8192 // top_k + 1, tokens // 2)):
        # distinct experts per token, skewed towards a few; expert 1 never chosen
        pw = rng.random(experts) ** 4
        pw[1 % experts] = 0.0
        pw /= pw.sum()
        idx = np.stack([rng.choice(experts, size=top_k, replace=False, p=pw) for _ in range(T)]).astype(np.int32)
        p = orc.permute(idx, experts, top_n)
        got = L.permute(torch.from_numpy(idx).cuda())
        for g, key in zip(got, ("counts", "offsets", "row_pair", "pair_row", "comp_counts")):
            np.testing.assert_array_equal(_to_np(g), p[key], err_msg=f"T={T} {key}")
    L.close()


def test_expert_ffn_and_combine(case):
    cfg, layer, L, x_bits, x, ref = case
    idx, w = L.route(x)
    counts, offsets, row_pair, pair_row, comp = L.permute(idx)
    y = L.expert_ffn(x, offsets, row_pair)
    err_rows = orc.rel_frobenius(_to_np(y), ref["y_rows"])
    out = L.combine(y, w, pair_row, x)
    err_out = orc.rel_frobenius(_to_np(out), ref["out"])
    per_tok = np.linalg.norm(_to_np(out) - ref["out"], axis=1) / np.linalg.norm(ref["out"], axis=1)
    print(f"[{cfg.name}] y_rows rel err {err_rows:.2e}, out rel err {err_out:.2e}, worst token {per_tok.max():.2e}")
    assert err_rows <= TOL and err_out <= TOL
    st = L.stats()
    from oracle import compress
    want = compress.staged_bytes(ref["perm"]["counts"], ref["perm"]["comp_counts"], cfg.hidden, cfg.ffn,
                                 cfg.bits, cfg.group, cfg.rank)
    P = 3 * cfg.hidden * cfg.ffn
    assert st["active_experts"] == want["active_experts"]
    assert st["comp_experts"] == (want["comp_experts"] if cfg.rank and cfg.top_n else 0)
    assert st["bytes_codes"] == want["bytes_codes"] + cfg.n_shared * P * cfg.shared_bits // 8
    assert st["bytes_meta"] == want["bytes_meta"] + cfg.n_shared * (P // cfg.group * 4)
    assert st["bytes_factors"] == (want["bytes_factors"] if cfg.top_n else 0)


def test_forward_matches_four_calls_and_is_deterministic(case):
    import torch
    cfg, layer, L, x_bits, x, ref = case
    idx, w = L.route(x)
    counts, offsets, row_pair, pair_row, comp = L.permute(idx)
    y = L.expert_ffn(x, offsets, row_pair)
    out4 = L.combine(y, w, pair_row, x).clone()
    out_a = L.forward(x).clone()
    out_b = L.forward(x).clone()
    assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16)), "two runs differ"
    # the composite equals the four calls up to rounding: it may add the fp32 K-block partial sums of
    # W2 in the combine instead of reading expert rows rounded to bf16 (one bf16 rounding, 2^-9, fewer)
    assert orc.rel_frobenius(_to_np(out_a), _to_np(out4)) <= 2.5e-3, "forward differs from the four calls by more than a rounding"
    e_fwd, e_four = orc.rel_frobenius(_to_np(out_a), ref["out"]), orc.rel_frobenius(_to_np(out4), ref["out"])
    print(f"[{cfg.name}] forward {e_fwd:.2e}, four calls {e_four:.2e}")
    assert e_fwd <= TOL and e_fwd <= e_four * 1.05 + 1e-4


def test_workspace_contents_do_not_matter(case):
    """The caller's workspace may hold anything: the forward pass (and the four calls) give the same
    bits after it was filled with 0xFF bytes (NaN patterns as fp16 or fp32, -1 as integers) as after
    zeros.  This covers the rows the kernels stage in place of rows past an expert's last one (kept
    at zero by the preparing launch of the same call) and every table the launches hand each other."""
    import torch
    cfg, layer, L, x_bits, x, ref = case
    T = x.shape[0]
    outs = []
    for fill in (0x00, 0xFF, 0x7E):
        L.workspace(T).fill_(fill)
        out = L.forward(x).clone()
        L.workspace(T).fill_(fill)
        idx, w = L.route(x)
        counts, offsets, row_pair, pair_row, comp = L.permute(idx)
        y = L.expert_ffn(x, offsets, row_pair)
        out4 = L.combine(y, w, pair_row, x).clone()
        outs.append((out, out4))
    for out, out4 in outs[1:]:
        assert torch.equal(out.view(torch.int16), outs[0][0].view(torch.int16)), "forward depends on what the workspace held"
        assert torch.equal(out4.view(torch.int16), outs[0][1].view(torch.int16)), "the four calls depend on what the workspace held"
    assert orc.rel_frobenius(_to_np(outs[1][0]), ref["out"]) <= TOL


def test_constructed_ties(amd):
    # duplicated gate rows and an all-zero token: lower index wins, on the GPU as in the oracle
    cfg = configs.TINY.with_(top_k=3, top_n=1, tokens=40, rank=0, name="ties")
    rng = np.random.default_rng(3)
    wg = rng.normal(size=(cfg.n_experts, cfg.hidden)).astype(np.float32)
    wg[5] = wg[2]; wg[7] = wg[2]
    xf = rng.normal(size=(cfg.tokens, cfg.hidden)).astype(np.float32)
    xf[0] = 0.0
    wg_bits, x_bits = synth.f32_to_bf16_bits(wg), synth.f32_to_bf16_bits(xf)
    ref = orc.route(x_bits, wg_bits, cfg.top_k)
    assert (ref["margin"] == 0).any()
    L = amd.Layer.from_config(cfg)
    L.set_gate(wg_bits)
    idx, w = L.route(amd.bf16_tensor(x_bits))
    np.testing.assert_array_equal(_to_np(idx), ref["idx"])
    np.testing.assert_allclose(_to_np(w), ref["w"], rtol=2e-6)
    assert list(_to_np(idx)[0]) == [0, 1, 2]
    L.close()


def test_n0_equals_rank0_layer_bitwise(amd):
    import torch
    cfg = configs.TINY.with_(top_n=0, name="n0")
    layer, L = _build(amd, cfg)
    cfg0 = configs.TINY.with_(rank=0, name="r0")
    layer0 = {"wg": layer["wg"], "bias": layer["bias"],
              "experts": [{m: dict(ex[m], A=None, B=None) for m in (0, 1, 2)} for ex in layer["experts"]]}
    L0 = amd.Layer.from_config(cfg0)
    L0.load(layer0)
    x_bits = synth.make_tokens(cfg)
    x = amd.bf16_tensor(x_bits)
    a, b = L.forward(x).clone(), L0.forward(x).clone()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    ref = fixtures.oracle_forward(cfg, layer, x_bits)
    assert orc.rel_frobenius(_to_np(a), ref["out"]) <= TOL
    L.close(); L0.close()


def test_large_scale_and_degenerate_groups(amd):
    # scales >= 1 (constant groups get scale 1) must not overflow the fp16 metadata
    cfg = configs.TINY.with_(rank=0, top_n=0, bits=2, name="degenerate")
    layer = fixtures.build_layer(cfg)
    ex = layer["experts"][0]
    for m in (0, 1, 2):
        ex[m]["codes"][:64, :] = 0
        s = ex[m]["scale"].view(np.float16).copy(); z = ex[m]["zero"].view(np.float16).copy()
        s[0, :] = 1.0; z[0, :] = 0.01
        s[1, ::2] = 3.0
        ex[m]["scale"], ex[m]["zero"] = s.view(np.uint16), z.view(np.uint16)
    L = amd.Layer.from_config(cfg)
    L.load(layer)
    x_bits = synth.make_tokens(cfg)
    ref = fixtures.oracle_forward(cfg, layer, x_bits)
    out = L.forward(amd.bf16_tensor(x_bits))
    assert np.isfinite(_to_np(out)).all()
    assert orc.rel_frobenius(_to_np(out), ref["out"]) <= TOL
    L.close()


def test_staged_mode_matches_resident(amd):
    import torch
    cfg = configs.TINY.with_(tokens=5, name="staged")     # few tokens: some experts stay on the host
    layer = fixtures.build_layer(cfg)
    # The device slots of a staged layer start out with whatever the allocation held.  Make that
    # NaN factors (a resident layer with poisoned factors, destroyed right before): an expert whose
    # factors are not brought in must not touch its factor slot.
    import copy
    poison = copy.deepcopy(layer)
    for ex in poison["experts"]:
        for a in ex.values():
            if a.get("A") is not None and np.size(a["A"]):
                a["A"] = np.full_like(a["A"], 0x7FC0)
                a["B"] = np.full_like(a["B"], 0x7FC0)
    Lp = amd.Layer.from_config(cfg, max_tokens=16)
    Lp.load(poison)
    Lp.close()
    Ls = amd.Layer.from_config(cfg, max_tokens=16, residency=amd.STAGED)
    Lr = amd.Layer.from_config(cfg, max_tokens=16)
    Lr.load(layer); Ls.load(layer)
    x_bits = synth.make_tokens(cfg)
    x = amd.bf16_tensor(x_bits)
    a, b = Lr.forward(x).clone(), Ls.forward(x).clone()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    ref = fixtures.oracle_forward(cfg, layer, x_bits)
    from oracle import compress
    want = compress.staged_bytes(ref["perm"]["counts"], ref["perm"]["comp_counts"], cfg.hidden, cfg.ffn,
                                 cfg.bits, cfg.group, cfg.rank)
    st = Ls.stats()
    assert want["active_experts"] < cfg.n_experts
    for k in ("active_experts", "comp_experts", "bytes_codes", "bytes_meta", "bytes_factors"):
        assert st[k] == want[k], k
    assert st["stage_ms"] > 0
    # a second batch that routes elsewhere must bring in its own experts
    cfg2 = cfg.with_(seed=99, tokens=7)
    x2_bits = synth.make_tokens(cfg2)
    x2 = amd.bf16_tensor(x2_bits)
    assert torch.equal(Lr.forward(x2).view(torch.int16), Ls.forward(x2).view(torch.int16))
    np.testing.assert_array_equal(_to_np(Ls.debug_unpack(3, 1)), layer["experts"][3][1]["codes"])
    Lr.close(); Ls.close()


def test_long_k_several_staging_phases(amd):
    """An FFN width of 36864: the decode flavour's W2 launch splits its K into 8 K-blocks of 18
    k-steps, i.e. two staging phases per block with one row tile and three with two (the Mixtral
    shape has one and two).  Two experts, k = 2: each holds every token, so 20 tokens take the
    two-row-tile body and their first 10 the one-row-tile body."""
    # the same for the fused projection, whose K is the hidden size and is not split into K-blocks:
    # the largest hidden size a layer accepts gives four and eight phases
    # (and 150 tokens: the grouped-GEMM flavour, two chunks per expert, over the same long K)
    for cfg in (configs.TINY.with_(n_experts=2, top_k=2, top_n=1, tokens=150, ffn=36864, bits=2, rank=8, name="long_k"),
                configs.TINY.with_(n_experts=2, top_k=2, top_n=1, tokens=150, hidden=16384, ffn=256, bits=3, rank=8, name="long_h")):
        layer, L = _build(amd, cfg)
        x_bits = synth.make_tokens(cfg)
        for T in (20, 10, 150):
            ref = fixtures.oracle_forward(cfg.with_(tokens=T), layer, x_bits[:T])
            out = L.forward(amd.bf16_tensor(x_bits[:T]))
            err = orc.rel_frobenius(_to_np(out), ref["out"])
            print(f"[{cfg.name}] T={T}: {err:.2e}")
            assert err <= TOL
        L.close()


def test_empty_batch(amd):
    """T = 0: every hot-path call returns without touching its per-token buffers (empty tensors have
    null data pointers); the grouping still reports zero rows for every expert."""
    import torch
    cfg = configs.TINY
    layer, L = _build(amd, cfg)
    x0 = torch.empty((0, cfg.hidden), dtype=torch.bfloat16, device="cuda")
    idx, w = L.route(x0)
    assert idx.shape == (0, cfg.top_k) and w.shape == (0, cfg.top_k)
    counts, offsets, row_pair, pair_row, comp = L.permute(idx)
    torch.cuda.synchronize()
    assert not counts.any() and not offsets.any() and not comp.any()
    y = L.expert_ffn(x0, offsets, row_pair)
    out = L.combine(y, w, pair_row, x0)
    assert y.shape == (0, cfg.hidden) and out.shape == (0, cfg.hidden)
    assert L.forward(x0).shape == (0, cfg.hidden)
    sentinel = torch.full((4, cfg.hidden), 1.5, dtype=torch.bfloat16, device="cuda")
    L.forward(x0, out=sentinel[:0])
    torch.cuda.synchronize()
    assert (sentinel == 1.5).all()
    # and the layer still works afterwards
    x_bits = synth.make_tokens(cfg)
    ref = fixtures.oracle_forward(cfg, layer, x_bits)
    assert orc.rel_frobenius(_to_np(L.forward(amd.bf16_tensor(x_bits))), ref["out"]) <= TOL
    L.close()


def test_hot_path_argument_errors(amd):
    import torch
    cfg = configs.TINY
    L = amd.Layer.from_config(cfg)
    x = amd.bf16_tensor(synth.make_tokens(cfg))
    with pytest.raises(amd.MoeLrcError) as ei:
        L.route(x)                                # gate not uploaded
    assert ei.value.code == -3
    wg, _ = synth.make_gate(cfg)
    L.set_gate(wg)
    with pytest.raises(amd.MoeLrcError) as ei:
        L.forward(x)                              # experts not uploaded
    assert ei.value.code == -3
    big = torch.zeros((cfg.tokens + 1, cfg.hidden), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(amd.MoeLrcError) as ei:
        L.route(big)                              # T > max_tokens
    assert ei.value.code == -3
    with pytest.raises(amd.MoeLrcError) as ei:
        L.set_expert(0, 0, np.full((256, 512), 9, np.uint8), np.zeros((4, 512), np.uint16),
                     np.zeros((4, 512), np.uint16), np.zeros((256, 8), np.uint16), np.zeros((8, 512), np.uint16))
    assert ei.value.code == -1                    # code out of range for 3 bits
    L.close()


@pytest.mark.parametrize("name", ["tiny", "deepseek_small"])
def test_forward_under_graph_capture_replays_like_eager(amd, name):
    """moe_lrc_forward allocates nothing, never synchronises in resident mode and clears nothing with
    a memset, so it can be captured into a HIP graph (with shared experts the capture forks to the
    layer's side stream and joins again).  Every replay, with the program's own eager work and
    synchronisations in between, must give the bits of the eager call on the same tokens."""
    import torch
    cfg = SMALL[name]
    layer = fixtures.build_layer(cfg)
    L = amd.Layer.from_config(cfg)
    L.load(layer)
    T = cfg.tokens
    xs = [amd.bf16_tensor(synth.make_tokens(cfg.with_(seed=cfg.seed + 17 * i))) for i in range(3)]
    eager = [L.forward(x).clone() for x in xs]           # (also the warm-up: function attributes are set)
    torch.cuda.synchronize()
    x_static = xs[0].clone()
    out = torch.empty((T, cfg.hidden), dtype=torch.bfloat16, device="cuda")
    ws = L.workspace(T)
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            L.forward_raw(x_static.data_ptr(), T, out.data_ptr(), ws.data_ptr(), ws.numel(),
                          torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for rep in range(2):
        for i, x in enumerate(xs):
            x_static.copy_(x)
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), eager[i].view(torch.int16)), (rep, i)
            again = L.forward(x)                          # eager work between the replays
            torch.cuda.synchronize()
            assert torch.equal(again.view(torch.int16), eager[i].view(torch.int16))
    L.close()


def test_route_tiled_path_many_tokens_and_experts(amd):
    """With >= 1024 tokens and >= 128 experts the logits come from the tiled fp64-matrix-core kernel
    (ragged token and expert tiles here: T = 1100, E = 136): indices bit-exact, ties included."""
    cfg = configs.QWEN3.with_(hidden=320, ffn=256, group=64, n_experts=136, tokens=1100, rank=0, top_n=0, name="route_tiled")
    wg, bias = synth.make_gate(cfg)
    wg = wg.copy()
    wg[5] = wg[77]                      # a duplicated gate row: equal logits, the lower index wins
    if bias is not None:
        bias = bias.copy(); bias[5] = bias[77]
    x_bits = synth.make_tokens(cfg)
    ref = orc.route(x_bits, wg, cfg.top_k, cfg.renormalize, bias)
    L = amd.Layer.from_config(cfg)
    L.set_gate(wg, bias)
    idx, w = L.route(amd.bf16_tensor(x_bits))
    np.testing.assert_array_equal(_to_np(idx), ref["idx"])
    np.testing.assert_allclose(_to_np(w), ref["w"], rtol=2e-6, atol=1e-30)
    L.close()


@pytest.mark.parametrize("hidden,experts", [(64, 8), (1024, 64), (2048, 8), (8192, 8), (8192, 64), (16384, 8), (16384, 130)])
def test_route_over_hidden_sizes(amd, hidden, experts):
    """Every variant of the per-token routing kernel (1 to 32 chunks of a row per lane, 4 or 16
    wavefronts per token), up to the largest hidden size a layer accepts: indices bit-exact."""
    cfg = configs.TINY.with_(hidden=hidden, ffn=64, group=64, n_experts=experts, top_k=min(6, experts), top_n=0, rank=0,
                             tokens=9, name=f"route_h{hidden}_e{experts}")
    wg, bias = synth.make_gate(cfg)
    wg = wg.copy()
    wg[1] = wg[experts - 1]             # equal logits: the lower index wins
    x_bits = synth.make_tokens(cfg)
    ref = orc.route(x_bits, wg, cfg.top_k, cfg.renormalize, bias)
    L = amd.Layer.from_config(cfg)
    L.set_gate(wg, bias)
    idx, w = L.route(amd.bf16_tensor(x_bits))
    np.testing.assert_array_equal(_to_np(idx), ref["idx"])
    np.testing.assert_allclose(_to_np(w), ref["w"], rtol=2e-6, atol=1e-30)
    L.close()


def test_route_with_several_blocks_per_token(amd):
    """With few tokens and 128 experts or more, several blocks share a token's gate rows and leave
    their logits in memory for the Top-k launch that follows.  Batches of different sizes, hence
    different numbers of blocks per token, one after the other on one layer: indices bit-exact every
    time, a duplicated gate row and a ragged expert count (136) included."""
    for E in (128, 136):
        cfg = configs.QWEN3.with_(hidden=512, ffn=256, group=64, n_experts=E, tokens=100, rank=0, top_n=0, name=f"route_split_{E}")
        wg, bias = synth.make_gate(cfg)
        wg = wg.copy()
        wg[3] = wg[E - 2]                   # equal logits in different blocks' shares: the lower index wins
        if bias is not None:
            bias = bias.copy(); bias[3] = bias[E - 2]
        x_bits = synth.make_tokens(cfg)
        ref = orc.route(x_bits, wg, cfg.top_k, cfg.renormalize, bias)
        L = amd.Layer.from_config(cfg)
        L.set_gate(wg, bias)
        x = amd.bf16_tensor(x_bits)
        for T in (1, 100, 3, 16, 1, 64, 17, 100):
            idx, w = L.route(x[:T])
            np.testing.assert_array_equal(_to_np(idx), ref["idx"][:T], err_msg=f"E={E} T={T}")
            np.testing.assert_allclose(_to_np(w), ref["w"][:T], rtol=2e-6, atol=1e-30)
        L.close()


@pytest.mark.parametrize("tokens", [16, 300])
def test_rank_per_projection_from_kurtosis(amd, tokens):
    """Section 3.1 step 1: the rank budget is spread over the expert matrices by their kurtosis, so
    every projection has a rank of its own (0 included, W1 and W3 of one expert may differ).
    Decode flavour (16 tokens) and grouped-GEMM flavour (300 tokens), resident and staged; the
    staged mode moves only the ranks uploaded."""
    import torch
    cfg = configs.TINY.with_(rank=32, tokens=tokens, name=f"ranks_T{tokens}")
    ranks = fixtures.kurtosis_ranks(cfg, 10, (0, 8, 16, 32))
    assert len(set(ranks.ravel().tolist())) >= 3 and (ranks[:, 0] != ranks[:, 1]).any()
    layer = fixtures.build_layer(cfg, ranks=ranks)
    x_bits = synth.make_tokens(cfg)
    x = amd.bf16_tensor(x_bits)
    ref = fixtures.oracle_forward(cfg, layer, x_bits)
    Lr = amd.Layer.from_config(cfg)
    Ls = amd.Layer.from_config(cfg, residency=amd.STAGED)
    Lr.load(layer); Ls.load(layer)
    out_r = Lr.forward(x).clone()
    torch.cuda.synchronize()
    out_s = Ls.forward(x).clone()
    torch.cuda.synchronize()
    err = orc.rel_frobenius(_to_np(out_r), ref["out"])
    print(f"\n[ranks_T{tokens}] ranks {ranks.tolist()} out rel err {err:.2e}", flush=True)
    assert err <= TOL
    assert torch.equal(out_r.view(torch.int16), out_s.view(torch.int16))
    st = Ls.stats()
    comp = np.asarray(ref["perm"]["comp_counts"]) > 0
    assert st["bytes_factors"] == int((ranks[comp].sum(axis=1) * (cfg.hidden + cfg.ffn) * 2).sum())
    # re-uploading a projection with a smaller rank leaves no trace of the larger one
    e = int(np.argmax(ranks[:, 0] == 32))
    a = dict(layer["experts"][e][0])
    Lr.set_expert(e, 0, a["codes"], a["scale"], a["zero"], None, None, rank=0)
    layer2 = {"wg": layer["wg"], "bias": layer["bias"], "experts": [dict(ex) for ex in layer["experts"]]}
    layer2["experts"][e][0] = dict(a, A=None, B=None, rank=0)
    ref2 = fixtures.oracle_forward(cfg, layer2, x_bits)
    assert orc.rel_frobenius(_to_np(Lr.forward(x)), ref2["out"]) <= TOL
    Lr.close(); Ls.close()


@pytest.mark.parametrize("tokens,rank", [(16, 16), (300, 32), (40, 24), (24, 72), (700, 64)])
def test_int3_factors(amd, tokens, rank):
    """Section 3.1 step 2 stores the factor pairs at INT3: uploaded as 3-bit codes + fp16 scale/zero
    per group of 64, kept at 3 bits in the pinned pool and on the device, and dequantized inside the
    kernels that consume them (both flavours of the (in A) and of the FFN kernels are reached: 16 to
    700 tokens).  Resident and staged layers agree bit for bit and match the oracle on the quantized
    factors; the staged byte counter counts a 4-bit cell + scale/zero per value."""
    import torch
    cfg = configs.TINY.with_(rank=rank, tokens=tokens, bits=2, name=f"int3_T{tokens}_r{rank}")
    layer = fixtures.build_layer(cfg, int3_factors=True)
    x_bits = synth.make_tokens(cfg)
    x = amd.bf16_tensor(x_bits)
    ref = fixtures.oracle_forward(cfg, layer, x_bits)
    Lr = amd.Layer.from_config(cfg)
    Ls = amd.Layer.from_config(cfg, residency=amd.STAGED)
    Lr.load(layer); Ls.load(layer)
    out_r = Lr.forward(x).clone()
    torch.cuda.synchronize()
    out_s = Ls.forward(x).clone()
    torch.cuda.synchronize()
    err = orc.rel_frobenius(_to_np(out_r), ref["out"])
    print(f"\n[{cfg.name}] out rel err {err:.2e}", flush=True)
    assert err <= TOL
    assert torch.equal(out_r.view(torch.int16), out_s.view(torch.int16))
    n_comp = int((np.asarray(ref["perm"]["comp_counts"]) > 0).sum())
    vals = 3 * rank * (cfg.hidden + cfg.ffn)
    assert Ls.stats()["bytes_factors"] == n_comp * (vals * 4 // 8 + vals // 64 * 4)
    # the compensation is really there: without it the output differs by far more than the tolerance
    assert orc.rel_frobenius(_to_np(out_r), fixtures.oracle_forward(cfg.with_(top_n=0), layer, x_bits)["out"]) > 5 * TOL
    Lr.close(); Ls.close()


@pytest.mark.parametrize("tokens", [16, 300, 700])
def test_int3_factors_with_a_rank_per_projection(amd, tokens):
    """Factor pairs at 3 bits whose ranks differ from matrix to matrix (Section 3.1 steps 1 and 2
    together): W1 and W3 of an expert run different numbers of rank steps, some projections have no
    pair at all, and the factor tiles past a projection's own rank are never read.  All three
    flavour mixes (16, 300, 700 tokens), resident against staged bit for bit."""
    import torch
    cfg = configs.TINY.with_(rank=64, tokens=tokens, bits=2, name=f"int3_ranks_T{tokens}")
    ranks = fixtures.kurtosis_ranks(cfg, 26, (0, 16, 32, 64))
    assert len(set(ranks.ravel().tolist())) >= 3 and (ranks[:, 0] != ranks[:, 1]).any()
    layer = fixtures.build_layer(cfg, ranks=ranks, int3_factors=True)
    x_bits = synth.make_tokens(cfg)
    x = amd.bf16_tensor(x_bits)
    ref = fixtures.oracle_forward(cfg, layer, x_bits)
    Lr = amd.Layer.from_config(cfg)
    Ls = amd.Layer.from_config(cfg, residency=amd.STAGED)
    Lr.load(layer); Ls.load(layer)
    out_r = Lr.forward(x).clone()
    torch.cuda.synchronize()
    out_s = Ls.forward(x).clone()
    torch.cuda.synchronize()
    err = orc.rel_frobenius(_to_np(out_r), ref["out"])
    print(f"\n[{cfg.name}] ranks {ranks.tolist()} out rel err {err:.2e}", flush=True)
    assert err <= TOL
    assert torch.equal(out_r.view(torch.int16), out_s.view(torch.int16))
    assert orc.rel_frobenius(_to_np(out_r), fixtures.oracle_forward(cfg.with_(top_n=0), layer, x_bits)["out"]) > 3 * TOL
    Lr.close(); Ls.close()


def test_mixed_fp16_and_int3_projections_staged(amd):
    """One expert may hold one projection's factors as an fp16 pair and the others at 3 bits: each
    pair lives in its own projection's factor sections, so neither upload disturbs the other, and
    the kernels take the format per projection from the expert table.  Staged and resident layers
    agree bit for bit and match the oracle."""
    import torch
    cfg = configs.TINY.with_(rank=32, tokens=24, bits=2, name="mixed_q3")
    bf = fixtures.build_layer(cfg)
    q3 = fixtures.build_layer(cfg, int3_factors=True)
    experts = []
    for e in range(cfg.n_experts):                       # W1 as a bf16 pair, W3 and W2 at 3 bits (and rotated per expert)
        keep = e % 3
        experts.append({m: (bf if m == keep else q3)["experts"][e][m] for m in (0, 1, 2)})
    layer = {"wg": bf["wg"], "bias": bf["bias"], "experts": experts}
    x_bits = synth.make_tokens(cfg)
    x = amd.bf16_tensor(x_bits)
    ref = fixtures.oracle_forward(cfg, layer, x_bits)
    Lr = amd.Layer.from_config(cfg)
    Ls = amd.Layer.from_config(cfg, residency=amd.STAGED)
    # upload order matters for an overlap bug: 3-bit blobs first on one layer, last on the other
    Lr.load(layer)
    Ls.set_gate(layer["wg"], layer["bias"])
    for e, ex in enumerate(experts):
        for m in (2, 1, 0):
            a = ex[m]
            if a.get("Aq") is not None:
                Ls.set_expert(e, m, a["codes"], a["scale"], a["zero"], None, None, 0)
                Ls.set_expert_factors_quantized(e, m, a["Aq"]["codes"].shape[1], a["Aq"], a["Bq"])
        for m in (0, 1, 2):
            a = ex[m]
            if a.get("Aq") is None:
                Ls.set_expert(e, m, a["codes"], a["scale"], a["zero"], a["A"], a["B"], cfg.rank)
    out_r = Lr.forward(x).clone()
    out_s = Ls.forward(x).clone()
    torch.cuda.synchronize()
    err = orc.rel_frobenius(_to_np(out_r), ref["out"])
    print(f"\n[{cfg.name}] out rel err {err:.2e}", flush=True)
    assert err <= TOL
    assert torch.equal(out_r.view(torch.int16), out_s.view(torch.int16))
    Lr.close(); Ls.close()


def test_stats_path_reports_the_flavour(amd):
    """moe_lrc_stats.path: bit 0 = W1|W3 ran as the grouped GEMM, bit 1 = W2 did."""
    import torch
    cfg = configs.TINY.with_(tokens=700, rank=8, name="path")
    layer = fixtures.sample_layer(cfg)
    L = amd.Layer.from_config(cfg)
    L.load(layer)
    for T, want in ((8, 0), (700, 3)):
        x = amd.bf16_tensor(synth.make_tokens(cfg, T))
        L.forward(x)
        torch.cuda.synchronize()
        assert L.stats()["path"] == want, (T, L.stats()["path"])
    L.close()


@pytest.mark.parametrize("tokens", [16, 100, 300, 700])
def test_ranks_from_the_papers_bucket_up_to_1024(amd, tokens):
    """Section 3.1 step 1 allocates every expert matrix a rank from the bucket {0, 16, 32, 128, 256,
    512, 1024}.  A layer whose projections cycle through the whole bucket (W1, W3 and W2 of one expert
    all different), at 16 tokens (skinny kernels, one row tile), 100 (two row tiles, several passes,
    the (in A) fragments of the large ranks taking the place of the staged activations), 300 (fused
    projection as grouped GEMM, W2 skinny) and 700 (both grouped GEMM, rank steps in chunks), against
    the oracle on the same stored factors; resident and staged layers agree bit for bit."""
    import torch
    bucket = (0, 16, 32, 128, 256, 512, 1024)
    cfg = configs.TINY.with_(rank=1024, tokens=tokens, bits=2, name=f"bucket_T{tokens}")
    layer = fixtures.sample_layer(cfg)
    for e, ex in enumerate(layer["experts"]):
        for m in (0, 1, 2):
            r = bucket[(3 * e + 2 * m) % len(bucket)]
            a = ex[m]
            a["rank"] = r
            a["A"] = np.ascontiguousarray(a["A"][:, :r]) if r else None
            a["B"] = np.ascontiguousarray(a["B"][:r]) if r else None
    x_bits = synth.make_tokens(cfg)
    x = amd.bf16_tensor(x_bits)
    ref = fixtures.oracle_forward(cfg, layer, x_bits)
    Lr = amd.Layer.from_config(cfg)
    Ls = amd.Layer.from_config(cfg, residency=amd.STAGED)
    Lr.load(layer); Ls.load(layer)
    out_r = Lr.forward(x).clone()
    torch.cuda.synchronize()
    out_s = Ls.forward(x).clone()
    torch.cuda.synchronize()
    err = orc.rel_frobenius(_to_np(out_r), ref["out"])
    none = orc.rel_frobenius(_to_np(out_r), fixtures.oracle_forward(cfg.with_(top_n=0), layer, x_bits)["out"])
    print(f"\n[{cfg.name}] out rel err {err:.2e} (the rank terms move the output by {none:.2e})", flush=True)
    assert err <= TOL and none > 10 * TOL
    assert torch.equal(out_r.view(torch.int16), out_s.view(torch.int16))
    Lr.close(); Ls.close()
