#!/usr/bin/env python3
"""Benchmark of one MoE layer's forward pass (route -> permute -> expert FFN -> combine) on one MI355X.

A step is one moe_lrc_forward over one batch of synthetic tokens, with packed experts, factors and
tokens already resident in HBM.  The timed calls rotate over several independent layer instances
so that every call streams weights that are cold in the 256 MB last-level cache, as in a real
multi-layer model.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mixtral_decode_T64_b2]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense fp16/bf16 MFMA, published



def counter_traffic(workload):
    """HBM bytes per launch of the dominant kernel from hardware counters (FETCH_SIZE + WRITE_SIZE,
    each scaled by what the same counter reads for a copy kernel of known size; two separate profiler
    runs of this script).  Counters cannot be read from inside a timed run: the figure is taken from
    the counter summary of this workload under profiles/ (a line `traffic_bytes_per_launch: N`), and
    is null when there is none.  Returns (bytes or None, file name or None)."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.md")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1].strip()), os.path.relpath(path, ROOT)
    except OSError:
        pass
    return None, None


def algorithmic_bytes(cfg, T, active, comp, fb=2.0):
    """Bytes each kernel must move per launch: packed codes + fp16 scale/zero of active experts,
    factor bytes of comp-active experts (fb bytes per factor value: 2 as fp16, 0.5625 at 3 bits in
    4-bit cells with fp16 scale/zero per 64), activations in and out."""
    H, F, b, g, r, k = cfg.hidden, cfg.ffn, cfg.bits, cfg.group, cfg.rank, cfg.top_k
    per_w = b / 8 + 4 / g                       # bytes per weight incl. scale/zero
    rows = T * k
    w13 = active * 2 * H * F * per_w + comp * 2 * r * F * fb + T * H * 2 + rows * F * 2
    w2 = active * H * F * per_w + comp * r * H * fb + rows * F * 2 + rows * H * 2
    xa13 = comp * 2 * H * r * fb
    xa2 = comp * F * r * fb
    shared = cfg.n_shared * 3 * H * F * (cfg.shared_bits / 8 + 4 / g)
    total = w13 + w2 + xa13 + xa2 + shared + T * H * 2 * 2
    return {"w13": w13, "w2": w2, "xa13": xa13, "xa2": xa2, "shared": shared, "total": total}


def algorithmic_flops(cfg, T):
    H, F, r, k, n = cfg.hidden, cfg.ffn, cfg.rank, cfg.top_k, cfg.top_n
    return T * k * 2 * 3 * H * F + T * n * 2 * 3 * r * (H + F) + T * cfg.n_shared * 2 * 3 * H * F


def cpu_baseline(cfg, layer, x_bits, budget_tokens=8):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload on the host cores."""
    from oracle import fixtures
    from oracle import moe_lrc_oracle as orc
    r = orc.route(x_bits, layer["wg"], cfg.top_k, cfg.renormalize, layer["bias"])
    mask = np.zeros(x_bits.shape[0], bool)
    mask[:min(budget_tokens, x_bits.shape[0])] = True
    t0 = time.perf_counter()
    fixtures.oracle_forward(cfg, layer, x_bits, token_mask=mask)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    n = int(mask.sum())
    return {"value": n / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"numpy fp64 oracle, routing of all {x_bits.shape[0]} tokens, expert FFN + combine of the "
                      f"first {n} tokens ({dt:.1f} s); tokens/s = {n} / time (extrapolates linearly in tokens)",
            "active_experts_full_batch": int((np.bincount(r['idx'].ravel(), minlength=cfg.n_experts) > 0).sum())}


def stack_bench(args, cfg):
    """Decode steps through a stack of layers whose experts live in pinned host memory and share a
    device slot pool (Section 4.3, case study 1).  Prints its own JSON line; never the headline value."""
    import torch
    import paper_2512_17073_amd as amd
    from workload import synth
    T, nl, E = cfg.tokens, args.stack, cfg.n_experts
    slots = args.slots or nl * E
    print(f"[bench] stack of {nl} x {cfg.name}, {slots} slots: generating artefacts", file=sys.stderr, flush=True)
    experts = [{m: synth.sample_artifacts(cfg, e, m) for m in (0, 1, 2)} for e in range(E + cfg.n_shared)]
    layers = []
    for i in range(nl):
        wg, bias = synth.make_gate(cfg.with_(seed=cfg.seed + 17 * i))          # a gate of its own per layer
        L = amd.Layer.from_config(cfg, residency=amd.POOLED)
        L.set_gate(wg, bias)
        for e in range(E + cfg.n_shared):
            src = experts[(e + i) % E] if e < E else experts[e]
            for m in (0, 1, 2):
                a = src[m]
                if args.int3_factors and e < E and cfg.rank > 0:
                    L.set_expert(e, m, a["codes"], a["scale"], a["zero"], None, None, 0)
                    L.set_expert_factors_quantized(e, m, cfg.rank, *synth.sample_factor_codes(cfg, (e + i) % E, m))
                else:
                    L.set_expert(e, m, a["codes"], a["scale"], a["zero"], a["A"], a["B"])
        layers.append(L)
        print(f"[bench] layer {i + 1}/{nl} packed into pinned memory", file=sys.stderr, flush=True)
    st = amd.Stack(layers, slots=slots, prefetch=not args.no_prefetch, residual=True)
    xs = [amd.bf16_tensor(synth.make_tokens(cfg.with_(seed=cfg.seed + 1000 + i))) for i in range(8)]
    out = torch.empty_like(xs[0])
    for i in range(args.warmup if args.warmup < 5 else 2):
        st.step(xs[i % 8], out)
    torch.cuda.synchronize()
    s0 = st.stats()
    step_ms, copy_ms = [], 0.0
    t0 = time.perf_counter()
    for i in range(args.steps if args.steps < 200 else 20):
        st.step(xs[(i + 3) % 8], out)
        s = st.stats()                       # (waits for the step's copies)
        step_ms.append(s["last_step_ms"]); copy_ms += s["last_copy_ms"]
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    s1 = st.stats()
    d = {k: s1[k] - s0[k] for k in ("expert_uses", "hits", "misses", "prefetched", "prefetch_hits", "factor_copies", "bytes_h2d")}
    n = len(step_ms)
    print(json.dumps({
        "metric": "stack_decode_tokens_per_s", "value": T * n / dt, "unit": "tokens/s", "n_gpus": 1, "steps": n,
        "ms_per_step": dt / n * 1e3, "ms_per_layer": dt / n / nl * 1e3, "higher_is_better": True, "data": "synthetic",
        "config": {"workload": cfg.name, "layers": nl, "slots": slots, "experts_per_layer": E, "tokens": T,
                   "prefetch": not args.no_prefetch, "residency": "pooled (pinned host memory)",
                   "factors": "int3" if args.int3_factors else "bf16"},
        "transfers": dict(d, hit_rate=d["hits"] / max(1, d["expert_uses"]),
                          h2d_gb_per_s_while_copying=d["bytes_h2d"] / max(copy_ms, 1e-9) / 1e6 if copy_ms else None,
                          h2d_gb_per_s_over_the_run=d["bytes_h2d"] / dt / 1e9),
        "step_ms_median": float(np.median(step_ms)), "step_ms_p10": float(np.percentile(step_ms, 10)),
        "step_ms_p90": float(np.percentile(step_ms, 90)),
    }))
    st.close()
    for L in layers:
        L.close()


def offline_bench(args, cfg):
    """The offline pipeline (quantizer, residual, rank-r factors) on one W1-shaped matrix of the
    workload, device against the oracle's numpy on the host.  A line of its own."""
    import torch
    import paper_2512_17073_amd as amd
    from oracle import compress
    K, N, r = cfg.hidden, cfg.ffn, max(cfg.rank, 8)
    rng = np.random.default_rng(cfg.seed)
    W = rng.standard_normal((K, N)) * 0.02
    omega = np.random.default_rng(1).standard_normal((N, r + 8))
    Wd, Od = torch.from_numpy(W).cuda(), torch.from_numpy(omega).cuda()
    res = {}
    for rep in range(2):                                       # (first pass untimed)
        torch.cuda.synchronize(); t0 = time.perf_counter()
        codes, scale, zero, E = amd.offline_quantize(Wd, cfg.bits, cfg.group)
        torch.cuda.synchronize(); t1 = time.perf_counter()
        A, B, sigma, Ab, Bb = amd.offline_factors(E, r, Od, power_iters=2)
        t2 = time.perf_counter()
        res = {"quantize_ms": (t1 - t0) * 1e3, "factors_ms": (t2 - t1) * 1e3}
    t0 = time.perf_counter()
    q = compress.quantize_groupwise(W, cfg.bits, cfg.group)
    Eo = W - compress.dequantize(q, cfg.group)
    t1 = time.perf_counter()
    A0, B0, S0 = compress.residual_factors(Eo, r, method="randomized", seed=1, power_iters=2)
    t2 = time.perf_counter()
    same = bool((codes.cpu().numpy() == q["codes"]).all())
    print(json.dumps({
        "metric": "offline_matrices_per_s", "value": 1e3 / (res["quantize_ms"] + res["factors_ms"]), "unit": "matrices/s",
        "config": {"workload": cfg.name, "K": K, "N": N, "bits": cfg.bits, "group": cfg.group, "rank": r, "sketch": r + 8, "power_iters": 2},
        "device_ms": res, "oracle_ms": {"quantize_ms": (t1 - t0) * 1e3, "factors_ms": (t2 - t1) * 1e3},
        "codes_equal_oracle": same, "sigma_rel_diff_max": float(np.max(np.abs(sigma - S0) / S0)),
        "dtype": "f64", "data": "synthetic"}))


def sample_clocks(step, torch, seconds: float = 4.0) -> dict:
    """Shader clock (MHz) as `rocm-smi --showclocks` reads it while `step` runs back to back for a few
    seconds, and again after the device has been idle for a second (read-only queries from a thread)."""
    import re
    import subprocess
    import threading

    def read_sclk():
        try:
            r = subprocess.run(["/opt/rocm/bin/rocm-smi", "--showclocks", "--json"], capture_output=True, text=True, timeout=20)
            m = re.search(r"sclk clock speed:\W+(\d+)Mhz", r.stdout)
            return int(m.group(1)) if m else None
        except Exception:
            return None

    busy, stop = [], threading.Event()

    def poll():
        while not stop.is_set():
            v = read_sclk()
            if v is not None:
                busy.append(v)
            time.sleep(0.1)

    th = threading.Thread(target=poll, daemon=True)
    t0 = time.time()
    th.start()
    i = 0
    while time.time() - t0 < seconds:
        for _ in range(200):
            step(i)
            i += 1
        torch.cuda.synchronize()
    stop.set()
    th.join(timeout=30)
    time.sleep(1.0)
    idle = read_sclk()
    busy = sorted(busy[1:])               # (the first reading may predate the loop)
    return {"sclk_mhz_under_load_median": busy[len(busy) // 2] if busy else None,
            "sclk_mhz_under_load_min": busy[0] if busy else None, "sclk_mhz_under_load_max": busy[-1] if busy else None,
            "samples": len(busy), "sclk_mhz_after_the_loop": idle, "forwards": i, "source": "rocm-smi --showclocks"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="mixtral_decode_T64_b2")
    ap.add_argument("--layers", type=int, default=0, help="layer instances to rotate over (0: enough for > 2 GB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true", help="replay one captured HIP graph per layer instance instead of launching eagerly")
    ap.add_argument("--cpu-tokens", type=int, default=64, help="tokens whose expert FFN the CPU oracle evaluates")
    ap.add_argument("--staged", action="store_true",
                    help="also time one layer in staged residency (packed experts and factors copied from the "
                         "pinned pool per call, chosen by the router) and report it under 'staging'; "
                         "never part of 'value'")
    ap.add_argument("--staged-int3", action="store_true",
                    help="with --staged: the factor pairs are held at 3 bits (in the pinned pool, on the bus and on the device)")
    ap.add_argument("--int3-factors", action="store_true",
                    help="the timed layers hold their factor pairs at 3 bits, dequantized inside the kernels "
                         "(config.factors says so; the default run keeps fp16 pairs)")
    ap.add_argument("--calibrate", action="store_true",
                    help="also measure what this device sustains (streaming read of 3 GiB, pinned host->device "
                         "copy, f16 MFMA rate) and report it as roofline.peak_measured beside the published peaks")
    ap.add_argument("--clocks", action="store_true",
                    help="also run the forward in a loop of a few seconds and report the shader clock rocm-smi reads meanwhile "
                         "(and after the loop): the clock under this load is set by power")
    ap.add_argument("--calib-copy", action="store_true",
                    help="after the timed region run an elementwise kernel that reads and writes 256 MiB, "
                         "so that a counter run can scale FETCH_SIZE / WRITE_SIZE by a known transfer")
    ap.add_argument("--stack", type=int, default=0,
                    help="instead of the single layer: decode steps through a stack of this many layers whose experts "
                         "live in pinned host memory (a line of its own, metric stack_decode_tokens_per_s)")
    ap.add_argument("--slots", type=int, default=0, help="with --stack: device slots of the shared pool (0: every expert fits)")
    ap.add_argument("--no-prefetch", action="store_true", help="with --stack: no copies ahead for the next layer")
    ap.add_argument("--offline", action="store_true",
                    help="instead of the layer: time the offline pipeline (quantizer + residual factors) on one "
                         "W1-shaped matrix of the workload, device against the oracle on the host")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2512_17073_amd as amd
    from workload import configs, synth
    amd.lib()
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)

    cfg = configs.get(args.workload)
    if args.stack > 0:
        stack_bench(args, cfg)
        return
    if args.offline:
        offline_bench(args, cfg)
        return
    T = cfg.tokens
    t_setup = time.time()
    print(f"[bench] workload {cfg.name}: generating artefacts", file=sys.stderr, flush=True)
    wg, bias = synth.make_gate(cfg)
    n_all = cfg.n_experts + cfg.n_shared
    experts = [{m: synth.sample_artifacts(cfg, e, m) for m in (0, 1, 2)} for e in range(n_all)]
    layer = {"wg": wg, "bias": bias, "experts": experts}
    x_bits = synth.make_tokens(cfg)

    per_layer = sum(a["codes"].size * synth.expert_bits(cfg, e) / 8 for e, ex in enumerate(experts) for a in ex.values())
    n_layers = args.layers or max(2, min(16, int(np.ceil(2.2e9 / per_layer))))
    layers = []
    E = cfg.n_experts
    for i in range(n_layers):
        L = amd.Layer.from_config(cfg)
        L.set_gate(wg, bias)
        for e in range(n_all):
            src = experts[(e + i) % E] if e < E else experts[e]     # rotate the routed experts per instance
            for m in (0, 1, 2):
                a = src[m]
                if args.int3_factors and e < E and cfg.rank > 0:
                    L.set_expert(e, m, a["codes"], a["scale"], a["zero"], None, None, 0)
                    L.set_expert_factors_quantized(e, m, cfg.rank, *synth.sample_factor_codes(cfg, (e + i) % E, m))
                else:
                    L.set_expert(e, m, a["codes"], a["scale"], a["zero"], a["A"], a["B"])
        layers.append(L)
        print(f"[bench] layer instance {i + 1}/{n_layers} uploaded ({time.time() - t_setup:.0f}s)", file=sys.stderr, flush=True)

    x = amd.bf16_tensor(x_bits)
    out = torch.empty((T, cfg.hidden), dtype=torch.bfloat16, device="cuda")
    ws_bytes = layers[0].workspace_bytes(T)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream

    def step(i):
        layers[i % n_layers].forward_raw(x.data_ptr(), T, out.data_ptr(), ws.data_ptr(), ws_bytes, stream)

    for i in range(max(args.warmup, n_layers)):     # eager warm-up (every instance at least once)
        step(i)
    torch.cuda.synchronize()
    eager_step = step
    use_graph = args.graph
    if use_graph:
        # one captured forward per layer instance: the launch sequence is fixed (no allocation, no
        # host synchronisation, no memset inside moe_lrc_forward), so a replay is the same work
        graphs = []
        cap_stream = torch.cuda.Stream()
        with torch.cuda.stream(cap_stream):
            for L in layers:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=cap_stream):
                    L.forward_raw(x.data_ptr(), T, out.data_ptr(), ws.data_ptr(), ws_bytes,
                                  torch.cuda.current_stream().cuda_stream)
                graphs.append(g)
        torch.cuda.synchronize()
        ref_out = out.clone()
        eager_step(n_layers - 1)
        torch.cuda.synchronize()
        ref_out.copy_(out)
        graphs[n_layers - 1].replay()
        torch.cuda.synchronize()
        assert torch.equal(ref_out.view(torch.int16), out.view(torch.int16)), "graph replay differs from eager"

        def step(i):
            graphs[i % n_layers].replay()
        for i in range(args.warmup):
            step(i)
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # spread: the same steps again, each bracketed by its own pair of events on the launch stream
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(args.steps, 200))]
    for i, (a, b) in enumerate(ev):
        a.record()
        step(i)
        b.record()
    torch.cuda.synchronize()
    each = np.array([a.elapsed_time(b) for a, b in ev])
    spread = {"median_ms": round(float(np.median(each)), 5), "p10_ms": round(float(np.percentile(each, 10)), 5),
              "p90_ms": round(float(np.percentile(each, 90)), 5), "n": len(ev),
              "note": "per-step HIP events (each pair adds a few microseconds to a step)"}
    other = None
    if not use_graph and not args.staged:
        # the same steps replayed from one captured HIP graph per layer instance, for comparison
        try:
            graphs = []
            cap_stream = torch.cuda.Stream()
            with torch.cuda.stream(cap_stream):
                for L in layers:
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=cap_stream):
                        L.forward_raw(x.data_ptr(), T, out.data_ptr(), ws.data_ptr(), ws_bytes,
                                      torch.cuda.current_stream().cuda_stream)
                    graphs.append(g)
            torch.cuda.synchronize()
            for i in range(max(args.warmup, n_layers)):
                graphs[i % n_layers].replay()
            torch.cuda.synchronize()
            tg = time.perf_counter()
            for i in range(args.steps):
                graphs[i % n_layers].replay()
            torch.cuda.synchronize()
            other = {"launch": "hip_graph", "ms_per_step": round((time.perf_counter() - tg) / args.steps * 1e3, 5)}
            del graphs
        except Exception as exc:     # the graph leg is extra information: never fail the bench line on it
            other = {"launch": "hip_graph", "error": str(exc)[:200]}

    # per-kernel durations: the same calls again with HIP events recorded on the stream between kernels
    for L in layers:
        L.profile_enable(True)
    stage_ms = {}
    reps = max(20, min(args.steps, 100))
    for i in range(reps):
        eager_step(i)
        prof = layers[i % n_layers].profile_read()
        for k, v in prof.items():
            stage_ms.setdefault(k, []).append(v)
    for L in layers:
        L.profile_enable(False)
    stage_avg = {k: float(np.mean(v)) for k, v in stage_ms.items()}

    st = layers[0].stats()
    ab = algorithmic_bytes(cfg, T, st["active_experts"], st["comp_experts"], 0.5625 if args.int3_factors else 2.0)
    flops = algorithmic_flops(cfg, T)
    dom = "w13"
    # A stage is bracketed by two event records, and a record itself takes stream time: without shared
    # experts the "shared" stage has nothing between its two records, so its duration is that cost,
    # and the kernel's own duration is its stage less that.
    ev_pair = stage_avg["shared"] if cfg.n_shared == 0 else 0.0
    dom_ms = max(stage_avg[dom] - ev_pair, 1e-6)
    rows_per_expert = T * cfg.top_k / cfg.n_experts
    if rows_per_expert > 40:     # (the library takes the grouped-GEMM flavour for W1|W3 from there on)
        # many rows per expert: the fused W1|W3 launch is a grouped GEMM, bound by the matrix cores
        w13_flops = T * cfg.top_k * 2 * 2 * cfg.hidden * cfg.ffn + T * cfg.top_n * 2 * 2 * cfg.rank * cfg.ffn
        achieved = w13_flops / (dom_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": "packed W1|W3 product + SwiGLU (qgemm_tile_kernel<bits,true,2>: 128-row chunks)",
                    "achieved": round(achieved, 1), "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / MFMA_F16_PEAK_TFLOPS, 4), "traffic": None,
                    "flops_per_launch": int(w13_flops), "avg_ms": round(dom_ms, 5),
                    "avg_ms_incl_event_pair": round(stage_avg[dom], 5), "event_pair_ms": round(ev_pair, 5)}
    else:
        achieved = ab[dom] / (dom_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "packed W1|W3 product + SwiGLU (qgemm_decode_kernel<bits,true> at decode sizes)",
                    "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": counter_traffic(cfg.name + ("_int3_factors" if args.int3_factors else ""))[0],
                    "traffic_source": counter_traffic(cfg.name + ("_int3_factors" if args.int3_factors else ""))[1],
                    "bytes_per_launch": int(ab[dom]), "avg_ms": round(dom_ms, 5),
                    "avg_ms_incl_event_pair": round(stage_avg[dom], 5), "event_pair_ms": round(ev_pair, 5)}
    if args.calibrate:
        print("[bench] calibration: streaming read, pinned copy, MFMA rate", file=sys.stderr, flush=True)
        roofline["peak_measured"] = {
            "hbm_read_gbs": round(amd.calibrate(amd.CAL_HBM_READ, 3 << 30, 5), 1),
            "h2d_pinned_gbs": round(amd.calibrate(amd.CAL_H2D, 256 << 20, 5), 1),
            "mfma_f16_tflops": round(amd.calibrate(amd.CAL_MFMA_F16, 0, 5), 1),
            "mfma_f16_32x32x16_tflops": round(amd.calibrate(amd.CAL_MFMA_F16_32, 0, 5), 1),
            "ns_per_mfma_16x16x32_with_n_packed_fmas": {str(n): round(amd.calibrate(amd.CAL_MFMA_VALU, n, 5), 2) for n in (0, 2, 4, 8, 16)},
            # a loop shaped like a sub-step of the decode kernel (16 vector operations make two operands,
            # 2 MT MFMAs use them), four wavefronts per SIMD: ns of SIMD time per wavefront sub-step
            "decode_substep_ns": {f"mt{mt}_{name}": round(amd.calibrate(amd.CAL_SUBSTEP, mt + 16 * mode, 5), 2)
                                  for mt in (1, 2) for mode, name in ((0, "both"), (1, "mfma_only"), (2, "valu_only"))},
            "note": "moe_lrc_calibrate on this device: 3 GiB streaming read, 256 MiB pinned copy, register-only MFMA loops "
                    "(the last: two wavefronts per SIMD, every MFMA followed by n independent v_pk_fma_f16)"}
    path_kernel_ms = sum(stage_avg.values())
    result = {
        "metric": "MoE-layer tokens/s (one layer forward, weights resident in HBM)",
        "value": round(T / (ms_per_step * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": cfg.name, "tokens": T, "hidden": cfg.hidden, "ffn": cfg.ffn,
                   "experts": cfg.n_experts, "shared": cfg.n_shared, "top_k": cfg.top_k, "top_n": cfg.top_n,
                   "bits": cfg.bits, "group": cfg.group, "rank": cfg.rank, "layer_instances": n_layers,
                   "active_experts": st["active_experts"], "comp_experts": st["comp_experts"],
                   "factors": "int3" if args.int3_factors else "bf16",
                   "launch": "hip_graph" if use_graph else "eager"},
        "roofline": roofline,
        "spread": spread,
        "other_launch_mode": other,
        "whole_path": {"algorithmic_bytes": int(ab["total"]), "hbm_gbs_wall": round(ab["total"] / (ms_per_step * 1e-3) / 1e9, 1),
                       "hbm_frac_wall": round(ab["total"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                       "hbm_gbs_kernels": round(ab["total"] / (path_kernel_ms * 1e-3) / 1e9, 1),
                       "tflops": round(flops / (ms_per_step * 1e-3) / 1e12, 2),
                       "mfma_frac": round(flops / (ms_per_step * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4),
                       "stage_ms": {k: round(v, 5) for k, v in stage_avg.items()}},
    }
    staging = None
    if args.staged:
        print("[bench] staged residency: one layer, packed experts copied from the pinned pool per call", file=sys.stderr, flush=True)
        Ls = amd.Layer.from_config(cfg, residency=amd.STAGED)
        Ls.set_gate(wg, bias)
        for e in range(n_all):
            for m in (0, 1, 2):
                a = experts[e][m]
                if args.staged_int3 and e < cfg.n_experts and cfg.rank > 0:
                    Ls.set_expert(e, m, a["codes"], a["scale"], a["zero"], None, None, 0)
                    Ls.set_expert_factors_quantized(e, m, cfg.rank, *synth.sample_factor_codes(cfg, e, m))
                else:
                    Ls.set_expert(e, m, a["codes"], a["scale"], a["zero"], a["A"], a["B"])
        for _ in range(3):
            Ls.forward_raw(x.data_ptr(), T, out.data_ptr(), ws.data_ptr(), ws_bytes, stream)
        torch.cuda.synchronize()
        reps_s = 20
        copy_ms = []
        t0s = time.perf_counter()
        for _ in range(reps_s):
            Ls.forward_raw(x.data_ptr(), T, out.data_ptr(), ws.data_ptr(), ws_bytes, stream)
            torch.cuda.synchronize()
            copy_ms.append(Ls.stats()["stage_ms"])
        dts = (time.perf_counter() - t0s) / reps_s * 1e3
        sst = Ls.stats()
        moved = sst["bytes_codes"] + sst["bytes_meta"] + sst["bytes_factors"]
        staging = {"ms_per_step_incl_copies": round(dts, 4), "copy_ms": round(float(np.mean(copy_ms)), 4),
                   "bytes_per_step": int(moved), "copy_gbs": round(moved / (float(np.mean(copy_ms)) * 1e-3) / 1e9, 1),
                   "tokens_per_s_incl_copies": round(T / (dts * 1e-3), 1),
                   "experts_copied": int(sst["active_experts"]), "factor_sets_copied": int(sst["comp_experts"]),
                   "bytes_factors": int(sst["bytes_factors"]), "factors": "int3" if args.staged_int3 else "bf16"}
        Ls.close()
    if args.clocks:
        result["clocks"] = sample_clocks(eager_step, torch)
    if args.calib_copy:
        src = torch.zeros(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)        # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    if staging is not None:
        result["staging"] = staging
    if not args.no_cpu_baseline:
        print("[bench] timing the CPU oracle on a bounded sample", file=sys.stderr, flush=True)
        result["cpu_baseline"] = cpu_baseline(cfg, layer, x_bits, args.cpu_tokens)
    else:
        result["cpu_baseline"] = None
    for L in layers:
        L.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
