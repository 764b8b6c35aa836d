"""Benchmark of the MoTE-layer forward on one MI355X.

One step = one pass of the whole hot path (router + Q_a(x), dispatch, routed gate-up GEMM
with SwiGLU, Q_a(h), routed down GEMM, shared FFN, combine) over one batch of synthetic
tokens whose inputs and weights already sit in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload headline|c2|c3|c5|c4_T<T>_n<n>|<c2|c3|c5|p05|p15|p3>_T<T>|ste_<shape>]

Without --workload the timed workload is the prefill shape (c3: d=2048, F=11008, E=16, top-2,
T=8192); the decode shapes (c4) and the skewed shape (c5) are measured after it and ride along in
the same JSON line under "decode" and "c5".
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_HBM_GBS = 8000.0
PEAK_I8_TOPS = 5000.0
PEAK_BF16_TFLOPS = 2500.0


def pick_config(name: str):
    import workloads as W
    if name == "c1":
        return W.C1
    if name == "c2":
        return W.C2
    if name == "c3":
        return W.C3
    if "_T" in name and name.split("_T")[0] in ("c2", "c3", "c5", "p05", "p15", "p3"):   # a shape at another batch size
        base, n_tok = name.split("_T")
        cfg = pick_config(base)
        return cfg.with_tokens(int(n_tok), name=f"{cfg.name.replace('_prefill', '')}_T{int(n_tok)}")
    if name == "c5":
        return W.C5
    if name in ("p05", "p15", "p3"):   # the paper's own layer: E = 4, top-1, T = 2048
        return {"p05": W.P05, "p15": W.P15, "p3": W.P3}[name]
    if name.startswith("c4"):
        n_tok, n_distinct = 64, 16
        for part in name.split("_")[1:]:
            if part[0] == "T":
                n_tok = int(part[1:])
            elif part[0] == "n":
                n_distinct = int(part[1:])
        return W.decode_config(n_tok, n_distinct)
    raise SystemExit(f"unknown workload {name}")


def stage_work(cfg, counts, shared_bits=0):
    """Algorithmic work per launch of each stage: (bound, amount, unit, peak).  shared_bits: 0 for the
    bf16 shared expert, 8 / 4 for the RTN-quantised one (bytes per weight = bits / 8, plus 4-byte row scales)."""
    T, d, F, E, k = cfg.n_tokens, cfg.d_model, cfg.d_ff, cfg.n_experts, cfg.top_k
    R = T * k
    n_active = int((counts > 0).sum())
    decode = cfg.name.startswith("c4")
    w = {}
    if decode:  # HBM-bound: packed expert bytes actually touched (+ their activations)
        w["routed_gate_up"] = ("hbm", n_active * 2 * d * F / 4 + R * d + R * F * 2, "GB/s", PEAK_HBM_GBS)
        w["routed_down"] = ("hbm", n_active * d * F / 4 + R * F + R * d * 4, "GB/s", PEAK_HBM_GBS)
        wb = (shared_bits or 16) / 8.0
        sc = 4 if shared_bits else 0
        w["shared_gate_up"] = ("hbm", 2 * d * F * wb + 2 * F * sc + T * d * 2 + T * F * 2, "GB/s", PEAK_HBM_GBS)
        w["shared_down"] = ("hbm", d * F * wb + d * sc + T * F * 2 + T * d * 4, "GB/s", PEAK_HBM_GBS)
    else:       # MFMA-bound
        w["routed_gate_up"] = ("mfma", 2.0 * R * 2 * d * F, "TFLOP/s", PEAK_I8_TOPS)
        w["routed_down"] = ("mfma", 2.0 * R * d * F, "TFLOP/s", PEAK_I8_TOPS)
        w["shared_gate_up"] = ("mfma", 2.0 * T * 2 * d * F, "TFLOP/s", PEAK_BF16_TFLOPS)
        w["shared_down"] = ("mfma", 2.0 * T * d * F, "TFLOP/s", PEAK_BF16_TFLOPS)
    w["router_quant"] = ("hbm", T * d * 2 + T * d + d * E * 2, "GB/s", PEAK_HBM_GBS)
    w["quant_h"] = ("hbm", R * F * 3, "GB/s", PEAK_HBM_GBS)
    w["combine"] = ("hbm", T * d * 4 + R * d * 4 + T * d * 2, "GB/s", PEAK_HBM_GBS)
    w["dispatch"] = ("hbm", R * 4 * 3, "GB/s", PEAK_HBM_GBS)
    return w


def read_traffic(stage: str, workload: str):
    """HBM bytes per launch of `stage`, from the committed rocprofv3 --pmc summary, if any."""
    path = os.path.join(ROOT, "profiles", f"pmc_traffic_{stage}_{workload}.txt")
    if not os.path.exists(path):
        return None
    with open(path) as fh:
        for line in fh:
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    return None


def measure_ste(workload: str, steps, warmup):
    """Straight-through gradients (Section 3.2) of the routed gate matrices of a configuration:
    R = T*k gradient rows of length d_ff, grouped by expert with seeded multinomial counts."""
    import numpy as np
    import torch
    import paper_2506_14435_amd as M
    cfg = pick_config(workload[4:])
    R, N, K, E = cfg.n_tokens * cfg.top_k, cfg.d_ff, cfg.d_model, cfg.n_experts
    steps = steps or 10
    warmup = 3 if warmup is None else warmup
    g = torch.Generator(device="cuda").manual_seed(cfg.seed)
    counts = np.random.default_rng(cfg.seed).multinomial(R, np.full(E, 1.0 / E))
    offsets = np.concatenate([[0], np.cumsum(counts)])
    packed, alpha = [], []
    for _ in range(E):
        w = torch.randn(N, K, generator=g, device="cuda") * 0.02
        pk, a = M.mote_pack_ternary(w)
        packed.append(pk.view(torch.uint8).reshape(-1))
        alpha.append(a)
    packed, alpha = torch.cat(packed), torch.cat(alpha)
    dy = torch.randn(R, N, generator=g, device="cuda").to(torch.bfloat16)
    q = torch.randint(-127, 128, (R, K), generator=g, device="cuda", dtype=torch.int8)
    beta = torch.rand(R, generator=g, device="cuda") * 4 + 1
    lib = M.load_library()
    ws = torch.empty(lib.mote_ste_backward_workspace_bytes(R, N, K, E), dtype=torch.uint8, device="cuda")
    run = lambda: M.mote_ste_linear_backward(dy, offsets, packed, alpha, 1, q, beta, N, K, workspace=ws)
    t0 = time.time()
    while time.time() - t0 < 0.1:
        run()
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(steps):
        run()
    end.record()
    torch.cuda.synchronize()
    ms = start.elapsed_time(end) / steps
    flops = 4.0 * R * N * K
    ach = flops / (ms * 1e-3) / 1e12
    return {"metric": "ste_backward_rows_per_s", "value": round(R / (ms * 1e-3), 1), "unit": "rows/s", "n_gpus": 1,
            "steps": steps, "warmup": warmup, "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"ste_backward_{cfg.name}", "rows": R, "n_out": N, "n_in": K, "n_experts": E},
            "roofline": {"kernel": "shared_gemm_kernel (dX and dW contractions)", "bound": "mfma", "achieved": round(ach, 2),
                         "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / PEAK_BF16_TFLOPS, 4), "traffic": None}}


def cpu_baseline(cfg, budget_s=20.0):
    """The CPU oracle as it stands, timed on the host cores on a bounded token sample."""
    import numpy as np
    from tests.mote_testlib import OracleProblem
    op = OracleProblem(cfg)
    n_probe = min(cfg.n_tokens, 32)
    stride = max(cfg.n_tokens // n_probe, 1)
    tokens = np.arange(0, cfg.n_tokens, stride)[:n_probe]
    t0 = time.perf_counter()
    ref = op.forward(tokens=tokens)          # also ternarises the touched experts (not timed below)
    t_probe = time.perf_counter() - t0
    needed = np.unique(ref["idx"])
    for e in needed:
        op.experts(int(e))
    t0 = time.perf_counter()
    op.forward(tokens=tokens)
    t_small = time.perf_counter() - t0
    # The probe's time is mostly fixed cost (router on all tokens), so the sample is grown until a
    # pass takes at least half the budget or covers the whole workload.
    n = len(tokens)
    while t_probe < 120 and n < cfg.n_tokens and t_small < 0.5 * budget_s:
        n = int(min(cfg.n_tokens, max(2 * n, n * 0.8 * budget_s / max(t_small, 1e-3))))
        stride = max(cfg.n_tokens // n, 1)
        tokens = np.arange(0, cfg.n_tokens, stride)[:n]
        n = len(tokens)
        t0 = time.perf_counter()
        op.forward(tokens=tokens)
        t_small = time.perf_counter() - t0
    reps = 1
    if t_small < 0.5 * budget_s and n == cfg.n_tokens:     # whole workload fits: repeat it to fill the budget
        reps = int(min(50, max(1, 0.5 * budget_s / t_small)))
        t0 = time.perf_counter()
        for _ in range(reps):
            op.forward(tokens=tokens)
        t_small = (time.perf_counter() - t0) / reps
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": n / t_small, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{n} of {cfg.n_tokens} tokens (every {max(cfg.n_tokens // n, 1)}th), router on all tokens, "
                      f"experts already ternarised; {reps} pass(es) of {t_small:.2f} s"}


def measure(workload: str, steps, warmup, graph: bool, calib_copy_mib: int, stage_steps_max: int = 200,
            shared_bits: int = 0):
    """Times one workload: whole forwards, then per-stage durations.  Returns the result dict
    (without cpu_baseline) and the config."""
    import torch
    import paper_2506_14435_amd as M
    from tests.mote_testlib import GpuProblem

    cfg = pick_config(workload)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev).manual_seed(cfg.seed + 977)

    def latent(e, m):  # fp32 latents drawn on the device; ternarised by mote_pack_ternary
        shape = (cfg.d_ff, cfg.d_model) if m < 2 else (cfg.d_model, cfg.d_ff)
        return torch.randn(*shape, device=dev, generator=gen) * cfg.sigma_latent

    gp = GpuProblem(cfg, dev, latent_source=latent if cfg.n_experts * cfg.d_model * cfg.d_ff > 5e7 else None,
                    shared_bits=shared_bits)
    out = torch.empty_like(gp.x)
    ws = gp.layer.workspace(cfg.n_tokens)
    taps = M.alloc_taps(gp.layer, cfg.n_tokens, ("counts",))

    # Decode shapes are HBM-bound and touch less than the 256 MB memory-side cache: rotate
    # over distinct copies of all weights so that every step really streams from HBM.
    layers = [gp.layer]
    keep = []
    if workload.startswith("c4"):
        step_bytes = sum(t.numel() * t.element_size() for t in (*gp.shared, *gp.wt))
        n_copies = max(2, int(-(-(1536 << 20) // step_bytes)))
        for _ in range(n_copies - 1):
            sh = tuple(t.clone() for t in gp.shared)
            wt = [t.clone() for t in gp.wt]
            keep.append((sh, wt))
            layers.append(M.MoteLayer(gp.w_router, *sh, *wt, gp.alpha, cfg.top_k, router_bias=gp.bias,
                                      shared_bits=shared_bits, shared_scales=gp.shared_scales))
    n_layers = len(layers)

    M.mote_layer_forward(gp.layer, gp.x, out=out, workspace=ws, taps=taps)
    torch.cuda.synchronize()
    counts = taps["counts"].cpu().numpy()

    if calib_copy_mib > 0:
        src = torch.full((calib_copy_mib << 20,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            M.mote_calib_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    # One step = one forward, launched eagerly.  --graph replays a HIP graph captured from the
    # same call instead (same kernels, one launch); measured 3-15 % slower than eager launches
    # on every workload, because the gaps between graph nodes exceed those between queued kernels.
    launch = "eager"
    fns = [lambda l=l: M.mote_layer_forward(l, gp.x, out=out, workspace=ws) for l in layers]
    if graph:
        try:
            graphs = [M.ForwardGraph(l, gp.x, out, ws) for l in layers]
            fns = [g.replay for g in graphs]
            launch = "hip_graph"
        except Exception as exc:  # noqa: BLE001
            print(f"bench.py: graph capture failed ({exc}); launching eagerly", file=sys.stderr)
    # Conditioning: an idle GPU needs some 50 ms of continuous work to reach its steady clocks (C2
    # reads 0.19 ms per forward right after start-up and 0.16 ms from then on), so forwards are
    # run for 0.1 s before the W warm-up steps, whatever W is; the probe also sizes the defaults.
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    conditioning = 0
    while conditioning < 5 or (time.perf_counter() - t0 < 0.1 and conditioning < 5000):
        for i in range(5):
            fns[(conditioning + i) % n_layers]()
        conditioning += 5
        torch.cuda.synchronize()
    probe_ms = (time.perf_counter() - t0) * 1e3 / conditioning
    if warmup is None:
        warmup = int(min(1000, max(10, 100.0 / probe_ms)))
    if steps is None:
        steps = int(min(2000, max(50, 300.0 / probe_ms)))
    for i in range(warmup):
        fns[i % n_layers]()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        fns[i % n_layers]()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / steps
    tokens_per_s = cfg.n_tokens * steps / elapsed

    # per-kernel durations: HIP events recorded by the library on the launch stream
    M.mote_stage_timing(True)
    acc = {n: 0.0 for n in M.STAGE_NAMES}
    stage_steps = min(steps, stage_steps_max)
    for i in range(stage_steps):
        M.mote_layer_forward(layers[i % n_layers], gp.x, out=out, workspace=ws)
        for n, v in M.mote_stage_times().items():
            acc[n] += v
    M.mote_stage_timing(False)
    stage_raw_ms = {n: v / stage_steps for n, v in acc.items()}
    # A stage time is event record to event record: the stage's kernel plus what two consecutive
    # event records read with nothing between them (about 5 us on this machine, measured here on
    # the same stream).  The kernel's launch duration is the stage time less that overhead; it is
    # what rocprofv3 --kernel-trace reports for the kernel (profiles/kernel_stats_*).
    torch.cuda.synchronize()
    event_pair_ms = min(M.mote_event_pair_overhead() for _ in range(3))
    stage_ms = {n: max(v - event_pair_ms, 0.1 * v) for n, v in stage_raw_ms.items()}

    work = stage_work(cfg, counts, shared_bits)
    candidates = ("routed_gate_up", "routed_down", "shared_gate_up", "shared_down")
    dom = max(candidates, key=lambda n: stage_ms[n])
    stages = {}
    for n in M.STAGE_NAMES:
        bound, amount, unit, peak = work[n]
        ach = amount / (stage_ms[n] * 1e-3) / (1e9 if unit == "GB/s" else 1e12)
        stages[n] = {"ms": round(stage_ms[n], 5), "event_to_event_ms": round(stage_raw_ms[n], 5), "bound": bound,
                     "achieved": round(ach, 2), "unit": unit, "frac": round(ach / peak, 4)}
    bound, amount, unit, peak = work[dom]
    achieved = amount / (stage_ms[dom] * 1e-3) / (1e9 if unit == "GB/s" else 1e12)
    roofline = {"kernel": dom, "bound": bound, "achieved": round(achieved, 2), "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4), "traffic": read_traffic(dom, workload),
                "avg_launch_ms": round(stage_ms[dom], 5), "event_to_event_ms": round(stage_raw_ms[dom], 5),
                "event_pair_overhead_ms": round(event_pair_ms, 5)}
    # The two figures the metric names: the routed GEMM pair against the int8 MFMA peak (large
    # batches) or its packed-weight stream against the HBM peak (decode).
    pair_ms = stage_ms["routed_gate_up"] + stage_ms["routed_down"]
    pair_amount = work["routed_gate_up"][1] + work["routed_down"][1]
    pair_peak = work["routed_gate_up"][3]
    pair_div = 1e9 if work["routed_gate_up"][2] == "GB/s" else 1e12
    routed_pair = {"bound": work["routed_gate_up"][0], "ms": round(pair_ms, 5),
                   "achieved": round(pair_amount / (pair_ms * 1e-3) / pair_div, 2),
                   "unit": work["routed_gate_up"][2], "peak": pair_peak,
                   "frac": round(pair_amount / (pair_ms * 1e-3) / pair_div / pair_peak, 4)}

    result = {
        "metric": "MoTE-layer tokens/s", "value": round(tokens_per_s, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "i8+bf16" if not shared_bits else f"i8+bf16 (shared expert weights int{shared_bits})",
        "data": "synthetic",
        "config": {"workload": cfg.name, "d_model": cfg.d_model, "d_ff": cfg.d_ff, "n_experts": cfg.n_experts,
                   "top_k": cfg.top_k, "tokens": cfg.n_tokens, "expert_loads": counts.tolist(),
                   "weight_copies_rotated": n_layers, "launch": launch, "conditioning_forwards": conditioning,
                   "shared_expert_bits": shared_bits or 16},
        "roofline": roofline,
        "routed_gemms": routed_pair,
        "stages": stages,
    }
    del fns, layers, keep, gp, out, ws, taps
    torch.cuda.empty_cache()
    return result, cfg


def brief(result):
    """The part of a workload's result that rides along in the headline line."""
    keep = ("value", "unit", "steps", "warmup", "ms_per_step", "roofline", "routed_gemms")
    b = {k: result[k] for k in keep}
    b["workload"] = result["config"]["workload"]
    b["tokens"] = result["config"]["tokens"]
    b["expert_loads"] = result["config"]["expert_loads"]
    b["weight_copies_rotated"] = result["config"]["weight_copies_rotated"]
    b["stage_frac"] = {n: s["frac"] for n, s in result["stages"].items()
                       if n in ("routed_gate_up", "routed_down", "shared_gate_up", "shared_down")}
    b["stage_ms"] = {n: s["ms"] for n, s in result["stages"].items()}
    return b


# decode batches of the benchmark definition: T tokens touching n distinct experts
DECODE_POINTS = ((1, 2), (4, 4), (16, 8), (64, 16))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed forwards (default: about 0.3 s of them, between 50 and 2000)")
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed forwards before the timed ones (default: about 0.1 s of them, between 10 and 1000)")
    ap.add_argument("--workload", default="headline",
                    help="headline (default): the prefill shape c3 as the timed workload, with the decode shapes "
                         "c4 (T = 1, 4, 16, 64) and the skewed shape c5 measured after it and carried in the same "
                         "JSON line; or one of c1 | c2 | c3 | c5 | c4_T<T>_n<n> | p05 | p15 | p3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="replay a captured HIP graph of the forward instead of launching its kernels eagerly")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run the library's plain copy kernel on this many MiB (three launches): the "
                         "known-size transfer that scales rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings")
    ap.add_argument("--shared-bits", type=int, default=0, choices=(0, 8, 4),
                    help="0: bf16 shared expert (the paper's layer); 8 / 4: RTN-quantised shared expert (Section 4.3)")
    ap.add_argument("--tune", action="append", default=[], metavar="KNOB=VALUE",
                    help="experiment knob of the library (mote_tuning_set), e.g. --tune no_fork=1")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU; the layer is token-parallel and shards without "
              "communication, so no multi-GPU figure is produced (run with --gpus 1).", file=sys.stderr)
        raise SystemExit(2)

    import torch
    import paper_2506_14435_amd as M

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU; there is no CPU fallback")
    M.load_library()
    for kv in args.tune:
        name, _, val = kv.partition("=")
        M.mote_tuning_set(name, int(val))
    if args.workload.startswith("ste_"):   # e.g. ste_c3: the training-side gradient GEMMs, a line of its own
        print(json.dumps(measure_ste(args.workload, args.steps, args.warmup)))
        return
    headline = args.workload == "headline"
    main_workload = "c3" if headline else args.workload
    result, cfg = measure(main_workload, args.steps, args.warmup, args.graph, args.calib_copy_mib,
                          shared_bits=args.shared_bits)
    if headline:
        # The metric names three figures: tokens/s of the layer, the decode shapes' packed-weight
        # stream against the HBM peak and the prefill shape's routed GEMMs against the int8 MFMA
        # peak.  The timed workload of this line is the prefill shape; the other shapes are
        # measured after it with their own default step counts.
        result["decode"] = [brief(measure(f"c4_T{t}_n{n}", None, None, args.graph, 0)[0]) for t, n in DECODE_POINTS]
        result["c5"] = brief(measure("c5", None, None, args.graph, 0)[0])
        # Section 4.3: the shared expert quantised to INT8 / INT4 (its bf16 weights are most of a small
        # decode step's bytes)
        result["decode_rtn_shared"] = [
            dict(brief(measure(f"c4_T{t}_n{n}", None, None, args.graph, 0, shared_bits=b)[0]), shared_expert_bits=b)
            for b in (8, 4) for t, n in ((1, 2), (4, 4), (64, 16))]
        d64 = result["decode"][-1]
        result["targets"] = {
            "prefill_routed_i8_frac": result["routed_gemms"]["frac"], "prefill_target": 0.5,
            "decode_routed_hbm_frac_T64": d64["routed_gemms"]["frac"],
            "decode_routed_gate_up_hbm_frac_T64": d64["stage_frac"]["routed_gate_up"],
            "decode_routed_down_hbm_frac_T64": d64["stage_frac"]["routed_down"], "decode_target": 0.7}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
