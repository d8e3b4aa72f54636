#!/usr/bin/env python3
"""Benchmark of the LONGER hot path on one MI355X.

A step is one ``longer_forward`` call (token merge -> cross-causal layer -> N self-causal
layers -> head) over one batch of the headline configuration C3 (256 users, L = 2000,
d = 128, bf16), inputs resident in HBM, rotating over three input buffers.  The line also
carries the KV-cache serving rate on configuration C5, the roofline figures of the
dominant kernel (the fused token-merge kernel, MFMA bound) measured with HIP events on
the launch stream, and the CPU oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-serving] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3        # MI355X dense fp32 MFMA (the fp32 configurations)
PEAK_HBM_GBS = 8000.0


def _oracle_flops(cfg, lens=None, B=None):
    # FLOP bookkeeping only (closed-form counts of Eq. 3 applied to the configuration)
    from oracle import longer_oracle as orc
    return orc.algorithmic_flops(cfg, lens, B=B), orc


def measured_traffic(cfg):
    """HBM bytes per launch of the merge kernel from the committed rocprofv3 counter summary
    (two --pmc runs, FETCH_SIZE and WRITE_SIZE, scaled by a copy kernel of known size); None
    when no summary exists for this workload."""
    path = os.path.join(ROOT, "profiles", "merge_%s_hbm_traffic.md" % cfg.name.lower())
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


def cpu_baseline(cfg, seconds_target=15.0):
    """Time the fp64 oracle on a bounded sample of users of the same workload."""
    import numpy as np
    import longer_synth as synth
    from oracle import longer_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    case = synth.make_case(cfg, users=1)
    t0 = time.perf_counter()
    orc.forward(case["cfg"], case["weights"], case["H"], case["G"], case["lens"])
    t1 = time.perf_counter() - t0
    users = int(max(1, min(2 * cfg.B, seconds_target / max(t1, 1e-3))))
    case = synth.make_case(cfg, users=users)
    t0 = time.perf_counter()
    orc.forward(case["cfg"], case["weights"], case["H"], case["G"], case["lens"])
    dt = time.perf_counter() - t0
    return {"value": users / dt, "unit": "user sequences/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d users of %s (L=%d, d=%d), one fp64 numpy pass, %.1f s" % (users, cfg.name, cfg.L, cfg.d, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="C3")
    ap.add_argument("--k-uniform", type=int, default=None,
                    help="sample this many of the k query slots uniformly from the older tokens instead of "
                         "taking the most recent k (Section 3.5.1); the default is the configuration's own")
    ap.add_argument("--q-learnable", action="store_true",
                    help="the k query slots hold learnable query tokens instead of sampled sequence tokens "
                         "(Section 3.5.1)")
    ap.add_argument("--from-inputs", type=int, default=0, metavar="D_E",
                    help="time longer_forward_from_inputs (input generation inside the merge kernel, Section 3.5.1) "
                         "on item embeddings of width D_E and time-difference features of width d - D_E, and "
                         "report the two-call sequence longer_input_generation + longer_forward beside it")
    ap.add_argument("--no-serving", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP graph replay measurement (profiler runs)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a kernel of known HBM traffic that "
                         "calibrates the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the forward path needs no collectives; users shard "
              "across GPUs with no exchange). --gpus %d is not supported." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import longer_synth as synth
    import paper_2505_04421_amd as lg

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    dev = "cuda:0"
    cfg = synth.CONFIGS[args.config]
    if args.k_uniform is not None:
        cfg = cfg.replace(k_uniform=args.k_uniform)
    if args.q_learnable:
        cfg = cfg.replace(q_learnable=True)
    case = synth.make_case(cfg)
    model = lg.DeviceModel(cfg, case["weights"], dev)
    B, L = cfg.B, cfg.L
    ws = model.workspace(B, L)
    lens_np = case["lens"]
    lens = None if lens_np is None else torch.from_numpy(lens_np.astype(np.int32)).to(dev)
    nbuf = 3
    Hs = [model.upload(case["H"])]
    for i in range(1, nbuf):        # distinct buffers so the input is not served from the last-level cache
        Hs.append(torch.roll(Hs[0], shifts=i, dims=0).contiguous() if lens is None else Hs[0].clone())
    G = model.upload(case["G"])
    Y = model.empty(B, cfg.n, cfg.d)
    logits = model.empty(B, dtype=torch.float32)

    def step(i):
        lg.longer_forward(model.ccfg, model.weights, Hs[i % nbuf], G, lens, B, L, Y, logits, ws)

    two_call_ms = None
    if args.from_inputs:
        d_e = args.from_inputs
        icase = synth.make_input_case(cfg.replace(ragged=False), d_e)
        mlp = {k: model.upload(v) for k, v in icase["mlp"].items()}
        iw = lg.CInputWeights(**{k: v.data_ptr() for k, v in mlp.items()})
        Es = [model.upload(icase["E"])]
        Ts = [model.upload(icase["tdiff"])]
        for i in range(1, nbuf):
            Es.append(torch.roll(Es[0], shifts=i, dims=0).contiguous())
            Ts.append(torch.roll(Ts[0], shifts=i, dims=0).contiguous())

        def two_calls(i):
            lg.longer_input_generation(model.ccfg, iw, Es[i % nbuf], Ts[i % nbuf], lens, B, L, d_e, Hs[i % nbuf], ws)
            lg.longer_forward(model.ccfg, model.weights, Hs[i % nbuf], G, lens, B, L, Y, logits, ws)

        for i in range(args.warmup):
            two_calls(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            two_calls(i)
        torch.cuda.synchronize()
        two_call_ms = (time.perf_counter() - t0) * 1e3 / args.steps

        def step(i):
            lg.longer_forward_from_inputs(model.ccfg, model.weights, iw, Es[i % nbuf], Ts[i % nbuf], d_e, G, lens, B, L,
                                          Y, logits, ws)

    if args.copy_probe_mib > 0:
        src = torch.empty(args.copy_probe_mib << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # Inside the timed region only the dominant launch is bracketed by the library's HIP events (on
    # the launch stream): the token merge, or the reduced stack where a narrow InnerTrans feeds a wide
    # main stack.  Every event pair adds a few microseconds of launch time to a step, so the other
    # stages are timed in a pass of their own below, outside the headline figure.
    # Which of the two it is comes from three untimed pilot steps with every stage timed.
    lg.longer_stage_timing(True)
    for i in range(3):
        step(i)
    torch.cuda.synchronize()
    pilot = lg.longer_stage_timing_read()
    dom = "attn" if pilot["attn"][0] > pilot["merge"][0] and pilot["attn"][1] == pilot["merge"][1] else "merge"
    lg.longer_stage_timing(True, stages=[dom])
    # markers between the steps (on the launch stream) give the per-step spread; the headline
    # figure is the wall-clock time of the whole timed region
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step(i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    dom_ms, dom_n = lg.longer_stage_timing_read()[dom]
    ms_per_step = dt * 1e3 / args.steps
    seq_per_s = B / (dt / args.steps)
    # per-stage breakdown: the same steps again with every launch group timed
    lg.longer_stage_timing(True)
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    stages = lg.longer_stage_timing_read()
    lg.longer_stage_timing(False)

    # the same steps replayed from HIP graphs (one per input buffer): the library allocates nothing and
    # only enqueues kernels, so a caller with a launch-bound batch size can capture it.  Reported
    # beside the eager figure, which stays the headline (the stage timers cannot run under capture)
    graph_ms = None
    try:
        if args.no_graph:
            raise RuntimeError("switched off with --no-graph")
        graphs = []
        for b in range(nbuf):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                step(b)
            graphs.append(g)
        for i in range(args.warmup):
            graphs[i % nbuf].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graphs[i % nbuf].replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        del graphs
    except Exception as e:        # reported, never fatal: the eager measurement above is complete
        print("bench.py: HIP graph replay not measured: %r" % (e,), file=sys.stderr)

    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_TFLOPS
    fl, _ = _oracle_flops(cfg, lens_np)
    if args.from_inputs:       # the MLP's two GEMMs on every valid raw token run inside the merge launch
        mlp_flop = 4.0 * cfg.d * cfg.ffn_mult * cfg.d * float(B * L if lens_np is None else lens_np.sum())
        fl = dict(fl, inner=fl["inner"] + mlp_flop, total=fl["total"] + mlp_flop)
    merge_ms, merge_n = (dom_ms, dom_n) if dom == "merge" else stages["merge"]
    merge_avg_ms = merge_ms / max(merge_n, 1)
    achieved = fl["inner"] / (merge_avg_ms * 1e-3) / 1e12
    total_tflops = fl["total"] / (ms_per_step * 1e-3) / 1e12
    # algorithmic HBM bytes of the merge kernel: each valid raw token read once, each merged token written once
    es = 2 if cfg.dtype == "bf16" else 4
    valid_tokens = float(B * L if lens_np is None else lens_np.sum())
    merged_tokens = float(B * cfg.T if lens_np is None else np.ceil(lens_np / cfg.K).sum())
    merge_bytes = valid_tokens * cfg.d_in * es + merged_tokens * cfg.d * 4
    roof_kernel = "block_kernel<MODE_MERGE> (fused gather + InnerTrans + pooling)"
    roof_ms, roof_flop = merge_avg_ms, fl["inner"]
    if dom == "attn":
        attn_ms, attn_n = dom_ms, max(dom_n, 1)
        # the reduced stack dominates (wide main stack over a narrow InnerTrans): price that launch instead.
        # Its work is everything but the InnerTrans and the cross layer's K/V projections (a launch of their own)
        Tu = np.full(B, cfg.T) if lens_np is None else np.ceil(lens_np / cfg.K)
        kv_flop = float(((cfg.m + Tu) * 4 * cfg.d * cfg.d).sum())
        roof_kernel = "block_kernel<MODE_STACK> (query side of the cross layer + all self layers)"
        roof_ms, roof_flop = attn_ms / attn_n, fl["total"] - fl["inner"] - kv_flop
        achieved = roof_flop / (roof_ms * 1e-3) / 1e12
    out = {
        "metric": "user sequences/s fwd at L=2000 bf16; candidates/s KV-cached; % MFMA peak",
        "value": seq_per_s, "unit": "user sequences/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
        "ms_per_step_hip_graph_replay": graph_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": "%s: longer_forward, B=%d users, L=%d, d=%d, m=%d, K=%d (T=%d), N_in=%d, k=%d, N=%d, heads=%d%s"
                   % (cfg.name, B, L, cfg.d, cfg.m, cfg.K, cfg.T, cfg.inner_layers, cfg.k_recent, cfg.n_self, cfg.heads,
                      (", merge by concatenation of raw width %d" % cfg.d_in if cfg.merge == "concat" else "")
                      + (", %d of the k query slots sampled uniformly" % cfg.k_uniform if cfg.k_uniform else "")
                      + (", learnable query tokens" if cfg.q_learnable else "")
                      + (", from raw inputs (item width %d + time-difference width %d, MLP inside the merge kernel)"
                         % (args.from_inputs, cfg.d - args.from_inputs) if args.from_inputs else "")),
                   "lens": "none" if lens_np is None else "uniform[%d,%d]" % (cfg.len_lo, cfg.len_hi)},
        "algorithmic_gflop_per_step": fl["total"] / 1e9,
        "mfma_peak_frac_whole_step": total_tflops / peak,
        "stage_ms_per_step": {k: v[0] / args.steps for k, v in stages.items() if v[1]},
        "roofline": {"kernel": roof_kernel, "bound": "mfma",
                     "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak,
                     "traffic": None if args.from_inputs else measured_traffic(cfg),
                     "avg_launch_ms": roof_ms, "algorithmic_gflop_per_launch": roof_flop / 1e9,
                     "merge_algorithmic_hbm_GBs": merge_bytes / (merge_avg_ms * 1e-3) / 1e9},
    }

    if two_call_ms is not None:
        out["input_generation_then_forward_ms_per_step"] = two_call_ms

    if not args.no_serving:
        c5 = synth.CONFIGS["C5"]
        case5 = synth.make_case(c5)
        m5 = lg.DeviceModel(c5, case5["weights"], dev)
        ws5 = m5.workspace(c5.B, c5.L, c5.C)
        H5, Gc5 = m5.upload(case5["H"]), m5.upload(case5["G_cand"])
        cache = m5.kv_cache(c5.B, c5.L)
        lg5 = m5.empty(c5.B, c5.C, dtype=torch.float32)
        for _ in range(2):
            lg.longer_kv_cache_build(m5.ccfg, m5.weights, H5, None, c5.B, c5.L, cache, ws5)
            lg.longer_score_candidates(m5.ccfg, m5.weights, cache, None, c5.B, c5.L, Gc5, c5.C, None, lg5, ws5)
        torch.cuda.synchronize()
        reps = max(3, args.steps // 3)
        t0 = time.perf_counter()
        for _ in range(reps):
            lg.longer_kv_cache_build(m5.ccfg, m5.weights, H5, None, c5.B, c5.L, cache, ws5)
        torch.cuda.synchronize()
        build_ms = (time.perf_counter() - t0) * 1e3 / reps
        t0 = time.perf_counter()
        for _ in range(reps):
            lg.longer_score_candidates(m5.ccfg, m5.weights, cache, None, c5.B, c5.L, Gc5, c5.C, None, lg5, ws5)
        torch.cuda.synchronize()
        score_ms = (time.perf_counter() - t0) * 1e3 / reps
        from oracle import longer_oracle as orc
        fl5 = orc.algorithmic_flops_score(c5, c5.T) * c5.B * c5.C
        out["serving"] = {"workload": "C5: %d users x %d candidates, L=%d, d=%d, K=%d (T=%d), k=%d, N=%d"
                          % (c5.B, c5.C, c5.L, c5.d, c5.K, c5.T, c5.k_recent, c5.n_self),
                          "candidates_per_s": c5.B * c5.C / (score_ms * 1e-3), "score_ms": score_ms,
                          "cache_build_ms": build_ms,
                          "candidates_per_s_incl_build": c5.B * c5.C / ((score_ms + build_ms) * 1e-3),
                          "score_mfma_peak_frac": fl5 / (score_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
        del m5, ws5, H5, Gc5, cache

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
