#!/usr/bin/env python3
"""Benchmark of the LONGER hot path on one MI355X.

A step is one ``longer_forward`` call (token merge -> cross-causal layer -> N self-causal
layers -> head) over one batch of the headline configuration C3 (256 users, L = 2000,
d = 128, bf16), inputs resident in HBM, rotating over three input buffers, parameters packed
once before the timed region (``longer_pack_weights``).  The line also carries

* ``roofline``: the dominant kernel (the fused token-merge kernel, MFMA bound) timed with HIP
  events on the launch stream, priced against the vendor peak and against the rate the matrix
  pipe sustains in an MFMA-only probe kernel run in the same process (``attainable``);
* ``microbench``: the library's instruction-rate probes (MFMA alone, VALU alone, both in the
  arrangements a kernel can choose between);
* ``all_configs``: the other forward configurations (C1, C2, C4), each with its own CPU-oracle leg
  (oracle rate on a sample of users and the GPU result's relative L2 error on that sample);
* ``serving``: KV-cache build and candidate scoring on configuration C5;
* ``cpu_baseline``: the fp64 oracle timed on a bounded sample of the headline workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-serving] [--no-cpu] [--no-others]
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

PROBE_MODES = {0: "mfma_only_two_waves_per_simd", 7: "mfma_only_one_wave_per_simd", 1: "valu_only",
               2: "mfma_phase_then_valu_phase_in_each_wave", 3: "mfma_waves_beside_valu_waves",
               9: "mfma_waves_beside_valu_waves_mfma_priority_raised",
               5: "each_mfma_followed_by_4_valu", 6: "each_mfma_followed_by_8_valu"}


def stored_traffic(cfg):
    """HBM bytes per launch of the merge kernel as stored in the committed rocprofv3 counter summary
    (two --pmc runs, FETCH_SIZE and WRITE_SIZE, scaled by a copy kernel of known size): (bytes, file)
    or (None, None).  Counters cannot be read inside this run; the figure is labelled as stored."""
    name = "merge_%s_hbm_traffic.md" % cfg.name.lower()
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1]), "profiles/" + name
    except OSError:
        pass
    return None, None


def cpu_oracle_leg(cfg, case_full, gpu_Y, seconds_target):
    """The CPU-baseline leg: the fp64 oracle on a bounded sample of the same workload's users (the
    first ones of the batch the GPU ran), timed; the GPU result of those users is compared with it."""
    import numpy as np
    from oracle import longer_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    w, H, G, lens = case_full["weights"], case_full["H"], case_full["G"], case_full["lens"]
    t0 = time.perf_counter()
    orc.forward(cfg, w, H[:1], G[:1], None if lens is None else lens[:1])
    t1 = time.perf_counter() - t0
    users = int(max(1, min(cfg.B, seconds_target / max(t1, 1e-3))))
    t0 = time.perf_counter()
    Y_ref, _ = orc.forward(cfg, w, H[:users], G[:users], None if lens is None else lens[:users])
    dt = time.perf_counter() - t0
    out = {"value": users / dt, "unit": "user sequences/s", "cores": int(cores), "kind": "oracle",
           "sample": "first %d users of %s (L=%d, d=%d), one fp64 numpy pass, %.1f s" % (users, cfg.name, cfg.L, cfg.d, dt)}
    if gpu_Y is not None:
        got = gpu_Y[:users].reshape(users, -1).astype(np.float64)
        ref = Y_ref.reshape(users, -1)
        den = np.linalg.norm(ref, axis=1)
        den = np.where(den > 0, den, 1.0)
        out["gpu_rel_l2_max_on_sample"] = float((np.linalg.norm(got - ref, axis=1) / den).max())
    return out


def probe_rates(lg, torch, modes=None, iters=2000):
    """Instruction-rate probes of the library: ns per iteration (per SIMD: the MFMA modes issue 16
    MFMAs per wave, the VALU modes 128 FMAs per wave) and the MFMA rate of mode 0."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.zeros(cus * 512, device="cuda")
    res = {}
    for mode, name in (modes or PROBE_MODES).items():
        lg.longer_probe_rate(mode, 50, cus, sink)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        lg.longer_probe_rate(mode, iters, cus, sink)
        e1.record()
        torch.cuda.synchronize()
        res[name] = e0.elapsed_time(e1) * 1e6 / iters
    # mode 0: 8 waves x 16 MFMAs x 32768 FLOP per workgroup and iteration
    attainable = cus * 8 * 16 * 32768.0 / (res[PROBE_MODES[0]] * 1e-9) / 1e12
    return {"compute_units": cus, "ns_per_iteration": res,
            "note": "one iteration per wave: 16 bf16 32x32x16 MFMAs and / or 128 fp32 FMAs; 512-thread workgroups, "
                    "one per compute unit"}, attainable


def run_merge_backward(lg, torch, cfg, case, steps):
    """Time longer_token_merge_backward (gradients of the token merge with recomputation) on the
    configuration's batch; inputs and the upstream gradient resident in HBM."""
    import numpy as np
    import longer_synth as synth
    from paper_2505_04421_amd import flops
    dev = "cuda:0"
    model = lg.DeviceModel(cfg, case["weights"], dev)
    B, L = cfg.B, cfg.L
    n_ws = lg.longer_backward_workspace_bytes(model.ccfg, B, L)
    nf = lg.longer_block_grad_floats(model.ccfg)
    if n_ws == 0 or nf == 0:
        return {"error": lg.longer_last_error()}
    ws = torch.empty(n_ws, dtype=torch.uint8, device=dev)
    H = model.upload(case["H"])
    lens = None if case["lens"] is None else torch.from_numpy(case["lens"].astype(np.int32)).to(dev)
    dM = torch.from_numpy(synth.draw_merge_gradient(cfg)).to(dev)
    dH = torch.empty(B, L, cfg.d_in, dtype=torch.float32, device=dev)
    grads = torch.empty(cfg.inner_layers * nf, dtype=torch.float32, device=dev)
    for _ in range(2):
        lg.longer_token_merge_backward(model.ccfg, model.inner, H, lens, B, L, dM, dH, grads, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        lg.longer_token_merge_backward(model.ccfg, model.inner, H, lens, B, L, dM, dH, grads, ws)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    work = flops.merge_backward_work(cfg, None if case["lens"] is None else case["lens"])
    grad_gflop = work["gradient_flops"] / 1e9     # d/d input and d/d parameter of every forward product
    return {"workload": "%s: longer_token_merge_backward, B=%d users, L=%d, InnerTrans width %d, %d block(s), K=%d"
                        % (cfg.name, B, L, cfg.d_in, cfg.inner_layers, cfg.K),
            "ms_per_step": ms, "steps": steps, "user_sequences_per_s": B / (ms * 1e-3),
            "gradient_gflop_per_step": grad_gflop,
            "recompute": "block inputs and every block's intermediates, from the raw tokens",
            "recompute_gflop_per_step": work["recompute_flops"] / 1e9,
            "mfma_peak_frac_gradient_flops": grad_gflop / 1e3 / (ms * 1e-3) / PEAK_BF16_TFLOPS,
            "roofline": {"bound": "hbm", "achieved": work["hbm_bytes"] / (ms * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                         "frac": work["hbm_bytes"] / (ms * 1e-3) / 1e9 / 8000.0,
                         "bytes_per_step": work["hbm_bytes"],
                         "traffic": 24.63e9 if cfg.name == "C3" else None,
                         "traffic_source": "profiles/merge_backward_c3_hbm_traffic.md" if cfg.name == "C3" else None,
                         "note": "chain of whole-batch kernels: every stored activation makes one trip through memory per use (tally in "
                                 "paper_2505_04421_amd/flops.py)"},
            "workspace_bytes": n_ws}


def run_forward_backward(lg, torch, cfg, case, steps):
    """Time longer_forward_backward: loss and every gradient of the whole model for one batch."""
    import numpy as np
    import longer_synth as synth
    from paper_2505_04421_amd import flops
    dev = "cuda:0"
    model = lg.DeviceModel(cfg, case["weights"], dev)
    B, L = cfg.B, cfg.L
    n_ws = lg.longer_forward_backward_workspace_bytes(model.ccfg, B, L)
    nf = lg.longer_model_grad_floats(model.ccfg)
    if n_ws == 0 or nf == 0:
        return {"error": lg.longer_last_error()}
    ws = torch.empty(n_ws, dtype=torch.uint8, device=dev)
    H, G = model.upload(case["H"]), model.upload(case["G"])
    lens = None if case["lens"] is None else torch.from_numpy(case["lens"].astype(np.int32)).to(dev)
    labels = torch.from_numpy(synth.draw_labels(cfg)).to(dev)
    dH = torch.empty(B, L, cfg.d_in, dtype=torch.float32, device=dev)
    dG = torch.empty(B, cfg.m, cfg.d, dtype=torch.float32, device=dev)
    grads = torch.empty(nf, dtype=torch.float32, device=dev)
    loss = torch.empty(4, dtype=torch.float32, device=dev)
    logits = torch.empty(B, dtype=torch.float32, device=dev)
    call = lambda: lg.longer_forward_backward(model.ccfg, model.weights, H, G, lens, B, L, labels, loss, logits, dH, dG, grads, ws)
    for _ in range(2):
        call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        call()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    fl = flops.forward_flops(cfg, None if case["lens"] is None else case["lens"])
    return {"workload": "%s: longer_forward_backward (loss of Eq. 2 and every gradient), B=%d users, L=%d" % (cfg.name, B, L),
            "ms_per_step": ms, "steps": steps, "user_sequences_per_s": B / (ms * 1e-3), "loss": float(loss[0].item()),
            "forward_plus_gradient_gflop_per_step": 3.0 * fl["total"] / 1e9,
            "mfma_peak_frac_forward_plus_gradient_flops": 3.0 * fl["total"] / 1e12 / (ms * 1e-3) / PEAK_BF16_TFLOPS,
            "workspace_bytes": n_ws}


def run_forward(lg, torch, synth, cfg, args, steps, warmup, want_graph=True):
    """Time longer_forward (or, with --from-inputs, longer_forward_from_inputs) on one configuration."""
    import numpy as np
    from paper_2505_04421_amd import flops
    dev = "cuda:0"
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

    iw = None
    two_call_ms = None
    from_inputs = args.from_inputs if cfg.name == args.config else 0
    if from_inputs:
        d_e = from_inputs
        icase = synth.make_input_case(cfg.replace(ragged=False), d_e)
        mlp = {k: model.upload(v) for k, v in icase["mlp"].items()}
        iw = lg.CInputWeights(**{k: v.data_ptr() for k, v in mlp.items()})
        Es = [model.upload(icase["E"])]
        Ts = [model.upload(icase["tdiff"])]
        for i in range(1, nbuf):
            Es.append(torch.roll(Es[0], shifts=i, dims=0).contiguous())
            Ts.append(torch.roll(Ts[0], shifts=i, dims=0).contiguous())
    # parameters packed once, outside the timed region (--pack-per-call: every call packs again)
    weights = model.weights if args.pack_per_call else model.pack(iw)

    def step(i):
        lg.longer_forward(model.ccfg, weights, Hs[i % nbuf], G, lens, B, L, Y, logits, ws)

    if from_inputs:
        def two_calls(i):
            lg.longer_input_generation(model.ccfg, iw, Es[i % nbuf], Ts[i % nbuf], lens, B, L, d_e, Hs[i % nbuf], ws)
            lg.longer_forward(model.ccfg, weights, Hs[i % nbuf], G, lens, B, L, Y, logits, ws)

        for i in range(warmup):
            two_calls(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            two_calls(i)
        torch.cuda.synchronize()
        two_call_ms = (time.perf_counter() - t0) * 1e3 / steps

        def step(i):
            lg.longer_forward_from_inputs(model.ccfg, weights, iw, Es[i % nbuf], Ts[i % nbuf], d_e, G, lens, B, L,
                                          Y, logits, ws)

    for i in range(warmup):
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
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        step(i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    dom_ms, dom_n = lg.longer_stage_timing_read()[dom]
    ms_per_step = dt * 1e3 / steps
    # per-stage breakdown: the same steps again with every launch group timed
    lg.longer_stage_timing(True)
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    stages = lg.longer_stage_timing_read()
    lg.longer_stage_timing(False)

    # the same steps replayed from HIP graphs (one per input buffer): the library allocates nothing and
    # only enqueues kernels, so a caller with a launch-bound batch size can capture it.  Reported
    # beside the eager figure, which stays the headline (the stage timers cannot run under capture)
    graph_ms = None
    if want_graph and not args.no_graph:
        try:
            graphs = []
            for b in range(nbuf):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    step(b)
                graphs.append(g)
            for i in range(warmup):
                graphs[i % nbuf].replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(steps):
                graphs[i % nbuf].replay()
            torch.cuda.synchronize()
            graph_ms = (time.perf_counter() - t0) * 1e3 / steps
            del graphs
        except Exception as e:        # reported, never fatal: the eager measurement above is complete
            print("bench.py: HIP graph replay not measured: %r" % (e,), file=sys.stderr)

    # one more step on buffer 0 whose result the CPU leg compares with the oracle
    step(0)
    torch.cuda.synchronize()
    Y_host = Y.float().cpu().numpy()

    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_TFLOPS
    fl = flops.forward_flops(cfg, lens_np)
    if from_inputs:       # the MLP's two GEMMs on every valid raw token run inside the merge launch
        mlp_flop = 4.0 * cfg.d * cfg.ffn_mult * cfg.d * float(B * L if lens_np is None else lens_np.sum())
        fl = dict(fl, inner=fl["inner"] + mlp_flop, total=fl["total"] + mlp_flop)
    merge_ms, merge_n = (dom_ms, dom_n) if dom == "merge" else stages["merge"]
    merge_avg_ms = merge_ms / max(merge_n, 1)
    # algorithmic HBM bytes of the merge kernel: each valid raw token read once, each merged token written once
    es = 2 if cfg.dtype == "bf16" else 4
    valid_tokens = float(B * L if lens_np is None else lens_np.sum())
    merged_tokens = float(B * cfg.T if lens_np is None else np.ceil(lens_np / cfg.K).sum())
    merge_bytes = valid_tokens * cfg.d_in * es + merged_tokens * cfg.d * 4
    roof_kernel = "block_kernel<MODE_MERGE> (fused gather + InnerTrans + pooling)"
    roof_ms, roof_flop = merge_avg_ms, fl["inner"]
    if dom == "attn":
        # the reduced stack dominates (wide main stack over a narrow InnerTrans): price that launch instead.
        # Its work is everything but the InnerTrans and the cross layer's K/V projections (a launch of their own)
        roof_kernel = "block_kernel<MODE_STACK> (query side of the cross layer + all self layers)"
        roof_ms, roof_flop = dom_ms / max(dom_n, 1), fl["total"] - fl["inner"] - fl["kv_cross"]
    achieved = roof_flop / (roof_ms * 1e-3) / 1e12
    total_tflops = fl["total"] / (ms_per_step * 1e-3) / 1e12
    res = {
        "cfg": cfg, "case": case, "Y_host": Y_host, "peak": peak,
        "ms_per_step": ms_per_step, "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
        "graph_ms": graph_ms, "seq_per_s": B / (dt / steps), "fl": fl, "total_tflops": total_tflops,
        "stage_ms": {k: v[0] / steps for k, v in stages.items() if v[1]},
        "roof_kernel": roof_kernel, "roof_ms": roof_ms, "roof_flop": roof_flop, "achieved": achieved,
        "merge_hbm_GBs": merge_bytes / (merge_avg_ms * 1e-3) / 1e9, "two_call_ms": two_call_ms,
        "lens": lens_np, "from_inputs": from_inputs,
    }
    del model, ws, Hs, G, Y, logits
    torch.cuda.empty_cache()
    return res


def workload_text(cfg, from_inputs=0):
    return ("%s: longer_forward, B=%d users, L=%d, d=%d, m=%d, K=%d (T=%d), N_in=%d, k=%d, N=%d, heads=%d%s"
            % (cfg.name, cfg.B, cfg.L, cfg.d, cfg.m, cfg.K, cfg.T, cfg.inner_layers, cfg.k_recent, cfg.n_self, cfg.heads,
               (", merge by concatenation of raw width %d" % cfg.d_in if cfg.merge == "concat" else "")
               + (", %d of the k query slots sampled uniformly" % cfg.k_uniform if cfg.k_uniform else "")
               + (", learnable query tokens" if cfg.q_learnable else "")
               + (", lens uniform[%d,%d]" % (cfg.len_lo, cfg.len_hi) if cfg.ragged else "")
               + (", from raw inputs (item width %d + time-difference width %d, MLP inside the merge kernel)"
                  % (from_inputs, cfg.d - from_inputs) if from_inputs else "")))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="C3")
    ap.add_argument("--k-recent", type=int, default=None,
                    help="number of sequence-side query slots k (the ablation's query number, Section 4.2.2); "
                         "above 128 - m the reduced stack runs one launch pair per layer")
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
    ap.add_argument("--pack-per-call", action="store_true",
                    help="let every call pack the parameters again instead of packing them once before the timed region")
    ap.add_argument("--no-serving", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the other forward configurations (all_configs)")
    ap.add_argument("--no-probe", action="store_true", help="skip the instruction-rate probes")
    ap.add_argument("--no-backward", action="store_true", help="skip the backward pass of the token merge")
    ap.add_argument("--merge-backward-only", action="store_true",
                    help="run nothing but the backward pass of the token merge (2 warm-up calls + --steps timed calls) and "
                         "print its block: for counter runs under rocprofv3")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP graph replay measurement (profiler runs)")
    ap.add_argument("--probe-all", action="store_true",
                    help="run every mode of the instruction-rate probe (include/longer.h lists them), print "
                         "{mode: ns per iteration} as one JSON line and exit")
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
    from paper_2505_04421_amd import flops

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    dev = "cuda:0"
    cfg = synth.CONFIGS[args.config]
    if args.k_recent is not None:
        cfg = cfg.replace(k_recent=args.k_recent)
    if args.k_uniform is not None:
        cfg = cfg.replace(k_uniform=args.k_uniform)
    if args.q_learnable:
        cfg = cfg.replace(q_learnable=True)

    if args.copy_probe_mib > 0:
        src = torch.empty(args.copy_probe_mib << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.merge_backward_only:
        print(json.dumps({"merge_backward": run_merge_backward(lg, torch, cfg, synth.make_case(cfg), args.steps)}))
        return

    if args.probe_all:
        modes = {0: PROBE_MODES[0]}
        modes.update({m: "mode_%d" % m for m in range(1, 22)})
        micro, attainable = probe_rates(lg, torch, modes, iters=4000)
        micro["attainable_mfma_tflops"] = attainable
        print(json.dumps(micro))
        return
    micro, attainable = (None, None)
    if not args.no_probe:
        micro, attainable = probe_rates(lg, torch)

    r = run_forward(lg, torch, synth, cfg, args, args.steps, args.warmup)
    traffic, traffic_src = (None, None) if r["from_inputs"] else stored_traffic(cfg)
    out = {
        "metric": "user sequences/s fwd at L=2000 bf16; candidates/s KV-cached; % MFMA peak",
        "value": r["seq_per_s"], "unit": "user sequences/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"], "ms_per_step_median": r["ms_per_step_median"], "ms_per_step_min": r["ms_per_step_min"],
        "ms_per_step_hip_graph_replay": r["graph_ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": workload_text(cfg, r["from_inputs"]),
                   "lens": "none" if r["lens"] is None else "uniform[%d,%d]" % (cfg.len_lo, cfg.len_hi),
                   "parameters": "packed on every call" if args.pack_per_call else "packed once (longer_pack_weights)"},
        "algorithmic_gflop_per_step": r["fl"]["total"] / 1e9,
        "mfma_peak_frac_whole_step": r["total_tflops"] / r["peak"],
        "mfma_attainable_frac_whole_step": None if not attainable or cfg.dtype != "bf16" else r["total_tflops"] / attainable,
        "stage_ms_per_step": r["stage_ms"],
        "roofline": {"kernel": r["roof_kernel"], "bound": "mfma",
                     "achieved": r["achieved"], "peak": r["peak"], "unit": "TFLOP/s",
                     "frac": r["achieved"] / r["peak"],
                     "attainable_tflops": attainable if cfg.dtype == "bf16" else None,
                     "frac_of_attainable": None if not attainable or cfg.dtype != "bf16" else r["achieved"] / attainable,
                     "traffic": traffic, "traffic_source": traffic_src,
                     "avg_launch_ms": r["roof_ms"], "algorithmic_gflop_per_launch": r["roof_flop"] / 1e9,
                     "merge_algorithmic_hbm_GBs": r["merge_hbm_GBs"]},
        "microbench": micro,
    }
    if r["two_call_ms"] is not None:
        out["input_generation_then_forward_ms_per_step"] = r["two_call_ms"]

    if not args.no_others and args.config == "C3":
        others = {}
        for name in ("C1", "C2", "C4"):
            oc = synth.CONFIGS[name]
            o = run_forward(lg, torch, synth, oc, args, max(10, args.steps // 2), max(3, args.warmup // 2), want_graph=True)
            entry = {"workload": workload_text(oc), "dtype": oc.dtype,
                     "ms_per_step": o["ms_per_step"], "ms_per_step_hip_graph_replay": o["graph_ms"],
                     "user_sequences_per_s": o["seq_per_s"],
                     "algorithmic_gflop_per_step": o["fl"]["total"] / 1e9,
                     "mfma_peak_frac_whole_step": o["total_tflops"] / o["peak"],
                     "stage_ms_per_step": o["stage_ms"],
                     "dominant_kernel": o["roof_kernel"], "dominant_kernel_ms": o["roof_ms"],
                     "dominant_kernel_frac": o["achieved"] / o["peak"]}
            if not args.no_cpu:
                entry["cpu_baseline"] = cpu_oracle_leg(oc, o["case"], o["Y_host"], 3.0)
            others[name] = entry
            del o
        out["all_configs"] = others

    if not args.no_serving:
        c5 = synth.CONFIGS["C5"]
        case5 = synth.make_case(c5)
        m5 = lg.DeviceModel(c5, case5["weights"], dev)
        w5 = m5.weights if args.pack_per_call else m5.pack()
        ws5 = m5.workspace(c5.B, c5.L)
        H5, Gc5 = m5.upload(case5["H"]), m5.upload(case5["G_cand"])
        cache = m5.kv_cache(c5.B, c5.L)
        lg5 = m5.empty(c5.B, c5.C, dtype=torch.float32)
        for _ in range(2):
            lg.longer_kv_cache_build(m5.ccfg, w5, H5, None, c5.B, c5.L, cache, ws5)
            lg.longer_score_candidates(m5.ccfg, w5, cache, None, c5.B, c5.L, Gc5, c5.C, None, lg5, ws5)
        torch.cuda.synchronize()
        reps = max(3, args.steps // 3)
        t0 = time.perf_counter()
        for _ in range(reps):
            lg.longer_kv_cache_build(m5.ccfg, w5, H5, None, c5.B, c5.L, cache, ws5)
        torch.cuda.synchronize()
        build_ms = (time.perf_counter() - t0) * 1e3 / reps
        t0 = time.perf_counter()
        for _ in range(reps):
            lg.longer_score_candidates(m5.ccfg, w5, cache, None, c5.B, c5.L, Gc5, c5.C, None, lg5, ws5)
        torch.cuda.synchronize()
        score_ms = (time.perf_counter() - t0) * 1e3 / reps
        fl5 = flops.score_flops(c5, c5.T) * c5.B * c5.C
        score_tflops = fl5 / (score_ms * 1e-3) / 1e12
        out["serving"] = {"workload": "C5: %d users x %d candidates, L=%d, d=%d, K=%d (T=%d), k=%d, N=%d"
                          % (c5.B, c5.C, c5.L, c5.d, c5.K, c5.T, c5.k_recent, c5.n_self),
                          "candidates_per_s": c5.B * c5.C / (score_ms * 1e-3), "score_ms": score_ms,
                          "cache_build_ms": build_ms,
                          "candidates_per_s_incl_build": c5.B * c5.C / ((score_ms + build_ms) * 1e-3),
                          "score_mfma_peak_frac": score_tflops / PEAK_BF16_TFLOPS,
                          "score_mfma_attainable_frac": None if not attainable else score_tflops / attainable}
        del m5, ws5, H5, Gc5, cache

    if not args.no_backward and cfg.dtype == "bf16" and not r["from_inputs"]:
        out["merge_backward"] = run_merge_backward(lg, torch, cfg, r["case"], max(3, args.steps // 5))
        out["forward_backward"] = run_forward_backward(lg, torch, cfg, r["case"], max(3, args.steps // 5))

    out["cpu_baseline"] = None if args.no_cpu else cpu_oracle_leg(cfg, r["case"], None if r["from_inputs"] else r["Y_host"], 15.0)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
