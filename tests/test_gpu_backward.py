"""GPU parity of longer_token_merge_backward (backward pass of the token merge with recomputation,
mixed precision) against the fp64 oracle ``oracle.longer_oracle_grad.token_merge_backward``.

Tolerance.  The oracle differentiates in fp64; the GPU pass rounds every GEMM operand and every stored
activation / activation gradient to bf16 (2^-9 relative, about 1.1e-3 rms per rounding).  A gradient
passes through about a dozen such roundings per InnerTrans block, independent of each other, so the
expected relative L2 error is sqrt(12) x 1.1e-3 = 4e-3 per block and 6e-3 over two; the bar is 2e-2
for the gradient of the raw tokens (per user) and for every parameter.  With ReLU the derivative is
a step: a hidden unit whose pre-activation lies within the forward pass's own rounding error of zero
(a few in a thousand) takes the other branch than in fp64, which is a difference of that unit's whole
contribution, not of a rounding; the bar there is 1e-1 (observed: 2e-2 at width 64, up to 7e-2 for a
parameter vector at width 32, where a block has only 64-128 hidden units).  The bar holds for the cases
drawn here; it is not a bound: over 60 further seeds of the random configurations below, five ReLU
configurations whose reduced stack has only 10-132 rows in the whole batch came out at 1.0e-1 to 1.6e-1 for
one parameter vector (a bias or LayerNorm shift of the main stack), and the same five configurations with
GELU at 1.2e-2 to 1.5e-2."""
import sys

import numpy as np
import pytest
import torch

import longer_synth as synth
from oracle import longer_oracle_grad as org

pytestmark = pytest.mark.gpu

TOL = 2e-2
TOL_RELU = 1e-1
PARAMS = org.PARAMS


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _rel(a, b):
    den = float(np.linalg.norm(b))
    return float(np.linalg.norm(a - b)) / (den if den > 0 else 1.0)


def _run_gpu(case, dM, ws_fill=None):
    import paper_2505_04421_amd as lg
    from gpu_util import guarded_empty
    cfg = case["cfg"]
    model = lg.DeviceModel(cfg, case["weights"])
    dev = model.device
    B, L = cfg.B, cfg.L
    H = model.upload(case["H"])
    lens = None if case["lens"] is None else torch.from_numpy(case["lens"].astype(np.int32)).to(dev)
    n_ws = lg.longer_backward_workspace_bytes(model.ccfg, B, L)
    nf = lg.longer_block_grad_floats(model.ccfg)
    assert n_ws > 0 and nf > 0, lg.longer_last_error()
    ws, g_ws = guarded_empty(dev, (n_ws,), torch.uint8)
    dH, g_dh = guarded_empty(dev, (B, L, cfg.d_in), torch.float32)
    grads, g_gr = guarded_empty(dev, (cfg.inner_layers * nf,), torch.float32)
    dM_t = torch.from_numpy(np.ascontiguousarray(dM, dtype=np.float32)).to(dev)
    if ws_fill is not None:
        ws.fill_(ws_fill)
    lg.longer_token_merge_backward(model.ccfg, model.inner, H, lens, B, L, dM_t, dH, grads, ws)
    torch.cuda.synchronize()
    for g, what in ((g_ws, "workspace"), (g_dh, "dH_out"), (g_gr, "grads_out")):
        g.check(what)
    views = lg.block_grad_views(cfg, grads)
    return dH.cpu().numpy().astype(np.float64), [{k: v.cpu().numpy().astype(np.float64) for k, v in blk.items()} for blk in views]


def _compare(name, case, dM, users=None, ws_fill=None):
    cfg = case["cfg"]
    _say("backward case %s: B=%d L=%d d_in=%d K=%d inner_layers=%d merge=%s act=%s" %
         (name, cfg.B, cfg.L, cfg.d_in, cfg.K, cfg.inner_layers, cfg.merge, cfg.act))
    dH, grads = _run_gpu(case, dM, ws_fill)
    assert np.isfinite(dH).all()
    TOL = TOL_RELU if cfg.act == "relu" else globals()["TOL"]
    sel = list(range(cfg.B)) if users is None else list(users)
    lens = case["lens"]
    sub_lens = None if lens is None else lens[sel]
    sub_cfg = cfg.replace(B=len(sel))
    dH_ref, g_ref = org.token_merge_backward(sub_cfg, case["weights"]["inner"], case["H"][sel], sub_lens, dM[sel],
                                             keep="input_only")
    worst = 0.0
    for i, u in enumerate(sel):
        if np.linalg.norm(dH_ref[i]) == 0:
            assert not dH[u].any(), "user %d: gradient must be zero" % u
            continue
        e = _rel(dH[u], dH_ref[i])
        worst = max(worst, e)
        assert e <= TOL, ("dH", u, e)
        # padded tokens: exact zeros
        ln = cfg.L if lens is None else int(min(lens[u], cfg.L))
        assert not dH[u, ln:].any(), "user %d: padded rows of dH are not zero" % u
    if users is not None:
        rest = np.setdiff1d(np.arange(cfg.B), sel)
        assert not dH[rest].any(), "users without an upstream gradient must get a zero gradient"
    _say("  dH: worst per-user rel-L2 %.3e (tol %.0e)" % (worst, TOL))
    for l in range(cfg.inner_layers):
        for k in PARAMS:
            got, ref = grads[l][k], g_ref[l][k]
            assert np.isfinite(got).all(), (l, k)
            if k == "bk":
                # zero in exact arithmetic (a shift of every key moves all scores of a query alike, and
                # softmax does not see it): judged against the size of b_Q's gradient, a sum of the
                # same kind over the same tokens
                e = float(np.linalg.norm(got - ref)) / (float(np.linalg.norm(g_ref[l]["bq"])) or 1.0)
            else:
                e = _rel(got, ref)
            _say("  block %d %-6s rel-L2 %.3e" % (l, k, e))
            assert e <= TOL, ("grad", l, k, e)


def _bf16_case(base, **kw):
    users = kw.pop("users", None)
    cfg = synth.CONFIGS[base].replace(dtype="bf16", **kw)
    return synth.make_case(cfg, users=users)


def test_backward_small_width32_one_block():
    case = _bf16_case("C1")
    _compare("C1 as bf16", case, synth.draw_merge_gradient(case["cfg"]))


def test_backward_c2_shape_ragged():
    case = _bf16_case("C2", users=6, L=203, ragged=True, len_lo=0, len_hi=203)
    case["lens"][0] = 0
    case["lens"][1] = 203
    case["lens"][2] = 5
    _compare("C2, 6 ragged users incl. an empty one", case, synth.draw_merge_gradient(case["cfg"]))


def test_backward_c3_shape_two_blocks():
    case = _bf16_case("C3", users=3, L=333, ragged=True, len_lo=1, len_hi=333)
    _compare("C3, 3 ragged users, two blocks", case, synth.draw_merge_gradient(case["cfg"]))


def test_backward_padded_rows_are_left_out_whatever_the_workspace_holds():
    """Tiles of padded rows are skipped and padded rows are never read: with a workspace full of NaN bit
    patterns (0xFF bytes) and NaN in the padded part of H, a ragged batch with long padded stretches (whole
    128-row tiles of padding, users of length 0) gives the same gradients."""
    cfg = synth.CONFIGS["C3"].replace(dtype="bf16", B=5, L=700, index=44)
    case = synth.make_case(cfg)                       # every row drawn; the lengths are set here
    case["lens"] = np.array([700, 0, 130, 3, 411], dtype=np.int32)
    case["H"] = np.where(np.arange(cfg.L)[None, :, None] < case["lens"][:, None, None], case["H"], np.float32("nan"))
    _compare("C3 shape, 5 ragged users, NaN workspace", case, synth.draw_merge_gradient(case["cfg"]), ws_fill=0xFF)


def test_backward_relu_and_head_width_32():
    case = _bf16_case("C2", users=4, L=130, act="relu", inner_heads=2)
    _compare("C2 with ReLU, head width 32", case, synth.draw_merge_gradient(case["cfg"]))


def test_backward_concat_merge():
    case = _bf16_case("P1", users=3, L=100, ragged=True, len_lo=3, len_hi=100)
    _compare("P1 (concat merge, raw width 32)", case, synth.draw_merge_gradient(case["cfg"]))


@pytest.mark.parametrize("K", [1, 16, 32])
def test_backward_group_sizes(K):
    case = _bf16_case("C2", users=3, L=97, K=K, ragged=True, len_lo=0, len_hi=97)
    _compare("C2 with K=%d" % K, case, synth.draw_merge_gradient(case["cfg"]))


def test_backward_c3_full_size_sampled_users():
    """The launch configuration the benchmark times (256 users x 2000 tokens): only four users get an
    upstream gradient, so every gradient of the batch is theirs and the oracle can compute it."""
    cfg = synth.CONFIGS["C3"]
    case = synth.make_case(cfg)
    users = [0, 100, 171, 255]
    _compare("C3 full size, upstream gradient on 4 users", case, synth.draw_merge_gradient(cfg, users=users), users=users)


def test_backward_argument_errors():
    import paper_2505_04421_amd as lg
    cfg = synth.CONFIGS["C1"]                      # fp32: no mixed-precision backward
    ccfg = lg.make_config(cfg)
    assert lg.longer_backward_workspace_bytes(ccfg, 4, 64) == 0
    assert "LONGER_BF16" in lg.longer_last_error()


# --------------------------------------------------------------------------- whole model
def _run_model_gpu(case, labels):
    import paper_2505_04421_amd as lg
    from gpu_util import guarded_empty
    cfg = case["cfg"]
    model = lg.DeviceModel(cfg, case["weights"])
    dev = model.device
    B, L = cfg.B, cfg.L
    H, G = model.upload(case["H"]), model.upload(case["G"])
    lens = None if case["lens"] is None else torch.from_numpy(case["lens"].astype(np.int32)).to(dev)
    n_ws = lg.longer_forward_backward_workspace_bytes(model.ccfg, B, L)
    nf = lg.longer_model_grad_floats(model.ccfg)
    assert n_ws > 0 and nf > 0, lg.longer_last_error()
    ws, g_ws = guarded_empty(dev, (n_ws,), torch.uint8)
    dH, g_dh = guarded_empty(dev, (B, L, cfg.d_in), torch.float32)
    dG, g_dg = guarded_empty(dev, (B, cfg.m, cfg.d), torch.float32)
    grads, g_gr = guarded_empty(dev, (nf,), torch.float32)
    logits, g_lg = guarded_empty(dev, (B,), torch.float32)
    loss, g_ls = guarded_empty(dev, (4,), torch.float32)
    lab = torch.from_numpy(labels.astype(np.float32)).to(dev)
    lg.longer_forward_backward(model.ccfg, model.weights, H, G, lens, B, L, lab, loss, logits, dH, dG, grads, ws)
    torch.cuda.synchronize()
    for g, what in ((g_ws, "workspace"), (g_dh, "dH_out"), (g_dg, "dG_out"), (g_gr, "grads_out"), (g_lg, "logits"), (g_ls, "loss")):
        g.check(what)
    views = lg.model_grad_views(cfg, grads)
    f64 = lambda t: t.cpu().numpy().astype(np.float64)
    host = {"inner": [{k: f64(v) for k, v in b.items()} for b in views["inner"]],
            "cross": {k: f64(v) for k, v in views["cross"].items()},
            "self": [{k: f64(v) for k, v in b.items()} for b in views["self"]],
            "head_w": f64(views["head_w"]), "head_b": f64(views["head_b"])}
    if "q_learn" in views:
        host["q_learn"] = f64(views["q_learn"])
    return float(loss[0].item()), f64(logits), f64(dH), f64(dG), host


def _compare_model(name, case):
    cfg = case["cfg"]
    labels = synth.draw_labels(cfg)
    _say("model backward case %s: B=%d L=%d d=%d m=%d k=%d n_self=%d inner_layers=%d k_uniform=%d gmask=%s" %
         (name, cfg.B, cfg.L, cfg.d, cfg.m, cfg.k_recent, cfg.n_self, cfg.inner_layers, cfg.k_uniform, cfg.gmask))
    loss, logits, dH, dG, grads = _run_model_gpu(case, labels)
    ref_loss, ref_logits, dH_ref, dG_ref, g_ref = org.model_backward(cfg, case["weights"], case["H"], case["G"], case["lens"], labels)
    scale = float(np.abs(ref_logits).max()) + 1.0
    assert np.abs(logits - ref_logits).max() <= 2e-2 * scale, (logits, ref_logits)
    assert abs(loss - ref_loss) <= 2e-2 * max(1.0, abs(ref_loss)), (loss, ref_loss)
    _say("  loss %.6f (oracle %.6f), logits max error %.3e" % (loss, ref_loss, np.abs(logits - ref_logits).max()))
    # The gradients are judged for the batch as a whole and per user: the loss gradient of a user is
    # (sigmoid(logit) - label) / B times its logit's gradient, so a logit that is 1e-2 off moves that
    # user's whole gradient by up to that share on top of the rounding of the backward pass itself.
    TOLM = 1e-1 if cfg.act == "relu" else 4e-2      # ReLU: units that take the other branch of the step, see the top
    e = _rel(dH, dH_ref)
    _say("  dH rel-L2 %.3e, dG rel-L2 %.3e" % (e, _rel(dG, dG_ref)))
    assert e <= TOLM and _rel(dG, dG_ref) <= TOLM
    lens = case["lens"]
    for u in range(cfg.B):
        ln = cfg.L if lens is None else int(min(lens[u], cfg.L))
        assert not dH[u, ln:].any(), "user %d: padded rows of dH are not zero" % u
        if np.linalg.norm(dH_ref[u]) > 0:
            assert _rel(dH[u], dH_ref[u]) <= 2 * TOLM, ("dH", u, _rel(dH[u], dH_ref[u]))
    groups = [("inner%d" % i, grads["inner"][i], g_ref["inner"][i]) for i in range(cfg.inner_layers)]
    groups.append(("cross", grads["cross"], g_ref["cross"]))
    groups += [("self%d" % i, grads["self"][i], g_ref["self"][i]) for i in range(cfg.n_self)]
    for gname, got, ref in groups:
        worst = 0.0
        for k in PARAMS:
            assert np.isfinite(got[k]).all(), (gname, k)
            if k == "bk":       # zero in exact arithmetic: judged against b_Q's size
                e = float(np.linalg.norm(got[k] - ref[k])) / (float(np.linalg.norm(ref["bq"])) or 1.0)
            else:
                e = _rel(got[k], ref[k])
            worst = max(worst, e)
            assert e <= TOLM, ("grad", gname, k, e)
        _say("  %-7s worst parameter rel-L2 %.3e" % (gname, worst))
    if cfg.q_learnable:
        e = _rel(grads["q_learn"], g_ref["q_learn"])
        _say("  learnable query tokens rel-L2 %.3e" % e)
        assert e <= TOLM
    assert _rel(grads["head_w"], g_ref["head_w"]) <= TOLM
    assert abs(grads["head_b"][0] - g_ref["head_b"][0]) <= TOLM * (abs(g_ref["head_b"][0]) + 1.0 / cfg.B)


def test_model_backward_long_sequence_many_queries():
    """975 merged tokens and 900 query slots per user: more rows than the attention kernels of the
    reduced stack stage in LDS per (user, head), so the row-per-thread kernels run instead."""
    case = _bf16_case("C2", users=2, L=7800, k_recent=900, ragged=True, len_lo=7000, len_hi=7800)
    case["lens"][0] = 7800
    _compare_model("C2 width, L = 7800, k = 900", case)


def test_model_backward_c2_shape_ragged():
    case = _bf16_case("C2", users=6, L=203, ragged=True, len_lo=0, len_hi=203)
    case["lens"][:3] = [0, 203, 5]
    _compare_model("C2, 6 ragged users", case)


def test_model_backward_c3_shape_sampled_queries_causal_globals():
    case = _bf16_case("C3", users=3, L=1010, k_uniform=40, gmask="causal", ragged=True, len_lo=500, len_hi=1010)
    _compare_model("C3, 3 users, recent 60 + uniform 40, causal globals", case)


@pytest.mark.parametrize("gmask", ["full", "causal"])
def test_model_backward_learnable_query_tokens(gmask):
    case = _bf16_case("C2", users=5, L=203, q_learnable=True, gmask=gmask, ragged=True, len_lo=0, len_hi=203)
    case["lens"][:2] = [0, 203]
    _compare_model("C2 with learnable query tokens, %s globals" % gmask, case)


def test_model_backward_head_width_32_relu():
    case = _bf16_case("C2", users=4, L=130, heads=2, inner_heads=2, act="relu", n_self=1)
    _compare_model("C2 with head width 32, ReLU", case)


def test_model_backward_concat_merge_d256():
    case = _bf16_case("P1", users=2, L=120, k_recent=12, n_self=1)
    _compare_model("P1 (concat merge into width 256)", case)


def test_model_backward_c3_full_size_sampled_users():
    """The headline batch (256 users x 2000 tokens): a user's input gradients and logit depend on that
    user alone (times 1 / B from the mean of Eq. 2), so the oracle computes them user by user."""
    cfg = synth.CONFIGS["C3"]
    case = synth.make_case(cfg)
    labels = synth.draw_labels(cfg)
    _say("model backward case C3 full size: B=%d L=%d" % (cfg.B, cfg.L))
    loss, logits, dH, dG, grads = _run_model_gpu(case, labels)
    assert np.isfinite(dH).all() and np.isfinite(dG).all() and np.isfinite(loss)
    for k, v in grads["cross"].items():
        assert np.isfinite(v).all(), k
    one = cfg.replace(B=1)
    for u in (0, 101, 255):
        _, lg_ref, dH_ref, dG_ref, _ = org.model_backward(one, case["weights"], case["H"][u:u + 1], case["G"][u:u + 1], None,
                                                          labels[u:u + 1])
        e_h, e_g = _rel(dH[u] * cfg.B, dH_ref[0]), _rel(dG[u] * cfg.B, dG_ref[0])
        _say("  user %3d: logit %.4f (oracle %.4f), dH rel-L2 %.3e, dG rel-L2 %.3e" % (u, logits[u], lg_ref[0], e_h, e_g))
        assert abs(logits[u] - lg_ref[0]) <= 2e-2 * (abs(lg_ref[0]) + 1.0)
        assert e_h <= 8e-2 and e_g <= 8e-2


def test_forward_backward_under_hip_graph_capture():
    """longer_forward_backward allocates nothing, never synchronises and enqueues kernels only: captured
    into a HIP graph and replayed three times on new inputs (eager work and synchronisation in between),
    it gives the eager call's input gradients bit for bit and its parameter gradients up to the order of
    their last atomic additions."""
    import paper_2505_04421_amd as lg
    cfg = synth.CONFIGS["C2"].replace(B=12, L=260, ragged=True, len_lo=0, len_hi=260, index=41)
    case = synth.make_case(cfg)
    model = lg.DeviceModel(cfg, case["weights"])
    dev = model.device
    B, L = cfg.B, cfg.L
    H, G = model.upload(case["H"]), model.upload(case["G"])
    lens = torch.from_numpy(case["lens"].astype(np.int32)).to(dev)
    labels = torch.from_numpy(synth.draw_labels(cfg)).to(dev)
    ws = torch.empty(lg.longer_forward_backward_workspace_bytes(model.ccfg, B, L), dtype=torch.uint8, device=dev)
    nf = lg.longer_model_grad_floats(model.ccfg)
    dH = torch.empty(B, L, cfg.d_in, dtype=torch.float32, device=dev)
    dG = torch.empty(B, cfg.m, cfg.d, dtype=torch.float32, device=dev)
    grads = torch.empty(nf, dtype=torch.float32, device=dev)
    loss = torch.empty(4, dtype=torch.float32, device=dev)
    logits = torch.empty(B, dtype=torch.float32, device=dev)

    def run():
        lg.longer_forward_backward(model.ccfg, model.weights, H, G, lens, B, L, labels, loss, logits, dH, dG, grads, ws)

    run()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    torch.cuda.synchronize()
    rng = np.random.default_rng(43)
    for it in range(3):
        H.copy_(model.upload(synth.round_bf16(rng.standard_normal(case["H"].shape).astype(np.float32))))
        G.copy_(model.upload(synth.round_bf16(rng.standard_normal(case["G"].shape).astype(np.float32))))
        for t in (dH, dG, grads, loss, logits):
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (dH, dG, grads, loss, logits)]
        for t in (dH, dG, grads, loss, logits):
            t.zero_()
        run()
        torch.cuda.synchronize()
        _say("  replay %d: loss %.6f (eager %.6f)" % (it, float(got[3][0]), float(loss[0])))
        assert torch.equal(got[0], dH) and torch.equal(got[1], dG) and torch.equal(got[4], logits)
        assert torch.allclose(got[2], grads, rtol=1e-4, atol=1e-6 * float(grads.abs().max()))
        assert abs(float(got[3][0]) - float(loss[0])) <= 1e-5 * max(1.0, abs(float(loss[0])))


def _random_bf16_config(seed):
    """A random small bf16 configuration over everything the backward pass accepts (widths, head widths,
    group sizes, global-set sizes, query counts and sampling, layer counts, merge modes, activations, masks)."""
    rng = np.random.default_rng(7000 + seed)
    d, dh = [(32, 16), (64, 16), (64, 32), (128, 16), (128, 32), (256, 32), (256, 16)][int(rng.integers(0, 7))]
    K = int(rng.choice([1, 2, 4, 8, 16, 32]))
    m = int(rng.choice([1, 2, 4, 8, 16]))
    merge = "mean"
    if d == 256 and rng.random() < 0.5:
        merge, K = "concat", int(rng.choice([4, 8]))
    di = d // K if merge == "concat" else d
    inner_heads = di // dh if di == d else di // 16
    L = int(rng.integers(2 * K, (40 if d < 256 else 12) * K))
    T = (L + K - 1) // K
    k = int(rng.integers(1, min(2 * T, 150 - m) + 1))
    ku = int(rng.integers(0, k + 1)) if rng.random() < 0.5 else 0
    return synth.Config("rndb", 700 + seed, B=int(rng.integers(2, 6)), L=L, d=d, heads=d // dh, m=m, K=K, k_recent=k,
                        n_self=int(rng.integers(0, 3)), inner_layers=int(rng.integers(1, 4)), inner_heads=inner_heads,
                        dtype="bf16", act=str(rng.choice(["gelu_erf", "gelu_erf", "relu"])),
                        gmask=str(rng.choice(["full", "causal"])), ragged=True, len_lo=0, len_hi=L, merge=merge,
                        k_uniform=ku, ffn_mult=int(rng.choice([2, 4])))


@pytest.mark.parametrize("seed", range(10))
def test_random_configurations_backward(seed):
    cfg = _random_bf16_config(seed)
    case = synth.make_case(cfg)
    if int(case["lens"].max()) == 0:
        case["lens"][0] = cfg.L
    _say("random configuration %d: %s" % (seed, cfg))
    _compare("random %d (token merge)" % seed, case, synth.draw_merge_gradient(cfg))
    _compare_model("random %d (whole model)" % seed, case)
