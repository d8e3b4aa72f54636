"""Parity of the HIP path (through the C ABI) against the fp64 oracle, element by
element on seeded inputs.  Tolerances: max relative L2 per user 1e-5 (fp32 mode) and
1e-2 (bf16 mode), the bar the benchmark definition states."""
import numpy as np
import pytest
import torch

import longer_synth as synth
from oracle import longer_oracle as orc

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 1e-2}


def _runner(case):
    from gpu_util import Runner
    return Runner(case)


def _say(msg):
    print(msg, flush=True)


def _gmodel(*a, **kw):
    from gpu_util import GuardedModel
    return GuardedModel(*a, **kw)


def test_mfma_register_layout_probe():
    import paper_2505_04421_amd as lg
    out = torch.zeros(2, 64, 16, dtype=torch.int32, device="cuda")
    lg.longer_probe_mfma_layout(out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    exp = np.zeros((64, 16), dtype=np.int64)
    for lane in range(64):
        for r in range(16):
            exp[lane, r] = (8 * (r // 4) + 4 * (lane // 32) + r % 4) * 32 + lane % 32
    assert np.array_equal(got[0], exp), got[0][:2]
    assert np.array_equal(got[1], exp), got[1][:2]


# A single row (one token's d features) is judged too, so that one bad row cannot hide among a
# user's many good ones: fp32 at the same bar, bf16 at ROW_SLACK times the per-user bar (a row
# has d values where a user has thousands, so its error norm fluctuates more).
ROW_SLACK = {"f32": 1.0, "bf16": 2.0}


def _check(name, got, ref, tol):
    from gpu_util import rel_l2_per_user, rel_l2_per_row, assert_zero_where_ref_zero_rows, check_all_guards
    check_all_guards()
    assert np.isfinite(got).all(), name + ": non-finite output"
    err = rel_l2_per_user(got, ref)
    row = rel_l2_per_row(got, ref) if got.ndim >= 3 else err
    row_tol = tol * (ROW_SLACK["f32"] if tol < 1e-3 else ROW_SLACK["bf16"])
    _say("  %-28s rel-L2 max %.3e (tol %.0e), worst row %.3e (tol %.0e)" % (name, err, tol, row, row_tol))
    assert err <= tol, (name, err)
    assert row <= row_tol, (name, "row", row)
    assert_zero_where_ref_zero_rows(got, ref)
    return err


def _check_logits_by_terms(name, logits, lg_ref, Yg_ref, head_w, tol):
    """A logit is a sum of m d signed terms: judge it against the size of those terms (a logit that
    happens to cancel to nearly zero has no meaningful relative error of its own)."""
    hw = np.abs(np.asarray(head_w, dtype=np.float64))
    terms = (np.abs(Yg_ref.reshape(-1, hw.size)) * hw[None, :]).sum(1).reshape(lg_ref.shape) + 1e-30
    err = float((np.abs(logits - lg_ref) / terms).max())
    _say("  %-28s max error / sum of |terms| %.3e (tol %.0e)" % (name, err, tol))
    assert np.isfinite(logits).all() and err <= tol, (name, err)


def _entry_points(case, tol, with_inner=True, logits_by_terms=False):
    cfg, w = case["cfg"], case["weights"]
    r = _runner(case)
    H, G, lens = case["H"], case["G"], case["lens"]
    M_ref = orc.token_merge(cfg, w["inner"], H, lens)
    _check("longer_token_merge", r.token_merge(), M_ref, tol)
    if with_inner:
        _check("longer_inner_transformer", r.inner_transformer(), orc.inner_transformer(cfg, w["inner"], H, lens), tol)
    # the later stages are checked on the oracle's own (rounded) intermediates so that each
    # entry point is compared in isolation, then end to end
    rnd = synth.round_bf16 if cfg.dtype == "bf16" else (lambda a: a.astype(np.float32))
    M_in = rnd(M_ref.astype(np.float32))
    X1_ref = orc.hybrid_cross_attn(cfg, w["cross"], G, M_in, lens, L=cfg.L, q_learn=w.get("q_learn"))
    _check("longer_hybrid_cross_attn", r.cross(G, M_in), X1_ref, tol)
    if cfg.n_self:
        X_in = rnd(X1_ref.astype(np.float32))
        X2_ref = orc.self_attn_layer(cfg, w["self"][0], X_in, lens, L=cfg.L)
        _check("longer_self_attn_layer", r.self_layer(X_in, 0), X2_ref, tol)
    Y_ref, lg_ref = orc.forward(cfg, w, H, G, lens)
    Y, logits = r.forward()
    _check("longer_forward Y", Y, Y_ref, tol)
    if logits_by_terms:
        _check_logits_by_terms("longer_forward logits", logits, lg_ref, Y_ref[:, :cfg.m], w["head_w"], tol)
    else:
        _check("longer_forward logits", logits[None, :], lg_ref[None, :], tol)


def test_c1_fp32_all_entry_points():
    _say("C1 fp32")
    _entry_points(synth.make_case(synth.CONFIGS["C1"]), TOL["f32"])


@pytest.mark.parametrize("gmask", ["full", "causal"])
def test_fp32_ragged_short_users_and_ragged_last_group(gmask):
    """L not a multiple of K, users shorter than k*K (invalid query slots), a user of
    length 0 and NaN in the padding."""
    cfg = synth.CONFIGS["C1"].replace(B=5, L=70, ragged=True, len_lo=1, len_hi=70, gmask=gmask, n_self=2, index=11)
    case = synth.make_case(cfg)
    case["lens"] = np.array([70, 0, 3, 29, 41], dtype=np.int32)
    H = np.random.default_rng(5).standard_normal(case["H"].shape).astype(np.float32)
    pos = np.arange(cfg.L)[None, :, None]
    case["H"] = np.where(pos < case["lens"][:, None, None], H, np.float32("nan")).astype(np.float32)
    _say("fp32 ragged, gmask=" + gmask)
    _entry_points(case, TOL["f32"])


def test_fp32_d64():
    cfg = synth.CONFIGS["C1"].replace(d=64, heads=4, inner_heads=4, m=4, K=8, L=96, k_recent=5, index=12, inner_layers=2)
    _say("fp32 d=64")
    _entry_points(synth.make_case(cfg), TOL["f32"])


def test_fp32_headline_width_d128():
    """The headline model shape (d = 128, 8 heads, two InnerTrans blocks, three self layers, m = 8, k = 100,
    K = 8) in fp32 on a few ragged users: the same kernels without bf16 rounding, so that an error of the
    logic at this width cannot hide inside the bf16 tolerance.  Forward entry points and serving."""
    cfg = synth.CONFIGS["C3"].replace(dtype="f32", B=3, L=333, ragged=True, len_lo=1, len_hi=333, index=31)
    case = synth.make_case(cfg)
    case["lens"][0] = 333
    _say("fp32 d=128 (C3's model shape, 3 ragged users)")
    _entry_points(case, TOL["f32"])
    scfg = cfg.replace(C=5, index=32)
    _say("fp32 d=128 serving")
    _serving(synth.make_case(scfg), TOL["f32"])


@pytest.mark.parametrize("k_recent,gmask", [(124, "full"), (150, "causal")])
def test_bf16_wide_query_sets(k_recent, gmask):
    """m + k = 128 fills the one-workgroup-per-user stack kernel exactly; m + k = 154 does not
    fit it, so longer_forward runs one K/V-projection + attention launch pair per layer.
    Ragged lengths, some users with fewer merged tokens than query slots."""
    cfg = synth.CONFIGS["C2"].replace(B=6, L=1400, K=8, m=4, k_recent=k_recent, n_self=2, gmask=gmask,
                                      ragged=True, len_lo=40, len_hi=1400, index=13)
    case = synth.make_case(cfg, pad_value=float("nan"))
    case["lens"][0] = 1400
    case["lens"][1] = 300          # 38 merged tokens < k
    case["H"][0] = synth.round_bf16(np.random.default_rng(7).standard_normal(case["H"][0].shape).astype(np.float32))
    case["H"][1, 300:] = np.nan
    _say("bf16 d=64, m + k = %d, gmask=%s" % (cfg.m + k_recent, gmask))
    _entry_points(case, TOL["bf16"], with_inner=False)


def test_fp32_single_user_single_group():
    """B = 1 and L < K: one (ragged) group, one merged token, every query slot but one invalid."""
    cfg = synth.CONFIGS["C1"].replace(B=1, L=3, K=4, index=14)
    _say("fp32 B=1, L=3 < K=4")
    _entry_points(synth.make_case(cfg), TOL["f32"])


@pytest.mark.parametrize("base,users", [("C1", None), ("C2", 8)])
def test_relu_activation(base, users):
    cfg = synth.CONFIGS[base].replace(act="relu", index=15)
    _say("%s with ReLU in the FFN" % base)
    _entry_points(synth.make_case(cfg, users=users), TOL[cfg.dtype], with_inner=(base == "C1"))


@pytest.mark.parametrize("K", [1, 2, 32])
def test_fp32_merge_group_sizes(K):
    """K = 1 (every token its own group), K = 2, and K = 32 (a whole tile is one group: the
    in-tile softmax runs over all 16 accumulator registers)."""
    cfg = synth.CONFIGS["C1"].replace(B=3, L=100, K=K, k_recent=3, ragged=True, len_lo=1, len_hi=100, index=16)
    case = synth.make_case(cfg, pad_value=float("nan"))
    case["lens"][0] = 100
    case["H"][0] = np.random.default_rng(9).standard_normal(case["H"][0].shape).astype(np.float32)
    _say("fp32 merge with K = %d" % K)
    _entry_points(case, TOL["f32"])


@pytest.mark.parametrize("m", [1, 16, 32])
def test_bf16_serving_global_set_sizes(m):
    """Candidate scoring with 1, 16 and 32 global tokens per candidate (32, 2 and 1 candidates
    per tile; the in-tile softmax windows of 4, 8 and 16 registers), ragged users."""
    cfg = synth.CONFIGS["C2"].replace(B=3, L=400, m=m, k_recent=20, C=7, gmask="causal" if m == 16 else "full",
                                      ragged=True, len_lo=30, len_hi=400, index=17)
    case = synth.make_case(cfg)
    case["lens"][0] = 37           # 5 merged tokens < k
    _say("bf16 serving with m = %d global tokens" % m)
    _serving(case, TOL["bf16"])


def test_bf16_d256_forward_entry_points():
    """The serving configuration's model (d = 256, head width 32) through the forward entry
    points: the d = 256 instantiations of the merge, K/V projection, attention and stack kernels."""
    cfg = synth.CONFIGS["C5"].replace(B=3, L=1200, C=0, ragged=True, len_lo=100, len_hi=1200, index=18)
    case = synth.make_case(cfg, pad_value=float("nan"))
    _say("bf16 d=256 forward (3 users, L=1200, K=16, k=64)")
    _entry_points(case, TOL["bf16"], with_inner=False)


def test_fp32_concat_merge_all_entry_points():
    """Merge by concatenation: raw tokens and InnerTrans at width 32, K = 2 outputs side by side,
    main stack at width 64.  Ragged lengths (a group with one valid token, a user of length 0),
    NaN in the padding."""
    cfg = synth.CONFIGS["C1"].replace(B=5, L=70, d=64, heads=4, K=2, m=4, k_recent=9, n_self=2, inner_layers=2,
                                      inner_heads=2, merge="concat", ragged=True, len_lo=1, len_hi=70, index=21)
    case = synth.make_case(cfg, pad_value=float("nan"))
    case["lens"] = np.array([70, 0, 3, 29, 41], dtype=np.int32)
    H = np.random.default_rng(6).standard_normal(case["H"].shape).astype(np.float32)
    pos = np.arange(cfg.L)[None, :, None]
    case["H"] = np.where(pos < case["lens"][:, None, None], H, np.float32("nan")).astype(np.float32)
    assert case["H"].shape[-1] == 32
    _say("fp32 concat merge 32 x 2 -> 64")
    _entry_points(case, TOL["f32"])


@pytest.mark.parametrize("K,inner_heads", [(4, 4), (8, 2)])
def test_bf16_concat_merge_all_entry_points_and_serving(K, inner_heads):
    """bf16, raw width 64 with K = 4, and the paper's typical raw width 32 (Section 3.4) with K = 8;
    main stack at 256 (the serving configuration's width)."""
    cfg = synth.CONFIGS["C5"].replace(B=3, L=1000, K=K, k_recent=40, inner_layers=2, inner_heads=inner_heads,
                                      merge="concat", ragged=True, len_lo=30, len_hi=1000, C=24, index=22)
    case = synth.make_case(cfg, pad_value=float("nan"))
    case["lens"][0] = 1000
    case["H"][0] = synth.round_bf16(np.random.default_rng(8).standard_normal(case["H"][0].shape).astype(np.float32))
    assert case["H"].shape[-1] == 256 // K
    _say("bf16 concat merge %d x %d -> 256" % (256 // K, K))
    _entry_points(case, TOL["bf16"])
    _serving(case, TOL["bf16"])


@pytest.mark.parametrize("k_uniform", [9, 4])
def test_fp32_sampled_query_slots(k_uniform):
    """Uniformly sampled query slots (all 9, or 4 older ones + the 5 most recent), ragged users
    including one with fewer merged tokens than slots and one of length 0; serving as well."""
    cfg = synth.CONFIGS["C1"].replace(B=5, L=70, k_recent=9, k_uniform=k_uniform, n_self=2, C=6,
                                      ragged=True, len_lo=1, len_hi=70, index=23)
    case = synth.make_case(cfg, pad_value=float("nan"))
    case["lens"] = np.array([70, 0, 13, 29, 41], dtype=np.int32)
    H = np.random.default_rng(10).standard_normal(case["H"].shape).astype(np.float32)
    pos = np.arange(cfg.L)[None, :, None]
    case["H"] = np.where(pos < case["lens"][:, None, None], H, np.float32("nan")).astype(np.float32)
    _say("fp32 sampled query slots, k_uniform=%d of 9" % k_uniform)
    _entry_points(case, TOL["f32"], with_inner=False)
    _serving(case, TOL["f32"])


@pytest.mark.parametrize("k_recent,k_uniform", [(100, 100), (100, 50), (150, 75)])
def test_bf16_sampled_query_slots(k_recent, k_uniform):
    """The ablation's strategies at its query count: uniform 100, recent 50 + uniform 50 (one
    workgroup per user runs the whole reduced stack), and 150 slots (one launch pair per layer)."""
    cfg = synth.CONFIGS["C2"].replace(B=6, L=2000, K=8, m=4, k_recent=k_recent, k_uniform=k_uniform, n_self=2,
                                      ragged=True, len_lo=40, len_hi=2000, C=10, index=24)
    case = synth.make_case(cfg, pad_value=float("nan"))
    case["lens"][0] = 2000
    case["lens"][1] = 300          # 38 merged tokens < slots
    case["H"][0] = synth.round_bf16(np.random.default_rng(11).standard_normal(case["H"][0].shape).astype(np.float32))
    case["H"][1, 300:] = np.nan
    _say("bf16 sampled query slots, k=%d, k_uniform=%d" % (k_recent, k_uniform))
    _entry_points(case, TOL["bf16"], with_inner=False)
    _serving(case, TOL["bf16"])


def test_fp32_learnable_query_tokens():
    """Learnable query tokens in place of sampled ones: ragged users, one with fewer merged tokens
    than slots (all slots still valid) and one of length 0 (no valid slot); serving as well."""
    cfg = synth.CONFIGS["C1"].replace(B=5, L=70, k_recent=9, q_learnable=True, n_self=2, C=6,
                                      ragged=True, len_lo=1, len_hi=70, index=25)
    case = synth.make_case(cfg, pad_value=float("nan"))
    case["lens"] = np.array([70, 0, 13, 29, 41], dtype=np.int32)
    H = np.random.default_rng(12).standard_normal(case["H"].shape).astype(np.float32)
    pos = np.arange(cfg.L)[None, :, None]
    case["H"] = np.where(pos < case["lens"][:, None, None], H, np.float32("nan")).astype(np.float32)
    _say("fp32 learnable query tokens")
    _entry_points(case, TOL["f32"], with_inner=False)
    _serving(case, TOL["f32"])


@pytest.mark.parametrize("k_recent,gmask", [(100, "full"), (150, "causal")])
def test_bf16_learnable_query_tokens(k_recent, gmask):
    """The ablation's 100 learnable queries (one workgroup per user runs the whole reduced stack)
    and 150 of them (one launch pair per layer); forward, every entry point, serving."""
    cfg = synth.CONFIGS["C2"].replace(B=6, L=2000, K=8, m=4, k_recent=k_recent, q_learnable=True, n_self=2,
                                      gmask=gmask, ragged=True, len_lo=40, len_hi=2000, C=10, index=26)
    case = synth.make_case(cfg, pad_value=float("nan"))
    case["lens"][0] = 2000
    case["lens"][1] = 300          # 38 merged tokens < slots
    case["lens"][2] = 0
    case["H"][0] = synth.round_bf16(np.random.default_rng(13).standard_normal(case["H"][0].shape).astype(np.float32))
    case["H"][1, 300:] = np.nan
    case["H"][2] = np.nan
    _say("bf16 learnable query tokens, k=%d, gmask %s" % (k_recent, gmask))
    _entry_points(case, TOL["bf16"], with_inner=False)
    _serving(case, TOL["bf16"])


def test_bf16_d32_all_entry_points_and_serving():
    """The narrowest bf16 width (the paper's typical raw width, Section 3.4) through every entry point."""
    cfg = synth.CONFIGS["C1"].replace(B=6, L=200, dtype="bf16", k_recent=20, n_self=2, inner_layers=2, C=12,
                                      ragged=True, len_lo=3, len_hi=200, index=25)
    case = synth.make_case(cfg, pad_value=float("nan"))
    case["lens"][0] = 200
    case["H"][0] = synth.round_bf16(np.random.default_rng(12).standard_normal(case["H"][0].shape).astype(np.float32))
    _say("bf16 d=32")
    _entry_points(case, TOL["bf16"])
    _serving(case, TOL["bf16"])


@pytest.mark.parametrize("base,ffn_mult,users", [("C1", 2, None), ("C2", 6, 6)])
def test_ffn_width_other_than_4d(base, ffn_mult, users):
    cfg = synth.CONFIGS[base].replace(ffn_mult=ffn_mult, index=26)
    _say("%s with FFN width %d d" % (base, ffn_mult))
    _entry_points(synth.make_case(cfg, users=users), TOL[cfg.dtype])


@pytest.mark.parametrize("d,heads,K", [(64, 2, 8), (128, 4, 8), (256, 16, 16)])
def test_bf16_other_head_widths(d, heads, K):
    """Head width 32 at d = 64 and 128, head width 16 at d = 256 (main stack and InnerTrans)."""
    cfg = synth.CONFIGS["C2"].replace(B=4, L=640, d=d, heads=heads, inner_heads=heads, K=K, m=8, k_recent=40, n_self=2,
                                      C=8, ragged=True, len_lo=50, len_hi=640, index=27)
    case = synth.make_case(cfg, pad_value=float("nan"))
    case["lens"][0] = 640
    case["H"][0] = synth.round_bf16(np.random.default_rng(13).standard_normal(case["H"][0].shape).astype(np.float32))
    _say("bf16 d=%d, %d heads of width %d" % (d, heads, d // heads))
    _entry_points(case, TOL["bf16"])
    _serving(case, TOL["bf16"])


@pytest.mark.parametrize("base,d_e,B,L", [("C1", 32, 3, 75), ("C3", 96, 5, 333)])
def test_input_generation(base, d_e, B, L):
    """H = MLP([E + pos ; tdiff]) (fp32 d = 64 as 32 + 32, bf16 d = 128 as 96 + 32), ragged lengths
    with NaN padding, then the library's own token merge over its output."""
    import paper_2505_04421_amd as lg
    import torch
    cfg = synth.CONFIGS[base].replace(B=B, L=L, ragged=True, len_lo=0, len_hi=L, index=28)
    if base == "C1":
        cfg = cfg.replace(d=64, heads=4, inner_heads=4)
    case = synth.make_input_case(cfg, d_e)
    case["lens"][0] = L            # one full-length user: give it real values where the draw had padding
    rnd = synth.round_bf16 if cfg.dtype == "bf16" else (lambda a: a)
    g = np.random.default_rng(14)
    case["E"][0] = rnd(g.standard_normal(case["E"][0].shape).astype(np.float32))
    case["tdiff"][0] = rnd(g.standard_normal(case["tdiff"][0].shape).astype(np.float32))
    tol = TOL[cfg.dtype]
    model = _gmodel(cfg, synth.draw_weights(cfg))
    mlp = {k: model.upload(v) for k, v in case["mlp"].items()}
    wts = lg.CInputWeights(**{k: v.data_ptr() for k, v in mlp.items()})
    Ed, Td = model.upload(case["E"]), model.upload(case["tdiff"])
    lens = torch.from_numpy(case["lens"].astype(np.int32)).to(model.device)
    H = model.empty(B, L, cfg.d)
    ws = model.workspace(B, L)
    _say("input generation %s d=%d = %d + %d" % (cfg.dtype, cfg.d, d_e, cfg.d - d_e))
    lg.longer_input_generation(model.ccfg, wts, Ed, Td, lens, B, L, d_e, H, ws)
    torch.cuda.synchronize()
    ref = orc.input_generation(cfg, case["mlp"], case["E"], case["tdiff"], case["lens"])
    _check("longer_input_generation", H.float().cpu().numpy().astype(np.float64), ref, tol)


@pytest.mark.parametrize("base,d_e,B,L", [("C1", 32, 3, 75), ("C3", 96, 5, 333), ("C2", 32, 4, 520)])
def test_forward_from_inputs(base, d_e, B, L):
    """The forward pass on the raw inputs (input generation inside the merge kernel) against the
    oracle's input_generation -> forward, and against the library's own two-call sequence.  Ragged
    lengths incl. a ragged last group, NaN padding, K = 4 / 8 / 8, one and two InnerTrans layers."""
    import paper_2505_04421_amd as lg
    import torch
    from gpu_util import rel_l2_per_user
    cfg = synth.CONFIGS[base].replace(B=B, L=L, ragged=True, len_lo=0, len_hi=L, index=29)
    if base == "C1":
        cfg = cfg.replace(d=64, heads=4, inner_heads=4, inner_layers=2)
    case = synth.make_input_case(cfg, d_e)
    case["lens"][0] = L
    case["lens"][1] = 0
    rnd = synth.round_bf16 if cfg.dtype == "bf16" else (lambda a: a)
    g = np.random.default_rng(15)
    case["E"][0] = rnd(g.standard_normal(case["E"][0].shape).astype(np.float32))
    case["tdiff"][0] = rnd(g.standard_normal(case["tdiff"][0].shape).astype(np.float32))
    G = rnd(g.standard_normal((B, cfg.m, cfg.d)).astype(np.float32))
    tol = TOL[cfg.dtype]
    w = synth.draw_weights(cfg)
    if cfg.dtype == "bf16":
        w = synth._map_tree(w, synth.round_bf16)
    model = _gmodel(cfg, w)
    mlp = {k: model.upload(v) for k, v in case["mlp"].items()}
    wts = lg.CInputWeights(**{k: v.data_ptr() for k, v in mlp.items()})
    Ed, Td, Gd = model.upload(case["E"]), model.upload(case["tdiff"]), model.upload(G)
    lens = torch.from_numpy(case["lens"].astype(np.int32)).to(model.device)
    ws = model.workspace(B, L)
    Y = model.empty(B, cfg.n, cfg.d)
    logits = model.empty(B, dtype=torch.float32)
    _say("forward from raw inputs %s d=%d = %d + %d, K=%d, %d InnerTrans layers"
         % (cfg.dtype, cfg.d, d_e, cfg.d - d_e, cfg.K, cfg.inner_layers))
    lg.longer_forward_from_inputs(model.ccfg, model.weights, wts, Ed, Td, d_e, Gd, lens, B, L, Y, logits, ws)
    torch.cuda.synchronize()
    H_ref = orc.input_generation(cfg, case["mlp"], case["E"], case["tdiff"], case["lens"])
    Y_ref, lg_ref = orc.forward(cfg, w, H_ref, G, case["lens"])
    Yh, lh = Y.float().cpu().numpy().astype(np.float64), logits.cpu().numpy().astype(np.float64)
    _check("longer_forward_from_inputs Y", Yh, Y_ref, tol)
    _check("longer_forward_from_inputs logits", lh[None, :], lg_ref[None, :], tol)
    # the two-call sequence (H rounded to the element type in between)
    H = model.empty(B, L, cfg.d)
    Y2 = model.empty(B, cfg.n, cfg.d)
    lg.longer_input_generation(model.ccfg, wts, Ed, Td, lens, B, L, d_e, H, ws)
    lg.longer_forward(model.ccfg, model.weights, H, Gd, lens, B, L, Y2, None, ws)
    torch.cuda.synchronize()
    err = rel_l2_per_user(Yh, Y2.float().cpu().numpy().astype(np.float64))
    _say("  fused vs two calls (GPU)      rel-L2 max %.3e" % err)
    assert err <= tol


def test_forward_and_scoring_under_hip_graph_capture():
    """The entry points allocate nothing, never synchronise and enqueue kernels only, so a caller may
    capture them into a HIP graph.  Replayed three times on new inputs, with eager work and
    synchronisation in between; every replay must equal the eager call bit for bit."""
    import paper_2505_04421_amd as lg
    cfg = synth.CONFIGS["C2"].replace(B=16, C=12, ragged=True, len_lo=0, len_hi=512, index=31)
    case = synth.make_case(cfg, pad_value=float("nan"))
    model = _gmodel(cfg, case["weights"])
    B, L = cfg.B, cfg.L
    ws = model.workspace(B, L, cfg.C)
    lens = torch.from_numpy(case["lens"].astype(np.int32)).to(model.device)
    H, G, Gc = model.upload(case["H"]), model.upload(case["G"]), model.upload(case["G_cand"])
    Y, logits = model.empty(B, cfg.n, cfg.d), model.empty(B, dtype=torch.float32)
    cache = model.kv_cache(B, L)
    sc = model.empty(B, cfg.C, dtype=torch.float32)

    def run():
        lg.longer_forward(model.ccfg, model.weights, H, G, lens, B, L, Y, logits, ws)
        lg.longer_kv_cache_build(model.ccfg, model.weights, H, lens, B, L, cache, ws)
        lg.longer_score_candidates(model.ccfg, model.weights, cache, lens, B, L, Gc, cfg.C, None, sc, ws)

    run()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    torch.cuda.synchronize()
    rng = np.random.default_rng(16)
    for it in range(3):
        Hn = np.where(np.isnan(case["H"]), np.float32("nan"), synth.round_bf16(rng.standard_normal(case["H"].shape).astype(np.float32)))
        H.copy_(model.upload(Hn)); G.copy_(model.upload(synth.round_bf16(rng.standard_normal(case["G"].shape).astype(np.float32))))
        Y.zero_(); logits.zero_(); sc.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = (Y.clone(), logits.clone(), sc.clone())
        Y.zero_(); logits.zero_(); sc.zero_()
        run()                                   # eager, same buffers
        torch.cuda.synchronize()
        _say("  replay %d: |Y| %.3e" % (it, float(Y.float().abs().sum())))
        assert torch.equal(got[0], Y) and torch.equal(got[1], logits) and torch.equal(got[2], sc)
    Y_ref, lg_ref = orc.forward(cfg, case["weights"], Hn, G.float().cpu().numpy(), case["lens"])
    _check("graph replay vs oracle Y", got[0].float().cpu().numpy().astype(np.float64), Y_ref, TOL["bf16"])


@pytest.mark.parametrize("scale", [16.0, 4096.0])
def test_bf16_large_ffn_preactivations(scale):
    """FFN pre-activations far outside the interval the bf16-mode GELU polynomial is fitted on (first
    FFN matrix of every block scaled up, the second scaled down): the clamp has to give x or 0, also
    where the fp16 square and the polynomial overflow (|x| of a few hundred at scale 16, of ten thousand
    at scale 4096, where the entries of the second matrix also fall into fp16's subnormal range)."""
    cfg = synth.CONFIGS["C2"].replace(B=4, L=200, n_self=1, ragged=True, len_lo=20, len_hi=200, C=5, index=33)
    case = synth.make_case(cfg)
    w = case["weights"]
    for blk in w["inner"] + [w["cross"]] + w["self"]:
        blk["w1"] = synth.round_bf16(blk["w1"] * np.float32(scale))
        blk["w2"] = synth.round_bf16(blk["w2"] / np.float32(scale))
    _say("bf16 FFN pre-activations x %g" % scale)
    _entry_points(case, TOL["bf16"], logits_by_terms=True)
    _serving(case, TOL["bf16"], logits_by_terms=True)


def test_forward_from_inputs_with_learnable_queries_and_wide_query_set():
    """Raw inputs + learnable query tokens + 150 query slots (one launch pair per layer instead of the
    one-workgroup stack): the combinations share one forward implementation and must compose."""
    import paper_2505_04421_amd as lg
    cfg = synth.CONFIGS["C2"].replace(B=3, L=300, k_recent=150, q_learnable=True, n_self=2, ragged=True,
                                      len_lo=0, len_hi=300, index=34, gmask="causal")
    d_e = 32
    case = synth.make_input_case(cfg, d_e)
    case["lens"][:] = [300, 0, 77]
    g = np.random.default_rng(17)
    for u, n in enumerate(case["lens"]):
        case["E"][u, :n] = synth.round_bf16(g.standard_normal((n, d_e)).astype(np.float32))
        case["tdiff"][u, :n] = synth.round_bf16(g.standard_normal((n, cfg.d - d_e)).astype(np.float32))
    G = synth.round_bf16(g.standard_normal((cfg.B, cfg.m, cfg.d)).astype(np.float32))
    w = synth._map_tree(synth.draw_weights(cfg), synth.round_bf16)
    model = _gmodel(cfg, w)
    mlp = {k: model.upload(v) for k, v in case["mlp"].items()}
    iw = lg.CInputWeights(**{k: v.data_ptr() for k, v in mlp.items()})
    lens = torch.from_numpy(case["lens"].astype(np.int32)).to(model.device)
    ws = model.workspace(cfg.B, cfg.L)
    Y = model.empty(cfg.B, cfg.n, cfg.d)
    logits = model.empty(cfg.B, dtype=torch.float32)
    _say("raw inputs + learnable queries + 150 slots")
    lg.longer_forward_from_inputs(model.ccfg, model.weights, iw, model.upload(case["E"]), model.upload(case["tdiff"]), d_e,
                                  model.upload(G), lens, cfg.B, cfg.L, Y, logits, ws)
    torch.cuda.synchronize()
    H_ref = orc.input_generation(cfg, case["mlp"], case["E"], case["tdiff"], case["lens"])
    Y_ref, lg_ref = orc.forward(cfg, w, H_ref, G, case["lens"])
    _check("Y", Y.float().cpu().numpy().astype(np.float64), Y_ref, TOL["bf16"])
    _check_logits_by_terms("logits", logits.cpu().numpy().astype(np.float64), lg_ref, Y_ref[:, :cfg.m], w["head_w"], TOL["bf16"])


@pytest.mark.parametrize("base,d_e,U,L", [("C1", 32, 3, 75), ("C3", 96, 4, 333)])
def test_serving_from_inputs(base, d_e, U, L):
    """Cache build on the raw inputs (input generation inside its merge kernel), then candidate scoring:
    against the oracle's input_generation -> kv_cache_build -> score_candidates, ragged users incl. an
    empty one, NaN padding."""
    import paper_2505_04421_amd as lg
    cfg = synth.CONFIGS[base].replace(B=U, L=L, C=7, n_self=2, ragged=True, len_lo=0, len_hi=L, index=35)
    if base == "C1":
        cfg = cfg.replace(d=64, heads=4, inner_heads=4)
    case = synth.make_input_case(cfg, d_e)
    case["lens"][0] = L
    case["lens"][1] = 0
    rnd = synth.round_bf16 if cfg.dtype == "bf16" else (lambda a: a)
    g = np.random.default_rng(18)
    case["E"][0] = rnd(g.standard_normal(case["E"][0].shape).astype(np.float32))
    case["tdiff"][0] = rnd(g.standard_normal(case["tdiff"][0].shape).astype(np.float32))
    Gc = rnd(g.standard_normal((U, cfg.C, cfg.m, cfg.d)).astype(np.float32))
    w = synth.draw_weights(cfg)
    if cfg.dtype == "bf16":
        w = synth._map_tree(w, synth.round_bf16)
    tol = TOL[cfg.dtype]
    model = _gmodel(cfg, w)
    mlp = {k: model.upload(v) for k, v in case["mlp"].items()}
    iw = lg.CInputWeights(**{k: v.data_ptr() for k, v in mlp.items()})
    lens = torch.from_numpy(case["lens"].astype(np.int32)).to(model.device)
    ws = model.workspace(U, L, cfg.C)
    cache = model.kv_cache(U, L)
    Yg = model.empty(U, cfg.C, cfg.m, cfg.d)
    logits = model.empty(U, cfg.C, dtype=torch.float32)
    _say("serving from raw inputs %s d=%d = %d + %d" % (cfg.dtype, cfg.d, d_e, cfg.d - d_e))
    lg.longer_kv_cache_build_from_inputs(model.ccfg, model.weights, iw, model.upload(case["E"]), model.upload(case["tdiff"]),
                                         d_e, lens, U, L, cache, ws)
    lg.longer_score_candidates(model.ccfg, model.weights, cache, lens, U, L, model.upload(Gc), cfg.C, Yg, logits, ws)
    torch.cuda.synchronize()
    H_ref = orc.input_generation(cfg, case["mlp"], case["E"], case["tdiff"], case["lens"])
    ref_cache = orc.kv_cache_build(cfg, w, H_ref, case["lens"])
    Yg_ref, lg_ref = orc.score_candidates(cfg, w, ref_cache, Gc)
    _check("Yg", Yg.float().cpu().numpy().astype(np.float64).reshape(U * cfg.C, cfg.m, cfg.d), Yg_ref.reshape(U * cfg.C, cfg.m, cfg.d), tol)
    _check_logits_by_terms("logits", logits.cpu().numpy().astype(np.float64), lg_ref, Yg_ref, w["head_w"], tol)


def test_rows_of_missing_tokens_are_never_read_by_the_layer_entry_points():
    """longer_hybrid_cross_attn and longer_self_attn_layer on caller-made inputs whose rows of
    tokens that do not exist (merged tokens past T_u, invalid query slots) hold NaN: those rows
    must not reach any K/V, so the results equal the oracle's, which never looks at them."""
    cfg = synth.CONFIGS["C2"].replace(B=5, L=512, n_self=1, ragged=True, len_lo=0, len_hi=512, index=41)
    case = synth.make_case(cfg, pad_value=float("nan"))
    case["lens"][:] = [512, 0, 37, 200, 263]
    w = case["weights"]
    r = _runner(case)
    g = np.random.default_rng(19)
    Tu = (case["lens"] + cfg.K - 1) // cfg.K
    M = synth.round_bf16(g.standard_normal((cfg.B, cfg.T, cfg.d)).astype(np.float32))
    for u in range(cfg.B):
        M[u, Tu[u]:] = np.nan
    G = case["G"]
    _say("NaN in the rows of missing tokens (cross layer: M past T_u)")
    X1_ref = orc.hybrid_cross_attn(cfg, w["cross"], G, np.nan_to_num(M), case["lens"], L=cfg.L)
    _check("longer_hybrid_cross_attn", r.cross(G, M), X1_ref, TOL["bf16"])
    X = synth.round_bf16(g.standard_normal((cfg.B, cfg.n, cfg.d)).astype(np.float32))
    for u in range(cfg.B):
        X[u, cfg.m:cfg.m + max(cfg.k_recent - Tu[u], 0)] = np.nan
    _say("NaN in the rows of missing tokens (self layer: invalid query slots)")
    X2_ref = orc.self_attn_layer(cfg, w["self"][0], np.nan_to_num(X), case["lens"], L=cfg.L)
    _check("longer_self_attn_layer", r.self_layer(X, 0), X2_ref, TOL["bf16"])


@pytest.mark.parametrize("k_recent", [32, 150])
def test_parameters_packed_once_equal_packing_per_call(k_recent):
    """longer_pack_weights + a longer_weights whose `packed` member is set give bit for bit what the
    same calls give when they pack per call: forward (both launch plans), forward from raw inputs,
    cache build + scoring."""
    import paper_2505_04421_amd as lg
    cfg = synth.CONFIGS["C2"].replace(B=5, L=400, k_recent=k_recent, n_self=2, C=9, ragged=True, len_lo=0, len_hi=400, index=42)
    d_e = 32
    case = synth.make_case(cfg, pad_value=float("nan"))
    icase = synth.make_input_case(cfg.replace(ragged=False), d_e)
    model = _gmodel(cfg, case["weights"])
    mlp = {k: model.upload(v) for k, v in icase["mlp"].items()}
    iw = lg.CInputWeights(**{k: v.data_ptr() for k, v in mlp.items()})
    packed = model.pack(iw)
    B, L = cfg.B, cfg.L
    lens = torch.from_numpy(case["lens"].astype(np.int32)).to(model.device)
    H, G, Gc = model.upload(case["H"]), model.upload(case["G"]), model.upload(case["G_cand"])
    Ed, Td = model.upload(icase["E"]), model.upload(icase["tdiff"])
    ws = model.workspace(B, L)
    _say("packed once vs packed per call, m + k = %d" % cfg.n)
    outs = []
    for wts in (model.weights, packed):
        Y, logits = model.empty(B, cfg.n, cfg.d), model.empty(B, dtype=torch.float32)
        Y2, logits2 = model.empty(B, cfg.n, cfg.d), model.empty(B, dtype=torch.float32)
        cache = model.kv_cache(B, L)
        Yg, sc = model.empty(B, cfg.C, cfg.m, cfg.d), model.empty(B, cfg.C, dtype=torch.float32)
        lg.longer_forward(model.ccfg, wts, H, G, lens, B, L, Y, logits, ws)
        lg.longer_forward_from_inputs(model.ccfg, wts, iw, Ed, Td, d_e, G, lens, B, L, Y2, logits2, ws)
        lg.longer_kv_cache_build(model.ccfg, wts, H, lens, B, L, cache, ws)
        lg.longer_score_candidates(model.ccfg, wts, cache, lens, B, L, Gc, cfg.C, Yg, sc, ws)
        torch.cuda.synchronize()
        ws.fill_(0xA5)       # the second round must not live on what the first one packed into the workspace
        outs.append((Y, logits, Y2, logits2, Yg, sc))
    from gpu_util import check_all_guards
    check_all_guards()
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    Y_ref, lg_ref = orc.forward(cfg, case["weights"], case["H"], case["G"], case["lens"])
    _check("packed once: longer_forward Y", outs[1][0].float().cpu().numpy().astype(np.float64), Y_ref, TOL["bf16"])


def _random_config(seed):
    """A random small configuration over everything the library accepts (widths, head widths, group
    sizes, global-set sizes, query counts and sampling, layer counts, merge modes, activations, masks)."""
    rng = np.random.default_rng(4000 + seed)
    dtype = str(rng.choice(["f32", "bf16"]))
    if dtype == "f32":
        d, dh = int(rng.choice([32, 64])), 16
    else:
        d, dh = [(32, 16), (64, 16), (64, 32), (128, 16), (128, 32), (256, 32), (256, 16)][int(rng.integers(0, 7))]
    K = int(rng.choice([1, 2, 4, 8, 16, 32]))
    m = int(rng.choice([1, 2, 4, 8, 16]))
    merge = "mean"
    if dtype == "bf16" and d == 256 and rng.random() < 0.5:
        merge, K = "concat", int(rng.choice([4, 8]))
    di = d // K if merge == "concat" else d
    inner_heads = di // dh if di == d else di // 16
    L = int(rng.integers(K, (40 if d < 256 else 12) * K))
    T = (L + K - 1) // K
    k = int(rng.integers(1, min(2 * T, 150 - m) + 1))
    ku = int(rng.integers(0, k + 1)) if rng.random() < 0.5 else 0
    return synth.Config("rnd", 600 + seed, B=int(rng.integers(1, 5)), L=L, d=d, heads=d // dh, m=m, K=K, k_recent=k,
                        n_self=int(rng.integers(0, 3)), inner_layers=int(rng.integers(1, 3)), inner_heads=inner_heads,
                        dtype=dtype, act=str(rng.choice(["gelu_erf", "relu"])), gmask=str(rng.choice(["full", "causal"])),
                        ragged=True, len_lo=0, len_hi=L, merge=merge, k_uniform=ku, ffn_mult=int(rng.choice([2, 4])),
                        C=int(rng.integers(1, 7)))


@pytest.mark.parametrize("seed", range(16))
def test_random_configurations_forward_and_serving(seed):
    from gpu_util import rel_l2_per_user, assert_zero_where_ref_zero_rows
    cfg = _random_config(seed)
    case = synth.make_case(cfg, pad_value=float("nan"))
    tol = TOL[cfg.dtype]
    _say("random configuration %d: %s" % (seed, cfg))
    r = _runner(case)
    w = case["weights"]
    Y_ref, lg_ref = orc.forward(cfg, w, case["H"], case["G"], case["lens"])
    Y, logits = r.forward()
    _check("longer_forward Y", Y, Y_ref, tol)
    # a logit is a sum of m d signed terms: judge it against the size of those terms (a logit that
    # happens to cancel to nearly zero has no meaningful relative error of its own)
    hw = np.abs(np.asarray(w["head_w"], dtype=np.float64))
    scale = (np.abs(Y_ref[:, :cfg.m].reshape(cfg.B, -1)) * hw[None, :]).sum(1) + 1e-30
    assert np.isfinite(logits).all() and (np.abs(logits - lg_ref) / scale).max() <= tol
    Yg, lgs = r.serve()
    cache = orc.kv_cache_build(cfg, w, case["H"], case["lens"])
    Yg_ref, lgs_ref = orc.score_candidates(cfg, w, cache, case["G_cand"])
    _check("longer_score_candidates Yg", Yg.reshape(cfg.B * cfg.C, cfg.m, cfg.d), Yg_ref.reshape(cfg.B * cfg.C, cfg.m, cfg.d), tol)
    sc2 = (np.abs(Yg_ref.reshape(cfg.B, cfg.C, -1)) * hw[None, None, :]).sum(2) + 1e-30
    assert np.isfinite(lgs).all() and (np.abs(lgs - lgs_ref) / sc2).max() <= tol


def test_c2_bf16_all_entry_points():
    _say("C2 bf16 (16 users)")
    _entry_points(synth.make_case(synth.CONFIGS["C2"], users=16), TOL["bf16"])


def test_c3_bf16_all_entry_points():
    _say("C3 bf16 (6 users)")
    _entry_points(synth.make_case(synth.CONFIGS["C3"], users=6), TOL["bf16"], with_inner=False)


def test_c4_bf16_ragged_nan_padding():
    _say("C4 bf16 ragged (6 users, NaN padding)")
    case = synth.make_case(synth.CONFIGS["C4"], users=6, pad_value=float("nan"))
    case["lens"][0] = 100        # fewer merged tokens (7) than query slots (64)
    case["lens"][1] = 5000       # a full-length user: the last group (5000 = 312*16 + 8) is ragged by L itself
    case["H"][0, 100:] = np.nan
    case["H"][1] = synth.round_bf16(np.random.default_rng(3).standard_normal(case["H"][1].shape).astype(np.float32))
    _entry_points(case, TOL["bf16"], with_inner=False)


def _serving(case, tol, logits_by_terms=False):
    from gpu_util import rel_l2_per_user
    cfg, w = case["cfg"], case["weights"]
    r = _runner(case)
    Yg, logits = r.serve()
    cache = orc.kv_cache_build(cfg, w, case["H"], case["lens"])
    Yg_ref, lg_ref = orc.score_candidates(cfg, w, cache, case["G_cand"])
    U, C = cfg.B, cfg.C
    _check("longer_score_candidates Yg", Yg.reshape(U * C, cfg.m, cfg.d), Yg_ref.reshape(U * C, cfg.m, cfg.d), tol)
    if logits_by_terms:
        _check_logits_by_terms("longer_score_candidates logit", logits, lg_ref, Yg_ref, w["head_w"], tol)
    else:
        _check("longer_score_candidates logit", logits, lg_ref, tol)
    # KV-cached scoring equals the full forward pass with that candidate's globals (GPU vs GPU)
    Yf, lf = r.forward(G=case["G_cand"][:, 0])
    err = rel_l2_per_user(Yg[:, 0], Yf[:, :cfg.m])
    _say("  cached vs full forward (GPU)  rel-L2 max %.3e" % err)
    assert err <= tol


def test_fp32_serving_small():
    cfg = synth.CONFIGS["C1"].replace(B=3, L=70, C=9, n_self=2, ragged=True, len_lo=5, len_hi=70, index=13)
    case = synth.make_case(cfg)
    case["lens"][0] = 9
    _say("fp32 serving")
    _serving(case, TOL["f32"])


def test_c5_bf16_serving():
    _say("C5 bf16 serving (2 users x 24 candidates)")
    _serving(synth.make_case(synth.CONFIGS["C5"], users=2, candidates=24), TOL["bf16"])


# --------------------------------------------------------------------------- full benchmark sizes
# The whole batch runs through the library in the launch configuration bench.py times; the
# oracle recomputes a sample of users (users are independent) and every sampled row is
# compared element by element.  All other users are checked for finiteness and for exact
# zeros in their invalid rows.
def _full_size_forward(name, sample, pad_value=0.0, packed=False):
    from gpu_util import Runner
    case = synth.make_case(synth.CONFIGS[name], pad_value=pad_value)
    cfg, w = case["cfg"], case["weights"]
    r = Runner(case, packed=packed)
    Y, logits = r.forward()
    assert np.isfinite(Y).all() and np.isfinite(logits).all()
    idx = np.arange(cfg.B) if sample is None else np.array(sample)
    lens = None if case["lens"] is None else case["lens"][idx]
    Y_ref, lg_ref = orc.forward(cfg, w, case["H"][idx], case["G"][idx], lens)
    tol = TOL[cfg.dtype]
    _check(name + " full batch, %d users Y" % len(idx), Y[idx], Y_ref, tol)
    _check(name + " full batch, logits", logits[idx][None, :], lg_ref[None, :], tol)
    if case["lens"] is not None:
        Tu = (case["lens"] + cfg.K - 1) // cfg.K
        for u in np.nonzero(Tu < cfg.k_recent)[0]:
            assert (Y[u, cfg.m:cfg.m + cfg.k_recent - Tu[u]] == 0).all()


def test_c2_full_size_all_users():
    _say("C2 full size (128 users), every user against the oracle")
    _full_size_forward("C2", None)


def test_c3_full_size_all_users():
    _say("C3 full size (256 users x 2000), every user against the oracle, parameters packed once")
    _full_size_forward("C3", None, packed=True)


def test_c4_full_size_sampled_users():
    _say("C4 full size (512 users, ragged, NaN padding), 40 users against the oracle")
    case = synth.make_case(synth.CONFIGS["C4"])
    order = np.argsort(case["lens"], kind="stable")
    # the four shortest, the four longest, the first and last of the batch and every 16th user in between
    pick = sorted(set(order[:4].tolist()) | set(order[-4:].tolist()) | {0, 511} | set(range(8, 512, 16)))
    _full_size_forward("C4", pick, pad_value=float("nan"))


def test_concat_production_shape_full_size_sampled_users():
    _say("P1 full size (256 users, raw width 32, K = 8, main stack at 256)")
    _full_size_forward("P1", [0, 131, 255])


def test_forward_from_inputs_full_size_sampled_users():
    """The C3 batch shape through longer_forward_from_inputs in the launch configuration the benchmark
    times (bench.py --from-inputs 96); the oracle recomputes a sample of users from their raw inputs."""
    import paper_2505_04421_amd as lg
    cfg = synth.CONFIGS["C3"]
    d_e = 96
    _say("C3 full size from raw inputs (256 users x 2000, item width 96 + time-difference width 32)")
    case = synth.make_case(cfg)
    icase = synth.make_input_case(cfg, d_e)
    w = case["weights"]
    model = _gmodel(cfg, w)
    mlp = {k: model.upload(v) for k, v in icase["mlp"].items()}
    iw = lg.CInputWeights(**{k: v.data_ptr() for k, v in mlp.items()})
    Ed, Td, Gd = model.upload(icase["E"]), model.upload(icase["tdiff"]), model.upload(case["G"])
    ws = model.workspace(cfg.B, cfg.L)
    Y = model.empty(cfg.B, cfg.n, cfg.d)
    logits = model.empty(cfg.B, dtype=torch.float32)
    lg.longer_forward_from_inputs(model.ccfg, model.weights, iw, Ed, Td, d_e, Gd, None, cfg.B, cfg.L, Y, logits, ws)
    torch.cuda.synchronize()
    Yh, lh = Y.float().cpu().numpy().astype(np.float64), logits.cpu().numpy().astype(np.float64)
    assert np.isfinite(Yh).all() and np.isfinite(lh).all()
    idx = np.array([0, 77, 255])
    H_ref = orc.input_generation(cfg, icase["mlp"], icase["E"][idx], icase["tdiff"][idx])
    Y_ref, lg_ref = orc.forward(cfg, w, H_ref, case["G"][idx])
    _check("from raw inputs, sampled users Y", Yh[idx], Y_ref, TOL["bf16"])
    _check("from raw inputs, sampled logits", lh[idx][None, :], lg_ref[None, :], TOL["bf16"])


def test_c5_full_size_whole_workgroups_of_candidates():
    """C5 in the launch configuration the benchmark times.  Per checked user: every candidate of the
    first workgroup of its candidate tiles (4 waves x 32 rows = 16 candidates), of a workgroup in the
    middle, and of the last (partially filled) workgroup.  Users 0, 7, 8 and 15 sit on different
    dies of the chip under the scoring launch's user placement (user u on die u mod 8)."""
    _say("C5 full size (16 users x 1000 candidates)")
    case = synth.make_case(synth.CONFIGS["C5"])
    cfg, w = case["cfg"], case["weights"]
    r = _runner(case)
    Yg, logits = r.serve()
    assert np.isfinite(Yg).all() and np.isfinite(logits).all()
    users = [0, 7, 8, 15]
    per_wg = 4 * 32 // cfg.m
    last_wg = (cfg.C - 1) // per_wg
    cands = sorted(set(range(0, per_wg)) | set(range(31 * per_wg, 32 * per_wg)) | set(range(last_wg * per_wg, cfg.C)))
    cache = orc.kv_cache_build(cfg, w, case["H"][users], None)
    Yg_ref, lg_ref = orc.score_candidates(cfg, w, cache, case["G_cand"][users][:, cands])
    got = Yg[users][:, cands]
    n = len(users) * len(cands)
    _say("  %d users x %d candidates against the oracle" % (len(users), len(cands)))
    _check("C5 Yg", got.reshape(n, cfg.m, cfg.d), Yg_ref.reshape(n, cfg.m, cfg.d), TOL["bf16"])
    _check("C5 logits", logits[users][:, cands], lg_ref, TOL["bf16"])
