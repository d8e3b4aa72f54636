"""Pins of the backward-pass oracle (oracle/longer_oracle_grad.py), no GPU needed: torch.autograd on
the library's encoder layer, central finite differences of the (separately pinned) forward oracle,
closed forms and invariants.  Section 3.6.2 of the paper: reverse-mode gradients with recomputation."""
import numpy as np
import pytest
import torch

import longer_synth as synth
from oracle import longer_oracle as orc
from oracle import longer_oracle_grad as grd

PARAMS = grd.PARAMS


def _blk(d, ff, seed):
    cfg = synth.CONFIGS["C1"].replace(d=d, heads=2, inner_heads=2, ffn_mult=ff, index=70 + seed)
    return {k: np.asarray(v, dtype=np.float64) for k, v in synth.draw_weights(cfg)["inner"][0].items()}


def _torch_layer(blk, d, heads, ff):
    layer = torch.nn.TransformerEncoderLayer(d, heads, ff * d, dropout=0.0, activation="gelu",
                                             batch_first=True, norm_first=True).double()
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    with torch.no_grad():
        layer.self_attn.in_proj_weight.copy_(torch.cat([t(blk["wq"]).T, t(blk["wk"]).T, t(blk["wv"]).T], 0))
        layer.self_attn.in_proj_bias.copy_(torch.cat([t(blk["bq"]), t(blk["bk"]), t(blk["bv"])]))
        layer.self_attn.out_proj.weight.copy_(t(blk["wo"]).T)
        layer.self_attn.out_proj.bias.copy_(t(blk["bo"]))
        layer.linear1.weight.copy_(t(blk["w1"]).T); layer.linear1.bias.copy_(t(blk["b1"]))
        layer.linear2.weight.copy_(t(blk["w2"]).T); layer.linear2.bias.copy_(t(blk["b2"]))
        layer.norm1.weight.copy_(t(blk["ln1_g"])); layer.norm1.bias.copy_(t(blk["ln1_b"]))
        layer.norm2.weight.copy_(t(blk["ln2_g"])); layer.norm2.bias.copy_(t(blk["ln2_b"]))
    return layer


def _torch_grads(layer, d):
    g = {}
    ipw, ipb = layer.self_attn.in_proj_weight.grad.numpy(), layer.self_attn.in_proj_bias.grad.numpy()
    g["wq"], g["wk"], g["wv"] = ipw[:d].T, ipw[d:2 * d].T, ipw[2 * d:].T
    g["bq"], g["bk"], g["bv"] = ipb[:d], ipb[d:2 * d], ipb[2 * d:]
    g["wo"], g["bo"] = layer.self_attn.out_proj.weight.grad.numpy().T, layer.self_attn.out_proj.bias.grad.numpy()
    g["w1"], g["b1"] = layer.linear1.weight.grad.numpy().T, layer.linear1.bias.grad.numpy()
    g["w2"], g["b2"] = layer.linear2.weight.grad.numpy().T, layer.linear2.bias.grad.numpy()
    g["ln1_g"], g["ln1_b"] = layer.norm1.weight.grad.numpy(), layer.norm1.bias.grad.numpy()
    g["ln2_g"], g["ln2_b"] = layer.norm2.weight.grad.numpy(), layer.norm2.bias.grad.numpy()
    return g


@pytest.mark.parametrize("padded", [False, True])
def test_block_backward_equals_autograd_of_the_library_encoder_layer(padded):
    d, heads, ff, G, K = 32, 2, 4, 5, 6
    rng = np.random.default_rng(1)
    blk = _blk(d, ff, 1)
    x = rng.standard_normal((G, K, d))
    dout = rng.standard_normal((G, K, d))
    valid = np.ones((G, K), dtype=bool)
    if padded:
        valid[1, 4:] = False
        valid[3, 1:] = False
    mask = valid[:, :, None] & valid[:, None, :]
    dout = np.where(valid[:, :, None], dout, 0.0)       # padded rows produce nothing downstream
    dxq, dxkv, g = grd.block_backward(dout, x, x, mask, blk, heads, 1e-5, "gelu_erf")
    dx = np.where(valid[:, :, None], dxq + dxkv, 0.0)
    layer = _torch_layer(blk, d, heads, ff)
    xt = torch.from_numpy(x).requires_grad_(True)
    kpm = torch.from_numpy(~valid) if padded else None
    # (the fused inference path of the library layer is not differentiable; training mode with dropout 0 is the same function)
    layer.train()
    out = layer(xt, src_key_padding_mask=kpm)
    (out * torch.from_numpy(dout)).sum().backward()
    ref_dx = np.where(valid[:, :, None], xt.grad.numpy(), 0.0)
    assert np.abs(dx - ref_dx).max() <= 1e-11 * max(1.0, np.abs(ref_dx).max())
    ref = _torch_grads(layer, d)
    for k in PARAMS:
        assert g[k].shape == ref[k].shape, k
        assert np.abs(g[k] - ref[k]).max() <= 1e-10 * max(1.0, np.abs(ref[k]).max()), k


def _fd(f, x, idx, h=1e-6):
    old = x[idx]
    x[idx] = old + h
    fp = f()
    x[idx] = old - h
    fm = f()
    x[idx] = old
    return (fp - fm) / (2 * h)


@pytest.mark.parametrize("act,cross", [("gelu_erf", False), ("relu", False), ("gelu_erf", True)])
def test_block_backward_against_finite_differences_of_the_forward_oracle(act, cross):
    """Central differences of longer_oracle.block (pinned on its own): self-attention with a random
    mask, and a cross block whose query rows differ from its key rows (Eq. 6)."""
    d, heads, nq, nk = 16, 2, 4, 7
    rng = np.random.default_rng(2)
    blk = {k: np.asarray(v, dtype=np.float64) for k, v in synth.draw_weights(
        synth.CONFIGS["C1"].replace(d=d, heads=heads, inner_heads=heads, ffn_mult=2, index=72))["inner"][0].items()}
    xkv = rng.standard_normal((nk, d))
    xq = rng.standard_normal((nq, d)) if cross else xkv
    n = xq.shape[0]
    mask = rng.random((n, nk)) < 0.7
    mask[:, 0] = True
    w = rng.standard_normal((n, d))
    loss = lambda: float((orc.block(xq, xkv if cross else xq, mask, blk, heads, 1e-5, act) * w).sum())
    dxq, dxkv, g = grd.block_backward(w, xq, xkv if cross else xq, mask, blk, heads, 1e-5, act)
    dx_self = None if cross else dxq + dxkv
    for _ in range(12):
        i, j = int(rng.integers(0, n)), int(rng.integers(0, d))
        num = _fd(loss, xq, (i, j))
        got = dxq[i, j] if cross else dx_self[i, j]
        assert abs(got - num) <= 2e-6 * max(1.0, abs(num)), ("xq", i, j, got, num)
    if cross:
        for _ in range(8):
            i, j = int(rng.integers(0, nk)), int(rng.integers(0, d))
            num = _fd(loss, xkv, (i, j))
            assert abs(dxkv[i, j] - num) <= 2e-6 * max(1.0, abs(num)), ("xkv", i, j)
    for k in PARAMS:
        p = blk[k]
        for _ in range(3):
            idx = tuple(int(rng.integers(0, s)) for s in p.shape)
            num = _fd(loss, p, idx)
            assert abs(g[k][idx] - num) <= 2e-6 * max(1.0, abs(num)), (k, idx, g[k][idx], num)


def _merge_case(merge, seed=3):
    cfg = synth.CONFIGS["C1"].replace(B=3, L=22, K=4, d=32 if merge == "mean" else 128, heads=2,
                                      inner_heads=2, inner_layers=2, merge=merge, ragged=True, len_lo=0, len_hi=22,
                                      index=73 + seed)
    case = synth.make_case(cfg, pad_value=float("nan"))
    case["lens"][:] = [22, 0, 9]
    rng = np.random.default_rng(seed)
    H = rng.standard_normal(case["H"].shape)
    pos = np.arange(cfg.L)[None, :, None]
    case["H"] = np.where(pos < case["lens"][:, None, None], H, np.nan)
    return cfg, case, rng


@pytest.mark.parametrize("merge", ["mean", "concat"])
def test_token_merge_backward_against_finite_differences(merge):
    """Two InnerTrans layers, ragged lengths with a ragged last group, an empty user, NaN padding."""
    cfg, case, rng = _merge_case(merge)
    inner = [{k: np.asarray(v, dtype=np.float64) for k, v in b.items()} for b in case["weights"]["inner"]]
    H, lens = case["H"], case["lens"]
    dM = rng.standard_normal((cfg.B, cfg.T, cfg.d))
    loss = lambda: float((orc.token_merge(cfg, inner, H, lens) * dM).sum())
    dH, grads = grd.token_merge_backward(cfg, inner, H, lens, dM)
    assert np.isfinite(dH).all()
    pos = np.arange(cfg.L)[None, :]
    assert (dH[pos >= lens[:, None]] == 0).all()            # padded tokens: exact zeros
    assert (dH[1] == 0).all()
    for _ in range(10):
        u = int(rng.choice([0, 2]))
        t, j = int(rng.integers(0, lens[u])), int(rng.integers(0, H.shape[-1]))
        num = _fd(loss, H, (u, t, j))
        assert abs(dH[u, t, j] - num) <= 5e-6 * max(1.0, abs(num)), (u, t, j, dH[u, t, j], num)
    for li in range(cfg.inner_layers):
        for k in ("wq", "wk", "wv", "wo", "w1", "w2", "ln1_g", "ln2_b", "bq", "bv", "b1", "b2"):
            p = inner[li][k]
            idx = tuple(int(rng.integers(0, s)) for s in p.shape)
            num = _fd(loss, p, idx)
            assert abs(grads[li][k][idx] - num) <= 5e-6 * max(1.0, abs(num)), (li, k, idx, grads[li][k][idx], num)


def test_key_bias_has_no_gradient_and_value_bias_passes_through():
    """Softmax drops a per-query constant, so d loss / d b_K = 0; the probabilities of a row sum to
    one, so d loss / d b_V = W_O applied to the summed gradient of the attention sub-block's output."""
    cfg, case, rng = _merge_case("mean", seed=4)
    inner = case["weights"]["inner"][:1]
    cfg = cfg.replace(inner_layers=1)
    dM = rng.standard_normal((cfg.B, cfg.T, cfg.d))
    _, grads = grd.token_merge_backward(cfg, inner, case["H"], case["lens"], dM)
    assert np.abs(grads[0]["bk"]).max() <= 1e-12 * np.abs(grads[0]["bq"]).max()
    assert np.abs(grads[0]["bv"] - np.asarray(inner[0]["wo"], dtype=np.float64) @ grads[0]["bo"]).max() <= 1e-10


def test_recomputation_changes_what_is_kept_not_the_gradients():
    cfg, case, rng = _merge_case("mean", seed=5)
    inner = case["weights"]["inner"]
    dM = rng.standard_normal((cfg.B, cfg.T, cfg.d))
    ref_dH, ref_g = grd.token_merge_backward(cfg, inner, case["H"], case["lens"], dM, keep="all")
    for keep in ("block_inputs", "input_only"):
        dH, g = grd.token_merge_backward(cfg, inner, case["H"], case["lens"], dM, keep=keep)
        assert np.array_equal(dH, ref_dH), keep
        for li in range(cfg.inner_layers):
            for k in PARAMS:
                assert np.array_equal(g[li][k], ref_g[li][k]), (keep, li, k)
    with pytest.raises(ValueError):
        grd.token_merge_backward(cfg, inner, case["H"], case["lens"], dM, keep="nothing")


def test_identity_block_gives_the_gradient_of_a_plain_mean():
    """W_O = b_O = W_2 = b_2 = 0 makes the block the identity: dH of a valid token is dM of its group
    divided by the group's valid count."""
    cfg, case, rng = _merge_case("mean", seed=6)
    cfg = cfg.replace(inner_layers=1)
    blk = dict(case["weights"]["inner"][0])
    for k in ("wo", "bo", "w2", "b2"):
        blk[k] = np.zeros_like(blk[k])
    dM = rng.standard_normal((cfg.B, cfg.T, cfg.d))
    dH, _ = grd.token_merge_backward(cfg, [blk], case["H"], case["lens"], dM)
    for u, n in enumerate(case["lens"]):
        for t in range(int(n)):
            grp = t // cfg.K
            cnt = min(cfg.K, int(n) - grp * cfg.K)
            assert np.allclose(dH[u, t], dM[u, grp] / cnt, rtol=0, atol=1e-15)


def test_gradients_are_linear_in_the_upstream_gradient():
    cfg, case, rng = _merge_case("mean", seed=7)
    inner = case["weights"]["inner"]
    a, b = rng.standard_normal((2, cfg.B, cfg.T, cfg.d))
    da, ga = grd.token_merge_backward(cfg, inner, case["H"], case["lens"], a)
    db, gb = grd.token_merge_backward(cfg, inner, case["H"], case["lens"], b)
    dc, gc = grd.token_merge_backward(cfg, inner, case["H"], case["lens"], 2.0 * a - 3.0 * b)
    assert np.abs(dc - (2.0 * da - 3.0 * db)).max() <= 1e-11 * np.abs(dc).max()
    assert np.abs(gc[0]["w1"] - (2.0 * ga[0]["w1"] - 3.0 * gb[0]["w1"])).max() <= 1e-11 * np.abs(gc[0]["w1"]).max()


def test_bce_loss_and_gradient_against_the_library():
    rng = np.random.default_rng(8)
    z = rng.standard_normal(17) * 6.0
    z[0], z[1] = 800.0, -800.0                      # saturated predictions must not overflow
    y = (rng.random(17) < 0.4).astype(np.float64)
    zt = torch.from_numpy(z).requires_grad_(True)
    ref = torch.nn.functional.binary_cross_entropy_with_logits(zt, torch.from_numpy(y))
    ref.backward()
    ref_v = float(ref.detach())
    assert abs(grd.bce_loss(z, y) - ref_v) <= 1e-12 * max(1.0, abs(ref_v))
    assert np.abs(grd.bce_loss_grad(z, y) - zt.grad.numpy()).max() <= 1e-15
    # Eq. 2 written out on unsaturated predictions
    p = 1.0 / (1.0 + np.exp(-z[2:]))
    assert abs(grd.bce_loss(z[2:], y[2:]) + np.mean(y[2:] * np.log(p) + (1 - y[2:]) * np.log(1 - p))) <= 1e-12


@pytest.mark.parametrize("k_uniform,gmask", [(0, "full"), (2, "causal")])
def test_model_backward_against_finite_differences_of_the_forward_oracle(k_uniform, gmask):
    """The whole model (merge, cross-causal layer, two self-causal layers, head, Eq. 1-2) on a tiny ragged
    batch with an empty user and a user shorter than the query set: every input and a sample of every
    parameter group against central differences of the loss computed by the forward oracle."""
    cfg = synth.tiny_config(B=4, L=22, d=8, heads=2, m=2, K=4, k_recent=4, n_self=2, inner_layers=1,
                            k_uniform=k_uniform, gmask=gmask, ragged=True, len_lo=0, len_hi=22)
    case = synth.make_case(cfg)
    case["lens"][:] = [22, 0, 5, 17]
    rng = np.random.default_rng(5 + k_uniform)
    w = case["weights"]
    w = {"inner": [{k: np.asarray(v, dtype=np.float64) for k, v in b.items()} for b in w["inner"]],
         "cross": {k: np.asarray(v, dtype=np.float64) for k, v in w["cross"].items()},
         "self": [{k: np.asarray(v, dtype=np.float64) for k, v in b.items()} for b in w["self"]],
         "head_w": np.asarray(w["head_w"], dtype=np.float64), "head_b": np.asarray(w["head_b"], dtype=np.float64)}
    H = np.asarray(case["H"], dtype=np.float64)
    G = np.asarray(case["G"], dtype=np.float64)
    lens = case["lens"]
    labels = np.array([1.0, 0.0, 1.0, 0.0])

    def loss():
        _, logits = orc.forward(cfg, w, H, G, lens)
        return grd.bce_loss(logits, labels)

    val, logits, dH, dG, grads = grd.model_backward(cfg, w, H, G, lens, labels)
    assert abs(val - loss()) <= 1e-12
    assert np.allclose(logits, orc.forward(cfg, w, H, G, lens)[1], atol=1e-12)
    pos = np.arange(cfg.L)[None, :]
    assert (dH[pos >= lens[:, None]] == 0).all()

    def close(a, num):      # step 1e-7: LayerNorm over 8 features bends sharply, 1e-6 leaves 3e-6 of truncation error
        return abs(a - num) <= 2e-6 * max(1e-2, abs(num))

    for u in (0, 2, 3):
        for _ in range(6):
            t, j = int(rng.integers(0, lens[u])), int(rng.integers(0, H.shape[-1]))
            num = _fd(loss, H, (u, t, j), h=1e-7)
            assert close(dH[u, t, j], num), ("dH", u, t, j, dH[u, t, j], num)
    for u in range(cfg.B):
        for _ in range(4):
            i, j = int(rng.integers(0, cfg.m)), int(rng.integers(0, cfg.d))
            num = _fd(loss, G, (u, i, j), h=1e-7)
            assert close(dG[u, i, j], num), ("dG", u, i, j, dG[u, i, j], num)
    groups = [("inner0", w["inner"][0], grads["inner"][0]), ("cross", w["cross"], grads["cross"]),
              ("self0", w["self"][0], grads["self"][0]), ("self1", w["self"][1], grads["self"][1])]
    for name, params, g in groups:
        for key in ("wq", "wk", "wv", "wo", "w1", "w2", "ln1_g", "ln1_b", "ln2_g", "bq", "bv", "bo", "b1", "b2"):
            p = params[key]
            idx = tuple(int(rng.integers(0, s)) for s in p.shape)
            num = _fd(loss, p, idx, h=1e-7)
            assert close(g[key][idx], num), (name, key, idx, g[key][idx], num)
    for _ in range(5):
        idx = (int(rng.integers(0, w["head_w"].size)),)
        num = _fd(loss, w["head_w"], idx, h=1e-7)
        assert close(grads["head_w"][idx], num), ("head_w", idx)
    num = _fd(loss, w["head_b"], (0,), h=1e-7)
    assert close(grads["head_b"][0], num)


def test_model_backward_a_token_outside_every_query_set_still_gets_its_gradient_through_the_keys():
    """A merged token older than the k sampled ones is not a query, but it is a key of the cross layer:
    its raw tokens' gradient is not zero; and a user's gradient does not depend on the other users."""
    cfg = synth.tiny_config(B=2, L=24, d=8, heads=2, m=2, K=4, k_recent=2, n_self=1, inner_layers=1)
    case = synth.make_case(cfg)
    w, H, G = case["weights"], case["H"], case["G"]
    labels = np.array([1.0, 0.0])
    _, _, dH, dG, _ = grd.model_backward(cfg, w, H, G, None, labels)
    assert np.abs(dH[0, :4]).max() > 0          # merged token 0 of 6: only ever a key
    one = cfg.replace(B=1)
    _, _, dH1, dG1, _ = grd.model_backward(one, w, H[1:], G[1:], None, labels[1:])
    # the mean of Eq. 2 runs over the batch: a batch of one user weighs it twice as much
    assert np.allclose(dH1[0], 2 * dH[1], rtol=1e-10, atol=1e-14) and np.allclose(dG1[0], 2 * dG[1], rtol=1e-10, atol=1e-14)


def test_model_backward_with_learnable_query_tokens_against_finite_differences():
    """Learnable query tokens (Section 3.5.1): the slots' rows are a parameter shared by all users; its
    gradient, and the gradients that reach H only through the keys of the cross layer."""
    cfg = synth.tiny_config(B=3, L=22, d=8, heads=2, m=2, K=4, k_recent=3, n_self=2, inner_layers=1,
                            q_learnable=True, ragged=True, len_lo=0, len_hi=22)
    case = synth.make_case(cfg)
    case["lens"][:] = [22, 0, 9]
    rng = np.random.default_rng(11)
    w = case["weights"]
    w = {"inner": [{k: np.asarray(v, dtype=np.float64) for k, v in b.items()} for b in w["inner"]],
         "cross": {k: np.asarray(v, dtype=np.float64) for k, v in w["cross"].items()},
         "self": [{k: np.asarray(v, dtype=np.float64) for k, v in b.items()} for b in w["self"]],
         "head_w": np.asarray(w["head_w"], dtype=np.float64), "head_b": np.asarray(w["head_b"], dtype=np.float64),
         "q_learn": np.asarray(w["q_learn"], dtype=np.float64)}
    H = np.asarray(case["H"], dtype=np.float64)
    G = np.asarray(case["G"], dtype=np.float64)
    lens = case["lens"]
    labels = np.array([1.0, 0.0, 1.0])

    def loss():
        return grd.bce_loss(orc.forward(cfg, w, H, G, lens)[1], labels)

    val, _, dH, dG, grads = grd.model_backward(cfg, w, H, G, lens, labels)
    assert abs(val - loss()) <= 1e-12

    def close(a, num):
        return abs(a - num) <= 2e-6 * max(1e-2, abs(num))

    for i in range(cfg.k_recent):
        for _ in range(3):
            j = int(rng.integers(0, cfg.d))
            num = _fd(loss, w["q_learn"], (i, j), h=1e-7)
            assert close(grads["q_learn"][i, j], num), ("q_learn", i, j, grads["q_learn"][i, j], num)
    for u in (0, 2):
        for _ in range(5):
            t, j = int(rng.integers(0, lens[u])), int(rng.integers(0, cfg.d))
            num = _fd(loss, H, (u, t, j), h=1e-7)
            assert close(dH[u, t, j], num), ("dH", u, t, j, dH[u, t, j], num)
    for key in ("wq", "wk", "wv", "w1"):
        p = w["cross"][key]
        idx = tuple(int(rng.integers(0, s)) for s in p.shape)
        assert close(grads["cross"][key][idx], _fd(loss, p, idx, h=1e-7)), key


def test_input_generation_backward_against_finite_differences():
    """Ragged users (one empty), NaN in the padding: every input and parameter of the input-generation
    stage against central differences of <input_generation(.), dH>."""
    cfg = synth.tiny_config(B=3, L=9, d=8, ragged=True, len_lo=0, len_hi=9)
    case = synth.make_input_case(cfg, 5)
    case["lens"][:] = [9, 0, 4]
    rng = np.random.default_rng(3)
    mlp = {k: np.asarray(v, dtype=np.float64) for k, v in case["mlp"].items()}
    E = np.asarray(case["E"], dtype=np.float64)
    td = np.asarray(case["tdiff"], dtype=np.float64)
    pos = np.arange(cfg.L)[None, :, None]
    E = np.where(pos < case["lens"][:, None, None], np.nan_to_num(E) + rng.standard_normal(E.shape), np.nan)
    td = np.where(pos < case["lens"][:, None, None], np.nan_to_num(td) + rng.standard_normal(td.shape), np.nan)
    lens = case["lens"]
    dH = rng.standard_normal((cfg.B, cfg.L, cfg.d))
    loss = lambda: float((orc.input_generation(cfg, mlp, E, td, lens) * dH).sum())
    dE, dtd, g = grd.input_generation_backward(cfg, mlp, E, td, lens, dH)
    assert (dE[1] == 0).all() and (dtd[1] == 0).all() and (dE[2, 4:] == 0).all() and (dtd[2, 4:] == 0).all()
    close = lambda a, num: abs(a - num) <= 2e-6 * max(1e-2, abs(num))
    for u in (0, 2):
        for _ in range(6):
            t = int(rng.integers(0, lens[u]))
            j = int(rng.integers(0, E.shape[-1])); k = int(rng.integers(0, td.shape[-1]))
            assert close(dE[u, t, j], _fd(loss, E, (u, t, j), h=1e-6)), ("dE", u, t, j)
            assert close(dtd[u, t, k], _fd(loss, td, (u, t, k), h=1e-6)), ("dtdiff", u, t, k)
    for key in ("pos", "w1", "b1", "w2", "b2"):
        p = mlp[key]
        for _ in range(4):
            idx = tuple(int(rng.integers(0, s)) for s in p.shape)
            assert close(g[key][idx], _fd(loss, p, idx, h=1e-6)), (key, idx, g[key][idx])
    assert (g["pos"][4:] != 0).any() and np.allclose(g["pos"][:4], dE[0, :4] + dE[2, :4])   # two users share positions 0..3
