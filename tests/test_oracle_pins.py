"""Pins for the CPU oracle: library routines, closed forms, values the paper
prints, brute force on tiny inputs and the model's invariants.  None of these
touch the HIP path."""
import math
import os

import numpy as np
import pytest
import torch

import longer_synth as synth
from oracle import longer_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if "=" in line:
                k, v = line.split("=")
                out[k.strip()] = float(v)
    return out


def _rng(seed):
    return np.random.default_rng(seed)


def _blk(seed, d):
    return synth.draw_block(_rng(seed), d)


# --------------------------------------------------------------------------- paper's printed numbers
def test_flops_worked_example_matches_paper():
    g = _golden("flops_worked_example.txt")
    L, d, K = int(g["L"]), int(g["d"]), int(g["K"])
    van = orc.flops_vanilla_layer(L, d)
    mer = orc.flops_merged_layer(L, d, K)
    assert round(van / 1e6) == g["vanilla_flops_M"]
    assert round(mer / 1e6) == g["merged_flops_M"]
    red = 100.0 * (1 - mer / van)
    assert abs(red - g["reduction_percent"]) < 0.06          # paper truncates 42.857 to 42.8
    assert math.isclose(mer / van, orc.merge_ratio(L, d, K), rel_tol=1e-12)


def test_table2_concat_ratios_follow_the_merge_formula():
    # the paper's Table 2 is a full model (several layers + non-attention parts), so only the
    # direction and rough size of the ratio can be compared with the single-layer formula
    g = _golden("flops_worked_example.txt")
    r4 = g["table2_merge4_concat"] / g["table2_no_merge"]
    r8 = g["table2_merge8_concat"] / g["table2_no_merge"]
    assert abs(r4 - orc.merge_ratio(2000, 32, 4)) < 0.02
    assert abs(r8 - orc.merge_ratio(2000, 32, 8)) < 0.02


@pytest.mark.parametrize("d", [8, 32, 128])
def test_block_owns_12d2_plus_13d_parameters(d):
    blk = _blk(1, d)
    assert orc.block_param_count(blk) == orc.params_vanilla_layer(d) == 12 * d * d + 13 * d
    assert orc.params_merged_layer(d, 4) == orc.params_vanilla_layer(4 * d)


def test_algorithmic_flops_of_a_full_block_reduces_to_eq3():
    # one inner layer over a single group of K = L tokens is exactly a vanilla layer over L tokens
    L, d = 16, 8
    cfg = synth.tiny_config(B=1, L=L, d=d, K=L, inner_layers=1, m=1, k_recent=1, n_self=0)
    fl = orc.algorithmic_flops(cfg)
    assert fl["inner"] == orc.flops_vanilla_layer(L, d)


def test_headline_flop_count():
    # 24 L d^2 N_in + 4 K d L N_in per user for the merge stage of the headline configuration
    cfg = synth.CONFIGS["C3"]
    fl = orc.algorithmic_flops(cfg, B=1)
    assert fl["inner"] == 2 * (24 * 2000 * 128 * 128 + 4 * 8 * 128 * 2000)
    assert abs(fl["total"] * 256 / 1e9 - 458.1) < 0.5


def test_scoring_flop_count_against_a_hand_count():
    # one candidate of the serving configuration (d = 256, m = 8 global rows, T = 625 cached merged
    # tokens, k = 64 cached slots in each of the 3 self layers, every global sees every global):
    #   per layer, projections + FFN of 8 rows (Eq. 3's 24 d^2 per token)  8 * 24 * 256^2 = 12 582 912
    #   first layer's attention, 4 d per query-key pair                    4 * 256 * 8 * (8 + 625) = 5 185 536
    #   a self layer's attention                                           4 * 256 * 8 * (8 + 64) = 589 824
    #   total 4 * 12 582 912 + 5 185 536 + 3 * 589 824 = 57 286 656
    cfg = synth.CONFIGS["C5"]
    assert orc.algorithmic_flops_score(cfg, cfg.T) == 57286656
    # fewer cached tokens than slots: the self layers see only the valid slots; no cached token at all
    assert orc.algorithmic_flops_score(cfg, 10) == 4 * 12582912 + 4 * 256 * 8 * (8 + 10) * 4
    assert orc.algorithmic_flops_score(cfg, 0) == 4 * 12582912 + 4 * 256 * 8 * 8 * 4
    # Eq. 8 read literally between the globals: 8 * 9 / 2 = 36 global pairs instead of 64
    causal = cfg.replace(gmask="causal")
    assert orc.algorithmic_flops_score(causal, cfg.T) == 57286656 - 4 * 4 * 256 * (64 - 36)


# --------------------------------------------------------------------------- library pins
def _torch_layer(blk, d, heads):
    layer = torch.nn.TransformerEncoderLayer(d, heads, 4 * d, dropout=0.0, activation="gelu",
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
    layer.eval()
    return layer


@pytest.mark.parametrize("d,heads,n", [(8, 2, 5), (32, 2, 4), (16, 1, 7)])
def test_block_equals_torch_encoder_layer(d, heads, n):
    blk = _blk(7, d)
    x = _rng(3).standard_normal((3, n, d))
    layer = _torch_layer(blk, d, heads)
    with torch.no_grad():
        ref = layer(torch.from_numpy(x)).numpy()
    got = orc.block(x, x, np.ones((3, n, n), bool), orc._f64(blk), heads, 1e-5, "gelu_erf")
    np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-12)


def test_block_with_key_padding_equals_torch():
    d, heads, n = 16, 2, 6
    blk = _blk(11, d)
    x = _rng(5).standard_normal((2, n, d))
    valid = np.array([[1, 1, 1, 1, 0, 0], [1, 1, 1, 1, 1, 1]], bool)
    layer = _torch_layer(blk, d, heads)
    # torch's fused fast path does not take padding masks on every build: use the plain path
    torch.backends.mha.set_fastpath_enabled(False)
    with torch.no_grad():
        ref = layer(torch.from_numpy(x), src_key_padding_mask=torch.from_numpy(~valid)).numpy()
    mask = valid[:, None, :] & np.ones((2, n, 1), bool)
    got = orc.block(x, x, mask, orc._f64(blk), heads, 1e-5, "gelu_erf")
    np.testing.assert_allclose(got[valid], ref[valid], rtol=1e-11, atol=1e-12)


def test_inner_transformer_equals_torch_layer_per_group():
    cfg = synth.tiny_config(B=2, L=16, d=8, K=4, inner_layers=2, inner_heads=2)
    blocks = [_blk(21, cfg.d), _blk(22, cfg.d)]
    H = _rng(9).standard_normal((cfg.B, cfg.L, cfg.d))
    Z = orc.inner_transformer(cfg, blocks, H)
    x = torch.from_numpy(H.reshape(cfg.B * cfg.T, cfg.K, cfg.d))
    with torch.no_grad():
        for b in blocks:
            x = _torch_layer(b, cfg.d, cfg.inner_heads)(x)
    np.testing.assert_allclose(Z.reshape(-1, cfg.K, cfg.d), x.numpy(), rtol=1e-10, atol=1e-11)
    M = orc.token_merge(cfg, blocks, H)
    np.testing.assert_allclose(M, x.numpy().reshape(cfg.B, cfg.T, cfg.K, cfg.d).mean(2), rtol=1e-10, atol=1e-11)


def test_inner_transformer_on_a_ragged_last_group_equals_torch_on_its_valid_tokens():
    """A group cut short by the user's length: its valid tokens attend to each other only, as if the
    group had that many tokens (torch's layer on the valid tokens alone); the rest of the group is zero
    and takes no part in the mean."""
    cfg = synth.tiny_config(B=2, L=12, d=8, K=4, inner_layers=2, inner_heads=2)
    blocks = [_blk(23, cfg.d), _blk(24, cfg.d)]
    H = _rng(10).standard_normal((cfg.B, cfg.L, cfg.d))
    lens = np.array([10, 5])                       # last groups hold 2 and 1 valid tokens
    Z = orc.inner_transformer(cfg, blocks, H, lens)
    M = orc.token_merge(cfg, blocks, H, lens)
    for u, (t, n) in enumerate([(2, 2), (1, 1)]):
        x = torch.from_numpy(H[u, t * cfg.K:t * cfg.K + n][None])
        with torch.no_grad():
            for b in blocks:
                x = _torch_layer(b, cfg.d, cfg.inner_heads)(x)
        np.testing.assert_allclose(Z[u, t, :n], x[0].numpy(), rtol=1e-10, atol=1e-11)
        assert (Z[u, t, n:] == 0).all() and (Z[u, t + 1:] == 0).all()
        np.testing.assert_allclose(M[u, t], x[0].numpy().mean(0), rtol=1e-10, atol=1e-11)
        assert (M[u, t + 1:] == 0).all()


def test_layernorm_and_gelu_equal_torch():
    x = _rng(2).standard_normal((5, 12)) * 3
    g, b = _rng(3).standard_normal(12), _rng(4).standard_normal(12)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (12,), torch.from_numpy(g), torch.from_numpy(b), 1e-5)
    np.testing.assert_allclose(orc.layer_norm(x, g, b, 1e-5), ref.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(orc.activation(x, "gelu_erf"), torch.nn.functional.gelu(torch.from_numpy(x)).numpy(),
                               rtol=1e-12, atol=1e-14)
    # closed-form points of the erf GELU
    assert orc.activation(np.array([0.0]), "gelu_erf")[0] == 0.0
    assert math.isclose(orc.activation(np.array([1.0]), "gelu_erf")[0], 0.5 * (1 + math.erf(1 / math.sqrt(2))))


# --------------------------------------------------------------------------- the mask against Eq. 8 as printed
def _eq8_mask_paper_order(m, Tu):
    """Eq. 8 literally: tokens numbered 1..m+Tu with the globals first, M_ij = 0 iff j >= i.
    The sequence part is numbered newest first (the only order under which 'j >= i' lets a
    sequence token see its own past and not its future)."""
    n = m + Tu
    return np.array([[j >= i for j in range(1, n + 1)] for i in range(1, n + 1)])


@pytest.mark.parametrize("m,T,Tu", [(2, 6, 6), (3, 5, 3), (1, 4, 4)])
def test_type_rule_is_eq8_after_index_mapping(m, T, Tu):
    keys = orc.key_tokens(m, T, Tu)
    got = orc._type_mask(keys, keys, "causal")                 # all tokens as queries
    paper = _eq8_mask_paper_order(m, Tu)
    # paper index of global a is a+1; of sequence token t (chronological) is m + (Tu - t)
    def pidx(tok):
        is_g, idx, _ = tok
        return idx if is_g else m + (Tu - 1 - idx)
    for qi, q in enumerate(keys):
        for ki, k in enumerate(keys):
            if not (q[2] and k[2]):
                assert not got[qi, ki]
                continue
            exp = paper[pidx(q), pidx(k)]
            if (not q[0]) and k[0]:
                exp = False       # text of Section 3.5.2: the sequence never sees the candidate side
            assert got[qi, ki] == exp, (q, k)
    full = orc._type_mask(keys, keys, "full")
    assert full[:m, :m].all() and (full[m:, :m] == False).all()
    np.testing.assert_array_equal(full[:, m:], got[:, m:])


def test_vectorised_mask_equals_scalar_rule():
    for gm in ("full", "causal"):
        q = orc.query_tokens(3, 4, 2)
        k = orc.key_tokens(3, 5, 2)
        got = orc._type_mask(q, k, gm)
        for i, (qg, qi, qv) in enumerate(q):
            for j, (kg, ki, kv) in enumerate(k):
                assert got[i, j] == (qv and kv and orc.visible(qg, qi, kg, ki, gm))


def test_cross_layer_equals_torch_mha_with_eq8_mask():
    """The whole first layer rebuilt from torch library modules with an explicit mask."""
    cfg = synth.tiny_config(B=1, L=20, d=16, heads=2, m=2, K=4, k_recent=3, gmask="causal")
    blk = _blk(31, cfg.d)
    G = _rng(1).standard_normal((1, cfg.m, cfg.d))
    M = _rng(2).standard_normal((1, cfg.T, cfg.d))
    X = orc.hybrid_cross_attn(cfg, blk, G, M)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    R = torch.cat([t(G[0]), t(M[0])], 0)
    O = torch.cat([t(G[0]), t(M[0, -cfg.k_recent:])], 0)
    ln = lambda x, g, b: torch.nn.functional.layer_norm(x, (cfg.d,), t(g), t(b), 1e-5)
    mha = torch.nn.MultiheadAttention(cfg.d, cfg.heads, dropout=0.0, bias=True, batch_first=True).double()
    with torch.no_grad():
        mha.in_proj_weight.copy_(torch.cat([t(blk["wq"]).T, t(blk["wk"]).T, t(blk["wv"]).T], 0))
        mha.in_proj_bias.copy_(torch.cat([t(blk["bq"]), t(blk["bk"]), t(blk["bv"])]))
        mha.out_proj.weight.copy_(t(blk["wo"]).T); mha.out_proj.bias.copy_(t(blk["bo"]))
    # mask rows: paper order index of each query; True = masked for torch
    full = _eq8_mask_paper_order(cfg.m, cfg.T)
    def pidx(is_g, idx):
        return idx if is_g else cfg.m + (cfg.T - 1 - idx)
    qtok = orc.query_tokens(cfg.m, cfg.k_recent, cfg.T)
    ktok = orc.key_tokens(cfg.m, cfg.T, cfg.T)
    allow = np.array([[full[pidx(q[0], q[1]), pidx(k[0], k[1])] and not ((not q[0]) and k[0]) for k in ktok] for q in qtok])
    with torch.no_grad():
        Rn, On = ln(R, blk["ln1_g"], blk["ln1_b"]), ln(O, blk["ln1_g"], blk["ln1_b"])
        a, _ = mha(On[None], Rn[None], Rn[None], attn_mask=torch.from_numpy(~allow), need_weights=False)
        x = O + a[0]
        hdn = torch.nn.functional.gelu(ln(x, blk["ln2_g"], blk["ln2_b"]) @ t(blk["w1"]) + t(blk["b1"]))
        ref = x + hdn @ t(blk["w2"]) + t(blk["b2"])
    np.testing.assert_allclose(X[0], ref.numpy(), rtol=1e-10, atol=1e-11)


# --------------------------------------------------------------------------- brute force
def _brute_attention_single_head(q, k, v, allow):
    """Eq. 7 with scalar loops: softmax(q k^T / sqrt(d) + M) v."""
    nq, d = len(q), len(q[0])
    out = [[0.0] * d for _ in range(nq)]
    for i in range(nq):
        sc = []
        for j in range(len(k)):
            if allow[i][j]:
                sc.append(sum(q[i][c] * k[j][c] for c in range(d)) / math.sqrt(d))
            else:
                sc.append(None)
        vis = [s for s in sc if s is not None]
        if not vis:
            continue
        mx = max(vis)
        den = sum(math.exp(s - mx) for s in vis)
        for j, s in enumerate(sc):
            if s is None:
                continue
            p = math.exp(s - mx) / den
            for c in range(d):
                out[i][c] += p * v[j][c]
    return out


def test_one_head_cross_layer_brute_force():
    """h = 1 is the paper's own Eq. 7 (scale 1/sqrt(d)); rebuilt with python scalars."""
    cfg = synth.tiny_config(B=1, L=12, d=4, heads=1, m=1, K=4, k_recent=2, gmask="full")
    blk = orc._f64(_blk(41, cfg.d))
    G = _rng(5).standard_normal((1, 1, 4))
    M = _rng(6).standard_normal((1, 3, 4))
    X = orc.hybrid_cross_attn(cfg, blk, G, M)

    def ln(row, g, b):
        mu = sum(row) / len(row)
        var = sum((x - mu) ** 2 for x in row) / len(row)
        return [(x - mu) / math.sqrt(var + 1e-5) * g[i] + b[i] for i, x in enumerate(row)]

    def lin(row, W, b):
        return [sum(row[i] * W[i][j] for i in range(len(row))) + b[j] for j in range(len(b))]

    R = [list(G[0, 0])] + [list(r) for r in M[0]]
    O = [list(G[0, 0]), list(M[0, 1]), list(M[0, 2])]
    # visibility written out by hand: global sees everything; slot t=1 sees merged 0,1; slot t=2 sees 0,1,2
    allow = [[True, True, True, True], [False, True, True, False], [False, True, True, True]]
    Rn = [ln(r, blk["ln1_g"], blk["ln1_b"]) for r in R]
    On = [ln(r, blk["ln1_g"], blk["ln1_b"]) for r in O]
    q = [lin(r, blk["wq"], blk["bq"]) for r in On]
    k = [lin(r, blk["wk"], blk["bk"]) for r in Rn]
    v = [lin(r, blk["wv"], blk["bv"]) for r in Rn]
    att = _brute_attention_single_head(q, k, v, allow)
    for i in range(3):
        x = [O[i][c] + y for c, y in enumerate(lin(att[i], blk["wo"], blk["bo"]))]
        hpre = lin(ln(x, blk["ln2_g"], blk["ln2_b"]), blk["w1"], blk["b1"])
        hid = [0.5 * z * (1 + math.erf(z / math.sqrt(2))) for z in hpre]
        y = [x[c] + z for c, z in enumerate(lin(hid, blk["w2"], blk["b2"]))]
        np.testing.assert_allclose(X[0, i], y, rtol=1e-11, atol=1e-12)


# --------------------------------------------------------------------------- invariants
def _identity_block(d, seed=0):
    blk = _blk(seed, d)
    for z in ("wo", "bo", "w2", "b2"):
        blk[z] = np.zeros_like(blk[z])
    return blk


def test_I1_K1_identity_inner_is_noop():
    cfg = synth.tiny_config(B=2, L=7, d=8, K=1)
    H = _rng(1).standard_normal((2, 7, 8))
    M = orc.token_merge(cfg, [_identity_block(8)], H)
    assert np.array_equal(M, H)


def test_I6_identity_inner_pools_valid_rows():
    cfg = synth.tiny_config(B=2, L=10, d=8, K=4)
    H = _rng(1).standard_normal((2, 10, 8))
    lens = np.array([10, 5])
    M = orc.token_merge(cfg, [_identity_block(8)], H, lens)
    np.testing.assert_allclose(M[0, 2], H[0, 8:10].mean(0), rtol=1e-14)     # ragged last group of L
    np.testing.assert_allclose(M[1, 1], H[1, 4], rtol=1e-14)               # one valid token
    np.testing.assert_allclose(M[1, 0], H[1, 0:4].mean(0), rtol=1e-14)
    assert (M[1, 2] == 0).all()


# --------------------------------------------------------------------------- merge by concatenation
def test_concat_merge_lays_torch_group_outputs_side_by_side():
    """Section 3.4, merge by concatenation after InnerTrans: the merged token of a group is its K
    block outputs side by side, oldest first (the block itself against torch's encoder layer)."""
    cfg = synth.tiny_config(B=2, L=16, d=32, K=4, inner_layers=2, inner_heads=2, merge="concat")
    assert cfg.d_in == 8
    blocks = [_blk(31, cfg.d_in), _blk(32, cfg.d_in)]
    H = _rng(19).standard_normal((cfg.B, cfg.L, cfg.d_in))
    x = torch.from_numpy(H.reshape(cfg.B * cfg.T, cfg.K, cfg.d_in))
    with torch.no_grad():
        for b in blocks:
            x = _torch_layer(b, cfg.d_in, cfg.inner_heads)(x)
    ref = x.numpy().reshape(cfg.B, cfg.T, cfg.K, cfg.d_in)
    M = orc.token_merge(cfg, blocks, H)
    assert M.shape == (cfg.B, cfg.T, cfg.d)
    for j in range(cfg.K):      # slot j of the merged token = output of the group's j-th token
        np.testing.assert_allclose(M[:, :, j * cfg.d_in:(j + 1) * cfg.d_in], ref[:, :, j], rtol=1e-10, atol=1e-11)


def test_concat_merge_identity_inner_is_a_reshape_with_zero_padding():
    cfg = synth.tiny_config(B=2, L=10, d=32, K=4, merge="concat")
    H = _rng(2).standard_normal((2, 10, 8))
    Hn = H.copy(); Hn[1, 5:] = np.nan
    M = orc.token_merge(cfg, [_identity_block(8)], Hn, np.array([10, 5]))
    assert np.array_equal(M[0, :2].reshape(8, 8), H[0, :8])
    assert np.array_equal(M[0, 2, :16].reshape(2, 8), H[0, 8:10]) and (M[0, 2, 16:] == 0).all()   # ragged last group of L
    assert np.array_equal(M[1, 1, :8], H[1, 4]) and (M[1, 1, 8:] == 0).all() and (M[1, 2] == 0).all()
    # K = 1: concatenation of one token is the token
    cfg1 = synth.tiny_config(B=2, L=7, d=8, K=1, merge="concat")
    H1 = _rng(3).standard_normal((2, 7, 8))
    assert np.array_equal(orc.token_merge(cfg1, [_identity_block(8)], H1), H1)


def test_concat_main_stack_has_eq4_parameters_and_ratio_flops():
    """Eq. 4: a layer of the main stack at the merged width K d owns 12 K^2 d^2 + 13 K d
    parameters; the complexity ratio's numerator is Eq. 3 at (L / K, K d)."""
    cfg = synth.tiny_config(B=1, L=2048, d=128, K=4, heads=2, merge="concat", inner_layers=1, n_self=1)
    w = synth.draw_weights(cfg)
    assert cfg.d_in == 32
    assert orc.block_param_count(w["cross"]) == orc.params_merged_layer(cfg.d_in, cfg.K) == 12 * 16 * 1024 + 13 * 128
    assert orc.block_param_count(w["inner"][0]) == orc.params_vanilla_layer(32)
    assert orc.flops_vanilla_layer(2048 // 4, 4 * 32) == orc.flops_merged_layer(2048, 32, 4)
    # the counter: a full-length user, all T merged tokens as queries of one self layer over
    # [m globals; T tokens] -- compare its GEMM part with 24 (m + T) (K d)^2
    cfgq = cfg.replace(k_recent=cfg.T)
    fl = orc.algorithmic_flops(cfgq)
    n = cfgq.m + cfgq.T
    causal_pairs = cfgq.m * cfgq.m + cfgq.m * cfgq.T + cfgq.T * (cfgq.T + 1) // 2
    assert fl["self_each"] == 24 * n * 128 * 128 + 4 * 128 * causal_pairs
    assert fl["inner"] == 2048 * 24 * 32 * 32 + 4 * 32 * (2048 // 4) * 16


def test_concat_forward_padding_and_cache_invariants():
    cfg = synth.tiny_config(B=2, L=23, d=16, K=4, heads=2, m=2, k_recent=3, n_self=2, inner_heads=1, merge="concat")
    w, H, G = _case(cfg)
    assert H.shape[-1] == 4 and w["inner"][0]["wq"].shape == (4, 4) and w["cross"]["wq"].shape == (16, 16)
    lens = np.array([23, 14])
    Y, lg = orc.forward(cfg, w, H, G, lens)
    Hn = H.copy(); Hn[1, 14:] = np.nan
    Yn, lgn = orc.forward(cfg, w, Hn, G, lens)
    assert np.array_equal(Y, Yn) and np.array_equal(lg, lgn)
    # forward = merge, then the same cross / self layers as in mean mode over M
    M = orc.token_merge(cfg, w["inner"], H, lens)
    X = orc.hybrid_cross_attn(cfg.replace(merge="mean"), w["cross"], G, M, lens, L=cfg.L)
    for blk in w["self"]:
        X = orc.self_attn_layer(cfg.replace(merge="mean"), blk, X, lens, L=cfg.L)
    assert np.array_equal(X, Y)
    # serving: scoring against the cache equals the full forward pass per candidate
    rng = _rng(5)
    Gc = rng.standard_normal((cfg.B, 3, cfg.m, cfg.d))
    cache = orc.kv_cache_build(cfg, w, H, lens)
    Yg, lgs = orc.score_candidates(cfg, w, cache, Gc)
    for c in range(3):
        Yc, lc = orc.forward(cfg, w, H, Gc[:, c], lens)
        np.testing.assert_allclose(Yg[:, c], Yc[:, :cfg.m], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(lgs[:, c], lc, rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------- input generation
def test_input_generation_equals_torch_mlp_on_concatenated_inputs():
    """Section 3.5.1: position added to the item embedding, time-difference feature concatenated,
    then an MLP -- rebuilt from torch.nn modules."""
    cfg = synth.tiny_config(B=3, L=9, d=16, ragged=True, len_lo=0, len_hi=9)
    case = synth.make_input_case(cfg, d_e=12)
    mlp, E, td = case["mlp"], case["E"], case["tdiff"]
    lens = np.array([9, 4, 0])
    H = orc.input_generation(cfg, mlp, E, td, lens)
    lin1, lin2 = torch.nn.Linear(16, 64).double(), torch.nn.Linear(64, 16).double()
    with torch.no_grad():
        lin1.weight.copy_(torch.from_numpy(mlp["w1"].astype(np.float64).T)); lin1.bias.copy_(torch.from_numpy(mlp["b1"].astype(np.float64)))
        lin2.weight.copy_(torch.from_numpy(mlp["w2"].astype(np.float64).T)); lin2.bias.copy_(torch.from_numpy(mlp["b2"].astype(np.float64)))
        net = torch.nn.Sequential(lin1, torch.nn.GELU(), lin2)
        for u in range(3):
            n = lens[u]
            x = torch.cat([torch.from_numpy(E[u, :n].astype(np.float64)) + torch.from_numpy(mlp["pos"][:n].astype(np.float64)),
                           torch.from_numpy(td[u, :n].astype(np.float64))], dim=1)
            np.testing.assert_allclose(H[u, :n], net(x).numpy(), rtol=1e-12, atol=1e-13)
            assert (H[u, n:] == 0).all()          # padded rows (NaN in the inputs) come out as zeros
    assert np.isfinite(H).all()
    # the position embedding is indexed by the token's position, not by anything user-specific
    H2 = orc.input_generation(cfg, mlp, np.roll(E, 1, axis=0), np.roll(td, 1, axis=0), np.roll(lens, 1))
    np.testing.assert_array_equal(H2, np.roll(H, 1, axis=0))


# --------------------------------------------------------------------------- query sampling strategies
def test_uniform_slots_are_evenly_spaced_increasing_and_end_at_the_newest_older_token():
    for Tu, k, ku in [(250, 100, 100), (250, 100, 50), (613, 64, 64), (101, 100, 37), (40, 8, 3)]:
        idx = [orc.slot_index(i, k, Tu, ku) for i in range(k)]
        r = k - ku
        assert idx[ku:] == list(range(Tu - r, Tu))                   # the recent part
        uni = np.array(idx[:ku])
        rest = Tu - r
        assert uni[-1] == rest - 1 and uni[0] >= 0 and (np.diff(uni) >= 1).all()
        gaps = np.diff(np.concatenate([[-1], uni]))                  # share sizes
        assert gaps.max() - gaps.min() <= 1 and gaps.sum() == rest
    # closed form when the share size is a whole number: every (rest / ku)-th token
    assert [orc.slot_index(i, 4, 20, 4) for i in range(4)] == [4, 9, 14, 19]
    assert [orc.slot_index(i, 6, 23, 4) for i in range(6)] == [4, 9, 14, 20, 21, 22]
    # no more tokens than slots: all of them, right-aligned, whatever the strategy
    assert [orc.slot_index(i, 5, 3, 5) for i in range(5)] == [-2, -1, 0, 1, 2]
    assert [orc.slot_index(i, 5, 5, 2) for i in range(5)] == [0, 1, 2, 3, 4]


def test_sampled_queries_follow_the_scalar_rule_and_eq8():
    """A uniformly sampled query sees exactly the keys Eq. 8 allows its token (mask rebuilt from the
    printed rule in paper order); gather and mask against scalar loops."""
    m, T, Tu, k, ku = 2, 11, 11, 4, 4
    cfg = synth.tiny_config(B=1, L=T * 2, d=8, K=2, m=m, k_recent=k, k_uniform=ku, gmask="causal", heads=1)
    q = orc.query_tokens(m, k, Tu, ku)
    assert [t for (_, t, _) in q[m:]] == [1, 4, 7, 10]
    keys = orc.key_tokens(m, T, Tu)
    got = orc._type_mask(q, keys, "causal")
    paper = _eq8_mask_paper_order(m, Tu)
    pidx = lambda tok: tok[1] if tok[0] else m + (Tu - 1 - tok[1])
    for qi, qq in enumerate(q):
        for ki, kk in enumerate(keys):
            exp = paper[pidx(qq), pidx(kk)] and not ((not qq[0]) and kk[0])
            assert got[qi, ki] == exp
    # the whole layer: each query row computed alone, one head, scalar softmax over its visible keys
    blk = orc._f64(_blk(41, 8))
    G = _rng(1).standard_normal((1, m, 8)); M = _rng(2).standard_normal((1, T, 8))
    X = orc.hybrid_cross_attn(cfg, blk, G, M)
    R = np.concatenate([G[0], M[0]], 0)
    Rn = orc.layer_norm(R, blk["ln1_g"], blk["ln1_b"], 1e-5)
    Kp, Vp = Rn @ blk["wk"] + blk["bk"], Rn @ blk["wv"] + blk["bv"]
    for si, t in enumerate([1, 4, 7, 10]):
        x = M[0, t]
        qv = orc.layer_norm(x[None], blk["ln1_g"], blk["ln1_b"], 1e-5)[0] @ blk["wq"] + blk["bq"]
        vis = [m + tt for tt in range(t + 1)]                         # own past and itself, no globals
        sc = np.array([qv @ Kp[j] / math.sqrt(8) for j in vis])
        pr = np.exp(sc - sc.max()); pr /= pr.sum()
        a = sum(pj * Vp[j] for pj, j in zip(pr, vis))
        y = x + a @ blk["wo"] + blk["bo"]
        h = orc.activation(orc.layer_norm(y[None], blk["ln2_g"], blk["ln2_b"], 1e-5)[0] @ blk["w1"] + blk["b1"], "gelu_erf")
        y = y + h @ blk["w2"] + blk["b2"]
        np.testing.assert_allclose(X[0, m + si], y, rtol=1e-11, atol=1e-12)


def test_sampling_strategies_reduce_to_recent_and_keep_the_invariants():
    base = synth.tiny_config(B=2, L=46, d=8, K=2, m=2, k_recent=6, n_self=2)
    w, H, G = _case(base)
    lens = np.array([46, 9])                 # second user: 5 merged tokens < 6 slots
    Y0, l0 = orc.forward(base, w, H, G, lens)
    Yz, lz = orc.forward(base.replace(k_uniform=0), w, H, G, lens)
    assert np.array_equal(Y0, Yz)
    for ku in (6, 3):
        cfg = base.replace(k_uniform=ku)
        Y, lgt = orc.forward(cfg, w, H, G, lens)
        assert not np.allclose(Y[0], Y0[0])
        assert np.array_equal(Y[1], Y0[1])   # a user with no more tokens than slots keeps all of them
        # a sampled row does not change when tokens newer than its own token change
        t_first = orc.slot_index(0, 6, 23, ku)
        H2 = H.copy(); H2[0, 2 * (t_first + 1):] += _rng(9).standard_normal(H2[0, 2 * (t_first + 1):].shape)
        Y2, _ = orc.forward(cfg, w, H2, G, lens)
        assert np.array_equal(Y2[0, cfg.m], Y[0, cfg.m]) and not np.allclose(Y2[0, cfg.m + 1], Y[0, cfg.m + 1])
        # serving: cached scoring equals the full pass
        Gc = _rng(4).standard_normal((2, 2, cfg.m, cfg.d))
        cache = orc.kv_cache_build(cfg, w, H, lens)
        Yg, lgs = orc.score_candidates(cfg, w, cache, Gc)
        for c in range(2):
            Yc, lc = orc.forward(cfg, w, H, Gc[:, c], lens)
            np.testing.assert_allclose(Yg[:, c], Yc[:, :cfg.m], rtol=1e-12, atol=1e-13)
    # every token sampled (k = T_u): the cross layer is a self layer, for any split
    cfgT = synth.tiny_config(B=2, L=16, d=8, K=4, m=2, k_recent=4, k_uniform=4)
    blk = _blk(3, 8)
    Gt = _rng(1).standard_normal((2, 2, 8)); Mt = _rng(2).standard_normal((2, 4, 8))
    np.testing.assert_allclose(orc.hybrid_cross_attn(cfgT, blk, Gt, Mt),
                               orc.self_attn_layer(cfgT, blk, np.concatenate([Gt, Mt], 1)), rtol=1e-13, atol=1e-14)


# --------------------------------------------------------------------------- learnable query tokens
def _torch_block_with_mask(blk, d, heads, O, R, allow):
    """One pre-LN block built from torch library modules: queries O [nq, d] over R [nk, d]
    under the boolean visibility ``allow`` [nq, nk]."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    ln = lambda x, g, b: torch.nn.functional.layer_norm(x, (d,), t(g), t(b), 1e-5)
    mha = torch.nn.MultiheadAttention(d, heads, dropout=0.0, bias=True, batch_first=True).double()
    with torch.no_grad():
        mha.in_proj_weight.copy_(torch.cat([t(blk["wq"]).T, t(blk["wk"]).T, t(blk["wv"]).T], 0))
        mha.in_proj_bias.copy_(torch.cat([t(blk["bq"]), t(blk["bk"]), t(blk["bv"])]))
        mha.out_proj.weight.copy_(t(blk["wo"]).T); mha.out_proj.bias.copy_(t(blk["bo"]))
        On, Rn = ln(t(O), blk["ln1_g"], blk["ln1_b"]), ln(t(R), blk["ln1_g"], blk["ln1_b"])
        a, _ = mha(On[None], Rn[None], Rn[None], attn_mask=torch.from_numpy(~np.asarray(allow)), need_weights=False)
        x = t(O) + a[0]
        hdn = torch.nn.functional.gelu(ln(x, blk["ln2_g"], blk["ln2_b"]) @ t(blk["w1"]) + t(blk["b1"]))
        return (x + hdn @ t(blk["w2"]) + t(blk["b2"])).numpy()


def test_learnable_queries_equal_torch_layers_with_the_masks_written_out():
    """First layer: [G; P] over [G; the user's valid merged tokens] -- a learnable slot sees every
    valid sequence token and no global; self layer: slots causal in slot order.  Both rebuilt
    from torch modules on the valid tokens only, masks written by hand."""
    m, k, d, K = 2, 3, 16, 4
    cfg = synth.tiny_config(B=2, L=24, d=d, heads=2, m=m, K=K, k_recent=k, q_learnable=True)
    blk, blk2 = _blk(31, d), _blk(32, d)
    G = _rng(1).standard_normal((2, m, d)); M = _rng(2).standard_normal((2, cfg.T, d))
    P = _rng(3).standard_normal((k, d))
    lens = np.array([24, 10])                                   # 6 and 3 valid merged tokens
    X = orc.hybrid_cross_attn(cfg, blk, G, M, lens, q_learn=P)
    Y = orc.self_attn_layer(cfg, blk2, X, lens)
    for u, Tu in enumerate((6, 3)):
        R = np.concatenate([G[u], M[u, :Tu]], 0)
        O = np.concatenate([G[u], P], 0)
        allow = np.zeros((m + k, m + Tu), dtype=bool)
        allow[:m, :] = True                                     # globals: everything (gmask full)
        allow[m:, m:] = True                                    # learnable slots: every valid sequence token
        ref = _torch_block_with_mask(blk, d, 2, O, R, allow)
        np.testing.assert_allclose(X[u], ref, rtol=1e-10, atol=1e-11)
        allow2 = np.zeros((m + k, m + k), dtype=bool)
        allow2[:m, :] = True
        for i in range(k):
            allow2[m + i, m:m + i + 1] = True                   # slot i: slots 0..i
        ref2 = _torch_block_with_mask(blk2, d, 2, ref, ref, allow2)
        np.testing.assert_allclose(Y[u], ref2, rtol=1e-10, atol=1e-11)


def test_learnable_query_descriptors_and_invariants():
    # descriptors against the rule written out: Eq. 8 for a token placed after the newest one
    q = orc.query_tokens(1, 3, 4, learnable=True)
    assert q[1:] == [(False, 4, True), (False, 5, True), (False, 6, True)]
    got = orc._type_mask(q, orc.key_tokens(1, 6, 4), "full")
    exp = np.array([[1, 1, 1, 1, 1, 0, 0]] + [[0, 1, 1, 1, 1, 0, 0]] * 3, dtype=bool)
    np.testing.assert_array_equal(got, exp)
    np.testing.assert_array_equal(orc._type_mask(q, q, "full"),
                                  np.array([[1, 1, 1, 1], [0, 1, 0, 0], [0, 1, 1, 0], [0, 1, 1, 1]], dtype=bool))
    assert all(not t[2] for t in orc.query_tokens(0, 3, 0, learnable=True))

    cfg = synth.tiny_config(B=3, L=24, d=8, K=4, m=2, k_recent=3, n_self=2, q_learnable=True)
    w, H, G = _case(cfg)
    assert w["q_learn"].shape == (3, 8)
    lens = np.array([24, 9, 0])
    Y, lg = orc.forward(cfg, w, H, G, lens)
    assert (Y[2, cfg.m:] == 0).all() and np.abs(Y[:2, cfg.m:]).min() > 0     # an empty user has no valid slot
    # the slots carry no position: their rows do not change when the valid merged tokens are reordered
    blk = w["cross"]
    M = _rng(5).standard_normal((1, 6, 8))
    perm = np.array([3, 0, 5, 1, 4, 2])
    Xa = orc.hybrid_cross_attn(cfg, blk, G[:1], M, q_learn=w["q_learn"])
    Xb = orc.hybrid_cross_attn(cfg, blk, G[:1], M[:, perm], q_learn=w["q_learn"])
    np.testing.assert_allclose(Xa, Xb, rtol=1e-12, atol=1e-13)
    # ... nor with the global tokens; and they differ from the sampled queries' rows
    Xc = orc.hybrid_cross_attn(cfg, blk, G[1:2], M, q_learn=w["q_learn"])
    assert np.array_equal(Xa[0, cfg.m:], Xc[0, cfg.m:])
    Xs = orc.hybrid_cross_attn(cfg.replace(q_learnable=False), blk, G[:1], M)
    np.testing.assert_allclose(Xs[0, :cfg.m], Xa[0, :cfg.m], rtol=1e-12, atol=1e-13)   # globals see the same keys
    assert not np.allclose(Xs[0, cfg.m:], Xa[0, cfg.m:])
    # padded tokens are never read
    H2 = H.copy(); H2[1, 9:] = np.nan
    Y2, lg2 = orc.forward(cfg, w, H2, G, lens)
    assert np.array_equal(Y2, Y) and np.array_equal(lg2, lg)
    # serving: cached scoring equals the full pass
    Gc = _rng(4).standard_normal((3, 2, cfg.m, cfg.d))
    cache = orc.kv_cache_build(cfg, w, H, lens)
    Yg, lgs = orc.score_candidates(cfg, w, cache, Gc)
    for c in range(2):
        Yc, lc = orc.forward(cfg, w, H, Gc[:, c], lens)
        np.testing.assert_allclose(Yg[:, c], Yc[:, :cfg.m], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(lgs[:, c], lc, rtol=1e-12, atol=1e-13)
    # FLOP count: k valid slots each paired with all T_u keys, for users with a token
    f = orc.algorithmic_flops(cfg, lens)
    f0 = orc.algorithmic_flops(cfg.replace(q_learnable=False), lens)
    d, k = cfg.d, cfg.k_recent
    extra_pairs = (3 * 6 - (4 + 5 + 6)) + 0 + 0            # user 0: recent slots see 4, 5, 6 keys; user 1: 3 tokens = 3 slots, sees 1, 2, 3
    extra_pairs += (3 * 3 - (1 + 2 + 3))
    assert f["cross"] - f0["cross"] == 4 * d * extra_pairs


def test_I2_all_tokens_as_queries_is_self_attention():
    for gm in ("full", "causal"):
        cfg = synth.tiny_config(B=2, L=16, d=8, K=4, m=2, k_recent=4, gmask=gm)      # k = T
        blk = _blk(3, 8)
        G = _rng(1).standard_normal((2, 2, 8))
        M = _rng(2).standard_normal((2, 4, 8))
        a = orc.hybrid_cross_attn(cfg, blk, G, M)
        b = orc.self_attn_layer(cfg, blk, np.concatenate([G, M], 1))
        np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-14)


def test_I3_softmax_rows_sum_to_one_and_masked_are_zero():
    cfg = synth.tiny_config(B=2, L=24, d=8, K=4, m=2, k_recent=3)
    blk = _blk(3, 8)
    G = _rng(1).standard_normal((2, 2, 8))
    M = _rng(2).standard_normal((2, 6, 8))
    lens = np.array([24, 9])
    probs = []
    orc.hybrid_cross_attn(cfg, blk, G, M, lens, probs_out=probs)
    assert len(probs) == 2 * cfg.heads
    for u in range(2):
        Tu = orc.merged_len(lens[u], cfg.K)
        mask = orc._type_mask(orc.query_tokens(2, 3, Tu), orc.key_tokens(2, 6, Tu), "full")
        for h in range(cfg.heads):
            p = probs[u * cfg.heads + h]
            assert (p[~mask] == 0).all()
            rows = mask.any(1)
            assert np.abs(p[rows].sum(1) - 1).max() < 1e-12
            assert (p[~rows] == 0).all()


def _case(cfg, seed=0):
    rng = _rng(seed)
    w = synth.draw_weights(cfg, rng)
    H = rng.standard_normal((cfg.B, cfg.L, cfg.d_in))
    G = rng.standard_normal((cfg.B, cfg.m, cfg.d))
    return w, H, G


@pytest.mark.parametrize("gm", ["full", "causal"])
def test_I4_kv_cache_scoring_equals_full_recompute(gm):
    cfg = synth.tiny_config(B=2, L=27, d=8, K=4, m=2, k_recent=3, n_self=2, gmask=gm)
    w, H, G = _case(cfg)
    lens = np.array([27, 6])          # second user has fewer merged tokens (2) than query slots (3)
    C = 3
    Gc = _rng(9).standard_normal((2, C, cfg.m, cfg.d))
    cache = orc.kv_cache_build(cfg, w, H, lens)
    Yg, logits = orc.score_candidates(cfg, w, cache, Gc)
    for c in range(C):
        Y, lg = orc.forward(cfg, w, H, Gc[:, c], lens)
        np.testing.assert_allclose(Yg[:, c], Y[:, :cfg.m], rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(logits[:, c], lg, rtol=1e-11, atol=1e-12)
    # sequence-side rows do not depend on the candidate
    Y0, _ = orc.forward(cfg, w, H, Gc[:, 0], lens)
    Y1, _ = orc.forward(cfg, w, H, Gc[:, 1], lens)
    assert np.array_equal(Y0[:, cfg.m:], Y1[:, cfg.m:])
    assert not np.allclose(Y0[:, :cfg.m], Y1[:, :cfg.m])


def test_I5_padding_and_causality():
    cfg = synth.tiny_config(B=1, L=23, d=8, K=4, m=2, k_recent=3, n_self=1)
    w, H, G = _case(cfg)
    lens = np.array([14])
    Y, lg = orc.forward(cfg, w, H, G, lens)
    Hn = H.copy(); Hn[0, 14:] = np.nan
    Yn, lgn = orc.forward(cfg, w, Hn, G, lens)
    assert np.array_equal(Y, Yn) and np.array_equal(lg, lgn)
    # same user stored without padding
    cfg2 = cfg.replace(L=14)
    Y2, lg2 = orc.forward(cfg2, w, H[:, :14], G, None)
    np.testing.assert_allclose(Y, Y2, rtol=1e-13, atol=1e-14)
    # a sequence row does not change when newer raw tokens change
    M = orc.token_merge(cfg, w["inner"], H, lens)
    X = orc.hybrid_cross_attn(cfg, w["cross"], G, M, lens, L=cfg.L)
    H3 = H.copy(); H3[0, 12:14] += _rng(77).standard_normal((2, cfg.d))   # last (ragged) group = merged token 3 = newest slot
    # (a constant shift would be invisible: LayerNorm removes it)
    M3 = orc.token_merge(cfg, w["inner"], H3, lens)
    X3 = orc.hybrid_cross_attn(cfg, w["cross"], G, M3, lens, L=cfg.L)
    assert np.array_equal(X[0, cfg.m:cfg.m + 2], X3[0, cfg.m:cfg.m + 2])
    assert not np.allclose(X[0, cfg.m + 2], X3[0, cfg.m + 2])
    assert not np.allclose(X[0, 0], X3[0, 0])    # globals see the whole sequence


def test_short_user_has_invalid_zero_slots():
    cfg = synth.tiny_config(B=1, L=12, d=8, K=4, m=2, k_recent=5, n_self=1)
    w, H, G = _case(cfg)
    Y, _ = orc.forward(cfg, w, H, G, np.array([7]))     # 2 merged tokens < 5 slots
    assert (Y[0, 2:5] == 0).all() and np.abs(Y[0, 5:]).min() > 0


def test_head_is_a_dot_product():
    cfg = synth.tiny_config()
    hw = _rng(1).standard_normal(cfg.m * cfg.d)
    hb = np.array([0.25])
    Yg = _rng(2).standard_normal((3, cfg.m, cfg.d))
    lg = orc.head_logits(cfg, hw, hb, Yg)
    for i in range(3):
        assert math.isclose(lg[i], sum(a * b for a, b in zip(hw, Yg[i].ravel())) + 0.25, rel_tol=1e-12)


# --------------------------------------------------------------------------- input generator
def test_bf16_rounding_is_nearest_even_and_idempotent():
    x = np.array([1.0, 1.00390625, 1.005859375, -3.14159, 1e-30, 65504.0], dtype=np.float32)
    r = synth.round_bf16(x)
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(r, t)
    assert np.array_equal(synth.round_bf16(r), r)
    assert np.array_equal(synth.bits_to_f32(synth.bf16_bits(r)), r)


def test_cases_are_seeded_and_shaped():
    a = synth.make_case(synth.CONFIGS["C1"])
    b = synth.make_case(synth.CONFIGS["C1"])
    assert np.array_equal(a["H"], b["H"]) and a["H"].shape == (4, 64, 32)
    assert np.array_equal(a["weights"]["cross"]["w1"], b["weights"]["cross"]["w1"])
    c4 = synth.make_case(synth.CONFIGS["C4"], users=3, pad_value=float("nan"))
    assert c4["lens"].min() >= 100 and c4["lens"].max() <= 5000
    assert np.isnan(c4["H"][0, c4["lens"][0]:]).all() and not np.isnan(c4["H"][0, :c4["lens"][0]]).any()
    assert np.array_equal(synth.round_bf16(c4["G"]), c4["G"])


# --------------------------------------------------------------------------- invariants over random small configurations
def _random_tiny(seed):
    rng = np.random.default_rng(9000 + seed)
    K = int(rng.choice([1, 2, 4]))
    merge = "concat" if (K > 1 and rng.random() < 0.4) else "mean"
    d_raw = int(rng.choice([4, 8]))
    d = d_raw * K if merge == "concat" else d_raw
    heads = int(rng.choice([1, 2]))
    k = int(rng.integers(1, 7))
    learn = bool(rng.random() < 0.3)
    ku = 0 if learn else int(rng.integers(0, k + 1))
    return synth.tiny_config(B=3, L=int(rng.integers(K, 9 * K)), d=d, heads=heads, inner_heads=int(rng.choice([1, 2])),
                             m=int(rng.integers(1, 4)), K=K, k_recent=k, k_uniform=ku, q_learnable=learn, merge=merge,
                             n_self=int(rng.integers(0, 3)), inner_layers=int(rng.integers(1, 3)),
                             gmask=str(rng.choice(["full", "causal"])), act=str(rng.choice(["gelu_erf", "relu"])),
                             ffn_mult=int(rng.choice([1, 4])), index=200 + seed)


@pytest.mark.parametrize("seed", range(12))
def test_invariants_hold_for_random_small_configurations(seed):
    """What must hold whatever the configuration (merge mode, query strategy, masks, layer counts):
    users are independent, padded storage is never read, a token cannot see its future, and the
    two-stage serving path equals the full pass."""
    cfg = _random_tiny(seed)
    rng = _rng(300 + seed)
    w = synth.draw_weights(cfg, rng)
    H = rng.standard_normal((cfg.B, cfg.L, cfg.d_in))
    G = rng.standard_normal((cfg.B, cfg.m, cfg.d))
    lens = rng.integers(0, cfg.L + 1, size=cfg.B)
    lens[0] = cfg.L
    Y, lg = orc.forward(cfg, w, H, G, lens)
    assert np.isfinite(Y).all() and np.isfinite(lg).all()
    # users are independent: any user alone gives the same rows
    for u in range(cfg.B):
        Yu, lu = orc.forward(cfg.replace(B=1), w, H[u:u + 1], G[u:u + 1], lens[u:u + 1])
        np.testing.assert_allclose(Yu[0], Y[u], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(lu[0], lg[u], rtol=1e-12, atol=1e-13)
    # padded storage is never read, and a longer padded length changes nothing
    Hn = H.copy()
    for u in range(cfg.B):
        Hn[u, lens[u]:] = np.nan
    Yn, _ = orc.forward(cfg, w, Hn, G, lens)
    assert np.array_equal(Yn, Y)
    Hp = np.concatenate([H, rng.standard_normal((cfg.B, 2 * cfg.K, cfg.d_in))], axis=1)
    for u in range(cfg.B):
        Hp[u, lens[u]:] = 0.0
    Yp, lp = orc.forward(cfg.replace(L=cfg.L + 2 * cfg.K), w, Hp, G, lens)
    np.testing.assert_allclose(Yp, Y, rtol=1e-12, atol=1e-13)
    # sequence-side rows never depend on the global tokens (what makes the KV cache valid)
    Y2, _ = orc.forward(cfg, w, H, G + 1.0, lens)
    assert np.array_equal(Y2[:, cfg.m:], Y[:, cfg.m:])
    # serving: cached scoring equals the full pass, candidate by candidate
    Gc = rng.standard_normal((cfg.B, 2, cfg.m, cfg.d))
    cache = orc.kv_cache_build(cfg, w, H, lens)
    Yg, lgs = orc.score_candidates(cfg, w, cache, Gc)
    for c in range(2):
        Yc, lc = orc.forward(cfg, w, H, Gc[:, c], lens)
        np.testing.assert_allclose(Yg[:, c], Yc[:, :cfg.m], rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(lgs[:, c], lc, rtol=1e-11, atol=1e-12)
    # causality of sampled sequence queries: changing the user's newest raw token leaves every slot that
    # holds an older merged token unchanged (learnable slots see everything and are exempt)
    if not cfg.q_learnable and lens[0] > cfg.K:
        H3 = H.copy(); H3[0, lens[0] - 1] += 1.0
        Y3, _ = orc.forward(cfg, w, H3, G, lens)
        Tu = orc.merged_len(lens[0], cfg.K)
        for i in range(cfg.k_recent):
            t = orc.slot_index(i, cfg.k_recent, Tu, cfg.k_uniform)
            if 0 <= t < Tu - 1:
                assert np.array_equal(Y3[0, cfg.m + i], Y[0, cfg.m + i])
