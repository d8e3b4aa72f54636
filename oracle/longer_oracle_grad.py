"""CPU oracle for the backward pass of LONGER with activation recomputation: the token merge (one
InnerTrans block stack and the group pooling), and the whole model (merge, cross-causal layer,
self-causal layers, head, loss).

TEST INFRASTRUCTURE ONLY, like ``longer_oracle``: plain fp64 numpy, written from the definitions;
never imported by the product path.  It states what the HIP backward pass (csrc/backward.hip) has to
reproduce.

What the paper fixes
--------------------
* Training minimises the binary cross-entropy of Eq. 2 over the predictions of Eq. 1.
* Gradients come from reverse-mode differentiation, which needs the forward pass's intermediate
  activations; selected activations are discarded in the forward pass and recomputed during the
  backward pass, trading computation for memory (Section 3.6.2, Mixed Precision Training and
  Recompute).  Recomputation changes what is kept, not what is computed: the gradients are those of
  the plain backward pass.
* The block that is differentiated is the encoder layer of Section 3.4 (Eq. 3) as ``longer_oracle``
  states it (pre-LayerNorm, W_Q / W_K / W_V / W_O with bias, FFN with exact-erf GELU or ReLU).

Readings (the paper gives no formulas for this part)
* what is kept under recomputation: the input rows of every block (``keep="block_inputs"``) or only
  the raw tokens (``keep="input_only"``); everything else of a block (normalised rows, Q, K, V,
  probabilities, attention output, FFN hidden values) is recomputed from its input when its
  gradient is taken;
* precision: fp64 throughout (the mixed-precision policy of Section 3.6.2 is a property of a GPU
  implementation, measured against this).

Parity status: ``block_backward`` is pinned to torch.autograd on torch.nn.TransformerEncoderLayer
(fp64, with and without key padding) and to central finite differences of ``longer_oracle.block``;
``token_merge_backward`` to finite differences of ``longer_oracle.token_merge``, to exact zeros on
padded tokens and to the closed form of a mean's gradient; the recomputing variants to bit equality
with the storing one; ``bce_loss`` / ``bce_loss_grad`` to torch's BCE-with-logits and its autograd.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
from scipy.special import erf as _erf

from . import longer_oracle as fwd

F64 = np.float64
PARAMS = ("ln1_g", "ln1_b", "wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


# --------------------------------------------------------------------------- loss (Eq. 1-2)
def bce_loss(logits: np.ndarray, y: np.ndarray) -> float:
    """Eq. 2: mean over the samples of -[y log p + (1 - y) log(1 - p)] with p = sigmoid(logit)
    (Eq. 1), written through log(1 + exp(.)) so that large logits do not overflow."""
    z = np.asarray(logits, dtype=F64)
    y = np.asarray(y, dtype=F64)
    return float(np.mean(np.maximum(z, 0.0) - z * y + np.log1p(np.exp(-np.abs(z)))))


def bce_loss_grad(logits: np.ndarray, y: np.ndarray) -> np.ndarray:
    """d loss / d logit = (sigmoid(logit) - y) / N."""
    z = np.asarray(logits, dtype=F64)
    y = np.asarray(y, dtype=F64)
    e = np.exp(-np.abs(z))                                   # sigmoid without overflow for large |logit|
    sig = np.where(z >= 0, 1.0 / (1.0 + e), e / (1.0 + e))
    return (sig - y) / z.size


# --------------------------------------------------------------------------- primitives
def _sum_lead(a: np.ndarray, keep: int) -> np.ndarray:
    """Sum over all leading axes, keeping the last ``keep`` ones (a parameter is shared by every row)."""
    return a.reshape((-1,) + a.shape[a.ndim - keep:]).sum(axis=0)


def _matT(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """sum over rows of a^T b: gradient of a weight from its input rows a [..., n, i] and the
    gradient of its output rows b [..., n, o]."""
    return a.reshape(-1, a.shape[-1]).T @ b.reshape(-1, b.shape[-1])


def layer_norm_backward(dy: np.ndarray, x: np.ndarray, g: np.ndarray, eps: float):
    """y = (x - mu) / sqrt(var + eps) * g + b with the biased variance: returns (dx, dg, db)."""
    D = x.shape[-1]
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xh = (x - mu) * rstd
    dxh = dy * g
    dx = rstd * (dxh - dxh.mean(axis=-1, keepdims=True) - xh * (dxh * xh).mean(axis=-1, keepdims=True))
    return dx, _sum_lead(dy * xh, 1), _sum_lead(dy, 1)


def activation_grad(x: np.ndarray, act: str) -> np.ndarray:
    if act == "gelu_erf":       # d/dx [x Phi(x)] = Phi(x) + x phi(x)
        return 0.5 * (1.0 + _erf(x / math.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)
    if act == "relu":
        return (x > 0).astype(F64)
    raise ValueError(act)


# --------------------------------------------------------------------------- one block
def block_forward_keep(xq, xkv, mask, blk, heads: int, eps: float, act: str) -> Tuple[np.ndarray, dict]:
    """``longer_oracle.block`` step by step, keeping every intermediate the backward pass reads."""
    d = xq.shape[-1]
    dh = d // heads
    c = {"xq": xq, "xkv": xkv, "mask": mask}
    c["nkv"] = fwd.layer_norm(xkv, blk["ln1_g"], blk["ln1_b"], eps)
    c["K"] = c["nkv"] @ blk["wk"] + blk["bk"]
    c["V"] = c["nkv"] @ blk["wv"] + blk["bv"]
    c["nq"] = fwd.layer_norm(xq, blk["ln1_g"], blk["ln1_b"], eps)
    c["q"] = c["nq"] @ blk["wq"] + blk["bq"]
    att = np.zeros_like(c["q"])
    c["p"] = []
    for h in range(heads):
        sl = slice(h * dh, (h + 1) * dh)
        s = c["q"][..., sl] @ np.swapaxes(c["K"][..., sl], -1, -2) / math.sqrt(dh)
        p = fwd.masked_softmax(s, mask)
        c["p"].append(p)
        att[..., sl] = p @ c["V"][..., sl]
    c["att"] = att
    c["x"] = xq + att @ blk["wo"] + blk["bo"]
    c["u"] = fwd.layer_norm(c["x"], blk["ln2_g"], blk["ln2_b"], eps)
    c["a"] = c["u"] @ blk["w1"] + blk["b1"]
    c["hdn"] = fwd.activation(c["a"], act)
    return c["x"] + c["hdn"] @ blk["w2"] + blk["b2"], c


def block_backward_kept(dout: np.ndarray, c: dict, blk, heads: int, eps: float, act: str):
    """Reverse of ``block_forward_keep``: returns (d xq, d xkv, {parameter: gradient})."""
    d = dout.shape[-1]
    dh = d // heads
    g: Dict[str, np.ndarray] = {}
    # FFN sub-block: out = x + act(LN2(x) W1 + b1) W2 + b2
    g["w2"] = _matT(c["hdn"], dout)
    g["b2"] = _sum_lead(dout, 1)
    da = (dout @ blk["w2"].T) * activation_grad(c["a"], act)
    g["w1"] = _matT(c["u"], da)
    g["b1"] = _sum_lead(da, 1)
    dx2, g["ln2_g"], g["ln2_b"] = layer_norm_backward(da @ blk["w1"].T, c["x"], blk["ln2_g"], eps)
    dx = dout + dx2
    # attention sub-block: x = xq + att W_O + b_O
    g["wo"] = _matT(c["att"], dx)
    g["bo"] = _sum_lead(dx, 1)
    datt = dx @ blk["wo"].T
    dq = np.zeros_like(c["q"])
    dK = np.zeros_like(c["K"])
    dV = np.zeros_like(c["V"])
    for h in range(heads):
        sl = slice(h * dh, (h + 1) * dh)
        p = c["p"][h]
        dp = datt[..., sl] @ np.swapaxes(c["V"][..., sl], -1, -2)
        dV[..., sl] = np.swapaxes(p, -1, -2) @ datt[..., sl]
        ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True)) / math.sqrt(dh)    # masked pairs: p = 0
        dq[..., sl] = ds @ c["K"][..., sl]
        dK[..., sl] = np.swapaxes(ds, -1, -2) @ c["q"][..., sl]
    g["wq"] = _matT(c["nq"], dq)
    g["bq"] = _sum_lead(dq, 1)
    g["wk"] = _matT(c["nkv"], dK)
    g["bk"] = _sum_lead(dK, 1)
    g["wv"] = _matT(c["nkv"], dV)
    g["bv"] = _sum_lead(dV, 1)
    dxq_n, gq, bq_ = layer_norm_backward(dq @ blk["wq"].T, c["xq"], blk["ln1_g"], eps)
    dxkv, gk, bk_ = layer_norm_backward(dK @ blk["wk"].T + dV @ blk["wv"].T, c["xkv"], blk["ln1_g"], eps)
    g["ln1_g"] = gq + gk          # LN1 normalises the query rows and the key rows
    g["ln1_b"] = bq_ + bk_
    return dx + dxq_n, dxkv, g


def block_backward(dout, xq, xkv, mask, blk, heads: int, eps: float, act: str):
    """Gradient of ``longer_oracle.block`` from its inputs alone: everything else is recomputed."""
    blk = fwd._f64(blk)
    _, c = block_forward_keep(np.asarray(xq, dtype=F64), np.asarray(xkv, dtype=F64), mask, blk, heads, eps, act)
    return block_backward_kept(np.asarray(dout, dtype=F64), c, blk, heads, eps, act)


# --------------------------------------------------------------------------- token merge
def token_merge_backward(cfg, inner_blocks: Sequence[dict], H: np.ndarray, lens, dM: np.ndarray,
                         keep: str = "all"):
    """Gradients of ``longer_oracle.token_merge`` (Section 3.4) for an upstream gradient dM [B, T, d]
    (merge "concat": [B, T, K d_raw]): returns (dH [B, L, d_raw], [per InnerTrans block {parameter:
    gradient}]).  Padded tokens get exact zeros.

    ``keep`` selects what the forward pass hands to the backward pass (Section 3.6.2):
      "all"           every intermediate of every block (plain reverse mode);
      "block_inputs"  the input rows of each block; a block's intermediates are recomputed;
      "input_only"    the raw tokens; the chain of block inputs is recomputed first.
    The three give the same numbers."""
    H = np.asarray(H)
    B, L, d = H.shape
    K = cfg.K
    T = (L + K - 1) // K
    lens = fwd._lens(lens, B, L)
    blocks = [fwd._f64(b) for b in inner_blocks]
    concat = getattr(cfg, "merge", "mean") == "concat"
    dM = np.asarray(dM, dtype=F64)
    dH = np.zeros((B, L, d), dtype=F64)
    grads = [{k: np.zeros_like(b[k]) for k in PARAMS} for b in blocks]
    for u in range(B):
        pos = np.arange(T * K).reshape(T, K)
        valid = pos < lens[u]
        nv = int(min(lens[u], L))
        E0 = np.zeros((T * K, d), dtype=F64)
        E0[:nv] = np.asarray(H[u, :nv], dtype=F64)
        E0 = E0.reshape(T, K, d)
        mask = valid[:, :, None] & valid[:, None, :]
        # ---- forward: what is kept depends on `keep`
        kept: List[object] = []
        E = E0
        for blk in blocks:
            out, c = block_forward_keep(E, E, mask, blk, cfg.inner_heads, cfg.ln_eps, cfg.act)
            kept.append(c if keep == "all" else (E if keep == "block_inputs" else None))
            E = out
        if keep == "input_only":          # recompute the chain of block inputs before going back
            E = E0
            for i, blk in enumerate(blocks):
                kept[i] = E
                E = fwd.block(E, E, mask, blk, cfg.inner_heads, cfg.ln_eps, cfg.act)
        elif keep not in ("all", "block_inputs"):
            raise ValueError(keep)
        # ---- gradient of the merge: mean over the valid tokens of a group, or concatenation
        if concat:
            dZ = dM[u].reshape(T, K, d)
        else:
            cnt = np.clip(lens[u] - np.arange(T) * K, 0, K)
            dZ = np.where(cnt[:, None, None] > 0, dM[u][:, None, :] / np.maximum(cnt, 1)[:, None, None], 0.0)
            dZ = np.broadcast_to(dZ, (T, K, d))
        dE = np.where(valid[:, :, None], dZ, 0.0)
        # ---- back through the blocks
        for i in reversed(range(len(blocks))):
            blk = blocks[i]
            if keep == "all":
                c = kept[i]
            else:
                _, c = block_forward_keep(kept[i], kept[i], mask, blk, cfg.inner_heads, cfg.ln_eps, cfg.act)
            dxq, dxkv, g = block_backward_kept(dE, c, blk, cfg.inner_heads, cfg.ln_eps, cfg.act)
            dE = np.where(valid[:, :, None], dxq + dxkv, 0.0)       # queries and keys are the same rows
            for k in PARAMS:
                grads[i][k] += g[k]
        dH[u, :nv] = dE.reshape(T * K, d)[:nv]
    return dH, grads


# --------------------------------------------------------------------------- whole model
def model_backward(cfg, weights: dict, H: np.ndarray, G: np.ndarray, lens, labels: np.ndarray, keep: str = "input_only"):
    """Loss (Eq. 2) of ``longer_oracle.forward`` (token merge, cross-causal layer over R = [G; M] with
    the query set O of Eq. 5, N self-causal layers, linear head on the global rows, Eq. 1) and its
    gradient with respect to every input and parameter:

        returns (loss, logits [B], dH [B, L, d_raw], dG [B, m, d],
                 {"inner": [per block], "cross": {...}, "self": [per block], "head_w", "head_b"}).

    With learnable query tokens (``q_learnable``) the slots' rows are the parameter ``q_learn`` [k, d]:
    the dict then holds its gradient ("q_learn": the sum over the users with at least one token of the
    slots' row gradients) and no gradient flows from the slots into the merged tokens.  The
    reduced stack keeps the input rows of every layer and recomputes a layer's intermediates when its
    gradient is taken; the token merge is differentiated by ``token_merge_backward(keep=...)``."""
    learn = bool(getattr(cfg, "q_learnable", False))
    q_learn = np.asarray(weights["q_learn"], dtype=F64) if learn else None
    H = np.asarray(H)
    G = np.asarray(G, dtype=F64)
    B, L, _ = H.shape
    m, k, d, T = cfg.m, cfg.k_recent, cfg.d, cfg.T
    lens_ = fwd._lens(lens, B, L)
    labels = np.asarray(labels, dtype=F64)
    cross = fwd._f64(weights["cross"])
    selfs = [fwd._f64(b) for b in weights["self"]]
    head_w = np.asarray(weights["head_w"], dtype=F64)
    head_b = float(np.asarray(weights["head_b"]).reshape(-1)[0])

    # ---- forward, keeping each layer's input rows per user
    M = fwd.token_merge(cfg, weights["inner"], H, lens)
    per_user = []
    logits = np.zeros(B, dtype=F64)
    for u in range(B):
        Tu = fwd.merged_len(lens_[u], cfg.K)
        Mu = np.where((np.arange(T) < Tu)[:, None], M[u], 0.0)
        R = np.concatenate([G[u], Mu], axis=0)
        qt = fwd._query_tokens(cfg, m, Tu)
        qvalid = np.array([t[2] for t in qt])
        O = fwd.gather_queries(cfg, G[u], Mu, Tu, q_learn)
        mask_c = fwd._type_mask(qt, fwd.key_tokens(m, T, Tu), cfg.gmask)
        mask_s = fwd._type_mask(qt, qt, cfg.gmask)
        X = np.where(qvalid[:, None], fwd.block(O, R, mask_c, cross, cfg.heads, cfg.ln_eps, cfg.act), 0.0)
        xs = []
        for blk in selfs:
            xs.append(X)
            X = np.where(qvalid[:, None], fwd.block(X, X, mask_s, blk, cfg.heads, cfg.ln_eps, cfg.act), 0.0)
        logits[u] = X[:m].reshape(-1) @ head_w + head_b
        per_user.append((Tu, qt, qvalid, O, R, mask_c, mask_s, xs, X))
    loss = bce_loss(logits, labels)

    # ---- backward
    dlogit = bce_loss_grad(logits, labels)
    g_cross = {p: np.zeros_like(cross[p]) for p in PARAMS}
    g_self = [{p: np.zeros_like(b[p]) for p in PARAMS} for b in selfs]
    g_hw = np.zeros_like(head_w)
    g_ql = np.zeros((k, d), dtype=F64)
    dG = np.zeros((B, m, d), dtype=F64)
    dM = np.zeros((B, T, d), dtype=F64)
    for u in range(B):
        Tu, qt, qvalid, O, R, mask_c, mask_s, xs, Y = per_user[u]
        g_hw += dlogit[u] * Y[:m].reshape(-1)
        dX = np.zeros((m + k, d), dtype=F64)
        dX[:m] = dlogit[u] * head_w.reshape(m, d)
        for i in reversed(range(len(selfs))):
            dX = np.where(qvalid[:, None], dX, 0.0)                # invalid rows were written as zeros
            dxq, dxkv, g = block_backward(dX, xs[i], xs[i], mask_s, selfs[i], cfg.heads, cfg.ln_eps, cfg.act)
            dX = dxq + dxkv                                         # queries and keys are the same rows
            for p in PARAMS:
                g_self[i][p] += g[p]
        dX = np.where(qvalid[:, None], dX, 0.0)
        dO, dR, g = block_backward(dX, O, R, mask_c, cross, cfg.heads, cfg.ln_eps, cfg.act)
        for p in PARAMS:
            g_cross[p] += g[p]
        dG[u] = dO[:m] + dR[:m]                                     # a global token is a query row and a key row
        dMu = dR[m:].copy()
        for i in range(k):
            t, v = qt[m + i][1], qt[m + i][2]
            if v and learn:
                g_ql[i] += dO[m + i]                                # slot i holds row i of the parameter
            elif v:
                dMu[t] += dO[m + i]                                 # slot i holds merged token t
        dM[u] = np.where((np.arange(T) < Tu)[:, None], dMu, 0.0)    # merged tokens past T_u were zeroed
    dH, g_inner = token_merge_backward(cfg, weights["inner"], H, lens, dM, keep=keep)
    grads = {"inner": g_inner, "cross": g_cross, "self": g_self, "head_w": g_hw, "head_b": np.array([dlogit.sum()])}
    if learn:
        grads["q_learn"] = g_ql
    return loss, logits, dH, dG, grads


# --------------------------------------------------------------------------- input generation
def input_generation_backward(cfg, mlp: dict, E: np.ndarray, tdiff: np.ndarray, lens, dH: np.ndarray):
    """Gradients of ``longer_oracle.input_generation`` (Section 3.5.1, Input Generation:
    H = act([E + pos ; tdiff] w1 + b1) w2 + b2 on the valid tokens) for an upstream gradient dH [B, L, d]:
    returns (dE [B, L, d_e], dtdiff [B, L, d - d_e], {"pos", "w1", "b1", "w2", "b2"}); padded tokens get
    exact zeros, the positional embedding's gradient is summed over the users that reach a position."""
    E = np.asarray(E)
    B, L, d_e = E.shape
    lens = fwd._lens(lens, B, L)
    w1, b1, w2, b2, pos = (np.asarray(mlp[k], dtype=F64) for k in ("w1", "b1", "w2", "b2", "pos"))
    dH = np.asarray(dH, dtype=F64)
    dE = np.zeros((B, L, d_e), dtype=F64)
    dtd = np.zeros((B, L, w1.shape[0] - d_e), dtype=F64)
    g = {"pos": np.zeros_like(pos), "w1": np.zeros_like(w1), "b1": np.zeros_like(b1), "w2": np.zeros_like(w2),
         "b2": np.zeros_like(b2)}
    for u in range(B):
        n = int(min(lens[u], L))
        x = np.concatenate([np.asarray(E[u, :n], dtype=F64) + pos[:n], np.asarray(tdiff[u, :n], dtype=F64)], axis=1)
        a = x @ w1 + b1
        hdn = fwd.activation(a, cfg.act)
        dy = dH[u, :n]
        g["w2"] += hdn.T @ dy
        g["b2"] += dy.sum(axis=0)
        da = (dy @ w2.T) * activation_grad(a, cfg.act)
        g["w1"] += x.T @ da
        g["b1"] += da.sum(axis=0)
        dx = da @ w1.T
        dE[u, :n] = dx[:, :d_e]
        g["pos"][:n] += dx[:, :d_e]          # the same embedding row serves every user at that position
        dtd[u, :n] = dx[:, d_e:]
    return dE, dtd, g
