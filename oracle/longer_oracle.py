"""CPU oracle for the LONGER forward pass and its KV-cache serving path.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 numpy statement of what
the hot path computes, written from the paper's definitions.  It shares no code
with the HIP library and must never be imported by the product path; only the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg may call it.

What the paper fixes and where each function follows it
-------------------------------------------------------
* Block structure: the "standard-structured transformer encoder layer" whose
  cost the paper gives as FLOPs = 24 L d^2 + 4 L^2 d and Params = 12 d^2 + 13 d
  (Token Merge, Section 3.4, Eq. 3).  The only decomposition giving both closed
  forms is four d x d projections with bias (4 d^2 + 4 d), an FFN d -> 4d -> d
  with biases (8 d^2 + 5 d) and two LayerNorms with gain and bias (4 d).
* Token merge with InnerTrans: a transformer block applied inside each group of
  K adjacent tokens (Section 3.4, InnerTrans equation).
* Query set O = [G; H_S] with the most recent k sequence tokens (Section 3.5.1,
  Eq. 5).
* Cross-causal attention of O over R = [G; H]: Q = O W_Q, K = R W_K, V = R W_V,
  softmax(Q K^T / sqrt(d) + M) V, then an FFN (Section 3.5.2, Eq. 6-8).
* N self-causal attention layers over the reduced set, each followed by an FFN
  (Section 3.5.3-3.5.4, Eq. 9-10).
* KV-cache serving: the sequence side is computed once per user, each candidate
  only attends from its global tokens to the cached sequence K/V (Section 3.6.3).

Readings taken where the paper is silent or ambiguous (all listed in the design
document as well):
* the K InnerTrans outputs of a group become one token of width d by a mean
  over the group's valid tokens (merge "mean"), or, with raw tokens of width
  d / K, by concatenation (merge "concat", the paper's own width-K d form);
  InnerTrans attention is bidirectional inside the group;
* pre-LayerNorm residual blocks, biased variance, eps = 1e-5, no final norm;
  FFN activation exact-erf GELU (ReLU selectable);
* multi-head attention with scale 1/sqrt(d_h); one head recovers Eq. 7;
* the mask of Eq. 8 is applied as a rule on token types over chronologically
  stored data (oldest first): a sequence query sees sequence keys that are not
  newer than itself and never a global key; a global query sees every valid
  sequence key and (gmask "full") every global key, or (gmask "causal", Eq. 8
  read literally) only globals with index >= its own;
* "recent k" = merged tokens T_u-k .. T_u-1, right-aligned in k slots; slots
  with a negative index are invalid;  invalid rows are returned as zeros;
  the other sampling strategies of Section 3.5.1 / the ablation table put
  uniformly sampled older tokens into the first ``k_uniform`` slots (each the
  newest token of one of k_uniform equal shares of the older tokens) and keep the
  most recent ones in the rest; slots stay in chronological order;
  ``q_learnable``: the k slots hold learnable query tokens (one [k, d] parameter for
  all users) that see every valid sequence token in the first layer and each other
  causally, in slot order, afterwards (see ``query_tokens``);
* the prediction head is logit = <head_w, flatten(Y[:m])> + head_b;
* input generation (``input_generation``): widths and MLP depth are this build's
  reading, see its docstring.

Parity status: every function below is pinned by tests/test_oracle_*.py to a
library routine, a closed form, brute force or one of the invariants, except
``head_logits`` whose definition is this build's own reading (the paper never
defines the head): parity unpinned beyond its closed form.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# --------------------------------------------------------------------------- closed forms
def flops_vanilla_layer(L: int, d: int) -> int:
    """Eq. 3: FLOPs of one encoder layer over L tokens of width d."""
    return 24 * L * d * d + 4 * L * L * d


def params_vanilla_layer(d: int) -> int:
    """Eq. 3: parameters of one encoder layer of width d."""
    return 12 * d * d + 13 * d


def flops_merged_layer(L: int, d: int, K: int) -> float:
    """Numerator of the complexity ratio in Section 3.4: a layer over L/K tokens
    of width K d (merge by concatenation)."""
    return 24 * L * d * d * K + 4 * L * L * d / K


def merge_ratio(L: int, d: int, K: int) -> float:
    """Closed-form ratio (6 d K + L / K) / (6 d + L) of Section 3.4."""
    return (6 * d * K + L / K) / (6 * d + L)


def params_merged_layer(d: int, K: int) -> int:
    """Eq. 4."""
    return 12 * K * K * d * d + 13 * K * d


def block_param_count(blk: Dict[str, np.ndarray]) -> int:
    return int(sum(np.asarray(v).size for v in blk.values()))


# --------------------------------------------------------------------------- primitives
def layer_norm(x: np.ndarray, g: np.ndarray, b: np.ndarray, eps: float) -> np.ndarray:
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g + b


def activation(x: np.ndarray, act: str) -> np.ndarray:
    if act == "gelu_erf":
        return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))
    if act == "relu":
        return np.maximum(x, 0.0)
    raise ValueError(act)


def masked_softmax(s: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Row softmax of ``s + M`` with M = 0 where ``mask`` else -inf (Eq. 7-8).
    Rows with no visible key give all zeros instead of NaN."""
    s = np.where(mask, s, -np.inf)
    mx = s.max(axis=-1, keepdims=True)
    mx = np.where(np.isfinite(mx), mx, 0.0)
    e = np.exp(s - mx)                      # exp(-inf) = 0 exactly
    den = e.sum(axis=-1, keepdims=True)
    return np.where(den > 0, e / np.where(den > 0, den, 1.0), 0.0)


def _f64(blk: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    return {k: np.asarray(v, dtype=F64) for k, v in blk.items()}


def project_kv(x: np.ndarray, blk, eps: float) -> Tuple[np.ndarray, np.ndarray]:
    """K = LN1(x) W_K + b_K, V = LN1(x) W_V + b_V (Eq. 6, key/value side)."""
    xn = layer_norm(x, blk["ln1_g"], blk["ln1_b"], eps)
    return xn @ blk["wk"] + blk["bk"], xn @ blk["wv"] + blk["bv"]


def attend_ffn(xq: np.ndarray, Kmat: np.ndarray, Vmat: np.ndarray, mask: np.ndarray, blk,
               heads: int, eps: float, act: str, probs_out: Optional[list] = None) -> np.ndarray:
    """Query side of a block: Q = LN1(xq) W_Q + b_Q, multi-head masked softmax
    attention over the given K/V (Eq. 7 / Eq. 9), output projection + residual
    from the query rows' own input, then the FFN sub-block with its residual.

    Shapes: xq [..., nq, d], Kmat/Vmat [..., nk, d], mask [..., nq, nk] bool.
    """
    d = xq.shape[-1]
    dh = d // heads
    q = layer_norm(xq, blk["ln1_g"], blk["ln1_b"], eps) @ blk["wq"] + blk["bq"]
    att = np.zeros_like(q)
    for h in range(heads):
        sl = slice(h * dh, (h + 1) * dh)
        s = q[..., sl] @ np.swapaxes(Kmat[..., sl], -1, -2) / math.sqrt(dh)
        p = masked_softmax(s, mask)
        if probs_out is not None:
            probs_out.append(p)
        att[..., sl] = p @ Vmat[..., sl]
    x = xq + att @ blk["wo"] + blk["bo"]
    hdn = activation(layer_norm(x, blk["ln2_g"], blk["ln2_b"], eps) @ blk["w1"] + blk["b1"], act)
    return x + hdn @ blk["w2"] + blk["b2"]


def block(xq: np.ndarray, xkv: np.ndarray, mask: np.ndarray, blk, heads: int, eps: float,
          act: str, probs_out: Optional[list] = None) -> np.ndarray:
    """A full pre-LN transformer block with queries from ``xq`` and keys/values
    from ``xkv`` (xq is xkv for self-attention)."""
    Kmat, Vmat = project_kv(xkv, blk, eps)
    return attend_ffn(xq, Kmat, Vmat, mask, blk, heads, eps, act, probs_out)


# --------------------------------------------------------------------------- masks
def visible(q_is_global: bool, q_idx: int, k_is_global: bool, k_idx: int, gmask: str) -> bool:
    """The rule of Eq. 8 on token types.  ``idx`` is the global token's index a
    for a global token, and the chronological merged-token index t for a
    sequence token.  Validity (padding) is handled by the caller."""
    if not q_is_global:
        return (not k_is_global) and k_idx <= q_idx
    if not k_is_global:
        return True
    return True if gmask == "full" else k_idx >= q_idx


def _type_mask(q_tokens, k_tokens, gmask: str) -> np.ndarray:
    """Boolean [nq, nk] from token descriptors (is_global, idx, valid): the rule
    of ``visible`` evaluated for all pairs at once, and-ed with validity."""
    qg = np.array([t[0] for t in q_tokens], dtype=bool)[:, None]
    qi = np.array([t[1] for t in q_tokens], dtype=np.int64)[:, None]
    qv = np.array([t[2] for t in q_tokens], dtype=bool)[:, None]
    kg = np.array([t[0] for t in k_tokens], dtype=bool)[None, :]
    ki = np.array([t[1] for t in k_tokens], dtype=np.int64)[None, :]
    kv = np.array([t[2] for t in k_tokens], dtype=bool)[None, :]
    glob_q = np.where(kg, True if gmask == "full" else (ki >= qi), True)   # global query row
    seq_q = (~kg) & (ki <= qi)                                              # sequence query row
    return np.where(qg, glob_q, seq_q) & qv & kv


def merged_len(length: int, K: int) -> int:
    """T_u = ceil(l_u / K): number of valid merged tokens of a user."""
    return (int(length) + K - 1) // K


def slot_index(i: int, k: int, Tu: int, k_uniform: int = 0) -> int:
    """Merged index held by slot i of the k sampled sequence tokens H_S (Section 3.5.1:
    a predefined sampling strategy; the ablation compares the most recent k, uniformly
    sampled tokens, and recent ones plus the rest sampled uniformly).  The last
    k - k_uniform slots hold the most recent tokens; the first k_uniform slots are spread
    evenly, oldest first, over the tokens before those, each holding the newest token of
    its share.  A user with no more than k tokens gets all of them, right-aligned (a
    negative index is an invalid slot)."""
    if Tu <= k or i >= k_uniform:
        return Tu - k + i
    rest = Tu - (k - k_uniform)          # tokens older than the recent part; more than k_uniform of them
    return ((i + 1) * rest) // k_uniform - 1


def query_tokens(m: int, k: int, Tu: int, k_uniform: int = 0, learnable: bool = False):
    """Descriptors of O = [G; H_S] (Eq. 5): slot i holds merged index
    ``slot_index(i, ...)`` (Tu - k + i for the default, most recent k), invalid when negative.

    ``learnable`` (Section 3.5.1: k learnable tokens as the query set, the strategy of the
    compression models cited there): the slots hold parameters, not sequence tokens.  They
    are placed after the user's newest token, in slot order: slot i carries the index
    Tu + i, so that under Eq. 8 it sees every valid sequence token in the first layer and
    the slots up to itself in the self-causal layers.  A user with no token at all has
    nothing to compress: its slots are invalid."""
    toks = [(True, a, True) for a in range(m)]
    for i in range(k):
        if learnable:
            toks.append((False, Tu + i, Tu > 0))
        else:
            t = slot_index(i, k, Tu, k_uniform)
            toks.append((False, t, t >= 0))
    return toks


def _query_tokens(cfg, m: int, Tu: int):
    """``query_tokens`` with the config's query strategy."""
    return query_tokens(m, cfg.k_recent, Tu, getattr(cfg, "k_uniform", 0), getattr(cfg, "q_learnable", False))


def key_tokens(m: int, T: int, Tu: int):
    """Descriptors of R = [G; M] (Section 3.5.1), merged tokens t >= Tu invalid."""
    return [(True, a, True) for a in range(m)] + [(False, t, t < Tu) for t in range(T)]


# --------------------------------------------------------------------------- input generation
def input_generation(cfg, mlp: dict, E: np.ndarray, tdiff: np.ndarray, lens=None) -> np.ndarray:
    """Sequence-token representations H [B, L, d] (Section 3.5.1, Input Generation): the
    learnable absolute positional embedding is added to each item embedding, the
    time-difference side information is concatenated to it, and the result goes through an
    MLP.  Readings (the paper fixes none of them): item and position width d_e, side
    information width d - d_e, a two-layer MLP d -> ffn_mult d -> d with the block's
    activation.  Rows of padded tokens are zero."""
    E = np.asarray(E)
    B, L, d_e = E.shape
    lens = _lens(lens, B, L)
    w1, b1, w2, b2, pos = (np.asarray(mlp[k], dtype=F64) for k in ("w1", "b1", "w2", "b2", "pos"))
    H = np.zeros((B, L, w2.shape[1]), dtype=F64)
    for u in range(B):
        n = int(min(lens[u], L))
        x = np.concatenate([np.asarray(E[u, :n], dtype=F64) + pos[:n], np.asarray(tdiff[u, :n], dtype=F64)], axis=1)
        H[u, :n] = activation(x @ w1 + b1, cfg.act) @ w2 + b2
    return H


# --------------------------------------------------------------------------- token merge
def _lens(lens, B: int, L: int) -> np.ndarray:
    if lens is None:
        return np.full(B, L, dtype=np.int64)
    return np.asarray(lens, dtype=np.int64)


def inner_transformer(cfg, inner_blocks: Sequence[dict], H: np.ndarray, lens=None) -> np.ndarray:
    """InnerTrans (Section 3.4): ``cfg.inner_layers`` transformer blocks applied
    inside every group of K adjacent tokens.  Returns the un-pooled group
    outputs Z [B, T, K, d]; rows of invalid (padded) tokens are zero."""
    H = np.asarray(H)
    B, L, d = H.shape
    K = cfg.K
    T = (L + K - 1) // K
    lens = _lens(lens, B, L)
    blocks = [_f64(b) for b in inner_blocks]
    Z = np.zeros((B, T, K, d), dtype=F64)
    for u in range(B):
        pos = np.arange(T * K).reshape(T, K)
        valid = pos < lens[u]                                   # [T, K]
        E = np.zeros((T * K, d), dtype=F64)
        nv = int(min(lens[u], L))
        E[:nv] = np.asarray(H[u, :nv], dtype=F64)               # padded values never read
        E = E.reshape(T, K, d)
        mask = valid[:, :, None] & valid[:, None, :]            # bidirectional inside the group
        for blk in blocks:
            E = block(E, E, mask, blk, cfg.inner_heads, cfg.ln_eps, cfg.act)
        Z[u] = np.where(valid[:, :, None], E, 0.0)
    return Z


def token_merge(cfg, inner_blocks: Sequence[dict], H: np.ndarray, lens=None) -> np.ndarray:
    """Merged tokens M [B, T, d].

    merge "mean" (default): mean of each group's valid InnerTrans outputs; groups
    with no valid token are zero.
    merge "concat" (Section 3.4: grouped representations formed by concatenation,
    after InnerTrans has let the group's tokens interact; the merged width K d is
    what Eq. 4 and the complexity ratio count): raw tokens of width d / K, the K
    InnerTrans outputs of a group laid side by side, oldest first; slots of
    invalid (padded) tokens are zero."""
    H = np.asarray(H)
    B, L, d = H.shape
    K = cfg.K
    T = (L + K - 1) // K
    lens = _lens(lens, B, L)
    Z = inner_transformer(cfg, inner_blocks, H, lens)
    if getattr(cfg, "merge", "mean") == "concat":
        return Z.reshape(B, T, K * d)
    M = np.zeros((B, T, d), dtype=F64)
    for u in range(B):
        cnt = np.clip(lens[u] - np.arange(T) * K, 0, K)         # valid tokens per group
        nz = cnt > 0
        M[u, nz] = Z[u, nz].sum(axis=1) / cnt[nz, None]
    return M


# --------------------------------------------------------------------------- hybrid attention
def slot_rows(cfg, M_u: np.ndarray, Tu: int, q_learn=None) -> np.ndarray:
    """The k sequence-side query rows of one user: the sampled merged tokens, or the
    learnable query tokens ``q_learn`` [k, d] (the same for every user); invalid slots zero."""
    k = cfg.k_recent
    Xs = np.zeros((k, M_u.shape[-1]), dtype=F64)
    for i, (_, t, v) in enumerate(_query_tokens(cfg, 0, Tu)):
        if v:
            Xs[i] = np.asarray(q_learn, dtype=F64)[i] if getattr(cfg, "q_learnable", False) else M_u[t]
    return Xs


def gather_queries(cfg, G_u: np.ndarray, M_u: np.ndarray, Tu: int, q_learn=None) -> np.ndarray:
    """O = [G; H_S] for one user (Eq. 5), invalid slots zero."""
    return np.concatenate([np.asarray(G_u, dtype=F64), slot_rows(cfg, M_u, Tu, q_learn)], axis=0)


def hybrid_cross_attn(cfg, cross_blk: dict, G: np.ndarray, M: np.ndarray, lens=None,
                      L: Optional[int] = None, probs_out: Optional[list] = None, q_learn=None) -> np.ndarray:
    """First layer (Section 3.5.2): queries O attend over R = [G; M].
    ``lens`` are raw lengths (None = all L); ``q_learn`` [k, d] are the learnable query
    tokens of a ``q_learnable`` configuration; returns X [B, m+k, d]."""
    G = np.asarray(G, dtype=F64)
    M = np.asarray(M, dtype=F64)
    B, T, d = M.shape
    L = T * cfg.K if L is None else L
    lens = _lens(lens, B, L)
    blk = _f64(cross_blk)
    X = np.zeros((B, cfg.m + cfg.k_recent, d), dtype=F64)
    for u in range(B):
        Tu = merged_len(lens[u], cfg.K)
        Mu = np.where((np.arange(T) < Tu)[:, None], M[u], 0.0)
        R = np.concatenate([G[u], Mu], axis=0)
        O = gather_queries(cfg, G[u], Mu, Tu, q_learn)
        qt = _query_tokens(cfg, cfg.m, Tu)
        mask = _type_mask(qt, key_tokens(cfg.m, T, Tu), cfg.gmask)
        out = block(O, R, mask, blk, cfg.heads, cfg.ln_eps, cfg.act, probs_out)
        qvalid = np.array([t[2] for t in qt])
        X[u] = np.where(qvalid[:, None], out, 0.0)
    return X


def self_attn_layer(cfg, blk: dict, X: np.ndarray, lens=None, L: Optional[int] = None,
                    probs_out: Optional[list] = None) -> np.ndarray:
    """One self-causal layer over the reduced set [G; k slots] (Section 3.5.3)."""
    X = np.asarray(X, dtype=F64)
    B, n, d = X.shape
    lens = _lens(lens, B, L if L is not None else 1 << 40)
    blk = _f64(blk)
    Y = np.zeros_like(X)
    for u in range(B):
        Tu = merged_len(lens[u], cfg.K)
        toks = _query_tokens(cfg, cfg.m, Tu)
        valid = np.array([t[2] for t in toks])
        Xu = np.where(valid[:, None], X[u], 0.0)
        mask = _type_mask(toks, toks, cfg.gmask)
        out = block(Xu, Xu, mask, blk, cfg.heads, cfg.ln_eps, cfg.act, probs_out)
        Y[u] = np.where(valid[:, None], out, 0.0)
    return Y


def head_logits(cfg, head_w: np.ndarray, head_b: np.ndarray, Yg: np.ndarray) -> np.ndarray:
    """logit = <head_w, flatten(global rows)> + head_b.  Yg [..., m, d]."""
    flat = np.asarray(Yg, dtype=F64).reshape(Yg.shape[:-2] + (-1,))
    return flat @ np.asarray(head_w, dtype=F64) + float(np.asarray(head_b).reshape(-1)[0])


def forward(cfg, weights: dict, H: np.ndarray, G: np.ndarray, lens=None):
    """CrossAttn(O, R) -> SelfAttn x N (Eq. 10) after token merge.
    Returns (Y [B, m+k, d], logits [B])."""
    H = np.asarray(H)
    B, L, d = H.shape
    M = token_merge(cfg, weights["inner"], H, lens)
    X = hybrid_cross_attn(cfg, weights["cross"], G, M, lens, L=L, q_learn=weights.get("q_learn"))
    for blk in weights["self"]:
        X = self_attn_layer(cfg, blk, X, lens, L=L)
    logits = head_logits(cfg, weights["head_w"], weights["head_b"], X[:, :cfg.m])
    return X, logits


# --------------------------------------------------------------------------- KV-cache serving
def kv_cache_build(cfg, weights: dict, H: np.ndarray, lens=None) -> dict:
    """Stage 1 of Section 3.6.3: everything that depends only on the user
    sequence.  Sequence tokens never see a global token, so their hidden states
    through all layers -- and hence their K/V in every layer -- are candidate
    independent.  Returns per layer the K/V of the sequence-side keys:
    layer 0 over the T merged tokens, layers 1..N over the k recent slots."""
    H = np.asarray(H)
    U, L, d = H.shape
    lens = _lens(lens, U, L)
    M = token_merge(cfg, weights["inner"], H, lens)
    T, d = M.shape[1], M.shape[2]          # the main stack's width (K times the raw width after a concat merge)
    k = cfg.k_recent
    blocks = [_f64(weights["cross"])] + [_f64(b) for b in weights["self"]]
    cache = {"K": [[] for _ in blocks], "V": [[] for _ in blocks], "valid": [[] for _ in blocks]}
    for u in range(U):
        Tu = merged_len(lens[u], cfg.K)
        Mu = np.where((np.arange(T) < Tu)[:, None], M[u], 0.0)
        # layer 0: keys are all merged tokens; queries are the k recent slots
        seq_keys = [(False, t, t < Tu) for t in range(T)]
        slots = _query_tokens(cfg, 0, Tu)
        svalid = np.array([s[2] for s in slots])
        Kc, Vc = project_kv(Mu, blocks[0], cfg.ln_eps)
        cache["K"][0].append(Kc); cache["V"][0].append(Vc)
        cache["valid"][0].append(np.array([s[2] for s in seq_keys]))
        Xs = slot_rows(cfg, Mu, Tu, weights.get("q_learn"))
        Xs = np.where(svalid[:, None],
                      attend_ffn(Xs, Kc, Vc, _type_mask(slots, seq_keys, cfg.gmask), blocks[0],
                                 cfg.heads, cfg.ln_eps, cfg.act), 0.0)
        for l in range(1, len(blocks)):
            Kc, Vc = project_kv(Xs, blocks[l], cfg.ln_eps)
            cache["K"][l].append(Kc); cache["V"][l].append(Vc)
            cache["valid"][l].append(svalid)
            if l + 1 < len(blocks):       # the last layer's sequence rows feed nothing
                Xs = np.where(svalid[:, None],
                              attend_ffn(Xs, Kc, Vc, _type_mask(slots, slots, cfg.gmask), blocks[l],
                                         cfg.heads, cfg.ln_eps, cfg.act), 0.0)
    return cache


def score_candidates(cfg, weights: dict, cache: dict, G_cand: np.ndarray):
    """Stage 2 of Section 3.6.3: each candidate's m global tokens run through the
    1 + N layers; their keys/values are their own globals plus the cached
    sequence K/V.  Returns (Yg [U, C, m, d], logits [U, C])."""
    G_cand = np.asarray(G_cand, dtype=F64)
    U, C, m, d = G_cand.shape
    blocks = [_f64(weights["cross"])] + [_f64(b) for b in weights["self"]]
    gg = np.array([[visible(True, a, True, b, cfg.gmask) for b in range(m)] for a in range(m)])
    Yg = np.zeros((U, C, m, d), dtype=F64)
    for u in range(U):
        for c in range(C):
            x = G_cand[u, c]
            for l, blk in enumerate(blocks):
                kg, vg = project_kv(x, blk, cfg.ln_eps)
                Kall = np.concatenate([kg, cache["K"][l][u]], axis=0)
                Vall = np.concatenate([vg, cache["V"][l][u]], axis=0)
                mask = np.concatenate([gg, np.broadcast_to(cache["valid"][l][u], (m, len(cache["valid"][l][u])))], axis=1)
                x = attend_ffn(x, Kall, Vall, mask, blk, cfg.heads, cfg.ln_eps, cfg.act)
            Yg[u, c] = x
    logits = head_logits(cfg, weights["head_w"], weights["head_b"], Yg)
    return Yg, logits


# --------------------------------------------------------------------------- algorithmic FLOPs
def algorithmic_flops(cfg, lens=None, B: Optional[int] = None, L: Optional[int] = None) -> dict:
    """FLOPs on valid tokens only, counted the way Eq. 3 counts them: 2 per
    multiply-add of every projection / FFN GEMM (24 d^2 per token of a block)
    and 4 d per unmasked query-key pair.  LayerNorm, softmax, GELU, pooling and
    the head are not counted."""
    B = cfg.B if B is None else B
    L = cfg.L if L is None else L
    lens = _lens(lens, B, L)
    d, m, k, K = cfg.d, cfg.m, cfg.k_recent, cfg.K
    f = cfg.ffn_mult
    per_tok_q = 2 * d * d + 2 * d * d + 4 * f * d * d      # W_Q, W_O, FFN
    per_tok_kv = 4 * d * d                                  # W_K, W_V
    di = d // K if getattr(cfg, "merge", "mean") == "concat" else d   # InnerTrans width
    per_tok_inner = (8 + 4 * f) * di * di
    inner = cross = selfl = 0
    for lu in lens:
        lu = int(lu)
        Tu = merged_len(lu, K)
        pairs = sum(min(K, lu - t * K) ** 2 for t in range(Tu))
        inner += cfg.inner_layers * (lu * per_tok_inner + 4 * di * pairs)
        slots = _query_tokens(cfg, 0, Tu)
        kv = sum(1 for s in slots if s[2])             # valid sequence-side query slots
        # cross layer: keys = m globals + Tu merged tokens; queries = m globals + kv slots
        gpairs = m * m if cfg.gmask == "full" else m * (m + 1) // 2
        seqpairs = sum(min(s[1] + 1, Tu) for s in slots if s[2])
        cross += (m + Tu) * per_tok_kv + (m + kv) * per_tok_q + 4 * d * (gpairs + m * Tu + seqpairs)
        spairs = kv * (kv + 1) // 2
        selfl += (m + kv) * (per_tok_q + per_tok_kv) + 4 * d * (gpairs + m * kv + spairs)
    total = inner + cross + cfg.n_self * selfl
    return {"inner": inner, "cross": cross, "self_each": selfl, "total": total}


def algorithmic_flops_score(cfg, Tu: int) -> int:
    """FLOPs to score one candidate against a cache with Tu valid merged tokens."""
    d, m, k = cfg.d, cfg.m, cfg.k_recent
    per_tok = (24 * d * d) if cfg.ffn_mult == 4 else (8 + 4 * cfg.ffn_mult) * d * d
    gp = m * m if cfg.gmask == "full" else m * (m + 1) // 2
    kv = sum(1 for t in _query_tokens(cfg, 0, Tu) if t[2])
    tot = m * per_tok + 4 * d * (gp + m * Tu)
    tot += cfg.n_self * (m * per_tok + 4 * d * (gp + m * kv))
    return tot
