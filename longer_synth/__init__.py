"""Seeded synthetic inputs for the LONGER forward / KV-cache hot path.

This module only *draws numbers and shapes them*: it holds none of the method's
arithmetic (no LayerNorm, attention, merge, mask).  Both the CPU oracle's tests
and the HIP path's tests / benchmark take their inputs from here, so the two
sides see the same values without sharing any model code.

The paper's own workload is proprietary behaviour logs (Experimental Setting,
Section 4.1); the tensors drawn here stand in for it with the shapes of the five
benchmark configurations.  Typical production shape in the paper: L = 2000,
d = 32 (Token Merge, Section 3.4), longest deployed sequence 10 000
(Introduction, contribution list).

Conventions
-----------
* everything is drawn in fp32 from ``numpy.random.Philox`` (a counter-based
  generator) seeded with ``SEED_BASE + config_index``; draw order is fixed:
  inner blocks, cross block, self blocks, head, (learnable query tokens), then H, G,
  G_cand, lens.
* weights are stored ``[in, out]`` so that ``y = x @ W + b`` (Eq. 6 writes
  ``Q = O W_Q``).
* in bf16 mode every tensor is rounded once to bf16 (round-to-nearest-even) and
  returned as fp32 values that are exactly representable in bf16; ``bf16_bits``
  gives the uint16 payload for the device.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Sequence

import numpy as np

SEED_BASE = 250504421

BLOCK_FIELDS = ("ln1_g", "ln1_b", "wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo",
                "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


@dataclasses.dataclass
class Config:
    """Model + workload shape.  Field names follow the paper's notation:
    d width, m global tokens, K merge group, k_recent sampled recent queries,
    n_self = N stacked self-attention layers (Section 3.4-3.5)."""
    name: str
    index: int
    B: int                 # users in the batch
    L: int                 # padded raw sequence length
    d: int
    heads: int
    m: int
    K: int
    k_recent: int
    n_self: int
    inner_layers: int
    inner_heads: int
    dtype: str             # "f32" | "bf16"
    ffn_mult: int = 4
    act: str = "gelu_erf"  # "gelu_erf" | "relu"
    gmask: str = "full"    # "full" | "causal"  (global->global visibility)
    ln_eps: float = 1e-5
    dist: str = "normal"   # "normal" | "lognormal_scaled"
    ragged: bool = False
    len_lo: int = 0
    len_hi: int = 0
    C: int = 0             # candidates per user (serving config only)
    k_uniform: int = 0     # of the k_recent query slots, how many are sampled uniformly from the older tokens
    merge: str = "mean"    # "mean": K outputs of a group pooled to one token of width d;
                           # "concat": raw tokens of width d / K, a group's K outputs concatenated
    q_learnable: bool = False  # the k_recent query slots hold learnable tokens (a [k_recent, d] parameter
                               # shared by all users) instead of tokens sampled from the sequence

    @property
    def T(self) -> int:
        return (self.L + self.K - 1) // self.K

    @property
    def d_in(self) -> int:
        """Width of the raw tokens H and of the InnerTrans blocks."""
        return self.d // self.K if self.merge == "concat" else self.d

    @property
    def n(self) -> int:
        return self.m + self.k_recent

    def replace(self, **kw) -> "Config":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[str, Config] = {
    # the five benchmark configurations, in order
    "C1": Config("C1", 0, B=4, L=64, d=32, heads=2, m=2, K=4, k_recent=8, n_self=1,
                 inner_layers=1, inner_heads=2, dtype="f32"),
    "C2": Config("C2", 1, B=128, L=512, d=64, heads=4, m=4, K=8, k_recent=32, n_self=2,
                 inner_layers=1, inner_heads=4, dtype="bf16"),
    "C3": Config("C3", 2, B=256, L=2000, d=128, heads=8, m=8, K=8, k_recent=100, n_self=3,
                 inner_layers=2, inner_heads=8, dtype="bf16", dist="lognormal_scaled"),
    "C4": Config("C4", 3, B=512, L=5000, d=128, heads=8, m=8, K=16, k_recent=64, n_self=3,
                 inner_layers=1, inner_heads=8, dtype="bf16", ragged=True, len_lo=100, len_hi=5000),
    "C5": Config("C5", 4, B=16, L=10000, d=256, heads=8, m=8, K=16, k_recent=64, n_self=3,
                 inner_layers=1, inner_heads=8, dtype="bf16", C=1000),
    # not a benchmark configuration: the paper's own typical shape (Section 3.4: L = 2000, raw width 32)
    # merged by concatenation, K = 8 -> main stack at width 256
    "P1": Config("P1", 5, B=256, L=2000, d=256, heads=8, m=8, K=8, k_recent=100, n_self=3,
                 inner_layers=1, inner_heads=2, dtype="bf16", dist="lognormal_scaled", merge="concat"),
}


# --------------------------------------------------------------------------- bf16
def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result is fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    out = r.astype(np.uint32).view(np.float32).reshape(x.shape)
    nan = np.isnan(x)
    if nan.any():
        out = out.copy()
        out[nan] = np.nan
    return out


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 payload of values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Inverse of ``bf16_bits``."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


# --------------------------------------------------------------------------- draws
def _rng(cfg: Config) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(SEED_BASE + cfg.index))


def _uniform(rng, shape, a) -> np.ndarray:
    return rng.uniform(-a, a, size=shape).astype(np.float32)


def draw_block(rng: np.random.Generator, d: int, ffn_mult: int = 4) -> Dict[str, np.ndarray]:
    """One transformer block's 12 d^2 + 13 d scalars (for ffn_mult = 4; Eq. 3, Params).
    Matrices are Xavier-uniform; biases and LayerNorm affine terms are drawn
    non-trivial so that every term of the block is exercised."""
    f = ffn_mult * d

    def xavier(fi, fo):
        return _uniform(rng, (fi, fo), np.sqrt(6.0 / (fi + fo)))

    blk = {}
    blk["ln1_g"] = rng.uniform(0.9, 1.1, size=d).astype(np.float32)
    blk["ln1_b"] = _uniform(rng, d, 0.05)
    for nm in ("q", "k", "v", "o"):
        blk["w" + nm] = xavier(d, d)
        blk["b" + nm] = _uniform(rng, d, 0.05)
    blk["ln2_g"] = rng.uniform(0.9, 1.1, size=d).astype(np.float32)
    blk["ln2_b"] = _uniform(rng, d, 0.05)
    blk["w1"] = xavier(d, f)
    blk["b1"] = _uniform(rng, f, 0.05)
    blk["w2"] = xavier(f, d)
    blk["b2"] = _uniform(rng, d, 0.05)
    return {k: blk[k] for k in BLOCK_FIELDS}


def draw_weights(cfg: Config, rng: Optional[np.random.Generator] = None) -> Dict[str, object]:
    rng = _rng(cfg) if rng is None else rng
    w = {
        "inner": [draw_block(rng, cfg.d_in, cfg.ffn_mult) for _ in range(cfg.inner_layers)],
        "cross": draw_block(rng, cfg.d, cfg.ffn_mult),
        "self": [draw_block(rng, cfg.d, cfg.ffn_mult) for _ in range(cfg.n_self)],
        "head_w": _uniform(rng, cfg.m * cfg.d, np.sqrt(6.0 / (cfg.m * cfg.d + 1))),
        "head_b": _uniform(rng, 1, 0.05),
    }
    if cfg.q_learnable:      # drawn last, so that the other parameters do not depend on the query strategy
        w["q_learn"] = rng.standard_normal(size=(cfg.k_recent, cfg.d), dtype=np.float32)
    return w


def draw_input_mlp(rng: np.random.Generator, cfg: "Config", d_e: int) -> Dict[str, np.ndarray]:
    """Parameters of the input-generation stage (Section 3.5.1, Input Generation): a learnable
    absolute positional embedding ``pos`` [L, d_e] added to the item embeddings, and a two-layer
    MLP d -> ffn_mult d -> d over [item + position ; time-difference feature]."""
    d, f = cfg.d, cfg.ffn_mult * cfg.d
    return {
        "pos": _uniform(rng, (cfg.L, d_e), 0.5),
        "w1": _uniform(rng, (d, f), np.sqrt(6.0 / (d + f))),
        "b1": _uniform(rng, f, 0.05),
        "w2": _uniform(rng, (f, d), np.sqrt(6.0 / (d + f))),
        "b2": _uniform(rng, d, 0.05),
    }


def make_input_case(cfg: "Config", d_e: int, seed_offset: int = 1000) -> Dict[str, object]:
    """Item embeddings E [B, L, d_e], time-difference features tdiff [B, L, d - d_e], the
    input-generation parameters and (ragged configurations) raw lengths; padded rows hold NaN."""
    rng = np.random.Generator(np.random.Philox(SEED_BASE + seed_offset + cfg.index))
    mlp = draw_input_mlp(rng, cfg, d_e)
    E = rng.standard_normal(size=(cfg.B, cfg.L, d_e), dtype=np.float32)
    tdiff = rng.standard_normal(size=(cfg.B, cfg.L, cfg.d - d_e), dtype=np.float32)
    lens = None
    if cfg.ragged:
        lens = rng.integers(cfg.len_lo, cfg.len_hi + 1, size=cfg.B).astype(np.int32)
        pos = np.arange(cfg.L)[None, :, None]
        E = np.where(pos < lens[:, None, None], E, np.float32("nan")).astype(np.float32)
        tdiff = np.where(pos < lens[:, None, None], tdiff, np.float32("nan")).astype(np.float32)
    case = {"cfg": cfg, "mlp": mlp, "E": E, "tdiff": tdiff, "lens": lens}
    if cfg.dtype == "bf16":
        case = _map_tree(case, round_bf16)
    return case


def _tokens(rng, shape, dist) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if dist == "lognormal_scaled":
        # every token row is scaled by exp(N(0,1)): heavy-tailed row norms
        s = np.exp(rng.standard_normal(size=shape[:-1] + (1,), dtype=np.float32))
        x = x * s
    return x.astype(np.float32)


def _map_tree(tree, fn):
    if isinstance(tree, dict):
        return {k: _map_tree(v, fn) for k, v in tree.items()}
    if isinstance(tree, list):
        return [_map_tree(v, fn) for v in tree]
    if isinstance(tree, np.ndarray) and tree.dtype == np.float32:
        return fn(tree)
    return tree


def make_case(cfg: Config, *, users: Optional[int] = None, candidates: Optional[int] = None,
              pad_value: float = 0.0) -> Dict[str, object]:
    """Draw weights and inputs for ``cfg``.

    ``users`` / ``candidates`` cut the batch (the first users / candidates of the
    full draw would differ: a cut case is its own seeded case, drawn at the cut
    shape).  ``pad_value`` fills the padded tail of ragged sequences (NaN in the
    padding-robustness parity runs, 0 in timing runs).

    Returns ``{"cfg", "weights", "H", "G", "lens", "G_cand"}``; float tensors are
    fp32 ndarrays (bf16-representable when ``cfg.dtype == "bf16"``); ``lens`` is
    int32 ``[B]`` or None.
    """
    if users is not None:
        cfg = cfg.replace(B=users)
    if candidates is not None:
        cfg = cfg.replace(C=candidates)
    rng = _rng(cfg)
    w = draw_weights(cfg, rng)
    H = _tokens(rng, (cfg.B, cfg.L, cfg.d_in), cfg.dist)
    G = _tokens(rng, (cfg.B, cfg.m, cfg.d), cfg.dist)
    G_cand = None
    if cfg.C > 0:
        G_cand = _tokens(rng, (cfg.B, cfg.C, cfg.m, cfg.d), cfg.dist)
    lens = None
    if cfg.ragged:
        lens = rng.integers(cfg.len_lo, cfg.len_hi + 1, size=cfg.B).astype(np.int32)
        pos = np.arange(cfg.L)[None, :, None]
        H = np.where(pos < lens[:, None, None], H, np.float32(pad_value)).astype(np.float32)
    case = {"cfg": cfg, "weights": w, "H": H, "G": G, "G_cand": G_cand, "lens": lens}
    if cfg.dtype == "bf16":
        case = _map_tree(case, round_bf16)
    return case


def tiny_config(**kw) -> Config:
    """A small fp32 configuration for brute-force and invariant tests."""
    base = dict(name="tiny", index=100, B=2, L=12, d=8, heads=2, m=2, K=4, k_recent=2, n_self=1,
                inner_layers=1, inner_heads=2, dtype="f32")
    base.update(kw)
    return Config(**base)


def draw_merge_gradient(cfg: Config, seed_offset: int = 7000, users: Optional[Sequence[int]] = None) -> np.ndarray:
    """Upstream gradient dM [B, T, d] (fp32, N(0, 1)) for the backward pass of the token merge: what the
    loss would hand back for the merged tokens.  ``users``: only these users get a non-zero gradient
    (the parameter gradients of a batch are then those of the chosen users alone)."""
    rng = np.random.default_rng(2505_04421 + 7919 * cfg.index + seed_offset)
    dM = rng.standard_normal((cfg.B, cfg.T, cfg.d)).astype(np.float32)
    if users is not None:
        keep = np.zeros(cfg.B, dtype=bool)
        keep[list(users)] = True
        dM[~keep] = 0.0
    return dM


def draw_labels(cfg: Config, seed_offset: int = 9000) -> np.ndarray:
    """Binary labels [B] (fp32 0 / 1) for the loss of Eq. 2."""
    rng = np.random.default_rng(2505_04421 + 7919 * cfg.index + seed_offset)
    return (rng.random(cfg.B) < 0.5).astype(np.float32)
