"""Algorithmic FLOP counts of the LONGER forward and scoring passes (bookkeeping for the
benchmark's roofline figures; nothing here runs on the data).

Counted the way Eq. 3 of the paper counts a transformer layer: 2 FLOP per multiply-add of every
projection / FFN GEMM (24 d^2 per token of a block with a 4d FFN) and 4 d per unmasked query-key
pair, on valid tokens only.  LayerNorm, softmax, the activation, pooling and the head are not
counted.
"""
from __future__ import annotations

from typing import Optional, Sequence


def _slot_tokens(k: int, tu: int, k_uniform: int, q_learnable: bool):
    """(newest merged token a valid query slot sees) for every valid one of a user's k slots
    (Section 3.5.1): learnable tokens see all tu tokens; sampled slots hold a token and see the
    tokens up to it."""
    if tu <= 0:
        return []
    if q_learnable:
        return [tu - 1] * k
    out = []
    for i in range(k):
        if tu <= k or i >= k_uniform:
            t = tu - k + i
        else:
            rest = tu - (k - k_uniform)
            t = ((i + 1) * rest) // k_uniform - 1
        if t >= 0:
            out.append(t)
    return out


def forward_flops(cfg, lens: Optional[Sequence[int]] = None, B: Optional[int] = None, L: Optional[int] = None) -> dict:
    """{"inner", "cross", "self_each", "kv_cross", "total"} for one longer_forward call."""
    B = cfg.B if B is None else B
    L = cfg.L if L is None else L
    lens = [L] * B if lens is None else [int(x) for x in lens]
    d, m, k, K, f = cfg.d, cfg.m, cfg.k_recent, cfg.K, cfg.ffn_mult
    q_side = (4 + 4 * f) * d * d            # W_Q, W_O and the FFN per query row
    kv_side = 4 * d * d                     # W_K, W_V per key row
    di = d // K if getattr(cfg, "merge", "mean") == "concat" else d
    inner_tok = (8 + 4 * f) * di * di
    gpairs = m * m if cfg.gmask == "full" else m * (m + 1) // 2
    inner = cross = selfl = kv_cross = 0
    for lu in lens:
        lu = min(max(lu, 0), L)
        tu = (lu + K - 1) // K
        full, rem = divmod(lu, K)
        inner += cfg.inner_layers * (lu * inner_tok + 4 * di * (full * K * K + rem * rem))
        slots = _slot_tokens(k, tu, getattr(cfg, "k_uniform", 0), getattr(cfg, "q_learnable", False))
        kv = len(slots)
        seqpairs = sum(min(t + 1, tu) for t in slots)
        kv_cross += (m + tu) * kv_side
        cross += (m + tu) * kv_side + (m + kv) * q_side + 4 * d * (gpairs + m * tu + seqpairs)
        selfl += (m + kv) * (q_side + kv_side) + 4 * d * (gpairs + m * kv + kv * (kv + 1) // 2)
    return {"inner": inner, "cross": cross, "self_each": selfl, "kv_cross": kv_cross,
            "total": inner + cross + cfg.n_self * selfl}


def score_flops(cfg, tu: int) -> int:
    """One candidate scored against a cache with tu valid merged tokens (Section 3.6.3, stage 2)."""
    d, m, f = cfg.d, cfg.m, cfg.ffn_mult
    per_row = (8 + 4 * f) * d * d
    gpairs = m * m if cfg.gmask == "full" else m * (m + 1) // 2
    kv = len(_slot_tokens(cfg.k_recent, tu, getattr(cfg, "k_uniform", 0), getattr(cfg, "q_learnable", False)))
    return m * per_row + 4 * d * (gpairs + m * tu) + cfg.n_self * (m * per_row + 4 * d * (gpairs + m * kv))


def merge_backward_work(cfg, lens: Optional[Sequence[int]] = None, B: Optional[int] = None, L: Optional[int] = None) -> dict:
    """Work of one longer_token_merge_backward call (Section 3.6.2: recomputation, mixed precision).

    ``gradient_flops``: the products a backward pass adds to the forward ones, two per forward
    product (the gradient of its input and of its weight): 2 x the InnerTrans forward count, on
    valid tokens.  ``recompute_flops``: the forward products that are computed again (the chain of
    block inputs: all blocks but the last; then every block's intermediates, without its second
    FFN product).  ``hbm_bytes``: what the pass's kernels read and write when every tensor makes one
    trip per use.  Per valid token and block 38 w bytes for the recomputed intermediates (up to the
    FFN's input; the hidden pre-activation is formed again inside the launch that takes its gradient and
    never stored) and 92 w + 10 f for the gradients, 6 w for every block input that the fused forward kernel recomputes (it
    reads the raw tokens and writes fp32 rows), 12 w once for the input copy and the merge gradient.  A
    padded token is never read; it costs the zeros written for it: 16 w per block (two LayerNorm outputs,
    two LayerNorm gradients with their bf16 copies), 4 w per recomputed block input, 10 w once."""
    B = cfg.B if B is None else B
    L = cfg.L if L is None else L
    w = cfg.d // cfg.K if getattr(cfg, "merge", "mean") == "concat" else cfg.d
    f = cfg.ffn_mult * w
    n = cfg.inner_layers
    inner = forward_flops(cfg, lens, B, L)["inner"]
    ffn2 = 4 * w * f // 2                                   # 2 w f FLOP per token: the second FFN product
    lens_ = [L] * B if lens is None else [min(max(int(x), 0), L) for x in lens]
    valid = sum(lens_)
    per_block = inner // max(n, 1)
    recompute = (n - 1) * per_block + n * (per_block - ffn2 * valid)
    per_token = (n - 1) * 6 * w + n * 38 * w + n * (92 * w + 10 * f) + 12 * w
    per_padded = (n - 1) * 4 * w + n * 16 * w + 10 * w
    return {"gradient_flops": 2 * inner, "recompute_flops": recompute,
            "hbm_bytes": per_token * valid + per_padded * (B * L - valid)}
