"""The benchmark's own FLOP counter (paper_2505_04421_amd.flops) against the oracle's counter, which
the paper's printed FLOP example pins (tests/test_oracle_pins.py).  No GPU needed."""
import numpy as np

import longer_synth as synth
from oracle import longer_oracle as orc


def test_benchmark_flop_counter_agrees_with_the_oracle_counter():
    """The benchmark prices its roofline figures with a counter of its own (the package's flops module,
    so that the product path never touches the oracle); the two counters are written independently
    and must agree on every configuration, query strategy and ragged length mix."""
    from paper_2505_04421_amd import flops
    rng = np.random.default_rng(77)
    cases = [(synth.CONFIGS[n], None) for n in ("C1", "C2", "C3", "C5", "P1")]
    c4 = synth.CONFIGS["C4"]
    cases.append((c4.replace(B=40), rng.integers(0, 5001, 40)))
    cases.append((synth.CONFIGS["C3"].replace(B=7, k_uniform=50), rng.integers(0, 2001, 7)))
    cases.append((synth.CONFIGS["C3"].replace(B=7, k_uniform=100, gmask="causal"), rng.integers(0, 2001, 7)))
    cases.append((synth.CONFIGS["C3"].replace(B=7, q_learnable=True), np.array([0, 1, 7, 8, 9, 1999, 2000])))
    cases.append((synth.CONFIGS["C2"].replace(B=5, ffn_mult=2, k_recent=150), np.array([512, 0, 100, 37, 511])))
    for cfg, lens in cases:
        a = orc.algorithmic_flops(cfg, lens)
        b = flops.forward_flops(cfg, lens)
        for key in ("inner", "cross", "self_each", "total"):
            assert a[key] == b[key], (cfg.name, key)
        for tu in (0, 1, cfg.k_recent - 1, cfg.k_recent, cfg.T):
            assert orc.algorithmic_flops_score(cfg, tu) == flops.score_flops(cfg, tu), (cfg.name, tu)
    # the K/V share of the cross layer, by hand at the headline shape: (8 + 250) key rows x 4 d^2
    assert flops.forward_flops(synth.CONFIGS["C3"], B=1)["kv_cross"] == 258 * 4 * 128 * 128


def test_backward_work_tally_by_hand_at_the_headline_shape():
    """C3: 512 000 tokens, width 128, FFN width 512, two InnerTrans blocks (Eq. 3: 24 d^2 per token and
    block + 4 K d of attention inside a group of K)."""
    from paper_2505_04421_amd import flops
    w = flops.merge_backward_work(synth.CONFIGS["C3"])
    tokens = 256 * 2000
    block = tokens * (24 * 128 * 128 + 4 * 8 * 128)
    assert w["gradient_flops"] == 2 * 2 * block
    # recomputed: block 0 in full (the chain of block inputs), then both blocks without the second FFN product
    assert w["recompute_flops"] == block + 2 * (block - tokens * 2 * 128 * 512)
    # bytes per token: 6 w for block 1's input, per block 38 w recomputed and 92 w + 10 f of gradients, 12 w once
    assert w["hbm_bytes"] == tokens * (6 * 128 + 2 * 38 * 128 + 2 * (92 * 128 + 10 * 512) + 12 * 128)
    # a ragged batch: FLOPs and bytes follow the valid tokens; a padded token costs the zeros written for it
    c = synth.CONFIGS["C2"].replace(B=3)                 # width 64, FFN width 256, one block
    r = flops.merge_backward_work(c, [0, 100, 512])
    assert r["gradient_flops"] == 2 * flops.forward_flops(c, [0, 100, 512])["inner"]
    assert r["hbm_bytes"] == 612 * (38 * 64 + (92 * 64 + 10 * 256) + 12 * 64) + (3 * 512 - 612) * (16 * 64 + 10 * 64)
