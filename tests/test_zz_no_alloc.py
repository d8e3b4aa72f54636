"""longer_score_candidates_static (the scoring entry point that takes no workspace and allocates
nothing) against longer_score_candidates, through the raw C ABI: two calls in a row, the second on
a smaller input, each bit for bit equal to the workspace-taking entry point on the same inputs."""
import ctypes

import numpy as np
import pytest
import torch

import longer_synth as synth

pytestmark = pytest.mark.gpu


def _serve_both_ways(cfg, seed_index):
    import paper_2505_04421_amd as lg
    lib = lg.load_library()
    case = synth.make_case(cfg.replace(index=seed_index), pad_value=float("nan"))
    model = lg.DeviceModel(cfg, case["weights"])
    U, L, C = cfg.B, cfg.L, cfg.C
    lens = torch.from_numpy(case["lens"].astype(np.int32)).to(model.device)
    H, Gc = model.upload(case["H"]), model.upload(case["G_cand"])
    ws = model.workspace(U, L)
    cache = model.kv_cache(U, L)
    lg.longer_kv_cache_build(model.ccfg, model.weights, H, lens, U, L, cache, ws)
    Yg_a, sc_a = model.empty(U, C, cfg.m, cfg.d), model.empty(U, C, dtype=torch.float32)
    Yg_b, sc_b = model.empty(U, C, cfg.m, cfg.d), model.empty(U, C, dtype=torch.float32)
    for t in (Yg_a, sc_a, Yg_b, sc_b):
        t.fill_(7.0)
    stream = torch.cuda.current_stream().cuda_stream or None
    print("  longer_score_candidates: %s, %d users x %d candidates" % (cfg.name, U, C), flush=True)
    rc = lib.longer_score_candidates(ctypes.byref(model.ccfg), ctypes.byref(model.weights), cache.data_ptr(), lens.data_ptr(),
                                     U, L, Gc.data_ptr(), C, Yg_a.data_ptr(), sc_a.data_ptr(), ws.data_ptr(), ws.numel(), stream)
    assert rc == 0, lg.longer_last_error()
    print("  longer_score_candidates_static", flush=True)
    rc = lib.longer_score_candidates_static(ctypes.byref(model.ccfg), ctypes.byref(model.weights), cache.data_ptr(), lens.data_ptr(),
                                            U, L, Gc.data_ptr(), C, Yg_b.data_ptr(), sc_b.data_ptr(), stream)
    assert rc == 0, lg.longer_last_error()
    torch.cuda.synchronize()
    assert torch.isfinite(sc_a).all() and torch.isfinite(Yg_a.float()).all()
    assert torch.equal(Yg_a, Yg_b) and torch.equal(sc_a, sc_b)
    return float(sc_a.abs().sum())


def test_static_scoring_equals_workspace_scoring_twice_in_a_row():
    big = synth.CONFIGS["C5"].replace(B=3, L=2000, C=40, ragged=True, len_lo=100, len_hi=2000)
    s1 = _serve_both_ways(big, 51)
    # the second call: a narrower model with fewer layers, users and candidates; the static array still
    # holds the first call's (larger) parameters
    small = synth.CONFIGS["C2"].replace(B=2, L=300, C=5, n_self=1, ragged=True, len_lo=0, len_hi=300)
    s2 = _serve_both_ways(small, 52)
    assert s1 > 0 and s2 > 0


def test_static_scoring_rejects_a_model_beyond_its_scratch():
    import paper_2505_04421_amd as lg
    lib = lg.load_library()
    cfg = lg.make_config(synth.CONFIGS["C5"].replace(n_self=6))      # 7 blocks of 1.5 MiB: more than 8 MiB
    blk = (lg.binding.CBlock * 8)()
    w = lg.binding.CWeights(inner=blk, cross=blk, self=blk, head_w=None, head_b=None, packed=None)
    fake = ctypes.c_void_p(4096)
    rc = lib.longer_score_candidates_static(ctypes.byref(cfg), ctypes.byref(w), fake, None, 2, 100, fake, 3, fake, fake, None)
    assert rc == -2 and "static scratch" in lg.longer_last_error()
