"""ctypes binding of liblonger.so.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

BLOCK_FIELDS = ("ln1_g", "ln1_b", "wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo",
                "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")
ENTRY_POINTS = ("longer_workspace_bytes", "longer_kv_cache_bytes", "longer_inner_transformer",
                "longer_token_merge", "longer_hybrid_cross_attn", "longer_self_attn_layer",
                "longer_forward", "longer_kv_cache_build", "longer_score_candidates", "longer_input_generation",
                "longer_forward_from_inputs", "longer_kv_cache_build_from_inputs",
                "longer_last_error", "longer_probe_mfma_layout", "longer_stage_timing",
                "longer_stage_timing_read", "longer_packed_weights_bytes", "longer_pack_weights",
                "longer_score_candidates_static", "longer_probe_rate",
                "longer_backward_workspace_bytes", "longer_block_grad_floats", "longer_token_merge_backward",
                "longer_model_grad_floats", "longer_forward_backward_workspace_bytes", "longer_forward_backward",
                "longer_input_backward_workspace_bytes", "longer_input_grad_floats", "longer_input_generation_backward")


class LongerError(RuntimeError):
    pass


class CConfig(ctypes.Structure):
    _fields_ = [("d", ctypes.c_int32), ("heads", ctypes.c_int32), ("ffn_mult", ctypes.c_int32),
                ("m", ctypes.c_int32), ("K", ctypes.c_int32), ("k_recent", ctypes.c_int32),
                ("n_self", ctypes.c_int32), ("inner_layers", ctypes.c_int32), ("inner_heads", ctypes.c_int32),
                ("act", ctypes.c_int32), ("gmask", ctypes.c_int32), ("ln_eps", ctypes.c_float),
                ("dtype", ctypes.c_int32), ("merge", ctypes.c_int32), ("k_uniform", ctypes.c_int32),
                ("q_learn", ctypes.c_void_p)]


class CBlock(ctypes.Structure):
    _fields_ = [(f, ctypes.c_void_p) for f in BLOCK_FIELDS]


class CWeights(ctypes.Structure):
    _fields_ = [("inner", ctypes.POINTER(CBlock)), ("cross", ctypes.POINTER(CBlock)),
                ("self", ctypes.POINTER(CBlock)), ("head_w", ctypes.c_void_p), ("head_b", ctypes.c_void_p),
                ("packed", ctypes.c_void_p)]


class CInputWeights(ctypes.Structure):
    _fields_ = [(f, ctypes.c_void_p) for f in ("pos", "w1", "b1", "w2", "b2")]


def library_path() -> str:
    return os.path.join(HERE, "liblonger.so")


def load_library() -> ctypes.CDLL:
    """Load the in-tree library; raises LongerError when it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise LongerError("liblonger.so is not built: run `python -m paper_2505_04421_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    lib = ctypes.CDLL(path)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    cfgp, blkp, wp = ctypes.POINTER(CConfig), ctypes.POINTER(CBlock), ctypes.POINTER(CWeights)
    lib.longer_workspace_bytes.restype = sz
    lib.longer_workspace_bytes.argtypes = [cfgp, i32, i32]
    lib.longer_kv_cache_bytes.restype = sz
    lib.longer_kv_cache_bytes.argtypes = [cfgp, i32, i32]
    lib.longer_inner_transformer.argtypes = [cfgp, blkp, vp, vp, i32, i32, vp, vp, sz, vp]
    lib.longer_token_merge.argtypes = [cfgp, blkp, vp, vp, i32, i32, vp, vp, sz, vp]
    lib.longer_hybrid_cross_attn.argtypes = [cfgp, blkp, vp, vp, vp, i32, i32, vp, vp, sz, vp]
    lib.longer_self_attn_layer.argtypes = [cfgp, blkp, vp, vp, i32, i32, vp, vp, sz, vp]
    lib.longer_forward.argtypes = [cfgp, wp, vp, vp, vp, i32, i32, vp, vp, vp, sz, vp]
    lib.longer_kv_cache_build.argtypes = [cfgp, wp, vp, vp, i32, i32, vp, vp, sz, vp]
    lib.longer_score_candidates.argtypes = [cfgp, wp, vp, vp, i32, i32, vp, i32, vp, vp, vp, sz, vp]
    lib.longer_input_generation.argtypes = [cfgp, ctypes.POINTER(CInputWeights), vp, vp, vp, i32, i32, i32, vp, vp, sz, vp]
    lib.longer_forward_from_inputs.argtypes = [cfgp, wp, ctypes.POINTER(CInputWeights), vp, vp, i32, vp, vp, i32, i32,
                                               vp, vp, vp, sz, vp]
    lib.longer_kv_cache_build_from_inputs.argtypes = [cfgp, wp, ctypes.POINTER(CInputWeights), vp, vp, i32, vp, i32, i32,
                                                      vp, vp, sz, vp]
    lib.longer_packed_weights_bytes.restype = sz
    lib.longer_packed_weights_bytes.argtypes = [cfgp]
    lib.longer_pack_weights.argtypes = [cfgp, wp, ctypes.POINTER(CInputWeights), vp, sz, vp]
    lib.longer_score_candidates_static.argtypes = [cfgp, wp, vp, vp, i32, i32, vp, i32, vp, vp, vp]
    lib.longer_probe_rate.argtypes = [i32, i32, i32, vp, vp]
    lib.longer_backward_workspace_bytes.restype = sz
    lib.longer_backward_workspace_bytes.argtypes = [cfgp, i32, i32]
    lib.longer_block_grad_floats.restype = sz
    lib.longer_block_grad_floats.argtypes = [cfgp]
    lib.longer_token_merge_backward.argtypes = [cfgp, blkp, vp, vp, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.longer_model_grad_floats.restype = sz
    lib.longer_model_grad_floats.argtypes = [cfgp]
    lib.longer_forward_backward_workspace_bytes.restype = sz
    lib.longer_forward_backward_workspace_bytes.argtypes = [cfgp, i32, i32]
    lib.longer_forward_backward.argtypes = [cfgp, wp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.longer_input_backward_workspace_bytes.restype = sz
    lib.longer_input_backward_workspace_bytes.argtypes = [cfgp, i32, i32, i32]
    lib.longer_input_grad_floats.restype = sz
    lib.longer_input_grad_floats.argtypes = [cfgp, i32, i32]
    lib.longer_input_generation_backward.argtypes = [cfgp, ctypes.POINTER(CInputWeights), vp, vp, vp, i32, i32, i32, vp, vp, vp, vp,
                                                     vp, sz, vp]
    lib.longer_last_error.restype = ctypes.c_char_p
    lib.longer_probe_mfma_layout.argtypes = [vp, vp]
    lib.longer_stage_timing.argtypes = [i32]
    lib.longer_stage_timing_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)]
    for name in ENTRY_POINTS:
        if name not in ("longer_workspace_bytes", "longer_kv_cache_bytes", "longer_packed_weights_bytes", "longer_last_error",
                        "longer_backward_workspace_bytes", "longer_block_grad_floats", "longer_model_grad_floats",
                        "longer_forward_backward_workspace_bytes", "longer_input_backward_workspace_bytes",
                        "longer_input_grad_floats"):
            getattr(lib, name).restype = ctypes.c_int
    _LIB = lib
    return lib


def exported_symbols() -> List[str]:
    lib = load_library()
    return [n for n in ENTRY_POINTS if hasattr(lib, n)]


def longer_last_error() -> str:
    return load_library().longer_last_error().decode()


def _check(rc: int, what: str):
    if rc != 0:
        raise LongerError("%s failed (%d): %s" % (what, rc, longer_last_error()))


_ACT = {"gelu_erf": 0, "relu": 1}
_GMASK = {"full": 0, "causal": 1}
_DTYPE = {"f32": 0, "bf16": 1}
_MERGE = {"mean": 0, "concat": 1}


def make_config(cfg, q_learn=None) -> CConfig:
    """From any object with the config's attribute names (e.g. longer_synth.Config); ``q_learn`` is the
    device tensor [k_recent, d] of learnable query tokens (the caller keeps it alive), or None."""
    return CConfig(q_learn=_ptr(q_learn), d=cfg.d, heads=cfg.heads, ffn_mult=cfg.ffn_mult, m=cfg.m, K=cfg.K, k_recent=cfg.k_recent,
                   n_self=cfg.n_self, inner_layers=cfg.inner_layers, inner_heads=cfg.inner_heads,
                   act=_ACT[cfg.act], gmask=_GMASK[cfg.gmask], ln_eps=cfg.ln_eps, dtype=_DTYPE[cfg.dtype],
                   merge=_MERGE[getattr(cfg, "merge", "mean")], k_uniform=getattr(cfg, "k_uniform", 0))


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda or not t.is_contiguous():
        raise LongerError("tensor arguments must be contiguous device tensors")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    import torch
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _require_gpu():
    import torch
    if not torch.cuda.is_available():
        raise LongerError("no GPU visible: the LONGER hot path has no CPU fallback")


class DeviceModel:
    """Uploads a weight tree (numpy fp32, see longer_synth.draw_weights) to the GPU in the
    config's element type and keeps the C structs that point at it."""

    def __init__(self, cfg, weights: Dict[str, object], device: str = "cuda:0"):
        import torch
        _require_gpu()
        self.cfg = cfg
        self.ccfg = make_config(cfg)
        self.device = torch.device(device)
        self.tdtype = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        self._keep = []
        self.inner = (CBlock * max(1, len(weights["inner"])))(*[self._block(b) for b in weights["inner"]])
        self.cross = (CBlock * 1)(self._block(weights["cross"]))
        self.self_ = (CBlock * max(1, len(weights["self"])))(*[self._block(b) for b in weights["self"]])
        hw, hb = self.upload(weights["head_w"]), self.upload(weights["head_b"])
        self._keep += [hw, hb]
        self.weights = CWeights(inner=self.inner, cross=self.cross, self=self.self_,
                                head_w=hw.data_ptr(), head_b=hb.data_ptr())
        if getattr(cfg, "q_learnable", False):
            self.q_learn = self.upload(weights["q_learn"])
            self.ccfg.q_learn = self.q_learn.data_ptr()

    def upload(self, a):
        import torch
        import numpy as np
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.device).to(self.tdtype).contiguous()

    def _block(self, blk) -> CBlock:
        ts = {f: self.upload(blk[f]) for f in BLOCK_FIELDS}
        self._keep.append(ts)
        return CBlock(**{f: ts[f].data_ptr() for f in BLOCK_FIELDS})

    def empty(self, *shape, dtype=None):
        import torch
        return torch.empty(*shape, dtype=dtype or self.tdtype, device=self.device)

    def workspace(self, B: int, L: int, C: int = 0):
        """Scratch for a batch of B users of padded length L (C, the candidate count, does not enter)."""
        import torch
        n = longer_workspace_bytes(self.ccfg, B, L)
        if n == 0:
            raise LongerError("workspace size query failed: " + longer_last_error())
        return torch.empty(n, dtype=torch.uint8, device=self.device)

    def pack(self, iweights=None):
        """Pack the parameters once (longer_pack_weights) and return a CWeights that streams from the
        packed buffer; the model keeps the buffer alive."""
        import torch
        n = longer_packed_weights_bytes(self.ccfg)
        if n == 0:
            raise LongerError("packed size query failed: " + longer_last_error())
        buf = torch.empty(n, dtype=torch.uint8, device=self.device)
        longer_pack_weights(self.ccfg, self.weights, iweights, buf)
        self._keep.append(buf)
        return CWeights(inner=self.inner, cross=self.cross, self=self.self_, head_w=self.weights.head_w,
                        head_b=self.weights.head_b, packed=buf.data_ptr())

    def kv_cache(self, U: int, L: int):
        import torch
        n = longer_kv_cache_bytes(self.ccfg, U, L)
        if n == 0:
            raise LongerError("cache size query failed: " + longer_last_error())
        return torch.empty(n, dtype=torch.uint8, device=self.device)


# ----------------------------------------------------------------------------- entry points
def longer_workspace_bytes(ccfg: CConfig, B: int, L: int) -> int:
    return int(load_library().longer_workspace_bytes(ctypes.byref(ccfg), B, L))


def longer_packed_weights_bytes(ccfg: CConfig) -> int:
    return int(load_library().longer_packed_weights_bytes(ctypes.byref(ccfg)))


def longer_pack_weights(ccfg, weights, iweights, packed_out, stream=None):
    _require_gpu()
    _check(load_library().longer_pack_weights(ctypes.byref(ccfg), ctypes.byref(weights),
                                              None if iweights is None else ctypes.byref(iweights),
                                              _ptr(packed_out), packed_out.numel(), _stream(stream)), "longer_pack_weights")


def longer_score_candidates_static(ccfg, weights, cache, lens, U, L, G_cand, C, Yg_out, logits_out, stream=None):
    _require_gpu()
    _check(load_library().longer_score_candidates_static(ctypes.byref(ccfg), ctypes.byref(weights), _ptr(cache), _ptr(lens),
                                                         U, L, _ptr(G_cand), C, _ptr(Yg_out), _ptr(logits_out),
                                                         _stream(stream)), "longer_score_candidates_static")


def longer_probe_rate(mode, iters, workgroups, out, stream=None):
    _require_gpu()
    if out.numel() < workgroups * 512:
        raise LongerError("longer_probe_rate: out must hold workgroups * 512 floats")
    _check(load_library().longer_probe_rate(mode, iters, workgroups, _ptr(out), _stream(stream)), "longer_probe_rate")


def longer_kv_cache_bytes(ccfg: CConfig, U: int, L: int) -> int:
    return int(load_library().longer_kv_cache_bytes(ctypes.byref(ccfg), U, L))


def longer_inner_transformer(ccfg, inner, H, lens, B, L, Z_out, ws, stream=None):
    _require_gpu()
    _check(load_library().longer_inner_transformer(ctypes.byref(ccfg), inner, _ptr(H), _ptr(lens), B, L, _ptr(Z_out),
                                                   _ptr(ws), ws.numel(), _stream(stream)), "longer_inner_transformer")


def longer_token_merge(ccfg, inner, H, lens, B, L, M_out, ws, stream=None):
    _require_gpu()
    _check(load_library().longer_token_merge(ctypes.byref(ccfg), inner, _ptr(H), _ptr(lens), B, L, _ptr(M_out),
                                             _ptr(ws), ws.numel(), _stream(stream)), "longer_token_merge")


def longer_hybrid_cross_attn(ccfg, cross, G, M, lens, B, L, X_out, ws, stream=None):
    _require_gpu()
    _check(load_library().longer_hybrid_cross_attn(ctypes.byref(ccfg), cross, _ptr(G), _ptr(M), _ptr(lens), B, L,
                                                   _ptr(X_out), _ptr(ws), ws.numel(), _stream(stream)),
           "longer_hybrid_cross_attn")


def longer_self_attn_layer(ccfg, blk, X_in, lens, B, L, X_out, ws, stream=None):
    _require_gpu()
    _check(load_library().longer_self_attn_layer(ctypes.byref(ccfg), blk, _ptr(X_in), _ptr(lens), B, L, _ptr(X_out),
                                                 _ptr(ws), ws.numel(), _stream(stream)), "longer_self_attn_layer")


def longer_forward(ccfg, weights, H, G, lens, B, L, Y_out, logits_out, ws, stream=None):
    _require_gpu()
    _check(load_library().longer_forward(ctypes.byref(ccfg), ctypes.byref(weights), _ptr(H), _ptr(G), _ptr(lens), B, L,
                                         _ptr(Y_out), _ptr(logits_out), _ptr(ws), ws.numel(), _stream(stream)),
           "longer_forward")


def longer_kv_cache_build(ccfg, weights, H, lens, U, L, cache, ws, stream=None):
    _require_gpu()
    _check(load_library().longer_kv_cache_build(ctypes.byref(ccfg), ctypes.byref(weights), _ptr(H), _ptr(lens), U, L,
                                                _ptr(cache), _ptr(ws), ws.numel(), _stream(stream)),
           "longer_kv_cache_build")


def longer_score_candidates(ccfg, weights, cache, lens, U, L, G_cand, C, Yg_out, logits_out, ws, stream=None):
    _require_gpu()
    _check(load_library().longer_score_candidates(ctypes.byref(ccfg), ctypes.byref(weights), _ptr(cache), _ptr(lens), U, L,
                                                  _ptr(G_cand), C, _ptr(Yg_out), _ptr(logits_out), _ptr(ws), ws.numel(),
                                                  _stream(stream)), "longer_score_candidates")


def longer_input_generation(ccfg, weights, E, tdiff, lens, B, L, d_e, H_out, ws, stream=None):
    _require_gpu()
    _check(load_library().longer_input_generation(ctypes.byref(ccfg), ctypes.byref(weights), _ptr(E), _ptr(tdiff), _ptr(lens),
                                                  B, L, d_e, _ptr(H_out), _ptr(ws), ws.numel(), _stream(stream)),
           "longer_input_generation")


def longer_forward_from_inputs(ccfg, weights, iweights, E, tdiff, d_e, G, lens, B, L, Y_out, logits_out, ws, stream=None):
    _require_gpu()
    _check(load_library().longer_forward_from_inputs(ctypes.byref(ccfg), ctypes.byref(weights), ctypes.byref(iweights),
                                                     _ptr(E), _ptr(tdiff), d_e, _ptr(G), _ptr(lens), B, L, _ptr(Y_out),
                                                     _ptr(logits_out), _ptr(ws), ws.numel(), _stream(stream)),
           "longer_forward_from_inputs")


def longer_kv_cache_build_from_inputs(ccfg, weights, iweights, E, tdiff, d_e, lens, U, L, cache, ws, stream=None):
    _require_gpu()
    _check(load_library().longer_kv_cache_build_from_inputs(ctypes.byref(ccfg), ctypes.byref(weights), ctypes.byref(iweights),
                                                            _ptr(E), _ptr(tdiff), d_e, _ptr(lens), U, L, _ptr(cache),
                                                            _ptr(ws), ws.numel(), _stream(stream)),
           "longer_kv_cache_build_from_inputs")


def longer_backward_workspace_bytes(ccfg: CConfig, B: int, L: int) -> int:
    return int(load_library().longer_backward_workspace_bytes(ctypes.byref(ccfg), B, L))


def longer_block_grad_floats(ccfg: CConfig) -> int:
    return int(load_library().longer_block_grad_floats(ctypes.byref(ccfg)))


def _block_views(grads, o, d, f):
    shapes = {"ln1_g": (d,), "ln1_b": (d,), "wq": (d, d), "bq": (d,), "wk": (d, d), "bk": (d,), "wv": (d, d), "bv": (d,),
              "wo": (d, d), "bo": (d,), "ln2_g": (d,), "ln2_b": (d,), "w1": (d, f), "b1": (f,), "w2": (f, d), "b2": (d,)}
    views = {}
    for name in BLOCK_FIELDS:
        n = 1
        for e in shapes[name]:
            n *= e
        views[name] = grads[o:o + n].view(*shapes[name])
        o += n
    return views, o


def block_grad_views(cfg, grads):
    """Split the flat fp32 gradient buffer of longer_token_merge_backward into one
    {parameter: tensor view} per InnerTrans block (the order and shapes of the longer_block members)."""
    d = cfg.d // cfg.K if getattr(cfg, "merge", "mean") == "concat" else cfg.d
    out, o = [], 0
    for _ in range(cfg.inner_layers):
        v, o = _block_views(grads, o, d, cfg.ffn_mult * d)
        out.append(v)
    return out


def model_grad_views(cfg, grads):
    """Split the gradient buffer of longer_forward_backward: {"inner": [...], "cross": {...}, "self": [...],
    "head_w": [m d], "head_b": [1] (, "q_learn": [k, d])} of tensor views."""
    di = cfg.d // cfg.K if getattr(cfg, "merge", "mean") == "concat" else cfg.d
    out = {"inner": [], "self": []}
    o = 0
    for _ in range(cfg.inner_layers):
        v, o = _block_views(grads, o, di, cfg.ffn_mult * di)
        out["inner"].append(v)
    out["cross"], o = _block_views(grads, o, cfg.d, cfg.ffn_mult * cfg.d)
    for _ in range(cfg.n_self):
        v, o = _block_views(grads, o, cfg.d, cfg.ffn_mult * cfg.d)
        out["self"].append(v)
    out["head_w"] = grads[o:o + cfg.m * cfg.d]
    out["head_b"] = grads[o + cfg.m * cfg.d:o + cfg.m * cfg.d + 1]
    o = (o + cfg.m * cfg.d + 1 + 3) // 4 * 4
    if getattr(cfg, "q_learnable", False):
        out["q_learn"] = grads[o:o + cfg.k_recent * cfg.d].view(cfg.k_recent, cfg.d)
    return out


def longer_model_grad_floats(ccfg: CConfig) -> int:
    return int(load_library().longer_model_grad_floats(ctypes.byref(ccfg)))


def longer_forward_backward_workspace_bytes(ccfg: CConfig, B: int, L: int) -> int:
    return int(load_library().longer_forward_backward_workspace_bytes(ctypes.byref(ccfg), B, L))


def longer_forward_backward(ccfg, weights, H, G, lens, B, L, labels, loss_out, logits_out, dH_out, dG_out, grads_out, ws,
                            stream=None):
    _require_gpu()
    _check(load_library().longer_forward_backward(ctypes.byref(ccfg), ctypes.byref(weights), _ptr(H), _ptr(G), _ptr(lens), B, L,
                                                  _ptr(labels), _ptr(loss_out), _ptr(logits_out), _ptr(dH_out), _ptr(dG_out),
                                                  _ptr(grads_out), _ptr(ws), ws.numel(), _stream(stream)),
           "longer_forward_backward")


def longer_token_merge_backward(ccfg, inner, H, lens, B, L, dM, dH_out, grads_out, ws, stream=None):
    _require_gpu()
    _check(load_library().longer_token_merge_backward(ctypes.byref(ccfg), inner, _ptr(H), _ptr(lens), B, L, _ptr(dM),
                                                      _ptr(dH_out), _ptr(grads_out), _ptr(ws), ws.numel(), _stream(stream)),
           "longer_token_merge_backward")


def longer_probe_mfma_layout(out, stream=None):
    _require_gpu()
    _check(load_library().longer_probe_mfma_layout(_ptr(out), _stream(stream)), "longer_probe_mfma_layout")


STAGES = ("pack", "merge", "kvproj", "attn", "score")


def longer_stage_timing(enable, stages=None):
    """Switch the per-stage event timers on (all stages, or only the named ones of STAGES) or off."""
    _require_gpu()
    code = 1 if enable else 0
    if enable and stages is not None:
        code = sum(2 << STAGES.index(s) for s in stages)
    _check(load_library().longer_stage_timing(code), "longer_stage_timing")


def longer_stage_timing_read():
    """{stage: (total_ms, launch_groups)} since the last read."""
    ms = (ctypes.c_double * len(STAGES))()
    n = (ctypes.c_int32 * len(STAGES))()
    _check(load_library().longer_stage_timing_read(ms, n), "longer_stage_timing_read")
    return {s: (ms[i], n[i]) for i, s in enumerate(STAGES)}


def longer_input_backward_workspace_bytes(ccfg: CConfig, B: int, L: int, d_e: int) -> int:
    return int(load_library().longer_input_backward_workspace_bytes(ctypes.byref(ccfg), B, L, d_e))


def longer_input_grad_floats(ccfg: CConfig, L: int, d_e: int) -> int:
    return int(load_library().longer_input_grad_floats(ctypes.byref(ccfg), L, d_e))


def input_grad_views(ccfg: CConfig, L: int, d_e: int, flat):
    """Split the gradient buffer of longer_input_generation_backward into {"pos", "w1", "b1", "w2", "b2"}."""
    d, f = ccfg.d, ccfg.ffn_mult * ccfg.d
    out, o = {}, 0
    for name, shape in (("pos", (L, d_e)), ("w1", (d, f)), ("b1", (f,)), ("w2", (f, d)), ("b2", (d,))):
        n = 1
        for v in shape:
            n *= v
        out[name] = flat[o:o + n].reshape(shape)
        o += n
    return out


def longer_input_generation_backward(ccfg, weights, E, tdiff, lens, B, L, d_e, dH, dE_out, dtdiff_out, grads_out, ws, stream=None):
    _require_gpu()
    _check(load_library().longer_input_generation_backward(ctypes.byref(ccfg), ctypes.byref(weights), _ptr(E), _ptr(tdiff),
                                                           _ptr(lens), B, L, d_e, _ptr(dH), _ptr(dE_out), _ptr(dtdiff_out),
                                                           _ptr(grads_out), _ptr(ws), ws.numel(), _stream(stream)),
           "longer_input_generation_backward")
