"""Helpers for the GPU parity tests: run the C-ABI entry points (through the Python
binding) on a seeded case and bring the results back as numpy arrays."""
import weakref

import numpy as np
import torch

import paper_2505_04421_amd as lg


GUARD = 4096          # bytes of sentinel on each side of every buffer the library writes
SENTINEL = 0xA5


class Guarded:
    """A device buffer between two sentinel-filled guard bands: a store that strays past either end
    of an output, the workspace or the cache shows up in check().  The body starts out filled with
    the sentinel too, so elements the library should have written and did not are not zeros by
    accident."""

    def __init__(self, device, nbytes):
        self.n = int(nbytes)
        self.raw = torch.full((self.n + 2 * GUARD,), SENTINEL, dtype=torch.uint8, device=device)
        self.body = self.raw[GUARD:GUARD + self.n]

    def tensor(self, dtype, shape):
        return self.body.view(dtype).view(*shape)

    def check(self, what=""):
        lo, hi = self.raw[:GUARD], self.raw[GUARD + self.n:]
        assert bool((lo == SENTINEL).all()) and bool((hi == SENTINEL).all()), "guard band overwritten: " + what


def guarded_empty(device, shape, dtype):
    """(tensor, guard) of the given shape inside a guarded buffer."""
    n = int(np.prod(shape)) * torch.empty(0, dtype=dtype).element_size()
    g = Guarded(device, n)
    return g.tensor(dtype, shape), g


class GuardedModel(lg.DeviceModel):
    """DeviceModel whose outputs, workspace and cache sit between guard bands; check_all_guards()
    (run by every comparison of the parity tests) looks at the bands of every live model."""
    LIVE = weakref.WeakSet()

    def __init__(self, *a, **kw):
        super().__init__(*a, **kw)
        self.guards = []
        GuardedModel.LIVE.add(self)

    def _guarded(self, shape, dtype):
        t, g = guarded_empty(self.device, shape, dtype)
        self.guards.append(g)
        return t

    def empty(self, *shape, dtype=None):
        return self._guarded(shape, dtype or self.tdtype)

    def workspace(self, B, L, C=0):
        n = lg.longer_workspace_bytes(self.ccfg, B, L)
        assert n > 0, lg.longer_last_error()
        return self._guarded((n,), torch.uint8)

    def kv_cache(self, U, L):
        n = lg.longer_kv_cache_bytes(self.ccfg, U, L)
        assert n > 0, lg.longer_last_error()
        return self._guarded((n,), torch.uint8)


def check_all_guards():
    torch.cuda.synchronize()
    for model in list(GuardedModel.LIVE):
        for g in model.guards:
            g.check("a buffer of a GuardedModel")


class Runner:
    def __init__(self, case, packed=False):
        self.case = case
        self.cfg = case["cfg"]
        self.model = lg.DeviceModel(self.cfg, case["weights"])
        self.B, self.L = self.cfg.B, self.cfg.L
        self.guards = []
        n_ws = lg.longer_workspace_bytes(self.model.ccfg, self.B, self.L)
        assert n_ws > 0, lg.longer_last_error()
        self.ws = self._guarded((n_ws,), torch.uint8, "workspace")
        self.lens = None
        if case["lens"] is not None:
            self.lens = torch.from_numpy(case["lens"].astype(np.int32)).to(self.model.device)
        # packed=True: the calls that take the whole model stream from a buffer packed once
        self.weights = self.model.pack() if packed else self.model.weights

    def _guarded(self, shape, dtype, what):
        t, g = guarded_empty(self.model.device, shape, dtype)
        self.guards.append((what, g))
        return t

    def empty(self, *shape, dtype=None, what="output"):
        return self._guarded(shape, dtype or self.model.tdtype, what)

    def up(self, a):
        return self.model.upload(a)

    def host(self, t):
        torch.cuda.synchronize()
        for what, g in self.guards:
            g.check(what)
        return t.float().cpu().numpy().astype(np.float64)

    def token_merge(self, H=None):
        c, m = self.cfg, self.model
        H = self.up(self.case["H"] if H is None else H)
        out = self.empty(self.B, c.T, c.d, what="M_out")
        lg.longer_token_merge(m.ccfg, m.inner, H, self.lens, self.B, self.L, out, self.ws)
        return self.host(out)

    def inner_transformer(self):
        c, m = self.cfg, self.model
        H = self.up(self.case["H"])
        out = self.empty(self.B, c.T, c.K, c.d_in, what="Z_out")
        lg.longer_inner_transformer(m.ccfg, m.inner, H, self.lens, self.B, self.L, out, self.ws)
        return self.host(out)

    def cross(self, G, M):
        c, m = self.cfg, self.model
        out = self.empty(self.B, c.n, c.d, what="X_out (cross)")
        lg.longer_hybrid_cross_attn(m.ccfg, m.cross, self.up(G), self.up(M), self.lens, self.B, self.L, out, self.ws)
        return self.host(out)

    def self_layer(self, X, i=0):
        c, m = self.cfg, self.model
        out = self.empty(self.B, c.n, c.d, what="X_out (self)")
        blk = (type(m.self_[0]) * 1)(m.self_[i])
        lg.longer_self_attn_layer(m.ccfg, blk, self.up(X), self.lens, self.B, self.L, out, self.ws)
        return self.host(out)

    def forward(self, H=None, G=None):
        c, m = self.cfg, self.model
        H = self.up(self.case["H"] if H is None else H)
        G = self.up(self.case["G"] if G is None else G)
        Y = self.empty(self.B, c.n, c.d, what="Y_out")
        logits = self.empty(self.B, dtype=torch.float32, what="logits_out")
        lg.longer_forward(m.ccfg, self.weights, H, G, self.lens, self.B, self.L, Y, logits, self.ws)
        return self.host(Y), self.host(logits)

    def serve(self, want_hidden=True):
        c, m = self.cfg, self.model
        H = self.up(self.case["H"])
        Gc = self.up(self.case["G_cand"])
        n_cache = lg.longer_kv_cache_bytes(m.ccfg, self.B, self.L)
        assert n_cache > 0, lg.longer_last_error()
        cache = self._guarded((n_cache,), torch.uint8, "kv cache")
        lg.longer_kv_cache_build(m.ccfg, self.weights, H, self.lens, self.B, self.L, cache, self.ws)
        Yg = self.empty(self.B, c.C, c.m, c.d, what="Yg_out") if want_hidden else None
        logits = self.empty(self.B, c.C, dtype=torch.float32, what="logits_out (scoring)")
        lg.longer_score_candidates(m.ccfg, self.weights, cache, self.lens, self.B, self.L, Gc, c.C, Yg, logits, self.ws)
        return (self.host(Yg) if want_hidden else None), self.host(logits)


def rel_l2_per_user(got, ref):
    """max over the leading (user) axis of ||got - ref|| / ||ref||."""
    got = got.reshape(got.shape[0], -1)
    ref = ref.reshape(ref.shape[0], -1)
    num = np.linalg.norm(got - ref, axis=1)
    den = np.linalg.norm(ref, axis=1)
    den = np.where(den > 0, den, 1.0)
    return float((num / den).max())


def rel_l2_per_row(got, ref):
    """max over the rows (last axis = features) that the reference marks valid (non-zero) of
    ||got - ref|| / ||ref||: one bad row cannot hide among a user's many good ones."""
    got = got.reshape(-1, got.shape[-1])
    ref = ref.reshape(-1, ref.shape[-1])
    den = np.linalg.norm(ref, axis=1)
    ok = den > 0
    if not ok.any():
        return 0.0
    num = np.linalg.norm(got - ref, axis=1)
    return float((num[ok] / den[ok]).max())


def assert_zero_where_ref_zero_rows(got, ref):
    """Rows that the oracle reports as invalid (all-zero) must be exact zeros."""
    zr = (ref == 0).all(axis=-1)
    assert (got[zr] == 0).all()
