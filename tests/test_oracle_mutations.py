"""Are the oracle's pins sharp?  Each case plants one plausible mistake in a COPY of the oracle's
source (a dropped term, a wrong sign or index, a transposed operand, a wrong constant) and runs the
pin tests against that copy in a scratch folder: at least one pin has to fail.  Everything happens
on the CPU; the real oracle and the HIP path are not touched."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTANTS = [
    ("layer norm: unbiased variance",
     "var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)",
     "var = ((x - mu) ** 2).sum(axis=-1, keepdims=True) / (x.shape[-1] - 1)"),
    ("layer norm: eps dropped", "np.sqrt(var + eps)", "np.sqrt(var)"),
    ("layer norm: shift dropped", "/ np.sqrt(var + eps) * g + b", "/ np.sqrt(var + eps) * g"),
    ("gelu: wrong erf argument", "_erf(x / math.sqrt(2.0))", "_erf(x / 2.0)"),
    ("attention: scale by the model width instead of the head width", "/ math.sqrt(dh)", "/ math.sqrt(d)"),
    ("attention: output bias dropped", 'x = xq + att @ blk["wo"] + blk["bo"]', 'x = xq + att @ blk["wo"]'),
    ("attention: residual dropped", 'x = xq + att @ blk["wo"] + blk["bo"]', 'x = att @ blk["wo"] + blk["bo"]'),
    ("ffn: residual dropped", 'return x + hdn @ blk["w2"] + blk["b2"]', 'return hdn @ blk["w2"] + blk["b2"]'),
    ("ffn: second norm skipped", 'activation(layer_norm(x, blk["ln2_g"], blk["ln2_b"], eps) @ blk["w1"]',
     'activation(x @ blk["w1"]'),
    ("K and V weights swapped", 'return xn @ blk["wk"] + blk["bk"], xn @ blk["wv"] + blk["bv"]',
     'return xn @ blk["wv"] + blk["bk"], xn @ blk["wk"] + blk["bv"]'),
    ("keys not normalised", 'xn = layer_norm(x, blk["ln1_g"], blk["ln1_b"], eps)\n    return xn @ blk["wk"]',
     'xn = x\n    return xn @ blk["wk"]'),
    ("mask: a sequence token does not see itself (both forms of the rule)",
     ["return (not k_is_global) and k_idx <= q_idx", "seq_q = (~kg) & (ki <= qi)"],
     ["return (not k_is_global) and k_idx < q_idx", "seq_q = (~kg) & (ki < qi)"]),
    ("mask: sequence tokens see the global tokens (both forms of the rule)",
     ["return (not k_is_global) and k_idx <= q_idx", "seq_q = (~kg) & (ki <= qi)"],
     ["return k_is_global or k_idx <= q_idx", "seq_q = kg | (ki <= qi)"]),
    ("mask: padded keys are visible", "return np.where(qg, glob_q, seq_q) & qv & kv", "return np.where(qg, glob_q, seq_q) & qv"),
    ("merge: mean over K instead of over the valid tokens", "M[u, nz] = Z[u, nz].sum(axis=1) / cnt[nz, None]",
     "M[u, nz] = Z[u, nz].sum(axis=1) / K"),
    ("merge: concatenation in the wrong order", "return Z.reshape(B, T, K * d)",
     "return Z.transpose(0, 1, 3, 2).reshape(B, T, K * d)"),
    ("inner transformer: padded tokens take part", "mask = valid[:, :, None] & valid[:, None, :]",
     "mask = np.ones_like(valid[:, :, None] & valid[:, None, :])"),
    ("recent slots shifted by one", "    if Tu <= k or i >= k_uniform:\n        return Tu - k + i",
     "    if Tu <= k or i >= k_uniform:\n        return Tu - k + i - 1"),
    ("uniform slots: oldest instead of newest token of a share", "return ((i + 1) * rest) // k_uniform - 1",
     "return (i * rest) // k_uniform"),
    ("learnable slots all at one position", "toks.append((False, Tu + i, Tu > 0))", "toks.append((False, Tu, Tu > 0))"),
    ("learnable slots miss the newest token", "toks.append((False, Tu + i, Tu > 0))", "toks.append((False, Tu - 2 + i, Tu > 0))"),
    ("head: bias dropped", 'return flat @ np.asarray(head_w, dtype=F64) + float(np.asarray(head_b).reshape(-1)[0])',
     'return flat @ np.asarray(head_w, dtype=F64)'),
    ("input generation: positional embedding dropped", "np.asarray(E[u, :n], dtype=F64) + pos[:n]", "np.asarray(E[u, :n], dtype=F64)"),
    ("input generation: output bias dropped", 'H[u, :n] = activation(x @ w1 + b1, cfg.act) @ w2 + b2',
     'H[u, :n] = activation(x @ w1 + b1, cfg.act) @ w2'),
    ("serving: the cached keys of a self layer come from the previous layer's input",
     "Kc, Vc = project_kv(Xs, blocks[l], cfg.ln_eps)\n            cache", "Kc, Vc = project_kv(Xs * 0 + Mu[:1], blocks[l], cfg.ln_eps)\n            cache"),
    ("flops: attention pairs counted once instead of twice", "4 * di * pairs", "2 * di * pairs"),
    ("scoring: global-global rule transposed", "visible(True, a, True, b, cfg.gmask)", "visible(True, b, True, a, cfg.gmask)"),
    ("scoring: invalid cached slots are visible", 'np.broadcast_to(cache["valid"][l][u], (m, len(cache["valid"][l][u])))',
     'np.ones((m, len(cache["valid"][l][u])), dtype=bool)'),
    ("padded merged tokens are valid keys", "[(False, t, t < Tu) for t in range(T)]", "[(False, t, True) for t in range(T)]"),
    ("merged length rounds down", "return (int(length) + K - 1) // K", "return int(length) // K"),
    ("query slot gathers the token before its own", "else M_u[t]", "else M_u[max(t - 1, 0)]"),
    ("causal global mask in the other direction (both forms of the rule)",
     ['return True if gmask == "full" else k_idx >= q_idx', 'True if gmask == "full" else (ki >= qi)'],
     ['return True if gmask == "full" else k_idx <= q_idx', 'True if gmask == "full" else (ki <= qi)']),
    ("softmax without the running maximum's guard for empty rows", "return np.where(den > 0, e / np.where(den > 0, den, 1.0), 0.0)",
     "return e / den"),
]


def _scratch(tmp_path, old, new):
    src = open(os.path.join(ROOT, "oracle", "longer_oracle.py")).read()
    olds, news = (old, new) if isinstance(old, list) else ([old], [new])
    for o, n in zip(olds, news):
        assert src.count(o) >= 1, "mutation target not found: " + o
        src = src.replace(o, n)
    os.makedirs(tmp_path / "oracle")
    (tmp_path / "oracle" / "__init__.py").write_text("")
    (tmp_path / "oracle" / "longer_oracle.py").write_text(src)
    shutil.copytree(os.path.join(ROOT, "longer_synth"), tmp_path / "longer_synth", ignore=shutil.ignore_patterns("__pycache__"))
    os.makedirs(tmp_path / "tests")
    for f in ("conftest.py", "test_oracle_pins.py"):
        shutil.copy(os.path.join(ROOT, "tests", f), tmp_path / "tests" / f)
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), tmp_path / "tests" / "golden")


def _run_pins(tmp_path):
    env = dict(os.environ, PYTHONPATH=str(tmp_path), PYTHONDONTWRITEBYTECODE="1")
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_oracle_pins.py"],
                          cwd=str(tmp_path), env=env, capture_output=True, text=True, timeout=600)


def test_the_unmodified_copy_passes(tmp_path):
    _scratch(tmp_path, "import math", "import math")
    r = _run_pins(tmp_path)
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(tmp_path, what, old, new):
    _scratch(tmp_path, old, new)
    r = _run_pins(tmp_path)
    assert r.returncode != 0, "no pin noticed: " + what
    assert " failed" in r.stdout or "Error" in r.stdout, r.stdout[-2000:]
