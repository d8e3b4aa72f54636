"""Are the pins of the backward-pass oracle sharp?  One plausible mistake at a time is planted in a COPY
of oracle/longer_oracle_grad.py (a dropped term, a wrong sign, a transposed operand) and the pins of
tests/test_oracle_grad_pins.py are run against the copy in a scratch folder: at least one has to fail.
CPU only; the real oracle is not touched."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTANTS = [
    ("layer norm backward: the mean of the gradient is not removed",
     "dx = rstd * (dxh - dxh.mean(axis=-1, keepdims=True) - xh * (dxh * xh).mean(axis=-1, keepdims=True))",
     "dx = rstd * (dxh - xh * (dxh * xh).mean(axis=-1, keepdims=True))"),
    ("layer norm backward: gain gradient from the un-normalised rows", "return dx, _sum_lead(dy * xh, 1), _sum_lead(dy, 1)",
     "return dx, _sum_lead(dy * x, 1), _sum_lead(dy, 1)"),
    ("gelu derivative without the density term",
     "return 0.5 * (1.0 + _erf(x / math.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)",
     "return 0.5 * (1.0 + _erf(x / math.sqrt(2.0)))"),
    ("FFN residual's gradient dropped", "    dx = dout + dx2", "    dx = dx2"),
    ("attention residual's gradient dropped", "    return dx + dxq_n, dxkv, g", "    return dxq_n, dxkv, g"),
    ("softmax backward without the row term", "ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True)) / math.sqrt(dh)",
     "ds = p * dp / math.sqrt(dh)"),
    ("softmax backward without the score scale", "ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True)) / math.sqrt(dh)",
     "ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))"),
    ("dK from the probabilities instead of their gradient", "dK[..., sl] = np.swapaxes(ds, -1, -2) @ c[\"q\"][..., sl]",
     "dK[..., sl] = np.swapaxes(p, -1, -2) @ c[\"q\"][..., sl]"),
    ("dV not transposed over the keys", "dV[..., sl] = np.swapaxes(p, -1, -2) @ datt[..., sl]",
     "dV[..., sl] = p[..., :dV.shape[-2], :].sum(axis=-2, keepdims=True).swapaxes(-1, -2) * datt[..., sl].mean(axis=-2, keepdims=True)"),
    ("key side of LN1 forgotten in the gain gradient", "    g[\"ln1_g\"] = gq + gk", "    g[\"ln1_g\"] = gq"),
    ("value path forgotten in the key rows' gradient", "dK @ blk[\"wk\"].T + dV @ blk[\"wv\"].T", "dK @ blk[\"wk\"].T"),
    ("merge: gradient divided by K instead of the valid count", "dM[u][:, None, :] / np.maximum(cnt, 1)[:, None, None]",
     "dM[u][:, None, :] / K"),
    ("merge: padded tokens keep a gradient", "        dE = np.where(valid[:, :, None], dZ, 0.0)", "        dE = dZ + 0.0"),
    ("queries' gradient forgotten when queries and keys are the same rows", "dE = np.where(valid[:, :, None], dxq + dxkv, 0.0)",
     "dE = np.where(valid[:, :, None], dxkv, 0.0)"),
    ("recomputation from the wrong block's input", "                kept[i] = E\n", "                kept[i] = E0\n"),
    ("loss gradient not averaged over the samples", "    return (sig - y) / z.size", "    return sig - y"),
    ("w1 gradient from the un-normalised rows", "g[\"w1\"] = _matT(c[\"u\"], da)", "g[\"w1\"] = _matT(c[\"x\"], da)"),
    ("model: a global token's gradient as a key row forgotten", "        dG[u] = dO[:m] + dR[:m]", "        dG[u] = dO[:m] + 0.0"),
    ("model: the query slots' gradient not returned to the merged tokens", "                dMu[t] += dO[m + i]", "                pass"),
    ("model: self layers, the key rows' gradient forgotten",
     "            dX = dxq + dxkv                                         # queries and keys are the same rows",
     "            dX = dxq"),
    ("model: learnable query tokens, gradient taken from users without any token too",
     "            if v and learn:\n                g_ql[i] += dO[m + i]", "            if learn:\n                g_ql[i] += dO[m + i] + 1.0 * (not v)"),
    ("input generation: the positional embedding's gradient not summed over the users",
     "        g[\"pos\"][:n] += dx[:, :d_e]", "        g[\"pos\"][:n] = dx[:, :d_e]"),
    ("input generation: the activation's derivative at the activated value",
     "        da = (dy @ w2.T) * activation_grad(a, cfg.act)", "        da = (dy @ w2.T) * activation_grad(hdn, cfg.act)"),
    ("model: head weights read feature-major", "        dX[:m] = dlogit[u] * head_w.reshape(m, d)",
     "        dX[:m] = dlogit[u] * head_w.reshape(d, m).T"),
]


def _scratch(tmp_path, old, new):
    src = open(os.path.join(ROOT, "oracle", "longer_oracle_grad.py")).read()
    assert src.count(old) >= 1, "mutation target not found: " + old
    src = src.replace(old, new)
    os.makedirs(tmp_path / "oracle")
    (tmp_path / "oracle" / "__init__.py").write_text("")
    (tmp_path / "oracle" / "longer_oracle_grad.py").write_text(src)
    shutil.copy(os.path.join(ROOT, "oracle", "longer_oracle.py"), tmp_path / "oracle" / "longer_oracle.py")
    shutil.copytree(os.path.join(ROOT, "longer_synth"), tmp_path / "longer_synth", ignore=shutil.ignore_patterns("__pycache__"))
    os.makedirs(tmp_path / "tests")
    for f in ("conftest.py", "test_oracle_grad_pins.py"):
        shutil.copy(os.path.join(ROOT, "tests", f), tmp_path / "tests" / f)


def _run_pins(tmp_path):
    env = dict(os.environ, PYTHONPATH=str(tmp_path), PYTHONDONTWRITEBYTECODE="1")
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_oracle_grad_pins.py"],
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
