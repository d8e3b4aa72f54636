"""The HIP path and the oracle share no code, and the benchmark refuses more than one GPU.
No GPU needed."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _sources(folder, exts):
    out = []
    for base, _, files in os.walk(os.path.join(ROOT, folder)):
        if "__pycache__" in base:
            continue
        out += [os.path.join(base, f) for f in files if f.endswith(exts)]
    return out


def test_product_path_never_touches_the_oracle():
    files = _sources("paper_2505_04421_amd", (".py", ".h", ".hip")) + _sources("include", (".h",))
    assert files
    for path in files:
        text = open(path).read()
        assert not re.search(r"\boracle\b", text), path + " mentions the oracle"


def test_oracle_is_independent_of_the_hip_path():
    files = _sources("oracle", (".py", ".c", ".h"))
    assert files
    for path in files:
        text = open(path).read()
        assert "paper_2505_04421_amd" not in text and "liblonger" not in text and "ctypes" not in text, path


def test_input_generator_holds_no_model_arithmetic():
    text = open(os.path.join(ROOT, "longer_synth", "__init__.py")).read()
    for word in ("softmax", "layer_norm", "erf(", "import torch", "paper_2505_04421_amd", "from oracle"):
        assert word not in text, word


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_benchmark_touches_the_oracle_only_in_its_cpu_baseline_leg():
    text = open(os.path.join(ROOT, "bench.py")).read()
    imports = [m.start() for m in re.finditer(r"from oracle import|import oracle", text)]
    assert len(imports) == 1
    leg = text.index("def cpu_oracle_leg(")
    nxt = text.index("\ndef ", leg + 1)
    assert leg < imports[0] < nxt
    assert "orc." not in text[:leg] and "orc." not in text[nxt:]
