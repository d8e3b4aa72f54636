"""The bf16-mode GELU of the HIP path (a clamped odd polynomial evaluated in packed fp16 on x / 4),
emulated step by step with numpy's float16 and compared with the erf form.  Checks its error
(max abs below 8e-3, N(0,1)-weighted rms below 1.2e-3, exact saturation far outside the fitted
interval) and that the kernel's fp16 coefficients are the fp32 polynomial's, rescaled.  No GPU needed."""
import os
import re

import numpy as np
from scipy.special import erf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
KERNEL = os.path.join(ROOT, "paper_2505_04421_amd", "csrc", "block_kernel.h")


def _coefficients():
    text = open(KERNEL).read()
    body = text[text.index("f16x8 gelu_quarter_h8"):]
    body = body[:body.index("return y * phi;")]
    k16 = [float(x) for x in re.findall(r"\(_Float16\)(-?[0-9.eE+-]+)f\)", body)][:5]      # k4, k3, k2, k1, k0
    body32 = text[text.index("float gelu_fn(float x)"):]
    body32 = body32[body32.index("const float u = x * x;"):body32.index("return x * phi;")]
    c32 = [float(x) for x in re.findall(r"(-?[0-9]\.[0-9]+(?:e-?[0-9]+)?)f", body32)][:5]   # c4 .. c0
    return k16, c32


def _fma16(a, b, c):
    return (a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)).astype(np.float16)


def _emulate(x, k):
    h = np.float16
    y = (x / 4.0).astype(np.float32)
    y16 = y.astype(h)
    toward_zero = np.abs(y16.astype(np.float32)) > np.abs(y)          # the kernel converts toward zero
    y16 = np.where(toward_zero, np.nextafter(y16, h(0)), y16).astype(h)
    v = (y16.astype(np.float64) ** 2).astype(h)
    pl = np.full_like(v, h(k[0]))
    for ki in k[1:]:
        pl = _fma16(pl, v, np.full_like(v, h(ki)))
    phi = np.clip(_fma16(y16, pl, np.full_like(v, h(0.5))).astype(np.float64), 0.0, 1.0).astype(h)
    return (y16.astype(np.float64) * phi.astype(np.float64)).astype(h).astype(np.float64) * 4.0


def test_fp16_coefficients_are_the_fp32_polynomial_rescaled():
    k16, c32 = _coefficients()
    assert len(k16) == 5 and len(c32) == 5
    for i, (k, c) in enumerate(zip(k16, c32)):
        power = 4 - i                                   # coefficient of u^power, u = x^2 = 16 v
        assert abs(k - 4.0 * 16.0 ** power * c) <= 1e-12 * abs(k)
        assert 0.5 < abs(k) < 8.0                       # of order 1: no fp16 subnormal among them


def test_fp16_gelu_error_against_the_erf_form():
    k16, _ = _coefficients()
    x = np.linspace(-8.0, 8.0, 200001)
    ref = 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))
    err = np.abs(_emulate(x, k16) - ref)
    assert err.max() < 8e-3
    w = np.exp(-x * x / 2.0)
    assert np.sqrt((err ** 2 * w).sum() / w.sum()) < 1.2e-3
    # saturation: far outside the fitted interval the clamp gives x and 0 up to the conversion's last
    # place, also where the square overflows fp16
    big = np.array([50.0, 300.0, 2000.0, 1e5])
    with np.errstate(over="ignore", invalid="ignore"):
        assert np.all(np.abs(_emulate(big, k16) - big) <= big * 2.0 ** -10)
        assert np.all(_emulate(-big, k16) == 0.0)
