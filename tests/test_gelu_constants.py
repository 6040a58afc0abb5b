"""The fp32 / fp64 GELU approximation of the HIP feature maps (Sec. 3.2 names GELU as the
activation of Eq. 1 and Eq. 2): the constants typed into csrc/lessdec_common.h are the ones
csrc/fit_gelu_poly.py derives, and evaluated as the kernels evaluate them they stay within the
error the header states, against the definition x Phi(x) computed with scipy's erfc."""
import importlib.util
import re
from pathlib import Path

import numpy as np
from scipy.special import erfc

CSRC = Path(__file__).resolve().parents[1] / "paper_2402_09398_amd" / "csrc"


def _fit_module():
    spec = importlib.util.spec_from_file_location("fit_gelu_poly", CSRC / "fit_gelu_poly.py")
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _header_constants(func):
    """c7 .. c1 (Horner order) and p as written in `func` of lessdec_common.h."""
    src = (CSRC / "lessdec_common.h").read_text()
    body = src[src.index(func):]
    body = body[:body.index("\n}\n")]
    p = float(re.search(r"fma[f]?\((0\.\d+)f?, t, 1\.0f?\)", body).group(1))
    first = float(re.search(r"a = (-?\d\.\d+e[-+]\d+)f?;", body).group(1))
    rest = [float(x) for x in re.findall(r"a = fma[f]?\(a, u, (-?\d\.\d+e[-+]\d+)f?\);", body)]
    return p, [first] + rest


def test_header_constants_are_the_fitted_ones():
    fit = _fit_module()
    c = fit.fit()                                   # c1 .. c7
    for func in ("gelu_fast_f32", "gelu_poly_f64"):
        p, horner = _header_constants(func)
        assert p == fit.P and len(horner) == fit.N
        np.testing.assert_allclose(horner[::-1], c, rtol=2e-6, atol=0)


def test_fp32_evaluation_error():
    fit = _fit_module()
    p, horner = _header_constants("gelu_fast_f32")
    x = np.linspace(-12, 12, 400001)
    exact = 0.5 * x * erfc(-x / np.sqrt(2))
    got = fit.gelu32(x, p, np.array(horner[::-1])).astype(np.float64)
    err = np.abs(got - exact)
    assert err[np.abs(x) <= 4].max() < 3e-7
    assert (err[np.abs(x) > 4] <= 1.2e-7 * np.abs(x[np.abs(x) > 4]) + 3e-7).all()


def test_fp64_evaluation_error():
    p, horner = _header_constants("gelu_poly_f64")
    x = np.linspace(-12, 12, 400001)
    t = np.abs(x)
    u = 1.0 / (1.0 + p * t)
    a = np.full_like(u, horner[0])
    for c in horner[1:]:
        a = a * u + c
    a = a * u
    tq = t * (a * np.exp(-0.5 * t * t))
    got = np.where(x >= 0, x - tq, -tq)
    assert np.abs(got - 0.5 * x * erfc(-x / np.sqrt(2))).max() < 2e-9
