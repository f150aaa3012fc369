"""The GELU kernels evaluate the normal CDF as 2^q(|z|) with a degree-10 polynomial whose coefficients are literals in
csrc/bias_act_dropout.hip.  This test reads those literals from the source and evaluates the same fp32 Horner chain
with numpy against scipy's erfc: a mistyped coefficient, a lost term or a wrong constant term shows here, without a GPU."""
import os
import re

import numpy as np
from scipy.special import erfc, ndtr

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2110_05722_amd", "csrc",
                   "bias_act_dropout.hip")


def _coefficients():
    text = open(SRC).read()
    body = text[text.index("float normal_cdf(float z)"):]
    body = body[:body.index("return z < 0.0f")]
    lead = re.search(r"float q = (-?[0-9.e+-]+)f;", body)
    rest = re.findall(r"q = fmaf\(q, u, (-?[0-9.e+-]+)f( - 1\.0f)?\);", body)
    coef = [np.float32(lead.group(1))] + [np.float32(np.float32(c) - np.float32(1.0)) if minus else np.float32(c) for c, minus in rest]
    clamp = np.float32(re.search(r"fminf\(fabsf\(z\), ([0-9.]+)f\)", body).group(1))
    return coef, clamp


def _normal_cdf_f32(z, coef, clamp):
    z = z.astype(np.float32)
    u = np.minimum(np.abs(z), clamp)
    q = np.full_like(u, coef[0])
    for c in coef[1:]:
        q = (q * u).astype(np.float32) + c          # an fma keeps the product unrounded: the difference is below the bound tested
        q = q.astype(np.float32)
    tail = np.exp2(q.astype(np.float64))
    return np.where(z < 0, tail, 1.0 - tail)


def test_source_polynomial_is_the_normal_cdf():
    coef, clamp = _coefficients()
    assert len(coef) == 11 and clamp == np.float32(6.5)
    z = np.linspace(-6.5, 6.5, 200001)
    got = _normal_cdf_f32(z, coef, clamp)
    ref = ndtr(z.astype(np.float32).astype(np.float64))
    # the lower tail keeps RELATIVE accuracy (it is what multiplies a large negative z in GELU), the upper one absolute
    lower = z < 0
    assert np.max(np.abs(got[lower] / ref[lower] - 1.0)) < 2e-5
    assert np.max(np.abs(got[~lower] - ref[~lower])) < 2e-6
    # the constant term carries the factor 1/2: Phi(0) = 1/2 from both sides
    assert abs(_normal_cdf_f32(np.array([0.0]), coef, clamp)[0] - 0.5) < 1e-6
    assert abs(_normal_cdf_f32(np.array([-0.0]), coef, clamp)[0] - 0.5) < 1e-6
    # beyond the clamp the tail is held: tiny, positive, and 2 Phi(-6.5) = erfc(6.5 / sqrt 2)
    far = _normal_cdf_f32(np.array([-9.0, 9.0]), coef, clamp)
    assert 0 < far[0] < 1e-10 and far[1] == 1.0 - far[0]
    assert abs(2 * far[0] / erfc(6.5 / np.sqrt(2.0)) - 1.0) < 2e-5
