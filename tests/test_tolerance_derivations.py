"""Bounds that the GPU kernels' documented approximations rest on, recomputed from the constants in the sources."""
import os
import re

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def source_constant(path, name):
    text = open(os.path.join(ROOT, path)).read()
    m = re.search(r"constexpr\s+float\s+%s\s*=\s*([0-9.eE+-]+)f?\s*;" % name, text)
    assert m, "%s not found in %s" % (name, path)
    return float(m.group(1))


def test_softcap_polynomial_stays_under_the_rounding_of_the_probabilities():
    """The 16-bit attention kernel takes cap*tanh(z) as cap*(z - z^3/3 + 2 z^5/15) while |z| <= CAP_POLY_Z.
    The logit error at the largest cap of the workloads (50) must stay well below 2^-9, the relative rounding
    step of a bf16 probability, and the alternating-series bound 17 z^7 / 315 must hold."""
    z0 = source_constant("paper_2604_03260_amd/csrc/focus_attn_mfma.hip", "CAP_POLY_Z")
    z = np.linspace(-z0, z0, 200001)
    poly = z - z ** 3 / 3.0 + 2.0 * z ** 5 / 15.0
    err = np.abs(np.tanh(z) - poly).max()
    assert err <= 17.0 * z0 ** 7 / 315.0 * (1.0 + 1e-9)
    assert 50.0 * err <= 2.0 ** -9 / 3.0                     # logit error (natural units) at cap = 50


def test_softcap_cubic_stays_under_the_same_bound():
    """Below CAP_CUBIC_Z some instantiations drop the z^5 term: cap*tanh(z) as cap*(z - z^3/3).  The error is below
    the next term of the alternating series, 2 z^5 / 15, and at cap 50 no larger than what the z^5 form is allowed."""
    z3 = source_constant("paper_2604_03260_amd/csrc/focus_attn_mfma.hip", "CAP_CUBIC_Z")
    z5 = source_constant("paper_2604_03260_amd/csrc/focus_attn_mfma.hip", "CAP_POLY_Z")
    assert 0.0 < z3 < z5
    z = np.linspace(-z3, z3, 200001)
    err = np.abs(np.tanh(z) - (z - z ** 3 / 3.0)).max()
    assert err <= 2.0 * z3 ** 5 / 15.0 * (1.0 + 1e-9)
    assert 50.0 * err <= 2.0 ** -9 / 3.0                     # logit error (natural units) at cap = 50
    assert err <= 17.0 * z5 ** 7 / 315.0                     # no worse than the z^5 form at the end of its range


def test_lazy_softmax_reference_keeps_probabilities_in_range():
    """Probabilities are taken against a reference that may lag the true maximum by RESCALE_THRESHOLD (log2
    units): they reach 2^threshold at most, far inside bf16 and fp16 range, and their fp32 row sum cannot
    overflow for any sequence length the library takes (2^24 keys)."""
    for path, name in (("paper_2604_03260_amd/csrc/focus_attn_mfma.hip", "RESCALE_THRESHOLD"),
                       ("paper_2604_03260_amd/csrc/focus_decode.hip", "DEC_RESCALE_THRESHOLD")):
        thr = source_constant(path, name)
        assert 2.0 ** thr <= 65504.0 / 64.0                  # fp16 holds it with room to spare
        assert 2.0 ** thr * 2.0 ** 24 < np.finfo(np.float32).max
