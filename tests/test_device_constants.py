"""Constants of the device code checked on the host (no GPU needed)."""
import math
import os
import re

import numpy as np


def test_device_gelu_polynomial_against_erf():
    # the bf16 kernels evaluate gelu(u) = max(u, 0) - a * 2^P(a), a = min(|u|, 6): take the
    # coefficients of P out of the device header and run the same fp32 arithmetic here against
    # the erf definition (section 2.1: the MLP's activation)
    hdr = open(os.path.join(os.path.dirname(__file__), "..", "paper_2110_14895_amd", "csrc", "ep_device.h")).read()
    body = re.search(r"#define EP_GELU_LOG2Q_COEFFS(.*?)\}", hdr, re.S).group(1)
    c = [np.float32(x.rstrip("f")) for x in re.findall(r"-?\d+\.\d+(?:e-?\d+)?f", body)]
    assert len(c) == 5
    u = np.concatenate([np.linspace(-12, 12, 480001), [0.0, -0.0, 1e-30, -1e-30, 50.0, -50.0]]).astype(np.float32)
    a = np.minimum(np.abs(u), np.float32(6.0))
    p = c[4] * a + c[3]
    for k in (2, 1, 0):
        p = (p * a + c[k]).astype(np.float32)
    got = (np.maximum(u, np.float32(0)) - np.exp2(p).astype(np.float32) * a).astype(np.float32)
    ref = np.array([0.5 * x * (1.0 + math.erf(x / math.sqrt(2.0))) for x in u.astype(np.float64)])
    err = np.abs(got.astype(np.float64) - ref)
    # the output format is bf16 (relative steps of 2^-8): the fit stays an order of magnitude
    # below it, 6.5e-6 absolute everywhere and 3.5e-4 relative on the positive side
    assert err.max() <= 6.5e-6, err.max()
    pos = u > 0
    assert np.all(err[pos] <= 3.5e-4 * ref[pos] + 1e-37), (err[pos] / np.maximum(ref[pos], 1e-300)).max()
    # far from the origin the correction term vanishes: identity on the right, zero on the left
    assert np.all(got[u >= 9] == u[u >= 9]) and np.all(np.abs(got[u <= -9]) < 1e-8)
