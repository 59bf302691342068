"""Pins for the oracle's gradients of the sequence mixer: central differences of S = sum <dy, mixer(...)> through
the forward oracle (the C implementation of the mixer), which is exact up to rounding for every argument in which
the mixer is linear and second-order accurate otherwise."""
import numpy as np
import pytest

import oracle
from oracle import layer
from paper_2310_12109_amd import workloads

KEYS = ("u", "K", "g_in", "g_out", "R1", "L1", "R2", "L2")


def _S(w, dy):
    return float(np.sum(dy * oracle.mixer(*(w[k] for k in KEYS))))


@pytest.mark.parametrize("b,gates", [(2, (True, True)), (3, (True, True)), (4, (False, False)), (4, (True, False)), (4, (False, True))])
def test_every_gradient_by_central_differences(b, gates):
    rng = np.random.default_rng(b)
    w = {k: (None if v is None else v.astype(np.float64)) for k, v in workloads.mixer_inputs(2, 3, b, seed=b, gates=gates).items()}
    dy = rng.standard_normal(w["u"].shape)
    g = layer.mixer_backward(*(w[k] for k in KEYS), dy)
    h = 1e-5
    for key, name in (("u", "du"), ("K", "dK"), ("g_in", "dg_in"), ("g_out", "dg_out"), ("R1", "dR1"), ("L1", "dL1"),
                      ("R2", "dR2"), ("L2", "dL2")):
        if w[key] is None:
            assert g[name] is None
            continue
        got = g[name]
        assert got.shape == w[key].shape
        for _ in range(10):
            idx = tuple(rng.integers(0, s) for s in w[key].shape)
            keep = w[key][idx]
            w[key][idx] = keep + h; up = _S(w, dy)
            w[key][idx] = keep - h; dn = _S(w, dy)
            w[key][idx] = keep
            assert abs((up - dn) / (2 * h) - got[idx]) < 1e-6 * max(1.0, abs(got[idx])), (name, idx)


def test_adjoint_identity_in_u():
    # the mixer is linear in u: <du, u> = <dy, y>
    w = {k: v.astype(np.float64) for k, v in workloads.mixer_inputs(3, 4, 4, seed=1).items()}
    dy = np.random.default_rng(2).standard_normal(w["u"].shape)
    g = layer.mixer_backward(*(w[k] for k in KEYS), dy)
    assert abs(np.sum(g["du"] * w["u"]) - _S(w, dy)) < 1e-9
    # and in K, in each gate and in each factor: <dX, X> = S as well (degree one in every argument)
    for key, name in (("K", "dK"), ("g_in", "dg_in"), ("g_out", "dg_out"), ("R1", "dR1"), ("L2", "dL2")):
        assert abs(np.sum(g[name] * w[key]) - _S(w, dy)) < 1e-9
