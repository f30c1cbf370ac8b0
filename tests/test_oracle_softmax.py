"""Pins for step 1 of the oracle (softmax of the target logits): an independent library
routine, closed forms, and exact widening of bf16."""
import numpy as np
from scipy.special import logsumexp, softmax

from oracle import oracle as O


def test_against_scipy_on_random_rows():
    rng = np.random.default_rng(1)
    for V, scale, tau in [(7, 1.0, 1.0), (1000, 3.0, 1.0), (4099, 8.0, 0.7), (32000, 2.0, 1.9)]:
        z = (rng.standard_normal(V) * scale).astype(np.float32)
        P, m, Z = O.softmax_row(z, O.F32, tau)
        y = z.astype(np.float64) * tau
        np.testing.assert_allclose(P, softmax(y), rtol=1e-12, atol=0)
        assert m == y.max()
        np.testing.assert_allclose(m + np.log(Z), logsumexp(y), rtol=1e-13)
        assert abs(P.sum() - 1.0) < 1e-12


def test_closed_forms():
    V = 64
    P, m, Z = O.softmax_row(np.full(V, 3.25, np.float32))
    assert m == 3.25 and Z == V and (P == 1.0 / V).all()
    # two distinct values: a logit of ln(3)-ish is not exact, use exact halves via exp(0)=1
    z = np.zeros(5, np.float32)
    z[2] = -np.inf
    P, m, Z = O.softmax_row(z)
    assert Z == 4.0 and P[2] == 0.0 and (P[[0, 1, 3, 4]] == 0.25).all()
    # shift invariance and the max landing where it should
    rng = np.random.default_rng(2)
    z = rng.standard_normal(300).astype(np.float32)
    P0, m0, Z0 = O.softmax_row(z)
    P1, m1, Z1 = O.softmax_row((z.astype(np.float64) + 5.0).astype(np.float32))
    np.testing.assert_allclose(P0, P1, rtol=2e-6)
    assert np.argmax(P0) == np.argmax(z) and m0 == float(z.max())


def test_temperature_scales_logits_not_probabilities():
    z = np.array([0.0, 1.0, 2.0, -1.0], np.float32)
    P, m, Z = O.softmax_row(z, O.F32, 2.0)
    want = np.exp(2.0 * z.astype(np.float64) - 4.0)
    np.testing.assert_allclose(P, want / want.sum(), rtol=1e-14)
    assert m == 4.0


def test_bf16_is_widened_exactly():
    rng = np.random.default_rng(3)
    z32 = (rng.standard_normal(999) * 4).astype(np.float32)
    bits = (z32.view(np.uint32) >> 16).astype(np.uint16)           # truncate to bf16
    widened = (bits.astype(np.uint32) << 16).view(np.float32)
    Pb, mb, Zb = O.softmax_row(bits, O.BF16, 1.3)
    Pf, mf, Zf = O.softmax_row(widened, O.F32, 1.3)
    assert (Pb == Pf).all() and mb == mf and Zb == Zf
