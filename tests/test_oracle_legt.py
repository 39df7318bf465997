"""Pins of the translated-Legendre oracle (oracle/legt.py): what mathematics fixes about it.

The paper prints no value for its LegT comparison, so every pin is a closed form, a library
routine that the oracle does not call, an invariant, or a brute force that shares none of its code.
"""

import numpy as np
import pytest
from scipy.special import eval_legendre, roots_legendre

import oracle.brute as brute
import oracle.legt as lg


def test_basis_equals_the_library_polynomials():
    """Bonnet's recurrence against scipy's evaluation (the oracle does not call it)."""
    for N, M in ((7, 7), (64, 33), (1000, 200)):
        P = lg.legt_basis(M, N)
        x = (2.0 * np.arange(N) + 1.0) / N - 1.0
        for m in (0, 1, 2, 3, M // 2, M - 1):
            assert np.allclose(P[:, m], eval_legendre(m, x), rtol=0, atol=2e-12), (N, m)
    assert np.all(np.abs(lg.legt_basis(300, 5000)) <= 1.0 + 1e-12)      # |P_m| <= 1 on [-1, 1]


def test_closed_forms_of_the_first_states():
    """c_0 is the plain sum; a constant has c_1 = 0 by symmetry; a ramp x_j has
    c_1 = sum x_j^2 = (N^2 - 1) / (3 N)."""
    N = 37
    x = lg.legt_positions(N)
    C = lg.legt_compress(np.stack([np.full(N, 2.5), x], axis=1), 3)
    assert C[0, 0] == pytest.approx(2.5 * N, rel=1e-14)
    assert abs(C[1, 0]) < 1e-12
    assert C[1, 1] == pytest.approx((N * N - 1) / (3.0 * N), rel=1e-13)
    assert abs(C[0, 1]) < 1e-12 and abs(C[2, 0] - 2.5 * np.sum(0.5 * (3 * x * x - 1))) < 1e-12


def test_reversing_the_segment_flips_the_odd_states():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((50, 3))
    C, Cr = lg.legt_compress(X, 9), lg.legt_compress(X[::-1], 9)
    sign = (-1.0) ** np.arange(9)
    assert np.allclose(Cr, sign[:, None] * C, atol=1e-12)


def test_gram_matrix_tends_to_the_weights_at_the_midpoint_rule_rate():
    """Sampled Legendre polynomials are orthogonal up to the quadrature error of the midpoint rule:
    diag(w) G -> I with an error that falls fourfold when N doubles."""
    M = 8
    errs = []
    for N in (200, 400, 800):
        P = lg.legt_basis(M, N)
        G = lg.legt_weights(M, N)[:, None] * (P.T @ P)
        errs.append(np.max(np.abs(G - np.eye(M))))
    assert errs[0] < 5e-3 and 3.5 < errs[0] / errs[1] < 4.5 and 3.5 < errs[1] / errs[2] < 4.5


def test_weights_are_the_inverse_continuous_norms():
    """(2m+1)/N against int P_m^2 by Gauss-Legendre quadrature (exact for these degrees)."""
    xg, wg = roots_legendre(40)
    N = 123
    for m in (0, 1, 5, 17):
        norm2 = float(np.sum(wg * eval_legendre(m, xg) ** 2))           # = 2 / (2m + 1)
        assert lg.legt_weights(m + 1, N)[m] == pytest.approx((2.0 / N) / norm2, rel=1e-12)


def test_polynomials_below_the_band_are_recovered_up_to_the_quadrature_error():
    N, M = 600, 6
    x = lg.legt_positions(N)
    f = 0.3 - 1.1 * x + 0.7 * x ** 3 - 0.2 * x ** 5            # degree 5 < M
    e1 = np.max(np.abs(lg.legt_reconstruct(lg.legt_compress(f[:, None], M), N)[:, 0] - f))
    x2 = lg.legt_positions(2 * N)
    f2 = 0.3 - 1.1 * x2 + 0.7 * x2 ** 3 - 0.2 * x2 ** 5
    e2 = np.max(np.abs(lg.legt_reconstruct(lg.legt_compress(f2[:, None], M), 2 * N)[:, 0] - f2))
    assert e1 < 1e-4 and 3.5 < e1 / e2 < 4.5
    # a polynomial ABOVE the band is not: P_7 is (nearly) orthogonal to every kept state
    p7 = eval_legendre(7, x)
    assert np.max(np.abs(lg.legt_reconstruct(lg.legt_compress(p7[:, None], M), N)[:, 0])) < 5e-3


def test_mse_is_the_definition_and_matches_brute_force():
    rng = np.random.default_rng(5)
    N, M = 23, 6
    X = rng.standard_normal((N, 2))
    mse = lg.legt_mse(X, M)
    for d in range(2):
        c, rebuilt = brute.legt_compress_rebuild([float(v) for v in X[:, d]], M)
        assert np.allclose(lg.legt_compress(X, M)[:, d], c, rtol=1e-11, atol=1e-11)
        assert mse[d] == pytest.approx(sum((a - b) ** 2 for a, b in zip(X[:, d], rebuilt)) / N, rel=1e-10)


@pytest.mark.parametrize("mutation", ["weights_2m", "positions_endpoints", "recurrence_sign"])
def test_planted_mistakes_are_caught(mutation, monkeypatch):
    """A plausible mistake planted in the oracle must fail at least one pin above."""
    if mutation == "weights_2m":
        monkeypatch.setattr(lg, "legt_weights", lambda M, N: 2.0 * np.arange(M) / N)
        with pytest.raises(AssertionError):
            test_weights_are_the_inverse_continuous_norms()
    elif mutation == "positions_endpoints":
        monkeypatch.setattr(lg, "legt_positions", lambda N: np.linspace(-1.0, 1.0, N))
        with pytest.raises(AssertionError):
            test_closed_forms_of_the_first_states()
    else:
        def bad_basis(M, N):
            x = lg.legt_positions(N)
            P = np.empty((N, M))
            P[:, 0] = 1.0
            if M > 1:
                P[:, 1] = x
            for m in range(1, M - 1):
                P[:, m + 1] = ((2 * m + 1) * x * P[:, m] + m * P[:, m - 1]) / (m + 1)
            return P
        monkeypatch.setattr(lg, "legt_basis", bad_basis)
        with pytest.raises(AssertionError):
            test_basis_equals_the_library_polynomials()
