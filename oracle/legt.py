"""fp64 numpy oracle of the translated-Legendre (HiPPO-LegT) alternative basis.

TEST INFRASTRUCTURE ONLY: never imported by the product path.

The paper names LegT ("Legendre polynomials in a translated fixed window", Section 3.2) as the
polynomial alternative to its Fourier basis and compares the two by how well each rebuilds KV
dimensions from the same number of states (Section 5.1, Table 3, the reconstruction figure).  It
gives no formula for its LegT; the reading taken here (listed in the design notes):

  * the window is the compressed segment itself: its N tokens sit at the midpoints
        x_j = (2 j + 1) / N - 1,   j = 0 .. N-1,
    of N equal cells of [-1, 1] (the uniform LegT measure on the window, sampled per token);
  * the state of a dimension is its inner products with the first M Legendre polynomials,
        c_m = sum_j P_m(x_j) x[j]            (plain sums, like the Fourier coefficients of Eq. 3);
  * reconstruction weights every polynomial by the inverse of its squared norm under that measure,
        x~[j] = sum_m (2 m + 1) / N * c_m * P_m(x_j),
    the midpoint-rule image of the continuous projector (int_{-1}^{1} P_m^2 = 2 / (2m+1), one cell
    is 2 / N wide).  Sampled Legendre polynomials are orthogonal only up to the O(1/N^2) error of
    that rule, so compress -> reconstruct is a projector only in the limit; both sides of the
    parity tests reproduce exactly this approximation.

P_m is evaluated by Bonnet's recurrence (m + 1) P_{m+1} = (2m + 1) x P_m - m P_{m-1}, which is
stable for |x| <= 1.  All arithmetic is float64.
"""

from __future__ import annotations

import numpy as np

__all__ = ["legt_positions", "legt_basis", "legt_weights", "legt_compress", "legt_reconstruct", "legt_mse"]


def legt_positions(N: int) -> np.ndarray:
    """Midpoints of N equal cells of [-1, 1]."""
    return (2.0 * np.arange(N, dtype=np.float64) + 1.0) / N - 1.0


def legt_basis(M: int, N: int) -> np.ndarray:
    """P[j, m] = Legendre polynomial of degree m at position x_j."""
    if M < 1 or N < 1:
        raise ValueError("need M >= 1 and N >= 1")
    x = legt_positions(N)
    P = np.empty((N, M), dtype=np.float64)
    P[:, 0] = 1.0
    if M > 1:
        P[:, 1] = x
    for m in range(1, M - 1):
        P[:, m + 1] = ((2 * m + 1) * x * P[:, m] - m * P[:, m - 1]) / (m + 1)
    return P


def legt_weights(M: int, N: int) -> np.ndarray:
    """(2m + 1) / N: inverse squared norm of P_m under the uniform measure, one cell = 2 / N."""
    return (2.0 * np.arange(M, dtype=np.float64) + 1.0) / N


def legt_compress(X, M: int) -> np.ndarray:
    """C[m, d] = sum_j P_m(x_j) X[j, d] for a segment X [N, d]."""
    X = np.asarray(X, dtype=np.float64)
    return legt_basis(M, X.shape[0]).T @ X


def legt_reconstruct(C, N: int) -> np.ndarray:
    """X~[j, d] = sum_m (2m+1)/N C[m, d] P_m(x_j)."""
    C = np.asarray(C, dtype=np.float64)
    M = C.shape[0]
    return legt_basis(M, N) @ (legt_weights(M, N)[:, None] * C)


def legt_mse(X, M: int) -> np.ndarray:
    """Per-dimension mean squared error of compressing X [N, d] to M LegT states and rebuilding it."""
    X = np.asarray(X, dtype=np.float64)
    R = legt_reconstruct(legt_compress(X, M), X.shape[0])
    return np.mean((X - R) ** 2, axis=0)
