"""Pure-Python, loop-by-loop statement of Eq. 1-6 for tiny shapes.

TEST INFRASTRUCTURE ONLY.  No numpy arithmetic: every sum is an explicit
loop over Python floats and every phase an exact Python integer, so that the
vectorised oracle in `fourier_kv.py` can be pinned to the definitions without
sharing its indexing.
"""

from __future__ import annotations

import math


def phi(m: int, pos: int, T: int) -> float:
    """m-th function of 1, cos(wt), sin(wt), cos(2wt), sin(2wt), ... (Eq. 4)."""
    if m == 0:
        return 1.0
    n = (m + 1) // 2
    ang = 2.0 * math.pi * ((n * pos) % T) / T
    return math.cos(ang) if m % 2 == 1 else math.sin(ang)


def weight(m: int, T: int) -> float:
    """1 / sum_{t<T} phi_m(t)^2, evaluated as the literal sum."""
    s = 0.0
    for t in range(T):
        v = phi(m, t, T)
        s += v * v
    return 1.0 / s


def compress(X, mask, M, T, t0=0):
    """Eq. 2-3: C[m][i] = sum_j phi_m(t0+j) X[j][idx_c[i]]; kept columns copied."""
    N = len(X)
    idx_c = [d for d, b in enumerate(mask) if b]
    idx_u = [d for d, b in enumerate(mask) if not b]
    C = [[0.0] * len(idx_c) for _ in range(M)]
    for m in range(M):
        for i, d in enumerate(idx_c):
            acc = 0.0
            for j in range(N):
                acc += phi(m, t0 + j, T) * X[j][d]
            C[m][i] = acc
    keep = [[X[j][d] for d in idx_u] for j in range(N)]
    return C, keep


def decode(q, Ck, kmask, Cv, vmask, T, t0, N, k_keep, v_keep, k_full, v_full, scale):
    """Eq. 6 for one KV head: q is a list of query vectors sharing the head."""
    d = len(kmask)
    M = len(Ck)

    def rebuild(C, keep, mask):
        idx_c = [x for x, b in enumerate(mask) if b]
        idx_u = [x for x, b in enumerate(mask) if not b]
        rows = []
        for j in range(N):
            row = [0.0] * d
            for i, dim in enumerate(idx_c):
                acc = 0.0
                for m in range(M):
                    acc += weight(m, T) * phi(m, t0 + j, T) * C[m][i]
                row[dim] = acc
            for i, dim in enumerate(idx_u):
                row[dim] = keep[j][i]
            rows.append(row)
        return rows

    Kt = [list(r) for r in k_full] + rebuild(Ck, k_keep, kmask)
    Vt = [list(r) for r in v_full] + rebuild(Cv, v_keep, vmask)
    outs = []
    for qv in q:
        s = []
        for row in Kt:
            acc = 0.0
            for x in range(d):
                acc += qv[x] * row[x]
            s.append(scale * acc)
        mx = max(s)
        e = [math.exp(v - mx) for v in s]
        z = sum(e)
        o = [0.0] * d
        for pj, row in zip(e, Vt):
            for x in range(d):
                o[x] += (pj / z) * row[x]
        outs.append(o)
    return outs


# ---------------------------------------------------------------------------
# translated-Legendre alternative (Section 3.2 / 5.1), stated without the recurrence
# ---------------------------------------------------------------------------
def legendre_explicit(m: int, x: float) -> float:
    """P_m(x) from its explicit power series, with exact integer coefficients:
    P_m(x) = 2^-m sum_k (-1)^k C(m, k) C(2m - 2k, m) x^(m - 2k)."""
    s = 0.0
    for k in range(m // 2 + 1):
        s += (-1) ** k * math.comb(m, k) * math.comb(2 * m - 2 * k, m) * x ** (m - 2 * k)
    return s / 2 ** m


def legt_compress_rebuild(xs, M):
    """(states, rebuilt values) of one dimension xs[0..N-1]: c_m = sum_j P_m(x_j) xs[j],
    rebuilt[j] = sum_m (2m+1)/N c_m P_m(x_j), positions x_j = (2j+1)/N - 1."""
    N = len(xs)
    pos = [(2 * j + 1) / N - 1.0 for j in range(N)]
    c = []
    for m in range(M):
        acc = 0.0
        for j in range(N):
            acc += legendre_explicit(m, pos[j]) * xs[j]
        c.append(acc)
    rebuilt = []
    for j in range(N):
        acc = 0.0
        for m in range(M):
            acc += (2 * m + 1) / N * c[m] * legendre_explicit(m, pos[j])
        rebuilt.append(acc)
    return c, rebuilt
