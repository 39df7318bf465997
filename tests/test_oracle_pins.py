"""Pins for the CPU oracle: closed forms, library routines, invariants, brute force.

None of these re-type the oracle's own formula.  Each check is a function of
the oracle module so that the mutation tests at the bottom can show that a
plausible mistake planted in the oracle (on the CPU) fails at least one pin.
"""

import math
import os

import numpy as np
import pytest
import scipy.special

import oracle.fourier_kv as fk
from oracle import brute

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------
# checks (each raises AssertionError on failure)
# --------------------------------------------------------------------------

def check_gram_is_inverse_weights():
    """Orthogonality over one period: Phi^T Phi = diag(1 / w)  (T = N, M = T)."""
    for T in (8, 9, 64, 381):
        phi = fk.basis_matrix(T, T, 0, T)
        gram = phi.T @ phi
        w = fk.basis_weights(T, T)
        assert np.allclose(gram, np.diag(1.0 / w), atol=1e-9 * T), T


def check_projector_matches_literal_eq4():
    """compress->reconstruct equals the orthogonal projector onto the row
    space of the paper's literal 2k x L matrix (Eq. 4, with its zero row)."""
    for (k, T) in ((3, 16), (5, 31), (8, 40)):
        t = np.arange(T)
        rows = []
        for n in range(k):
            rows.append(np.cos(2 * np.pi * n * t / T))
            rows.append(np.sin(2 * np.pi * n * t / T))
        F = np.stack(rows)                                   # [2k, T]
        P_lit = np.linalg.pinv(F) @ F
        M = 2 * k - 1
        mask = np.ones(1, dtype=np.uint8)
        P = np.empty((T, T))
        for j in range(T):
            e = np.zeros((T, 1)); e[j, 0] = 1.0
            C, keep = fk.compress_segment(e, mask, M, T)
            P[:, j] = fk.reconstruct_segment(C, keep, mask, T, 0, T)[:, 0]
        assert np.allclose(P, P_lit, atol=1e-12), (k, T)


def _read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *nums = line.split()
            vals[key] = np.array([float(v) for v in nums])
    return vals


def check_worked_example():
    g = _read_golden("worked_projection_T8.txt")
    C, keep = fk.compress_segment(g["x"][:, None], np.ones(1, np.uint8), 8, 8)
    assert keep.shape == (8, 0)
    assert np.allclose(C[:, 0], g["C"], atol=1e-13)


def check_rfft_equality():
    """T = N: cosine coefficients are Re(rfft), sine coefficients are -Im(rfft)."""
    rng = np.random.default_rng(7)
    for N in (16, 45, 380):
        x = rng.standard_normal((N, 3))
        M = N if N % 2 == 1 else N  # full band
        C, _ = fk.compress_segment(x, np.ones(3, np.uint8), M, N)
        X = np.fft.rfft(x, axis=0)
        assert np.allclose(C[0], X[0].real, atol=1e-10)
        for m in range(1, M):
            n = (m + 1) // 2
            want = X[n].real if m % 2 == 1 else -X[n].imag
            assert np.allclose(C[m], want, atol=1e-10), (N, m)


def check_additivity_and_streaming():
    """Linearity in tokens: chunks add up; Eq. 5 is the one-token chunk."""
    rng = np.random.default_rng(11)
    N, T, M = 50, 64, 21
    x = rng.standard_normal((N, 6))
    mask = np.array([1, 0, 1, 1, 0, 1], np.uint8)
    C_all, keep_all = fk.compress_segment(x, mask, M, T, t0=3)
    a = 17
    C1, k1 = fk.compress_segment(x[:a], mask, M, T, t0=3)
    C2, k2 = fk.compress_segment(x[a:], mask, M, T, t0=3 + a, C_prev=C1)
    assert np.allclose(C2, C_all, atol=1e-12)
    assert np.array_equal(np.concatenate([k1, k2]), keep_all)
    C = np.zeros_like(C_all)
    for j in range(N):
        C, _ = fk.compress_segment(x[j:j + 1], mask, M, T, t0=3 + j, C_prev=C)
    assert np.allclose(C, C_all, atol=1e-12)
    # kept columns are the unmasked ones in ascending order, untouched
    assert np.array_equal(keep_all, x[:, [1, 4]])


def check_reconstruction_closed_forms():
    rng = np.random.default_rng(3)
    # M = N = T: exact reconstruction, odd and even N
    for N in (8, 9, 380):
        x = rng.standard_normal((N, 4))
        mask = np.array([1, 1, 0, 1], np.uint8)
        C, keep = fk.compress_segment(x, mask, N, N)
        xr = fk.reconstruct_segment(C, keep, mask, N, 0, N)
        assert np.allclose(xr, x, atol=1e-11), N
    # in-band signal recovered exactly by a band that covers it
    N = 120
    j = np.arange(N)
    sig = 0.7 + 1.3 * np.cos(2 * np.pi * 5 * j / N + 0.4) - 0.8 * np.sin(2 * np.pi * 9 * j / N)
    for M in (19, 20, 33):
        C, keep = fk.compress_segment(sig[:, None], np.ones(1, np.uint8), M, N)
        xr = fk.reconstruct_segment(C, keep, np.ones(1, np.uint8), N, 0, N)
        assert np.allclose(xr[:, 0], sig, atol=1e-12), M
    # out-of-band component is removed entirely
    hi = np.cos(2 * np.pi * 30 * j / N)
    C, keep = fk.compress_segment(hi[:, None], np.ones(1, np.uint8), 21, N)
    assert np.allclose(C, 0.0, atol=1e-11)
    # projector: symmetric, idempotent, trace = M
    M = 14
    phi = fk.basis_matrix(M, N, 0, N)
    P = phi @ (fk.basis_weights(M, N)[:, None] * phi.T)
    assert np.allclose(P, P.T, atol=1e-13)
    assert np.allclose(P @ P, P, atol=1e-12)
    assert abs(np.trace(P) - M) < 1e-10


def _vanilla(q, K, V, scale):
    p = scipy.special.softmax(scale * (K @ q))
    return p @ V


def _rand_case(rng, G=2, d=16, N=40, W=6, Dkc=9, Dvc=12):
    q = rng.standard_normal((G, d))
    K = rng.standard_normal((N + W, d))
    V = rng.standard_normal((N + W, d))
    kmask = np.zeros(d, np.uint8); kmask[rng.choice(d, Dkc, replace=False)] = 1
    vmask = np.zeros(d, np.uint8); vmask[rng.choice(d, Dvc, replace=False)] = 1
    return q, K, V, kmask, vmask


def _run_decode(q, K, V, kmask, vmask, N, W, M, T, t0=0, scale=None, perm=None):
    """Compress rows W.. (the middle) and decode; first W rows stay full-width."""
    Ck, kk = fk.compress_segment(K[W:], kmask, M, T, t0)
    Cv, vk = fk.compress_segment(V[W:], vmask, M, T, t0)
    kf, vf = K[:W], V[:W]
    if perm is not None:
        kf, vf = kf[perm], vf[perm]
    return fk.decode_head_group(q, Ck, kmask, Cv, vmask, T, t0, N, kk, vk, kf, vf, scale)


def check_attention_special_cases():
    rng = np.random.default_rng(5)
    G, d, N, W = 2, 16, 40, 6
    q, K, V, kmask, vmask = _rand_case(rng, G, d, N, W)
    scale = 1.0 / math.sqrt(d)
    want = np.stack([_vanilla(q[g], K, V, scale) for g in range(G)])
    # nothing compressed -> vanilla attention over all rows
    zero = np.zeros(d, np.uint8)
    got = _run_decode(q, K, V, zero, zero, N, W, 7, N)
    assert np.allclose(got, want, atol=1e-13)
    # full band (M = N = T) -> vanilla attention on the original K, V
    got = _run_decode(q, K, V, kmask, vmask, N, W, N, N)
    assert np.allclose(got, want, atol=1e-11)
    # explicit scale is honoured
    got = _run_decode(q, K, V, kmask, vmask, N, W, N, N, scale=0.37)
    want2 = np.stack([_vanilla(q[g], K, V, 0.37) for g in range(G)])
    assert np.allclose(got, want2, atol=1e-11)
    # q = 0, T = N: uniform weights -> column mean of the original V, any M >= 1
    for M in (1, 2, 5, 12, N):
        got = _run_decode(np.zeros((1, d)), K, V, kmask, vmask, N, W, M, N)
        assert np.allclose(got[0], V.mean(axis=0), atol=1e-12), M
    # order of the full-width rows does not matter
    perm = rng.permutation(W)
    a = _run_decode(q, K, V, kmask, vmask, N, W, 9, N)
    b = _run_decode(q, K, V, kmask, vmask, N, W, 9, N, perm=perm)
    assert np.allclose(a, b, atol=1e-13)
    # two query heads of a group with the same q give the same output
    qq = np.stack([q[0], q[0]])
    o = _run_decode(qq, K, V, kmask, vmask, N, W, 9, N)
    assert np.array_equal(o[0], o[1])
    # a compressed K dimension that is a pure in-band sinusoid is seen exactly:
    Ks = K.copy()
    jj = np.arange(N)
    for dim in np.flatnonzero(kmask):
        Ks[W:, dim] = np.cos(2 * np.pi * 3 * jj / N + dim)
    Vs = V.copy()
    for dim in np.flatnonzero(vmask):
        Vs[W:, dim] = 0.5 + np.sin(2 * np.pi * 2 * jj / N + dim)
    got = _run_decode(q, Ks, Vs, kmask, vmask, N, W, 9, N)
    want3 = np.stack([_vanilla(q[g], Ks, Vs, scale) for g in range(G)])
    assert np.allclose(got, want3, atol=1e-12)


def check_brute_force():
    rng = np.random.default_rng(21)
    G, d, N, W = 2, 8, 12, 3
    for M, T, t0 in ((1, 12, 0), (4, 12, 0), (5, 12, 0), (12, 12, 0), (6, 20, 5)):
        q, K, V, kmask, vmask = _rand_case(rng, G, d, N, W, Dkc=5, Dvc=3)
        Ck, kk = fk.compress_segment(K[W:], kmask, M, T, t0)
        Cv, vk = fk.compress_segment(V[W:], vmask, M, T, t0)
        Cb, kb = brute.compress(K[W:].tolist(), kmask.tolist(), M, T, t0)
        assert np.allclose(Ck, np.array(Cb).reshape(M, -1), atol=1e-12)
        assert np.array_equal(kk, np.array(kb).reshape(N, -1))
        w = [brute.weight(m, T) for m in range(M)]
        assert np.allclose(fk.basis_weights(M, T), w, rtol=1e-12)
        scale = 1.0 / math.sqrt(d)
        got = fk.decode_head_group(q, Ck, kmask, Cv, vmask, T, t0, N, kk, vk, K[:W], V[:W])
        want = brute.decode(q.tolist(), Ck.tolist(), kmask.tolist(), Cv.tolist(), vmask.tolist(),
                            T, t0, N, kk.tolist(), vk.tolist(), K[:W].tolist(), V[:W].tolist(), scale)
        assert np.allclose(got, np.array(want), atol=1e-12), (M, T, t0)


def check_large_phase_is_exact():
    """order*position beyond 2^24 must not lose the phase (integer reduction)."""
    T, M = 129020, 512
    t0 = T - 4
    phi = fk.basis_matrix(M, T, t0, 4)
    # positions T-4..T-1 are positions -4..-1 by periodicity
    for r, p in enumerate((-4, -3, -2, -1)):
        for m in (1, 2, 255, 256, 511):
            n = (m + 1) // 2
            ang = 2 * math.pi * n * p / T
            want = math.cos(ang) if m % 2 else math.sin(ang)
            assert abs(phi[r, m] - want) < 1e-12, (p, m)


def check_batched_wrappers():
    rng = np.random.default_rng(9)
    B, Hkv, G, d, N, W, M = 2, 2, 2, 8, 10, 3, 5
    X = rng.standard_normal((B, Hkv, N + W, d))
    Y = rng.standard_normal((B, Hkv, N + W, d))
    q = rng.standard_normal((B, Hkv * G, d))
    km = np.zeros((B, Hkv, d), np.uint8); vm = np.zeros((B, Hkv, d), np.uint8)
    for b in range(B):
        for h in range(Hkv):
            km[b, h, rng.choice(d, 3, replace=False)] = 1
            vm[b, h, rng.choice(d, 5, replace=False)] = 1
    Ck, kk = fk.compress_batched(X[:, :, W:], km, M, N)
    Cv, vk = fk.compress_batched(Y[:, :, W:], vm, M, N)
    out = fk.decode_batched(q, Ck, km, Cv, vm, N, 0, N, kk, vk, X[:, :, :W], Y[:, :, :W])
    for b in range(B):
        for hq in range(Hkv * G):
            h = hq // G
            one = _run_decode(q[b, hq:hq + 1], X[b, h], Y[b, h], km[b, h], vm[b, h], N, W, M, N)
            assert np.allclose(out[b, hq], one[0], atol=1e-13)


def check_varlen_decode():
    """decode_varlen: equal lengths = decode_batched; every sequence = vanilla attention over exactly
    its own rows when the band is full (M = its row count = T); rows past a sequence's counts are
    invisible to it, rows inside are not; a sequence without rows gives zeros."""
    rng = np.random.default_rng(21)
    B, Hkv, G, d, N, W, M = 3, 2, 2, 8, 12, 4, 5
    T = 16
    Xk = rng.standard_normal((B, Hkv, N, d)); Xv = rng.standard_normal((B, Hkv, N, d))
    Kf = rng.standard_normal((B, Hkv, W, d)); Vf = rng.standard_normal((B, Hkv, W, d))
    q = rng.standard_normal((B, Hkv * G, d))
    km = np.zeros((B, Hkv, d), np.uint8); vm = np.zeros((B, Hkv, d), np.uint8)
    for b in range(B):
        for h in range(Hkv):
            km[b, h, rng.choice(d, 3, replace=False)] = 1
            vm[b, h, rng.choice(d, 5, replace=False)] = 1

    def state(seq_n):
        Ck = np.zeros((B, Hkv, M, 3)); Cv = np.zeros((B, Hkv, M, 5))
        kk = rng.standard_normal((B, Hkv, N, d - 3)); vk = rng.standard_normal((B, Hkv, N, d - 5))   # rows past n: junk
        for b in range(B):
            for h in range(Hkv):
                n = seq_n[b]
                Ck[b, h], kk[b, h, :n] = fk.compress_segment(Xk[b, h, :n], km[b, h], M, T, 0)
                Cv[b, h], vk[b, h, :n] = fk.compress_segment(Xv[b, h, :n], vm[b, h], M, T, 0)
        return Ck, Cv, kk, vk

    # equal lengths: the batched wrapper
    full = [N] * B
    Ck, Cv, kk, vk = state(full)
    a = fk.decode_varlen(q, Ck, km, Cv, vm, T, 0, full, kk, vk, Kf, Vf, [W] * B)
    b_ = fk.decode_batched(q, Ck, km, Cv, vm, T, 0, N, kk, vk, Kf, Vf)
    assert np.allclose(a, b_, atol=1e-14)
    # different lengths: each sequence alone
    seq_n, seq_w = [12, 0, 7], [4, 3, 0]
    Ck, Cv, kk, vk = state(seq_n)
    out = fk.decode_varlen(q, Ck, km, Cv, vm, T, 0, seq_n, kk, vk, Kf, Vf, seq_w)
    for b in range(B):
        for h in range(Hkv):
            n, w = seq_n[b], seq_w[b]
            one = fk.decode_head_group(q[b, h * G:(h + 1) * G], Ck[b, h], km[b, h], Cv[b, h], vm[b, h], T, 0, n,
                                       kk[b, h, :n], vk[b, h, :n], Kf[b, h, :w], Vf[b, h, :w])
            assert np.allclose(out[b, h * G:(h + 1) * G], one, atol=1e-14)
    # rows past the counts are invisible, rows inside are not
    kk2, Kf2 = kk.copy(), Kf.copy()
    kk2[2, :, 7:] += 100.0; Kf2[1, :, 3:] += 100.0
    assert np.array_equal(fk.decode_varlen(q, Ck, km, Cv, vm, T, 0, seq_n, kk2, vk, Kf2, Vf, seq_w), out)
    kk2 = kk.copy(); kk2[2, :, 6] += 1.0
    assert not np.allclose(fk.decode_varlen(q, Ck, km, Cv, vm, T, 0, seq_n, kk2, vk, Kf, Vf, seq_w)[2], out[2])
    # full band on a sequence's own rows (M = n = T): vanilla attention over exactly those rows
    n, w = 7, 2
    km0 = km[:1]; vm0 = vm[:1]
    Ck1 = np.zeros((1, Hkv, n, 3)); Cv1 = np.zeros((1, Hkv, n, 5))
    kk1 = np.zeros((1, Hkv, N, d - 3)); vk1 = np.zeros((1, Hkv, N, d - 5))
    for h in range(Hkv):
        Ck1[0, h], kk1[0, h, :n] = fk.compress_segment(Xk[0, h, :n], km0[0, h], n, n, 0)
        Cv1[0, h], vk1[0, h, :n] = fk.compress_segment(Xv[0, h, :n], vm0[0, h], n, n, 0)
    got = fk.decode_varlen(q[:1], Ck1, km0, Cv1, vm0, n, 0, [n], kk1, vk1, Kf[:1], Vf[:1], [w])
    for h in range(Hkv):
        Kt = np.concatenate([Kf[0, h, :w], Xk[0, h, :n]]); Vt = np.concatenate([Vf[0, h, :w], Xv[0, h, :n]])
        for g in range(G):
            s_ = Kt @ q[0, h * G + g] / np.sqrt(d)
            p_ = np.exp(s_ - s_.max()); p_ /= p_.sum()
            assert np.allclose(got[0, h * G + g], p_ @ Vt, atol=1e-10)
    # no rows at all: zeros
    z = fk.decode_varlen(q, Ck, km, Cv, vm, T, 0, [0, 0, 0], kk, vk, Kf, Vf, [0, 0, 0])
    assert not z.any()


ALL_CHECKS = (
    check_gram_is_inverse_weights,
    check_projector_matches_literal_eq4,
    check_worked_example,
    check_rfft_equality,
    check_additivity_and_streaming,
    check_reconstruction_closed_forms,
    check_attention_special_cases,
    check_brute_force,
    check_large_phase_is_exact,
    check_batched_wrappers,
    check_varlen_decode,
)


@pytest.mark.parametrize("check", ALL_CHECKS, ids=lambda f: f.__name__)
def test_pin(check):
    check()


# --------------------------------------------------------------------------
# mutation tests: mistakes planted in the oracle must trip a pin
# --------------------------------------------------------------------------

def _some_pin_fails():
    for check in ALL_CHECKS:
        try:
            check()
        except (AssertionError, ValueError, IndexError):
            return True
    return False


def _mut_swap_trig(orig):
    def f(M, T, t0, N):
        phi = orig(M, T, t0, N).copy()
        odd = phi[:, 1::2].copy()
        k = min(odd.shape[1], phi[:, 2::2].shape[1])
        phi[:, 1:1 + 2 * k:2], phi[:, 2:2 + 2 * k:2] = phi[:, 2:2 + 2 * k:2].copy(), odd[:, :k]
        return phi
    return f


def _mut_sine_sign(orig):
    def f(M, T, t0, N):
        phi = orig(M, T, t0, N).copy()
        phi[:, 2::2] *= -1.0
        return phi
    return f


def _mut_ignore_t0(orig):
    return lambda M, T, t0, N: orig(M, T, 0, N)


def _mut_order_off_by_one(orig):
    def f(M, T, t0, N):
        phi = orig(min(M + 2, T), T, t0, N)
        out = phi[:, :M].copy()
        if M > 2:
            out[:, 1:] = orig(min(M + 2, T), T, t0, N)[:, 3:M + 2] if M + 2 <= T else out[:, 1:]
        return out
    return f


def _mut_dc_weight(orig):
    def f(M, T):
        w = orig(M, T).copy()
        w[0] = 2.0 / T
        return w
    return f


def _mut_paper_one_over_k(orig):
    def f(M, T):
        k = (M + 1) // 2
        return np.full(M, 1.0 / k)
    return f


def _mut_nyquist_weight(orig):
    def f(M, T):
        return np.where(np.arange(M) == 0, 1.0 / T, 2.0 / T)
    return f


@pytest.mark.parametrize("name,target,mut", [
    ("swap_cos_sin", "basis_matrix", _mut_swap_trig),
    ("sine_sign", "basis_matrix", _mut_sine_sign),
    ("ignore_t0", "basis_matrix", _mut_ignore_t0),
    ("order_off_by_one", "basis_matrix", _mut_order_off_by_one),
    ("dc_weight", "basis_weights", _mut_dc_weight),
    ("one_over_k", "basis_weights", _mut_paper_one_over_k),
    ("nyquist_weight", "basis_weights", _mut_nyquist_weight),
])
def test_planted_mistake_is_caught(monkeypatch, name, target, mut):
    monkeypatch.setattr(fk, target, mut(getattr(fk, target)))
    assert _some_pin_fails(), name


def test_planted_mistakes_in_attention_are_caught(monkeypatch):
    # dropped softmax normalisation
    def attend_no_norm(q, K, V, scale):
        s = scale * (K @ q)
        return np.exp(s - s.max()) @ V
    monkeypatch.setattr(fk, "attend", attend_no_norm)
    assert _some_pin_fails()
    monkeypatch.undo()

    # transposed operand: V reconstructed from K's coefficients (the paper's typo taken literally)
    orig = fk.decode_head_group

    def decode_typo(q, Ck, kmask, Cv, vmask, T, t0, N, kk, vk, kf, vf, scale=None):
        return orig(q, Ck, kmask, Ck if Ck.shape == Cv.shape else Cv * 0, vmask, T, t0, N, kk, vk, kf, vf, scale)
    monkeypatch.setattr(fk, "decode_head_group", decode_typo)
    assert _some_pin_fails()
    monkeypatch.undo()

    # kept columns written in the wrong order
    orig_c = fk.compress_segment

    def compress_rev(X, mask, M, T, t0=0, C_prev=None):
        C, keep = orig_c(X, mask, M, T, t0, C_prev)
        return C, keep[:, ::-1]
    monkeypatch.setattr(fk, "compress_segment", compress_rev)
    assert _some_pin_fails()


# ---------------------------------------------------------------------------
# streaming maintenance (Eq. 5 + the window of Eq. 1)
# ---------------------------------------------------------------------------
def test_append_token_equals_recompression_of_the_longer_segment():
    """Feeding tokens one at a time through the window must leave exactly the state that
    compressing the longer middle segment in one shot gives, and attention over that state
    must equal attention over the one-shot state (Eq. 5 is Eq. 3 restricted to one row)."""
    rng = np.random.default_rng(77)
    d, Li, Lw, N0, steps, M = 16, 2, 5, 20, 9, 7
    T = N0 + steps
    kmask = np.zeros(d, np.uint8); kmask[rng.choice(d, 11, replace=False)] = 1
    vmask = np.zeros(d, np.uint8); vmask[rng.choice(d, 9, replace=False)] = 1
    total = Li + N0 + Lw + steps
    K = rng.standard_normal((total, d)); V = rng.standard_normal((total, d))
    # state after prefill: sink rows, N0 middle rows compressed, a full window
    Ck, kk = fk.compress_segment(K[Li:Li + N0], kmask, M, T, 0)
    Cv, vk = fk.compress_segment(V[Li:Li + N0], vmask, M, T, 0)
    k_full = np.concatenate([K[:Li], K[Li + N0:Li + N0 + Lw]]); v_full = np.concatenate([V[:Li], V[Li + N0:Li + N0 + Lw]])
    for s in range(steps):
        slot = Li + s % Lw            # ring: the oldest window row
        t_new = Li + N0 + Lw + s
        Ck, Cv, kk, vk, k_full, v_full = fk.append_token(Ck, Cv, kmask, vmask, kk, vk, k_full, v_full, slot,
                                                         K[t_new], V[t_new], T, N0 + s, True)
    # one-shot reference over the longer segment
    Ck1, kk1 = fk.compress_segment(K[Li:Li + N0 + steps], kmask, M, T, 0)
    Cv1, vk1 = fk.compress_segment(V[Li:Li + N0 + steps], vmask, M, T, 0)
    assert np.allclose(Ck, Ck1, atol=1e-12) and np.allclose(Cv, Cv1, atol=1e-12)
    assert np.array_equal(kk, kk1) and np.array_equal(vk, vk1)
    # the window holds the last Lw tokens (as a set of rows), the sink rows are untouched
    want = K[total - Lw:]
    got = k_full[Li:]
    assert np.array_equal(np.sort(got, axis=0), np.sort(want, axis=0))
    assert np.array_equal(k_full[:Li], K[:Li])
    q = rng.standard_normal((2, d))
    o_stream = fk.decode_head_group(q, Ck, kmask, Cv, vmask, T, 0, N0 + steps, kk, vk, k_full, v_full)
    o_shot = fk.decode_head_group(q, Ck1, kmask, Cv1, vmask, T, 0, N0 + steps, kk1, vk1,
                                  np.concatenate([K[:Li], K[total - Lw:]]), np.concatenate([V[:Li], V[total - Lw:]]))
    assert np.allclose(o_stream, o_shot, atol=1e-12)


def test_append_token_without_eviction_only_fills_the_window():
    rng = np.random.default_rng(5)
    d, M, T = 8, 5, 40
    kmask = np.array([1, 0, 1, 1, 0, 0, 1, 0], np.uint8); vmask = kmask[::-1].copy()
    Ck = rng.standard_normal((M, 4)); Cv = rng.standard_normal((M, 4))
    kk = rng.standard_normal((3, 4)); vk = rng.standard_normal((3, 4))
    k_full = rng.standard_normal((6, d)); v_full = rng.standard_normal((6, d))
    kn, vn = rng.standard_normal(d), rng.standard_normal(d)
    out = fk.append_token(Ck, Cv, kmask, vmask, kk, vk, k_full, v_full, 4, kn, vn, T, 3, False)
    assert np.array_equal(out[0], Ck) and np.array_equal(out[1], Cv)
    assert np.array_equal(out[2], kk) and np.array_equal(out[3], vk)
    assert np.array_equal(out[4][4], kn) and np.array_equal(out[5][4], vn)
    assert np.array_equal(np.delete(out[4], 4, axis=0), np.delete(k_full, 4, axis=0))


# --------------------------------------------------------------------------
# dimension selection (Section 3.4)
# --------------------------------------------------------------------------

def _mse_from_fft(X, M):
    """Independent route to the reconstruction error: with the segment spanning one period the
    first M real basis functions span the DC bin and the lowest complex bins of numpy's FFT, so
    the error is the energy of the discarded bins (Parseval), no basis matrix involved."""
    N = X.shape[0]
    F = np.fft.rfft(X, axis=0)                      # bins 0 .. N//2
    power = np.abs(F) ** 2
    power[1:(N + 1) // 2] *= 2.0                    # bins with a conjugate twin count twice
    kept = np.zeros(F.shape[0])
    nfull = (M - 1) // 2                            # orders with both cosine and sine kept
    kept[: nfull + 1] = 1.0
    err = (power * (1.0 - kept)[:, None]).sum(axis=0) / N
    if M % 2 == 0:                                  # one more cosine without its sine
        n = M // 2
        if 2 * n == N:                              # the Nyquist bin is real: its cosine is all of it
            err -= power[n] / N
        else:
            err -= 2.0 * F[n].real ** 2 / N         # cosine part of bin n (half of the doubled power)
    return err / N


def test_reconstruction_mse_is_the_energy_of_the_discarded_fft_bins():
    rng = np.random.default_rng(5)
    for N, M in ((64, 9), (64, 10), (50, 50), (50, 49), (37, 1), (128, 64), (33, 33)):
        X = rng.standard_normal((N, 5))
        got = fk.reconstruction_mse(X, M)
        want = _mse_from_fft(X, M)
        assert np.allclose(got, want, rtol=1e-9, atol=1e-12), (N, M, got, want)


def test_select_dims_picks_the_band_limited_dimensions():
    rng = np.random.default_rng(6)
    N, d, M = 240, 12, 17
    t = np.arange(N)
    X = rng.standard_normal((N, d))
    smooth = [1, 4, 5, 9]
    for i, dim in enumerate(smooth):                # in-band tones (orders <= 8) plus a little noise
        X[:, dim] = np.cos(2 * np.pi * (i + 1) * t / N + 0.3 * i) + 0.5 * np.sin(2 * np.pi * (i + 3) * t / N) \
            + 0.01 * rng.standard_normal(N)
    mask, mse = fk.select_dims(X, M, len(smooth))
    assert sorted(np.flatnonzero(mask)) == smooth
    assert mse[smooth].max() < 2e-4 and np.delete(mse, smooth).min() > 0.5
    # ties go to the lower index, and the count is exact
    Z = np.zeros((N, 6))
    m0, e0 = fk.select_dims(Z, M, 4)
    assert m0.tolist() == [1, 1, 1, 1, 0, 0] and not e0.any()
    assert fk.select_dims(X, M, 0)[0].sum() == 0 and fk.select_dims(X, M, d)[0].sum() == d


def test_reconstruction_mse_brute_force_tiny():
    rng = np.random.default_rng(7)
    N, M = 7, 4
    X = rng.standard_normal((N, 2))
    want = np.zeros(2)
    for dcol in range(2):
        x = X[:, dcol]
        # plain loops: coefficients, weights, rebuilt samples
        fn = [lambda j: 1.0,
              lambda j: math.cos(2 * math.pi * j / N), lambda j: math.sin(2 * math.pi * j / N),
              lambda j: math.cos(4 * math.pi * j / N)]
        c = [sum(f(j) * x[j] for j in range(N)) for f in fn]
        w = [1.0 / N, 2.0 / N, 2.0 / N, 2.0 / N]
        for j in range(N):
            xr = sum(w[m] * c[m] * fn[m](j) for m in range(M))
            want[dcol] += (x[j] - xr) ** 2 / N
    assert np.allclose(fk.reconstruction_mse(X, M), want, rtol=1e-12, atol=1e-14)


# --------------------------------------------------------------------------
# several query tokens per step (causal among the new tokens)
# --------------------------------------------------------------------------

def _mq_case(seed=11, N=40, W=9, d=8, G=2, Tq=3, M=7):
    rng = np.random.default_rng(seed)
    kmask = (rng.random(d) < 0.5).astype(np.uint8)
    vmask = (rng.random(d) < 0.5).astype(np.uint8)
    K, V = rng.standard_normal((N, d)), rng.standard_normal((N, d))
    Ck, kk = fk.compress_segment(K, kmask, M, N, 0)
    Cv, vk = fk.compress_segment(V, vmask, M, N, 0)
    kf, vf = rng.standard_normal((W, d)), rng.standard_normal((W, d))
    q = rng.standard_normal((Tq, G, d))
    return dict(q=q, Ck=Ck, kmask=kmask, Cv=Cv, vmask=vmask, T=N, t0=0, N=N, k_keep=kk, v_keep=vk,
                k_full=kf, v_full=vf)


def test_multi_query_decode_is_causal_among_the_new_tokens():
    c = _mq_case()
    base = fk.decode_multi_query(**c)
    Tq, W = c["q"].shape[0], c["k_full"].shape[0]
    # one query token = the ordinary decode over all rows
    one = fk.decode_multi_query(**dict(c, q=c["q"][-1:]))
    assert np.allclose(one[0], fk.decode_head_group(c["q"][-1], c["Ck"], c["kmask"], c["Cv"], c["vmask"], c["T"], 0,
                                                    c["N"], c["k_keep"], c["v_keep"], c["k_full"], c["v_full"]))
    # the last query sees everything: same as the ordinary decode too
    assert np.allclose(base[-1], one[0])
    # changing new token t leaves the outputs of queries < t untouched and changes query t
    for t in range(1, Tq):
        kf2, vf2 = c["k_full"].copy(), c["v_full"].copy()
        kf2[W - Tq + t] += 1.0
        vf2[W - Tq + t] -= 2.0
        alt = fk.decode_multi_query(**dict(c, k_full=kf2, v_full=vf2))
        assert np.array_equal(alt[:t], base[:t])
        assert not np.allclose(alt[t], base[t])
    # an older row is visible to every query
    kf3 = c["k_full"].copy()
    kf3[0] += 3.0
    alt = fk.decode_multi_query(**dict(c, k_full=kf3))
    assert all(not np.allclose(alt[t], base[t]) for t in range(Tq))


def test_multi_query_decode_brute_force():
    c = _mq_case(seed=12, N=12, W=5, d=4, G=1, Tq=2, M=5)
    got = fk.decode_multi_query(**c)
    Km = fk.reconstruct_segment(c["Ck"], c["k_keep"], c["kmask"], c["T"], 0, c["N"])
    Vm = fk.reconstruct_segment(c["Cv"], c["v_keep"], c["vmask"], c["T"], 0, c["N"])
    W, Tq, d = 5, 2, 4
    for t in range(Tq):
        rows_k = [c["k_full"][j] for j in range(W) if j <= W - Tq + t] + [Km[j] for j in range(c["N"])]
        rows_v = [c["v_full"][j] for j in range(W) if j <= W - Tq + t] + [Vm[j] for j in range(c["N"])]
        s = [sum(c["q"][t, 0, i] * rk[i] for i in range(d)) / math.sqrt(d) for rk in rows_k]
        mx = max(s)
        e = [math.exp(x - mx) for x in s]
        z = sum(e)
        want = [sum(e[j] / z * rows_v[j][i] for j in range(len(e))) for i in range(d)]
        assert np.allclose(got[t, 0], want, rtol=1e-12, atol=1e-14)

