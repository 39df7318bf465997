"""fp64 numpy oracle of FourierAttention's compression and decode steps.

TEST INFRASTRUCTURE ONLY: never imported by the product path.

Notation (paper, Section 3.3):
  K, V            per-head caches of shape [L, d]
  L_init, L_local sink and recent-window lengths (Eq. 1)
  D^kc, D^ku ...  compressed / kept head-dimension index sets (Eq. 2)
  F               real Fourier compression matrix (Eq. 4)
  K^mc, V^mc      fixed-length coefficient states (Eq. 3, updated by Eq. 5)
  K~, V~          reconstructed caches used for attention (Eq. 6)

Readings of the paper taken here (each is listed in the design notes):
  * The basis index is relative to the compressed segment: the first
    compressed token sits at position t0 (0 for a fresh segment).
  * Eq. 4 lists 2k rows of which row 1 (sine of order 0) is identically zero.
    `M` counts the live functions of the ordered system
        1, cos(w t), sin(w t), cos(2 w t), sin(2 w t), ...   (w = 2 pi / T)
    so the paper's k complex orders correspond to M = 2k - 1.
  * Coefficients are the plain inner products of Eq. 3 (no normalisation), so
    Eq. 5's rank-one update is literally `+=`.  The `1/k` in Eq. 6 is replaced
    by the inverse squared norm of each basis function over one period,
        w_m = 1/T for the constant (and the Nyquist cosine when 2n = T),
        w_m = 2/T otherwise,
    which makes compress->reconstruct the orthogonal projector onto the kept
    band whenever the segment spans exactly one period.
  * Eq. 6's V line reuses K^mc; that is read as V^mc.
  * softmax scale defaults to 1/sqrt(d); query head i attends KV head
    i // (Hq/Hkv); a single decode query sees every cached token.

All arithmetic is float64.  Phases are reduced in exact integer arithmetic
before the trigonometric call so that large order*position products lose
nothing.
"""

from __future__ import annotations

import numpy as np

__all__ = [
    "basis_matrix",
    "basis_weights",
    "compress_segment",
    "reconstruct_segment",
    "attend",
    "decode_head_group",
    "compress_batched",
    "decode_batched",
    "decode_varlen",
    "append_token",
    "reconstruction_mse",
    "select_dims",
    "decode_multi_query",
]


def _orders(M: int) -> np.ndarray:
    """Harmonic order n of basis function m: 0, 1, 1, 2, 2, 3, 3, ..."""
    m = np.arange(M, dtype=np.int64)
    return (m + 1) // 2


def basis_matrix(M: int, T: int, t0: int, N: int) -> np.ndarray:
    """Phi[j, m] = m-th real Fourier basis function at position t0 + j.

    Eq. 4 (transposed: rows are positions, columns are basis functions), with
    the identically-zero sine of order 0 dropped.  Column 0 is the constant;
    odd columns are cosines and even columns (> 0) sines of order (m+1)//2.
    """
    if not (1 <= M <= T):
        raise ValueError("need 1 <= M <= T")
    if t0 < 0 or N < 0 or t0 + N > T:
        raise ValueError("need 0 <= t0 and t0 + N <= T")
    pos = t0 + np.arange(N, dtype=np.int64)
    n = _orders(M)
    r = (pos[:, None] * n[None, :]) % T          # exact integer phase, [N, M]
    ang = (2.0 * np.pi / T) * r.astype(np.float64)
    m = np.arange(M)
    phi = np.where((m % 2 == 1)[None, :], np.cos(ang), np.sin(ang))
    phi[:, 0] = 1.0
    return phi


def basis_weights(M: int, T: int) -> np.ndarray:
    """w[m] = 1 / (sum over one period of phi_m^2).

    Replaces the 1/k factor of Eq. 6 (see module docstring).
    """
    n = _orders(M)
    w = np.full(M, 2.0 / T)
    w[(n == 0) | (2 * n == T)] = 1.0 / T
    return w


def _split_dims(mask: np.ndarray):
    mask = np.asarray(mask).astype(bool)
    return np.flatnonzero(mask), np.flatnonzero(~mask)


def compress_segment(X, mask, M: int, T: int, t0: int = 0, C_prev=None):
    """Eq. 2-3 (and Eq. 5 when C_prev is given) for one head.

    X     [N, d]  rows L_init .. L-L_local of K (or V)
    mask  [d]     1 = dimension is compressed
    Returns (C [M, |Dc|], X_keep [N, d-|Dc|]); columns in ascending dim order.
    """
    X = np.asarray(X, dtype=np.float64)
    idx_c, idx_u = _split_dims(mask)
    N = X.shape[0]
    phi = basis_matrix(M, T, t0, N)              # [N, M]
    C = phi.T @ X[:, idx_c]                      # F K^mn
    if C_prev is not None:
        C = np.asarray(C_prev, dtype=np.float64) + C
    return C, X[:, idx_u].copy()


def reconstruct_segment(C, X_keep, mask, T: int, t0: int, N: int) -> np.ndarray:
    """Eq. 6, first and third lines: rebuild the [N, d] middle segment."""
    C = np.asarray(C, dtype=np.float64)
    idx_c, idx_u = _split_dims(mask)
    d = len(idx_c) + len(idx_u)
    M = C.shape[0]
    phi = basis_matrix(M, T, t0, N)
    w = basis_weights(M, T)
    Xr = np.empty((N, d), dtype=np.float64)
    Xr[:, idx_c] = phi @ (w[:, None] * C)        # weighted F^T K^mc
    Xr[:, idx_u] = np.asarray(X_keep, dtype=np.float64).reshape(N, len(idx_u))
    return Xr


def attend(q, K, V, scale: float) -> np.ndarray:
    """softmax(scale * K q) V for one query vector: plain attention."""
    s = scale * (K @ q)
    s = s - np.max(s)
    p = np.exp(s)
    p = p / np.sum(p)
    return p @ V


def decode_head_group(q, Ck, kmask, Cv, vmask, T, t0, N,
                      k_keep, v_keep, k_full, v_full, scale=None) -> np.ndarray:
    """Eq. 6 for one KV head and the G query heads that share it.

    q       [G, d]
    Ck, Cv  [M, |Dkc|], [M, |Dvc|]
    k_keep  [N, d-|Dkc|], v_keep [N, d-|Dvc|]
    k_full  [W, d], v_full [W, d]   sink rows then window rows
    Returns out [G, d].
    """
    q = np.asarray(q, dtype=np.float64)
    d = q.shape[1]
    if scale is None or scale <= 0:
        scale = 1.0 / np.sqrt(d)
    Km = reconstruct_segment(Ck, k_keep, kmask, T, t0, N)
    Vm = reconstruct_segment(Cv, v_keep, vmask, T, t0, N)
    Kt = np.concatenate([np.asarray(k_full, np.float64).reshape(-1, d), Km], axis=0)
    Vt = np.concatenate([np.asarray(v_full, np.float64).reshape(-1, d), Vm], axis=0)
    return np.stack([attend(q[g], Kt, Vt, scale) for g in range(q.shape[0])])


def compress_batched(X, masks, M, T, t0=0, C_prev=None):
    """compress_segment over [B, H]: X [B,H,N,d], masks [B,H,d]."""
    X = np.asarray(X)
    B, H, N, d = X.shape
    Dc = int(np.asarray(masks[0, 0]).astype(bool).sum())
    C = np.empty((B, H, M, Dc))
    Xk = np.empty((B, H, N, d - Dc))
    for b in range(B):
        for h in range(H):
            prev = None if C_prev is None else C_prev[b, h]
            C[b, h], Xk[b, h] = compress_segment(X[b, h], masks[b, h], M, T, t0, prev)
    return C, Xk


def decode_batched(q, Ck, kmask, Cv, vmask, T, t0, N,
                   k_keep, v_keep, k_full, v_full, scale=None):
    """decode_head_group over [B, Hkv]; q [B,Hq,d] -> out [B,Hq,d]."""
    q = np.asarray(q, dtype=np.float64)
    B, Hq, d = q.shape
    Hkv = np.asarray(kmask).shape[1]
    G = Hq // Hkv
    out = np.empty((B, Hq, d))
    for b in range(B):
        for h in range(Hkv):
            out[b, h * G:(h + 1) * G] = decode_head_group(
                q[b, h * G:(h + 1) * G], Ck[b, h], kmask[b, h], Cv[b, h], vmask[b, h],
                T, t0, N, k_keep[b, h], v_keep[b, h], k_full[b, h], v_full[b, h], scale)
    return out


def decode_varlen(q, Ck, kmask, Cv, vmask, T, t0, seq_n, k_keep, v_keep, k_full, v_full, seq_w, scale=None):
    """Eq. 6 for a batch whose sequences stand at different positions: sequence b has seq_n[b]
    middle rows (the first seq_n[b] rows of its k_keep / v_keep, and coefficient states that hold
    exactly those tokens) and seq_w[b] full-width rows (the first seq_w[b] rows of k_full /
    v_full).  Every sequence is one decode_head_group call on its own rows: nothing of a longer
    neighbour is visible to it.  A sequence without any row has no softmax; its output is zero.
    q [B,Hq,d] -> out [B,Hq,d]."""
    q = np.asarray(q, dtype=np.float64)
    B, Hq, d = q.shape
    Hkv = np.asarray(kmask).shape[1]
    G = Hq // Hkv
    out = np.zeros((B, Hq, d))
    for b in range(B):
        n, w = int(seq_n[b]), int(seq_w[b])
        if n + w == 0:
            continue
        for h in range(Hkv):
            out[b, h * G:(h + 1) * G] = decode_head_group(
                q[b, h * G:(h + 1) * G], Ck[b, h], kmask[b, h], Cv[b, h], vmask[b, h], T, t0, n,
                np.asarray(k_keep[b, h])[:n], np.asarray(v_keep[b, h])[:n],
                np.asarray(k_full[b, h])[:w], np.asarray(v_full[b, h])[:w], scale)
    return out


def append_token(Ck, Cv, kmask, vmask, k_keep, v_keep, k_full, v_full, slot: int, k_new, v_new,
                 T: int, n_mid: int, evict: bool):
    """One decode step of cache maintenance for one KV head (Eq. 5 and the window of Eq. 1).

    The recent window lives in rows of k_full / v_full (their order never matters to Eq. 6);
    `slot` is the row that holds the oldest window token.  With `evict`, that token leaves the
    window and becomes middle token number n_mid: its compressed dims are folded into the
    coefficient states by the rank-one update of Eq. 5 (the basis column taken at the token's own
    position n_mid), its kept dims are appended to K^mu / V^mu.  The new token then takes the row.

    Returns new (Ck, Cv, k_keep, v_keep, k_full, v_full); nothing is modified in place.
    """
    Ck = np.asarray(Ck, dtype=np.float64)
    Cv = np.asarray(Cv, dtype=np.float64)
    k_keep = np.asarray(k_keep, dtype=np.float64)
    v_keep = np.asarray(v_keep, dtype=np.float64)
    k_full = np.array(k_full, dtype=np.float64, copy=True)
    v_full = np.array(v_full, dtype=np.float64, copy=True)
    if evict:
        Ck, ku = compress_segment(k_full[slot][None, :], kmask, Ck.shape[0], T, n_mid, C_prev=Ck)
        Cv, vu = compress_segment(v_full[slot][None, :], vmask, Cv.shape[0], T, n_mid, C_prev=Cv)
        k_keep = np.concatenate([k_keep.reshape(-1, ku.shape[1]), ku], axis=0)
        v_keep = np.concatenate([v_keep.reshape(-1, vu.shape[1]), vu], axis=0)
    k_full[slot] = np.asarray(k_new, dtype=np.float64)
    v_full[slot] = np.asarray(v_new, dtype=np.float64)
    return Ck, Cv, k_keep, v_keep, k_full, v_full


def reconstruction_mse(X, M: int) -> np.ndarray:
    """Section 3.4: per head dimension, the mean squared error of compressing the
    whole segment onto the first M basis functions and rebuilding it (Eq. 3 then
    Eq. 6), with the segment spanning exactly one period (T = N, t0 = 0).

    X [N, d] -> mse [d].  Written as the definition: compress every dim, rebuild
    every row, subtract.
    """
    X = np.asarray(X, dtype=np.float64)
    N, d = X.shape
    ones = np.ones(d, dtype=np.uint8)
    C, keep = compress_segment(X, ones, M, N, 0)
    Xr = reconstruct_segment(C, keep, ones, N, 0, N)
    return np.mean((X - Xr) ** 2, axis=0)


def select_dims(X, M: int, Dc: int):
    """Section 3.4: the Dc head dimensions with the lowest reconstruction error are
    the ones to compress.  Equal errors go to the lower dimension index.

    Returns (mask uint8 [d] with Dc ones, mse [d]).
    """
    mse = reconstruction_mse(X, M)
    order = np.argsort(mse, kind="stable")
    mask = np.zeros(mse.shape[0], dtype=np.uint8)
    mask[order[:Dc]] = 1
    return mask, mse


def decode_multi_query(q, Ck, kmask, Cv, vmask, T, t0, N,
                       k_keep, v_keep, k_full, v_full, scale=None) -> np.ndarray:
    """Eq. 6 for Tq consecutive query tokens of one KV head (chunked decoding / verification of
    drafted tokens, the FlashAttention side of Section 3.3's kernel).

    q [Tq, G, d].  The last Tq rows of k_full / v_full are the Tq new tokens in order; query t sees
    every other row and the new tokens 0 .. t (causal among the new tokens, everything older is
    visible to all).  Returns out [Tq, G, d]: each query is an ordinary single-query decode over
    the rows it may see.
    """
    q = np.asarray(q, dtype=np.float64)
    Tq = q.shape[0]
    k_full = np.asarray(k_full, np.float64)
    v_full = np.asarray(v_full, np.float64)
    W = k_full.shape[0]
    if Tq < 1 or Tq > W:
        raise ValueError("need 1 <= Tq <= number of full-width rows")
    out = []
    for t in range(Tq):
        vis = W - Tq + t + 1
        out.append(decode_head_group(q[t], Ck, kmask, Cv, vmask, T, t0, N, k_keep, v_keep,
                                     k_full[:vis], v_full[:vis], scale))
    return np.stack(out)

