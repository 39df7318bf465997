"""Seeded synthetic KV caches with the signal structure the paper describes.

The paper's workloads are LLaMA KV caches on long prompts; neither the models
nor the prompts are available, so these inputs stand in for them.  They take
the paper's shapes (GQA / MHA head layouts, 4 sink tokens, a recent window of
about a thousand tokens, 75-88 % of head dimensions compressed) and its
qualitative observation that compressible dimensions vary smoothly in time
(Section 3.4) while the others do not.

Recipe (per sequence and KV head, K and V drawn independently):
  * masks: a uniformly random subset of `Dc` of the `D` dims, seed 2000+index;
  * a compressed dim at context position t (sink, middle and window alike):
        x(t) = sum_{r<3} a_r cos(2 pi n_r (t - Li) / T + psi_r) + eps_t
    with n_r integer uniform in [1, max(1, (M-1)//2)], a_r ~ U(0.5, 1.5),
    psi_r ~ U(0, 2 pi), eps ~ N(0, 0.1^2);
  * every other K/V entry and q ~ N(0, 1), seed 1000+index;
  * values are rounded to the config's dtype on the host, so that both the
    oracle and the GPU path see identical bits.

Nothing here evaluates the method's basis, projection or attention.
"""

from __future__ import annotations

import numpy as np


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bfloat16 (nearest-even) and return the uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array holding exactly the bfloat16-representable roundings of x."""
    bits = bf16_bits(x).astype(np.uint32) << np.uint32(16)
    return bits.view(np.float32).reshape(np.shape(x))


def _round(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.asarray(x, dtype=np.float32)
    return round_to_bf16(x) if dtype == "bf16" else x


def make_masks(cfg):
    """(kmask, vmask): uint8 [B, Hkv, D], exactly Dkc / Dvc ones per row."""
    rng = np.random.default_rng(2000 + cfg.index)

    def draw(Dc):
        m = np.zeros((cfg.B, cfg.Hkv, cfg.D), dtype=np.uint8)
        for b in range(cfg.B):
            for h in range(cfg.Hkv):
                m[b, h, rng.choice(cfg.D, size=Dc, replace=False)] = 1
        return m

    return draw(cfg.Dkc), draw(cfg.Dvc)


def _cache(cfg, rng, mask, Dc):
    """One K or V cache [B, Hkv, L, D] (fp32) following the recipe above."""
    L, T = cfg.L, cfg.T
    out = np.empty((cfg.B, cfg.Hkv, L, cfg.D), dtype=np.float32)
    j = (np.arange(L, dtype=np.float64) - cfg.Li)[:, None]            # [L, 1]
    n_hi = max(1, (cfg.M - 1) // 2)
    for b in range(cfg.B):
        for h in range(cfg.Hkv):
            x = rng.standard_normal((L, cfg.D), dtype=np.float32)
            if Dc:
                idx = np.flatnonzero(mask[b, h])
                n_r = rng.integers(1, n_hi + 1, size=(3, Dc)).astype(np.float64)
                a_r = rng.uniform(0.5, 1.5, size=(3, Dc))
                psi = rng.uniform(0.0, 2.0 * np.pi, size=(3, Dc))
                sig = np.zeros((L, Dc))
                for r in range(3):
                    sig += a_r[r] * np.cos((2.0 * np.pi / T) * j * n_r[r] + psi[r])
                sig += 0.1 * rng.standard_normal((L, Dc))
                x[:, idx] = sig.astype(np.float32)
            out[b, h] = x
    return out


def make_context(cfg):
    """Synthetic decode-step state for `cfg`.

    Returns a dict of fp32 numpy arrays already rounded to cfg.dtype:
      q       [B, Hq, D]
      k_mid   [B, Hkv, N, D]   rows Li .. Li+N of K (what gets compressed)
      v_mid   [B, Hkv, N, D]
      k_full  [B, Hkv, W, D]   sink rows followed by recent-window rows
      v_full  [B, Hkv, W, D]
      kmask, vmask  uint8 [B, Hkv, D]
    """
    kmask, vmask = make_masks(cfg)
    rng = np.random.default_rng(1000 + cfg.index)
    K = _round(_cache(cfg, rng, kmask, cfg.Dkc), cfg.dtype)
    V = _round(_cache(cfg, rng, vmask, cfg.Dvc), cfg.dtype)
    q = _round(rng.standard_normal((cfg.B, cfg.Hq, cfg.D), dtype=np.float32), cfg.dtype)
    Li, N = cfg.Li, cfg.N
    sel_full = np.r_[0:Li, Li + N:cfg.L]
    return {
        "q": q,
        "k_mid": np.ascontiguousarray(K[:, :, Li:Li + N]),
        "v_mid": np.ascontiguousarray(V[:, :, Li:Li + N]),
        "k_full": np.ascontiguousarray(K[:, :, sel_full]),
        "v_full": np.ascontiguousarray(V[:, :, sel_full]),
        "kmask": kmask,
        "vmask": vmask,
    }


def rel_err(got, want, floor: float = 0.0) -> float:
    """max |got - want| / max |want| over one tensor: the parity metric.

    Elementwise relative error is meaningless for entries that are ~0
    (out-of-band coefficients, near-cancelling outputs), so the error is
    normalised by the largest magnitude of the reference tensor.  `floor`
    bounds the denominator from below for tensors that are small only through
    cancellation (e.g. a band that misses every component of the signal).
    """
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    denom = max(float(np.max(np.abs(want))) if want.size else 0.0, float(floor))
    if denom == 0.0:
        return float(np.max(np.abs(got))) if got.size else 0.0
    return float(np.max(np.abs(got - want)) / denom)
