"""Helpers shared by the GPU parity tests (no method arithmetic here)."""

from __future__ import annotations

import numpy as np
import torch

import oracle.fourier_kv as fk
from workloads import make_context


def torch_dtype(cfg):
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def to_dev(a: np.ndarray, cfg=None, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if t.dtype == torch.float32 and (cfg is not None or dtype is not None):
        t = t.to(dtype if dtype is not None else torch_dtype(cfg))
    return t.cuda()


def rows_to_tok8(x: np.ndarray) -> np.ndarray:
    """[..., n, Du] rows -> [..., ceil(n/8)*Du*8] token-interleaved-by-8 slab."""
    *lead, n, du = x.shape
    g = (n + 7) // 8
    pad = np.zeros((*lead, g * 8, du), dtype=x.dtype)
    pad[..., :n, :] = x
    return np.ascontiguousarray(pad.reshape(*lead, g, 8, du).swapaxes(-1, -2)).reshape(*lead, g * du * 8)


def rows_pad8(x: np.ndarray) -> np.ndarray:
    """[..., n, Du] rows -> [..., n, Du rounded up to 8] with zero pad columns."""
    *lead, n, du = x.shape
    pitch = (du + 7) // 8 * 8
    out = np.zeros((*lead, n, pitch), dtype=x.dtype)
    out[..., :du] = x
    return out


def oracle_state(cfg, ctx, heads=None):
    """Oracle compression of the middle segment.  `heads`: list of (b, hkv) to
    evaluate (others left as zeros), None = all.  Coefficients are rounded to
    fp32, which is what the decode step is handed."""
    B, H, N, D, M, T = cfg.B, cfg.Hkv, cfg.N, cfg.D, cfg.M, cfg.T
    ck = np.zeros((B, H, M, cfg.Dkc)); cv = np.zeros((B, H, M, cfg.Dvc))
    kk = np.zeros((B, H, N, D - cfg.Dkc), np.float32); vk = np.zeros((B, H, N, D - cfg.Dvc), np.float32)
    todo = heads if heads is not None else [(b, h) for b in range(B) for h in range(H)]
    for b, h in todo:
        c, k = fk.compress_segment(ctx["k_mid"][b, h], ctx["kmask"][b, h], M, T, cfg.t0)
        ck[b, h], kk[b, h] = c, k
        c, k = fk.compress_segment(ctx["v_mid"][b, h], ctx["vmask"][b, h], M, T, cfg.t0)
        cv[b, h], vk[b, h] = c, k
    return {"ck": ck, "cv": cv, "kk": kk, "vk": vk,
            "ck32": ck.astype(np.float32), "cv32": cv.astype(np.float32)}


def oracle_decode_heads(cfg, ctx, st, heads, from_f32_coeffs=True):
    """Oracle outputs for the listed (b, hkv): dict (b,h) -> [G, D]."""
    out = {}
    G = cfg.G
    for b, h in heads:
        ck = st["ck32"][b, h].astype(np.float64) if from_f32_coeffs else st["ck"][b, h]
        cv = st["cv32"][b, h].astype(np.float64) if from_f32_coeffs else st["cv"][b, h]
        out[(b, h)] = fk.decode_head_group(
            ctx["q"][b, h * G:(h + 1) * G], ck, ctx["kmask"][b, h], cv, ctx["vmask"][b, h],
            cfg.T, cfg.t0, cfg.N, st["kk"][b, h], st["vk"][b, h], ctx["k_full"][b, h], ctx["v_full"][b, h])
    return out


def sample_heads(cfg, k, seed=0):
    allh = [(b, h) for b in range(cfg.B) for h in range(cfg.Hkv)]
    if k is None or k >= len(allh):
        return allh
    rng = np.random.default_rng(seed)
    idx = sorted(rng.choice(len(allh), size=k, replace=False))
    return [allh[i] for i in idx]


def cached_context(cfg, _cache={}):
    key = (cfg.name, cfg.index)
    if key not in _cache:
        _cache.clear()  # keep at most one big context alive
        _cache[key] = make_context(cfg)
    return _cache[key]
