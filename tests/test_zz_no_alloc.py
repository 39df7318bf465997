"""fa_decode_static: the entry point that allocates nothing (split-K state in the library's static
device array) against fa_decode with a caller workspace, through the C ABI.  Collected last: the file
name sorts after every other test file."""

import numpy as np
import pytest
import torch

from workloads import small_variants
from fa_testlib import cached_context, oracle_state, rows_pad8, rows_to_tok8, sample_heads, to_dev

pytestmark = pytest.mark.gpu


def _inputs(cfg):
    ctx = cached_context(cfg)
    st = oracle_state(cfg, ctx, sample_heads(cfg, None))
    return (to_dev(ctx["q"], cfg), to_dev(st["ck32"]), to_dev(ctx["kmask"]), to_dev(st["cv32"]), to_dev(ctx["vmask"]),
            cfg.M, cfg.T, cfg.t0, cfg.N, to_dev(rows_pad8(st["kk"]), cfg), to_dev(rows_to_tok8(st["vk"]), cfg),
            to_dev(ctx["k_full"], cfg), to_dev(ctx["v_full"], cfg))


def test_static_scratch_decode_matches_workspace_decode_twice_in_a_row():
    """Two calls in a row on the same GPU, the second with a smaller input: the array keeps the first
    call's contents, and nothing of it may leak into the second result.  Same kernels, same launch
    configuration, so the results must be identical to fa_decode's bit for bit."""
    import paper_2506_11886_amd as fa
    small = {c.name: c for c in small_variants()}
    big, little = small["mha_ragged"], small["tiny_bf16"]
    for cfg in (big, little):
        print(f"[case] static scratch {cfg}", flush=True)
        args = _inputs(cfg)
        want = fa.fa_decode(*args, num_splits=cfg.num_splits)
        out = torch.full((cfg.B, cfg.Hq, cfg.D), float("nan"), dtype=torch.float32, device="cuda")
        before = torch.cuda.memory_allocated()
        fa.fa_decode_static(*args, num_splits=cfg.num_splits, out=out)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert torch.isfinite(out).all()
        assert torch.equal(out, want), (cfg.name, (out - want).abs().max().item())


def test_static_scratch_decode_in_the_one_launch_form():
    """The same two calls in a row on shapes that run as one launch (num_splits = 1): that form keeps all
    of its state in LDS, the static array is not even touched."""
    import paper_2506_11886_amd as fa
    from workloads import one_launch_variants
    shapes = one_launch_variants()
    for cfg in (shapes[0], shapes[4]):
        print(f"[case] static scratch, one launch {cfg}", flush=True)
        args = _inputs(cfg)
        want = fa.fa_decode(*args, num_splits=1)
        out = torch.full((cfg.B, cfg.Hq, cfg.D), float("nan"), dtype=torch.float32, device="cuda")
        before = torch.cuda.memory_allocated()
        fa.fa_decode_static(*args, num_splits=1, out=out)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert torch.isfinite(out).all()
        assert torch.equal(out, want), (cfg.name, (out - want).abs().max().item())
