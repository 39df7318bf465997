"""Host-side checks of the synthetic input generators (no method arithmetic)."""

import numpy as np
import torch

from workloads import CONFIGS, get_config, make_context, make_masks, round_to_bf16, bf16_bits, small_variants


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(10000) * 10.0 ** rng.integers(-6, 6, 10000)).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(round_to_bf16(x), want.float().numpy())
    assert np.array_equal(bf16_bits(x), want.view(torch.int16).numpy().view(np.uint16))


def test_masks_have_exact_popcount_and_differ():
    cfg = get_config(3)
    km, vm = make_masks(cfg)
    assert km.shape == (cfg.B, cfg.Hkv, cfg.D)
    assert (km.sum(-1) == cfg.Dkc).all() and (vm.sum(-1) == cfg.Dvc).all()
    assert not np.array_equal(km[0, 0], km[1, 0])
    assert not np.array_equal(km, vm)


def test_context_shapes_dtype_and_determinism():
    for cfg in small_variants():
        a = make_context(cfg)
        b = make_context(cfg)
        assert a["q"].shape == (cfg.B, cfg.Hq, cfg.D)
        assert a["k_mid"].shape == (cfg.B, cfg.Hkv, cfg.N, cfg.D)
        assert a["v_full"].shape == (cfg.B, cfg.Hkv, cfg.W, cfg.D)
        for key in a:
            assert np.array_equal(a[key], b[key]), key
        if cfg.dtype == "bf16":
            for key in ("q", "k_mid", "v_mid", "k_full", "v_full"):
                assert np.array_equal(a[key], round_to_bf16(a[key])), key


def test_config_table_matches_stated_sizes():
    c2, c3, c4, c5 = (get_config(i) for i in (2, 3, 4, 5))
    assert (c2.L, c3.L, c4.L) == (32768, 8192, 131072)
    assert c5.N == 4096 and c5.W == 516
    assert abs(c2.decode_bytes() / 1e6 - 38.3) < 0.2
    assert abs(c3.decode_bytes() / 1e6 - 172.6) < 0.5
    assert abs(c4.decode_bytes() / 1e6 - 78.2) < 0.3
    assert abs(c5.decode_bytes() / 1e6 - 252.4) < 0.5
    assert abs(2 * c5.compress_flops(96) / 1e9 - 103.1) < 0.2
    assert len(CONFIGS) == 5


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU's share only: any other count exits with a message, before touching a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and not r.stdout.strip()
