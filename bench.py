#!/usr/bin/env python3
"""Benchmark of the FourierAttention hot path on one MI355X.

A step is one pass of the whole path on one synthetic batch that is already
resident in HBM: fa_compress(K), fa_compress(V), fa_decode.  The headline
value is context tokens per second over that step (B * L / t_step); the
decode-only and compress-only rates and their rooflines are reported beside
it.  Inputs rotate over enough distinct buffer sets that consecutive steps
cannot be served from the 256 MB last-level cache.

Prints ONE JSON line on stdout.
"""

from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "Fourier-KV decode context tokens/s/GPU + achieved HBM GB/s (% of peak)"
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch from hardware counters (FETCH_SIZE + WRITE_SIZE, each scaled by what the
# same counter reads for the --copy-probe kernel), keyed by (kernel, config index).
# Source: profiles/bench_cfg*_hbm_traffic.txt; null for anything not measured there.
MEASURED_TRAFFIC = {
    # compress_project = the K | V pair launch (both tensors); cfg2: 130.3 MB read + 81.3 MB written,
    # 48.8 MB of it chunk partials
    ("compress_project", 2): 211520000, ("decode_partial", 2): 39270000,
    ("compress_project", 3): 654170000, ("decode_partial", 3): 165390000,
    ("compress_project", 4): 660390000, ("decode_partial", 4): 80510000,   # M = 512: X is read by two row blocks
    ("compress_project", 5): 721580000, ("decode_partial", 5): 205500000,
}
MFMA_BF16_PEAK_TFLOPS = 2500.0
FP32_MATRIX_PEAK_TFLOPS = 157.3
LLC_BYTES = 256 << 20


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="2", help="config index (1-5) or name")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch a converting copy of known size (bf16 -> fp32, 64 MiB read, "
                         "128 MiB written) three times: the yardstick that HBM counter runs are scaled by")
    ap.add_argument("--extras", action="store_true",
                    help="also time the calls outside the step: fa_append (one token per sequence and KV head) "
                         "and fa_select_dims (the K segment) -> phases.append / phases.select")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (one GPU's share of the path at its "
              "real shape); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2506_11886_amd as fa
    from workloads import get_config, make_context

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = get_config(args.workload)
    dt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    ctx = make_context(cfg)

    def dev(a):
        t = torch.from_numpy(a)
        return (t.to(dt) if t.dtype == torch.float32 else t).cuda()

    B, Hq, Hkv, D, N, W, M, T = cfg.B, cfg.Hq, cfg.Hkv, cfg.D, cfg.N, cfg.W, cfg.M, cfg.T
    Dku, Dvu = D - cfg.Dkc, D - cfg.Dvc
    dec_bytes = cfg.decode_bytes()
    cmp_bytes = cfg.compress_bytes(cfg.Dkc) + cfg.compress_bytes(cfg.Dvc)
    cmp_flops = cfg.compress_flops(cfg.Dkc) + cfg.compress_flops(cfg.Dvc)
    n_sets = int(min(16, max(2, math.ceil(2.0 * LLC_BYTES / dec_bytes))))

    master = {k: dev(ctx[k]) for k in ("q", "k_mid", "v_mid", "k_full", "v_full", "kmask", "vmask")}
    sets = []
    for _ in range(n_sets):
        s = {k: v.clone() for k, v in master.items()}
        s["ck"] = torch.empty((B, Hkv, M, cfg.Dkc), dtype=torch.float32, device="cuda")
        s["cv"] = torch.empty((B, Hkv, M, cfg.Dvc), dtype=torch.float32, device="cuda")
        s["kk"] = torch.empty((B, Hkv, N, fa.keep_rows_pitch(Dku)), dtype=dt, device="cuda")
        s["vk"] = torch.zeros((B, Hkv, fa.tok8_numel(N, Dvu)), dtype=dt, device="cuda")
        s["out"] = torch.empty((B, Hq, D), dtype=torch.float32, device="cuda")
        sets.append(s)
    ws_c = torch.empty(max(256, fa.compress_kv_workspace_bytes(B, Hkv, N, D, cfg.Dkc, cfg.Dvc, M)),
                       dtype=torch.uint8, device="cuda")
    ws_d = torch.empty(max(256, fa.decode_workspace_bytes(B, Hq, Hkv, D, cfg.Dkc, cfg.Dvc, M, N, W,
                                                          cfg.num_splits)),
                       dtype=torch.uint8, device="cuda")

    def compress(s, kms=None):   # K and V of the same tokens: one call (one projection launch when both qualify)
        fa.fa_compress_kv(s["k_mid"], s["v_mid"], s["kmask"], s["vmask"], cfg.Dkc, cfg.Dvc, M, T, ck=s["ck"],
                          cv=s["cv"], k_keep=s["kk"], v_keep=s["vk"], workspace=ws_c, kernel_ms=kms)

    def decode(s, kms=None):
        fa.fa_decode(s["q"], s["ck"], s["kmask"], s["cv"], s["vmask"], M, T, 0, N, s["kk"], s["vk"],
                     s["k_full"], s["v_full"], num_splits=cfg.num_splits, out=s["out"],
                     workspace=ws_d, kernel_ms=kms)

    def step(i):
        s = sets[i % n_sets]
        compress(s)
        decode(s)

    def timed_loop(fn, steps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    for s in sets:               # every set holds valid coefficients before decode-only timing
        compress(s)
    for i in range(args.warmup):
        step(i)
    t_step = timed_loop(step, args.steps)
    t_dec = timed_loop(lambda i: decode(sets[i % n_sets]), args.steps)
    t_cmp = timed_loop(lambda i: compress(sets[i % n_sets]), args.steps)

    # per-kernel durations from HIP events recorded around each kernel on the launch stream
    reps = max(4, min(args.steps, 40))
    kd, kc = [], []
    for i in range(reps):
        decode(sets[i % n_sets], kd)
        compress(sets[i % n_sets], kc)
    kd = np.array(kd).reshape(reps, 3).mean(0) * 1e-3        # prepare, partial, finish [s]
    kc = np.array(kc).reshape(reps, 2).mean(0) * 1e-3        # [projection of K and V, their reductions] [s]
    t_partial = float(kd[1])
    t_project = float(kc[0])                                   # K and V projections together

    def roof_hbm(bytes_, t, kernel):
        a = bytes_ / t / 1e9
        return {"kernel": kernel, "bound": "hbm", "achieved": round(a, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(a / HBM_PEAK_GBS, 4),
                "traffic": MEASURED_TRAFFIC.get((kernel, cfg.index))}

    mm_peak = MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else FP32_MATRIX_PEAK_TFLOPS
    roof_dec = roof_hbm(dec_bytes, t_partial, "decode_partial")
    # compress: the binding roof is whichever ideal time is longer for this workload
    if cmp_bytes / (HBM_PEAK_GBS * 1e9) >= cmp_flops / (mm_peak * 1e12):
        roof_cmp = roof_hbm(cmp_bytes, t_project, "compress_project")
    else:
        a = cmp_flops / t_project / 1e12
        roof_cmp = {"kernel": "compress_project", "bound": "mfma", "achieved": round(a, 1),
                    "peak": mm_peak, "unit": "TFLOP/s", "frac": round(a / mm_peak, 4),
                    "traffic": MEASURED_TRAFFIC.get(("compress_project", cfg.index))}
    roof_cmp["launches_per_step"] = 1       # K and V in one launch; achieved = bytes (flop) of both / its duration
    roof_cmp["mfma_tflops"] = round(cmp_flops / t_project / 1e12, 1)
    roof_cmp["mfma_frac"] = round(cmp_flops / t_project / 1e12 / mm_peak, 4)
    dominant = roof_cmp if t_project > t_partial else roof_dec

    result = {
        "metric": METRIC,
        "value": round(B * cfg.L / t_step, 1),
        "unit": "context tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(t_step * 1e3, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {
            "workload": f"cfg{cfg.index} {cfg.name}: B={B} Hq={Hq} Hkv={Hkv} D={D} L={cfg.L} "
                        f"(sink {cfg.Li} + middle {N} + window {cfg.Lw}) Dkc={cfg.Dkc} Dvc={cfg.Dvc} M={M}",
            "step": "fa_compress_kv(K, V) + fa_decode",
            "buffer_sets": n_sets,
        },
        "roofline": dominant,
        "phases": {
            "decode": {"ms": round(t_dec * 1e3, 5), "context_tokens_per_s": round(B * cfg.L / t_dec, 1),
                       "algorithmic_bytes": dec_bytes,
                       "call_GBps": round(dec_bytes / t_dec / 1e9, 1),
                       "kernel_ms": {"prepare": round(float(kd[0]) * 1e3, 5),
                                     "partial": round(float(kd[1]) * 1e3, 5),
                                     "finish": round(float(kd[2]) * 1e3, 5)},
                       "roofline": roof_dec},
            "compress": {"ms": round(t_cmp * 1e3, 5), "tokens_per_s": round(B * N / t_cmp, 1),
                         "algorithmic_bytes": cmp_bytes, "flop": cmp_flops,
                         "kernel_ms": {"project_kv": round(float(kc[0]) * 1e3, 5),
                                       "reduce_kv": round(float(kc[1]) * 1e3, 5)},
                         "roofline": roof_cmp},
        },
    }

    if args.extras:
        s0 = sets[0]
        k_new = torch.randn((B, Hkv, D), device="cuda").to(dt)
        v_new = torch.randn((B, Hkv, D), device="cuda").to(dt)
        kk_ap = torch.zeros((B, Hkv, N + 64, fa.keep_rows_pitch(Dku)), dtype=dt, device="cuda")
        vk_ap = torch.zeros((B, Hkv, fa.tok8_numel(N + 64, Dvu)), dtype=dt, device="cuda")
        T_ap = T + 64

        def append(i):   # evicting appends at successive middle positions (the state drifts: timing only)
            fa.fa_append(k_new, v_new, s0["k_full"], s0["v_full"], cfg.Li + i % max(cfg.Lw, 1), cfg.Lw > 0,
                         s0["kmask"], s0["vmask"], M, T_ap, N + i % 64, s0["ck"], s0["cv"], kk_ap, vk_ap)
        if W > 0:
            for i in range(8):
                append(i)
            t_app = timed_loop(append, min(args.steps, 64))
            app_bytes = B * Hkv * (2 * M * (cfg.Dkc + cfg.Dvc) * 4 + 4 * D * (2 if dt == torch.bfloat16 else 4))
            result["phases"]["append"] = {"ms": round(t_app * 1e3, 5), "algorithmic_bytes": app_bytes,
                                          "GBps": round(app_bytes / t_app / 1e9, 1)}
        Tq = max(1, 16 // (Hq // Hkv))
        if Tq > 1 and W >= Tq:   # as many query tokens per step as the group limit allows
            q_mq = torch.randn((B, Hkv, Tq, Hq // Hkv, D), device="cuda").to(dt)
            out_mq = torch.empty((B, Hkv, Tq, Hq // Hkv, D), dtype=torch.float32, device="cuda")
            ws_mq = torch.empty(max(256, fa.decode_workspace_bytes(B, Hq * Tq, Hkv, D, cfg.Dkc, cfg.Dvc, M, N, W,
                                                                   cfg.num_splits)), dtype=torch.uint8, device="cuda")

            def decode_mq(i):
                s = sets[i % n_sets]
                fa.fa_decode_mq(q_mq, s["ck"], s["kmask"], s["cv"], s["vmask"], M, T, 0, N, s["kk"], s["vk"],
                                s["k_full"], s["v_full"], num_splits=cfg.num_splits, out=out_mq, workspace=ws_mq)
            for i in range(4):
                decode_mq(i)
            t_mq = timed_loop(decode_mq, args.steps)
            result["phases"]["decode_mq"] = {"query_tokens": Tq, "ms": round(t_mq * 1e3, 5),
                                             "ms_per_query_token": round(t_mq * 1e3 / Tq, 5),
                                             "call_GBps": round(dec_bytes / t_mq / 1e9, 1)}
        if N >= M:
            ws_s = torch.empty(max(256, fa.select_workspace_bytes(fa.FA_BF16 if dt == torch.bfloat16 else fa.FA_F32,
                                                                  B, Hkv, N, D, M)), dtype=torch.uint8, device="cuda")
            sel = lambda i: fa.fa_select_dims(sets[i % n_sets]["k_mid"], M, cfg.Dkc, workspace=ws_s)
            for i in range(2):
                sel(i)
            t_sel = timed_loop(sel, max(4, min(args.steps, 20)))
            sel_flop = 2.0 * B * Hkv * N * M * D
            result["phases"]["select"] = {"ms": round(t_sel * 1e3, 5), "flop": sel_flop,
                                          "fp32_matrix_tflops": round(sel_flop / t_sel / 1e12, 1),
                                          "fp32_matrix_frac": round(sel_flop / t_sel / 1e12 / FP32_MATRIX_PEAK_TFLOPS, 4)}

    if args.copy_probe:
        src = torch.ones(32 << 20, dtype=torch.bfloat16, device="cuda")
        dst = torch.empty(32 << 20, dtype=torch.float32, device="cuda")
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        result["copy_probe"] = {"read_bytes": src.numel() * 2, "written_bytes": dst.numel() * 4, "launches": 3}

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, ctx, args.cpu_seconds)
    print(json.dumps(result), flush=True)


def cpu_baseline(cfg, ctx, budget_s):
    """The fp64 oracle, as it stands, on a bounded sample of (sequence, KV head)
    pairs of the same workload: compress K, compress V, decode."""
    import numpy as np
    import oracle.fourier_kv as fk
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    heads = [(b, h) for b in range(cfg.B) for h in range(cfg.Hkv)]
    G = cfg.G
    done, t_used = 0, 0.0
    for b, h in heads:
        t0 = time.perf_counter()
        ck, kk = fk.compress_segment(ctx["k_mid"][b, h], ctx["kmask"][b, h], cfg.M, cfg.T, 0)
        cv, vk = fk.compress_segment(ctx["v_mid"][b, h], ctx["vmask"][b, h], cfg.M, cfg.T, 0)
        fk.decode_head_group(ctx["q"][b, h * G:(h + 1) * G], ck, ctx["kmask"][b, h], cv, ctx["vmask"][b, h],
                             cfg.T, 0, cfg.N, kk, vk, ctx["k_full"][b, h], ctx["v_full"][b, h])
        t_used += time.perf_counter() - t0
        done += 1
        if t_used + t_used / done > budget_s:
            break
    tokens = cfg.B * cfg.L * done / len(heads)
    return {"value": round(tokens / t_used, 1), "unit": "context tokens/s", "cores": int(cores),
            "kind": "oracle",
            "sample": f"{done} of {len(heads)} (sequence, KV head) pairs of the same workload, "
                      f"compress K + compress V + decode, {t_used:.1f} s wall"}


if __name__ == "__main__":
    main()
