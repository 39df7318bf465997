#!/usr/bin/env python3
"""Benchmark of the FourierAttention hot path on one MI355X.

Headline (`value`): decode context tokens per second, B * L / t_decode, of one
`fa_decode` call (one layer, one new token per sequence) on the largest
configuration (cfg4: 131072 tokens of context).  `roofline` is that call
against the HBM peak: algorithmic bytes of the call over the summed durations
of its kernels, with the dominant kernel beside it.  A "step" of the timed loop
is one pass of the whole path on one synthetic batch that is already resident
in HBM - fa_compress_kv(K, V) then fa_decode - and `ms_per_step` is that; the
decode-only and compress-only loops are timed the same way and reported under
`phases`.  The other configurations (cfg2, cfg3, cfg5) are measured in the same
run with fewer steps and reported under `other_workloads`.  Inputs rotate over
enough distinct buffer sets that consecutive steps cannot be served from the
256 MB last-level cache.

Prints ONE JSON line on stdout.
"""

from __future__ import annotations

import argparse
import hashlib
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "Fourier-KV decode context tokens/s/GPU + achieved HBM GB/s (% of peak)"
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
FP32_MATRIX_PEAK_TFLOPS = 157.3
LLC_BYTES = 256 << 20
CSRC = os.path.join(ROOT, "paper_2506_11886_amd", "csrc")


def source_digest(*names):
    """Short digest of kernel sources: a counter summary under profiles/ is only quoted while the
    kernels it measured are the ones in the tree."""
    h = hashlib.sha256()
    for n in names:
        with open(os.path.join(CSRC, n), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(index):
    """HBM bytes per launch from the hardware-counter summary profiles/bench_cfg<index>_hbm_traffic.txt
    (FETCH_SIZE + WRITE_SIZE, each scaled by the copy probe): {kernel name prefix: bytes}.  Empty when
    the file is missing or was made from other kernel sources than the ones in the tree."""
    path = os.path.join(ROOT, "profiles", f"bench_cfg{index}_hbm_traffic.txt")
    try:
        text = open(path).read()
    except OSError:
        return {}
    m = re.search(r"kernel sources digest:\s*([0-9a-f]{16})", text)
    if not m or m.group(1) != source_digest("fa_decode.hip", "fa_compress.hip", "fa_common.hpp", "fa_mma.hpp"):
        return {}
    out = {}
    for line in text.splitlines():
        f = line.split()
        if len(f) >= 6 and re.match(r"(decode_|compress_)", f[0]):
            try:
                out[f[0].split("<")[0]] = out.get(f[0].split("<")[0], 0) + int(round(float(f[-1]) * 1e6))
            except ValueError:
                pass
    return out


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="4", help="config index (1-5) or name of the headline workload")
    ap.add_argument("--only", action="store_true", help="measure the headline workload only (no other_workloads)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch a converting copy of known size (bf16 -> fp32, 64 MiB read, "
                         "128 MiB written) three times: the yardstick that HBM counter runs are scaled by")
    ap.add_argument("--extras", action="store_true",
                    help="also time the calls outside the step: fa_append (one token per sequence and KV head), "
                         "fa_decode_mq and fa_select_dims (the K segment) -> phases.append / decode_mq / select")
    return ap.parse_args()


def timed_loop(torch, fn, steps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        fn(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def measure(cfg, steps, warmup, extras=False):
    """Time the path on one configuration; returns (result dict, context)."""
    import numpy as np
    import torch

    import paper_2506_11886_amd as fa
    from workloads import make_context

    dt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    ctx = make_context(cfg)

    def dev(a):
        t = torch.from_numpy(a)
        return (t.to(dt) if t.dtype == torch.float32 else t).cuda()

    B, Hq, Hkv, D, N, W, M, T = cfg.B, cfg.Hq, cfg.Hkv, cfg.D, cfg.N, cfg.W, cfg.M, cfg.T
    e = cfg.elem_bytes()
    Dku, Dvu = D - cfg.Dkc, D - cfg.Dvc
    dec_bytes = cfg.decode_bytes()
    cmp_bytes = cfg.compress_bytes(cfg.Dkc) + cfg.compress_bytes(cfg.Dvc)
    cmp_flops = cfg.compress_flops(cfg.Dkc) + cfg.compress_flops(cfg.Dvc)
    n_sets = int(min(16, max(2, math.ceil(2.0 * LLC_BYTES / dec_bytes))))
    # what each kernel of the decode call has to move (the split-K records between them are overhead)
    bh = B * Hkv
    # (with more than 256 series slots the full-width sink / window rows are processed in the launch that
    # forms the series coefficients, otherwise in the launch of the middle rows)
    full_rows = bh * W * D * 2 * e
    early = M > 257
    kb = {"prepare": bh * M * cfg.Dkc * 4 + B * Hq * D * e + bh * D + (full_rows if early else 0),
          "partial": bh * N * (Dku + Dvu) * e + B * Hq * D * e + (0 if early else full_rows),
          "finish": bh * M * cfg.Dvc * 4 + bh * D + B * Hq * D * 4}

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
    del master
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

    for s in sets:               # every set holds valid coefficients before decode-only timing
        compress(s)
    for i in range(warmup):
        step(i)
    t_step = timed_loop(torch, step, steps)
    t_dec = timed_loop(torch, lambda i: decode(sets[i % n_sets]), steps)
    t_cmp = timed_loop(torch, lambda i: compress(sets[i % n_sets]), steps)

    # per-kernel durations: every kernel is launched with its own HIP event pair on the launch stream
    reps = max(4, min(steps, 40))
    kd, kc = [], []
    for i in range(reps):
        decode(sets[i % n_sets], kd)
        compress(sets[i % n_sets], kc)
    kd = np.array(kd).reshape(reps, 3).mean(0) * 1e-3        # prepare, partial, finish [s]
    kc = np.array(kc).reshape(reps, 2).mean(0) * 1e-3        # [projection of K and V, their reductions] [s]
    t_kernels = float(kd.sum())
    t_project = float(kc[0])
    traffic = measured_traffic(cfg.index)

    def hbm(bytes_, t):
        a = bytes_ / t / 1e9 if t > 0 else 0.0
        return {"achieved": round(a, 1), "frac": round(a / HBM_PEAK_GBS, 4)}

    names = ("prepare", "partial", "finish")
    what = ("fa_decode call = decode_prepare (series coefficients) + decode_partial (middle rows; "
            "full-width rows in either) + decode_finish")
    if kd[0] == 0.0 and kd[2] == 0.0:   # the one-launch form: one workgroup per (sequence, KV head) does it all
        names, kd, kb = ("fused",), kd[1:2], {"fused": dec_bytes}
        what = "fa_decode call = decode_fused (series coefficients, all rows and the merge in one launch)"
    def kernel_traffic(prefix):   # counter summary lines are keyed by kernel name (decode_prepare2, decode_partial_fast8, ...)
        hits = [v for k, v in traffic.items() if k.startswith(prefix)]
        return sum(hits) if hits else None

    per_kernel = {}
    for i, n in enumerate(names):
        per_kernel["decode_" + n] = {"ms": round(float(kd[i]) * 1e3, 5), "algorithmic_bytes": kb[n],
                                     **hbm(kb[n], float(kd[i])), "traffic": kernel_traffic("decode_" + n)}
    dom = "decode_" + names[int(np.argmax(kd))]
    call_traffic = [kernel_traffic("decode_" + n) for n in names]
    roof_dec = {"kernel": what,
                "bound": "hbm", **hbm(dec_bytes, t_kernels), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "algorithmic_bytes": dec_bytes, "kernels_ms": round(t_kernels * 1e3, 5),
                "traffic": (sum(call_traffic) if all(v is not None for v in call_traffic) else None),
                "dominant_kernel": {"kernel": dom, **per_kernel[dom], "peak": HBM_PEAK_GBS, "unit": "GB/s"},
                "kernels": per_kernel}
    # order the keys the way the contract lists them
    roof_dec = {k: roof_dec[k] for k in ("kernel", "bound", "achieved", "peak", "unit", "frac", "traffic",
                                         "algorithmic_bytes", "kernels_ms", "dominant_kernel", "kernels")}

    mm_peak = MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else FP32_MATRIX_PEAK_TFLOPS
    tfl = cmp_flops / t_project / 1e12
    hb = hbm(cmp_bytes, t_project)
    hbm_bound = cmp_bytes / (HBM_PEAK_GBS * 1e9) >= cmp_flops / (mm_peak * 1e12)
    roof_cmp = {"kernel": "compress_project (K and V in one launch)",
                "bound": "hbm" if hbm_bound else "mfma",
                "achieved": hb["achieved"] if hbm_bound else round(tfl, 1),
                "peak": HBM_PEAK_GBS if hbm_bound else mm_peak,
                "unit": "GB/s" if hbm_bound else "TFLOP/s",
                "frac": hb["frac"] if hbm_bound else round(tfl / mm_peak, 4),
                "traffic": traffic.get("compress_project_fast_kv", traffic.get("compress_project")),
                "hbm_GBps": hb["achieved"], "hbm_frac": hb["frac"],
                "mfma_tflops": round(tfl, 1), "mfma_frac": round(tfl / mm_peak, 4)}

    res = {
        "workload": f"cfg{cfg.index} {cfg.name}: B={B} Hq={Hq} Hkv={Hkv} D={D} L={cfg.L} "
                    f"(sink {cfg.Li} + middle {N} + window {cfg.Lw}) Dkc={cfg.Dkc} Dvc={cfg.Dvc} M={M}",
        "dtype": cfg.dtype, "steps": steps, "buffer_sets": n_sets,
        "decode_context_tokens_per_s": round(B * cfg.L / t_dec, 1),
        "ms_per_step": round(t_step * 1e3, 5),
        "roofline": roof_dec,
        "phases": {
            "decode": {"ms": round(t_dec * 1e3, 5), "context_tokens_per_s": round(B * cfg.L / t_dec, 1),
                       "algorithmic_bytes": dec_bytes, "wall_GBps": round(dec_bytes / t_dec / 1e9, 1),
                       "wall_frac": round(dec_bytes / t_dec / 1e9 / HBM_PEAK_GBS, 4)},
            "compress": {"ms": round(t_cmp * 1e3, 5), "tokens_per_s": round(B * N / t_cmp, 1),
                         "algorithmic_bytes": cmp_bytes, "flop": cmp_flops,
                         "kernel_ms": {"project_kv": round(float(kc[0]) * 1e3, 5),
                                       "reduce_kv": round(float(kc[1]) * 1e3, 5)},
                         "roofline": roof_cmp},
            "step": {"ms": round(t_step * 1e3, 5), "context_tokens_per_s": round(B * cfg.L / t_step, 1)},
        },
    }

    if extras:
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
            t_app = timed_loop(torch, append, min(steps, 64))
            app_bytes = B * Hkv * (2 * M * (cfg.Dkc + cfg.Dvc) * 4 + 4 * D * e)
            res["phases"]["append"] = {"ms": round(t_app * 1e3, 5), "algorithmic_bytes": app_bytes,
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
            t_mq = timed_loop(torch, decode_mq, steps)
            res["phases"]["decode_mq"] = {"query_tokens": Tq, "ms": round(t_mq * 1e3, 5),
                                          "ms_per_query_token": round(t_mq * 1e3 / Tq, 5),
                                          "wall_GBps": round(dec_bytes / t_mq / 1e9, 1)}
        if B > 1:   # the same batch with its sequences at different positions (a quarter to all of the rows each)
            g = torch.Generator().manual_seed(4000 + cfg.index)
            seq_n = (torch.randint(N // 4, N + 1, (B,), generator=g)).to(torch.int32).cuda()
            seq_w = torch.full((B,), W, dtype=torch.int32).cuda()
            out_vl = torch.empty((B, Hq, D), dtype=torch.float32, device="cuda")

            def decode_vl(i):
                s = sets[i % n_sets]
                fa.fa_decode_varlen(s["q"], s["ck"], s["kmask"], s["cv"], s["vmask"], M, T, 0, N, seq_n, s["kk"], s["vk"],
                                    s["k_full"], s["v_full"], seq_w, num_splits=cfg.num_splits, out=out_vl, workspace=ws_d)
            for i in range(4):
                decode_vl(i)
            t_vl = timed_loop(torch, decode_vl, steps)
            rows = int(seq_n.sum().item()) + B * W
            res["phases"]["decode_varlen"] = {"ms": round(t_vl * 1e3, 5), "context_tokens": rows,
                                              "context_tokens_per_s": round(rows / t_vl, 1),
                                              "mean_fill": round(float(seq_n.float().mean().item()) / N, 3)}
        if N >= M:
            ws_s = torch.empty(max(256, fa.select_workspace_bytes(fa.FA_BF16 if dt == torch.bfloat16 else fa.FA_F32,
                                                                  B, Hkv, N, D, M)), dtype=torch.uint8, device="cuda")
            sel = lambda i: fa.fa_select_dims(sets[i % n_sets]["k_mid"], M, cfg.Dkc, workspace=ws_s)
            for i in range(2):
                sel(i)
            t_sel = timed_loop(torch, sel, max(4, min(steps, 20)))
            sel_flop = 2.0 * B * Hkv * N * M * D
            res["phases"]["select"] = {"ms": round(t_sel * 1e3, 5), "flop": sel_flop,
                                       "fp32_matrix_tflops": round(sel_flop / t_sel / 1e12, 1),
                                       "fp32_matrix_frac": round(sel_flop / t_sel / 1e12 / FP32_MATRIX_PEAK_TFLOPS, 4)}
            # Fourier against translated Legendre at the same number of states (the paper's basis comparison,
            # on the synthetic law): mean reconstruction error of the planted (smooth) dims and of the others
            Ml = min(M, 256)
            ws_l = torch.empty(max(256, fa.legt_workspace_bytes(B, Hkv, N, D, Ml)), dtype=torch.uint8, device="cuda")
            x0 = sets[0]["k_mid"]
            leg = lambda i: fa.fa_legt(x0, Ml, workspace=ws_l)
            leg(0)
            t_leg = timed_loop(torch, leg, 3)
            _, mse_l = fa.fa_legt(x0, Ml, workspace=ws_l)
            _, mse_f = fa.fa_select_dims(x0, Ml, cfg.Dkc, workspace=ws_s)
            torch.cuda.synchronize()
            planted = sets[0]["kmask"].bool()
            res["phases"]["basis_comparison"] = {
                "states": Ml, "legt_ms": round(t_leg * 1e3, 4),
                "legt_fp32_vector_tflops": round(4.0 * B * Hkv * N * Ml * D / t_leg / 1e12, 2),
                "mse_smooth_dims": {"fourier": float(mse_f[planted].mean()), "legt": float(mse_l[planted].mean())},
                "mse_other_dims": {"fourier": float(mse_f[~planted].mean()), "legt": float(mse_l[~planted].mean())}}
    del sets, ws_c, ws_d
    torch.cuda.empty_cache()
    return res, ctx


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (one GPU's share of the path at its "
              "real shape); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from workloads import CONFIGS, get_config

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = get_config(args.workload)
    res, ctx = measure(cfg, args.steps, args.warmup, args.extras)

    result = {
        "metric": METRIC,
        "value": res["decode_context_tokens_per_s"],
        "unit": "context tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {
            "workload": res["workload"],
            "value_is": "B * L / t of the fa_decode call alone (decode context tokens/s); each of the "
                        "decode-only, compress-only and whole-step loops times exactly `steps` calls",
            "step": "fa_compress_kv(K, V) + fa_decode (ms_per_step)",
            "buffer_sets": res["buffer_sets"],
        },
        "roofline": res["roofline"],
        "phases": res["phases"],
    }

    if not args.only:
        others = {}
        for c in CONFIGS[1:]:
            if c.index == cfg.index:
                continue
            r, _ = measure(c, max(10, min(args.steps, 60)), max(2, min(args.warmup, 10)))
            others[f"cfg{c.index}"] = {
                "workload": r["workload"], "steps": r["steps"],
                "decode_context_tokens_per_s": r["decode_context_tokens_per_s"],
                "decode_ms": r["phases"]["decode"]["ms"], "ms_per_step": r["ms_per_step"],
                "roofline": {k: r["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic",
                                                           "kernels_ms")},
                "decode_kernels": {k: {"ms": v["ms"], "frac": v["frac"]} for k, v in r["roofline"]["kernels"].items()},
                "compress": {"ms": r["phases"]["compress"]["ms"], "kernel_ms": r["phases"]["compress"]["kernel_ms"],
                             "roofline": r["phases"]["compress"]["roofline"]},
            }
        result["other_workloads"] = others

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
    pairs of the same workload: the decode step the headline value measures (the
    oracle's compression of the sample is needed first and is timed beside it)."""
    import oracle.fourier_kv as fk
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    heads = [(b, h) for b in range(cfg.B) for h in range(cfg.Hkv)]
    G = cfg.G
    done, t_dec, t_cmp = 0, 0.0, 0.0
    for b, h in heads:
        t0 = time.perf_counter()
        ck, kk = fk.compress_segment(ctx["k_mid"][b, h], ctx["kmask"][b, h], cfg.M, cfg.T, 0)
        cv, vk = fk.compress_segment(ctx["v_mid"][b, h], ctx["vmask"][b, h], cfg.M, cfg.T, 0)
        t1 = time.perf_counter()
        fk.decode_head_group(ctx["q"][b, h * G:(h + 1) * G], ck, ctx["kmask"][b, h], cv, ctx["vmask"][b, h],
                             cfg.T, 0, cfg.N, kk, vk, ctx["k_full"][b, h], ctx["v_full"][b, h])
        t2 = time.perf_counter()
        t_cmp += t1 - t0
        t_dec += t2 - t1
        done += 1
        if (t_cmp + t_dec) * (1.0 + 1.0 / done) > budget_s:
            break
    tokens = cfg.B * cfg.L * done / len(heads)
    return {"value": round(tokens / t_dec, 1), "unit": "context tokens/s", "cores": int(cores),
            "kind": "oracle",
            "sample": f"{done} of {len(heads)} (sequence, KV head) pairs of the same workload: oracle decode "
                      f"{t_dec:.1f} s wall (its compression of the sample, {t_cmp:.1f} s, is not in the value; "
                      f"whole path {tokens / (t_dec + t_cmp):.1f} context tokens/s)"}


if __name__ == "__main__":
    main()
