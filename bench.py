#!/usr/bin/env python3
"""Benchmark of the block-wise causal attention hot path on one MI355X.

One "step" is one pass of the hot path over one batch of synthetic input: for the
training form the forward call; for the cached forms the cache append of the new
frames and the forward over the cache (nfd_kvcache_append_attn_fwd: one call).  Inputs are resident in HBM before the timed
region.  Prints ONE JSON line on stdout.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 matrix-core peak (published)
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E peak (published)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2_train")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cache-sets", type=int, default=16,
                    help="cached forms (decode, speculative): number of distinct K/V caches the steps rotate over")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--settle-ms", type=float, default=150.0,
                    help="the warm-up runs its --warmup steps and then keeps stepping until this much GPU time has passed: "
                         "from idle the chip boosts, overshoots its power limit, throttles and needs about 60 launches of the "
                         "training form (20-30 ms) to settle; 0 = exactly --warmup steps")
    ap.add_argument("--no-check", action="store_true", help="skip the comparison of the timed output with the oracle")
    ap.add_argument("--all", action="store_true", help="also time the other workloads (reported on stderr)")
    ap.add_argument("--bwd", action="store_true",
                    help="also time the training step of the attention: forward with log-sum-exp + backward (stderr and 'backward')")
    ap.add_argument("--rope", action="store_true",
                    help="also time the fused 3D rotary embedding + cache write on the workload's new frames (stderr and 'pre_op')")
    ap.add_argument("--fp8kv", action="store_true",
                    help="also time the cached workloads over the 8-bit (E4M3) KV cache: quantising append + forward "
                         "(stderr and 'fp8_kv_cache')")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 1 GiB device copy a few times (a kernel of known HBM bytes, for scaling profiler counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2506_01380_amd import binding as nb
    from paper_2506_01380_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    attn = nb.Attention("bf16")

    def oracle_check(tensors, cfg):
        """The output the last timed step left behind against the fp64 oracle on the same device-drawn inputs, on
        sampled query rows (first and last row of every query frame plus a few seeded random ones; all heads)."""
        from oracle import nfd_oracle as orc
        q, k, v, out = tensors[:4]
        T, kvf, qf = cfg["T"], cfg["kv_frames"], cfg["q_frames"]
        rows = wl.sample_rows(T, qf, 2 if qf * T > 20000 else 6, cfg["seed"])
        host = lambda t: t.float().cpu().numpy().astype(np.float64)
        torch.cuda.synchronize()
        ref = orc.block_causal_attn(host(q), host(k[:, :, : kvf * T]), host(v[:, :, : kvf * T]), T, kv_frames=kvf, q_frames=qf, rows=rows)
        got = host(out[:, :, torch.from_numpy(rows).to(out.device)])
        d = got - ref
        row = np.sqrt((d ** 2).sum(-1)) / np.sqrt((ref ** 2).sum(-1))
        return dict(max_abs=float(np.abs(d).max()), rel_l2=float(np.linalg.norm(d) / np.linalg.norm(ref)),
                    worst_row_rel_l2=float(row.max()), rows_per_head=int(len(rows)), finite=bool(np.isfinite(got).all()))

    def time_workload(name, steps, warmup, kv8=False):
        cfg = wl.CONFIGS[name] if name in wl.CONFIGS else wl.EXTRA_CONFIGS[name]
        B, H, D, T, kvf, qf, F = (cfg[x] for x in ("B", "H", "D", "T", "kv_frames", "q_frames", "F"))
        # cached forms run "cold": every step takes the next of --cache-sets distinct K/V caches (one per layer of
        # a model; together larger than the 256 MB last-level cache), so K and V come from HBM
        rotate = max(1, args.cache_sets) if qf < kvf else 1
        gen = torch.Generator(device="cuda").manual_seed(cfg["seed"])
        mk = lambda *s: torch.randn(*s, device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
        cached = qf < kvf
        sets = []
        if kv8:  # the same step over the 8-bit cache: quantising append of the new frames, then the forward
            nbytes = nb.nfd_fp8_cache_bytes(B, H, F, T, D)
            ksc = torch.full((B, H), 6.0 / 448.0, device="cuda")  # 6 sigma of N(0,1) at the top of the E4M3 range
            vsc = torch.full((B, H), 6.0 / 448.0, device="cuda")
        for _ in range(rotate):
            q = mk(B, H, qf * T, D)
            if kv8:
                k, v = torch.zeros(nbytes, dtype=torch.uint8, device="cuda"), torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
                kn, vn = mk(B, H, kvf * T, D), mk(B, H, kvf * T, D)
                nb.nfd_kvcache_append_fp8(attn.h, k, v, ksc, vsc, kn, vn, B, H, F, T, D, 0, kvf)
                kn, vn = kn[:, :, (kvf - qf) * T:].clone(), vn[:, :, (kvf - qf) * T:].clone()
            else:
                k, v = mk(B, H, F * T, D), mk(B, H, F * T, D)
                kn = k[:, :, (kvf - qf) * T: kvf * T].clone() if cached else None
                vn = v[:, :, (kvf - qf) * T: kvf * T].clone() if cached else None
            sets.append((q, k, v, torch.empty_like(q), kn, vn))

        def step(i):
            q, k, v, out, kn, vn = sets[i % rotate]
            if kv8:
                nb.nfd_kvcache_append_fp8(attn.h, k, v, ksc, vsc, kn, vn, B, H, F, T, D, kvf - qf, qf)
                nb.nfd_block_causal_attn_fwd_fp8kv(attn.h, q, k, v, ksc, vsc, out, B, H, F, T, D, kvf, qf)
                return
            if cached:  # cache write of the new frames and the attention over the cache, one call
                nb.nfd_kvcache_append_attn_fwd(attn.h, q, k, v, kn, vn, out, B, H, F, T, D, kvf, qf)
            else:
                nb.nfd_block_causal_attn_fwd(attn.h, q, k, v, out, B, H, F, T, D, kvf, qf)

        w0, w1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        w0.record()
        for i in range(warmup):
            step(i)
        warm = warmup
        while args.settle_ms > 0:  # untimed: let clock and power management settle under this very load
            w1.record()
            torch.cuda.synchronize()
            if w0.elapsed_time(w1) >= args.settle_ms:
                break
            for i in range(max(1, warmup)):
                step(warm + i)
            warm += max(1, warmup)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(steps):
            step(i)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        # a second, untimed-for-the-headline pass with one event pair per step: median and minimum
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(steps, 200))]
        for i, (a0, a1) in enumerate(evs):
            a0.record()
            step(i)
            a1.record()
        torch.cuda.synchronize()
        per = sorted(a0.elapsed_time(a1) for a0, a1 in evs)
        check = None  # after all timing: the oracle runs on the host and the GPU idles meanwhile
        if not args.no_check and not kv8:
            check = oracle_check(sets[(steps - 1) % rotate], cfg)
        flops = nb.unmasked_flops(B, H, D, T, kvf, qf)
        min_bytes = (2 * kvf * T + 2 * qf * T) * D * 2 * B * H
        # which roof binds: the larger of the times the algorithmic FLOPs and the minimum HBM bytes need at the peaks
        t_mfma, t_hbm = flops / (PEAK_BF16_TFLOPS * 1e9), min_bytes / (PEAK_HBM_GBS * 1e6)  # ms
        return dict(workload=name, ms_per_step=ms, ms_median=per[len(per) // 2], ms_min=per[0], tflops=flops / ms * 1e-9, gbs=min_bytes / ms * 1e-6,
                    pct_mfma_peak=100 * t_mfma / ms, pct_hbm_peak=100 * t_hbm / ms, bound="mfma" if t_mfma >= t_hbm else "hbm",
                    frames_per_s=B * qf / ms * 1e3, flops=flops, min_bytes=min_bytes, cfg=cfg, warmup_steps_run=warm,
                    vs_oracle=check, cache_sets=rotate, plan=nb.nfd_attn_plan(nb.NFD_BF16, B, H, F, T, D, kvf, qf))

    main_res = time_workload(args.workload, args.steps, args.warmup)
    cfg = main_res["cfg"]

    if args.calibrate_copy:
        # kvcache_append is a plain copy: here exactly 1 GiB read and 1 GiB written per launch (K and V, 512 MiB each)
        cb, ch, cf, ct, cd = 4, 16, 64, 1024, 64
        kc = torch.zeros((cb, ch, cf * ct, cd), dtype=torch.bfloat16, device="cuda")
        vc = torch.zeros_like(kc)
        kn = torch.ones_like(kc)
        vn = torch.ones_like(kc)
        for _ in range(4):
            nb.nfd_kvcache_append(attn.h, kc, vc, kn, vn, cb, ch, cf, ct, cd, 0, cf)
        torch.cuda.synchronize()
        del kc, vc, kn, vn

    def time_rope(name, steps, warmup, kv8=False):
        """The step before the attention call: rotate q and k of the workload's query frames, write k and v
        into the cache.  HBM-bound streaming: 3 tensors in, 3 out (kv8: k and v out as 8-bit codes)."""
        c = wl.CONFIGS[name]
        B, H, D, T, kvf, qf, F = (c[x] for x in ("B", "H", "D", "T", "kv_frames", "q_frames", "F"))
        grid = (24, T // 24)          # 24 x 14 latent grid at T = 336, 24 x 24 at T = 576
        sections = (16, 24, 24)       # [n_T, n_H, n_W] of a 64-wide head
        gen = torch.Generator(device="cuda").manual_seed(c["seed"] + 5)
        mk = lambda *s: torch.randn(*s, device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
        sets = []
        if kv8:
            n8 = nb.nfd_fp8_cache_bytes(B, H, F, T, D)
            ksc = torch.full((B, H), 6.0 / 448.0, device="cuda")
            vsc = torch.full((B, H), 6.0 / 448.0, device="cuda")
        for _ in range(4):
            cache = (lambda: torch.zeros(n8, dtype=torch.uint8, device="cuda")) if kv8 else \
                (lambda: torch.zeros(B, H, F * T, D, device="cuda", dtype=torch.bfloat16))
            sets.append((mk(B, H, qf * T, D), mk(B, H, qf * T, D), mk(B, H, qf * T, D),
                         torch.empty(B, H, qf * T, D, device="cuda", dtype=torch.bfloat16), cache(), cache()))

        def step(i):
            q, kn, vn, qo, kc, vc = sets[i % len(sets)]
            if kv8:
                nb.nfd_rope_kvcache_append_fp8(attn.h, q, qo, kc, vc, ksc, vsc, kn, vn, B, H, F, T, D, kvf - qf, qf, 0,
                                               grid[0], grid[1], sections[0], sections[1], sections[2], 10000.0)
                return
            nb.nfd_rope_kvcache_append(attn.h, q, qo, kc, vc, kn, vn, B, H, F, T, D, kvf - qf, qf, 0,
                                       grid[0], grid[1], sections[0], sections[1], sections[2], 10000.0)

        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(steps):
            step(i)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        nbytes = (5 if kv8 else 6) * B * H * qf * T * D * 2  # q, k, v read; q, k, v written (k, v as one byte each with kv8)
        return dict(kernel="rope_kvcache_append" + ("<.., true> (8-bit cache)" if kv8 else ""), workload=name, us_per_call=round(ms * 1e3, 2), bytes=nbytes,
                    gbs=round(nbytes / ms * 1e-6, 1), frac_hbm_peak=round(nbytes / ms * 1e-6 / PEAK_HBM_GBS, 4))

    def time_bwd(name, steps, warmup):
        """Forward that keeps the log-sum-exp, then the backward (dq kernel, then dk/dv kernel).  FLOPs counted:
        forward 4.D per visible pair, backward 10.D (five products), the recomputation in the second
        backward kernel is not counted."""
        c = wl.CONFIGS[name]
        B, H, D, T, kvf, qf, F = (c[x] for x in ("B", "H", "D", "T", "kv_frames", "q_frames", "F"))
        gen = torch.Generator(device="cuda").manual_seed(c["seed"] + 7)
        mk = lambda *s: torch.randn(*s, device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
        q, k, v, g = mk(B, H, qf * T, D), mk(B, H, F * T, D), mk(B, H, F * T, D), mk(B, H, qf * T, D)
        out = torch.empty_like(q)
        lse = torch.empty((B, H, qf * T), dtype=torch.float32, device="cuda")
        dq, dk, dv = torch.empty_like(q), torch.zeros_like(k), torch.zeros_like(v)

        def fwd():
            nb.nfd_block_causal_attn_fwd_lse(attn.h, q, k, v, out, lse, B, H, F, T, D, kvf, qf)

        def bwd():
            nb.nfd_block_causal_attn_bwd(attn.h, q, k, v, out, g, lse, dq, dk, dv, B, H, F, T, D, kvf, qf)

        def timed(fn):
            for _ in range(warmup):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / steps

        fwd()
        ms_f, ms_b = timed(fwd), timed(bwd)
        fl = nb.unmasked_flops(B, H, D, T, kvf, qf)
        return dict(kernel="attn_bwd_dq_bf16_d64 + attn_bwd_dkdv_bf16_d64", workload=name,
                    fwd_lse_ms=round(ms_f, 5), bwd_ms=round(ms_b, 5), bwd_tflops=round(2.5 * fl / ms_b * 1e-9, 2),
                    bwd_frac_mfma_peak=round(2.5 * fl / ms_b * 1e-9 / PEAK_BF16_TFLOPS, 4),
                    fwd_bwd_tflops=round(3.5 * fl / (ms_f + ms_b) * 1e-9, 2))

    backward = None
    if args.bwd:
        backward = time_bwd(args.workload, max(10, args.steps // 2), args.warmup)
        print(json.dumps(backward), file=sys.stderr, flush=True)

    pre_op = None
    if args.rope:
        pre_op = time_rope(args.workload, args.steps, args.warmup)
        print(json.dumps(pre_op), file=sys.stderr, flush=True)
        if args.fp8kv:
            pre_op = [pre_op, time_rope(args.workload, args.steps, args.warmup, kv8=True)]
            print(json.dumps(pre_op[1]), file=sys.stderr, flush=True)

    others = []
    if args.all:
        for name in wl.CONFIGS:
            if name == args.workload or wl.CONFIGS[name]["dtype"] != "bf16":
                continue
            steps = 20 if name == "c5a_long_train" else 200
            r = time_workload(name, steps, 10)
            r.pop("cfg")
            others.append(r)
            print(json.dumps(r), file=sys.stderr, flush=True)

    fp8kv = []
    if args.fp8kv:
        # the workload named on the command line if it is a cached form, otherwise every cached form
        main_cached = cfg["q_frames"] < cfg["kv_frames"]
        for name in ([args.workload] if main_cached else list(wl.CONFIGS)):
            c = wl.CONFIGS[name] if name in wl.CONFIGS else wl.EXTRA_CONFIGS[name]
            if c["dtype"] != "bf16" or c["q_frames"] == c["kv_frames"]:
                continue
            r = time_workload(name, args.steps if main_cached else 200, args.warmup if main_cached else 10, kv8=True)
            r.pop("cfg")
            fp8kv.append({k: (round(v, 4) if isinstance(v, float) else v) for k, v in r.items()
                          if k in ("workload", "ms_per_step", "ms_median", "ms_min", "tflops", "frames_per_s")})
            print(json.dumps({"fp8_kv_cache": fp8kv[-1]}), file=sys.stderr, flush=True)

    def oracle_rate(name, seconds):
        """The fp64 oracle on the host cores on a bounded sample of the workload (whole rows, all heads)."""
        from oracle import nfd_oracle as orc
        c, q, k, v = wl.make_config(name)
        B, H, D, T, kvf, qf = (c[x] for x in ("B", "H", "D", "T", "kv_frames", "q_frames"))
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        q64, k64, v64 = (np.asarray(x, dtype=np.float64) for x in (q, k, v))  # exact widening, outside the timed part
        P = kvf - qf

        def run_rows(rows):
            t0 = time.perf_counter()
            orc.block_causal_attn(q64, k64, v64, T, kv_frames=kvf, q_frames=qf, rows=rows)
            dt = time.perf_counter() - t0
            idx = np.arange(qf * T) if rows is None else rows
            pairs = int(sum((P + int(r) // T + 1) * T for r in idx)) * B * H
            return dt, 4 * D * pairs, len(idx)

        # calibrate on two rows per frame, then size the sample for about `seconds` of oracle time
        dt0, fl0, n0 = run_rows(wl.sample_rows(T, qf, 0, c["seed"]))
        rows_fit = int(n0 * seconds / max(dt0, 1e-4))
        if rows_fit >= qf * T:
            dt, fl, n = run_rows(None)
            what = "all %d query rows of all %d heads (the whole workload)" % (qf * T, B * H)
        else:
            per_frame = max(1, rows_fit // qf - 2)
            dt, fl, n = run_rows(wl.sample_rows(T, qf, per_frame, c["seed"]))
            what = "%d of %d query rows per head (first, last and %d random rows of each frame), all %d heads" % (
                n, qf * T, per_frame, B * H)
        model = "unknown"
        try:
            with open("/proc/cpuinfo") as f:
                model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), "unknown")
        except OSError:
            pass
        return dict(value=round(fl / dt * 1e-12, 5), unit="TFLOP/s", cores=cores, kind="oracle",
                    sample="%s, %.1f s of oracle time" % (what, dt), cpu=model)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = oracle_rate(args.workload, args.cpu_seconds)
        for r in others:  # --all: the oracle beside every GPU time, a few seconds each
            r["cpu_baseline"] = oracle_rate(r["workload"], min(args.cpu_seconds, 4.0))
            print(json.dumps({"workload": r["workload"], "cpu_baseline": r["cpu_baseline"]}), file=sys.stderr, flush=True)

    # HBM bytes per launch come from rocprofv3 counter runs kept under profiles/, not from this run
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get(args.workload, {}).get("bytes_per_launch")
    frac = main_res["tflops"] / PEAK_BF16_TFLOPS
    hbm_frac = main_res["gbs"] / PEAK_HBM_GBS
    if main_res["bound"] == "mfma":
        roof = {"bound": "mfma", "achieved": round(main_res["tflops"], 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(frac, 4)}
    else:
        roof = {"bound": "hbm", "achieved": round(main_res["gbs"], 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(hbm_frac, 4)}
    roof.update({"traffic": traffic, "traffic_source": "profiles/hbm_traffic.json (rocprofv3 --pmc runs; not measured in this run)",
                 "kernel": "attn_fwd_bf16_d64_m16" if main_res["plan"]["block_m"] == 256 else "attn_fwd_bf16_d64<1>",
                 # both roofs, always: the algorithmic FLOPs against the matrix-core peak, the minimum bytes against HBM
                 "mfma": {"achieved_tflops": round(main_res["tflops"], 2), "peak": PEAK_BF16_TFLOPS, "frac": round(frac, 4)},
                 "hbm": {"achieved_gbs": round(main_res["gbs"], 1), "peak": PEAK_HBM_GBS, "frac": round(hbm_frac, 4),
                         "min_bytes": main_res["min_bytes"]}})
    line = {
        "metric": "block-causal attn TFLOP/s (unmasked) + % bf16 MFMA peak; attn-layer frames/s",
        "value": round(main_res["tflops"], 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(main_res["ms_per_step"], 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "B": cfg["B"], "H": cfg["H"], "D": cfg["D"], "T": cfg["T"],
                   "kv_frames": cfg["kv_frames"], "q_frames": cfg["q_frames"],
                   "pct_bf16_mfma_peak": round(100 * frac, 2), "gbs": round(main_res["gbs"], 1),
                   "pct_hbm_peak": round(100 * hbm_frac, 2), "bound": main_res["bound"],
                   "warmup_steps_run": main_res["warmup_steps_run"], "settle_ms": args.settle_ms,
                   "attn_layer_frames_per_s": round(main_res["frames_per_s"], 1),
                   "ms_per_step_median": round(main_res["ms_median"], 5), "ms_per_step_min": round(main_res["ms_min"], 5),
                   "cache_sets": main_res["cache_sets"], "plan": main_res["plan"]},
        "roofline": roof,
        "cpu_baseline": cpu,
        "vs_oracle": main_res["vs_oracle"],
    }
    if backward:
        line["backward"] = backward
    if pre_op:
        line["pre_op"] = pre_op
    if fp8kv:
        line["fp8_kv_cache"] = fp8kv
    if others:
        line["other_workloads"] = [{k: (round(v, 4) if isinstance(v, float) else v) for k, v in r.items()
                                    if k in ("workload", "ms_per_step", "ms_median", "ms_min", "tflops", "pct_mfma_peak", "gbs", "pct_hbm_peak", "bound",
                                             "frames_per_s", "vs_oracle", "cpu_baseline")}
                                   for r in others]
    attn.close()
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
