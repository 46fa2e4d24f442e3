"""Benchmark of the FLASH-D attention forward path on one MI355X.

A step is one flashd_attn_fwd call (the whole hot path: Q load, K/V streaming, scores,
mask, weight recurrence, blend, store) on the LLaMA-7B-like causal bf16 prefill workload;
the inputs are resident in HBM before the timed region and rotate over several independent
sets so that the last-level cache is not flattering.  One JSON line is printed.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--settle-ms T] [--no-cpu] [--no-decode]
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import sys
import time

import numpy as np
import torch

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16/fp16 matrix peak
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E peak
# fp32 vector fma without packed instructions (this build compiles them out): 256 CUs x 4 SIMDs
# x 16 lanes x 2 flop x 2.4 GHz = 78.6 TFLOP/s, half the published 157.3 that counts packed issue
PEAK_FP32_FMA = 78.6

# HBM-side bytes per launch of the dominant kernel, from the profiler's FETCH_SIZE and
# WRITE_SIZE counters scaled by a 1 GiB device copy (the summaries under profiles/ give the
# commands and the raw readings); they cannot be read from inside this process.
TRAFFIC_PREFILL_BYTES = 343.8e6
TRAFFIC_DECODE_BYTES = 2148.6e6


SETTLE_MS = 150.0
SETTLE = {"ms": SETTLE_MS}      # set from --settle-ms


def settle(fn, nsets, ms=None):
    """Untimed launches for `ms` of GPU time.  The clock governor takes the GPU from its idle
    clock to the steady one over about 40 ms of load (a run timed from idle reads 15 % low on
    the first 10 ms), so every timed leg starts with this."""
    ms = SETTLE["ms"] if ms is None else ms
    if ms <= 0:
        return 0
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    n = 0
    ev0.record()
    while True:
        for i in range(8):
            fn((n + i) % nsets)
        n += 8
        ev1.record()
        ev1.synchronize()
        if ev0.elapsed_time(ev1) >= ms:
            return n


def time_calls(fn, steps, warmup, nsets):
    """Wall time and HIP-event time (on the launch stream) of `steps` calls of fn(i % nsets),
    after the clock-settling launches and `warmup` more untimed calls."""
    settle(fn, nsets)
    for i in range(warmup):
        fn(i % nsets)
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(steps):
        fn(i % nsets)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return wall_ms, ev0.elapsed_time(ev1)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--sets", type=int, default=4, help="independent input sets to rotate over")
    ap.add_argument("--settle-ms", type=float, default=SETTLE_MS,
                    help="GPU time of untimed launches before each timed leg (clock ramp)")
    ap.add_argument("--workload", type=int, default=1, choices=[1, 2, 4],
                    help="index of the prefill configuration that is timed (1 = the headline "
                         "causal bf16 prefill, the default; 2 = long non-causal bf16; "
                         "4 = fp16 stress): the others are there for profiles")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode side measurement")
    ap.add_argument("--no-ablation", action="store_true")
    ap.add_argument("--no-kv8", action="store_true", help="skip the fp8 K/V decode measurement")
    ap.add_argument("--no-decode16", action="store_true",
                    help="skip the decode measurement with 16 query positions per head")
    ap.add_argument("--no-state", action="store_true",
                    help="skip the two-chunk run through flashd_attn_fwd_state")
    ap.add_argument("--no-skip-stats", action="store_true",
                    help="skip the static skip-range statistics (Sec. III-C) of two workloads")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain device copy of 1 GiB, 10 times (reference for "
                         "scaling the profiler's HBM byte counters)")
    args = ap.parse_args()
    SETTLE["ms"] = args.settle_ms
    if args.gpus != 1:
        print("bench.py measures one GPU; this build has no multi-GPU path (--gpus must be 1)",
              file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 256)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": 1 << 30, "bytes_written": 1 << 30,
                                               "launches": 10}}))
        return 0

    from paper_2505_14201_amd import flashd, synthetic

    w = synthetic.CONFIGS[args.workload]
    q, k, v, _ = synthetic.make_qkv(w)
    sets = []
    for s in range(args.sets):
        if s == 0:
            qs, ks, vs = q, k, v
        else:   # further sets: same distribution, different seed
            qs, ks, vs, _ = synthetic.make_qkv(dataclasses.replace(w, seed=w.seed + 100 * s))
        qg, kg, vg = qs.cuda(), ks.cuda(), vs.cuda()
        sets.append((qg, kg, vg, torch.empty_like(qg)))
    torch.cuda.synchronize()

    def step(i):
        qg, kg, vg, og = sets[i]
        flashd.attn_fwd(qg, kg, vg, og, w.causal, w.scale)

    wall_ms, ev_ms = time_calls(step, args.steps, args.warmup, args.sets)
    ms_per_step = wall_ms / args.steps
    kern_ms = ev_ms / args.steps
    flops = w.flops()
    value = flops / (ms_per_step * 1e-3) / 1e12
    achieved = flops / (kern_ms * 1e-3) / 1e12

    out = {
        "metric": "attention fwd TFLOP/s (%s %s prefill, FLASH-D form)"
                  % ("causal" if w.causal else "non-causal", w.dtype),
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "settle_ms": args.settle_ms,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "Lq": w.Lq,
                   "Lk": w.Lk, "d": w.d, "causal": w.causal, "input_sets": args.sets,
                   "flop_per_step": flops},
        "roofline": {"bound": "mfma",
                     "kernel": "tile_kernel<%s,%d> (flashd_attn_fwd)" % (w.dtype.upper(), w.d),
                     "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     "traffic": TRAFFIC_PREFILL_BYTES if args.workload == 1 else None,
                     "kernel_ms": round(kern_ms, 4)},
    }

    # parity of what was just timed, against the oracle, and the oracle's own speed
    if not args.no_cpu:
        from oracle import attention as oa
        # The oracle does about 0.09 TFLOP/s on the host cores: the whole headline workload
        # takes seconds; larger ones are sampled by query rows (seeded, spread over all
        # heads) so that the leg stays near 20 s.
        nrows_all = w.B * w.Hq * w.Lq
        budget_flop = 2.0e12
        if flops <= budget_flop:
            rows, nrows, what = None, nrows_all, "the whole workload (all B*Hq*Lq rows)"
        else:
            nrows = max(1024, int(nrows_all * budget_flop / flops))
            rng = np.random.default_rng(12345)
            flat = np.sort(rng.choice(nrows_all, size=nrows, replace=False))
            rows = np.stack([flat // (w.Hq * w.Lq), (flat // w.Lq) % w.Hq, flat % w.Lq], axis=1)
            what = "%d of %d query rows, seeded uniform sample" % (nrows, nrows_all)
        t0 = time.perf_counter()
        ref = oa.attn(q, k, v, w.causal, w.scale, "definition", rows)
        cpu_s = time.perf_counter() - t0
        got = sets[0][3].cpu().double().numpy()
        if rows is not None:
            got = got[rows[:, 0], rows[:, 1], rows[:, 2]]
            if w.causal:
                vis = np.clip(rows[:, 2] + (w.Lk - w.Lq) + 1, 0, w.Lk).sum()
            else:
                vis = float(nrows) * w.Lk
            cpu_flops = 4.0 * w.d * float(vis)
        else:
            cpu_flops = flops
        err = np.abs(got - ref)
        out["parity"] = {"max_abs_err": float(err.max()),
                         "rel_rms_err": float(np.sqrt((err ** 2).sum() / (ref ** 2).sum())),
                         "rows_checked": int(nrows)}
        out["cpu_baseline"] = {"value": round(cpu_flops / cpu_s / 1e12, 5), "unit": "TFLOP/s",
                               "cores": oa.num_threads(), "kind": "oracle",
                               "sample": what + ", fp64 definition",
                               "seconds": round(cpu_s, 2)}
        del ref, got, err

    if not args.no_ablation:
        def step_abl(i):
            qg, kg, vg, og = sets[i]
            flashd.attn_fwd_ex(qg, kg, vg, og, w.causal, w.scale, flashd.VARIANT_ONLINE_SOFTMAX, 1)
        _, ev_abl = time_calls(step_abl, args.steps, args.warmup, args.sets)
        out["ablation_online_softmax"] = {
            "kernel_ms": round(ev_abl / args.steps, 4),
            "TFLOP/s": round(flops / (ev_abl / args.steps * 1e-3) / 1e12, 2)}

    if not args.no_ablation:
        # Alg. 3 literally, one sigmoid per key on the vector ALUs (variant PER_KEY): what
        # lifting the recurrence to key tiles on the matrix cores buys
        pk_steps = 5

        def step_pk(i):
            qg, kg, vg, og = sets[i]
            flashd.attn_fwd_ex(qg, kg, vg, og, w.causal, w.scale, flashd.VARIANT_PER_KEY, 1)
        step_pk(0)
        _, ev_pk = time_calls(step_pk, pk_steps, 0, args.sets)
        out["per_key_literal"] = {
            "kernel_ms": round(ev_pk / pk_steps, 3),
            "TFLOP/s": round(flops / (ev_pk / pk_steps * 1e-3) / 1e12, 2)}

    if not args.no_skip_stats:
        # Sec. III-C / Table I on synthetic inputs: share of Alg. 3 steps whose score
        # difference leaves the static range [-6, 11]
        def rates(wl, qg, kg):
            cnt = torch.empty(3, dtype=torch.int64, device="cuda")
            flashd.skip_stats(qg, kg, wl.causal, wl.scale, counts=cnt)       # warm-up
            reps = 20
            _, ms = time_calls(lambda _i: flashd.skip_stats(qg, kg, wl.causal, wl.scale,
                                                            counts=cnt), reps, 0, 1)
            ms /= reps
            steps, low, high = (int(x) for x in cnt.cpu())
            tf = 2.0 * wl.d * steps / (ms * 1e-3) / 1e12      # one fp32 fma per element
            return {"workload": wl.name, "steps": steps, "low_frac": round(low / steps, 6),
                    "high_frac": round(high / steps, 6), "kernel_ms": round(ms, 3),
                    "roofline": {"bound": "alu", "achieved": round(tf, 2), "peak": PEAK_FP32_FMA,
                                 "unit": "TFLOP/s", "frac": round(tf / PEAK_FP32_FMA, 4)}}
        ws = synthetic.CONFIGS[4]
        qs_, ks_, _, _ = synthetic.make_qkv(ws)
        out["skip_stats"] = [rates(w, sets[0][0], sets[0][1]), rates(ws, qs_.cuda(), ks_.cuda())]

    if not args.no_state:
        # the same workload fed as two chunks of keys with the Alg. 3 state handed on
        # (flashd_attn_fwd_state): chunked prefill through the state primitive
        qg, kg, vg, og = sets[0]
        half = w.Lk // 2
        kc = [kg[:, :, :half].contiguous(), kg[:, :, half:].contiguous()]
        vc = [vg[:, :, :half].contiguous(), vg[:, :, half:].contiguous()]
        st = torch.empty(w.B, w.Hq, w.Lq, w.d + 2, dtype=torch.float32, device="cuda")

        def step_state(_i):
            flashd.attn_fwd_state(qg, kc[0], vc[0], w.causal, w.scale, state_out=st,
                                  causal_shift=w.Lk - w.Lq)
            flashd.attn_fwd_state(qg, kc[1], vc[1], w.causal, w.scale, o=og, state_in=st,
                                  causal_shift=w.Lk - w.Lq - half)
        _, ev_st = time_calls(step_state, max(5, args.steps // 5), 2, 1)
        ms_st = ev_st / max(5, args.steps // 5)
        out["state_two_chunks"] = {"ms_per_step": round(ms_st, 4),
                                   "TFLOP/s": round(flops / (ms_st * 1e-3) / 1e12, 2)}
        del kc, vc, st

    del sets
    torch.cuda.empty_cache()

    if not args.no_decode:
        wd = synthetic.CONFIGS[3]
        qd, kd, vd, _ = synthetic.make_qkv(wd)
        qg, kg, vg = qd.cuda(), kd.cuda(), vd.cuda()
        og = torch.empty_like(qg)

        def step_dec(_):
            flashd.attn_fwd(qg, kg, vg, og, wd.causal, wd.scale)
        dsteps = max(10, args.steps // 2)
        _, ev_dec = time_calls(step_dec, dsteps, 5, 1)
        dms = ev_dec / dsteps
        gbs = wd.bytes_io() / (dms * 1e-3) / 1e9
        out["decode"] = {"workload": wd.name, "ms_per_step": round(dms, 4),
                         "bytes_per_step": wd.bytes_io(),
                         "roofline": {"bound": "hbm", "achieved": round(gbs, 1),
                                      "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                      "frac": round(gbs / PEAK_HBM_GBS, 4),
                                      "traffic": TRAFFIC_DECODE_BYTES}}
        if not args.no_decode16:
            # the same KV cache read for 16 query positions per head at once (speculative decoding,
            # a short chunk): (Hq / Hkv) * Lq = 64 rows per kv head, past the decode kernel's 32, so
            # the tile kernel runs it with the heads of a kv group as one head, key range split
            gen = torch.Generator().manual_seed(wd.seed + 16)
            q16 = torch.randn((wd.B, wd.Hq, 16, wd.d), generator=gen).to(qg.dtype).cuda()
            o16 = torch.empty_like(q16)

            def step_16(_):
                flashd.attn_fwd(q16, kg, vg, o16, True, wd.scale)
            _, ev16 = time_calls(step_16, dsteps, 5, 1)
            ms16 = ev16 / dsteps
            bytes16 = (kg.numel() + vg.numel() + 2 * q16.numel()) * kg.element_size()
            gbs16 = bytes16 / (ms16 * 1e-3) / 1e9
            out["decode_16_positions"] = {"ms_per_step": round(ms16, 4), "bytes_per_step": bytes16,
                                          "roofline": {"bound": "hbm", "achieved": round(gbs16, 1),
                                                       "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                                       "frac": round(gbs16 / PEAK_HBM_GBS, 4),
                                                       "traffic": None}}
            del q16, o16
        if not args.no_kv8:
            # the same decode workload with K and V stored as fp8 (flashd_attn_fwd_kv8)
            ks_, vs_ = 2.0 ** -5, 2.0 ** -5
            k8 = (kd.float() / ks_).to(torch.float8_e4m3fn).cuda()
            v8 = (vd.float() / vs_).to(torch.float8_e4m3fn).cuda()

            def step_kv8(_):
                flashd.attn_fwd_kv8(qg, k8, v8, og, wd.causal, wd.scale, ks_, vs_)
            _, ev8 = time_calls(step_kv8, dsteps, 5, 1)
            ms8 = ev8 / dsteps
            bytes8 = k8.numel() + v8.numel() + 2 * qg.numel() * qg.element_size()
            gbs8 = bytes8 / (ms8 * 1e-3) / 1e9
            out["decode_fp8_kv"] = {"ms_per_step": round(ms8, 4), "bytes_per_step": bytes8,
                                    "speedup_vs_bf16_kv": round(dms / ms8, 3),
                                    "roofline": {"bound": "hbm", "achieved": round(gbs8, 1),
                                                 "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                                 "frac": round(gbs8 / PEAK_HBM_GBS, 4),
                                                 "traffic": None}}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
