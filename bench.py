"""Benchmark of the FLASH-D attention forward path on one MI355X.

A step is one flashd_attn_fwd call (the whole hot path: Q load, K/V streaming, scores,
mask, weight recurrence, blend, store) on the LLaMA-7B-like causal bf16 prefill workload;
the inputs are resident in HBM before the timed region and rotate over several independent
sets so that the last-level cache is not flattering.  One JSON line is printed.

The other four configurations ride in the same line: the long non-causal prefill and the fp16
stress prefill as legs of their own (kernel time, TFLOP/s, roofline, the Alg. 2 ablation and
the per-tile blend on the same inputs, parity against the oracle), the single fp32 head in
microseconds, the GQA decode with its HBM roofline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--settle-ms T] [--no-cpu] [--no-decode]
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import re
import sys
import time

import numpy as np
import torch

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16/fp16 matrix peak
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E peak
# profiles/ summary that holds the HBM traffic of each prefill configuration's kernel
PREFILL_PROFILE = {1: "wide_kernel_bf16_d128_causal_prefill.txt",
                   2: "wide_kernel_bf16_d128_long_noncausal_prefill.txt",
                   4: "tile_kernel_f16_d64_stress_prefill.txt"}
# fp32 vector peak as published (157.3 TFLOP/s: 256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz,
# doubled by packed issue).  This build compiles the packed fp32 instructions out, so what its
# plain fma code can reach is half of that, 78.6 TFLOP/s; both fractions are reported.
PEAK_FP32 = 157.3
PEAK_FP32_FMA = 78.6

# HBM-side bytes per launch of a kernel cannot be read from inside this process: they come from
# the profiler's FETCH_SIZE and WRITE_SIZE counters scaled by a 1 GiB device copy.  The
# summaries under profiles/ hold the commands, the raw readings and the line this function
# looks for; the JSON line names the file next to the figure ("traffic_source").
PROFILE_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles")


def profile_traffic(fname):
    """(bytes per launch, relative path) from a profiles/ summary, or (None, None)."""
    path = os.path.join(PROFILE_DIR, fname)
    try:
        for line in open(path):
            m = re.match(r"\s*HBM-side traffic per launch:\s*([0-9.]+)\s*MB", line)
            if m:
                return float(m.group(1)) * 1e6, "profiles/" + fname
    except OSError:
        pass
    return None, None



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


def make_sets(w, nsets):
    """nsets independent input sets of a workload on the GPU (set 0 is the workload's own seed)."""
    from paper_2505_14201_amd import synthetic
    host, sets = None, []
    for s in range(nsets):
        qs, ks, vs, _ = synthetic.make_qkv(w if s == 0 else dataclasses.replace(w, seed=w.seed + 100 * s))
        if s == 0:
            host = (qs, ks, vs)
        qg, kg, vg = qs.cuda(), ks.cuda(), vs.cuda()
        sets.append((qg, kg, vg, torch.empty_like(qg)))
    torch.cuda.synchronize()
    return host, sets


def oracle_leg(w, host, got, budget_flop=2.0e12):
    """Parity of `got` (GPU output for input set 0, CPU tensor) against the oracle, and the
    oracle's own speed.  Workloads above budget_flop are sampled by query rows (seeded, spread
    over all heads) so that the leg stays near 20 s on the machine's host cores."""
    from oracle import attention as oa
    q, k, v = host
    flops = w.flops()
    nrows_all = w.B * w.Hq * w.Lq
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
    g = got.double().numpy()
    if rows is not None:
        g = g[rows[:, 0], rows[:, 1], rows[:, 2]]
        vis = (np.clip(rows[:, 2] + (w.Lk - w.Lq) + 1, 0, w.Lk).sum() if w.causal
               else float(nrows) * w.Lk)
        cpu_flops = 4.0 * w.d * float(vis)
    else:
        cpu_flops = flops
    err = np.abs(g - ref)
    parity = {"max_abs_err": float(err.max()),
              "rel_rms_err": float(np.sqrt((err ** 2).sum() / (ref ** 2).sum())),
              "rows_checked": int(nrows)}
    cpu = {"value": round(cpu_flops / cpu_s / 1e12, 5), "unit": "TFLOP/s",
           "cores": oa.num_threads(), "kind": "oracle", "sample": what + ", fp64 definition",
           "seconds": round(cpu_s, 2)}
    return parity, cpu


def auto_variant(w):
    """The variant flashd_attn_fwd takes for this workload (the library's own answer)."""
    from paper_2505_14201_amd import flashd
    code = {"bf16": flashd.BF16, "f16": flashd.F16, "f32": flashd.F32}[w.dtype]
    return flashd.auto_variant(w.B, w.Hq, w.Hkv, w.Lq, w.Lk, w.d, code, w.causal)


def prefill_kernel_name(w):
    from paper_2505_14201_amd import flashd
    kern = "wide_kernel" if auto_variant(w) == flashd.VARIANT_TILE_256 else "tile_kernel"
    return "%s<%s,%d> (flashd_attn_fwd)" % (kern, w.dtype.upper(), w.d)


def variant_legs(w, sets, steps, warmup):
    """Kernel time of the Alg. 2 ablation, of the per-tile blend and (d = 128, where it applies)
    of the prefill kernel the automatic choice did not take (256 or 128 rows per workgroup) on
    the same inputs."""
    from paper_2505_14201_amd import flashd
    out = {}
    legs = [("ablation_online_softmax", flashd.VARIANT_ONLINE_SOFTMAX),
            ("tile_blend", flashd.VARIANT_TILE_BLEND)]
    if auto_variant(w) == flashd.VARIANT_TILE_256:
        legs.append(("tile_128_rows", flashd.VARIANT_TILE))
    elif w.d == 128:
        legs.append(("tile_256_rows", flashd.VARIANT_TILE_256))
    for key, var in legs:
        def step_var(i, var=var):
            qg, kg, vg, og = sets[i]
            flashd.attn_fwd_ex(qg, kg, vg, og, w.causal, w.scale, var, 1)
        _, ev = time_calls(step_var, steps, warmup, len(sets))
        out[key] = {"kernel_ms": round(ev / steps, 4),
                    "TFLOP/s": round(w.flops() / (ev / steps * 1e-3) / 1e12, 2)}
    return out


def prefill_leg(w, steps, warmup, nsets, profile, cpu=True, variants=True, budget_flop=2.0e12):
    """One prefill configuration other than the headline one: flashd_attn_fwd timed with HIP
    events on the launch stream, its roofline, the other variants, parity and oracle speed."""
    from paper_2505_14201_amd import flashd
    host, sets = make_sets(w, nsets)

    def step(i):
        qg, kg, vg, og = sets[i]
        flashd.attn_fwd(qg, kg, vg, og, w.causal, w.scale)
    _, ev = time_calls(step, steps, warmup, nsets)
    ms = ev / steps
    tf = w.flops() / (ms * 1e-3) / 1e12
    traffic, src = profile_traffic(profile) if profile else (None, None)
    leg = {"workload": w.name, "dtype": w.dtype, "steps": steps, "input_sets": nsets,
           "flop_per_step": w.flops(), "kernel_ms": round(ms, 4), "TFLOP/s": round(tf, 2),
           "roofline": {"bound": "mfma",
                        "kernel": prefill_kernel_name(w),
                        "achieved": round(tf, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(tf / PEAK_BF16_TFLOPS, 4), "traffic": traffic,
                        "traffic_source": src}}
    if cpu:
        step(0)
        torch.cuda.synchronize()
        leg["parity"], leg["cpu_baseline"] = oracle_leg(w, host, sets[0][3].cpu(), budget_flop)
    if variants:
        leg.update(variant_legs(w, sets, steps, warmup))
    del sets
    torch.cuda.empty_cache()
    return leg


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
    ap.add_argument("--no-other-prefill", action="store_true",
                    help="skip the legs of the long non-causal, the stress and the single-head "
                         "configurations")
    ap.add_argument("--no-long-causal", action="store_true",
                    help="skip the leg of the causal mask at 16384 positions (not one of the "
                         "five configurations)")
    ap.add_argument("--no-kv8", action="store_true", help="skip the fp8 K/V decode measurement")
    ap.add_argument("--no-skipv", action="store_true",
                    help="skip the peaked-score decode measurement (saturation skip on V)")
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
    (q, k, v), sets = make_sets(w, args.sets)
    steps = args.steps if args.workload != 2 else min(args.steps, 50)    # 4 ms per step there

    def step(i):
        qg, kg, vg, og = sets[i]
        flashd.attn_fwd(qg, kg, vg, og, w.causal, w.scale)

    wall_ms, ev_ms = time_calls(step, steps, args.warmup, args.sets)
    ms_per_step = wall_ms / steps
    kern_ms = ev_ms / steps
    flops = w.flops()
    value = flops / (ms_per_step * 1e-3) / 1e12
    achieved = flops / (kern_ms * 1e-3) / 1e12
    traffic, traffic_src = profile_traffic(PREFILL_PROFILE[args.workload])

    out = {
        "metric": "attention fwd TFLOP/s (%s %s prefill, FLASH-D tile form: blend factor "
                  "carried per row as beta = 1 / sum 2^(s - R), applied at the store)"
                  % ("causal" if w.causal else "non-causal", w.dtype),
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": steps,
        "warmup": args.warmup, "settle_ms": args.settle_ms,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "Lq": w.Lq,
                   "Lk": w.Lk, "d": w.d, "causal": w.causal, "input_sets": args.sets,
                   "flop_per_step": flops},
        "roofline": {"bound": "mfma",
                     "kernel": prefill_kernel_name(w),
                     "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic, "traffic_source": traffic_src,
                     "kernel_ms": round(kern_ms, 4)},
    }

    # parity of what was just timed, against the oracle, and the oracle's own speed
    if not args.no_cpu:
        out["parity"], out["cpu_baseline"] = oracle_leg(w, (q, k, v), sets[0][3].cpu())

    if not args.no_ablation:
        out.update(variant_legs(w, sets, steps, args.warmup))

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
                    "roofline": {"bound": "alu", "achieved": round(tf, 2), "peak": PEAK_FP32,
                                 "unit": "TFLOP/s", "frac": round(tf / PEAK_FP32, 4),
                                 "frac_of_unpacked_fma_rate": round(tf / PEAK_FP32_FMA, 4)}}
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

    if not args.no_other_prefill and args.workload == 1:
        # the other two prefill configurations, each with its ablation, blend and parity legs
        out["prefill_c3"] = prefill_leg(synthetic.CONFIGS[2], min(args.steps, 40), 4, 2,
                                        PREFILL_PROFILE[2], cpu=not args.no_cpu,
                                        variants=not args.no_ablation)
        out["prefill_c5"] = prefill_leg(synthetic.CONFIGS[4], args.steps, args.warmup, args.sets,
                                        PREFILL_PROFILE[4], cpu=not args.no_cpu,
                                        variants=not args.no_ablation)
        # beside the five configurations: the causal mask at the length of the long workload
        # (one sequence of 16384 positions), where a row tile's fixed costs weigh less than at
        # the 2048 positions of the headline workload
        if not args.no_long_causal:
            wl = synthetic.small("x1_long_causal_prefill_bf16", 1, 32, 32, 16384, 16384, 128,
                                 "bf16", True, seed=1602)
            out["prefill_causal_16k"] = prefill_leg(wl, min(args.steps, 40), 4, 2, None,
                                                    cpu=not args.no_cpu, variants=False,
                                                    budget_flop=2.0e11)
        # the single fp32 head: launch-latency bound, reported in microseconds with its parity
        w1 = synthetic.CONFIGS[0]
        (q1, k1, v1), s1 = make_sets(w1, 1)

        def step_c1(_i):
            flashd.attn_fwd(s1[0][0], s1[0][1], s1[0][2], s1[0][3], w1.causal, w1.scale)
        n1 = max(1000, args.steps)
        wall1, ev1 = time_calls(step_c1, n1, 20, 1)
        leg = {"workload": w1.name, "dtype": w1.dtype, "steps": n1,
               "kernel": "perkey_kernel<F32,64> (flashd_attn_fwd)",
               "us_per_call_stream": round(ev1 / n1 * 1e3, 2),
               "us_per_call_wall": round(wall1 / n1 * 1e3, 2)}
        if not args.no_cpu:
            leg["parity"], leg["cpu_baseline"] = oracle_leg(w1, (q1, k1, v1), s1[0][3].cpu())
        out["c1_single_head_f32"] = leg
        del s1

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
        dec_traffic, dec_src = profile_traffic("decode_kernel_bf16_d128_gqa_decode.txt")
        out["decode"] = {"workload": wd.name, "ms_per_step": round(dms, 4),
                         "bytes_per_step": wd.bytes_io(),
                         "roofline": {"bound": "hbm", "achieved": round(gbs, 1),
                                      "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                      "frac": round(gbs / PEAK_HBM_GBS, 4),
                                      "traffic": dec_traffic, "traffic_source": dec_src}}
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
        if not args.no_decode16:
            # one sequence with a long context: 8 workgroups' worth of (b, kv head) units, so
            # the keys are split 64 ways and merge_splits_kernel folds the partial states
            gen = torch.Generator().manual_seed(wd.seed + 17)
            Ll = 131072
            q1 = torch.randn((1, wd.Hq, 1, wd.d), generator=gen).to(qg.dtype).cuda()
            k1 = torch.randn((1, wd.Hkv, Ll, wd.d), generator=gen).to(qg.dtype).cuda()
            v1 = torch.randn((1, wd.Hkv, Ll, wd.d), generator=gen).to(qg.dtype).cuda()
            o1 = torch.empty_like(q1)

            def step_long(_):
                flashd.attn_fwd(q1, k1, v1, o1, False, wd.scale)
            _, evl = time_calls(step_long, dsteps, 5, 1)
            msl = evl / dsteps
            bytesl = (k1.numel() + v1.numel() + 2 * q1.numel()) * k1.element_size()
            out["decode_single_sequence_128k"] = {
                "ms_per_step": round(msl, 4), "bytes_per_step": bytesl,
                "splits": flashd.auto_splits(1, wd.Hq, wd.Hkv, 1, Ll, wd.d, flashd.BF16),
                "roofline": {"bound": "hbm", "achieved": round(bytesl / (msl * 1e-3) / 1e9, 1),
                             "peak": PEAK_HBM_GBS, "unit": "GB/s",
                             "frac": round(bytesl / (msl * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                             "traffic": None}}
            del q1, k1, v1, o1
        if not args.no_skipv:
            # Saturation skip of Sec. III-C on the V fetch, on the decode shape with peaked
            # scores (a dominant early key per kv group): the kernel with and without the skip
            # on the same input, and how many 32-key blocks went without their V
            del qg, kg, vg, og
            torch.cuda.empty_cache()
            wp = synthetic.PEAKED_DECODE
            qp, kp, vp, _ = synthetic.make_qkv(wp)
            qg, kg, vg = qp.cuda(), kp.cuda(), vp.cuda()
            og = torch.empty_like(qg)
            cnt = torch.zeros(2, dtype=torch.int64, device="cuda")
            flashd.attn_fwd_skipv(qg, kg, vg, og, wp.causal, wp.scale, 1, None, cnt)
            torch.cuda.synchronize()
            visited, skipped = (int(x) for x in cnt.cpu())
            _, ev_ns = time_calls(lambda _i: flashd.attn_fwd_ex(qg, kg, vg, og, wp.causal, wp.scale,
                                                                flashd.VARIANT_TILE, 1),
                                  dsteps, 5, 1)
            _, ev_sk = time_calls(lambda _i: flashd.attn_fwd(qg, kg, vg, og, wp.causal, wp.scale),
                                  dsteps, 5, 1)
            ms_ns, ms_sk = ev_ns / dsteps, ev_sk / dsteps
            block_bytes = 32 * wp.d * 2
            fetched = wp.bytes_io() - skipped * block_bytes          # K, Q, O and the V blocks taken
            out["decode_peaked_skipv"] = {
                "workload": wp.name, "blocks_visited": visited, "v_blocks_not_fetched": skipped,
                "ms_per_step_unskipped": round(ms_ns, 4), "ms_per_step": round(ms_sk, 4),
                "speedup": round(ms_ns / ms_sk, 3), "bytes_algorithmic": wp.bytes_io(),
                "bytes_fetched_by_count": fetched,
                "GB/s_equivalent": round(wp.bytes_io() / (ms_sk * 1e-3) / 1e9, 1),
                "roofline": {"bound": "hbm", "achieved": round(fetched / (ms_sk * 1e-3) / 1e9, 1),
                             "peak": PEAK_HBM_GBS, "unit": "GB/s",
                             "frac": round(fetched / (ms_sk * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                             "traffic": None}}
            if not args.no_cpu:
                from oracle import attention as oa
                ref = oa.attn(qp, kp, vp, wp.causal, wp.scale)
                err = np.abs(og.cpu().double().numpy() - ref)
                out["decode_peaked_skipv"]["parity"] = {"max_abs_err": float(err.max())}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
