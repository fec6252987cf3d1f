#!/usr/bin/env python3
"""Benchmark of the hybrid key-switching hot path on one MI355X.

Default workload: the bootstrapping-level key-switch (N = 2^16, L = 24 ciphertext primes, K = 8 special
primes, dnum = 3, one ciphertext per call).  A "step" is one ks_keyswitch call, i.e. the whole chain INTT,
ModUp base conversion, NTT, inner product with the evaluation key, INTT, ModDown base conversion, NTT and
the final subtract-and-scale.  All inputs are resident in HBM before the timed region.  To keep the 256 MB
last-level cache from flattering the number, steps rotate over several disjoint sets of (d, evk, out,
workspace); `hot_value` reports the single-set figure next to it.

Prints ONE JSON line.  `roofline` describes the kernel with the largest share of the step time: its
algorithmic bytes (what one launch must read plus write) divided by its average duration, measured with
HIP events on the launch stream in a separate instrumented pass over the same workload.
`cpu_baseline` is the plain-C reference timed on this machine's host cores on a bounded sample.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP64_VECTOR_PEAK_TFLOPS = 78.6   # 256 CU x 4 SIMD x 16 lanes x 2 flop x 2.4 GHz
MIB = 1024.0 * 1024.0
GIB = 1024.0 * MIB
CHUNK = 8                        # ciphertexts per internal pass of the batched pipelines (the key is read once per chunk)

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (profiles/keyswitch_cfg2_hbm_traffic.txt,
# "measured" column: FETCH_SIZE and WRITE_SIZE scaled by what the same counters read for a 1 GiB device copy, summed, per
# launch), keyed by workload and kernel.  tests/test_profiles_consistent.py checks these against that file.
MEASURED_TRAFFIC_BYTES: dict = {
    ("keyswitch", "rows_inner_product"): 178500631,
    ("keyswitch", "rows_moddown_finish"): 68023405,
    ("keyswitch", "bconv_mfma_ntt_cols"): 53443678,  # mean of the ModUp and the ModDown launch
    ("keyswitch", "ntt_inv_rows"): 27089621,
    ("keyswitch", "ntt_inv_cols"): 21370488,         # mean of the 24-limb and the 16-limb launch
}

# Algorithmic bytes of the other workloads (fused-plan accounting: every transform = two passes over its limbs, base
# conversion and products fused into them, keys read once per chunk of ciphertexts), per unit of work.
CFG3_BYTES_PER_CALL = 222.5 * GIB          # 64 ciphertexts x 16 hoisted rotations
CFG4_BYTES_PER_DIRECTION = 2 * 2 * 1920 * 65536 * 8.0   # 1920 limb transforms, two passes, read + write
CFG5_BYTES_PER_HMULT = 698.0 * MIB


def _keyswitch_bytes(L, K, dnum, N, batch=1):
    """Algorithmic traffic of one key-switch in bytes: compulsory (read d and the key, write out) and the
    fused-plan model (every transform = two passes over its limbs, base conversion and products fused).  In a batched
    call the key is read once per chunk of min(batch, 8) ciphertexts, so each ciphertext is charged that share of it."""
    limb = N * 8
    alpha = -(-L // dnum)
    E = L + K
    new_limbs = sum(E - (min((j + 1) * alpha, L) - j * alpha) for j in range(dnum))
    key_limbs = dnum * 2 * E / min(batch, CHUNK)
    compulsory = (L + key_limbs + 2 * L) * limb
    fused = (2 * L                                       # INTT rows
             + L + new_limbs                             # INTT cols + conversion + NTT cols
             + new_limbs + L + key_limbs + 2 * E         # NTT rows + inner product
             + 2 * 2 * K                                 # INTT rows of special limbs
             + 2 * K + 2 * L                             # INTT cols + conversion + NTT cols
             + 2 * L + 2 * L + 2 * L) * limb             # NTT rows + subtract-scale
    return compulsory, fused


def _keyswitch_bytes_moved(L, K, dnum, N, batch=1):
    """What the library's chain moves per key-switch: the fused-plan model with the ciphertext limbs of both
    accumulators written and read back as 5-byte packed residues instead of 8-byte words (2 * 2 * L limbs at 3/8 less)."""
    return _keyswitch_bytes(L, K, dnum, N, batch)[1] - 2 * 2 * L * N * 3.0


def _apply_options(ctx, args):
    """--opt ID=VALUE pairs: tuning options of the context (see ks_ctx_set_option)."""
    for item in args.opt or []:
        k, v = item.split("=")
        ctx.set_option(int(k), int(v))


def _median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2] if len(xs) % 2 else 0.5 * (xs[len(xs) // 2 - 1] + xs[len(xs) // 2])


def _event_timed(torch, issue, calls):
    """Milliseconds per call of `calls` back-to-back calls on the current stream (HIP events around the lot)."""
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    issue(calls)
    t1.record()
    torch.cuda.synchronize()
    return t0.elapsed_time(t1) / calls


def bench_keyswitch(args, torch, K, ks_inputs):
    cfg = ks_inputs.CONFIGS[2]
    q, p = ks_inputs.moduli(cfg)
    logN, L, Kk, dnum = cfg["logN"], cfg["L"], cfg["K"], cfg["dnum"]
    N = 1 << logN
    ctx = K.Context(logN, q, p, dnum)
    _apply_options(ctx, args)
    ws_words = K.ks_workspace_bytes(ctx, K.KS_OP_KEYSWITCH, L, 1) // 8
    sets = []
    for s in range(args.sets):
        d = ks_inputs.uniform_residues(cfg["seed"], 100 * s + 1, (1,), q, N, device="cuda")
        evk = ks_inputs.uniform_residues(cfg["seed"], 100 * s + 2, (dnum, 2), q + p, N, device="cuda")
        out = torch.empty((1, 2, L, N), dtype=torch.int64, device="cuda")
        ws = torch.empty(ws_words, dtype=torch.int64, device="cuda")
        sets.append((d, evk, out, ws))
    state = {"i": 0}

    def run(n, rotate=True):
        for _ in range(n):
            d, evk, out, ws = sets[state["i"] % len(sets)] if rotate else sets[0]
            state["i"] += 1
            K.ks_keyswitch(ctx, d, L, evk, out, ws)

    # Timing protocol: W warm-up calls, then `repeats` runs of max(K, 200) calls each, HIP events around each run;
    # the headline is the MEDIAN run.  The run of exactly K calls the command line asks for is reported beside it.
    calls = max(args.steps, args.min_calls)
    run(args.warmup)
    exact_k = _event_timed(torch, run, args.steps)
    runs = [_event_timed(torch, run, calls) for _ in range(args.repeats)]
    ms = _median(runs)
    run(args.warmup, False)
    ms_hot = _median([_event_timed(torch, lambda n: run(n, False), calls) for _ in range(3)])

    def timed_streams(n, n_streams):
        """Independent key-switches issued round-robin on several streams (default priority), wall-clocked between
        device-wide synchronisations over at least 200 calls: a serving loop with several requests in flight."""
        streams = [torch.cuda.Stream() for _ in range(n_streams)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            with torch.cuda.stream(streams[i % n_streams]):
                d, evk, out, ws = sets[i % len(sets)]
                K.ks_keyswitch(ctx, d, L, evk, out, ws)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    ms_streams = {}
    if args.sets >= 2 and not args.no_batched:
        for ns in (2, 3):
            if ns <= args.sets:
                timed_streams(max(args.warmup, 30), ns)
                trials = [timed_streams(calls, ns) for _ in range(3)]
                ms_streams[ns] = {"median": _median(trials), "best": min(trials), "worst": max(trials)}

    # the same key-switch over a batch of independent ciphertexts in one call (one key): what a serving loop or an
    # encrypted matrix product issues; every launch then fills the chip
    batched = {}
    for nb in (() if args.no_batched else (16,)):
        d_b = ks_inputs.uniform_residues(cfg["seed"], 7001, (nb,), q, N, device="cuda")
        out_b = torch.empty((nb, 2, L, N), dtype=torch.int64, device="cuda")
        ws_b = torch.empty(K.ks_workspace_bytes(ctx, K.KS_OP_KEYSWITCH, L, nb) // 8, dtype=torch.int64, device="cuda")
        issue = lambda n: [K.ks_keyswitch(ctx, d_b, L, sets[0][1], out_b, ws_b) for _ in range(n)]
        issue(2)
        reps = max(13, calls // nb)                      # at least 200 key-switches per run
        batched[nb] = _median([_event_timed(torch, issue, reps) for _ in range(3)]) / nb
        del d_b, out_b, ws_b

    # instrumented pass: per-kernel durations from HIP events recorded by the library on the launch stream
    K.ks_profile_enable(True)
    prof_steps = 24
    run(prof_steps)
    torch.cuda.synchronize()
    kernels = K.ks_profile_report()
    K.ks_profile_enable(False)
    for k in kernels:
        k["avg_us"] = 1000.0 * k["total_ms"] / k["launches"]
        k["ms_per_step"] = k["total_ms"] / prof_steps
        k["achieved_GBs"] = k["total_bytes"] / (k["total_ms"] * 1e-3) / 1e9
        k["bytes_per_launch"] = k["total_bytes"] / k["launches"]
        # fp64 vector instruction slots, priced as FMA slots against the 78.6 TFLOP/s vector peak
        k["achieved_TFLOPs"] = 2.0 * k.get("total_ops", 0.0) / (k["total_ms"] * 1e-3) / 1e12
        k["hbm_frac"] = k["achieved_GBs"] / HBM_PEAK_GBS
        k["alu_frac"] = k["achieved_TFLOPs"] / FP64_VECTOR_PEAK_TFLOPS
    dom = max(kernels, key=lambda k: k["total_ms"])
    traffic = MEASURED_TRAFFIC_BYTES.get(("keyswitch", dom["kernel"]))
    if dom["alu_frac"] > dom["hbm_frac"]:
        roofline = {"bound": "alu", "kernel": dom["kernel"], "achieved": round(dom["achieved_TFLOPs"], 2),
                    "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(dom["alu_frac"], 4), "traffic": traffic,
                    "algorithmic_ops_per_launch": dom["total_ops"] / dom["launches"]}
    else:
        roofline = {"bound": "hbm", "kernel": dom["kernel"], "achieved": round(dom["achieved_GBs"], 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(dom["hbm_frac"], 4), "traffic": traffic}
    roofline.update({"algorithmic_bytes_per_launch": dom["bytes_per_launch"], "avg_launch_us": round(dom["avg_us"], 2),
                     "launches_per_step": dom["launches"] / prof_steps})
    compulsory, fused = _keyswitch_bytes(L, Kk, dnum, N)
    # what a plain device copy of 1 GiB reaches on this GPU: the practical ceiling beside the 8 TB/s data-sheet peak
    copy_gbs = bench_copy(args, torch)["value"] if not args.no_batched else None
    frac = lambda nbytes, t_ms: round(nbytes / (t_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    path = {"fused_plan_MiB": fused / MIB, "compulsory_MiB": compulsory / MIB,
            "fused_plan_GBs": round(fused / (ms * 1e-3) / 1e9, 1), "fused_plan_frac_of_peak": frac(fused, ms),
            "target_frac_of_peak": 0.60,
            # the same with the packed accumulator limbs counted at their 5 bytes: the bytes the chain really moves
            "moved_MiB": round(_keyswitch_bytes_moved(L, Kk, dnum, N) / MIB, 1),
            "moved_frac_of_peak": frac(_keyswitch_bytes_moved(L, Kk, dnum, N), ms),
            "compulsory_GBs": round(compulsory / (ms * 1e-3) / 1e9, 1),
            "sum_kernel_ms_per_step": round(sum(k["ms_per_step"] for k in kernels), 4),
            # algorithmic traffic per ciphertext of a batched call, the key charged once per chunk of 8 (part of this
            # traffic is served by the last-level cache: one key and one workspace are reused by the whole batch)
            "batched_fused_plan_MiB_per_keyswitch": {str(nb): round(_keyswitch_bytes(L, Kk, dnum, N, nb)[1] / MIB, 1) for nb in batched},
            "batched_fused_plan_frac_of_peak": {str(nb): frac(_keyswitch_bytes(L, Kk, dnum, N, nb)[1], v) for nb, v in batched.items()},
            "device_copy_GBs": copy_gbs,
            "fused_plan_frac_of_device_copy": round(fused / (ms * 1e-3) / 1e9 / copy_gbs, 4) if copy_gbs else None}
    result = {
        "metric": "key_switches_per_sec", "value": round(1000.0 / ms, 2), "unit": "key-switch/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "bootstrap-keyswitch N=2^16 L=24 K=8 dnum=3 batch=1 (36-bit primes in 64-bit words)",
                   "buffer_sets_rotated": args.sets},
        "timing": {"protocol": "median of repeats; each repeat = calls_per_repeat back-to-back calls between two HIP events",
                   "repeats": args.repeats, "calls_per_repeat": calls, "ms_per_step_min": round(min(runs), 5),
                   "ms_per_step_max": round(max(runs), 5), "ms_per_step_exactly_steps_calls": round(exact_k, 5)},
        "hot_value": round(1000.0 / ms_hot, 2),
        "multi_stream_value": {str(ns): {k2: round(1000.0 / v2, 2) for k2, v2 in v.items()} for ns, v in ms_streams.items()},
        "batched_value": {str(nb): round(1000.0 / v, 2) for nb, v in batched.items()},
        "roofline": roofline, "path": path,
        "kernels": [{"kernel": k["kernel"], "launches_per_step": k["launches"] / prof_steps, "avg_us": round(k["avg_us"], 2),
                     "ms_per_step": round(k["ms_per_step"], 4), "achieved_GBs": round(k["achieved_GBs"], 1),
                     "hbm_frac": round(k["hbm_frac"], 3), "alu_frac": round(k["alu_frac"], 3)} for k in kernels],
        "paper_context": "paper reports only end-to-end times on NVIDIA GPUs (bootstrapping 7.5 ms on 8xB200, BERT-Base 8.8 s, "
                         "Llama3-8B 134 s); no per-key-switch figure exists to compare with",
    }
    first = sets[0]
    del sets
    return result, (cfg, q, p, first)


def other_workloads(args, torch, K, ks_inputs):
    """Configurations 3, 4 and 5 in the same run, compactly: throughput and the fraction of the HBM peak their
    algorithmic (fused-plan) bytes move at.  Few repetitions: the calls are tens of milliseconds long."""
    import copy
    import gc
    a = copy.copy(args)
    a.steps = 120
    out = {}

    def compact(r, nbytes_per_ms_step):
        gbs = nbytes_per_ms_step / (r["ms_per_step"] * 1e-3) / 1e9
        return {"value": r["value"], "unit": r["unit"], "ms_per_call": r["ms_per_step"], "workload": r["config"]["workload"],
                "algorithmic_GBs": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}

    for name, fn, nbytes in (("cfg3_hoisted_rotations", lambda: bench_rotate(a, torch, K, ks_inputs), CFG3_BYTES_PER_CALL),
                             ("cfg4_batched_ntt", lambda: bench_ntt(a, torch, K, ks_inputs), 2 * CFG4_BYTES_PER_DIRECTION),
                             ("cfg5_hmult", lambda: bench_hmult(a, torch, K, ks_inputs), 256 * CFG5_BYTES_PER_HMULT),
                             ("cfg5_hmult_moddown_merged", lambda: bench_hmult(a, torch, K, ks_inputs, merged=True), 256 * CFG5_BYTES_PER_HMULT)):
        out[name] = compact(fn(), nbytes)
        gc.collect()
        torch.cuda.empty_cache()
    return out


def cpu_baseline_keyswitch(cfg, q, p, first_set, ks_inputs, budget_s=12.0):
    """The plain-C reference as it stands on this machine's host cores: all cores, then one thread."""
    import ctypes
    from oracle import c_tier
    from oracle import ckks_ref as R
    logN, dnum = cfg["logN"], cfg["dnum"]
    ref = c_tier.COracle(logN, q, p, dnum, [R.minimal_psi(m, logN) for m in q + p])
    d = ks_inputs.as_u64(first_set[0])
    evk = ks_inputs.as_u64(first_set[1])
    ref.keyswitch(d, evk)                       # warm the tables / page in
    cores = c_tier.max_threads()
    n, t0 = 0, time.time()
    while n < 4 or (time.time() - t0 < budget_s and n < 200):
        ref.keyswitch(d, evk)
        n += 1
    dt = time.time() - t0
    single = None
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
        gomp.omp_set_num_threads(1)
        n1, t1 = 0, time.time()
        while n1 < 2 or (time.time() - t1 < 6.0 and n1 < 20):
            ref.keyswitch(d, evk)
            n1 += 1
        single = {"value": round(n1 / (time.time() - t1), 3), "cores": 1, "sample": f"{n1} key-switches"}
        gomp.omp_set_num_threads(cores)
    except OSError:
        pass
    return {"value": round(n / dt, 3), "unit": "key-switch/s", "cores": cores, "kind": "oracle",
            "sample": f"{n} key-switches of the same workload (same seeded d and evk), {dt:.1f} s wall", "single_thread": single}


def _kernel_breakdown(K, torch, fn, units):
    """Run fn once with the library's event instrumentation on; per-kernel time per unit of work and rooflines."""
    K.ks_profile_enable(True)
    fn()
    torch.cuda.synchronize()
    kernels = K.ks_profile_report()
    K.ks_profile_enable(False)
    out = []
    for k in kernels:
        gbs = k["total_bytes"] / (k["total_ms"] * 1e-3) / 1e9
        tfl = 2.0 * k.get("total_ops", 0.0) / (k["total_ms"] * 1e-3) / 1e12
        out.append({"kernel": k["kernel"], "launches": k["launches"], "us_per_unit": round(k["total_ms"] * 1e3 / units, 3),
                    "achieved_GBs": round(gbs, 1), "hbm_frac": round(gbs / HBM_PEAK_GBS, 3),
                    "alu_frac": round(tfl / FP64_VECTOR_PEAK_TFLOPS, 3), "total_ms": k["total_ms"]})
    return out


def _dominant_roofline(kernels):
    dom = max(kernels, key=lambda k: k["total_ms"])
    if dom["alu_frac"] > dom["hbm_frac"]:
        rl = {"bound": "alu", "kernel": dom["kernel"], "achieved": round(dom["alu_frac"] * FP64_VECTOR_PEAK_TFLOPS, 2),
              "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": dom["alu_frac"], "traffic": None}
    else:
        rl = {"bound": "hbm", "kernel": dom["kernel"], "achieved": dom["achieved_GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
              "frac": dom["hbm_frac"], "traffic": None}
    for k in kernels:
        k.pop("total_ms", None)
    return rl


def _time_calls(torch, fn, reps):
    fn()
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for _ in range(reps):
        fn()
    t1.record()
    torch.cuda.synchronize()
    return t0.elapsed_time(t1) / reps


def _words(args, torch, cfg):
    """(cfg, dtype, narrow, tag) for the word size asked for: 64-bit words with the configuration's own primes, or the
    paper's word size (28-bit primes, one residue per 32-bit word) through the _u32 entry points."""
    if args.word_size == 32:
        return dict(cfg, bits=28), torch.int32, (lambda t: None if t is None else t.to(torch.int32)), ", 28-bit primes in 32-bit words"
    return cfg, torch.int64, (lambda t: t), ""


def bench_keyswitch_u32(args, torch, K, ks_inputs):
    """Configuration 2's shape with the paper's word size: 28-bit primes, d / key / result in 32-bit words."""
    cfg = dict(ks_inputs.CONFIGS[2], bits=28)
    q, p = ks_inputs.moduli(cfg)
    logN, L, Kk, dnum = cfg["logN"], cfg["L"], cfg["K"], cfg["dnum"]
    N = 1 << logN
    ctx = K.Context(logN, q, p, dnum)
    _apply_options(ctx, args)
    i32 = lambda t: t.to(torch.int32)
    sets = []
    for sidx in range(args.sets):
        d = i32(ks_inputs.uniform_residues(cfg["seed"], 100 * sidx + 1, (1,), q, N, device="cuda"))
        evk = i32(ks_inputs.uniform_residues(cfg["seed"], 100 * sidx + 2, (dnum, 2), q + p, N, device="cuda"))
        out = torch.empty((1, 2, L, N), dtype=torch.int32, device="cuda")
        ws = torch.empty(K.ks_workspace_bytes(ctx, K.KS_OP_KEYSWITCH, L, 1) // 8, dtype=torch.int64, device="cuda")
        sets.append((d, evk, out, ws))
    state = {"i": 0}

    def one():
        d, evk, out, ws = sets[state["i"] % len(sets)]
        state["i"] += 1
        K.ks_keyswitch_u32(ctx, d, L, evk, out, ws)

    for _ in range(args.warmup):
        one()
    ms = _time_calls(torch, one, args.steps)
    nb = 16
    d_b = i32(ks_inputs.uniform_residues(cfg["seed"], 7001, (nb,), q, N, device="cuda"))
    out_b = torch.empty((nb, 2, L, N), dtype=torch.int32, device="cuda")
    ws_b = torch.empty(K.ks_workspace_bytes(ctx, K.KS_OP_KEYSWITCH, L, nb) // 8, dtype=torch.int64, device="cuda")
    batched = lambda: K.ks_keyswitch_u32(ctx, d_b, L, sets[0][1], out_b, ws_b)
    ms_b = _time_calls(torch, batched, max(2, min(20, args.steps // nb + 1))) / nb
    kernels = _kernel_breakdown(K, torch, lambda: [one() for _ in range(24)], 24)
    return {"metric": "key_switches_per_sec", "value": round(1000.0 / ms, 2), "unit": "key-switch/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f64", "data": "synthetic", "batched_value": {str(nb): round(1000.0 / ms_b, 2)},
            "config": {"workload": "bootstrap-keyswitch N=2^16 L=24 K=8 dnum=3 batch=1, 28-bit primes, d / key / result in 32-bit words",
                       "buffer_sets_rotated": args.sets},
            "roofline": _dominant_roofline(kernels), "kernels": kernels}


def bench_rotate(args, torch, K, ks_inputs):
    """Configuration 3: 64 ciphertexts x 16 hoisted rotations per call (one ModUp per ciphertext, 16 rotation keys)."""
    cfg, dtype, narrow, tag = _words(args, torch, ks_inputs.CONFIGS[3])
    w32 = args.word_size == 32
    q, p = ks_inputs.moduli(cfg)
    logN, L, B, R, dnum = cfg["logN"], cfg["L"], cfg["batch"], cfg["n_rot"], cfg["dnum"]
    N = 1 << logN
    ctx = K.Context(logN, q, p, dnum)
    _apply_options(ctx, args)
    ct = narrow(ks_inputs.uniform_residues(cfg["seed"], 1, (B, 2), q, N, device="cuda"))
    keys = [narrow(ks_inputs.uniform_residues(cfg["seed"], 10 + r, (dnum, 2), q + p, N, device="cuda")) for r in range(R)]
    gal = ks_inputs.galois_elements(logN, R)
    out = torch.empty((B, R, 2, L, N), dtype=dtype, device="cuda")
    op = K.KS_OP_ROTATE_HOISTED_U32 if w32 else K.KS_OP_ROTATE_HOISTED
    ws = torch.empty(K.ks_workspace_bytes(ctx, op, L, B, R) // 8, dtype=torch.int64, device="cuda")
    entry = K.ks_rotate_hoisted_u32 if w32 else K.ks_rotate_hoisted
    fn = lambda: entry(ctx, ct, L, gal, keys, out, ws)
    reps = max(2, args.steps // 60)
    ms = _time_calls(torch, fn, reps)
    kernels = _kernel_breakdown(K, torch, fn, B * R)
    return {"metric": "rotations_per_sec", "value": round(B * R / (ms * 1e-3), 1), "unit": "rotation/s", "n_gpus": 1, "steps": reps,
            "warmup": 1, "ms_per_step": round(ms, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f64", "data": "synthetic",
            "config": {"workload": "hoisted-rotations N=2^16 L=24 K=8 dnum=3, 64 ciphertexts x 16 Galois elements per call" + tag},
            "roofline": _dominant_roofline(kernels), "kernels": kernels}


def bench_rotate_mac(args, torch, K, ks_inputs):
    """Configuration 3's shape through the double-hoisted entry point: per ciphertext the 16 rotations are multiplied by
    plaintext diagonals and summed on the extended basis, with one division by P for the sum."""
    cfg, dtype, narrow, tag = _words(args, torch, ks_inputs.CONFIGS[3])
    w32 = args.word_size == 32
    q, p = ks_inputs.moduli(cfg)
    logN, L, B, R, dnum = cfg["logN"], cfg["L"], cfg["batch"], cfg["n_rot"], cfg["dnum"]
    N = 1 << logN
    ctx = K.Context(logN, q, p, dnum)
    _apply_options(ctx, args)
    ct = narrow(ks_inputs.uniform_residues(cfg["seed"], 1, (B, 2), q, N, device="cuda"))
    keys = [narrow(ks_inputs.uniform_residues(cfg["seed"], 10 + r, (dnum, 2), q + p, N, device="cuda")) for r in range(R)]
    pts = [narrow(ks_inputs.uniform_residues(cfg["seed"], 100 + r, (), q + p, N, device="cuda")) for r in range(R)]
    gal = ks_inputs.galois_elements(logN, R)
    out = torch.empty((B, 2, L, N), dtype=dtype, device="cuda")
    op = K.KS_OP_ROTATE_HOISTED_U32 if w32 else K.KS_OP_ROTATE_HOISTED
    ws = torch.empty(K.ks_workspace_bytes(ctx, op, L, B, R) // 8, dtype=torch.int64, device="cuda")
    entry = K.ks_rotate_mac_hoisted_u32 if w32 else K.ks_rotate_mac_hoisted
    fn = lambda: entry(ctx, ct, L, gal, keys, pts, out, ws)
    reps = max(2, args.steps // 30)
    ms = _time_calls(torch, fn, reps)
    kernels = _kernel_breakdown(K, torch, fn, B * R)
    return {"metric": "rotations_per_sec", "value": round(B * R / (ms * 1e-3), 1), "unit": "rotation/s", "n_gpus": 1, "steps": reps,
            "warmup": 1, "ms_per_step": round(ms, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f64", "data": "synthetic",
            "config": {"workload": "double-hoisted rotate-multiply-accumulate N=2^16 L=24 K=8 dnum=3, 64 ciphertexts x 16 Galois "
                                   "elements per call, one ModDown per ciphertext" + tag},
            "roofline": _dominant_roofline(kernels), "kernels": kernels}


def bench_bsgs(args, torch, K, ks_inputs):
    """Baby-step giant-step linear transform with configuration 3's parameters: 64 ciphertexts, 16 x 16 = 256 plaintext
    diagonals per ciphertext (rotation 0 of either level is the identity and needs no key)."""
    cfg, dtype, narrow, tag = _words(args, torch, ks_inputs.CONFIGS[3])
    w32 = args.word_size == 32
    q, p = ks_inputs.moduli(cfg)
    logN, L, B, dnum = cfg["logN"], cfg["L"], cfg["batch"], cfg["dnum"]
    n1 = n2 = 16
    N = 1 << logN
    ctx = K.Context(logN, q, p, dnum)
    _apply_options(ctx, args)
    gal = ks_inputs.galois_elements(logN, n1 + n2)
    baby, giant = [1] + gal[:n1 - 1], [1] + gal[n1:n1 + n2 - 1]
    key = lambda tid, g: None if g == 1 else narrow(ks_inputs.uniform_residues(cfg["seed"], tid, (dnum, 2), q + p, N, device="cuda"))
    bkeys = [key(10 + i, g) for i, g in enumerate(baby)]
    gkeys = [key(40 + i, g) for i, g in enumerate(giant)]
    pts = [[narrow(ks_inputs.uniform_residues(cfg["seed"], 100 + g * n1 + b, (), q + p, N, device="cuda")) for b in range(n1)]
           for g in range(n2)]
    ct = narrow(ks_inputs.uniform_residues(cfg["seed"], 1, (B, 2), q, N, device="cuda"))
    out = torch.empty((B, 2, L, N), dtype=dtype, device="cuda")
    ws = torch.empty(K.ks_workspace_bytes(ctx, K.KS_OP_BSGS_U32 if w32 else K.KS_OP_BSGS, L, B) // 8, dtype=torch.int64, device="cuda")
    entry = K.ks_bsgs_linear_transform_u32 if w32 else K.ks_bsgs_linear_transform
    fn = lambda: entry(ctx, ct, L, baby, bkeys, giant, gkeys, pts, out, ws)
    reps = max(2, args.steps // 100)
    ms = _time_calls(torch, fn, reps)
    kernels = _kernel_breakdown(K, torch, fn, B * n1 * n2)
    return {"metric": "bsgs_diagonal_terms_per_sec", "value": round(B * n1 * n2 / (ms * 1e-3), 1), "unit": "rotated-and-multiplied term/s",
            "n_gpus": 1, "steps": reps, "warmup": 1, "ms_per_step": round(ms, 3), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f64", "data": "synthetic", "transforms_per_sec": round(B / (ms * 1e-3), 1),
            "config": {"workload": "bsgs linear transform N=2^16 L=24 K=8 dnum=3, 64 ciphertexts x (16 baby x 16 giant) diagonals per call" + tag},
            "roofline": _dominant_roofline(kernels), "kernels": kernels}


def bench_hmult(args, torch, K, ks_inputs, merged=False):
    """Configuration 5: 256 ciphertext pairs per call: tensor product, relinearisation, rescale (merged: the division
    by P and the rescale done as one division by P q_last)."""
    cfg, dtype, narrow, tag = _words(args, torch, ks_inputs.CONFIGS[5])
    q, p = ks_inputs.moduli(cfg)
    logN, L, B, dnum = cfg["logN"], cfg["L"], cfg["batch"], cfg["dnum"]
    N = 1 << logN
    ctx = K.Context(logN, q, p, dnum)
    _apply_options(ctx, args)
    cta = narrow(ks_inputs.uniform_residues(cfg["seed"], 1, (B, 2), q, N, device="cuda"))
    ctb = narrow(ks_inputs.uniform_residues(cfg["seed"], 2, (B, 2), q, N, device="cuda"))
    rlk = narrow(ks_inputs.uniform_residues(cfg["seed"], 3, (dnum, 2), q + p, N, device="cuda"))
    out = torch.empty((B, 2, L - 1, N), dtype=dtype, device="cuda")
    ws = torch.empty(K.ks_workspace_bytes(ctx, K.KS_OP_HMULT_RELIN_RESCALE, L, B) // 8, dtype=torch.int64, device="cuda")
    if args.word_size == 32:
        entry = K.hmult_relin_rescale_merged_u32 if merged else K.hmult_relin_rescale_u32
    else:
        entry = K.hmult_relin_rescale_merged if merged else K.hmult_relin_rescale
    fn = lambda: entry(ctx, cta, ctb, L, rlk, out, ws)
    reps = max(2, args.steps // 60)
    ms = _time_calls(torch, fn, reps)
    kernels = _kernel_breakdown(K, torch, fn, B)
    return {"metric": "hmults_per_sec", "value": round(B / (ms * 1e-3), 1), "unit": "HMult+relin+rescale/s", "n_gpus": 1, "steps": reps,
            "warmup": 1, "ms_per_step": round(ms, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f64", "data": "synthetic",
            "config": {"workload": "hmult-relin-rescale N=2^16 L=35 K=12 dnum=3, 256 ciphertext pairs per call"
                                   + (", ModDown merged with rescale" if merged else "") + tag},
            "roofline": _dominant_roofline(kernels), "kernels": kernels}


def bench_ntt(args, torch, K, ks_inputs):
    cfg, dtype, narrow, tag = _words(args, torch, ks_inputs.CONFIGS[4])
    q, p = ks_inputs.moduli(cfg)
    logN, L, batch = cfg["logN"], cfg["L"], cfg["batch"]
    N = 1 << logN
    ctx = K.Context(logN, q, p, 1)
    _apply_options(ctx, args)
    ids = list(range(L))
    data = narrow(ks_inputs.uniform_residues(cfg["seed"], 1, (batch,), q, N, device="cuda"))
    fwd, inv = (K.ntt_fwd_u32, K.ntt_inv_u32) if args.word_size == 32 else (K.ntt_fwd, K.ntt_inv)
    fwd(ctx, data, ids)
    inv(ctx, data, ids)
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    steps = max(2, args.steps // 10)
    t0.record()
    for _ in range(steps):
        fwd(ctx, data, ids)
        inv(ctx, data, ids)
    t1.record()
    torch.cuda.synchronize()
    ms = t0.elapsed_time(t1) / steps
    limbs = 2 * L * batch
    bytes_one_pass = limbs * N * (args.word_size // 8) * 2.0
    kernels = _kernel_breakdown(K, torch, lambda: (fwd(ctx, data, ids), inv(ctx, data, ids)), limbs)
    _dominant_roofline(kernels)
    return {"metric": "limb_ntts_per_sec", "kernels": kernels, "value": round(limbs / (ms * 1e-3), 1), "unit": "limb-NTT/s (2^16 points)", "n_gpus": 1,
            "steps": steps, "warmup": 1, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f64", "data": "synthetic",
            "config": {"workload": "batched-ntt N=2^16 60 limbs x 32 polynomials, forward then inverse" + tag},
            "roofline": {"bound": "hbm", "kernel": "ntt_fwd+ntt_inv (two passes each)", "achieved": round(2 * bytes_one_pass / (ms * 1e-3) / 1e9, 1),
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(2 * bytes_one_pass / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                         "traffic": None}}


def bench_bconv(args, torch, K, ks_inputs):
    """The standalone base conversion at the two shapes the key-switch uses most (configuration 2's ModUp digit: 8 -> 24
    moduli; configuration 5's: 12 -> 35), vector kernel against the int8 matrix-core kernel, one polynomial and 64."""
    rows = []
    for cfg_id, n_src, n_dst in ((2, 8, 24), (5, 12, 35)):
        cfg = ks_inputs.CONFIGS[cfg_id]
        q, p = ks_inputs.moduli(cfg)
        logN = cfg["logN"]
        N = 1 << logN
        ctx = K.Context(logN, q, p, cfg["dnum"])
        src, dst = list(range(n_src)), list(range(n_src, n_src + n_dst))
        K.bconv_prepare(ctx, src, dst)
        for batch in (1, 64):
            x = ks_inputs.uniform_residues(cfg["seed"], 1, (batch,), [(q + p)[i] for i in src], N, device="cuda")
            out = torch.empty((batch, n_dst, N), dtype=torch.int64, device="cuda")
            row = {"shape": f"{n_src}->{n_dst} moduli, N=2^{logN}, {batch} polynomial(s)", "bytes": (n_src + n_dst) * batch * N * 8}
            for name, kernel in (("vector", 1), ("int8_mfma", 2)):
                ctx.set_option(K.KS_OPT_BCONV_KERNEL, kernel)
                fn = lambda: K.bconv(ctx, x, src, out, dst)
                fn()
                # kernel durations from the library's own HIP events (a single-polynomial launch is shorter than the
                # host-side cost of a call, so back-to-back wall time would measure the host)
                reps, trials = (100 if batch == 1 else 20), []
                for _ in range(3):
                    torch.cuda.synchronize()
                    K.ks_profile_enable(True)
                    for _ in range(reps):
                        fn()
                    torch.cuda.synchronize()
                    rec = K.ks_profile_report()
                    K.ks_profile_enable(False)
                    trials.append(sum(k["total_ms"] for k in rec) * 1e3 / reps)
                us = sorted(trials)[1]
                row[name + "_us"] = round(us, 2)
                row[name + "_GBs"] = round(row["bytes"] / (us * 1e-6) / 1e9, 1)
            ctx.set_option(K.KS_OPT_BCONV_KERNEL, 0)
            rows.append(row)
    big = rows[1]
    return {"metric": "bconv_GBps", "value": big["vector_GBs"], "unit": "GB/s", "n_gpus": 1, "steps": 20, "warmup": 1,
            "ms_per_step": round(big["vector_us"] * 1e-3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f64 (vector) / int8 (matrix cores)", "data": "synthetic",
            "config": {"workload": "standalone base conversion, vector kernel vs int8 matrix-core kernel"}, "shapes": rows,
            "roofline": {"bound": "hbm", "kernel": "bconv_kernel", "achieved": big["vector_GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(big["vector_GBs"] / HBM_PEAK_GBS, 4), "traffic": None}}


def bench_copy(args, torch):
    """A plain device copy of known size: the yardstick the HBM counters of the profiling runs are scaled by."""
    n = 1 << 27  # 1 GiB of int64
    a = torch.ones(n, dtype=torch.int64, device="cuda")
    b = torch.empty_like(a)
    b.copy_(a)
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for _ in range(10):
        b.copy_(a)
    t1.record()
    torch.cuda.synchronize()
    ms = t0.elapsed_time(t1) / 10
    return {"metric": "copy_GBps", "value": round(2 * n * 8 / (ms * 1e-3) / 1e9, 1), "unit": "GB/s", "n_gpus": 1, "steps": 10,
            "warmup": 1, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "int64", "data": "synthetic", "config": {"workload": "device copy, 1 GiB read + 1 GiB written per launch"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--sets", type=int, default=6, help="disjoint buffer sets rotated through (cold-cache figure)")
    ap.add_argument("--no-batched", action="store_true", help="skip the batched key-switch measurement (counter runs)")
    ap.add_argument("--workload", default="keyswitch", choices=["keyswitch", "keyswitch_u32", "ntt", "rotate", "rotate_mac", "bsgs", "hmult", "hmult_merged", "bconv", "copy"])
    ap.add_argument("--word-size", type=int, default=64, choices=[64, 32],
                    help="32: the rotate / rotate_mac / bsgs / hmult / hmult_merged / ntt workloads with 28-bit primes in 32-bit words")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--repeats", type=int, default=5, help="timed runs of the headline workload (the median is reported)")
    ap.add_argument("--min-calls", type=int, default=200,
                    help="calls per timed repeat are max(steps, this); counter-collection runs lower it to keep them short")
    ap.add_argument("--no-extras", action="store_true", help="skip configurations 3, 4 and 5 (profiling runs)")
    ap.add_argument("--opt", action="append", help="context tuning option ID=VALUE (ks_ctx_set_option), repeatable")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one key-switch stream on one MI355X); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import ks_inputs
    import paper_2512_11269_amd as K
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.workload == "copy":
        result = bench_copy(args, torch)
    elif args.workload == "bconv":
        result = bench_bconv(args, torch, K, ks_inputs)
    elif args.workload == "ntt":
        result = bench_ntt(args, torch, K, ks_inputs)
    elif args.workload == "keyswitch_u32":
        result = bench_keyswitch_u32(args, torch, K, ks_inputs)
    elif args.workload == "rotate":
        result = bench_rotate(args, torch, K, ks_inputs)
    elif args.workload == "rotate_mac":
        result = bench_rotate_mac(args, torch, K, ks_inputs)
    elif args.workload == "bsgs":
        result = bench_bsgs(args, torch, K, ks_inputs)
    elif args.workload in ("hmult", "hmult_merged"):
        result = bench_hmult(args, torch, K, ks_inputs, merged=args.workload == "hmult_merged")
    else:
        result, (cfg, q, p, first_set) = bench_keyswitch(args, torch, K, ks_inputs)
        if not args.no_cpu_baseline:
            result["cpu_baseline"] = cpu_baseline_keyswitch(cfg, q, p, first_set, ks_inputs)
        del first_set
        torch.cuda.empty_cache()
        if not (args.no_extras or args.no_batched):
            result["other_workloads"] = other_workloads(args, torch, K, ks_inputs)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
