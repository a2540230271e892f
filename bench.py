#!/usr/bin/env python3
"""Benchmark of the EARS verification step on one MI355X.

A step is one whole `ears_verify_bf16` call (row statistics, decision scan, replacement / bonus
sampling) over one synthetic batch already resident in HBM.  Prints ONE JSON line on stdout.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
WORKLOAD_INDEX = 2              # B=256, K=8, V=128256, bf16: the configuration the metric is quoted on
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_row_stats_c2.json")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    for rel in ("paper_2512_13194_amd/csrc/row_stats.h", "paper_2512_13194_amd/csrc/ears_device.h"):
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic():
    """HBM bytes per row-statistics launch from the committed rocprofv3 counter runs, or None when
    there are none or the kernel source has changed since they were taken."""
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
    except OSError:
        return None
    if t.get("kernel_source_hash") != kernel_source_hash():
        return None
    return t.get("hbm_bytes_per_launch")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also run the plain copy kernel over a buffer of known size (for scaling "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU; sequences are independent, so more GPUs would "
            "each take a share of the batch with no exchange. Re-run with --gpus 1.")
        return 2

    import torch
    import paper_2512_13194_amd as ears
    from paper_2512_13194_amd import inputs

    ears.lib()                    # raises when libears.so is missing: there is no fallback path
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 3
    torch.cuda.set_device(0)
    cfg = inputs.CONFIGS[WORKLOAD_INDEX]
    B, K, V = cfg["B"], cfg["K"], cfg["V"]
    T = cfg["temperatures"][0]
    betas = cfg["betas"]
    seed0 = cfg["seed"]
    esz = 2
    log("generating workload %s on the GPU ..." % cfg["name"])
    batch = inputs.make_config(WORKLOAD_INDEX, device="cuda")
    acc = torch.empty(B, dtype=torch.int32, device="cuda")
    tok = torch.empty(B, K + 1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()

    def step(i):
        # beta cycles through the workload's sweep; the seed changes every step as it would
        # between decoding steps
        ears.ears_verify_bf16(batch.target, batch.draft, batch.tokens, T, betas[i % len(betas)],
                              seed0 + i, out_accept_len=acc, out_tokens=tok)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    positions_per_s = B * K / (ms_per_step * 1e-3)

    # algorithmic bytes of a whole call: every target row 0..K-1 and every draft row once, plus
    # the row pair (rejected) or the single bonus row (all accepted) the sampler re-reads
    rejected = []
    for i in range(len(betas)):
        step(i)
        torch.cuda.synchronize()
        rejected.append(int((acc < K).sum().item()))
    mean_rej = sum(rejected) / len(rejected)
    k1_bytes = 2 * B * K * V * esz
    call_bytes = k1_bytes + (2 * mean_rej + (B - mean_rej)) * V * esz
    call_gbps = call_bytes / (ms_per_step * 1e-3) / 1e9

    # dominant kernel: the row-statistics pass.  Its average launch duration is measured with HIP
    # events on the stream it is launched on (torch's current stream, which the binding passes to
    # the library): `steps` launches of the statistics stage back to back between two events, so
    # that the events' own cost is spread over all of them.
    ws = torch.empty(ears.ears_workspace_bytes(B * K, B, V), dtype=torch.uint8, device="cuda")

    def stats_only(i):
        ears.ears_verify_ex(batch.target, batch.draft, batch.tokens, temperature=T, beta=betas[0],
                            seed=seed0 + i, workspace=ws, stages=ears.EARS_STAGE_STATS,
                            out_accept_len=acc, out_tokens=tok.view(-1))

    for i in range(max(10, args.warmup)):   # the clock settles within a few launches
        stats_only(i)
    torch.cuda.synchronize()
    k0, k1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    k0.record()
    for i in range(args.steps):
        stats_only(i)
    k1.record()
    torch.cuda.synchronize()
    k1_ms = k0.elapsed_time(k1) / args.steps
    k1_gbps = k1_bytes / (k1_ms * 1e-3) / 1e9

    # practical ceiling: a read-only streaming kernel over one buffer that holds exactly the rows
    # the statistics kernel reads (target rows 0..K-1, then the draft rows), one launch per pass
    rows = torch.cat([batch.target[:, :K].reshape(-1), batch.draft.reshape(-1)])
    assert rows.numel() * esz == k1_bytes
    sink = None
    for _ in range(3):
        sink = ears.ears_bench_read(rows, sink)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    reps = 20
    for _ in range(reps):
        ears.ears_bench_read(rows, sink)
    e1.record()
    torch.cuda.synchronize()
    read_gbps = k1_bytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del rows

    # the two widened paths on the same batch, each as `reps` whole calls between two events
    def timed_ms(fn, reps=20):
        for _ in range(3):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    ent_ms = timed_ms(lambda: ears.ears_verify_ex(
        batch.target, batch.draft, batch.tokens, temperature=T, beta=betas[1], seed=seed0,
        uncertainty=ears.EARS_UNCERTAINTY_ENTROPY, workspace=ws, out_accept_len=acc,
        out_tokens=tok.view(-1)))
    var_ms = timed_ms(lambda: ears.ears_verify_ex(
        batch.target, batch.draft, batch.tokens, temperature=T, beta=betas[1], seed=seed0,
        uncertainty=ears.EARS_UNCERTAINTY_VARIANCE, workspace=ws, out_accept_len=acc,
        out_tokens=tok.view(-1)))
    greedy_tokens = batch.target[:, :K].float().argmax(-1).to(torch.int32)
    greedy_tokens[::2, K // 2] = 0        # half of the sequences stop in the middle
    greedy_ms = timed_ms(lambda: ears.ears_verify_greedy(
        batch.target, greedy_tokens, workspace=ws, out_accept_len=acc, out_tokens=tok))
    greedy_bytes = B * (K + 1) * V * esz
    other_paths = {
        "entropy_uncertainty": {"ms_per_call": ent_ms, "positions_per_s": B * K / (ent_ms * 1e-3)},
        "variance_uncertainty": {"ms_per_call": var_ms, "positions_per_s": B * K / (var_ms * 1e-3)},
        "greedy_temperature_0": {"ms_per_call": greedy_ms,
                                 "positions_per_s": B * K / (greedy_ms * 1e-3),
                                 "algorithmic_bytes": greedy_bytes,
                                 "achieved_GBps": greedy_bytes / (greedy_ms * 1e-3) / 1e9}}

    # producer-side fusion: the vocabulary projection that emits this batch's target logits
    # (N = B (K + 1) rows, hidden size 4096) with the statistics epilogue; dense bf16 MFMA peak
    lm_D = 4096
    lm_N = B * (K + 1)
    g = torch.Generator(device="cuda").manual_seed(7)
    hidden = torch.randn(lm_N, lm_D, generator=g, device="cuda").to(torch.bfloat16)
    weight = (torch.randn(V, lm_D, generator=g, device="cuda") * (2.5 / lm_D ** 0.5)).to(torch.bfloat16)
    lm_logits = torch.empty(lm_N, V, dtype=torch.bfloat16, device="cuda")
    lm_max = torch.empty(lm_N, dtype=torch.float32, device="cuda")
    lm_sum = torch.empty(lm_N, dtype=torch.float64, device="cuda")
    lm_ws = torch.empty(ears.ears_lm_head_workspace_bytes(lm_N, V), dtype=torch.uint8, device="cuda")
    lm_ms = timed_ms(lambda: ears.ears_lm_head_bf16(
        hidden, weight, temperature=T, out_logits=lm_logits, out_row_max=lm_max,
        out_row_sumexp=lm_sum, workspace=lm_ws), reps=10)
    lm_flop = 2.0 * lm_N * lm_D * V
    other_paths["lm_head_with_statistics"] = {
        "ms_per_call": lm_ms, "N": lm_N, "D": lm_D, "V": V, "bound": "mfma",
        "achieved_TFLOPs": lm_flop / (lm_ms * 1e-3) / 1e12, "peak_TFLOPs": 2500.0,
        "frac": lm_flop / (lm_ms * 1e-3) / 1e12 / 2500.0}
    del hidden, weight, lm_ws, lm_logits

    # the same shape with four times the sequences: what the fixed costs of the headline batch weigh
    big = inputs.make_config(WORKLOAD_INDEX, device="cuda", scale_B=4 * B)   # same recipe
    big_ws = torch.empty(ears.ears_workspace_bytes(4 * B * K, 4 * B, V), dtype=torch.uint8, device="cuda")
    big_acc = torch.empty(4 * B, dtype=torch.int32, device="cuda")
    big_tok = torch.empty(4 * B * (K + 1), dtype=torch.int32, device="cuda")
    big_ms = timed_ms(lambda: ears.ears_verify_ex(
        big.target, big.draft, big.tokens, temperature=T, beta=betas[1], seed=seed0, workspace=big_ws,
        out_accept_len=big_acc, out_tokens=big_tok), reps=10)
    big_rej = int((big_acc < K).sum().item())
    big_bytes = (2 * 4 * B * K + 2 * big_rej + (4 * B - big_rej)) * V * esz
    other_paths["four_times_the_batch"] = {
        "B": 4 * B, "ms_per_call": big_ms, "positions_per_s": 4 * B * K / (big_ms * 1e-3),
        "algorithmic_bytes": big_bytes, "achieved_GBps": big_bytes / (big_ms * 1e-3) / 1e9,
        "frac_of_hbm_peak": big_bytes / (big_ms * 1e-3) / 1e9 / 8000.0}
    del big, big_ws

    if args.traffic_calibration:
        # plain copy of the draft buffer: reads and writes exactly draft.numel() * 2 bytes
        dst = torch.empty_like(batch.draft)
        for _ in range(4):
            ears.ears_bench_copy(dst, batch.draft)
        torch.cuda.synchronize()
        log("traffic calibration: ears_bench_copy of %d bytes, 4 times" % (batch.draft.numel() * esz))
        del dst

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        try:
            ncores = len(os.sched_getaffinity(0))
        except AttributeError:
            ncores = os.cpu_count() or 1
        threads = max(1, min(16, ncores))
        tgt = inputs.logits_to_numpy(batch.target)
        drf = inputs.logits_to_numpy(batch.draft)
        tk = batch.tokens.cpu().numpy()
        c0 = time.perf_counter()
        for beta in betas:
            oracle.verify(tgt, drf, tk, T, beta, seed0, nthreads=threads)
        c1 = time.perf_counter()
        cpu = {"value": len(betas) * B * K / (c1 - c0), "unit": "positions/s", "cores": threads,
               "kind": "oracle",
               "sample": "the whole %s batch (%d sequences) once per beta of its sweep %s, fp64 "
                         "three-pass oracle, one OpenMP thread per sequence, %.1f s wall on %d threads"
                         % (cfg["name"], B, betas, c1 - c0, threads)}

    out = {
        "metric": "verified_draft_positions_per_sec",
        "value": positions_per_s,
        "unit": "positions/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": cfg["name"], "B": B, "K": K, "V": V, "temperature": T,
                   "betas_cycled": betas, "entry_point": "ears_verify_bf16",
                   "mean_rejected_sequences": mean_rej},
        "whole_call": {"algorithmic_bytes": call_bytes, "achieved_GBps": call_gbps,
                       "frac_of_hbm_peak": call_gbps / HBM_PEAK_GBPS},
        "roofline": {"bound": "hbm", "kernel": "row_stats_kernel<BF16>", "achieved": k1_gbps,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": k1_gbps / HBM_PEAK_GBPS,
                     "traffic": measured_traffic(), "algorithmic_bytes_per_launch": k1_bytes,
                     "avg_launch_ms": k1_ms,
                     "stream_read_ceiling_GBps": read_gbps},
        "cpu_baseline": cpu,
        "other_paths": other_paths,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
