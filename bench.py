#!/usr/bin/env python3
"""Benchmark of the EARS verification step on one MI355X.

A step is one whole `ears_verify_bf16` call (row statistics with the per-position decisions, then
the accept-length scan and the replacement / bonus sampling) over one synthetic batch already
resident in HBM.  Prints ONE JSON line on stdout.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
# plain vector-ALU issue: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz
VALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9
WORKLOAD_INDEX = 2              # B=256, K=8, V=128256, bf16: the configuration the metric is quoted on
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_verify_c2.json")
FILTER_FILE = os.path.join(ROOT, "profiles", "filter_counters_c2.json")
KERNEL_SOURCES = ("paper_2512_13194_amd/csrc/row_stats.h", "paper_2512_13194_amd/csrc/ears_device.h",
                  "paper_2512_13194_amd/csrc/decide.h", "paper_2512_13194_amd/csrc/sample.h",
                  "paper_2512_13194_amd/csrc/verify.h",
                  "paper_2512_13194_amd/csrc/ears_kernels.hip", "paper_2512_13194_amd/build.py")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_source_hash() -> str:
    """Hash of everything that shapes the verification kernels and their launches (sources,
    launch code, build flags): a committed counter figure is only reported while it matches."""
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def committed_counters(path):
    """A committed rocprofv3 counter summary, or None when there is none or the kernel sources have
    changed since it was taken."""
    try:
        with open(path) as f:
            t = json.load(f)
    except OSError:
        return None
    if t.get("kernel_source_hash") != kernel_source_hash():
        return None
    return t


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--settle-ms", type=float, default=300.0,
                    help="keep the GPU busy with whole calls for this long before the warm-up steps: after "
                         "an idle spell its clocks take about 25 ms of work (some 120 calls) to come back up, "
                         "which is longer than a short timed region; 0 turns it off")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the other workloads and paths (short runs under a profiler)")
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

    # ---- the timed region: exactly `steps` whole calls between two synchronisations -------------
    # (before the warm-up steps the GPU's clocks are given time to settle, see --settle-ms)
    settle_calls = 0
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for i in range(20):
            step(i)
        torch.cuda.synchronize()
        settle_calls += 20
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

    def per_launch_ms(fn, reps):
        """Each launch between its own pair of HIP events on the launch stream."""
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(reps)]
        for i, (a, b) in enumerate(ev):
            a.record()
            fn(i)
            b.record()
        torch.cuda.synchronize()
        return [a.elapsed_time(b) for a, b in ev]

    def spread(ms):
        s = sorted(ms)
        return {"median_ms": statistics.median(s), "mean_ms": sum(s) / len(s), "min_ms": s[0],
                "p90_ms": s[(9 * len(s)) // 10], "launches": len(s)}

    reps = max(20, args.steps)
    call_ms = spread(per_launch_ms(step, reps))

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

    # ---- dominant kernel: verify_kernel<BF16, 8, 0>, the ONE launch of a whole call -----------------
    # (statistics workgroups, then the sampling workgroups that wait for them).  Its launches are
    # timed with HIP events on the stream they run on (torch's current stream, which the binding
    # hands to the library): back to back between two events for the average, and one pair of
    # events per launch (call_ms above) for the median.
    v0, v1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    v0.record()
    for i in range(reps):
        step(i)
    v1.record()
    torch.cuda.synchronize()
    vk_ms = v0.elapsed_time(v1) / reps
    vk_gbps = call_bytes / (vk_ms * 1e-3) / 1e9

    # ---- the statistics stage as a launch of its own ------------------------------------------------
    # A statistics-stage call (what a pipeline that computes the statistics ahead of time makes)
    # launches row_stats_kernel<BF16, 8, 0>: the same statistics and per-position decisions, and
    # nothing else.  Timed the same way.
    ws = torch.empty(ears.ears_workspace_bytes(B * K, B, V), dtype=torch.uint8, device="cuda")

    def stats_only(i):
        ears.ears_verify_ex(batch.target, batch.draft, batch.tokens, temperature=T,
                            beta=betas[i % len(betas)], seed=seed0 + i, workspace=ws,
                            stages=ears.EARS_STAGE_STATS, out_accept_len=acc, out_tokens=tok.view(-1))

    for i in range(max(10, args.warmup)):   # the clock settles within a few launches
        stats_only(i)
    torch.cuda.synchronize()
    k0, k1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    k0.record()
    for i in range(reps):
        stats_only(i)
    k1.record()
    torch.cuda.synchronize()
    k1_ms = k0.elapsed_time(k1) / reps
    k1_gbps = k1_bytes / (k1_ms * 1e-3) / 1e9
    k1_spread = spread(per_launch_ms(stats_only, reps))

    # ---- the sampling stage as a launch of its own, timed in place ------------------------------------
    # Statistics + decisions, then the sampling stage of the same call as a launch of its own, with
    # the events around the sampling launch only: the rows it reads are as cold as in a whole call.
    def stats_decide(i):
        ears.ears_verify_ex(batch.target, batch.draft, batch.tokens, temperature=T,
                            beta=betas[i % len(betas)], seed=seed0 + i, workspace=ws,
                            stages=ears.EARS_STAGE_STATS | ears.EARS_STAGE_DECIDE, out_accept_len=acc,
                            out_tokens=tok.view(-1))

    def sample_only(i):
        ears.ears_verify_ex(batch.target, batch.draft, batch.tokens, temperature=T,
                            beta=betas[i % len(betas)], seed=seed0 + i, workspace=ws,
                            stages=ears.EARS_STAGE_SAMPLE, out_accept_len=acc, out_tokens=tok.view(-1))

    samp_ev = []
    for i in range(reps):
        stats_decide(i)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        sample_only(i)
        b.record()
        samp_ev.append((a, b))
    torch.cuda.synchronize()
    samp = spread([a.elapsed_time(b) for a, b in samp_ev])
    filt = committed_counters(FILTER_FILE)
    # Its bound is the memory stream too: the kernel's first 15 us are paced by the arrival of the
    # rejected / bonus target rows (cold: the statistics kernel read them with non-temporal loads),
    # the rest is the dependent start and the tail through the exact choice.  Algorithmic bytes: one
    # target row per sequence.
    samp_bytes = B * V * esz
    filter_roofline = {
        "kernel": "sample_select_kernel<BF16, 2, false> (scan, filter and exact choice as a launch of "
                  "their own: a SAMPLE-stage call; in a whole call the same code runs as the second "
                  "part of verify_kernel)",
        "bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBPS,
        "achieved": samp_bytes / (samp["median_ms"] * 1e-3) / 1e9,
        "frac": samp_bytes / (samp["median_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "algorithmic_bytes_per_launch": samp_bytes,
        "launch_ms": samp,
    }
    if filt is not None:
        lane_ops = filt["valu_wave_instructions_per_launch"] * 64
        filter_roofline["vector_alu"] = {
            "wave_instructions_per_launch": filt["valu_wave_instructions_per_launch"],
            "lane_ops_per_s": lane_ops / (samp["median_ms"] * 1e-3),
            "frac_of_issue_peak": lane_ops / (samp["median_ms"] * 1e-3) / VALU_PEAK_LANE_OPS,
            "counters_from": filt.get("source")}

    # practical ceiling: a read-only streaming kernel over one buffer that holds exactly the rows
    # the statistics kernel reads (target rows 0..K-1, then the draft rows), one launch per pass
    rows = torch.cat([batch.target[:, :K].reshape(-1), batch.draft.reshape(-1)])
    assert rows.numel() * esz == k1_bytes
    sink = None
    for _ in range(3):
        sink = ears.ears_bench_read(rows, sink)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        ears.ears_bench_read(rows, sink)
    e1.record()
    torch.cuda.synchronize()
    read_gbps = k1_bytes * 20 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del rows

    def timed_ms(fn, reps=20):
        # a kernel with other arithmetic than the one before it runs some tens of launches before
        # its time settles (the entropy variant: 200 us after 3 launches, 181-185 us after 30)
        for _ in range(30):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    other_paths = {}
    if not args.headline_only:
        other_paths = _other_paths(torch, ears, inputs, batch, ws, acc, tok, T, betas, seed0, timed_ms)

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
        n1 = 16                                    # sequences of the single-threaded sample
        s0 = time.perf_counter()
        oracle.verify(tgt[:n1], drf[:n1], tk[:n1], T, betas[1], seed0, nthreads=1)
        s1 = time.perf_counter()
        cpu = {"value": len(betas) * B * K / (c1 - c0), "unit": "positions/s", "cores": threads,
               "kind": "oracle",
               "sample": "the whole %s batch (%d sequences) once per beta of its sweep %s, fp64 "
                         "three-pass oracle, one OpenMP thread per sequence, %.1f s wall on %d threads"
                         % (cfg["name"], B, betas, c1 - c0, threads),
               "single_thread": {"value": n1 * K / (s1 - s0), "unit": "positions/s", "cores": 1,
                                 "sample": "the first %d sequences of the same batch, beta %.2f, "
                                           "%.1f s wall" % (n1, betas[1], s1 - s0)}}

    traffic = committed_counters(TRAFFIC_FILE)
    out = {
        "metric": "verified_draft_positions_per_sec",
        "value": positions_per_s,
        "unit": "positions/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle": {"ms": args.settle_ms, "whole_calls_before_the_warmup_steps": settle_calls},
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
                       "frac_of_hbm_peak": call_gbps / HBM_PEAK_GBPS,
                       "per_launch_events": call_ms,
                       "frac_of_hbm_peak_at_median": call_bytes / (call_ms["median_ms"] * 1e-3) / 1e9
                                                     / HBM_PEAK_GBPS},
        "roofline": {"bound": "hbm",
                     "kernel": "verify_kernel<BF16, 8, 0> (the one launch of the timed call: statistics "
                               "and decision of every position, then filter and exact choice)",
                     "achieved": vk_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": vk_gbps / HBM_PEAK_GBPS,
                     "traffic": None if traffic is None else traffic.get("hbm_bytes_per_launch"),
                     "traffic_source": None if traffic is None else
                     "committed rocprofv3 counter runs (%s), valid for the current kernel sources"
                     % traffic.get("source"),
                     "algorithmic_bytes_per_launch": call_bytes,
                     "avg_launch_ms": vk_ms, "per_launch_events": call_ms,
                     "stream_read_ceiling_GBps": read_gbps},
        "roofline_statistics_stage": {
            "bound": "hbm",
            "kernel": "row_stats_kernel<BF16, 8, 0> (a STATS-stage call: statistics + per-position "
                      "decision as a launch of their own; in a whole call the same code runs as the "
                      "first part of verify_kernel)",
            "achieved": k1_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": k1_gbps / HBM_PEAK_GBPS,
            "algorithmic_bytes_per_launch": k1_bytes, "avg_launch_ms": k1_ms,
            "per_launch_events": k1_spread},
        "roofline_sampling_stage": filter_roofline,
        "cpu_baseline": cpu,
        "other_paths": other_paths,
    }
    print(json.dumps(out), flush=True)
    return 0


def _whole_call_entry(torch, ears, inputs, index, timed_ms, rotate=1):
    """Whole calls on another workload: time per call, positions/s, algorithmic bytes and their
    fraction of the HBM peak.  `rotate` input sets (generated with different data seeds) are taken
    in turn, so that a batch smaller than the caches is not simply re-read from them."""
    cfg = inputs.CONFIGS[index]
    sets = []
    for j in range(rotate):
        if j == 0:
            sets.append(inputs.make_config(index, device="cuda"))
        else:
            sets.append(inputs.make_rect(cfg["B"], cfg["K"], cfg["V"], inputs._TORCH_DTYPE[cfg["dtype"]],
                                         T=cfg["temperatures"][0], data_seed=cfg["data_seed"] + 100 * j,
                                         device="cuda", **cfg["gen"]))
    b0 = sets[0]
    esz = b0.target.element_size()
    V = b0.V
    ragged = b0.row_offsets is not None
    R = b0.total_draft_rows
    Bn = b0.B
    acc = torch.empty(Bn, dtype=torch.int32, device="cuda")
    tok = torch.empty(R + Bn, dtype=torch.int32, device="cuda")
    state = {"i": 0}
    if ragged:
        fn = ears.ears_verify_ragged_bf16

        def call():
            bt = sets[state["i"] % rotate]
            state["i"] += 1
            fn(bt.target, bt.draft, bt.tokens, bt.row_offsets, bt.temperature, bt.beta,
               cfg["seed"] + state["i"], out_accept_len=acc, out_tokens=tok)
        Ks = (b0.row_offsets[1:] - b0.row_offsets[:-1]).to(torch.int32)
    else:
        fn = ears.ears_verify_f32 if b0.target.dtype == torch.float32 else ears.ears_verify_bf16
        T = cfg["temperatures"][0]
        beta = cfg["betas"][-1]

        def call():
            bt = sets[state["i"] % rotate]
            state["i"] += 1
            fn(bt.target, bt.draft, bt.tokens, T, beta, cfg["seed"] + state["i"], out_accept_len=acc,
               out_tokens=tok.view(Bn, -1))
        Ks = torch.full((Bn,), b0.K, dtype=torch.int32, device="cuda")
    ms = timed_ms(call, reps=40 if R * V < 1e8 else 20)
    rej = int((acc < Ks).sum().item())
    nbytes = (2 * R + 2 * rej + (Bn - rej)) * V * esz
    entry = {"workload": cfg["name"], "ms_per_call": ms, "positions_per_s": R / (ms * 1e-3),
             "algorithmic_bytes": nbytes, "achieved_GBps": nbytes / (ms * 1e-3) / 1e9,
             "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
    if rotate > 1:
        entry["input_sets_rotated"] = rotate
    if nbytes < 5e6:
        entry["note"] = "latency-bound: a few megabytes, three dependent kernel phases"
    return entry


def _other_paths(torch, ears, inputs, batch, ws, acc, tok, T, betas, seed0, timed_ms):
    B, K, V = batch.B, batch.K, batch.V
    esz = 2
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
    other = {
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
    other["lm_head_with_statistics"] = {
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
    other["four_times_the_batch"] = {
        "B": 4 * B, "ms_per_call": big_ms, "positions_per_s": 4 * B * K / (big_ms * 1e-3),
        "algorithmic_bytes": big_bytes, "achieved_GBps": big_bytes / (big_ms * 1e-3) / 1e9,
        "frac_of_hbm_peak": big_bytes / (big_ms * 1e-3) / 1e9 / 8000.0}
    del big, big_ws
    torch.cuda.empty_cache()

    # the other workloads as whole calls (workload 1 is smaller than the caches: eight input sets
    # in turn; workload 0 is a megabyte and measures latency, not bandwidth)
    other["workload_0"] = _whole_call_entry(torch, ears, inputs, 0, timed_ms, rotate=8)
    other["workload_1"] = _whole_call_entry(torch, ears, inputs, 1, timed_ms, rotate=8)
    other["workload_3"] = _whole_call_entry(torch, ears, inputs, 3, timed_ms)
    torch.cuda.empty_cache()
    other["workload_4"] = _whole_call_entry(torch, ears, inputs, 4, timed_ms)
    torch.cuda.empty_cache()
    return other


if __name__ == "__main__":
    sys.exit(main())
