#!/usr/bin/env python3
"""Benchmark of the PPOW window-scoring hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic windows already
resident in HBM: ppow_score_windows (row-pair streaming reduction + window
epilogue) followed by ppow_select_windows (top-M).  Prints ONE JSON line with the
whole-job throughput in windows/s, the roofline figures of the dominant kernel
(the row-pair streaming reduction, HBM-bound) and the CPU oracle timed on a
bounded sample of the same inputs.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
"""
import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="rejection_bf16_128k")
    ap.add_argument("--windows", type=int, default=0,
                    help="override the window count B (0: the workload's own)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="CPU time budget of the oracle baseline (0 disables it)")
    ap.add_argument("--expected-accept", action="store_true",
                    help="force the expected-acceptance second pass on for this workload")
    ap.add_argument("--copy-calibration", type=float, default=0.0, metavar="GIB",
                    help="only run a plain device copy of this many GiB (counter calibration)")
    return ap.parse_args()


def cpu_baseline(w, inputs, gpu_out, seconds):
    """Time the oracle, as it stands, on the first windows of the same inputs."""
    import numpy as np
    import oracle

    def run(n):
        a = inputs["target_logits"][:n].cpu()
        b = inputs["draft_logits"][:n].cpu()
        tok = inputs["draft_tokens"][:n].cpu().numpy()
        u = inputs["uniforms"]
        u = None if u is None else u[:n].cpu().numpy()
        want = ("kl", "confidence", "accept_prob") + (("expected_accept",) if w.expected_accept else ())
        t0 = time.perf_counter()
        res = oracle.score_windows(b, a, tok, u, cost_ratio=w.cost_ratio, prox_eps=w.prox_eps,
                                   prox_eta=w.prox_eta,
                                   verify=oracle.GREEDY if w.verify == "greedy" else oracle.REJECTION,
                                   want=want)
        oracle.select_windows(res.adaw_score, max(1, min(w.M, n)))
        return res, time.perf_counter() - t0

    probe = min(w.B, 32)
    res, dt = run(probe)
    n = int(min(w.B, max(probe, probe * seconds / max(dt, 1e-6))))
    if n > probe:
        res, dt = run(n)
    # single-thread rate on a small fixed subset, for a per-core figure
    one = min(w.B, 16)
    oracle.set_threads(1)
    _, dt1 = run(one)
    oracle.set_threads(res.threads)
    k_gpu = gpu_out.accepted_len[:n].cpu().numpy()
    s_gpu = gpu_out.adaw_score[:n].cpu().numpy().astype(np.float64)
    rtol = 2e-3 if w.dtype == "bf16" else 1e-4
    agrees = bool(np.array_equal(k_gpu, res.accepted_len) and
                  np.all(np.abs(s_gpu - res.adaw_score) <= rtol * np.abs(res.adaw_score) + 1e-6))
    return {"value": n / dt, "unit": "windows/s", "cores": res.threads, "kind": "oracle",
            "sample": f"first {n} of {w.B} windows of the timed batch, scoring + selection, "
                      f"{dt:.1f} s", "single_thread_value": one / dt1,
            "single_thread_sample": f"first {one} windows, 1 thread, {dt1:.1f} s",
            "gpu_matches_oracle_on_sample": agrees}


def measured_traffic(name):
    """HBM bytes per launch of the row kernel from committed rocprofv3 counter runs, if any."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as fh:
        return json.load(fh).get(name, {}).get("bytes_per_launch")


def bench_sequences(args, w, dev):
    """Sequence-mode ADAW: a step scores N sequences of T positions once, forms every
    overlapping window score, draws one start per sequence and ranks all windows."""
    import torch
    import paper_2605_14978_amd as ppow
    from workloads import generate_sequences

    N, T, K, V = w.B, w.seq_len, w.K, w.V
    W = T - K + 1
    t0 = time.perf_counter()
    d = generate_sequences(w, device=dev)
    torch.cuda.synchronize()
    print(f"# generated {N} sequences of {T} positions in {time.perf_counter() - t0:.1f} s",
          file=sys.stderr, flush=True)
    code = ppow.PPOW_BF16 if w.dtype == "bf16" else ppow.PPOW_F32
    buf = ppow.SequenceBuffers(N, T, V, K, code, dev)
    selbuf = ppow.SelectBuffers(N * W, w.M, dev)

    def score():
        ppow.ppow_adaw_sequence(d["draft_logits"], d["target_logits"], K, d["uniforms"], buffers=buf)

    def select():
        ppow.ppow_select_windows(buf.window_score.view(-1), w.M, buffers=selbuf)

    for _ in range(args.warmup):
        score()
        select()
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        starts[i].record()
        score()
        stops[i].record()
        select()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    score_ms = sum(s.elapsed_time(e) for s, e in zip(starts, stops)) / args.steps
    algorithmic_bytes = 2 * N * T * V * w.elem_bytes
    achieved = algorithmic_bytes / (score_ms * 1e-3) / 1e9
    result = {
        "metric": "speculative windows scored/sec", "value": N * W / (ms_per_step * 1e-3),
        "unit": "windows/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": w.name, "sequences": N, "positions": T, "K": K, "V": V, "M": w.M,
                   "windows": N * W, "logit_gigabytes_per_step": algorithmic_bytes / 1e9},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": measured_traffic(w.name),
                     "kernel": "row_stats_kernel", "kernel_ms": score_ms,
                     "algorithmic_bytes_per_launch": algorithmic_bytes},
    }
    if args.cpu_seconds > 0:
        import numpy as np
        import oracle
        n = 1
        t0 = time.perf_counter()
        v_ref, s_ref = oracle.adaw_sequence(d["draft_logits"][:n].cpu(), d["target_logits"][:n].cpu(), K)
        oracle.sample_starts(s_ref, d["uniforms"][:n].cpu().numpy().astype(np.float64))
        dt = time.perf_counter() - t0
        s_gpu = buf.window_score[:n].cpu().numpy().astype(np.float64)
        rtol = 2e-3 if w.dtype == "bf16" else 1e-4
        agrees = bool(np.all(np.abs(s_gpu - s_ref) <= rtol * np.abs(s_ref) + 1e-6))
        result["cpu_baseline"] = {"value": n * W / dt, "unit": "windows/s", "cores": os.cpu_count(),
                                  "kind": "oracle", "sample": f"first {n} of {N} sequences ({T} rows), {dt:.1f} s",
                                  "gpu_matches_oracle_on_sample": agrees}
    print(json.dumps(result), flush=True)


def main():
    args = parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (windows are independent, so more "
                 "GPUs would each score their own share); run with --gpus 1")
    import torch
    import paper_2605_14978_amd as ppow
    from workloads import WORKLOADS, generate
    from workloads.generate import accepted_length_histogram, describe

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    ppow.lib()                                     # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    dev = "cuda:0"

    if args.copy_calibration > 0:
        # A plain elementwise copy of known size: rocprofv3's FETCH_SIZE / WRITE_SIZE for this
        # kernel give the factor that converts the counters to bytes.
        n = int(args.copy_calibration * (1 << 30)) // 4
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(max(1, args.steps)):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n * 4, "bytes_written": n * 4,
                          "launches": max(1, args.steps)}), flush=True)
        return

    w = WORKLOADS[args.workload]
    if args.windows:
        w = w.scaled(args.windows)
    if args.expected_accept:
        w = dataclasses.replace(w, expected_accept=True)
    print(f"# {describe(w)}", file=sys.stderr, flush=True)

    if w.seq_len:
        return bench_sequences(args, w, dev)

    # A workload of several chunks streams them through the scoring call one after another
    # (they would not all fit in HBM); up to MAX_RESIDENT distinct chunks are kept resident and
    # cycled, so every call still reads its logits from HBM.
    MAX_RESIDENT = 4
    n_resident = min(w.chunks, MAX_RESIDENT)
    total = w.B * w.chunks
    t0 = time.perf_counter()
    chunks = [generate(w, device=dev, chunk=c) for c in range(n_resident)]
    inputs = chunks[0]
    torch.cuda.synchronize()
    print(f"# generated {n_resident} resident chunk(s) in {time.perf_counter() - t0:.1f} s",
          file=sys.stderr, flush=True)

    code = ppow.PPOW_BF16 if w.dtype == "bf16" else ppow.PPOW_F32
    flags = ppow.PPOW_FLAG_EXPECTED_ACCEPT if w.expected_accept else 0
    optional = ("expected_accept",) if w.expected_accept else ()
    sbuf = ppow.ScoreBuffers(total, w.K, w.V, code, dev, optional, flags)
    slices = [sbuf.window_slice(c * w.B, (c + 1) * w.B) for c in range(w.chunks)]
    selbuf = ppow.SelectBuffers(total, w.M, dev)
    verify = ppow.PPOW_VERIFY_GREEDY if w.verify == "greedy" else ppow.PPOW_VERIFY_REJECTION

    def score():
        for c in range(w.chunks):
            d = chunks[c % n_resident]
            ppow.ppow_score_windows(d["draft_logits"], d["target_logits"], d["draft_tokens"],
                                    d["uniforms"], cost_ratio=w.cost_ratio, prox_eps=w.prox_eps,
                                    prox_eta=w.prox_eta, verify=verify, flags=flags,
                                    buffers=slices[c])

    def select():
        ppow.ppow_select_windows(sbuf.adaw_score, w.M, buffers=selbuf)

    for _ in range(args.warmup):
        score()
        select()
    torch.cuda.synchronize()

    # HIP events on the launch stream (torch's current stream) bracket the scoring calls of
    # each step: the row kernel(s) plus the microsecond-scale window epilogue(s).
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        starts[i].record()
        score()
        stops[i].record()
        select()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ms_per_step = elapsed * 1e3 / args.steps
    score_ms = sum(s.elapsed_time(e) for s, e in zip(starts, stops)) / args.steps / w.chunks
    algorithmic_bytes = w.B * w.logit_bytes_per_window          # per launch of the row kernel
    achieved = algorithmic_bytes / (score_ms * 1e-3) / 1e9
    hist = accepted_length_histogram(sbuf.accepted_len, w.K)
    print(f"# accepted-length histogram 0..K: {hist}", file=sys.stderr, flush=True)

    result = {
        "metric": "speculative windows scored/sec",
        "value": total / (ms_per_step * 1e-3),
        "unit": "windows/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype if w.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "chunks": w.chunks, "K": w.K, "V": w.V, "M": w.M,
                   "verify": w.verify, "cost_ratio": w.cost_ratio,
                   "expected_accept_pass": w.expected_accept,
                   "logit_gigabytes_per_step": algorithmic_bytes * w.chunks / 1e9},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": measured_traffic(w.name),
                     "kernel": "row_%s_kernel" % ("cluster" if ppow.last_row_kernel() == "cluster" else "stats"),
                     "kernel_ms": score_ms,
                     "algorithmic_bytes_per_launch": algorithmic_bytes},
    }
    if args.cpu_seconds > 0:
        result["cpu_baseline"] = cpu_baseline(w, inputs, sbuf, args.cpu_seconds)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
