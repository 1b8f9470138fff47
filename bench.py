#!/usr/bin/env python3
"""Benchmark of the PPOW window-scoring hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic windows already
resident in HBM: ppow_score_windows (row-pair streaming reduction + window
epilogue) followed by ppow_select_windows (top-M).  Prints ONE JSON line: the
headline workload's whole-job throughput in windows/s with the roofline figures of
its dominant kernel (the row-pair streaming reduction, HBM-bound) and the CPU
oracle timed on a bounded sample of the same inputs, plus -- unless one workload is
asked for with --workload -- a "configs" array with the same measurements for the
other benchmark workloads.

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
HEADLINE = "rejection_bf16_128k"
# the other workloads of the benchmark, reported in "configs" (the tiny fp32 case is a
# parity-test case only: its whole input is 1 MB)
OTHERS = ["greedy_bf16_32k", "twopass_f32_152k", "stream_bf16_128k", "sequence_bf16_128k"]
RTOL = {"f32": 1e-4, "bf16": 1e-4}     # the parity tests' bound (bf16 inputs held to the fp32 one)
ATOL = 1e-6
ATOL_DIVERGENCE = 4e-6                  # floor for divergences: two log-sum-exps cancel


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None,
                    help=f"measure this workload only (default: {HEADLINE} as the headline and "
                         "the other workloads in \"configs\")")
    ap.add_argument("--windows", type=int, default=0,
                    help="override the window count B (0: the workload's own)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="CPU time budget of the headline's oracle baseline (0 disables every "
                         "oracle leg; the other workloads get a quarter of it each)")
    ap.add_argument("--expected-accept", action="store_true",
                    help="force the expected-acceptance second pass on for this workload")
    ap.add_argument("--copy-calibration", type=float, default=0.0, metavar="GIB",
                    help="only run a plain device copy of this many GiB (counter calibration)")
    return ap.parse_args()


def needed_rtol(got, ref, atol=ATOL):
    """Smallest rtol for which |got - ref| <= rtol*|ref| + atol holds on every element."""
    import numpy as np
    got = np.asarray(got, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    excess = np.maximum(np.abs(got - ref) - atol, 0.0)
    with np.errstate(divide="ignore", invalid="ignore"):
        need = np.where(excess > 0, excess / np.abs(ref), 0.0)
    return float(need.max()) if need.size else 0.0


def cpu_baseline(w, inputs, gpu_out, seconds, single_thread_windows):
    """Time the oracle, as it stands, on the first windows of the same inputs, and compare the
    GPU's outputs for those windows with it."""
    import math
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
    out = {"value": n / dt, "unit": "windows/s", "cores": res.threads, "kind": "oracle",
           "sample": f"first {n} of {w.B} windows of the timed batch, scoring + selection, "
                     f"{dt:.1f} s"}
    if single_thread_windows:
        # per-core figure: a fixed subset on one thread
        one = min(w.B, single_thread_windows)
        oracle.set_threads(1)
        _, dt1 = run(one)
        oracle.set_threads(res.threads)
        out["single_thread_value"] = one / dt1
        out["single_thread_sample"] = f"first {one} windows, 1 thread, {dt1:.1f} s"

    k_gpu = gpu_out.accepted_len[:n].cpu().numpy()
    rp_gpu = gpu_out.r_proximity[:n].cpu().numpy().astype(np.float64)
    errors = {"r_speedup": needed_rtol(gpu_out.r_speedup[:n].cpu(), res.r_speedup),
              "adaw_score": needed_rtol(gpu_out.adaw_score[:n].cpu(), res.adaw_score, ATOL_DIVERGENCE),
              "delta": needed_rtol(gpu_out.delta[:n].cpu(), res.delta, ATOL * math.log(w.V)),
              "kl": needed_rtol(gpu_out.kl[:n].cpu(), res.kl, ATOL_DIVERGENCE),
              "confidence": needed_rtol(gpu_out.confidence[:n].cpu(), res.confidence),
              "accept_prob": needed_rtol(gpu_out.accept_prob[:n].cpu(), res.accept_prob)}
    if w.expected_accept:
        errors["expected_accept"] = needed_rtol(gpu_out.expected_accept[:n].cpu(), res.expected_accept)
    rtol = RTOL[w.dtype]
    out["gpu_matches_oracle_on_sample"] = bool(
        np.array_equal(k_gpu, res.accepted_len) and np.array_equal(rp_gpu, res.r_proximity)
        and all(e <= rtol for e in errors.values()))
    out["max_rel_error"] = errors
    out["max_rel_error_note"] = ("per output, the rtol that |gpu - oracle| <= rtol*|oracle| + atol would "
                                 "have needed on the sample (atol 1e-6, x ln V for delta, 4e-6 for kl "
                                 f"and adaw_score); the bound is {rtol:g}; accepted_len and r_proximity "
                                 "are exact")
    return out


def measured_traffic(name):
    """HBM bytes per launch of the row kernel from committed rocprofv3 counter runs, if any
    (profiles/hbm_traffic.json says which commit they were taken at)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as fh:
        return json.load(fh).get(name, {}).get("bytes_per_launch")


def bench_sequences(args, w, dev, cpu_seconds):
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
    if cpu_seconds > 0:
        import numpy as np
        import oracle
        n = 1
        t0 = time.perf_counter()
        v_ref, s_ref = oracle.adaw_sequence(d["draft_logits"][:n].cpu(), d["target_logits"][:n].cpu(), K)
        picks = oracle.sample_starts(s_ref, d["uniforms"][:n].cpu().numpy().astype(np.float64))
        dt = time.perf_counter() - t0
        errors = {"criticality": needed_rtol(buf.criticality[:n].cpu(), v_ref, ATOL_DIVERGENCE),
                  "window_score": needed_rtol(buf.window_score[:n].cpu(), s_ref, ATOL_DIVERGENCE)}
        rtol = RTOL[w.dtype]
        # the start is drawn from fp32 scores on the GPU: compare with the oracle's draw on those
        s_gpu = buf.window_score[:n].cpu().numpy().astype(np.float64)
        own = oracle.sample_starts(s_gpu, d["uniforms"][:n].cpu().numpy().astype(np.float64))
        agrees = bool(all(e <= rtol for e in errors.values()) and
                      np.array_equal(buf.sampled_start[:n].cpu().numpy(), own))
        result["cpu_baseline"] = {"value": n * W / dt, "unit": "windows/s", "cores": os.cpu_count(),
                                  "kind": "oracle", "sample": f"first {n} of {N} sequences ({T} rows), {dt:.1f} s",
                                  "gpu_matches_oracle_on_sample": agrees, "max_rel_error": errors,
                                  "start_drawn_as_by_the_oracle_from_its_own_scores":
                                      bool(np.array_equal(picks, own))}
    del d, buf, selbuf
    torch.cuda.empty_cache()
    return result


def bench_windows(args, w, dev, cpu_seconds, single_thread_windows):
    import torch
    import paper_2605_14978_amd as ppow
    from workloads import generate
    from workloads.generate import accepted_length_histogram

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
    optional = ("delta", "kl", "confidence", "accept_prob") if cpu_seconds > 0 else ()
    optional += ("expected_accept",) if w.expected_accept else ()
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
    firing = float((sbuf.r_proximity != 0).float().mean().item())
    print(f"# accepted-length histogram 0..K: {hist}; windows with a proximity reward: "
          f"{100 * firing:.2f} %", file=sys.stderr, flush=True)

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
        "accepted_length_histogram": hist,
        "proximity_reward_fraction": firing,
    }
    if cpu_seconds > 0:
        result["cpu_baseline"] = cpu_baseline(w, inputs, sbuf, cpu_seconds, single_thread_windows)
    del chunks, inputs, sbuf, slices, selbuf
    torch.cuda.empty_cache()
    return result


def bench_one(args, name, dev, cpu_seconds, single_thread_windows=0):
    from workloads import WORKLOADS
    from workloads.generate import describe
    w = WORKLOADS[name]
    if args.windows:
        w = w.scaled(args.windows)
    if args.expected_accept:
        w = dataclasses.replace(w, expected_accept=True)
    print(f"# {describe(w)}", file=sys.stderr, flush=True)
    if w.seq_len:
        return bench_sequences(args, w, dev, cpu_seconds)
    return bench_windows(args, w, dev, cpu_seconds, single_thread_windows)


def main():
    args = parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (windows are independent, so more "
                 "GPUs would each score their own share); run with --gpus 1")
    import torch
    import paper_2605_14978_amd as ppow

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

    if args.workload:
        result = bench_one(args, args.workload, dev, args.cpu_seconds, single_thread_windows=256)
    else:
        result = bench_one(args, HEADLINE, dev, args.cpu_seconds, single_thread_windows=256)
        configs = []
        for name in OTHERS:
            r = bench_one(args, name, dev, args.cpu_seconds / 4)
            entry = {"workload": name, "value": r["value"], "unit": r["unit"],
                     "ms_per_step": r["ms_per_step"], "dtype": r["dtype"], "config": r["config"],
                     "kernel": r["roofline"]["kernel"], "kernel_ms": r["roofline"]["kernel_ms"],
                     "achieved": r["roofline"]["achieved"], "frac": r["roofline"]["frac"],
                     "traffic": r["roofline"]["traffic"],
                     "algorithmic_bytes_per_launch": r["roofline"]["algorithmic_bytes_per_launch"]}
            for key in ("accepted_length_histogram", "proximity_reward_fraction"):
                if key in r:
                    entry[key] = r[key]
            if "cpu_baseline" in r:
                cb = r["cpu_baseline"]
                entry["oracle_windows_per_s"] = cb["value"]
                entry["oracle_sample"] = cb["sample"]
                entry["gpu_matches_oracle_on_sample"] = cb["gpu_matches_oracle_on_sample"]
                entry["max_rel_error"] = cb["max_rel_error"]
            configs.append(entry)
        result["configs"] = configs
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
