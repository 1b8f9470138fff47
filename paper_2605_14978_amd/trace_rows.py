"""Per-workgroup timeline of one launch of the row kernel (a tuning aid, needs an MI355X).

Builds a variant of the library with PPOW_ROW_TRACE=1, in which thread 0 of every workgroup of
`row_stats_kernel` records when it began and ended (100 MHz clock) and where it ran (XCD, CU),
scores one batch of a benchmark workload with it and prints what the launch looked like: row
durations, occupied workgroup slots over time, rows and mean row duration per XCD, and how long
the compute units idle at the end of the launch.

    python -m paper_2605_14978_amd.trace_rows --workload greedy_bf16_32k
    python -m paper_2605_14978_amd.trace_rows --workload rejection_bf16_128k --windows 4096

At most 40 000 row pairs (windows x K) are traced.
"""
import argparse
import os
import subprocess
import sys
import tempfile

TRACE_ROWS = 40000          # as in row_stats.hip
TRACE_OFFSET = 4096


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--workload", default="greedy_bf16_32k")
    ap.add_argument("--windows", type=int, default=0, help="window count (0: the workload's own)")
    ap.add_argument("--library", default=None,
                    help="a library already built with PPOW_ROW_TRACE=1 (default: build one)")
    args = ap.parse_args()

    here = os.path.dirname(os.path.abspath(__file__))
    sys.path.insert(0, os.path.dirname(here))
    from paper_2605_14978_amd.build import build
    library = args.library
    if library is None:
        tmp = tempfile.mkdtemp(prefix="ppow_trace_")
        library = build(defines=["PPOW_ROW_TRACE=1"], output=os.path.join(tmp, "libppow_trace.so"))
    if os.environ.get("PPOW_LIBRARY") != library:
        # the binding fixes its library when the package is imported, which has happened by
        # now: measure in a child process that starts with the variant selected
        env = dict(os.environ, PPOW_LIBRARY=library)
        child = subprocess.run([sys.executable, "-m", "paper_2605_14978_amd.trace_rows", "--workload",
                                args.workload, "--windows", str(args.windows), "--library", library],
                               env=env, cwd=os.path.dirname(here))
        raise SystemExit(child.returncode)

    import numpy as np
    import torch
    import paper_2605_14978_amd as ppow
    from workloads import WORKLOADS, generate

    w = WORKLOADS[args.workload]
    if args.windows:
        w = w.scaled(args.windows)
    if w.seq_len or w.expected_accept:
        raise SystemExit("the trace covers the single-pass window workloads")
    if w.B * w.K > TRACE_ROWS:
        raise SystemExit(f"{w.B * w.K} row pairs: at most {TRACE_ROWS} are traced, pass --windows")
    dev = "cuda:0"
    d = generate(w, device=dev)
    code = ppow.PPOW_BF16 if w.dtype == "bf16" else ppow.PPOW_F32
    buf = ppow.ScoreBuffers(w.B, w.K, w.V, code, dev)
    verify = ppow.PPOW_VERIFY_GREEDY if w.verify == "greedy" else ppow.PPOW_VERIFY_REJECTION
    for _ in range(3):                              # the last launch is the one that is read
        ppow.ppow_score_windows(d["draft_logits"], d["target_logits"], d["draft_tokens"], d["uniforms"],
                                cost_ratio=w.cost_ratio, verify=verify, buffers=buf)
    torch.cuda.synchronize()
    rows = w.B * w.K
    raw = buf.workspace[TRACE_OFFSET:TRACE_OFFSET + 20 * TRACE_ROWS].cpu().numpy()
    when = raw[:16 * TRACE_ROWS].view(np.uint64).reshape(-1, 2)[:rows].astype(np.int64)
    hw = raw[16 * TRACE_ROWS:].view(np.uint32)[:rows]

    t0 = when[:, 0].min()
    begin, end = (when[:, 0] - t0) / 100.0, (when[:, 1] - t0) / 100.0      # microseconds
    dur, span = end - begin, float(end.max())
    gbytes = rows * 2 * w.V * w.elem_bytes / 1e9
    print(f"{w.name}: {rows} row pairs, {gbytes:.2f} GB, launch {span:.1f} us "
          f"({gbytes / (span * 1e-6):.0f} GB/s from first begin to last end)")
    pct = np.percentile(dur, [5, 50, 95])
    print(f"row duration: mean {dur.mean():.1f} us, 5th/50th/95th percentile "
          f"{pct[0]:.1f} / {pct[1]:.1f} / {pct[2]:.1f}, longest {dur.max():.1f}")
    first = np.sort(begin)
    resident = int(np.sum(first < first[0] + 2.0))
    print(f"workgroups begun within 2 us of the first: {resident}")
    grid = np.linspace(0.0, span, 21)
    print("occupied slots at 0, 5, ... 100 % of the launch:",
          " ".join(str(int(np.sum((begin <= t) & (end > t)))) for t in grid))
    tail = np.linspace(span - 2.0 * dur.mean(), span, 11)
    print("occupied slots over the last two mean row durations:",
          " ".join(str(int(np.sum((begin <= t) & (end > t)))) for t in tail))
    xcc = hw >> 16
    cu = (xcc.astype(np.int64) << 16) | (hw & 0xff00)          # XCD, shader engine/array, CU
    print("rows per XCD:         ", " ".join(f"{int(np.sum(xcc == x)):6d}" for x in range(8)))
    print("mean row duration/XCD:", " ".join(f"{dur[xcc == x].mean():6.1f}" if np.any(xcc == x) else "     -"
                                              for x in range(8)))
    last = np.array([end[cu == c].max() for c in np.unique(cu)])
    print(f"compute units seen: {len(last)}; a compute unit idles {np.mean(span - last):.1f} us at the end "
          f"of the launch on average ({100 * np.mean(span - last) / span:.1f} % of it)")
    print(f"slot occupancy over the launch: {dur.sum() / span:.0f} workgroups on average")


if __name__ == "__main__":
    main()
