"""Throughput of bpe_encode_batch on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C]

A step is one whole bpe_encode_batch call (length binning, per-string merge kernels, offset scan, packing)
over one synthetic batch that is already resident in HBM.  The default workload is configuration 2
(32,000 merges, 1,024 strings x 1 KiB).  Prints one JSON line: input GB/s as `value`, plus tokens/s, the
HBM roofline of the encode kernel and the CPU oracle timed on this host as a baseline.
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

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E peak, GB/s


def measured_traffic(config: int):
    """HBM-side bytes per encode-kernel launch from the committed rocprofv3 counter summary, if there is one
    for this workload (the counters cannot be read from inside this process)."""
    import re

    path = os.path.join(ROOT, "profiles", f"encode_kernel_config{config}_pmc.md")
    try:
        m = re.search(r"^traffic_bytes_per_launch\s*=\s*(\d+)", open(path).read(), flags=re.M)
    except OSError:
        return None
    return int(m.group(1)) if m else None


VALU_PEAK_GIPS = 256 * 4 * 2.4 / 4      # 256 CUs x 4 SIMDs, one wave64 vector instruction per 4 cycles at 2.4 GHz


def measured_valu(config: int):
    """Vector wave-instructions per encode-kernel launch from the committed SQ counter summary, if it has a
    figure for this workload."""
    import re

    try:
        text = open(os.path.join(ROOT, "profiles", "encode_kernel_sq_counters.md")).read()
    except OSError:
        return None
    m = re.search(rf"^valu_wave_instructions_per_launch_config{config}\s*=\s*(\d+)", text, flags=re.M)
    return int(m.group(1)) if m else None


def stream_copy_gbs(dev, nbytes=1 << 30, reps=5):
    """Read + written bytes per second of a plain device-to-device copy: the ceiling an HBM-bound kernel could
    reach on this machine, for comparison with the published peak."""
    import torch

    src = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(reps):
        dst.copy_(src)
    ev1.record()
    torch.cuda.synchronize()
    return 2.0 * nbytes * reps / (ev0.elapsed_time(ev1) * 1e-3) / 1e9


def cpu_baseline(merges, data, offsets, target_seconds=1.5):
    """The oracle's textbook sequential encoder on all host threads, on repetitions of the same batch."""
    import oracle

    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    table = oracle.Table(merges)
    t0 = time.perf_counter()
    ids, _ = table.encode_batch(data, offsets, tier=oracle.TEXTBOOK, nthreads=cores)
    once = time.perf_counter() - t0
    reps = max(1, min(200, int(target_seconds / max(once, 1e-6))))
    t0 = time.perf_counter()
    for _ in range(reps):
        table.encode_batch(data, offsets, tier=oracle.TEXTBOOK, nthreads=cores)
    wall = time.perf_counter() - t0
    # the work model of the one-rank-per-pass view (section 4.2) on a few strings: passes and token visits
    sample = min(len(offsets) - 1, 16)
    _, _, st = table.encode_batch(data[: int(offsets[sample])], offsets[: sample + 1], tier=oracle.PASSES,
                                  nthreads=cores, stats=True)
    sample_bytes = max(int(offsets[sample]), 1)
    return {
        "pass_view": {"strings": sample, "passes_per_string": st["passes"] / max(sample, 1),
                      "token_visits_per_byte": st["visits"] / sample_bytes},
        "value": len(data) * reps / wall / 1e9,
        "unit": "GB/s",
        "tokens_per_s": len(ids) * reps / wall,
        "cores": cores,
        "kind": "oracle",
        "sample": f"whole batch ({len(offsets) - 1} strings, {len(data)} bytes) x {reps} repetitions, "
                  f"textbook sequential encoder, {wall:.1f} s wall",
    }, ids


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="workload configuration 1..5 (default 2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 256 MiB device copy (a kernel of known traffic for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: strings are independent, so more GPUs only split the batch; "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2507_11941_amd as bpe
    import workloads

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    bpe.load_library()
    cfg = workloads.CONFIGS[args.config]
    merges = workloads.load_merges(cfg.table)
    data, offsets = workloads.batch(args.config)
    batch = len(offsets) - 1
    total = int(offsets[-1])
    max_len = int(np.diff(offsets).max())

    dev = torch.device("cuda:0")
    table = bpe.build_table(merges)
    d_data = torch.from_numpy(data).to(dev)
    d_off = torch.from_numpy(offsets).to(dev)
    out_ids = torch.empty(total, dtype=torch.int32, device=dev)
    out_off = torch.empty(batch + 1, dtype=torch.int64, device=dev)
    ws = torch.empty(bpe.workspace_bytes(batch, total, max_len), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream(dev)

    def step():
        bpe.encode_batch(table, d_data, d_off, max_len, out_ids, out_off, ws, stream)

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    n_tokens = int(out_off[-1].item())

    # the timed region: exactly `steps` calls, nothing else on the stream
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    ms_total = ev0.elapsed_time(ev1)
    # the encode kernel's own duration: the same calls again with an event pair around the encode launches of
    # each (on `stream`).  Kept out of the timed region because an event record between two kernels costs the
    # stream about 3 us, a twentieth of a step here.
    bpe.set_profiling(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    kernel_ms_total, kernel_calls = bpe.read_profile()
    bpe.set_profiling(False)
    ms_per_step = ms_total / args.steps
    kernel_ms = kernel_ms_total / max(kernel_calls, 1)

    # algorithmic HBM bytes of one encode: read every input byte and two offsets per string, write every id
    # and one count per string
    algo_bytes = total + 4 * n_tokens + 16 * batch
    achieved = algo_bytes / (kernel_ms * 1e-3) / 1e9

    result = {
        "metric": "bpe_encode_batch input throughput",
        "value": total / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "tokens_per_s": n_tokens / (ms_per_step * 1e-3),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",                           # all arithmetic is on 32-bit unsigned words (ranks, ids, masks)
        "io": "u8 bytes in, i32 ids and i64 offsets out",
        "data": "synthetic",
        "config": {"workload": f"config {args.config}: {cfg.name}", "table_merges": int(len(merges)),
                   "batch": batch, "input_bytes": total, "max_len": max_len, "tokens": n_tokens},
        "hbm_fraction_input": total / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "kernel": "encode_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(args.config),
                     "algorithmic_bytes_per_launch": algo_bytes, "kernel_ms": kernel_ms,
                     "kernel_calls_timed": kernel_calls},
    }
    valu = measured_valu(args.config)
    if valu is not None:                                 # how busy the vector ALUs are: the limit that applies
        rate = valu / (kernel_ms * 1e-3) / 1e9
        result["issue"] = {"bound": "alu", "achieved": rate, "peak": VALU_PEAK_GIPS, "unit": "G wave-instr/s",
                           "frac": rate / VALU_PEAK_GIPS, "valu_wave_instructions_per_launch": valu}
    if not args.no_cpu_baseline:
        result["stream_copy_GBs"] = stream_copy_gbs(dev)
        base, want = cpu_baseline(merges, data, offsets)
        got = out_ids[:n_tokens].cpu().numpy()
        result["cpu_baseline"] = base
        result["matches_oracle"] = bool(len(want) == len(got) and np.array_equal(want, got))
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
