"""Throughput of bpe_encode_batch on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C]

A step is one whole bpe_encode_batch call (cutting long strings into pieces, the per-piece merge kernels, the
offset scan and the packing) over one synthetic batch that is already resident in HBM.  The default workload
is configuration 5, the throughput configuration: 100,000 merges, 65,536 strings with log-normal lengths
(64 B - 64 KiB), 211 MiB of input.  Prints one JSON line: input GB/s as `value`, plus tokens/s, the HBM roofline
of the encode kernel, the CPU oracle timed on this host as a baseline, and a short timing of the other four
configurations under `extra.per_config`.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E peak, GB/s
VALU_PEAK_GIPS = 256 * 4 * 2.4 / 4      # 256 CUs x 4 SIMDs, one wave64 vector instruction per 4 cycles at 2.4 GHz


def kernel_source_sha16() -> str:
    """Identifies the kernels a counter summary under profiles/ was taken with: a hash over the library's
    sources.  Counter figures are only quoted beside a run of the same sources."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2507_11941_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".h", ".hip")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def committed_counters(config: int):
    """Figures that cannot be read from inside this process (rocprofv3 --pmc runs of this same command): HBM-side
    bytes and vector wave-instructions per encode-kernel launch, from profiles/bpe_encode_batch_config<C>.md.
    Returns (traffic, valu, sha16 of the sources they were measured with); all None if there is no summary."""
    path = os.path.join(ROOT, "profiles", f"bpe_encode_batch_config{config}.md")
    try:
        text = open(path).read()
    except OSError:
        return None, None, None

    def find(key, conv):
        m = re.search(rf"^{key}\s*=\s*(\S+)", text, flags=re.M)
        return conv(m.group(1)) if m else None

    return (find("traffic_bytes_per_launch", int), find("valu_wave_instructions_per_launch", int),
            find("kernel_source_sha16", str))


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


def host_threads() -> int:
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    return max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores))))


def cpu_baseline(merges, data, offsets, budget_seconds=12.0):
    """The oracle's textbook sequential encoder, as it stands, on this host: (i) all threads over a prefix of the
    batch sized to the time budget (the whole batch when it fits), (ii) one thread on the first strings."""
    import numpy as np

    import oracle

    cores = host_threads()
    table = oracle.Table(merges)
    batch = len(offsets) - 1

    def run(n_strings, threads):
        sub = data[: int(offsets[n_strings])]
        t0 = time.perf_counter()
        ids, _ = table.encode_batch(sub, offsets[: n_strings + 1], tier=oracle.TEXTBOOK, nthreads=threads)
        return time.perf_counter() - t0, len(sub), len(ids)

    # the textbook encoder is quadratic in the string length, so time is not proportional to bytes: probe a small
    # prefix and grow it until the budget is in sight
    n = min(batch, max(64, 4 * cores))
    wall, nbytes, ntok = run(n, cores)
    while n < batch and wall < budget_seconds / 4:
        n = min(batch, max(n * 2, int(n * (budget_seconds / 2) / max(wall, 1e-3))))
        wall, nbytes, ntok = run(n, cores)
    n1 = min(batch, 256)
    while n1 > 8 and wall * cores * n1 / n > budget_seconds:     # keep the one-thread leg inside the budget too
        n1 //= 2
    wall1, nbytes1, _ = run(n1, 1)
    sample = min(batch, 16)
    _, _, st = table.encode_batch(data[: int(offsets[sample])], offsets[: sample + 1], tier=oracle.PASSES,
                                  nthreads=cores, stats=True)
    return {
        "value": nbytes / wall / 1e9,
        "unit": "GB/s",
        "tokens_per_s": ntok / wall,
        "cores": cores,
        "kind": "oracle",
        "sample": f"first {n} of {batch} strings ({nbytes} bytes), textbook sequential encoder on {cores} threads, "
                  f"{wall:.1f} s wall",
        "single_thread": {"value": nbytes1 / wall1 / 1e9, "unit": "GB/s", "cores": 1,
                          "sample": f"first {n1} strings ({nbytes1} bytes), {wall1:.1f} s wall"},
        # the work model of the one-rank-per-pass view (section 4.2) on a few strings: passes and token visits
        "pass_view": {"strings": sample, "passes_per_string": st["passes"] / max(sample, 1),
                      "token_visits_per_byte": st["visits"] / max(int(offsets[sample]), 1)},
    }


class Workload:
    """One configuration's batch, resident on the device, with its outputs and workspace."""

    def __init__(self, config: int, dev, tables):
        import numpy as np
        import torch

        import paper_2507_11941_amd as bpe
        import workloads

        self.cfg = workloads.CONFIGS[config]
        if self.cfg.table not in tables:
            merges = workloads.load_merges(self.cfg.table)
            tables[self.cfg.table] = (merges, bpe.build_table(merges))
        self.merges, self.table = tables[self.cfg.table]
        self.data, self.offsets = workloads.batch(config)
        self.batch = len(self.offsets) - 1
        self.total = int(self.offsets[-1])
        self.max_len = int(np.diff(self.offsets).max())
        self.d_data = torch.from_numpy(self.data).to(dev)
        self.d_off = torch.from_numpy(self.offsets).to(dev)
        self.out_ids = torch.empty(self.total, dtype=torch.int32, device=dev)
        self.out_off = torch.empty(self.batch + 1, dtype=torch.int64, device=dev)
        self.ws = torch.empty(bpe.workspace_bytes(self.batch, self.total, self.max_len), dtype=torch.uint8,
                              device=dev)
        self.stream = torch.cuda.current_stream(dev)
        self._encode = bpe.encode_batch

    def step(self):
        self._encode(self.table, self.d_data, self.d_off, self.max_len, self.out_ids, self.out_off, self.ws,
                     self.stream)

    def time_steps(self, steps, warmup):
        """(ms per step over exactly `steps` back-to-back calls, tokens).  Nothing else is on the stream."""
        import torch

        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record(self.stream)
        for _ in range(steps):
            self.step()
        ev1.record(self.stream)
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / steps, int(self.out_off[-1].item())

    def time_each(self, steps):
        """Per-step and per-encode-kernel durations of `steps` more calls: every call sits between two events on
        the stream, and the library records an event pair around its encode kernels.  Kept out of the timed region
        because an event record between two kernels costs the stream a few microseconds."""
        import torch

        import paper_2507_11941_amd as bpe

        steps = min(steps, 512)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        bpe.set_profiling(True)
        marks[0].record(self.stream)
        for i in range(steps):
            self.step()
            marks[i + 1].record(self.stream)
        torch.cuda.synchronize()
        kernel_ms_total, kernel_calls = bpe.read_profile()
        bpe.set_profiling(False)
        each = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
        return each, kernel_ms_total / max(kernel_calls, 1), kernel_calls

    def release(self):
        self.d_data = self.d_off = self.out_ids = self.out_off = self.ws = None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, help="workload configuration 1..5 (default 5); 6 = 256 strings of 64 KiB of one byte each, which "
                         "only the HBM-staged kernel variant can take")
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the oracle legs (baseline and comparison) and the other configurations")
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

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    bpe.load_library()
    dev = torch.device("cuda:0")
    tables = {}
    w = Workload(args.config, dev, tables)

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ms_per_step, n_tokens = w.time_steps(args.steps, args.warmup)        # the timed region
    each, kernel_ms, kernel_calls = w.time_each(args.steps)

    # algorithmic HBM bytes of one encode: read every input byte and two offsets per string, write every id
    # and one count per string
    algo_bytes = w.total + 4 * n_tokens + 16 * w.batch
    achieved = algo_bytes / (kernel_ms * 1e-3) / 1e9
    traffic, valu, profiled_sha = committed_counters(args.config)
    current = profiled_sha == kernel_source_sha16()

    result = {
        "metric": "bpe_encode_batch input throughput",
        "value": w.total / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "tokens_per_s": n_tokens / (ms_per_step * 1e-3),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_median": each[len(each) // 2],
        "ms_per_step_min": each[0],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",                           # all arithmetic is on 32-bit unsigned words (ranks, ids, masks)
        "io": "u8 bytes in, i32 ids and i64 offsets out",
        "data": "synthetic",
        "config": {"workload": f"config {args.config}: {w.cfg.name}", "table_merges": int(len(w.merges)),
                   "batch": w.batch, "input_bytes": w.total, "max_len": w.max_len, "tokens": n_tokens},
        "hbm_fraction_input": w.total / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "kernel": "encode kernels of one call", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     # from the committed rocprofv3 counter runs of this command; null unless they were taken with
                     # the kernels that are running now
                     "traffic": traffic if current else None,
                     "traffic_source": (f"profiles/bpe_encode_batch_config{args.config}.md" if current and traffic
                                        else None),
                     "algorithmic_bytes_per_launch": algo_bytes, "kernel_ms": kernel_ms,
                     "kernel_calls_timed": kernel_calls},
    }
    # the method's own look-up counts (section 4.2: every pair is looked up once, when it comes into being): the
    # n - 1 initial byte pairs of a string go to the direct 256 x 256 table, and each of the n - k merges creates
    # at most two pairs that go to the hash table
    result["work"] = {"direct_table_lookups": w.total - w.batch, "merges": w.total - n_tokens,
                      "hash_probes_upper_bound": 2 * (w.total - n_tokens)}
    if valu is not None and current:                     # how busy the vector ALUs are: the limit that applies
        rate = valu / (kernel_ms * 1e-3) / 1e9
        result["issue"] = {"bound": "alu", "achieved": rate, "peak": VALU_PEAK_GIPS, "unit": "G wave-instr/s",
                           "frac": rate / VALU_PEAK_GIPS, "valu_wave_instructions_per_launch": valu,
                           "source": f"profiles/bpe_encode_batch_config{args.config}.md (same kernel sources)"}
    if not args.no_cpu_baseline:
        import oracle

        result["stream_copy_GBs"] = stream_copy_gbs(dev)
        # the whole batch against the oracle's heap encoder (all threads): ids and offsets
        got_off = w.out_off.cpu().numpy()
        got_ids = w.out_ids[:n_tokens].cpu().numpy()
        want_ids, want_off = oracle.Table(w.merges).encode_batch(w.data, w.offsets, tier=oracle.HEAP,
                                                                 nthreads=host_threads())
        result["matches_oracle"] = bool(np.array_equal(got_off, want_off) and np.array_equal(got_ids, want_ids))
        del want_ids, got_ids
        result["cpu_baseline"] = cpu_baseline(w.merges, w.data, w.offsets)
        # the other configurations, briefly (same call, same timing method)
        per_config = []
        w.release()
        for c in (1, 2, 3, 4, 5):
            if c == args.config:
                continue
            o = Workload(c, dev, tables)
            ms, tok = o.time_steps(max(10, min(args.steps, 200 if o.total < (8 << 20) else 20)), 3)
            _, kms, _ = o.time_each(10)
            per_config.append({"workload": f"config {c}: {o.cfg.name}", "input_bytes": o.total, "tokens": tok,
                               "ms_per_step": ms, "GB/s": o.total / (ms * 1e-3) / 1e9,
                               "tokens_per_s": tok / (ms * 1e-3), "encode_kernel_ms": kms})
            o.release()
        result["extra"] = {"per_config": per_config}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
