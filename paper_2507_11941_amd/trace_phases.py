"""Per-phase time breakdown of the encode kernel (developer tool).

    python -m paper_2507_11941_amd.trace_phases [--counts | --probes] [config] [batch]

Builds a second copy of the library with -DBPE_TRACE (libbpe_hip_trace.so), encodes `batch` strings of the
configuration once and prints, for the first string that workgroup 0 encodes, the shader-clock ticks thread 0
spent in each phase of the pass loop, plus the pass count.
"""
from __future__ import annotations

import ctypes
import os
import sys

import numpy as np

PHASES = ["load", "minima sweep", "scans+neighbours+candidates", "walk1", "parity scan", "walk2",
          "successor exchange", "probes",
          "refresh+publish", "emit", "passes", "total"]


def main() -> int:
    args = [a for a in sys.argv[1:] if not a.startswith("--")]
    counts = "--counts" in sys.argv[1:]        # loop-trip and per-lane counts instead of clean clock figures
    probes = "--probes" in sys.argv[1:]        # extra clock points inside the probe loop (they lengthen it)
    cfg = int(args[0]) if len(args) > 0 else 2
    batch = int(args[1]) if len(args) > 1 else 1
    import torch

    from . import _binding, build as hip_build

    lib_path = os.path.join(os.path.dirname(os.path.abspath(__file__)),
                            "libbpe_hip_counts.so" if counts else
                            "libbpe_hip_probes.so" if probes else "libbpe_hip_trace.so")
    saved = hip_build.LIB
    hip_build.LIB = lib_path
    try:
        hip_build.build(force=False, extra_flags=("-DBPE_TRACE", "-DBPE_TRACE_COUNTS") if counts else
                        ("-DBPE_TRACE", "-DBPE_TRACE_PROBES") if probes else ("-DBPE_TRACE",))   # only if missing or older than the sources
    finally:
        hip_build.LIB = saved
    _binding._LIB_PATH = lib_path
    lib = _binding.load_library()
    lib.bpe_debug_trace.argtypes = [ctypes.c_void_p, ctypes.c_int]

    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import workloads

    c = workloads.CONFIGS[cfg]
    table = _binding.build_table(workloads.load_merges(c.table))
    data, off = workloads.batch(cfg, batch_override=batch)
    dev = torch.device("cuda:0")
    d, o = torch.from_numpy(data).to(dev), torch.from_numpy(off).to(dev)
    max_len = int(np.diff(off).max())
    for _ in range(3):
        _binding.encode_batch(table, d, o, max_len)
    torch.cuda.synchronize()
    lib.bpe_debug_trace(None, 1)
    _binding.encode_batch(table, d, o, max_len)
    torch.cuda.synchronize()
    t = np.zeros(128, dtype=np.uint64)
    lib.bpe_debug_trace(t.ctypes.data, 0)
    passes = max(int(t[10]), 1)
    print(f"config {cfg}, batch {batch}: {int(t[10])} passes, {int(t[11])} ticks in all")
    if counts:
        print(f"  loop trips of the wave: walk1 {int(t[12])}, walk2 {int(t[13])}, probe loop {int(t[8])};  "
              f"summed over lanes: candidates {int(t[15])}, applied {int(t[16])}, look-ups {int(t[14])}, "
              f"of which sent to the table {int(t[20])}")
        return 0
    if probes:
        print(f"  inside the probe loop: operands from LDS {int(t[19])}, hash + loads + wait {int(t[17])}, "
              f"compare + store {int(t[18])}")
    if "--per-pass" in sys.argv[1:]:
        print("  per pass: " + " | ".join(PHASES[1:8]))
        for ps in range(12):
            row = [int(t[32 + 8 * ps + ph]) for ph in range(1, 8)]
            if any(row):
                print(f"  pass {ps + 1:2d}: " + " ".join(f"{x:7d}" for x in row))
    print("  ticks of pass 1, 2, ...: " + ", ".join(str(int(x)) for x in t[21:32] if int(x)))
    for name, v in zip(PHASES[:10], t[:10]):
        if name == "refresh+publish":
            continue
        per = f"{int(v) / passes:9.0f} / pass" if name not in ("load", "emit") else ""
        print(f"  {name:28s} {int(v):10d} ticks {100.0 * int(v) / max(int(t[11]), 1):5.1f} %  {per}")
    return 0


if __name__ == "__main__":
    sys.exit(main())
