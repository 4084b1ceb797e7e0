"""Train and store the merge tables of the benchmark configurations.

    python oracle/make_tables.py [1k] [32k] [100k]

For each table: regenerate its seeded corpus (``workloads.corpus``), run the oracle's greedy trainer on it
and write the rows as little-endian int32 pairs to ``workloads/tables/merges_<key>.bin`` (row index = rank,
merged id = 256 + rank).  The stored files are inputs to both the oracle and the HIP path; they are produced
here, by the oracle's trainer alone.
"""
from __future__ import annotations

import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import oracle  # noqa: E402
import workloads  # noqa: E402


def make(key: str) -> None:
    style, nbytes, seed, n_merges = workloads.TABLES[key]
    t0 = time.time()
    corpus = workloads.corpus(key)
    t1 = time.time()
    merges = oracle.train(corpus, n_merges)
    t2 = time.time()
    if len(merges) != n_merges:
        raise SystemExit(f"table {key}: corpus sustained only {len(merges)} of {n_merges} merges")
    path = workloads.table_path(key)
    os.makedirs(os.path.dirname(path), exist_ok=True)
    merges.astype("<i4").tofile(path)
    print(f"table {key}: style {style}, corpus {nbytes} B seed {seed} ({t1 - t0:.1f} s), "
          f"{n_merges} merges trained in {t2 - t1:.1f} s -> {path}", flush=True)


if __name__ == "__main__":
    for k in (sys.argv[1:] or list(workloads.TABLES)):
        make(k)
