"""The oracle's three fast encoders against each other at scale, on the stored tables: the heap encoder is the
whole-batch checker of the large GPU parity runs, so it is admitted here on more than 10^5 strings of the
benchmark's own text styles (and on the adversarial strings) by agreeing with the textbook one-merge-at-a-time
encoder and with the one-rank-per-pass view; the pass invariants are checked on a sample of the same strings."""
import numpy as np
import pytest

import oracle
import workloads

THREADS = 8


def ragged(style, seed, count, lo, hi):
    rng = np.random.default_rng(seed)
    lens = rng.integers(lo, hi + 1, size=count)
    off = np.zeros(count + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    return workloads.text(style, seed, int(off[-1])), off


@pytest.mark.parametrize("key,style,count", [("32k", 2, 60_000), ("100k", 3, 60_000)])
def test_heap_textbook_and_pass_view_agree_on_text(key, style, count):
    table = oracle.Table(workloads.load_merges(key))
    data, off = ragged(style, 4242 + style, count, 8, 160)
    want_ids, want_off = table.encode_batch(data, off, tier=oracle.TEXTBOOK, nthreads=THREADS)
    for tier in (oracle.HEAP, oracle.PASSES):
        ids, o = table.encode_batch(data, off, tier=tier, nthreads=THREADS)
        assert np.array_equal(o, want_off) and np.array_equal(ids, want_ids), tier
    # I6 / I7 on a sample: strictly increasing ranks, every pass merges, live counts add up
    for i in range(0, count, 997):
        s = data[off[i]:off[i + 1]].tobytes()
        live, last = len(s), -1
        for rank, live_before, merges in table.pass_trace(s):
            assert rank > last and live_before == live and merges >= 1
            live, last = live - merges, rank
        assert live == want_off[i + 1] - want_off[i]


def test_heap_textbook_and_pass_view_agree_on_adversarial_strings():
    """Configuration 4's runs and repeated motifs (overlapping self pairs, deep merge chains), cut to 1 KiB."""
    table = oracle.Table(workloads.load_merges("100k"))
    data = workloads.adversarial(workloads.BATCH_SEED, 64, 16384).reshape(-1, 1024)[:768].reshape(-1)
    off = np.arange(769, dtype=np.int64) * 1024
    want_ids, want_off = table.encode_batch(data, off, tier=oracle.TEXTBOOK, nthreads=THREADS)
    for tier in (oracle.HEAP, oracle.PASSES):
        ids, o = table.encode_batch(data, off, tier=tier, nthreads=THREADS)
        assert np.array_equal(o, want_off) and np.array_equal(ids, want_ids), tier
