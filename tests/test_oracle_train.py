"""Pins for the oracle's greedy trainer.  The paper uses pretrained tables, so the trainer's definition is
this build's own; it is pinned to hand-worked runs, to a direct pair count, and to a pure-Python recount."""
import collections
import random

import numpy as np
import pytest

import oracle
import workloads
from conftest import parse_rows, read_golden

WS = b" \t\n\r"


def python_trainer(corpus: bytes, n_merges: int):
    """Independent recount trainer in pure Python (same definition, nothing shared with the oracle)."""
    chunks, start = collections.Counter(), 0
    for i in range(1, len(corpus) + 1):
        if i == len(corpus) or corpus[i] in WS:
            if i > start:
                chunks[corpus[start:i]] += 1
            start = i
    words = [(list(c), f) for c, f in chunks.items()]
    rows = []
    for step in range(n_merges):
        counts = collections.Counter()
        for w, f in words:
            for p in zip(w, w[1:]):
                counts[p] += f
        if not counts:
            break
        best = min(counts, key=lambda p: (-counts[p], p))
        rows.append(best)
        for w, _ in words:
            i, out = 0, []
            while i < len(w):
                if i + 1 < len(w) and (w[i], w[i + 1]) == best:
                    out.append(256 + step)
                    i += 2
                else:
                    out.append(w[i])
                    i += 1
            w[:] = out
    return rows


@pytest.mark.parametrize("row", read_golden("hand_worked_training.txt"))
def test_hand_worked_training(row):
    corpus, n, expected = row[0], int(row[1]), parse_rows(row[2])
    for naive in (True, False):
        got = oracle.train(corpus, n, naive=naive)
        assert [tuple(r) for r in got.tolist()] == expected, f"naive={naive}"


def test_incremental_equals_naive_equals_python_on_small_corpora():
    rng = random.Random(7)
    for trial in range(12):
        alphabet = b"abcde \n" if trial % 2 else b"ab "
        corpus = bytes(rng.choice(alphabet) for _ in range(rng.randint(1, 600)))
        n = rng.randint(1, 60)
        want = python_trainer(corpus, n)
        assert [tuple(r) for r in oracle.train(corpus, n, naive=True).tolist()] == want
        assert [tuple(r) for r in oracle.train(corpus, n, naive=False).tolist()] == want


def test_trained_on_generated_text():
    corpus = workloads.text(1, 4242, 40_000)
    inc = oracle.train(corpus, 300)
    assert len(inc) == 300
    assert np.array_equal(inc, oracle.train(corpus, 300, naive=True))
    assert [tuple(r) for r in inc[:40].tolist()] == python_trainer(corpus.tobytes(), 40)
    # first row = most frequent adjacent pair inside chunks, counted directly
    counts = collections.Counter()
    b = corpus.tobytes()
    for i in range(len(b) - 1):
        if b[i + 1] not in WS:          # a pair never crosses into the next chunk
            counts[(b[i], b[i + 1])] += 1
    top = min(counts, key=lambda p: (-counts[p], p))
    assert tuple(inc[0].tolist()) == top
    # rows reference only existing tokens, and never repeat
    for r, (a, c) in enumerate(inc.tolist()):
        assert 0 <= a < 256 + r and 0 <= c < 256 + r
    assert len({tuple(r) for r in inc.tolist()}) == len(inc)


def test_stored_tables_are_wellformed():
    for key, (_, _, _, n_merges) in workloads.TABLES.items():
        m = workloads.load_merges(key)
        assert m.shape == (n_merges, 2)
        r = np.arange(n_merges)
        assert (m >= 0).all() and (m[:, 0] < 256 + r).all() and (m[:, 1] < 256 + r).all()
        packed = m[:, 0].astype(np.int64) << 32 | m[:, 1]
        assert len(np.unique(packed)) == n_merges


def test_stored_tiny_table_is_what_the_trainer_produces():
    got = oracle.train(workloads.corpus("1k"), 1000)
    assert np.array_equal(got, workloads.load_merges("1k"))
