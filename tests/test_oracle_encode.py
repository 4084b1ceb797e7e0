"""Pins for the CPU oracle's encoders: values and properties fixed by the paper's Algorithm 1 and by
mathematics, none of them produced by the oracle itself."""
import itertools
import random

import numpy as np
import pytest

import oracle
from conftest import parse_ids, parse_rows, read_golden

TIERS = [oracle.BRUTE, oracle.TEXTBOOK, oracle.PASSES, oracle.HEAP]


def naive_python_bpe(merges, data: bytes):
    """Independent transcription of Algorithm 1 (section 3.1) in pure Python: O(n^2) merge loop."""
    rank = {}
    for r, (a, b) in enumerate(merges):
        rank.setdefault((a, b), r)
    toks = list(data)
    while True:
        cands = [(rank[p], i) for i, p in enumerate(zip(toks, toks[1:])) if p in rank]
        if not cands:
            return toks
        r, i = min(cands)          # lowest rank, then left-most
        toks[i:i + 2] = [256 + r]


@pytest.mark.parametrize("row", read_golden("hand_worked_encodings.txt"))
def test_hand_worked_examples(row):
    rows, text, expected, passes = parse_rows(row[0]), row[1], parse_ids(row[2]), int(row[3])
    t = oracle.Table(rows)
    for tier in TIERS:
        assert t.encode(text, tier).tolist() == expected, f"tier {tier}"
    _, st = t.encode(text, oracle.PASSES, stats=True)
    assert st["passes"] == passes
    assert st["merges"] == len(text.encode()) - len(expected)


def test_doubling_chain_closed_form():
    """Rows (a,a), (256,256), (257,257), ...: 'a'*n with n = q*2^D + rem encodes to q top-level tokens
    followed by one token per set bit of rem, high bit first; passes = min(D, floor(log2 n))."""
    D = 5
    rows = [(97, 97)] + [(255 + j, 255 + j) for j in range(1, D)]
    level = [97] + [255 + j for j in range(1, D + 1)]          # token of 2^j letters
    t = oracle.Table(rows)
    for n in range(0, 200):
        q, rem = divmod(n, 1 << D)
        expected = [level[D]] * q + [level[j] for j in range(D - 1, -1, -1) if rem >> j & 1]
        for tier in TIERS:
            assert t.encode("a" * n, tier).tolist() == expected, (n, tier)
        _, st = t.encode("a" * n, oracle.PASSES, stats=True)
        assert st["passes"] == (0 if n == 0 else min(D, n.bit_length() - 1))


def test_alternating_pair_and_empty_table():
    t = oracle.Table([(120, 121)])
    for k in range(0, 40):
        for tier in TIERS:
            assert t.encode("xy" * k, tier).tolist() == [256] * k
            assert t.encode("xy" * k + "x", tier).tolist() == [256] * k + [120]
            assert t.encode("y" + "xy" * k, tier).tolist() == [121] + [256] * k
    e = oracle.Table(np.zeros((0, 2), dtype=np.int32))
    data = bytes(range(256)) * 2
    for tier in TIERS:
        assert e.encode(data, tier).tolist() == list(data)
    _, st = e.encode(data, oracle.PASSES, stats=True)
    assert st == {"passes": 0, "visits": 0, "merges": 0}


SMALL_TABLES = [
    [(97, 97)],
    [(97, 98), (98, 97)],
    [(97, 98), (98, 99), (256, 99), (258, 258)],
    [(98, 99), (97, 98), (257, 99), (97, 256)],
    [(97, 97), (256, 97), (97, 256), (256, 256), (98, 98), (260, 260), (99, 97)],
    [(99, 99), (256, 256), (257, 99), (99, 257), (97, 99), (98, 258)],
]


@pytest.mark.parametrize("rows", SMALL_TABLES)
def test_exhaustive_small_alphabet_against_python_transcription(rows):
    """Every string over {a,b,c} up to length 9: all four encoders equal the pure-Python Algorithm 1."""
    t = oracle.Table(rows)
    for n in range(0, 10):
        for tup in itertools.product(b"abc", repeat=n):
            data = bytes(tup)
            want = naive_python_bpe(rows, data)
            for tier in TIERS:
                assert t.encode(data, tier).tolist() == want, (data, tier)


def random_monotone_table(rng, n_rows, alphabet):
    """Random table with the trained-table property: a row's operands exist before the row."""
    rows, seen = [], set()
    while len(rows) < n_rows:
        pool = list(alphabet) + [256 + r for r in range(len(rows))]
        p = (rng.choice(pool), rng.choice(pool))
        if p not in seen:
            seen.add(p)
            rows.append(p)
    return rows


def test_random_tables_against_python_transcription():
    rng = random.Random(1234)
    for trial in range(60):
        alphabet = rng.sample(range(256), rng.randint(2, 5))
        rows = random_monotone_table(rng, rng.randint(1, 40), alphabet)
        t = oracle.Table(rows)
        for _ in range(20):
            data = bytes(rng.choice(alphabet) for _ in range(rng.randint(0, 80)))
            want = naive_python_bpe(rows, data)
            for tier in TIERS:
                assert t.encode(data, tier).tolist() == want, (rows, data, tier)


def expand(rows, tok):
    return bytes([tok]) if tok < 256 else expand(rows, rows[tok - 256][0]) + expand(rows, rows[tok - 256][1])


def test_invariants_on_random_inputs():
    """Round trip, fixed point, length bounds, prefix-table property, strictly increasing pass ranks."""
    rng = random.Random(99)
    for trial in range(40):
        alphabet = rng.sample(range(256), rng.randint(2, 6))
        rows = random_monotone_table(rng, rng.randint(1, 60), alphabet)
        keys = set(rows)
        t = oracle.Table(rows)
        for _ in range(10):
            data = bytes(rng.choice(alphabet) for _ in range(rng.randint(0, 300)))
            ids = t.encode(data, oracle.TEXTBOOK).tolist()
            # decode(encode(x)) == x, by the oracle's decoder and by an independent expansion
            assert t.decode(ids) == data
            assert b"".join(expand(rows, i) for i in ids) == data
            # fixed point: no adjacent output pair is in the table
            assert not any(p in keys for p in zip(ids, ids[1:]))
            # k <= n, k == n iff no pair of x is in the table, k == 0 iff n == 0
            assert len(ids) <= len(data)
            assert (len(ids) == len(data)) == (not any(p in keys for p in zip(data, data[1:])))
            assert all(0 <= i < 256 + len(rows) for i in ids)
            # encoding with the first m rows, then continuing with all rows, equals encoding with all rows
            m = rng.randint(0, len(rows))
            part = oracle.Table(rows[:m]).encode(data, oracle.TEXTBOOK).tolist()
            assert continue_encoding(rows, part) == ids
            assert t.encode(data, oracle.HEAP).tolist() == ids
            assert t.encode(data, oracle.PASSES).tolist() == ids
            check_pass_invariants(t, data, len(ids))


def check_pass_invariants(table, data, n_tokens):
    """The one-rank-per-pass view (section 4.2) of a table whose rows only use older tokens: the rank applied
    strictly increases from pass to pass, every pass applies at least one merge, and a pass that starts with
    L live tokens and applies m merges leaves L - m."""
    trace = table.pass_trace(data)
    live = len(data)
    last_rank = -1
    for rank, live_before, merges in trace:
        assert rank > last_rank, trace
        assert live_before == live and merges >= 1
        live -= merges
        last_rank = rank
    assert live == n_tokens


def test_pass_trace_hand_worked():
    """'abcabcabc' with rows ab, bc, (ab)c, (abc)(abc): rank 0 three times, rank 2 three times, rank 3 once (row 1,
    'bc', never applies: its b is taken by 'ab' first)."""
    t = oracle.Table([(97, 98), (98, 99), (256, 99), (258, 258)])
    assert t.pass_trace("abcabcabc") == [(0, 9, 3), (2, 6, 3), (3, 3, 1)]
    assert t.pass_trace("") == [] and t.pass_trace("zzz") == []
    # a table that breaks the operand-order rule is where the pass view leaves Algorithm 1: the invariant is
    # a property of valid tables, not of the code (ranks go 1, then 0: not increasing)
    bad = oracle.Table([(256 + 1, 99), (97, 98)])
    assert [r for r, _, _ in bad.pass_trace("abc")] == [1, 0]


def continue_encoding(rows, toks):
    rank = {p: r for r, p in reversed(list(enumerate(rows)))}
    toks = list(toks)
    while True:
        cands = [(rank[p], i) for i, p in enumerate(zip(toks, toks[1:])) if p in rank]
        if not cands:
            return toks
        r, i = min(cands)
        toks[i:i + 2] = [256 + r]


def test_pass_counters_match_their_definition():
    """passes = number of distinct ranks applied; visits = sum of live tokens at the start of each pass."""
    rows = [(97, 98), (98, 99), (256, 99), (258, 258)]
    t = oracle.Table(rows)
    # "abcabcabc": 9 tokens -> pass rank 0 (3 merges) -> 6 -> pass rank 2 (3 merges) -> 3 -> pass rank 3 -> 2
    _, st = t.encode("abcabcabc", oracle.PASSES, stats=True)
    assert st == {"passes": 3, "visits": 9 + 6 + 3, "merges": 3 + 3 + 1}


def test_batch_is_independent_of_neighbours_and_threads():
    rng = random.Random(5)
    rows = random_monotone_table(rng, 50, [97, 98, 99, 32])
    t = oracle.Table(rows)
    strings = [bytes(rng.choice([97, 98, 99, 32]) for _ in range(rng.randint(0, 120))) for _ in range(37)]
    strings[5] = b""
    data = np.frombuffer(b"".join(strings), dtype=np.uint8)
    offsets = np.cumsum([0] + [len(s) for s in strings])
    for tier in (oracle.TEXTBOOK, oracle.HEAP):
        for nthreads in (1, 4):
            ids, off = t.encode_batch(data, offsets, tier=tier, nthreads=nthreads)
            assert off[0] == 0 and len(off) == len(strings) + 1 and off[-1] == len(ids)
            for i, s in enumerate(strings):
                assert ids[off[i]:off[i + 1]].tolist() == naive_python_bpe(rows, s)
