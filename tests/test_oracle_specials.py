"""Pins of the oracle's special-token handling (section 4.1): hand-worked examples, and the defining property
that an occurrence splits the string into parts that are encoded on their own by a table that knows nothing
about special tokens."""
import random

import pytest

import oracle
from conftest import parse_ids, parse_rows, read_golden

TIERS = (oracle.BRUTE, oracle.TEXTBOOK, oracle.PASSES, oracle.HEAP)


def parse_specials(spec):
    return {k.encode(): int(v) for k, v in (item.split("=") for item in spec.split(";"))}


@pytest.mark.parametrize("row", read_golden("hand_worked_specials.txt"))
def test_hand_worked_special_examples(row):
    t = oracle.Table(parse_rows(row[0]))
    t.set_specials(parse_specials(row[1]))
    for tier in TIERS:
        got = t.encode(row[2].encode(), tier)
        assert got.tolist() == parse_ids(row[3]), (row, tier)
        assert t.decode(got) == row[2].encode()


def random_monotone_table(rng, n_rows, alphabet):
    rows, seen = [], set()
    while len(rows) < n_rows:
        pool = list(alphabet) + [256 + r for r in range(len(rows))]
        p = (rng.choice(pool), rng.choice(pool))
        if p not in seen:
            seen.add(p)
            rows.append(p)
    return rows


def test_an_occurrence_splits_the_string():
    rng = random.Random(21)
    specials = {b"<|x|>": 5000, b"<|x|>!": 5001, b"[SEP]": 5002}
    for trial in range(30):
        alphabet = [ord(c) for c in "abS|x"]             # letters of the specials take part in merges too
        rows = random_monotone_table(rng, rng.randint(1, 40), alphabet)
        plain = oracle.Table(rows)
        marked = oracle.Table(rows)
        marked.set_specials(specials)
        parts = [bytes(rng.choice(alphabet) for _ in range(rng.randint(0, 30))) for _ in range(4)]
        seps = [rng.choice(list(specials)) for _ in range(3)]
        # a part that follows "<|x|>" must not start with "!" (it does not: '!' is not in the alphabet)
        text = parts[0] + b"".join(s + p for s, p in zip(seps, parts[1:]))
        want = plain.encode(parts[0]).tolist()
        for s, p in zip(seps, parts[1:]):
            want += [specials[s]] + plain.encode(p).tolist()
        for tier in TIERS:
            assert marked.encode(text, tier).tolist() == want, (rows, text, tier)
        # removing the specials restores the plain encoding
        marked.set_specials({})
        assert marked.encode(text).tolist() == plain.encode(text).tolist()
