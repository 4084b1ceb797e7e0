"""Pins of the oracle's vocabulary numbering (section 4.1: initial ids by lookup; a merge yields the
vocabulary's id of the merged token): hand-worked examples, and invariance of Algorithm 1 under renaming the
tokens, which ties it to the default numbering that the other pins fix."""
import random

import numpy as np
import pytest

import oracle
from conftest import read_golden

TIERS = (oracle.BRUTE, oracle.TEXTBOOK, oracle.PASSES, oracle.HEAP)


def parse_vocab(byte_spec, row_spec):
    byte_ids = np.arange(256, dtype=np.int32) + 1000
    for item in byte_spec.split(","):
        ch, val = item.split("=")
        byte_ids[ord(ch)] = int(val)
    merges, merged = [], []
    for item in row_spec.split(","):
        pair, m = item.split(">")
        l, r = pair.split(":")
        merges.append((int(l), int(r)))
        merged.append(int(m))
    return byte_ids, merges, merged


@pytest.mark.parametrize("row", read_golden("hand_worked_vocab.txt"))
def test_hand_worked_vocab_examples(row):
    byte_ids, merges, merged = parse_vocab(row[0], row[1])
    want = [int(x) for x in row[3].split(",") if x.strip()]
    t = oracle.Table(merges, byte_ids, merged)
    for tier in TIERS:
        got = t.encode(row[2].encode(), tier)
        assert got.tolist() == want, (row, tier)
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


def random_renaming(rng, n_rows):
    """A random injective renaming of the 256 + n_rows default ids."""
    return np.array(rng.sample(range(4 * (256 + n_rows) + 7), 256 + n_rows), dtype=np.int32)


def test_renaming_the_tokens_renames_the_result():
    rng = random.Random(77)
    for trial in range(40):
        alphabet = rng.sample(range(256), rng.randint(2, 5))
        rows = random_monotone_table(rng, rng.randint(1, 40), alphabet)
        phi = random_renaming(rng, len(rows))
        plain = oracle.Table(rows)
        named = oracle.Table([(phi[a], phi[b]) for a, b in rows], phi[:256], phi[256:])
        for _ in range(15):
            data = bytes(rng.choice(alphabet) for _ in range(rng.randint(0, 80)))
            want = phi[plain.encode(data, oracle.BRUTE)].tolist() if data else []
            for tier in TIERS:
                got = named.encode(data, tier)
                assert got.tolist() == want, (rows, data, tier)
            assert named.decode(named.encode(data)) == data


def test_default_numbering_is_the_identity_vocabulary():
    rng = random.Random(5)
    rows = random_monotone_table(rng, 30, [97, 98, 99])
    ident = np.arange(256 + len(rows), dtype=np.int32)
    a, b = oracle.Table(rows), oracle.Table(rows, ident[:256], ident[256:])
    for _ in range(30):
        data = bytes(rng.choice([97, 98, 99]) for _ in range(rng.randint(0, 60)))
        assert a.encode(data).tolist() == b.encode(data).tolist()
