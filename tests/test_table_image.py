"""Host logic of the merge-table builder, checked on the table image without a GPU.

The test restates the table format (paper_2507_11941_amd/csrc/table_format.h) in Python -- placement of a
pair, tags, value fields, horizon code -- and checks the image the library builds against definitions taken
directly from the merge list: every row is found with its rank, other pairs are not found, the capability bits
say which tokens are operands of later rows, a row's limit is a valid lower bound of the first rank that uses
its token, and a byte bigram is marked as a cut exactly when it lies at no row's junction."""
import random

import numpy as np
import pytest

import paper_2507_11941_amd as bpe
import workloads

NO_RANK, CUT = 0xFFFFFFFF, 0xFFFFFFFD
M32 = 0xFFFFFFFF


SLOTS = 2                                        # per bucket; a bucket is 16 bytes, eight share a 128-byte line
FLAG_LEFT, FLAG_RIGHT, HORIZON_SHIFT = 1 << 10, 1 << 11, 2


def mul24(x, y):
    return ((x & 0xFFFFFF) * (y & 0xFFFFFF)) & M32


def place_pair(a, b, log2_buckets):
    b2 = b ^ (mul24(a, 0x9E3779) >> 12)
    a2 = a ^ (mul24(b2, 0x85EBCB) >> 12)
    return a2 & ((1 << log2_buckets) - 1), ((a2 >> log2_buckets) << 20) | b2


def lookup(words, log2_buckets, a, b):
    """Value stored for (a, b) or NO_RANK, reading the buckets as the format prescribes: the home bucket, and
    the buckets bucket ^ 1 .. bucket ^ d of its line only where the home bucket is full and records, in spare
    value bits of its two slots, that its keys reach as far as displacement d."""
    bucket, fp = place_pair(a, b, log2_buckets)
    assert fp < 1 << 27
    home = [int(x) for x in words[bucket * 2 * SLOTS:(bucket + 1) * 2 * SLOTS]]
    for k in range(SLOTS):
        if home[2 * k + 1] == fp:
            return home[2 * k] & ~3
    if home[3] != M32:
        reach = (home[0] & 3) | ((home[2] & 3) << 2)
        for d in range(1, reach + 1):
            other = [int(x) for x in words[(bucket ^ d) * 2 * SLOTS:((bucket ^ d) + 1) * 2 * SLOTS]]
            for k in range(SLOTS):
                if other[2 * k + 1] == (fp | (d << 28)):
                    return other[2 * k] & ~3
    return NO_RANK


def horizon_decode(code):
    e, m = code >> 4, code & 15
    return ((16 | m) << (e - 1)) if e else m


def random_monotone_table(rng, n_rows, alphabet):
    rows, seen = [], set()
    while len(rows) < n_rows:
        pool = list(alphabet) + [256 + r for r in range(len(rows))]
        p = (rng.choice(pool), rng.choice(pool))
        if p not in seen:
            seen.add(p)
            rows.append(p)
    return rows


def check_image(merges):
    merges = [tuple(map(int, r)) for r in merges]
    n = len(merges)
    words, log2 = bpe.table_image(merges)
    n_bucket_words = (1 << log2) * 2 * SLOTS
    assert len(words) == n_bucket_words + 256 + 65536
    assert SLOTS * (1 << log2) * 2 >= 5 * n                   # load at most 0.4
    byte_word = words[n_bucket_words:n_bucket_words + 256]
    byte_pair = words[n_bucket_words + 256:]

    first_left, first_right = {}, {}
    for r, (a, b) in enumerate(merges):
        first_left.setdefault(a, r)
        first_right.setdefault(b, r)

    # every row is found, with its own rank and a sound description of the token it creates
    for r, (a, b) in enumerate(merges):
        v = lookup(words, log2, a, b)
        assert v != NO_RANK and v >> 12 == r, (r, a, b)
        tok = 256 + r
        assert bool(v & FLAG_LEFT) == (tok in first_left) and bool(v & FLAG_RIGHT) == (tok in first_right)
        uses = [x for x in (first_left.get(tok), first_right.get(tok)) if x is not None]
        code = (v >> HORIZON_SHIFT) & 0xFF
        if uses:
            limit = r + 1 + horizon_decode(code)
            assert code != 255 and r < limit <= min(uses), (r, limit, uses)
            # the code is the tightest one: the next code up would overshoot
            assert code == 254 or r + 1 + horizon_decode(code + 1) > min(uses)
        else:
            assert code == 255
        if a < 256 and b < 256:
            assert int(byte_pair[a << 8 | b]) == v     # (the direct table never carries the overflow bit)
    # the occupied slots are exactly the rows
    tags = words[1:n_bucket_words:2]
    assert int((tags != M32).sum()) == n

    # pairs that are no row are not found
    rng = random.Random(n)
    keys = set(merges)
    for _ in range(3000):
        a, b = rng.randrange(256 + n), rng.randrange(256 + n)
        if (a, b) not in keys:
            assert lookup(words, log2, a, b) == NO_RANK

    # token words of the bytes
    for b in range(256):
        w = int(byte_word[b])
        assert w & 0xFFFFF == b
        assert bool(w & (1 << 30)) == (b in first_left) and bool(w & (1 << 31)) == (b in first_right)

    # cuts: a byte bigram is a junction iff some row joins a token ending in x with one starting in y
    first_byte, last_byte = list(range(256)), list(range(256))
    junction = set()
    for a, b in merges:
        junction.add((last_byte[a], first_byte[b]))
        first_byte.append(first_byte[a])
        last_byte.append(last_byte[b])
    for x in range(256):
        for y in range(256):
            e = int(byte_pair[x << 8 | y])
            if (x, y) in keys:
                assert e >> 12 == merges.index((x, y)) if n < 2000 else e not in (NO_RANK, CUT)
            elif (x, y) in junction:
                assert e == NO_RANK, (x, y)
            else:
                assert e == CUT, (x, y)


def test_empty_and_tiny_tables():
    check_image([])
    check_image([(97, 97)])
    check_image([(97, 98), (98, 99), (256, 99), (258, 258)])


def test_random_tables():
    rng = random.Random(99)
    for trial in range(25):
        alphabet = rng.sample(range(256), rng.randint(2, 40))
        check_image(random_monotone_table(rng, rng.randint(1, 600), alphabet))


def test_doubling_chain_horizons():
    """Row r = (token r-1 twice): each token is used by the very next row, so every limit is rank + 1."""
    rows = [(97, 97)] + [(256 + r, 256 + r) for r in range(40)]
    words, log2 = bpe.table_image(rows)
    for r, (a, b) in enumerate(rows):
        v = lookup(words, log2, a, b)
        assert v >> 12 == r
        assert ((v >> HORIZON_SHIFT) & 0xFF) == (0 if r + 1 < len(rows) else 255)


@pytest.mark.parametrize("key", ["1k", "32k", "100k"])
def test_trained_tables(key):
    check_image(workloads.load_merges(key))


def test_image_rejects_what_build_table_rejects():
    with pytest.raises(bpe.BpeError) as e:
        bpe.table_image([(97, 98), (258, 99)])
    assert e.value.code == -2
    with pytest.raises(bpe.BpeError) as e:
        bpe.table_image([(97, 98), (97, 98)])
    assert e.value.code == -3
