"""Randomised differential test: random merge tables (alphabets of 1 to 60 bytes, 0 to 2,000 rows, deep
chains), random batches of strings of every kernel variant's size (with bytes that are in no row, i.e. cuts,
at three densities), optionally a vocabulary's own ids and special tokens -- GPU path against the oracle."""
import random

import numpy as np
import pytest

import oracle
from gpu_util import assert_same_encoding, gpu_encode, to_batch

pytestmark = pytest.mark.gpu

LENGTHS = [0, 1, 2, 3, 15, 16, 17, 63, 64, 65, 100, 500, 1000, 1023, 1024, 1025, 2000, 4096, 4097, 10000, 16384,
           16385, 30000, 65536]


@pytest.fixture(scope="module")
def bpe():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_11941_amd as bpe

    bpe.load_library()
    return bpe


def chained_table(rng, n_rows, alphabet):
    """Random rows whose operands exist before the row, biased towards recent tokens so that chains get deep."""
    rows, seen = [], set()
    while len(rows) < n_rows:
        pool = list(alphabet) + [256 + r for r in range(len(rows))]
        a = rng.choice(pool) if rng.random() < 0.6 else rng.choice(pool[-20:])
        b = rng.choice(pool) if rng.random() < 0.6 else rng.choice(pool[-20:])
        if (a, b) not in seen:
            seen.add((a, b))
            rows.append((a, b))
    return rows


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_tables_batches_vocabularies_and_specials(bpe, seed):
    rng = random.Random(seed)
    for trial in range(60):
        alphabet = rng.sample(range(256), rng.choice([1, 2, 3, 5, 8, 20, 60]))
        rows = chained_table(rng, rng.choice([0, 1, 5, 40, 300, 2000]), alphabet)
        merges = np.array(rows, dtype=np.int32).reshape(-1, 2)
        extra = rng.sample(range(256), rng.choice([0, 0, 2, 10]))      # bytes in no row: every bigram with them is a cut
        lens = [rng.choice(LENGTHS) for _ in range(rng.choice([1, 3, 20, 100]))]
        if sum(lens) > 400000:
            lens = lens[:10]
        pool = alphabet + extra
        weights = [1.0] * len(alphabet) + [rng.choice([0.02, 0.2, 1.0])] * len(extra)
        strings = [bytes(rng.choices(pool, weights=weights, k=n)) if n else b"" for n in lens]
        specials = {}
        if rng.random() < 0.3:
            specials = {b"<|s|>": 900001, b"[Q]": 900002}
            strings = [(s[: len(s) // 2] + rng.choice(list(specials)) + s[len(s) // 2:])[:65536]
                       if rng.random() < 0.5 else s for s in strings]
        if rng.random() < 0.3:
            phi = np.array(rng.sample(range(3 * (256 + len(rows)) + 10), 256 + len(rows)), dtype=np.int32)
            named = phi[merges]
            orc = oracle.Table(named, phi[:256], phi[256:])
            table = bpe.build_table_vocab(phi[:256], named, phi[256:])
        else:
            orc = oracle.Table(merges)
            table = bpe.build_table(merges)
        if specials:
            orc.set_specials(specials)
            table.set_specials(specials)
        data, off = to_batch(strings)
        ids, out_off = gpu_encode(table, data, off)
        want_ids, want_off = orc.encode_batch(data, off, tier=oracle.HEAP, nthreads=16)
        assert_same_encoding(ids, out_off, want_ids, want_off,
                             f"seed {seed} trial {trial}: {len(rows)} rows, alphabet {len(alphabet)}, lengths {lens[:6]}")
        table.free()
