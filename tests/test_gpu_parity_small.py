"""GPU parity, small cases: the HIP path (through the C ABI) against the CPU oracle and against the
hand-worked values, bit for bit.  Token ids are integers: the bar is exact equality."""
import random

import numpy as np
import pytest

import oracle
import workloads
from conftest import parse_ids, parse_rows, read_golden
from gpu_util import assert_same_encoding, gpu_encode, to_batch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bpe():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_11941_amd as bpe

    bpe.load_library()
    return bpe


def test_hand_worked_examples(bpe):
    by_table = {}
    for row in read_golden("hand_worked_encodings.txt"):
        by_table.setdefault(row[0], []).append((row[1].encode(), parse_ids(row[2])))
    for spec, cases in by_table.items():
        table = bpe.build_table(parse_rows(spec))
        data, off = to_batch([c[0] for c in cases])
        ids, out_off = gpu_encode(table, data, off)
        for i, (text, want) in enumerate(cases):
            assert ids[out_off[i]:out_off[i + 1]].tolist() == want, (spec, text)
        # and one string per call
        for text, want in cases:
            ids1, off1 = gpu_encode(table, *to_batch([text]))
            assert ids1.tolist() == want and off1.tolist() == [0, len(want)]
        table.free()


def test_doubling_chain_closed_form(bpe):
    """'a'*n under rows (a,a),(256,256),...: q top-level tokens then one token per set bit of the rest."""
    D = 5
    rows = [(97, 97)] + [(255 + j, 255 + j) for j in range(1, D)]
    level = [97] + [255 + j for j in range(1, D + 1)]
    table = bpe.build_table(rows)
    lengths = list(range(0, 200)) + [1023, 1024, 1025, 4095, 4096, 4097, 16384, 16385, 50001, 65535, 65536]
    data, off = to_batch([b"a" * n for n in lengths])
    ids, out_off = gpu_encode(table, data, off)
    for i, n in enumerate(lengths):
        q, rem = divmod(n, 1 << D)
        want = [level[D]] * q + [level[j] for j in range(D - 1, -1, -1) if rem >> j & 1]
        assert ids[out_off[i]:out_off[i + 1]].tolist() == want, n


def test_deep_doubling_chain(bpe):
    """16 levels of doubling: 65536 letters collapse to one token; every pass is a self pair."""
    D = 16
    rows = [(97, 97)] + [(255 + j, 255 + j) for j in range(1, D)]
    table = bpe.build_table(rows)
    orc = oracle.Table(rows)
    lengths = [65536, 65535, 40000, 16384, 4096, 1000, 3]
    data, off = to_batch([b"a" * n for n in lengths])
    ids, out_off = gpu_encode(table, data, off)
    want_ids, want_off = orc.encode_batch(data, off, tier=oracle.HEAP)
    assert_same_encoding(ids, out_off, want_ids, want_off, "deep doubling")
    assert ids[:1].tolist() == [255 + D]


def random_monotone_table(rng, n_rows, alphabet):
    rows, seen = [], set()
    while len(rows) < n_rows:
        pool = list(alphabet) + [256 + r for r in range(len(rows))]
        p = (rng.choice(pool), rng.choice(pool))
        if p not in seen:
            seen.add(p)
            rows.append(p)
    return rows


def test_random_tables_and_strings(bpe):
    """Small alphabets and random tables make overlaps, self pairs and deep chains frequent."""
    rng = random.Random(2024)
    for trial in range(25):
        alphabet = rng.sample(range(256), rng.randint(2, 5))
        rows = random_monotone_table(rng, rng.randint(1, 200), alphabet)
        strings = [bytes(rng.choice(alphabet) for _ in range(rng.choice([0, 1, 2, 3, 17, 64, 65, 300, 1500, 5000])))
                   for _ in range(40)]
        data, off = to_batch(strings)
        table = bpe.build_table(rows)
        ids, out_off = gpu_encode(table, data, off)
        want_ids, want_off = oracle.Table(rows).encode_batch(data, off, tier=oracle.TEXTBOOK, nthreads=8)
        assert_same_encoding(ids, out_off, want_ids, want_off, f"trial {trial}")
        table.free()


def test_empty_and_degenerate_batches(bpe):
    table = bpe.build_table([(97, 98), (256, 99)])
    ids, off = gpu_encode(table, np.zeros(0, np.uint8), np.zeros(1, np.int64), max_len=0)
    assert ids.tolist() == [] and off.tolist() == [0]
    ids, off = gpu_encode(table, *to_batch([b"", b"", b""]))
    assert ids.tolist() == [] and off.tolist() == [0, 0, 0, 0]
    ids, off = gpu_encode(table, *to_batch([b"", b"a", b"", b"abc", b"ab", b""]))
    assert ids.tolist() == [97, 257, 256] and off.tolist() == [0, 0, 1, 1, 2, 3, 3]
    # empty table: ids are the bytes
    empty = bpe.build_table(np.zeros((0, 2), np.int32))
    raw = bytes(range(256)) * 5
    ids, off = gpu_encode(empty, *to_batch([raw, b"xyz"]))
    assert ids.tolist() == list(raw) + [120, 121, 122] and off.tolist() == [0, len(raw), len(raw) + 3]


def test_max_len_too_small_is_harmless(bpe):
    """A string longer than max_len has unspecified output (encoded, or no tokens); the others are exact."""
    table = bpe.build_table([(97, 98)])
    strings = [b"ab" * 10, b"ab" * 3000, b"ab"]
    ids, off = gpu_encode(table, *to_batch(strings), max_len=64)
    assert off[0] == 0 and off[1] == 10 and off[3] - off[2] == 1
    assert ids[:10].tolist() == [256] * 10 and ids[off[2]:off[3]].tolist() == [256]
    assert off[2] - off[1] in (0, 3000)
    ids, off = gpu_encode(table, *to_batch(strings), max_len=6000)
    assert off.tolist() == [0, 10, 3010, 3011] and (ids == 256).all()


def test_encode_rejects_bad_arguments(bpe):
    import torch

    table = bpe.build_table([(97, 98)])
    data = torch.zeros(16, dtype=torch.uint8, device="cuda:0")
    offsets = torch.tensor([0, 16], dtype=torch.int64, device="cuda:0")
    with pytest.raises(bpe.BpeError):
        bpe.encode_batch(table, data, offsets, max_len=bpe.MAX_STRING_BYTES + 1)
    short = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(bpe.BpeError):
        bpe.encode_batch(table, data, offsets, max_len=16, workspace=short)
    torch.cuda.synchronize()


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


def test_hand_worked_vocab_examples(bpe):
    by_table = {}
    for row in read_golden("hand_worked_vocab.txt"):
        by_table.setdefault((row[0], row[1]), []).append((row[2].encode(), parse_ids(row[3])))
    for (byte_spec, row_spec), cases in by_table.items():
        table = bpe.build_table_vocab(*parse_vocab(byte_spec, row_spec))
        ids, out_off = gpu_encode(table, *to_batch([c[0] for c in cases]))
        for i, (text, want) in enumerate(cases):
            assert ids[out_off[i]:out_off[i + 1]].tolist() == want, (byte_spec, row_spec, text)
        table.free()


def test_random_vocabularies(bpe):
    """Random tables under a random renaming of the tokens, against the oracle built over the same vocabulary."""
    rng = random.Random(4321)
    for trial in range(12):
        alphabet = rng.sample(range(256), rng.randint(2, 6))
        rows = random_monotone_table(rng, rng.randint(1, 60), alphabet)
        phi = np.array(rng.sample(range(4 * (256 + len(rows))), 256 + len(rows)), dtype=np.int32)
        named = [(int(phi[a]), int(phi[b])) for a, b in rows]
        orc = oracle.Table(named, phi[:256], phi[256:])
        table = bpe.build_table_vocab(phi[:256], named, phi[256:])
        strings = [bytes(rng.choice(alphabet) for _ in range(rng.choice([0, 1, 2, 5, 64, 65, 300, 1100, 2500])))
                   for _ in range(40)]
        data, off = to_batch(strings)
        ids, out_off = gpu_encode(table, data, off)
        want_ids, want_off = orc.encode_batch(data, off, tier=oracle.TEXTBOOK, nthreads=8)
        assert_same_encoding(ids, out_off, want_ids, want_off, f"vocabulary trial {trial}")
        table.free()


def parse_specials(spec):
    return {k.encode(): int(v) for k, v in (item.split("=") for item in spec.split(";"))}


def test_hand_worked_special_examples(bpe):
    by_table = {}
    for row in read_golden("hand_worked_specials.txt"):
        by_table.setdefault((row[0], row[1]), []).append((row[2].encode(), parse_ids(row[3])))
    for (spec, specials), cases in by_table.items():
        table = bpe.build_table(parse_rows(spec))
        table.set_specials(parse_specials(specials))
        ids, out_off = gpu_encode(table, *to_batch([c[0] for c in cases]))
        for i, (text, want) in enumerate(cases):
            assert ids[out_off[i]:out_off[i + 1]].tolist() == want, (spec, specials, text)
        table.free()


def test_special_sets_that_could_overlap_are_rejected(bpe):
    table = bpe.build_table([(97, 98)])
    for bad in ({b"aa": 1}, {b"<a>": 1, b"a": 2}, {b"<a>": 1, b"a><": 2}, {b"ab": 1, b"bc": 2}, {b"": 1},
                {b"x" * 65: 1}, {b"<a>": -4}):
        with pytest.raises(bpe.BpeError):
            table.set_specials(bad)
    table.set_specials({b"<a>": 1, b"<a>b": 2, b"[x]": 3})      # a special may begin a longer one
    ids, _ = gpu_encode(table, *to_batch([b"ab<a>b[x]<a>"]))
    assert ids.tolist() == [256, 2, 3, 1]
    table.set_specials({})
    ids, _ = gpu_encode(table, *to_batch([b"ab<a>"]))
    assert ids.tolist() == [256, 60, 97, 62]
    table.free()


def test_random_texts_with_special_tokens(bpe):
    """Specials sprinkled over random strings of every kernel variant's size, default and vocabulary ids."""
    rng = random.Random(99)
    specials = {b"<|endoftext|>": 70001, b"<|endoftext|>2": 70002, b"[SEP]": 70003, b"\x00": 70004,
                b"<" + b"q" * 62 + b">": 70005}
    for trial in range(6):
        alphabet = [ord(c) for c in "ab|<>e "] + rng.sample(range(128, 256), 2)
        rows = random_monotone_table(rng, rng.randint(5, 200), alphabet)
        if trial % 2:
            phi = np.array(rng.sample(range(60000), 256 + len(rows)), dtype=np.int32)
            named = [(int(phi[a]), int(phi[b])) for a, b in rows]
            orc = oracle.Table(named, phi[:256], phi[256:])
            table = bpe.build_table_vocab(phi[:256], named, phi[256:])
        else:
            orc = oracle.Table(rows)
            table = bpe.build_table(rows)
        orc.set_specials(specials)
        table.set_specials(specials)
        strings = []
        for n in (0, 1, 13, 14, 64, 200, 1000, 1024, 1500, 5000, 20000, 65536):
            s = bytearray()
            while len(s) < n:
                if rng.random() < 0.15:
                    s += rng.choice(list(specials))
                else:
                    s += bytes(rng.choice(alphabet) for _ in range(rng.choice((1, 3, 20, 150))))
            strings.append(bytes(s[:n]))
        strings += list(specials) + [b"".join(specials) * 3]
        data, off = to_batch(strings)
        ids, out_off = gpu_encode(table, data, off)
        want_ids, want_off = orc.encode_batch(data, off, tier=oracle.HEAP, nthreads=8)
        assert_same_encoding(ids, out_off, want_ids, want_off, f"specials trial {trial}")
        table.free()


def test_encode_strings_convenience(bpe):
    """Host strings in, one id array per string out: str and bytes, empty strings, a string above 1 KiB."""
    merges = workloads.load_merges("1k")
    table = bpe.build_table(merges)
    orc = oracle.Table(merges)
    text = workloads.text(1, 77, 3000).tobytes()
    strings = ["the quick brown fox", b"", text[:10], text[10:1500], "", text[1500:]]
    got = bpe.encode_strings(table, strings)
    assert len(got) == len(strings)
    for s, ids in zip(strings, got):
        raw = s.encode() if isinstance(s, str) else s
        assert ids.tolist() == orc.encode(raw, oracle.TEXTBOOK).tolist()
    assert bpe.encode_strings(table, []) == []
    table.free()

