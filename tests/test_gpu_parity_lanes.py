"""GPU parity on the boundaries of the lane-per-segment kernel: segments of exactly the 32 bytes a lane can take
and of one byte more (which send the item to the wave-per-item kernel), items of exactly 1 KiB, items that are all
two-byte segments (the longest possible segment list) or all one-byte segments (an empty list), and the three
launch paths: one workgroup per string, listed strings, pieces of long strings.  All against the CPU oracle."""
import numpy as np
import pytest

import oracle
from gpu_util import assert_same_encoding, gpu_encode, to_batch

pytestmark = pytest.mark.gpu

THREADS = 16

# 'a' doubles five times (aa, aaaa, ... 32 a's); 'b' 'c' merge; every other bigram, and so every bigram with
# 'x', is a cut.  "a" * n is one segment of n bytes, "bc" * k is k segments of two bytes.
CHAIN = [(97, 97)] + [(255 + j, 255 + j) for j in range(1, 5)] + [(98, 99)]


@pytest.fixture(scope="module")
def bpe():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_11941_amd as bpe

    bpe.load_library()
    return bpe


def check(bpe, rows, strings, what):
    data, off = to_batch(strings)
    table, orc = bpe.build_table(rows), oracle.Table(rows)
    ids, out_off = gpu_encode(table, data, off)
    want_ids, want_off = orc.encode_batch(data, off, tier=oracle.HEAP, nthreads=THREADS)
    assert_same_encoding(ids, out_off, want_ids, want_off, what)
    table.free()
    return ids, out_off


def run_of(n):
    return b"a" * n


def test_segment_lengths_around_what_a_lane_takes(bpe):
    """One workgroup per string: runs of 1..70 'a' between cuts; 32 is the last length a lane takes itself."""
    strings = [b"x" + run_of(n) + b"x" + b"bc" * 3 + b"x" + run_of(n) for n in range(1, 71)]
    ids, off = check(bpe, CHAIN, strings, "runs of 1..70")
    # closed form for the run of 32: one token of level 5 (id 260); of 33: that token and a single 'a'
    s32 = ids[off[31]:off[32]].tolist()
    assert s32 == [120, 260, 120, 261, 261, 261, 120, 260]
    s33 = ids[off[32]:off[33]].tolist()
    assert s33 == [120, 260, 97, 120, 261, 261, 261, 120, 260, 97]


@pytest.mark.parametrize("batch", [1, 700, 5000])
def test_items_of_exactly_one_kib(bpe, batch):
    """1,024-byte strings in the three shapes a list can take: all two-byte segments (512 of them), all one-byte
    segments (none listed), 32-byte runs back to back with cuts between them; one workgroup per string (small
    batches) and listed strings (more strings than resident workgroups)."""
    shapes = [b"bc" * 512, b"x" * 1024, (run_of(31) + b"x") * 32, (run_of(32) + b"x") * 31 + b"x",
              b"bc" * 300 + run_of(33) + b"x" * 391, run_of(1024)]
    strings = [shapes[i % len(shapes)] for i in range(batch)]
    check(bpe, CHAIN, strings, f"1 KiB items, batch {batch}")


def test_pieces_of_long_strings_with_and_without_long_segments(bpe):
    """Strings above 1 KiB are cut into pieces: pieces whose segments all fit a lane, pieces that hold one run of
    33..900 bytes (handed on to the wave-per-item kernel through the list), and a string without any cut."""
    rng = np.random.default_rng(5)
    strings = []
    for i in range(300):
        parts = []
        while sum(map(len, parts)) < 3000 + 10 * i:
            kind = rng.integers(0, 4)
            if kind == 0:
                parts.append(b"bc" * int(rng.integers(1, 40)) + b"x")
            elif kind == 1:
                parts.append(run_of(int(rng.integers(1, 33))) + b"x")
            elif kind == 2 and i % 3 == 0:
                parts.append(run_of(int(rng.integers(33, 900))) + b"x")
            else:
                parts.append(b"x" * int(rng.integers(1, 9)))
        strings.append(b"".join(parts))
    strings.append(run_of(5000))
    strings.append(b"")
    check(bpe, CHAIN, strings, "pieces")
