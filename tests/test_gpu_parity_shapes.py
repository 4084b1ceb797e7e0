"""GPU parity on batch shapes and table structures chosen to sit on the boundaries between the launch paths:
batch sizes around the resident grid and the fused scan/pack limit, string lengths around the piece target,
tables without any segment cut (nothing can be split, every kernel variant is used) and tables where every
bigram is a cut, and very many very short strings.  All against the CPU oracle, bit for bit."""
import random

import numpy as np
import pytest

import oracle
import workloads
from gpu_util import assert_same_encoding, gpu_encode, to_batch

pytestmark = pytest.mark.gpu

THREADS = 16


@pytest.fixture(scope="module")
def bpe():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_11941_amd as bpe

    bpe.load_library()
    return bpe


def check(bpe, rows, data, off, what, tier=oracle.HEAP):
    table = bpe.build_table(rows)
    orc = oracle.Table(rows)
    ids, out_off = gpu_encode(table, data, off)
    want_ids, want_off = orc.encode_batch(data, off, tier=tier, nthreads=THREADS)
    assert_same_encoding(ids, out_off, want_ids, want_off, what)
    table.free()


@pytest.mark.parametrize("batch", [1, 2, 63, 3071, 3072, 3073, 4095, 4096, 4097, 9000])
def test_batch_sizes_around_the_launch_path_limits(bpe, batch):
    merges = workloads.load_merges("32k")
    text = workloads.text(2, 500 + batch, 200 * batch)
    rng = np.random.default_rng(batch)
    lens = rng.integers(0, 400, size=batch)
    lens = (lens * (200 * batch / max(int(lens.sum()), 1))).astype(np.int64)
    off = np.zeros(batch + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    check(bpe, merges, text[: int(off[-1])], off, f"batch {batch}")


def test_lengths_around_the_piece_target(bpe):
    merges = workloads.load_merges("100k")
    lens = [767, 768, 769, 895, 896, 897, 1023, 1024, 1025, 1151, 1152, 1153, 1791, 1792, 1793, 2047, 2048, 2049,
            2687, 2688, 2689, 8960, 8961]
    off = np.zeros(len(lens) + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    check(bpe, merges, workloads.text(3, 31, int(off[-1])), off, "piece target", tier=oracle.TEXTBOOK)
    # the same lengths as one-string batches (max_len then equals the string)
    data = workloads.text(3, 32, max(lens))
    for n in lens:
        check(bpe, merges, data[:n], np.array([0, n], dtype=np.int64), f"single string of {n}", tier=oracle.TEXTBOOK)


def random_monotone_table(rng, n_rows, alphabet, first_rows=()):
    rows = list(first_rows)
    seen = set(rows)
    while len(rows) < n_rows:
        pool = list(alphabet) + [256 + r for r in range(len(rows))]
        p = (rng.choice(pool), rng.choice(pool))
        if p not in seen:
            seen.add(p)
            rows.append(p)
    return rows


def test_table_without_cuts_uses_every_variant(bpe):
    """Two letters whose four bigrams are all rows: no cut anywhere, so no string can be split into pieces and
    the four-wave, sixteen-wave and staged variants all run, with whole-string horizons."""
    rng = random.Random(8)
    a, b = ord("a"), ord("b")
    rows = random_monotone_table(rng, 300, [a, b], first_rows=[(a, a), (a, b), (b, a), (b, b)])
    lens = [0, 1, 2, 65, 1000, 1024, 1025, 3000, 4096, 4097, 9000, 16384, 16385, 40000, 65536]
    strings = [bytes(rng.choice((a, b)) for _ in range(n)) for n in lens]
    data, off = to_batch(strings)
    check(bpe, rows, data, off, "no cuts")


def test_partly_cut_strings_leave_void_slots(bpe):
    """Long stretches without a cut between stretches full of them: slots whose window holds no cut are void
    and the piece before them runs on, into the bigger variants."""
    rng = random.Random(9)
    a, b, c = ord("a"), ord("b"), ord("c")
    rows = random_monotone_table(rng, 120, [a, b], first_rows=[(a, a), (a, b), (b, a), (b, b)])
    # 'c' is in no row: every bigram with it is a cut
    strings = []
    for n in (1500, 5000, 20000, 65536):
        s = bytearray()
        while len(s) < n:
            if rng.random() < 0.5:
                s += bytes(rng.choice((a, b)) for _ in range(rng.choice((30, 200, 900, 2500))))
            else:
                s += bytes(rng.choice((a, b, c)) for _ in range(rng.choice((5, 100, 1000))))
        strings.append(bytes(s[:n]))
    data, off = to_batch(strings)
    check(bpe, rows, data, off, "void slots")


def test_the_only_cut_at_every_distance_before_a_piece_boundary(bpe):
    """Runs of 'a' under a doubling table (no cut inside a run) with a single 'b' -- the only place to cut --
    placed so that the last cut before the piece boundary at byte 896 lies d bytes before it, for every d the
    search window covers and a few beyond (then the slot is void and the piece runs on into a bigger variant)."""
    a, b = ord("a"), ord("b")
    rows = [(a, a)] + [(255 + j, 255 + j) for j in range(1, 10)]
    strings = []
    for d in list(range(0, 130)) + [200, 500]:
        s = bytearray(b"a" * 1900)
        s[896 - d - 1] = b                              # cuts before this byte and after it: the later one wins
        strings.append(bytes(s))
    strings.append(b"a" * 1900)                         # no cut at all
    data, off = to_batch(strings)
    check(bpe, rows, data, off, "cut distances", tier=oracle.TEXTBOOK)


def test_table_where_every_bigram_is_a_cut(bpe):
    data, off = workloads.batch(3, batch_override=64)
    check(bpe, np.zeros((0, 2), dtype=np.int32), data, off, "empty table")
    # one row only: everything except "ab" is a cut
    check(bpe, [(ord("a"), ord("b"))], data, off, "one row")


def test_very_many_very_short_strings(bpe):
    merges = workloads.load_merges("1k")
    text = workloads.text(1, 3, 200000)
    for n_strings, length in ((65536, 1), (100000, 0), (50000, 3)):
        off = np.arange(n_strings + 1, dtype=np.int64) * length
        check(bpe, merges, text[: int(off[-1])], off, f"{n_strings} strings of {length}")


def test_two_streams_and_graph_replay(bpe):
    """bpe_encode_batch only enqueues: two calls on two streams with their own workspaces do not disturb each
    other, and a call captured into a HIP graph gives the eager result on every replay, also after the input
    buffer's contents have changed."""
    import torch

    merges = workloads.load_merges("32k")
    table = bpe.build_table(merges)
    orc = oracle.Table(merges)
    dev = torch.device("cuda:0")
    batches = [workloads.batch(2, batch_override=700), workloads.batch(3, batch_override=40)]
    wants = [orc.encode_batch(d, o, tier=oracle.HEAP, nthreads=THREADS) for d, o in batches]
    streams = [torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)]
    outs = []
    for (data, off), stream in zip(batches, streams):
        d, o = torch.from_numpy(data).to(dev), torch.from_numpy(off).to(dev)
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            for _ in range(3):
                ids, out_off = bpe.encode_batch(table, d, o, int(np.diff(off).max()), stream=stream)
        outs.append((ids, out_off))
    torch.cuda.synchronize()
    for (ids, out_off), (want_ids, want_off) in zip(outs, wants):
        out_off = out_off.cpu().numpy()
        assert_same_encoding(ids[: int(out_off[-1])].cpu().numpy(), out_off, want_ids, want_off, "two streams")

    # graph capture of one call, replayed over changing inputs of the same shape
    data, off = batches[0]
    lens_max = int(np.diff(off).max())
    d, o = torch.from_numpy(data).to(dev), torch.from_numpy(off).to(dev)
    out_ids = torch.empty(len(data), dtype=torch.int32, device=dev)
    out_off = torch.empty(len(off), dtype=torch.int64, device=dev)
    ws = torch.empty(bpe.workspace_bytes(len(off) - 1, len(data), lens_max), dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream(device=dev)
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        bpe.encode_batch(table, d, o, lens_max, out_ids, out_off, ws, stream=torch.cuda.current_stream(dev))
    rng = np.random.default_rng(5)
    for replay in range(4):
        if replay:                                        # same offsets, other bytes
            data = workloads.text(2, 900 + replay, len(data))
            d.copy_(torch.from_numpy(data).to(dev))
        out_ids.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want_ids, want_off = orc.encode_batch(data, off, tier=oracle.HEAP, nthreads=THREADS)
        got_off = out_off.cpu().numpy()
        assert_same_encoding(out_ids[: int(got_off[-1])].cpu().numpy(), got_off, want_ids, want_off,
                             f"graph replay {replay}")
    table.free()
