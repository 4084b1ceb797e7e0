"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py times:
the HIP path (through the C ABI) against the CPU oracle, bit for bit.

The whole batch is compared with the oracle's heap encoder (admitted by agreeing with Algorithm 1 in the
CPU tests) and a spread of strings -- always including the longest -- with the textbook one-merge-at-a-time
encoder.  Round trip and fixed-point properties are checked on the GPU output directly."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import assert_same_encoding, gpu_encode, to_batch

pytestmark = pytest.mark.gpu

ORACLE_THREADS = 16


@pytest.fixture(scope="module")
def bpe():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_11941_amd as bpe

    bpe.load_library()
    return bpe


_tables = {}


def tables(bpe, key):
    if key not in _tables:
        merges = workloads.load_merges(key)
        _tables[key] = (bpe.build_table(merges), oracle.Table(merges), merges)
    return _tables[key]


def check_properties(merges, orc, data, off, ids, out_off, picks):
    keys = set(map(tuple, merges.tolist()))
    for i in picks:
        s = data[off[i]:off[i + 1]].tobytes()
        t = ids[out_off[i]:out_off[i + 1]]
        assert orc.decode(t) == s, f"round trip of string {i}"
        assert not any((int(a), int(b)) in keys for a, b in zip(t[:-1], t[1:])), f"string {i} is not a fixed point"
        assert len(t) <= len(s)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_config_full_size(bpe, cfg):
    c = workloads.CONFIGS[cfg]
    table, orc, merges = tables(bpe, c.table)
    data, off = workloads.batch(cfg)
    b = len(off) - 1
    print(f"config {cfg}: {b} strings, {len(data)} bytes", flush=True)
    ids, out_off = gpu_encode(table, data, off)
    want_ids, want_off = orc.encode_batch(data, off, tier=oracle.HEAP, nthreads=ORACLE_THREADS)
    assert_same_encoding(ids, out_off, want_ids, want_off, f"config {cfg} vs heap oracle")
    # a spread of strings, and the longest, against the textbook encoder
    lens = np.diff(off)
    picks = sorted(set(np.linspace(0, b - 1, 24).astype(int).tolist() + [int(np.argmax(lens)), int(np.argmin(lens))]))
    sub, sub_off = to_batch([data[off[i]:off[i + 1]].tobytes() for i in picks])
    t_ids, t_off = orc.encode_batch(sub, sub_off, tier=oracle.TEXTBOOK, nthreads=ORACLE_THREADS)
    for j, i in enumerate(picks):
        assert np.array_equal(ids[out_off[i]:out_off[i + 1]], t_ids[t_off[j]:t_off[j + 1]]), f"string {i} vs textbook"
    check_properties(merges, orc, data, off, ids, out_off, picks[:8])
    assert ids.max() < 256 + len(merges)


@pytest.mark.parametrize("cfg", [2, 3])
def test_config_under_a_vocabulary(bpe, cfg):
    """The same batches with the tokens renamed by a random injection (a vocabulary's own ids): all three
    packing paths write vocabulary ids, compared with the oracle built over that vocabulary."""
    c = workloads.CONFIGS[cfg]
    merges = workloads.load_merges(c.table)
    rng = np.random.default_rng(2024 + cfg)
    phi = rng.permutation(3 * (256 + len(merges)))[: 256 + len(merges)].astype(np.int32)
    named = phi[merges]
    table = bpe.build_table_vocab(phi[:256], named, phi[256:])
    orc = oracle.Table(named, phi[:256], phi[256:])
    data, off = workloads.batch(cfg)
    ids, out_off = gpu_encode(table, data, off)
    want_ids, want_off = orc.encode_batch(data, off, tier=oracle.HEAP, nthreads=ORACLE_THREADS)
    assert_same_encoding(ids, out_off, want_ids, want_off, f"config {cfg} under a vocabulary")
    # a batch above 4096 strings of at most 1 KiB takes the third packing path
    if cfg == 2:
        many, many_off = workloads.batch(cfg, batch_override=5000)
        ids, out_off = gpu_encode(table, many, many_off)
        want_ids, want_off = orc.encode_batch(many, many_off, tier=oracle.HEAP, nthreads=ORACLE_THREADS)
        assert_same_encoding(ids, out_off, want_ids, want_off, "5000 strings under a vocabulary")
    table.free()


def test_ragged_lengths_and_unaligned_starts(bpe):
    """Lengths 0..~70 around every kernel-variant boundary, cut from one text stream so starts are unaligned."""
    table, orc, _ = tables(bpe, "100k")
    rng = np.random.default_rng(11)
    lens = [0, 1, 2, 3, 63, 64, 65, 127, 129, 1023, 1024, 1025, 4095, 4096, 4097, 16383, 16384, 16385,
            65535, 65536, 33333, 7, 0, 5000, 999, 20000]
    lens += rng.integers(0, 3000, size=200).tolist()
    off = np.zeros(len(lens) + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    data = workloads.text(3, 77, int(off[-1]))
    ids, out_off = gpu_encode(table, data, off)
    want_ids, want_off = orc.encode_batch(data, off, tier=oracle.TEXTBOOK, nthreads=ORACLE_THREADS)
    assert_same_encoding(ids, out_off, want_ids, want_off, "ragged")


def test_batch_order_and_repeat_determinism(bpe):
    """A string's encoding does not depend on its neighbours, its position, or the run."""
    table, orc, _ = tables(bpe, "32k")
    data, off = workloads.batch(2, batch_override=300)
    ids, out_off = gpu_encode(table, data, off)
    ids2, out_off2 = gpu_encode(table, data, off)
    assert np.array_equal(ids, ids2) and np.array_equal(out_off, out_off2)
    perm = np.random.default_rng(3).permutation(300)
    strings = [data[off[i]:off[i + 1]].tobytes() for i in perm]
    p_ids, p_off = gpu_encode(table, *to_batch(strings))
    for j, i in enumerate(perm):
        assert np.array_equal(p_ids[p_off[j]:p_off[j + 1]], ids[out_off[i]:out_off[i + 1]])


def test_adversarial_runs_with_doubling_table(bpe):
    """Long single-byte runs under a table that keeps doubling them: deep chains of self-pair passes."""
    rows = []
    for byte in (ord("a"), ord("0"), ord(" ")):
        prev = byte
        for _ in range(12):
            rows.append((prev, prev))
            prev = 256 + len(rows) - 1
    rows += [(ord("a"), ord("b")), (ord("b"), ord("a"))]
    table = bpe.build_table(rows)
    orc = oracle.Table(rows)
    data, off = workloads.batch(4, batch_override=24)
    ids, out_off = gpu_encode(table, data, off)
    want_ids, want_off = orc.encode_batch(data, off, tier=oracle.TEXTBOOK, nthreads=ORACLE_THREADS)
    assert_same_encoding(ids, out_off, want_ids, want_off, "doubling table on adversarial strings")
