"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI and fetch the result."""
from __future__ import annotations

import numpy as np


def to_batch(strings):
    """list of bytes -> (uint8 array, int64 offsets)."""
    data = np.frombuffer(b"".join(strings), dtype=np.uint8).copy()
    offsets = np.zeros(len(strings) + 1, dtype=np.int64)
    np.cumsum([len(s) for s in strings], out=offsets[1:])
    return data, offsets


def gpu_encode(table, data, offsets, max_len=None):
    """Encode on cuda:0 via bpe_encode_batch; returns (ids int32[total], out_offsets int64[B+1]) on the host."""
    import torch

    import paper_2507_11941_amd as bpe

    data = np.ascontiguousarray(data, dtype=np.uint8)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    if max_len is None:
        max_len = int(np.diff(offsets).max()) if len(offsets) > 1 else 0
    dev = torch.device("cuda:0")
    d = torch.from_numpy(data).to(dev) if len(data) else torch.empty(0, dtype=torch.uint8, device=dev)
    o = torch.from_numpy(offsets).to(dev)
    ids, out_off = bpe.encode_batch(table, d, o, max_len)
    torch.cuda.synchronize()
    out_off = out_off.cpu().numpy()
    ids = ids[: int(out_off[-1])].cpu().numpy()
    return ids, out_off


def assert_same_encoding(got_ids, got_off, want_ids, want_off, what=""):
    """Element-by-element comparison of two dense encodings, reporting the first string that differs."""
    assert got_off[0] == 0
    if not np.array_equal(got_off, want_off):
        bad = int(np.flatnonzero(got_off != want_off)[0]) - 1
        raise AssertionError(f"{what}: token count of string {bad} differs: "
                             f"got {got_off[bad + 1] - got_off[bad]}, want {want_off[bad + 1] - want_off[bad]}")
    if not np.array_equal(got_ids, want_ids):
        pos = int(np.flatnonzero(got_ids != want_ids)[0])
        s = int(np.searchsorted(want_off, pos, side="right")) - 1
        raise AssertionError(f"{what}: string {s} differs at token {pos - want_off[s]}: "
                             f"got {got_ids[pos]}, want {want_ids[pos]}")
