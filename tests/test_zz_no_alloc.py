"""bpe_encode_batch_static (the entry point that allocates nothing and keeps its scratch in the library's own
device array) against bpe_encode_batch, through the C ABI: two calls in a row on the shared scratch, the second
on a smaller input, then a ragged batch; and the size limits."""
import ctypes

import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu


def encode_both(lib, table, data, offsets):
    """(ids, offsets) from bpe_encode_batch and from bpe_encode_batch_static, both called through ctypes."""
    import torch

    import paper_2507_11941_amd as bpe

    dev = torch.device("cuda:0")
    batch, total = len(offsets) - 1, len(data)
    max_len = int(np.diff(offsets).max()) if batch else 0
    d = torch.from_numpy(data).to(dev) if total else torch.empty(0, dtype=torch.uint8, device=dev)
    o = torch.from_numpy(offsets).to(dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    results = []
    for static in (False, True):
        ids = torch.full((max(total, 1),), -1, dtype=torch.int32, device=dev)
        off = torch.full((batch + 1,), -1, dtype=torch.int64, device=dev)
        if static:
            code = lib.bpe_encode_batch_static(table.handle, d.data_ptr(), o.data_ptr(), batch, total, max_len,
                                               ids.data_ptr(), off.data_ptr(), stream)
        else:
            ws = torch.empty(bpe.workspace_bytes(batch, total, max_len), dtype=torch.uint8, device=dev)
            code = lib.bpe_encode_batch(table.handle, d.data_ptr(), o.data_ptr(), batch, total, max_len,
                                        ids.data_ptr(), off.data_ptr(), ws.data_ptr(), ws.numel(), stream)
        assert code == 0, (static, code)
        torch.cuda.synchronize()
        off_h = off.cpu().numpy()
        results.append((ids[: int(off_h[-1])].cpu().numpy(), off_h))
    return results


def test_static_entry_point_matches_the_workspace_one():
    import paper_2507_11941_amd as bpe

    lib = bpe.load_library()
    table = bpe.build_table(workloads.load_merges("100k"))
    # 1: 600 strings x 4 KiB, cut into pieces (2.4 MiB); 2: right after it, 100 strings x 1 KiB (one workgroup
    # per string); 3: ragged lengths with empty strings, up to 16 KiB
    first = workloads.batch(3, batch_override=600)
    second = workloads.batch(2, batch_override=100)
    rng = np.random.default_rng(7)
    lens = rng.integers(0, 3000, size=500)
    lens[::50] = 0
    lens[3] = 16384
    off3 = np.zeros(len(lens) + 1, dtype=np.int64)
    np.cumsum(lens, out=off3[1:])
    third = (workloads.text(3, 11, int(off3[-1])), off3)
    for name, (data, offsets) in (("4 KiB strings", first), ("smaller, 1 KiB strings", second), ("ragged", third)):
        (want_ids, want_off), (got_ids, got_off) = encode_both(lib, table, data, offsets)
        assert want_off[-1] > 0, name
        assert np.array_equal(got_off, want_off), name
        assert np.array_equal(got_ids, want_ids), name


def test_static_entry_point_rejects_what_exceeds_its_scratch():
    import torch

    import paper_2507_11941_amd as bpe

    lib = bpe.load_library()
    table = bpe.build_table(workloads.load_merges("1k"))
    dev = torch.device("cuda:0")
    d = torch.zeros(64, dtype=torch.uint8, device=dev)
    o = torch.zeros(2, dtype=torch.int64, device=dev)
    ids = torch.zeros(64, dtype=torch.int32, device=dev)
    off = torch.zeros(2, dtype=torch.int64, device=dev)
    args = (d.data_ptr(), o.data_ptr())
    outs = (ids.data_ptr(), off.data_ptr(), None)
    too_big = -6
    assert lib.bpe_encode_batch_static(table.handle, *args, 4097, 64, 64, *outs) == too_big
    assert lib.bpe_encode_batch_static(table.handle, *args, 1, (4 << 20) + 1, 64, *outs) == too_big
    assert lib.bpe_encode_batch_static(table.handle, *args, 1, 64, 16385, *outs) == too_big
    assert lib.bpe_encode_batch_static(None, *args, 1, 64, 64, *outs) == -1
    assert lib.bpe_encode_batch_static(table.handle, *args, 1, 64, 64, None, off.data_ptr(), None) == -1
    torch.cuda.synchronize()
