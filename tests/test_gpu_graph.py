"""bpe_encode_batch captured in a HIP graph: the call only enqueues kernels (no allocation, no synchronisation,
no memset nodes -- the kernels clear their own counters), so a caller may capture it once and replay it on new
input of the same sizes.  Every replay is compared with the oracle; between replays the test changes the input
and does eager work and synchronisations of its own."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kind", ["direct", "split"])
def test_replays_of_a_captured_call_match_the_oracle(kind):
    import torch

    import paper_2507_11941_amd as bpe

    dev = torch.device("cuda:0")
    merges = workloads.load_merges("32k")
    table = bpe.build_table(merges)
    orc = oracle.Table(merges)
    if kind == "direct":                                 # one workgroup per string, two launches
        batch, length = 96, 1024
    else:                                                # strings cut into pieces, work lists, tiled scan
        batch, length = 64, 6000
    total = batch * length
    offsets = np.arange(batch + 1, dtype=np.int64) * length
    inputs = [workloads.text(2, 100 + r, total) for r in range(4)]

    d = torch.zeros(total, dtype=torch.uint8, device=dev)
    o = torch.from_numpy(offsets).to(dev)
    ids = torch.zeros(total, dtype=torch.int32, device=dev)
    off = torch.zeros(batch + 1, dtype=torch.int64, device=dev)
    ws = torch.empty(bpe.workspace_bytes(batch, total, length), dtype=torch.uint8, device=dev)

    # an eager call first: one-time set-up of the library (kernel attributes) must not fall into the capture
    d.copy_(torch.from_numpy(inputs[0]))
    bpe.encode_batch(table, d, o, length, out_ids=ids, out_offsets=off, workspace=ws)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        bpe.encode_batch(table, d, o, length, out_ids=ids, out_offsets=off, workspace=ws)
    torch.cuda.synchronize()

    for r in (1, 2, 3, 1):
        d.copy_(torch.from_numpy(inputs[r]))
        ids.fill_(-1)                                    # eager work between the replays
        off.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want_ids, want_off = orc.encode_batch(inputs[r], offsets, tier=oracle.HEAP)
        got_off = off.cpu().numpy()
        assert np.array_equal(got_off, want_off), (kind, r)
        assert np.array_equal(ids[: int(got_off[-1])].cpu().numpy(), want_ids), (kind, r)
