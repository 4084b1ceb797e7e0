"""Section 5.2's similarity between this library's byte-level encoding (GPU) and a regex-pretokenised BPE over the
same table (`tokenizers`), on the synthetic texts of the benchmark configurations.  Table 1's datasets and model
are not available here, so its figures are not reproduced ("parity unpinned" for them); what is pinned is the
metric itself (tests/test_quality.py) and, here, that with the regex switched off the library's BPE and the GPU
agree token for token."""
import numpy as np
import pytest

import workloads
from gpu_util import gpu_encode, to_batch
from paper_2507_11941_amd import quality

tokenizers = pytest.importorskip("tokenizers")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bpe():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_11941_amd as bpe

    bpe.load_library()
    return bpe


@pytest.mark.parametrize("cfg,count", [(1, 64), (2, 512), (3, 256), (5, 600)])
def test_similarity_to_regex_pretokenised_bpe(bpe, cfg, count):
    c = workloads.CONFIGS[cfg]
    merges = workloads.load_merges(c.table)
    data, off = workloads.batch(cfg, batch_override=count)
    strings = [quality.whole_characters(data[off[i]:off[i + 1]].tobytes()) for i in range(count)]
    strings = [s for s in strings if len(s) <= 16384]                 # (keeps the distance computation short)
    table = bpe.build_table(merges)
    ids, out_off = gpu_encode(table, *to_batch(strings))
    ours = [ids[out_off[i]:out_off[i + 1]] for i in range(len(strings))]
    lengths = [len(s) for s in strings]

    plain = quality.reference_ids(quality.regex_reference(merges, use_regex=False), strings)
    for i, (a, b) in enumerate(zip(plain, ours)):
        assert np.array_equal(a, b), f"string {i}: the library's BPE without pre-tokenisation differs from the GPU"
    assert quality.similarity(plain, ours, lengths) == 1.0

    sim = quality.similarity(quality.reference_ids(quality.regex_reference(merges, use_regex=True), strings), ours,
                             lengths)
    print(f"config {cfg} ({c.name}): similarity to regex-pretokenised BPE over the same table = {sim:.4f} "
          f"on {len(strings)} strings")
    assert 0.5 < sim <= 1.0
    table.free()
