"""The rules the GPU kernels use instead of Algorithm 1's one-merge-at-a-time loop, as a plain Python model,
checked against the oracle (and so against Algorithm 1) on random tables whose rows only use older tokens and on
the stored trained tables.  The model shares no code with the oracle or the kernels; it takes the horizon codes
from the host image of the table the library builds, so that the codes the kernels see are the ones modelled.

Three rules:
  cuts      a byte bigram that lies at no row's junction (last byte of the left operand, first byte of the right
            operand) can never be merged across: the string falls into segments that are encoded on their own.
            This is what lets long strings be cut into pieces and what the lane-per-segment kernel relies on.
  lanes     inside a segment: positions never move, a merge keeps the merged token at the left position and kills
            the right one, pair values are cached per position and only the two pairs next to a merge are looked
            up again; the next merge is the lowest value, left-most on ties (value and position in one key).
  fusion    (wave-per-item kernels) per segment, all pairs whose rank lies below the horizon E = min limit(pair)
            are settled in one pass: along a run of adjacent candidates whose ranks do not decrease the applied
            ones alternate from the run's head, and a candidate whose right neighbour has a strictly lower rank
            waits for the next pass.
"""
import random

import numpy as np
import pytest

import oracle
import paper_2507_11941_amd as bpe
import workloads

INF = 1 << 40
NO_RANK, CUT = 0xFFFFFFFF, 0xFFFFFFFD
HORIZON_SHIFT, SLOTS = 2, 2


def random_monotone_table(rng, n_rows, alphabet):
    rows, seen = [], set()
    while len(rows) < n_rows:
        pool = list(alphabet) + [256 + r for r in range(len(rows))]
        p = (rng.choice(pool), rng.choice(pool))
        if p not in seen:
            seen.add(p)
            rows.append(p)
    return rows


def horizon_decode(code):
    e, m = code >> 4, code & 15
    return ((16 | m) << (e - 1)) if e else m


class Model:
    """What the kernels know about a table: rank of a pair, limit of a row (from the image's horizon codes),
    and which byte bigrams are cuts (from the image's byte-pair table)."""

    def __init__(self, merges):
        self.rows = [tuple(map(int, r)) for r in merges]
        self.rank = {p: r for r, p in enumerate(self.rows)}
        words, log2 = bpe.table_image(self.rows)
        n_bucket_words = (1 << log2) * 2 * SLOTS
        self.byte_pair = words[n_bucket_words + 256:]
        # value of every row, found by scanning the occupied slots (tag != empty): rank -> horizon code
        slots = words[:n_bucket_words].reshape(-1, 2)
        occupied = slots[slots[:, 1] != NO_RANK]
        code = {int(v) >> 12: (int(v) >> HORIZON_SHIFT) & 0xFF for v in occupied[:, 0]}
        assert len(code) == len(self.rows)
        self.limit = [INF if code[r] == 255 else r + 1 + horizon_decode(code[r]) for r in range(len(self.rows))]

    def segments(self, data: bytes):
        out, start = [], 0
        for i in range(len(data) - 1):
            if int(self.byte_pair[data[i] << 8 | data[i + 1]]) == CUT:
                out.append(data[start:i + 1])
                start = i + 1
        out.append(data[start:])
        return out

    # -- lane-per-segment rule --
    def encode_segment_lane(self, seg: bytes):
        n = len(seg)
        tok = list(seg)
        live = [True] * n
        val = [self.rank.get((seg[i], seg[i + 1]), INF) if i + 1 < n else INF for i in range(n)]
        while True:
            r, k = min(((val[i], i) for i in range(n) if live[i]), default=(INF, 0))   # lowest value, left-most
            if r == INF:
                break
            right = next(i for i in range(k + 1, n) if live[i])
            tok[k] = 256 + r
            live[right] = False
            val[right] = INF
            after = next((i for i in range(right + 1, n) if live[i]), None)
            left = next((i for i in range(k - 1, -1, -1) if live[i]), None)
            val[k] = self.rank.get((tok[k], tok[after]), INF) if after is not None else INF
            if left is not None:
                val[left] = self.rank.get((tok[left], tok[k]), INF)
        return [tok[i] for i in range(n) if live[i]]

    # -- fused passes with a horizon --
    def encode_segment_fused(self, seg: bytes, passes=None):
        T = list(seg)
        count = 0
        while True:
            R = [self.rank.get((T[i], T[i + 1]), INF) for i in range(len(T) - 1)]
            present = [r for r in R if r < INF]
            if not present:
                break
            E = min(self.limit[r] for r in present)
            count += 1
            L = len(R)
            S = [r < E for r in R]                                   # candidates
            beaten_left = [i > 0 and S[i] and S[i - 1] and R[i - 1] <= R[i] for i in range(L)]
            beaten_right = [i + 1 < L and S[i] and S[i + 1] and R[i + 1] < R[i] for i in range(L)]
            applied, run = [False] * L, 0
            for i in range(L):
                run = run + 1 if beaten_left[i] else 0                # place in the run of left-beaten candidates
                applied[i] = S[i] and not beaten_right[i] and run % 2 == 0
            assert any(applied)                                       # a pass always makes progress
            out, i = [], 0
            while i < len(T):
                if i < L and applied[i]:
                    out.append(256 + R[i])
                    i += 2
                else:
                    out.append(T[i])
                    i += 1
            T = out
        if passes is not None:
            passes.append(count)
        return T

    def encode(self, data: bytes, rule):
        out = []
        for seg in self.segments(data):
            out += rule(seg)
        return out


def check(model, orc, data):
    want = orc.encode(data, oracle.TEXTBOOK).tolist()
    assert model.encode(data, model.encode_segment_lane) == want, ("lanes", model.rows[:8], data)
    assert model.encode(data, model.encode_segment_fused) == want, ("fused", model.rows[:8], data)
    assert model.encode_segment_fused(data) == want, ("fused, whole string", model.rows[:8], data)


def test_rules_on_random_tables():
    rng = random.Random(7)
    for trial in range(120):
        alphabet = rng.sample(range(256), rng.randint(2, 5))
        rows = random_monotone_table(rng, rng.randint(1, 120), alphabet)
        model, orc = Model(rows), oracle.Table(rows)
        for _ in range(12):
            check(model, orc, bytes(rng.choice(alphabet) for _ in range(rng.randint(0, 200))))


def test_cuts_exist_and_split_what_they_should():
    """Rows ab, cd, (ab)(cd): 'bc' is a junction (row 2), 'da' is not: "abcdabcd" has one cut, in the middle."""
    model = Model([(97, 98), (99, 100), (256, 257)])
    assert model.segments(b"abcdabcd") == [b"abcd", b"abcd"]
    assert model.encode(b"abcdabcd", model.encode_segment_lane) == [258, 258]
    assert model.segments(b"") == [b""] and model.encode(b"", model.encode_segment_lane) == []


@pytest.mark.parametrize("key,cfg,count", [("1k", 1, 64), ("32k", 2, 24), ("100k", 4, 2)])
def test_rules_on_trained_tables(key, cfg, count):
    merges = workloads.load_merges(key)
    model, orc = Model(merges), oracle.Table(merges)
    data, off = workloads.batch(cfg, batch_override=count)
    fused_passes, longest = [], 0
    for s in range(count):
        d = data[off[s]:min(off[s + 1], off[s] + 1024)].tobytes()
        check(model, orc, d)
        model.encode(d, lambda seg: model.encode_segment_fused(seg, fused_passes))
        longest = max(longest, max(len(x) for x in model.segments(d)))
    assert max(fused_passes) <= 64 or cfg == 4           # segment horizons keep the pass count low on text
    assert longest <= 32 or cfg == 4                     # text segments fit a lane; the adversarial runs do not
