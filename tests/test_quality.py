"""The tokenization-quality measure of section 5.2: Levenshtein distance and the similarity formula against
hand-worked values and a brute-force recursion; the byte alphabet against the byte-level pre-tokeniser of the
`tokenizers` library; and that library's BPE model, with pre-tokenisation switched off, against the oracle's
textbook encoder on the stored tables -- an implementation of Algorithm 1 that neither side of this build wrote."""
import functools
import random

import numpy as np
import pytest

import oracle
import workloads
from paper_2507_11941_amd import quality

tokenizers = pytest.importorskip("tokenizers")


def brute_force_distance(a, b):
    @functools.lru_cache(maxsize=None)
    def d(i, j):
        if i == 0 or j == 0:
            return i + j
        return min(d(i - 1, j) + 1, d(i, j - 1) + 1, d(i - 1, j - 1) + (a[i - 1] != b[j - 1]))
    return d(len(a), len(b))


def test_levenshtein_known_values_and_brute_force():
    assert quality.levenshtein(list(b"kitten"), list(b"sitting")) == 3
    assert quality.levenshtein([], []) == 0
    assert quality.levenshtein([1, 2, 3], []) == 3 and quality.levenshtein([], [7]) == 1
    assert quality.levenshtein([5, 6, 7], [5, 6, 7]) == 0
    assert quality.levenshtein([1] * 10, [2] * 10) == 10
    rng = random.Random(3)
    for _ in range(300):
        a = tuple(rng.randrange(4) for _ in range(rng.randrange(0, 12)))
        b = tuple(rng.randrange(4) for _ in range(rng.randrange(0, 12)))
        assert quality.levenshtein(a, b) == brute_force_distance(a, b), (a, b)


def test_similarity_hand_worked():
    # "abcd" (4 bytes): reference [ab, c, d], ours [ab, cd]: substitute one token, delete one -> d_L = 2 -> 1 - 2/4
    # "xy" (2 bytes): equal -> 1.  Mean = 0.75
    sim = quality.similarity([[256, 99, 100], [300]], [[256, 257], [300]], [4, 2])
    assert sim == pytest.approx(0.75)
    assert quality.similarity([[1, 2]], [[1, 2]], [5]) == 1.0
    assert quality.similarity([[]], [[]], [0]) == 1.0          # empty strings are left out


def test_byte_alphabet_is_the_byte_level_pre_tokenisers():
    chars = quality.byte_alphabet()
    assert len(set(chars.values())) == 256
    assert set(chars.values()) == set(tokenizers.pre_tokenizers.ByteLevel.alphabet())
    pre = tokenizers.pre_tokenizers.ByteLevel(add_prefix_space=False, use_regex=False)
    for text in ["A", " ", "\n", "\t", "~", "\x7f", "é", "ß", "€", "日本", "\U0001F600", "a b\r\n"]:
        mapped = "".join(piece for piece, _ in pre.pre_tokenize_str(text))
        assert mapped == "".join(chars[b] for b in text.encode("utf-8")), text


@pytest.mark.parametrize("key,style", [("1k", 1), ("32k", 2), ("100k", 3)])
def test_library_bpe_without_pre_tokenisation_equals_algorithm_1(key, style):
    merges = workloads.load_merges(key)
    ref = quality.regex_reference(merges, use_regex=False)
    orc = oracle.Table(merges)
    rng = np.random.default_rng(11)
    text = workloads.text(style, 77, 64 * 1024).tobytes()
    strings = []
    at = 0
    while at < len(text) - 600:
        n = int(rng.integers(1, 500))
        strings.append(quality.whole_characters(text[at:at + n]))
        at += n
    got = quality.reference_ids(ref, strings)
    for s, ids in zip(strings, got):
        assert ids.tolist() == orc.encode(s, oracle.TEXTBOOK).tolist(), s


def test_regex_pre_tokenisation_changes_some_encodings():
    """With the word / number / punctuation split in front, merges that cross such a boundary cannot happen: on
    punctuated text the reference differs from Algorithm 1 in places, and the similarity says by how much."""
    merges = workloads.load_merges("32k")
    orc = oracle.Table(merges)
    ref = quality.regex_reference(merges, use_regex=True)
    text = workloads.text(2, 5, 32 * 1024).tobytes()
    strings = [text[i:i + 1024] for i in range(0, len(text), 1024)]
    ours = [orc.encode(s, oracle.TEXTBOOK) for s in strings]
    sim = quality.similarity(quality.reference_ids(ref, strings), ours, [len(s) for s in strings])
    assert 0.5 < sim <= 1.0
    print(f"similarity, 32k table, style-2 text: {sim:.4f}")
