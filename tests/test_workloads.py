"""The seeded input generators: determinism, shapes, and the statistical recipe of each configuration."""
import hashlib

import numpy as np

import workloads


def test_streams_are_deterministic_and_prefix_stable():
    for style in (1, 2, 3):
        a = workloads.text(style, 0, 5000)
        b = workloads.text(style, 0, 5000)
        assert np.array_equal(a, b)
        assert np.array_equal(workloads.text(style, 0, 1200), a[:1200])
        assert not np.array_equal(workloads.text(style, 1, 5000), a)


def test_style1_alphabet_and_word_lengths():
    t = workloads.text(1, 3, 200_000).tobytes()
    assert set(t) <= set(b"abcdefghijklmnopqrstuvwxyz ")
    words = t[: t.rindex(b" ")].split(b" ")
    assert all(1 <= len(w) <= 12 for w in words)
    # Zipf head: the most frequent word carries a visible share of the stream
    _, counts = np.unique(np.array(words, dtype=object), return_counts=True)
    assert counts.max() / len(words) > 0.05


def test_style2_has_capitals_digits_punctuation_and_newlines():
    t = workloads.text(2, 3, 300_000).tobytes()
    assert all(b < 128 for b in t)
    lines = t.split(b"\n")
    assert len(lines) > 1000 and max(len(x) for x in lines[:-1]) < 80 + 16
    words = t.replace(b"\n", b" ").split(b" ")
    alpha = [w for w in words if w.isalpha()]
    cap = sum(1 for w in alpha if w[:1].isupper()) / len(alpha)
    assert 0.10 < cap < 0.20
    assert any(w.isdigit() for w in words) and any(not w.isalnum() for w in words if w)


def test_style3_is_wellformed_utf8_with_multibyte_share():
    t = workloads.text(3, 3, 400_000).tobytes()
    t = t[: max(t.rindex(b" "), t.rindex(b"\n"))]      # drop the possibly cut last word
    s = t.decode("utf-8")                              # raises if malformed
    words = s.split()
    multi = [w for w in words if ord(w[0]) >= 0x80]
    assert 0.12 < len(multi) / len(words) < 0.18
    assert all(1 <= len(w) <= 6 for w in multi)
    assert {len(w[0].encode()) for w in multi} == {2, 3, 4}
    assert not any(0xD800 <= ord(ch) <= 0xDFFF for w in multi for ch in w)


def test_config_batches_have_the_stated_shapes():
    for cfg, (b, n) in {1: (64, 256), 2: (1024, 1024)}.items():
        data, off = workloads.batch(cfg)
        assert len(off) == b + 1 and off[0] == 0 and off[-1] == len(data) == b * n
        assert (np.diff(off) == n).all()
    data, off = workloads.batch(4, batch_override=8)
    assert len(data) == 8 * 16384
    s = data[:16384].tobytes()
    # long runs of one byte exist
    best, cur = 1, 1
    for i in range(1, len(s)):
        cur = cur + 1 if s[i] == s[i - 1] else 1
        best = max(best, cur)
    assert best >= 16


def test_lognormal_lengths_recipe():
    lens = workloads.lognormal_lengths(0, 65536, 2048.0, 1.0, 64, 65536)
    assert lens.min() >= 64 and lens.max() <= 65536
    assert 1900 < np.median(lens) < 2200
    assert 190 * 2**20 < lens.sum() < 230 * 2**20
    data, off = workloads.batch(5, batch_override=256)
    assert np.array_equal(np.diff(off), lens[:256]) and len(data) == off[-1]


def test_generator_regression_hashes():
    """The byte streams themselves are fixed: a change here changes every stored table and result."""
    got = {s: hashlib.sha256(workloads.text(s, 0, 4096).tobytes()).hexdigest()[:16] for s in (1, 2, 3)}
    got["adv"] = hashlib.sha256(workloads.adversarial(0, 2, 4096).tobytes()).hexdigest()[:16]
    assert got == EXPECTED_HASHES, got


EXPECTED_HASHES = {1: '67d7c93ee2c1d8ec', 2: 'fcad8362c319486d', 3: 'fa32c59cd043632b', 'adv': '1886a9462b3e539d'}
