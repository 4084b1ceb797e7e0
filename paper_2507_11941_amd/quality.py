"""Tokenization-quality harness (section 5.2 of the paper): how close the byte-level encoding -- what this
library computes, with no regular-expression pre-tokenisation -- comes to the encoding a regex-pretokenised BPE
gives with the same merge table.

The paper's measure: for every input string s_i, the Levenshtein distance d_L between the two token sequences,
divided by |s_i|, subtracted from one, averaged over the batch:

    sim = 1/n * sum_i ( 1 - d_L(t_i_ref, t_i_ours) / |s_i| )

The paper does not say in what unit |s_i| is taken; here it is the string's length in bytes (the unit the
byte-level method works in), so that a string whose every token differs still scores above zero.  The reference
side of the paper is HuggingFace Tokenizers; `regex_reference` builds exactly that from a merge list (a BPE model
over the table with the byte-level regex pre-tokeniser in front).  Nothing in the encode path uses this module.
"""
from __future__ import annotations

import numpy as np


def levenshtein(a, b) -> int:
    """Edit distance (insert, delete, substitute, each at cost 1) between two sequences of token ids."""
    a = np.asarray(a, dtype=np.int64).ravel()
    b = np.asarray(b, dtype=np.int64).ravel()
    if len(a) < len(b):
        a, b = b, a
    if len(b) == 0:
        return int(len(a))
    # one row of the dynamic programme per element of a; the dependence of a cell on its left neighbour
    # (an insertion chain) is a running minimum of (cell - column), which numpy can do in one call
    cols = np.arange(len(b) + 1, dtype=np.int64)
    row = cols.copy()
    for i, x in enumerate(a, start=1):
        cand = np.empty_like(row)
        cand[0] = i
        cand[1:] = np.minimum(row[1:] + 1, row[:-1] + (b != x))
        row = np.minimum.accumulate(cand - cols) + cols
    return int(row[-1])


def similarity(reference, ours, lengths) -> float:
    """The paper's sim over a batch: `reference` and `ours` are lists of id sequences, `lengths` the strings'
    byte lengths.  Strings of length zero are left out (both sides are empty there)."""
    terms = []
    for ref, got, n in zip(reference, ours, lengths):
        if n > 0:
            terms.append(1.0 - levenshtein(ref, got) / float(n))
    return float(np.mean(terms)) if terms else 1.0


def byte_alphabet():
    """The byte -> printable character map of byte-level BPE vocabularies (printable Latin-1 bytes stand for
    themselves, the others take the code points from 256 on, in byte order)."""
    keep = list(range(ord("!"), ord("~") + 1)) + list(range(0xA1, 0xAC + 1)) + list(range(0xAE, 0xFF + 1))
    chars, extra = {}, 0
    for b in range(256):
        if b in keep:
            chars[b] = chr(b)
        else:
            chars[b] = chr(256 + extra)
            extra += 1
    return chars


def regex_reference(merges, use_regex: bool = True):
    """A HuggingFace `tokenizers.Tokenizer` over the merge list (row index = rank, ids as this library numbers
    them: byte b = b, row r = 256 + r) with the byte-level pre-tokeniser in front: with `use_regex` it splits the
    text with the usual word / number / punctuation pattern before any merge (the paper's ground truth), without
    it the whole text is one word (then it must agree with Algorithm 1 on the bytes).
    Raises ValueError if two tokens of the table spell the same bytes (a string-keyed vocabulary cannot hold both)."""
    from tokenizers import Tokenizer, models, pre_tokenizers

    chars = byte_alphabet()
    spell = [chars[b] for b in range(256)]
    pairs = []
    for a, b in np.asarray(merges, dtype=np.int64).reshape(-1, 2).tolist():
        pairs.append((spell[a], spell[b]))
        spell.append(spell[a] + spell[b])
    vocab = {s: i for i, s in enumerate(spell)}
    if len(vocab) != len(spell):
        raise ValueError("two tokens of the table spell the same bytes")
    tok = Tokenizer(models.BPE(vocab=vocab, merges=pairs))
    tok.pre_tokenizer = pre_tokenizers.ByteLevel(add_prefix_space=False, use_regex=use_regex)
    return tok


def reference_ids(tokenizer, strings):
    """Token ids of each byte string (which must be valid UTF-8) under `tokenizer`."""
    return [np.asarray(e.ids, dtype=np.int64)
            for e in tokenizer.encode_batch([s.decode("utf-8") for s in strings], add_special_tokens=False)]


def whole_characters(data: bytes) -> bytes:
    """`data` without the incomplete UTF-8 sequences a cut may have left at its ends."""
    return data.decode("utf-8", errors="ignore").encode("utf-8")
