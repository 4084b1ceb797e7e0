"""CPU oracle for byte-level BPE encoding -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``bpe_oracle.cpp`` (built with g++ into ``liboracle.so``).  Only ``tests/``, the smoke
check and the benchmark's cpu-baseline leg may import this package; the product path never does.  It shares
no code with the HIP library.

Encoder tiers: 0 = Algorithm 1 literally (brute force), 1 = textbook sequential with cached ranks,
2 = pass view (one rank per pass, also counts passes / token visits), 3 = heap + linked list.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bpe_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

BRUTE, TEXTBOOK, PASSES, HEAP = 0, 1, 2, 3


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-pthread", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, i32, i64, ci = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int
        lib.orc_table_new.argtypes = [vp, i32]
        lib.orc_table_new.restype = vp
        lib.orc_table_new_vocab.argtypes = [vp, vp, vp, i32]
        lib.orc_table_new_vocab.restype = vp
        lib.orc_table_free.argtypes = [vp]
        lib.orc_table_free.restype = None
        lib.orc_table_set_specials.argtypes = [vp, vp, vp, vp, i32]
        lib.orc_table_set_specials.restype = None
        lib.orc_encode.argtypes = [vp, ci, vp, i64, vp, vp]
        lib.orc_encode.restype = i64
        lib.orc_encode_batch.argtypes = [vp, ci, vp, vp, i64, ci, vp, vp, vp]
        lib.orc_encode_batch.restype = i64
        lib.orc_pass_trace.argtypes = [vp, vp, i64, vp, i64]
        lib.orc_pass_trace.restype = i64
        lib.orc_decode.argtypes = [vp, vp, i64, vp, i64]
        lib.orc_decode.restype = i64
        lib.orc_train.argtypes = [vp, i64, i32, vp, ci]
        lib.orc_train.restype = i64
        _lib = lib
    return _lib


def _as_bytes(s) -> np.ndarray:
    if isinstance(s, str):
        s = s.encode("utf-8")
    if isinstance(s, (bytes, bytearray)):
        return np.frombuffer(bytes(s), dtype=np.uint8)
    return np.ascontiguousarray(s, dtype=np.uint8)


class Table:
    """A merge table: rows of (left_id, right_id); rank = row index; merged id = 256 + rank.

    With a vocabulary (`byte_ids[256]`: id of each single byte; `merged_ids[rows]`: id of the token each row
    creates) the rows and the results are in the vocabulary's ids instead."""

    def __init__(self, merges, byte_ids=None, merged_ids=None):
        self.merges = np.ascontiguousarray(np.asarray(merges, dtype=np.int32).reshape(-1, 2))
        if (byte_ids is None) != (merged_ids is None):
            raise ValueError("give both byte_ids and merged_ids, or neither")
        if byte_ids is None:
            self._h = _load().orc_table_new(self.merges.ctypes.data, len(self.merges))
        else:
            self.byte_ids = np.ascontiguousarray(np.asarray(byte_ids, dtype=np.int32))
            self.merged_ids = np.ascontiguousarray(np.asarray(merged_ids, dtype=np.int32))
            if self.byte_ids.shape != (256,) or self.merged_ids.shape != (len(self.merges),):
                raise ValueError("byte_ids must have 256 entries and merged_ids one per row")
            self._h = _load().orc_table_new_vocab(self.byte_ids.ctypes.data, self.merges.ctypes.data,
                                                  self.merged_ids.ctypes.data, len(self.merges))

    def set_specials(self, specials):
        """specials: {bytes: id}.  Their occurrences (left to right, the longest where several match) become
        one token each; the text between them is encoded on its own.  An empty dict removes them."""
        items = [(bytes(k), int(v)) for k, v in dict(specials).items()]
        text = np.frombuffer(b"".join(k for k, _ in items), dtype=np.uint8).copy()
        off = np.zeros(len(items) + 1, dtype=np.int32)
        np.cumsum([len(k) for k, _ in items], out=off[1:])
        ids = np.array([v for _, v in items], dtype=np.int32)
        _load().orc_table_set_specials(self._h, text.ctypes.data if len(text) else None, off.ctypes.data,
                                       ids.ctypes.data if len(ids) else None, len(items))

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.orc_table_free(self._h)
            self._h = None

    def __len__(self):
        return len(self.merges)

    def encode(self, s, tier: int = TEXTBOOK, stats: bool = False):
        b = _as_bytes(s)
        out = np.empty(max(len(b), 1), dtype=np.int32)
        st = np.zeros(3, dtype=np.int64)
        k = _load().orc_encode(self._h, tier, b.ctypes.data, len(b), out.ctypes.data, st.ctypes.data)
        ids = out[:k].copy()
        if stats:
            return ids, {"passes": int(st[0]), "visits": int(st[1]), "merges": int(st[2])}
        return ids

    def pass_trace(self, s):
        """What each pass of the pass view (one rank per pass, section 4.2) did on s: a list of
        (rank applied, live tokens at the start of the pass, merges applied by the pass)."""
        b = _as_bytes(s)
        cap = max(len(b), 1)
        out = np.zeros(3 * cap, dtype=np.int64)
        passes = _load().orc_pass_trace(self._h, b.ctypes.data, len(b), out.ctypes.data, cap)
        return [tuple(int(x) for x in out[3 * i:3 * i + 3]) for i in range(min(passes, cap))]

    def encode_batch(self, data, offsets, tier: int = TEXTBOOK, nthreads: int = 1, stats: bool = False):
        """Dense (ids int32[total_tokens], out_offsets int64[B+1]) for a batch of strings."""
        data = _as_bytes(data)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        b = len(offsets) - 1
        out = np.empty(max(int(offsets[-1]), 1), dtype=np.int32)
        out_off = np.zeros(b + 1, dtype=np.int64)
        st = np.zeros(3, dtype=np.int64)
        k = _load().orc_encode_batch(self._h, tier, data.ctypes.data, offsets.ctypes.data, b, nthreads,
                                     out.ctypes.data, out_off.ctypes.data, st.ctypes.data)
        ids = out[:k].copy()
        if stats:
            return ids, out_off, {"passes": int(st[0]), "visits": int(st[1]), "merges": int(st[2])}
        return ids, out_off

    def decode(self, ids) -> bytes:
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        cap = 64
        while True:
            out = np.empty(cap, dtype=np.uint8)
            n = _load().orc_decode(self._h, ids.ctypes.data, len(ids), out.ctypes.data, cap)
            if n <= cap:
                return out[:n].tobytes()
            cap = int(n)


def train(corpus, n_merges: int, naive: bool = False) -> np.ndarray:
    """Greedy most-frequent-pair trainer; returns int32[rows, 2] (rows <= n_merges if pairs run out)."""
    c = _as_bytes(corpus)
    out = np.zeros((max(n_merges, 1), 2), dtype=np.int32)
    rows = _load().orc_train(c.ctypes.data, len(c), n_merges, out.ctypes.data, 1 if naive else 0)
    return out[:rows].copy()
