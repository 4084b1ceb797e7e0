"""Seeded synthetic inputs for the five benchmark configurations.

Holds input generation only (text streams, adversarial strings, length mixes, and the loader for the stored
merge tables).  None of the method's arithmetic lives here; the CPU oracle and the HIP path both take their
inputs from this module and neither is imported by it.

The generators are native (``gen.cpp`` -> ``libworkloads.so``, built on first use with g++).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.cpp")
_LIB = os.path.join(_HERE, "libworkloads.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile gen.cpp into libworkloads.so (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.wl_text.argtypes = [ctypes.c_int, ctypes.c_uint64, ctypes.c_void_p, ctypes.c_int64]
        lib.wl_text.restype = ctypes.c_int
        lib.wl_adversarial.argtypes = [ctypes.c_uint64, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64]
        lib.wl_adversarial.restype = ctypes.c_int
        lib.wl_lognormal_lengths.argtypes = [ctypes.c_uint64, ctypes.c_void_p, ctypes.c_int64,
                                             ctypes.c_double, ctypes.c_double, ctypes.c_int64, ctypes.c_int64]
        lib.wl_lognormal_lengths.restype = ctypes.c_int
        _lib = lib
    return _lib


def text(style: int, seed: int, nbytes: int) -> np.ndarray:
    """nbytes of the style's word stream as a uint8 array."""
    out = np.empty(nbytes, dtype=np.uint8)
    rc = _load().wl_text(style, seed, out.ctypes.data, nbytes)
    if rc != 0:
        raise ValueError(f"wl_text({style}, {seed}, {nbytes}) failed")
    return out


def adversarial(seed: int, nstrings: int, length: int) -> np.ndarray:
    out = np.empty(nstrings * length, dtype=np.uint8)
    rc = _load().wl_adversarial(seed, out.ctypes.data, nstrings, length)
    if rc != 0:
        raise ValueError("wl_adversarial failed")
    return out


def lognormal_lengths(seed: int, count: int, median: float, sigma: float, lo: int, hi: int) -> np.ndarray:
    out = np.empty(count, dtype=np.int64)
    rc = _load().wl_lognormal_lengths(seed, out.ctypes.data, count, median, sigma, lo, hi)
    if rc != 0:
        raise ValueError("wl_lognormal_lengths failed")
    return out


@dataclass(frozen=True)
class Config:
    """One benchmark configuration: which table it uses and the shape of its encode batch."""
    index: int
    name: str
    table: str            # key into TABLES
    batch: int
    length: int           # bytes per string (0 = log-normal mix)
    kind: str             # "text", "adversarial" or "lognormal"
    style: int            # text style of the batch strings


# table key -> (text style of the training corpus, corpus bytes, corpus seed, number of merges)
TABLES = {
    "1k": (1, 1 << 20, 1001, 1_000),
    "32k": (2, 64 << 20, 1002, 32_000),
    "100k": (3, 256 << 20, 1003, 100_000),
}

CONFIGS = {
    1: Config(1, "tiny", "1k", 64, 256, "text", 1),
    2: Config(2, "32k-merges 1024x1KiB", "32k", 1024, 1024, "text", 2),
    3: Config(3, "100k-merges 8192x4KiB", "100k", 8192, 4096, "text", 3),
    4: Config(4, "adversarial 2048x16KiB", "100k", 2048, 16384, "adversarial", 3),
    5: Config(5, "throughput 65536 lognormal", "100k", 65536, 0, "lognormal", 3),
    # not one of the five benchmark configurations: whole 64 KiB strings of one repeated byte each, the input
    # that has no place to cut and so exercises the encoder for strings that exceed on-chip memory
    6: Config(6, "long runs 256x64KiB", "100k", 256, 65536, "runs", 3),
}

BATCH_SEED = 0


def corpus(table: str) -> np.ndarray:
    """The training corpus of a table (regenerated from its seed; never stored)."""
    style, nbytes, seed, _ = TABLES[table]
    return text(style, seed, nbytes)


def batch(cfg: int, batch_override: int | None = None):
    """(bytes uint8[total], offsets int64[B+1]) of a configuration's encode batch, seed 0.

    ``batch_override`` keeps the recipe but generates fewer (or more) strings; a prefix of the full
    batch for the fixed-length configurations.
    """
    c = CONFIGS[cfg]
    b = c.batch if batch_override is None else int(batch_override)
    if c.kind == "text":
        data = text(c.style, BATCH_SEED, b * c.length)
        offsets = np.arange(b + 1, dtype=np.int64) * c.length
    elif c.kind == "runs":
        run_bytes = np.frombuffer(b"a0 e", dtype=np.uint8)
        data = np.repeat(run_bytes[np.arange(b) % len(run_bytes)], c.length)
        offsets = np.arange(b + 1, dtype=np.int64) * c.length
    elif c.kind == "adversarial":
        data = adversarial(BATCH_SEED, b, c.length)
        offsets = np.arange(b + 1, dtype=np.int64) * c.length
    else:
        lens = lognormal_lengths(BATCH_SEED, b, 2048.0, 1.0, 64, 65536)
        offsets = np.zeros(b + 1, dtype=np.int64)
        np.cumsum(lens, out=offsets[1:])
        data = text(c.style, BATCH_SEED, int(offsets[-1]))
    return data, offsets


def table_path(table: str) -> str:
    return os.path.join(_HERE, "tables", f"merges_{table}.bin")


def load_merges(table: str) -> np.ndarray:
    """The stored merge list of a table as int32[n_merges, 2]; row index = rank, merged id = 256 + rank.

    The files are written by ``oracle/make_tables.py`` (the oracle's trainer run on ``corpus(table)``).
    """
    path = table_path(table)
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: run `python oracle/make_tables.py {table}`")
    m = np.fromfile(path, dtype=np.int32)
    return m.reshape(-1, 2)
