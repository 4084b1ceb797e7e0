"""The C-ABI library: loads without a GPU, exports every symbol the header declares, and rejects bad
arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2507_11941_amd as bpe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "bpe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bpe_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = bpe.load_library()
    names = declared_functions()
    assert {"bpe_build_table", "bpe_free_table", "bpe_encode_batch", "bpe_workspace_bytes",
            "bpe_strerror"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_error_strings():
    lib = bpe.load_library()
    for code in (0, -1, -2, -3, -4, -5, -6, -7):
        assert lib.bpe_strerror(code)
    assert lib.bpe_strerror(0) == b"ok"


def build_raw(merges, n=None):
    lib = bpe.load_library()
    m = np.ascontiguousarray(np.asarray(merges, dtype=np.int32).reshape(-1, 2))
    handle, bad = ctypes.c_void_p(), ctypes.c_int32(-7)
    code = lib.bpe_build_table(m.ctypes.data, len(m) if n is None else n, ctypes.byref(handle), ctypes.byref(bad))
    return code, bad.value, handle.value


def test_build_table_rejects_malformed_tables_on_the_host():
    # forward reference: row 1 uses id 258 which row 1 itself would create at the earliest
    assert build_raw([(97, 98), (258, 99)])[:2] == (-2, 1)
    assert build_raw([(97, 256)])[:2] == (-2, 0)          # a row cannot use its own token
    assert build_raw([(-1, 98)])[:2] == (-2, 0)
    # duplicate pair
    assert build_raw([(97, 98), (98, 99), (97, 98)])[:2] == (-3, 2)
    # negative count, null output
    assert build_raw([(97, 98)], n=-1)[0] == -1
    lib = bpe.load_library()
    assert lib.bpe_build_table(None, 1, None, None) == -1
    with pytest.raises(bpe.BpeError):
        bpe.build_table([(97, 98), (97, 98)])


def build_vocab_raw(byte_ids, merges, merged):
    lib = bpe.load_library()
    b = np.ascontiguousarray(byte_ids, dtype=np.int32)
    m = np.ascontiguousarray(np.asarray(merges, dtype=np.int32).reshape(-1, 2))
    g = np.ascontiguousarray(merged, dtype=np.int32)
    handle, bad = ctypes.c_void_p(), ctypes.c_int32(-7)
    code = lib.bpe_build_table_vocab(b.ctypes.data, m.ctypes.data, g.ctypes.data, len(m), ctypes.byref(handle),
                                     ctypes.byref(bad))
    return code, bad.value


def test_build_table_vocab_rejects_malformed_vocabularies_on_the_host():
    ids = np.arange(256, dtype=np.int32) + 1000
    a, b, c = 1097, 1098, 1099
    # an operand that is neither a byte id nor created by an earlier row
    assert build_vocab_raw(ids, [(a, b), (7, c)], [5, 6]) == (-2, 1)
    assert build_vocab_raw(ids, [(5, b)], [5]) == (-2, 0)           # a row cannot use its own token
    assert build_vocab_raw(ids, [(97, 98)], [5]) == (-2, 0)         # default byte values are not ids here
    # ids must be unique: merged id equal to a byte id, to an earlier merged id, two bytes alike
    assert build_vocab_raw(ids, [(a, b)], [a]) == (-7, 0)
    assert build_vocab_raw(ids, [(a, b), (b, c)], [5, 5]) == (-7, 1)
    twice = ids.copy()
    twice[3] = twice[200]
    assert build_vocab_raw(twice, [(a, b)], [5]) == (-7, -1)
    # the same pair in two rows
    assert build_vocab_raw(ids, [(a, b), (b, c), (a, b)], [5, 6, 7]) == (-3, 2)
    # negative ids, null arrays
    assert build_vocab_raw(ids, [(a, b)], [-5])[0] == -1
    lib = bpe.load_library()
    assert lib.bpe_build_table_vocab(None, None, None, 0, None, None) == -1
    with pytest.raises(bpe.BpeError):
        bpe.build_table_vocab(ids, [(a, b)], [a])


def test_workspace_bytes():
    assert bpe.workspace_bytes(-1, 0, 0) == 0
    assert bpe.workspace_bytes(1, -1, 0) == 0
    assert bpe.workspace_bytes(1, 10, bpe.MAX_STRING_BYTES + 1) == 0
    small = bpe.workspace_bytes(64, 64 * 256, 256)
    assert small >= 64 * 256 * 4 and small % 256 == 0
    assert bpe.workspace_bytes(64, 64 * 256, 65536) > small       # staging for strings beyond LDS
    assert bpe.workspace_bytes(0, 0, 0) > 0


def test_encode_rejects_bad_arguments_without_a_device():
    lib = bpe.load_library()
    assert lib.bpe_encode_batch(None, None, None, 0, 0, 0, None, None, None, 0, None) == -1
    assert lib.bpe_table_n_merges(None) == 0
    lib.bpe_free_table(None)
    assert lib.bpe_read_profile(None, None) == -1


def test_static_entry_point_limits_fit_its_scratch():
    """The limits of bpe_encode_batch_static are such that the workspace of any call within them fits the
    24 MiB array the library carries (the workspace grows with each of the three sizes)."""
    text = open(os.path.join(ROOT, "include", "bpe.h")).read()
    lim = {k: int(eval(v)) for k, v in re.findall(r"#define (BPE_STATIC_MAX_\w+) (.+)", text)}
    assert lim == {"BPE_STATIC_MAX_BATCH": 4096, "BPE_STATIC_MAX_TOTAL_BYTES": 4 << 20,
                   "BPE_STATIC_MAX_STRING_BYTES": 16384}
    worst = bpe.workspace_bytes(lim["BPE_STATIC_MAX_BATCH"], lim["BPE_STATIC_MAX_TOTAL_BYTES"],
                                lim["BPE_STATIC_MAX_STRING_BYTES"])
    assert 0 < worst <= 24 << 20
    for batch, total, max_len in ((4096, 4 << 20, 1024), (1, 4 << 20, 16384), (4096, 4096, 1), (0, 0, 0)):
        assert bpe.workspace_bytes(batch, total, max_len) <= worst
