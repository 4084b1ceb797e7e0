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
    for code in (0, -1, -2, -3, -4, -5, -6):
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
