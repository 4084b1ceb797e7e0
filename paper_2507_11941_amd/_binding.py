"""ctypes binding of include/bpe.h: argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbpe_hip.so")
_lib = None

MAX_STRING_BYTES = 65536


class BpeError(RuntimeError):
    def __init__(self, code: int, what: str, detail: str = ""):
        self.code = code
        super().__init__(f"{what}: {detail or code}")


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libbpe_hip.so (built by ``paper_2507_11941_amd.build``).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch ships its own HIP runtime under the same soname as the system one; whichever is loaded first
    # serves the whole process.  Load torch's first so that the library shares the runtime (streams,
    # device pointers) of the tensors it is handed.
    import torch  # noqa: F401

    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(f"{_LIB_PATH} not built: run `python -m paper_2507_11941_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.bpe_build_table.argtypes = [vp, i32, ctypes.POINTER(vp), ctypes.POINTER(i32)]
    lib.bpe_build_table.restype = ctypes.c_int
    lib.bpe_build_table_vocab.argtypes = [vp, vp, vp, i32, ctypes.POINTER(vp), ctypes.POINTER(i32)]
    lib.bpe_build_table_vocab.restype = ctypes.c_int
    lib.bpe_table_image.argtypes = [vp, i32, vp, ctypes.c_int64, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.bpe_table_image.restype = ctypes.c_int64
    lib.bpe_table_set_specials.argtypes = [vp, vp, vp, vp, i32]
    lib.bpe_table_set_specials.restype = ctypes.c_int
    lib.bpe_free_table.argtypes = [vp]
    lib.bpe_free_table.restype = None
    lib.bpe_table_n_merges.argtypes = [vp]
    lib.bpe_table_n_merges.restype = i32
    lib.bpe_workspace_bytes.argtypes = [i32, i64, i32]
    lib.bpe_workspace_bytes.restype = ctypes.c_size_t
    lib.bpe_encode_batch.argtypes = [vp, vp, vp, i32, i64, i32, vp, vp, vp, ctypes.c_size_t, vp]
    lib.bpe_encode_batch.restype = ctypes.c_int
    lib.bpe_encode_batch_static.argtypes = [vp, vp, vp, i32, i64, i32, vp, vp, vp]
    lib.bpe_encode_batch_static.restype = ctypes.c_int
    lib.bpe_read_profile.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
    lib.bpe_read_profile.restype = ctypes.c_int
    lib.bpe_set_profiling.argtypes = [ctypes.c_int]
    lib.bpe_set_profiling.restype = ctypes.c_int
    lib.bpe_strerror.argtypes = [ctypes.c_int]
    lib.bpe_strerror.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(code: int, what: str):
    if code != 0:
        raise BpeError(code, what, load_library().bpe_strerror(code).decode())


class Table:
    """Handle of a GPU-resident merge table (bpe_build_table / bpe_free_table)."""

    def __init__(self, handle: int, n_merges: int):
        self._h = handle
        self.n_merges = n_merges

    @property
    def handle(self) -> int:
        return self._h

    def set_specials(self, specials):
        """specials: {bytes: id}; every occurrence of one of the byte strings becomes one token with that id
        (bpe_table_set_specials).  An empty dict removes them."""
        items = [(bytes(k), int(v)) for k, v in dict(specials).items()]
        text = np.frombuffer(b"".join(k for k, _ in items), dtype=np.uint8).copy()
        off = np.zeros(len(items) + 1, dtype=np.int32)
        np.cumsum([len(k) for k, _ in items], out=off[1:])
        ids = np.array([v for _, v in items], dtype=np.int32)
        _check(load_library().bpe_table_set_specials(self._h, text.ctypes.data if len(text) else None,
                                                     off.ctypes.data, ids.ctypes.data if len(ids) else None,
                                                     len(items)), "bpe_table_set_specials")

    def free(self):
        if self._h:
            load_library().bpe_free_table(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def build_table(merges) -> Table:
    """merges: int32[n, 2] on the host; row index = rank, merged id = 256 + rank."""
    lib = load_library()
    m = np.ascontiguousarray(np.asarray(merges, dtype=np.int32).reshape(-1, 2))
    handle = ctypes.c_void_p()
    bad = ctypes.c_int32(-1)
    code = lib.bpe_build_table(m.ctypes.data if len(m) else None, len(m), ctypes.byref(handle), ctypes.byref(bad))
    if code != 0:
        raise BpeError(code, "bpe_build_table", f"{lib.bpe_strerror(code).decode()} (row {bad.value})")
    return Table(handle.value, len(m))


def table_image(merges):
    """The host-memory image of the table (uint32 array) and log2 of its bucket count; needs no GPU."""
    lib = load_library()
    m = np.ascontiguousarray(np.asarray(merges, dtype=np.int32).reshape(-1, 2))
    ptr = m.ctypes.data if len(m) else None
    bad, log2 = ctypes.c_int32(-1), ctypes.c_int32(0)
    n = lib.bpe_table_image(ptr, len(m), None, 0, ctypes.byref(log2), ctypes.byref(bad))
    if n < 0:
        raise BpeError(int(n), "bpe_table_image", f"{lib.bpe_strerror(int(n)).decode()} (row {bad.value})")
    words = np.empty(n, dtype=np.uint32)
    lib.bpe_table_image(ptr, len(m), words.ctypes.data, n, ctypes.byref(log2), ctypes.byref(bad))
    return words, log2.value


def build_table_vocab(byte_ids, merges, merged_ids) -> Table:
    """Table over a vocabulary's own ids: byte_ids int32[256], merges int32[n, 2] in vocabulary ids,
    merged_ids int32[n] (id of the token each row creates); encode_batch then returns vocabulary ids."""
    lib = load_library()
    b = np.ascontiguousarray(np.asarray(byte_ids, dtype=np.int32))
    m = np.ascontiguousarray(np.asarray(merges, dtype=np.int32).reshape(-1, 2))
    g = np.ascontiguousarray(np.asarray(merged_ids, dtype=np.int32))
    if b.shape != (256,) or g.shape != (len(m),):
        raise ValueError("byte_ids must have 256 entries and merged_ids one per row")
    handle = ctypes.c_void_p()
    bad = ctypes.c_int32(-1)
    code = lib.bpe_build_table_vocab(b.ctypes.data, m.ctypes.data if len(m) else None,
                                     g.ctypes.data if len(m) else None, len(m), ctypes.byref(handle),
                                     ctypes.byref(bad))
    if code != 0:
        raise BpeError(code, "bpe_build_table_vocab", f"{lib.bpe_strerror(code).decode()} (row {bad.value})")
    return Table(handle.value, len(m))


def workspace_bytes(batch: int, total_bytes: int, max_len: int) -> int:
    return int(load_library().bpe_workspace_bytes(batch, total_bytes, max_len))


def encode_batch(table: Table, data, offsets, max_len: int, out_ids=None, out_offsets=None, workspace=None,
                 stream=None):
    """Enqueue one batch encode on ``stream`` (default: torch's current stream); returns
    (out_ids int32[capacity], out_offsets int64[B+1]) device tensors.  ``data`` is a uint8 CUDA tensor with
    the strings back to back, ``offsets`` an int64 CUDA tensor [B+1].  Nothing is synchronised."""
    import torch

    lib = load_library()
    if not (data.is_cuda and offsets.is_cuda):
        raise ValueError("encode_batch needs device tensors")
    if data.dtype != torch.uint8 or offsets.dtype != torch.int64:
        raise ValueError("data must be uint8 and offsets int64")
    data = data.contiguous()
    offsets = offsets.contiguous()
    batch = offsets.numel() - 1
    total = data.numel()
    dev = data.device
    if out_ids is None:
        out_ids = torch.empty(max(total, 1), dtype=torch.int32, device=dev)
    if out_offsets is None:
        out_offsets = torch.empty(batch + 1, dtype=torch.int64, device=dev)
    need = workspace_bytes(batch, total, max_len)
    if need == 0:
        raise BpeError(-1, "bpe_workspace_bytes", "invalid sizes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    if stream is None:
        stream = torch.cuda.current_stream(dev)
    if stream != torch.cuda.current_stream(dev):
        # tensors made above belong to torch's current stream: tell the allocator that `stream` uses them too,
        # so that their memory is not handed out again while the encode kernels still run
        for t in (out_ids, out_offsets, workspace):
            t.record_stream(stream)
    code = lib.bpe_encode_batch(table.handle, data.data_ptr(), offsets.data_ptr(), batch, total, max_len,
                                out_ids.data_ptr(), out_offsets.data_ptr(), workspace.data_ptr(),
                                workspace.numel(), stream.cuda_stream)
    _check(code, "bpe_encode_batch")
    return out_ids, out_offsets


STATIC_MAX_BATCH, STATIC_MAX_TOTAL_BYTES, STATIC_MAX_STRING_BYTES = 4096, 4 << 20, 16384


def encode_batch_static(table: Table, data, offsets, max_len: int, out_ids, out_offsets, stream=None):
    """bpe_encode_batch_static: the same encode with the library's built-in scratch instead of a workspace, for
    callers that cannot allocate; outputs are the caller's.  Calls on one GPU must not overlap."""
    import torch

    lib = load_library()
    if not (data.is_cuda and offsets.is_cuda and out_ids.is_cuda and out_offsets.is_cuda):
        raise ValueError("encode_batch_static needs device tensors")
    if data.dtype != torch.uint8 or offsets.dtype != torch.int64 or out_ids.dtype != torch.int32 \
            or out_offsets.dtype != torch.int64:
        raise ValueError("data must be uint8, offsets and out_offsets int64, out_ids int32")
    if not (data.is_contiguous() and offsets.is_contiguous() and out_ids.is_contiguous()
            and out_offsets.is_contiguous()):
        raise ValueError("encode_batch_static takes contiguous tensors (it makes no copies)")
    batch = offsets.numel() - 1
    if out_ids.numel() < data.numel() or out_offsets.numel() < batch + 1:
        raise ValueError("outputs too small")
    if stream is None:
        stream = torch.cuda.current_stream(data.device)
    code = lib.bpe_encode_batch_static(table.handle, data.data_ptr(), offsets.data_ptr(), batch, data.numel(),
                                       max_len, out_ids.data_ptr(), out_offsets.data_ptr(), stream.cuda_stream)
    _check(code, "bpe_encode_batch_static")
    return out_ids, out_offsets


def encode_strings(table: Table, strings, device=None):
    """Convenience for callers that start from host strings: ``strings`` is a sequence of ``bytes`` (or ``str``,
    encoded as UTF-8); returns one int32 numpy array of token ids per string.  Marshalling only: the bytes are
    joined, copied to the device, encoded by ``encode_batch`` and the ids copied back (this synchronises)."""
    import numpy as np
    import torch

    raw = [s.encode("utf-8") if isinstance(s, str) else bytes(s) for s in strings]
    lens = np.fromiter((len(b) for b in raw), dtype=np.int64, count=len(raw))
    offsets = np.zeros(len(raw) + 1, dtype=np.int64)
    np.cumsum(lens, out=offsets[1:])
    max_len = int(lens.max()) if len(raw) else 0
    if max_len > MAX_STRING_BYTES:
        raise ValueError(f"a string has {max_len} bytes; the encoder takes at most {MAX_STRING_BYTES}")
    dev = torch.device(device if device is not None else "cuda:0")
    data = np.frombuffer(b"".join(raw), dtype=np.uint8)
    d = torch.from_numpy(data.copy()).to(dev) if len(data) else torch.empty(0, dtype=torch.uint8, device=dev)
    o = torch.from_numpy(offsets).to(dev)
    with torch.cuda.device(dev):
        ids, out_off = encode_batch(table, d, o, max_len)
    out_off = out_off.cpu().numpy()
    ids = ids[: int(out_off[-1])].cpu().numpy()
    return [ids[out_off[i]:out_off[i + 1]] for i in range(len(raw))]


def set_profiling(enabled: bool) -> None:
    _check(load_library().bpe_set_profiling(1 if enabled else 0), "bpe_set_profiling")


def read_profile():
    """(total encode-kernel milliseconds, number of calls) recorded since set_profiling(True)."""
    total, calls = ctypes.c_float(0.0), ctypes.c_int32(0)
    _check(load_library().bpe_read_profile(ctypes.byref(total), ctypes.byref(calls)), "bpe_read_profile")
    return float(total.value), int(calls.value)
