"""ctypes binding of the tokenization pipeline (include/tokpipe.h): argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtokpipe.so")

EXPORTED_SYMBOLS = (
    "tokpipe_last_error", "tokpipe_index_jsonl", "tokpipe_tokenize",
    "tokfile_open", "tokfile_close", "tokfile_num_docs", "tokfile_num_tokens", "tokfile_token_bytes", "tokfile_doc",
)


class TokPipeError(RuntimeError):
    pass


class Stats(C.Structure):
    _fields_ = [("n_docs", C.c_uint64), ("n_tokens", C.c_uint64), ("bytes_read", C.c_uint64), ("seconds", C.c_double),
                ("cache_hits", C.c_uint64), ("cache_misses", C.c_uint64)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise TokPipeError(f"{LIB_PATH} is not built: run python -m paper_2602_08387_amd.build")
    l = C.CDLL(LIB_PATH)
    l.tokpipe_last_error.restype = C.c_char_p
    l.tokpipe_index_jsonl.restype = C.c_int
    l.tokpipe_index_jsonl.argtypes = [C.c_char_p, C.c_char_p, C.c_int, C.POINTER(C.c_uint64)]
    l.tokpipe_tokenize.restype = C.c_int
    l.tokpipe_tokenize.argtypes = [C.c_char_p, C.c_char_p, C.c_char_p, C.c_void_p, C.c_uint32, C.c_char_p, C.c_int64,
                                   C.c_int, C.c_int, C.c_int, C.POINTER(Stats)]
    l.tokfile_open.restype = C.c_void_p
    l.tokfile_open.argtypes = [C.c_char_p]
    l.tokfile_close.restype = None
    l.tokfile_close.argtypes = [C.c_void_p]
    for name in ("tokfile_num_docs", "tokfile_num_tokens"):
        getattr(l, name).restype = C.c_uint64
        getattr(l, name).argtypes = [C.c_void_p]
    l.tokfile_token_bytes.restype = C.c_uint32
    l.tokfile_token_bytes.argtypes = [C.c_void_p]
    l.tokfile_doc.restype = C.c_int
    l.tokfile_doc.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(C.c_void_p), C.POINTER(C.c_uint64)]
    return l


lib = _load()


def _check(rc, what):
    if rc != 0:
        raise TokPipeError(f"{what}: {lib.tokpipe_last_error().decode()}")


def index_jsonl(jsonl_path, index_path, n_threads=1) -> int:
    n = C.c_uint64(0)
    _check(lib.tokpipe_index_jsonl(os.fsencode(jsonl_path), os.fsencode(index_path), n_threads, C.byref(n)), "tokpipe_index_jsonl")
    return int(n.value)


def tokenize(jsonl_path, index_path, out_path, merges, key="text", eod_token=-1, n_workers=1, batch_docs=64,
             queue_depth=8) -> Stats:
    m = np.ascontiguousarray(np.asarray(merges, dtype=np.uint32).reshape(-1, 2))
    st = Stats()
    _check(lib.tokpipe_tokenize(os.fsencode(jsonl_path), os.fsencode(index_path), os.fsencode(out_path),
                                m.ctypes.data_as(C.c_void_p) if len(m) else None, len(m), key.encode(), int(eod_token),
                                n_workers, batch_docs, queue_depth, C.byref(st)), "tokpipe_tokenize")
    return st


class TokenFile:
    """Memory-mapped token file; doc(i) returns a NumPy view of document i's tokens."""

    def __init__(self, path):
        self._h = lib.tokfile_open(os.fsencode(path))
        if not self._h:
            raise TokPipeError(f"tokfile_open: {lib.tokpipe_last_error().decode()}")
        self.num_docs = int(lib.tokfile_num_docs(self._h))
        self.num_tokens = int(lib.tokfile_num_tokens(self._h))
        self.token_bytes = int(lib.tokfile_token_bytes(self._h))

    def doc(self, i) -> np.ndarray:
        p, n = C.c_void_p(), C.c_uint64()
        _check(lib.tokfile_doc(self._h, int(i), C.byref(p), C.byref(n)), "tokfile_doc")
        if n.value == 0:
            return np.zeros(0, np.uint16 if self.token_bytes == 2 else np.uint32)
        ctype = C.c_uint16 if self.token_bytes == 2 else C.c_uint32
        return np.ctypeslib.as_array(C.cast(p, C.POINTER(ctype)), shape=(int(n.value),))

    def close(self):
        if self._h:
            lib.tokfile_close(self._h)
            self._h = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()
