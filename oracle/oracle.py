"""ctypes front end of the reference codec in ``zm_oracle.c``.

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports it, and it
never imports the product package.

The C file follows ZipMoE (arXiv 2601.21198) Sec. 2.2 (bf16 fields), Sec. 3.1
(offline initialisation: split, shard, compress, pack, serialise) and Sec. 3.3
(tensor recovery).  This module only moves numpy arrays in and out of it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zm_oracle.c")
_LIB = os.path.join(_HERE, "libzm_oracle.so")

OK, E_ARG, E_SIZE, E_FORMAT, E_NOMEM = 0, -1, -2, -3, -4
MODE_CODED, MODE_RAW = 0, 1
MAX_LEN = 12
TILE = 512


def build(force: bool = False) -> str:
    """Compile ``zm_oracle.c`` with gcc (building the checker is not using it)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", _LIB]
        )
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        u8p, u16p, u64p = (ctypes.POINTER(t) for t in (ctypes.c_uint8, ctypes.c_uint16, ctypes.c_uint64))
        sz = ctypes.c_size_t
        L.zo_split.argtypes = [u16p, sz, u8p, u8p]
        L.zo_split.restype = None
        L.zo_merge.argtypes = [u8p, u8p, sz, u16p]
        L.zo_merge.restype = None
        L.zo_histogram.argtypes = [u8p, sz, u64p]
        L.zo_histogram.restype = None
        L.zo_code_lengths.argtypes = [u64p, ctypes.c_int, u8p]
        L.zo_code_lengths.restype = ctypes.c_int
        L.zo_canonical.argtypes = [u8p, u16p]
        L.zo_canonical.restype = ctypes.c_int
        L.zo_kraft_units.argtypes = [u8p]
        L.zo_kraft_units.restype = ctypes.c_uint32
        L.zo_encode_bound.argtypes = [sz, ctypes.c_uint32, ctypes.c_uint32]
        L.zo_encode_bound.restype = sz
        L.zo_encode.argtypes = [u16p, sz, ctypes.c_uint32, ctypes.c_uint32, u8p, u8p, sz, ctypes.POINTER(sz)]
        L.zo_encode.restype = ctypes.c_int
        L.zo_blob_values.argtypes = [u8p, sz]
        L.zo_blob_values.restype = ctypes.c_uint64
        L.zo_decode.argtypes = [u8p, sz, u16p, sz]
        L.zo_decode.restype = ctypes.c_int
        L.zo_decode_chunks.argtypes = [u8p, sz, sz, sz, u16p]
        L.zo_decode_chunks.restype = ctypes.c_int
        L.zo_check_table.argtypes = [u8p, sz]
        L.zo_check_table.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(a: np.ndarray, t):
    return a.ctypes.data_as(ctypes.POINTER(t))


def _u16(words) -> np.ndarray:
    a = np.ascontiguousarray(words)
    if a.dtype != np.uint16:
        raise TypeError("bf16 words are passed as uint16")
    return a.reshape(-1)


class OracleError(Exception):
    def __init__(self, code: int):
        super().__init__(f"oracle returned {code}")
        self.code = code


def split(words):
    w = _u16(words)
    e = np.empty(w.size, np.uint8)
    sm = np.empty(w.size, np.uint8)
    lib().zo_split(_p(w, ctypes.c_uint16), w.size, _p(e, ctypes.c_uint8), _p(sm, ctypes.c_uint8))
    return e, sm


def merge(e, sm):
    e = np.ascontiguousarray(e, np.uint8).reshape(-1)
    sm = np.ascontiguousarray(sm, np.uint8).reshape(-1)
    assert e.size == sm.size
    w = np.empty(e.size, np.uint16)
    lib().zo_merge(_p(e, ctypes.c_uint8), _p(sm, ctypes.c_uint8), e.size, _p(w, ctypes.c_uint16))
    return w


def histogram(e):
    e = np.ascontiguousarray(e, np.uint8).reshape(-1)
    h = np.zeros(256, np.uint64)
    lib().zo_histogram(_p(e, ctypes.c_uint8), e.size, _p(h, ctypes.c_uint64))
    return h


def code_lengths(hist, max_len: int = 8):
    h = np.ascontiguousarray(hist, np.uint64)
    assert h.shape == (256,)
    out = np.zeros(256, np.uint8)
    rc = lib().zo_code_lengths(_p(h, ctypes.c_uint64), max_len, _p(out, ctypes.c_uint8))
    if rc != OK:
        raise OracleError(rc)
    return out


def canonical(lengths):
    l = np.ascontiguousarray(lengths, np.uint8)
    assert l.shape == (256,)
    code = np.zeros(256, np.uint16)
    n = lib().zo_canonical(_p(l, ctypes.c_uint8), _p(code, ctypes.c_uint16))
    return code, n


def kraft_units(lengths) -> int:
    l = np.ascontiguousarray(lengths, np.uint8)
    return int(lib().zo_kraft_units(_p(l, ctypes.c_uint8)))


def encode(words, chunk_values: int, stream_values: int, lengths) -> np.ndarray:
    """Serialise one tensor; returns the object as a uint8 array."""
    w = _u16(words)
    l = np.ascontiguousarray(lengths, np.uint8)
    cap = lib().zo_encode_bound(w.size, chunk_values, stream_values)
    blob = np.zeros(cap, np.uint8)
    size = ctypes.c_size_t(0)
    rc = lib().zo_encode(_p(w, ctypes.c_uint16), w.size, chunk_values, stream_values,
                         _p(l, ctypes.c_uint8), _p(blob, ctypes.c_uint8), cap, ctypes.byref(size))
    if rc != OK:
        raise OracleError(rc)
    return blob[: size.value].copy()


def encode_tensor(words, chunk_values: int, stream_values: int, max_len: int = 8):
    """split -> histogram -> code lengths -> serialise, the whole offline path."""
    e, _ = split(words)
    lengths = code_lengths(histogram(e), max_len)
    return encode(words, chunk_values, stream_values, lengths), lengths


def blob_values(blob) -> int:
    b = np.ascontiguousarray(blob, np.uint8)
    return int(lib().zo_blob_values(_p(b, ctypes.c_uint8), b.size))


def decode(blob) -> np.ndarray:
    b = np.ascontiguousarray(blob, np.uint8)
    n = blob_values(b)
    out = np.zeros(n, np.uint16)
    rc = lib().zo_decode(_p(b, ctypes.c_uint8), b.size, _p(out, ctypes.c_uint16), n)
    if rc != OK:
        raise OracleError(rc)
    return out


def decode_chunks(blob, c0: int, c1: int, out: np.ndarray) -> None:
    """Decode chunks [c0, c1) into ``out`` (a uint16 array of the whole tensor's length)."""
    b = np.ascontiguousarray(blob, np.uint8)
    assert out.dtype == np.uint16 and out.flags.c_contiguous and out.size >= blob_values(b)
    rc = lib().zo_decode_chunks(_p(b, ctypes.c_uint8), b.size, c0, c1, _p(out, ctypes.c_uint16))
    if rc != OK:
        raise OracleError(rc)


def check_table(blob) -> int:
    b = np.ascontiguousarray(blob, np.uint8)
    return int(lib().zo_check_table(_p(b, ctypes.c_uint8), b.size))


def header(blob) -> dict:
    """The header fields of a serialised tensor, read with numpy only."""
    b = np.ascontiguousarray(blob, np.uint8)
    u32 = lambda o: int(b[o:o + 4].view("<u4")[0])
    u64 = lambda o: int(b[o:o + 8].view("<u8")[0])
    return dict(magic=u32(0), version=u32(4), n_values=u64(8), chunk_values=u32(16), stream_values=u32(20),
                n_chunks=u32(24), L=u32(28), quantum=u32(32), n_present=u32(36), pad_symbol=u32(40), table_stride=u32(44),
                len_offset=u64(48), lut_offset=u64(56), table_offset=u64(64), sm_offset=u64(72),
                e_offset=u64(80), blob_size=u64(88))
