"""CPU oracle for the byte-level BPE merge loop (encoder, decoder, trainer).

TEST INFRASTRUCTURE ONLY.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the HIP library
and its Python binding never do, and share no code with it.

The arithmetic lives in ``bpe_oracle.c`` (plain C) and ``bpe_trainer.cpp``;
this module only compiles them with gcc/g++ and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "_build", "liboracle.so")
_SOURCES = [os.path.join(_HERE, "bpe_oracle.c"), os.path.join(_HERE, "bpe_trainer.cpp")]
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with the host compilers (no GPU code involved)."""
    os.makedirs(os.path.dirname(_LIB_PATH), exist_ok=True)
    stale = force or not os.path.exists(_LIB_PATH) or any(
        os.path.getmtime(s) > os.path.getmtime(_LIB_PATH) for s in _SOURCES)
    if stale:
        bdir = os.path.dirname(_LIB_PATH)
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-Wall", "-c", _SOURCES[0],
                               "-o", os.path.join(bdir, "bpe_oracle.o")])
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fPIC", "-Wall", "-c", _SOURCES[1],
                               "-o", os.path.join(bdir, "bpe_trainer.o")])
        subprocess.check_call(["g++", "-shared", "-o", _LIB_PATH,
                               os.path.join(bdir, "bpe_oracle.o"),
                               os.path.join(bdir, "bpe_trainer.o"), "-lpthread"])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        lib.oracle_table_create.restype = vp
        lib.oracle_table_create.argtypes = [vp, vp, vp, i64]
        lib.oracle_table_free.argtypes = [vp]
        lib.oracle_lookup.restype = i32
        lib.oracle_lookup.argtypes = [vp, i32, i32, vp, vp]
        lib.oracle_encode.restype = i64
        lib.oracle_encode.argtypes = [vp, vp, vp, i64, vp, vp, i32]
        lib.oracle_decode.restype = i64
        lib.oracle_decode.argtypes = [vp, vp, i64, vp, i64]
        lib.oracle_token_byte_offsets.restype = i64
        lib.oracle_token_byte_offsets.argtypes = [vp, vp, i64, vp]
        lib.oracle_pretokenize.restype = i64
        lib.oracle_pretokenize.argtypes = [vp, i64, vp, i64, vp, vp]
        lib.oracle_train.restype = i64
        lib.oracle_train.argtypes = [vp, vp, i64, i64, vp]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


class Table:
    """Merge table: row k of ``merges`` is (left id, right id); its rank is
    ``ranks[k]`` (default k) and its merged id ``merged_ids[k]`` (default 256 + rank)."""

    def __init__(self, merges, ranks=None, merged_ids=None):
        self.merges = np.ascontiguousarray(np.asarray(merges, dtype=np.int32).reshape(-1, 2))
        n = self.merges.shape[0]
        self.ranks = np.ascontiguousarray(
            np.arange(n, dtype=np.int32) if ranks is None else np.asarray(ranks, dtype=np.int32))
        self.merged_ids = None if merged_ids is None else np.ascontiguousarray(
            np.asarray(merged_ids, dtype=np.int32))
        self._h = _load().oracle_table_create(
            _ptr(self.merges), _ptr(self.ranks),
            None if self.merged_ids is None else _ptr(self.merged_ids), n)

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.oracle_table_free(self._h)
            self._h = None

    def lookup(self, a: int, b: int):
        """(rank, merged id) of pair (a, b), or None."""
        r, m = ctypes.c_int32(), ctypes.c_int32()
        ok = _load().oracle_lookup(self._h, int(a), int(b), ctypes.byref(r), ctypes.byref(m))
        return (r.value, m.value) if ok else None


def encode(table: Table, data, piece_offsets, n_threads: int = 1):
    """Greedy BPE of every piece ``data[off[p]:off[p+1]]``.  Returns
    (ids int32[total], out_offsets int32[n_pieces+1])."""
    data = np.ascontiguousarray(np.asarray(data, dtype=np.uint8))
    off = np.ascontiguousarray(np.asarray(piece_offsets, dtype=np.int32))
    n_pieces = off.size - 1
    assert n_pieces >= 0 and off[0] == 0 and off[-1] == data.size and (np.diff(off) >= 0).all()
    ids = np.empty(max(int(data.size), 1), dtype=np.int32)
    out_off = np.zeros(n_pieces + 1, dtype=np.int32)
    total = _load().oracle_encode(table._h, _ptr(data), _ptr(off), n_pieces,
                                  _ptr(ids), _ptr(out_off), int(n_threads))
    return ids[:total].copy(), out_off


def pretokenize(data, seq_offsets=None):
    """Piece boundaries of ``data``: a piece starts at byte 0, at every sequence
    start and at every byte 0x20.  Returns (piece_offsets int32[n_pieces+1],
    seq_first_piece int32[n_seqs+1]); without ``seq_offsets`` the data is one sequence."""
    data = np.ascontiguousarray(np.asarray(data, dtype=np.uint8))
    if seq_offsets is None:
        seq_offsets = [0, data.size]
    seq = np.ascontiguousarray(np.asarray(seq_offsets, dtype=np.int32))
    n_seqs = seq.size - 1
    assert n_seqs >= 0 and seq[0] == 0 and seq[-1] == data.size and (np.diff(seq) >= 0).all()
    off = np.zeros(data.size + 1, dtype=np.int32)
    first = np.zeros(n_seqs + 1, dtype=np.int32)
    n_pieces = _load().oracle_pretokenize(_ptr(data), data.size, _ptr(seq), n_seqs, _ptr(off), _ptr(first))
    return off[:n_pieces + 1].copy(), first


def encode_raw(table: Table, data, seq_offsets=None, n_threads: int = 1):
    """Pre-tokenize, then encode every piece.  Returns (ids, seq_token_offsets
    int32[n_seqs+1], piece_offsets, out_offsets): sequence k owns
    ids[seq_token_offsets[k]:seq_token_offsets[k+1]]."""
    off, first = pretokenize(data, seq_offsets)
    ids, out_off = encode(table, data, off, n_threads=n_threads)
    return ids, out_off[first].copy(), off, out_off


def decode(table: Table, ids) -> np.ndarray:
    """Bytes the token ids expand to (merged ids replaced by their parts, recursively)."""
    ids = np.ascontiguousarray(np.asarray(ids, dtype=np.int32))
    n = _load().oracle_decode(table._h, _ptr(ids), ids.size, None, 0)
    if n < 0:
        raise ValueError("unknown token id")
    out = np.empty(max(n, 1), dtype=np.uint8)
    _load().oracle_decode(table._h, _ptr(ids), ids.size, _ptr(out), n)
    return out[:n]


def token_byte_offsets(table: Table, ids) -> np.ndarray:
    """int64 [n + 1]: where the bytes of every token start in ``decode(table, ids)``; last = total."""
    ids = np.ascontiguousarray(np.asarray(ids, dtype=np.int32))
    out = np.zeros(ids.size + 1, dtype=np.int64)
    if _load().oracle_token_byte_offsets(table._h, _ptr(ids), ids.size, _ptr(out)) < 0:
        raise ValueError("unknown token id")
    return out


def map_ids(ids, output_ids, to_output_ids: bool = True) -> np.ndarray:
    """Renumber token ids with the table ``output_ids[id]`` of a vocabulary, or
    back (``to_output_ids=False``); -1 for a value the table does not know."""
    ids = np.asarray(ids, dtype=np.int64)
    output_ids = np.asarray(output_ids, dtype=np.int64)
    out = np.full(ids.shape, -1, dtype=np.int32)
    if to_output_ids:
        for i, v in enumerate(ids):
            if 0 <= v < output_ids.size:
                out[i] = output_ids[v]
    else:
        back = {int(o): k for k, o in enumerate(output_ids)}
        for i, v in enumerate(ids):
            out[i] = back.get(int(v), -1)
    return out


def train(data, piece_offsets, n_merges: int) -> np.ndarray:
    """Learn up to ``n_merges`` merges; returns int32 [n, 2], row k = pair of rank k."""
    data = np.ascontiguousarray(np.asarray(data, dtype=np.uint8))
    off = np.ascontiguousarray(np.asarray(piece_offsets, dtype=np.int32))
    out = np.zeros((max(n_merges, 1), 2), dtype=np.int32)
    n = _load().oracle_train(_ptr(data), _ptr(off), off.size - 1, int(n_merges), _ptr(out))
    return out[:n].copy()
