"""ctypes binding of libbpe_mi355x.so: argument marshalling only.

Function names follow include/bpe_mi355x.h.  Device buffers are torch tensors
on the GPU (torch supplies memory and streams, nothing else); every step of
the path runs in the library's kernels.  There is no CPU fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "lib", "libbpe_mi355x.so")
_lib = None

EXPORTS = [
    "bpe_last_error", "bpe_table_capacity", "bpe_table_image_build", "bpe_table_build",
    "bpe_table_free", "bpe_table_info", "bpe_table_lookup", "bpe_workspace_bytes", "bpe_dedup_workspace_bytes", "bpe_encode", "bpe_encode_static",
    "bpe_encode_timed", "bpe_encode_plan", "bpe_encode_raw_plan", "bpe_encode_status", "bpe_status_from_words", "bpe_pool_create", "bpe_pool_destroy", "bpe_pool_workspace",
    "bpe_pretokenize_workspace_bytes", "bpe_pretokenize", "bpe_encode_raw_workspace_bytes", "bpe_encode_raw",
    "bpe_encode_raw_timed", "bpe_vocab_build", "bpe_vocab_free", "bpe_vocab_info", "bpe_map_ids",
    "bpe_decode_workspace_bytes", "bpe_decode",
]


class BpeError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"bpe_mi355x error {code}: {message}")
        self.code = code


class _TableInfo(ctypes.Structure):
    _fields_ = [("n_merges", ctypes.c_int64), ("capacity", ctypes.c_int64),
                ("device_bytes", ctypes.c_int64), ("hash_attempt", ctypes.c_int32),
                ("max_id", ctypes.c_int32)]


class _VocabInfo(ctypes.Structure):
    _fields_ = [("n_ids", ctypes.c_int64), ("n_output_ids", ctypes.c_int64), ("pool_bytes", ctypes.c_int64),
                ("device_bytes", ctypes.c_int64), ("max_token_bytes", ctypes.c_int32),
                ("has_output_ids", ctypes.c_int32)]


class _PlanLaunch(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_char * 32), ("grid", ctypes.c_int64), ("block", ctypes.c_int32),
                ("interval", ctypes.c_int32)]


class _Plan(ctypes.Structure):
    _fields_ = [("n_launches", ctypes.c_int32), ("single_kernel", ctypes.c_int32),
                ("selection_level", ctypes.c_int32), ("pieces_per_wave", ctypes.c_int32),
                ("waves_per_tile", ctypes.c_int32), ("reserved", ctypes.c_int32), ("n_tiles", ctypes.c_int64),
                ("launch", _PlanLaunch * 8)]


class _Options(ctypes.Structure):
    _fields_ = [("selection_level", ctypes.c_int32), ("pieces_per_wave", ctypes.c_int32),
                ("tiny_max_len", ctypes.c_int32), ("wave_max_len", ctypes.c_int32),
                ("wave_lds_max_len", ctypes.c_int32), ("lds_max_len", ctypes.c_int32),
                ("fused", ctypes.c_int32), ("pretokenize_tile_kib", ctypes.c_int32),
                ("paper_kernel", ctypes.c_int32), ("column_max_len", ctypes.c_int32),
                ("dedup", ctypes.c_int32), ("long_groups", ctypes.c_int32)]


@dataclass
class EncodeOptions:
    selection_level: int = 0
    pieces_per_wave: int = 0
    tiny_max_len: int = 0
    wave_max_len: int = 0
    wave_lds_max_len: int = 0
    lds_max_len: int = 0
    fused: int = 0
    pretokenize_tile_kib: int = 0
    paper_kernel: int = 0
    column_max_len: int = 0
    dedup: int = 0
    long_groups: int = 0

    def _c(self):
        return _Options(self.selection_level, self.pieces_per_wave, self.tiny_max_len,
                        self.wave_max_len, self.wave_lds_max_len, self.lds_max_len, self.fused,
                        self.pretokenize_tile_kib, self.paper_kernel, self.column_max_len, self.dedup, self.long_groups)


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the built library; build it first if it was never built or was built from
    other sources than the ones that are there now (a hash of the sources travels with it)."""
    global _lib
    if _lib is not None:
        return _lib
    from .build import build_library, library_is_current
    if not library_is_current():
        build_library()
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    lib.bpe_last_error.restype = ctypes.c_char_p
    lib.bpe_table_capacity.restype = i64
    lib.bpe_table_capacity.argtypes = [i64]
    lib.bpe_table_image_build.restype = i32
    lib.bpe_table_image_build.argtypes = [vp, vp, vp, i64, vp, i64, ctypes.POINTER(_TableInfo)]
    lib.bpe_table_build.restype = i32
    lib.bpe_table_build.argtypes = [vp, vp, vp, i64, ctypes.POINTER(vp)]
    lib.bpe_table_free.restype = i32
    lib.bpe_table_free.argtypes = [vp]
    lib.bpe_table_info.restype = i32
    lib.bpe_table_info.argtypes = [vp, ctypes.POINTER(_TableInfo)]
    lib.bpe_table_lookup.restype = i32
    lib.bpe_table_lookup.argtypes = [vp, vp, i64, vp, vp, vp]
    lib.bpe_workspace_bytes.restype = i64
    lib.bpe_workspace_bytes.argtypes = [i64, i64]
    lib.bpe_dedup_workspace_bytes.restype = i64
    lib.bpe_dedup_workspace_bytes.argtypes = [i64, i64]
    lib.bpe_encode.restype = i32
    lib.bpe_encode.argtypes = [vp, vp, vp, i64, i64, vp, vp, vp, i64, ctypes.POINTER(_Options), vp]
    lib.bpe_encode_static.restype = i32
    lib.bpe_encode_static.argtypes = [vp, vp, vp, i64, i64, vp, vp, ctypes.POINTER(_Options), vp]
    lib.bpe_encode_timed.restype = i32
    lib.bpe_encode_timed.argtypes = lib.bpe_encode.argtypes + [vp]
    lib.bpe_encode_plan.restype = i32
    lib.bpe_encode_plan.argtypes = [i64, i64, ctypes.POINTER(_Options), ctypes.POINTER(_Plan)]
    lib.bpe_encode_raw_plan.restype = i32
    lib.bpe_encode_raw_plan.argtypes = [i64, i64, i64, i32, i32, ctypes.POINTER(_Options), ctypes.POINTER(_Plan)]
    lib.bpe_status_from_words.restype = i32
    lib.bpe_status_from_words.argtypes = [vp]
    lib.bpe_encode_status.restype = i32
    lib.bpe_encode_status.argtypes = [vp, vp]
    lib.bpe_pretokenize_workspace_bytes.restype = i64
    lib.bpe_pretokenize_workspace_bytes.argtypes = [i64]
    lib.bpe_pretokenize.restype = i32
    lib.bpe_pretokenize.argtypes = [vp, i64, vp, i64, vp, i64, vp, vp, vp, i64, ctypes.POINTER(_Options), vp]
    lib.bpe_encode_raw_workspace_bytes.restype = i64
    lib.bpe_encode_raw_workspace_bytes.argtypes = [i64, i64, i64]
    lib.bpe_encode_raw.restype = i32
    lib.bpe_encode_raw.argtypes = [vp, vp, i64, vp, i64, i64, vp, vp, vp, vp, vp, vp, i64,
                                   ctypes.POINTER(_Options), vp]
    lib.bpe_encode_raw_timed.restype = i32
    lib.bpe_encode_raw_timed.argtypes = lib.bpe_encode_raw.argtypes + [vp]
    lib.bpe_vocab_build.restype = i32
    lib.bpe_vocab_build.argtypes = [vp, vp, vp, i64, vp, i64, ctypes.POINTER(vp)]
    lib.bpe_vocab_free.restype = i32
    lib.bpe_vocab_free.argtypes = [vp]
    lib.bpe_vocab_info.restype = i32
    lib.bpe_vocab_info.argtypes = [vp, ctypes.POINTER(_VocabInfo)]
    lib.bpe_map_ids.restype = i32
    lib.bpe_map_ids.argtypes = [vp, vp, vp, i64, vp, i32, vp]
    lib.bpe_decode_workspace_bytes.restype = i64
    lib.bpe_decode_workspace_bytes.argtypes = [i64]
    lib.bpe_decode.restype = i32
    lib.bpe_decode.argtypes = [vp, vp, i64, vp, i32, vp, i64, vp, vp, vp, i64, vp]
    lib.bpe_pool_create.restype = i32
    lib.bpe_pool_create.argtypes = [i64, i64, ctypes.POINTER(vp)]
    lib.bpe_pool_destroy.restype = i32
    lib.bpe_pool_destroy.argtypes = [vp]
    lib.bpe_pool_workspace.restype = i32
    lib.bpe_pool_workspace.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(i64)]
    _lib = lib
    return lib


def _check(rc: int):
    if rc < 0:
        raise BpeError(rc, load_library().bpe_last_error().decode(errors="replace"))
    return rc


def _host_i32(a, shape=None):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(np.asarray(a, dtype=np.int32))
    if shape is not None:
        arr = arr.reshape(shape)
    return arr, arr.ctypes.data_as(ctypes.c_void_p)


def _dev_ptr(t, dtype_name: str):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or not t.is_contiguous():
        raise TypeError("expected a contiguous torch tensor on the GPU")
    if str(t.dtype) != f"torch.{dtype_name}":
        raise TypeError(f"expected dtype {dtype_name}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def bpe_table_capacity(n_merges: int) -> int:
    return _check(load_library().bpe_table_capacity(int(n_merges)))


def bpe_table_image_build(merges, ranks=None, merged_ids=None):
    """Host-only: validate the rules and return (slots uint64[capacity, 2], info dict)."""
    lib = load_library()
    m, mp = _host_i32(merges, (-1, 2))
    n = m.shape[0]
    _, rp = _host_i32(ranks)
    _, ip = _host_i32(merged_ids)
    cap = bpe_table_capacity(n)
    slots = np.zeros((cap, 2), dtype=np.uint64)
    info = _TableInfo()
    _check(lib.bpe_table_image_build(mp, rp, ip, n, slots.ctypes.data_as(ctypes.c_void_p), cap,
                                     ctypes.byref(info)))
    return slots, {f: getattr(info, f) for f, _ in _TableInfo._fields_}


class Table:
    """Device-resident merge table (owns its device memory)."""

    def __init__(self, merges, ranks=None, merged_ids=None):
        lib = load_library()
        m, mp = _host_i32(merges, (-1, 2))
        _, rp = _host_i32(ranks)
        _, ip = _host_i32(merged_ids)
        h = ctypes.c_void_p()
        _check(lib.bpe_table_build(mp, rp, ip, m.shape[0], ctypes.byref(h)))
        self._h = h
        info = _TableInfo()
        _check(lib.bpe_table_info(self._h, ctypes.byref(info)))
        self.info = {f: getattr(info, f) for f, _ in _TableInfo._fields_}

    def free(self):
        if getattr(self, "_h", None):
            load_library().bpe_table_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def bpe_table_build(merges, ranks=None, merged_ids=None) -> Table:
    return Table(merges, ranks, merged_ids)


def bpe_table_lookup(table: Table, pairs, out_rank, out_merged, stream=None):
    n = pairs.shape[0]
    _check(load_library().bpe_table_lookup(table._h, _dev_ptr(pairs, "int32"), n,
                                           _dev_ptr(out_rank, "int32"), _dev_ptr(out_merged, "int32"),
                                           _stream_ptr(stream)))


def bpe_workspace_bytes(n_bytes: int, n_pieces: int) -> int:
    return _check(load_library().bpe_workspace_bytes(int(n_bytes), int(n_pieces)))


def bpe_dedup_workspace_bytes(n_bytes: int, n_pieces: int) -> int:
    return _check(load_library().bpe_dedup_workspace_bytes(int(n_bytes), int(n_pieces)))


def bpe_encode(table: Table, data, piece_offsets, out_ids, out_offsets, workspace,
               opts: EncodeOptions | None = None, stream=None):
    """Enqueue one encode; all tensors live on the GPU.  Does not synchronise."""
    n_bytes = data.numel()
    n_pieces = piece_offsets.numel() - 1
    if out_offsets.numel() < n_pieces + 1 or out_ids.numel() < n_bytes:
        raise ValueError("output tensors are too small")
    c_opts = ctypes.byref(opts._c()) if opts is not None else None
    _check(load_library().bpe_encode(
        table._h, _dev_ptr(data, "uint8"), _dev_ptr(piece_offsets, "int32"), n_bytes, n_pieces,
        _dev_ptr(out_ids, "int32"), _dev_ptr(out_offsets, "int32"),
        _dev_ptr(workspace, "uint8"), workspace.numel(), c_opts, _stream_ptr(stream)))


STATIC_SCRATCH_BYTES = 16 << 20   # what bpe_encode_static's built-in array holds


def bpe_encode_static(table: Table, data, piece_offsets, out_ids, out_offsets,
                      opts: EncodeOptions | None = None, stream=None):
    """bpe_encode on the library's built-in scratch array: no workspace, no allocation."""
    n_bytes = data.numel()
    n_pieces = piece_offsets.numel() - 1
    if out_offsets.numel() < n_pieces + 1 or out_ids.numel() < n_bytes:
        raise ValueError("output tensors are too small")
    c_opts = ctypes.byref(opts._c()) if opts is not None else None
    _check(load_library().bpe_encode_static(
        table._h, _dev_ptr(data, "uint8"), _dev_ptr(piece_offsets, "int32"), n_bytes, n_pieces,
        _dev_ptr(out_ids, "int32"), _dev_ptr(out_offsets, "int32"), c_opts, _stream_ptr(stream)))


N_TIMED_INTERVALS = 3       # bpe_encode_timed: merge (the whole path in the single kernel), tile scan, emit
N_RAW_TIMED_INTERVALS = 5   # bpe_encode_raw_timed: pre-tokenizer, merge, tile scan, emit, sequence offsets


def _plan_dict(plan: _Plan) -> dict:
    d = {f: getattr(plan, f) for f in ("single_kernel", "selection_level", "pieces_per_wave", "waves_per_tile",
                                        "n_tiles")}
    d["launches"] = [{"kernel": plan.launch[i].kernel.decode(), "grid": plan.launch[i].grid,
                      "block": plan.launch[i].block, "interval": plan.launch[i].interval}
                     for i in range(plan.n_launches)]
    return d


def bpe_encode_plan(n_bytes: int, n_pieces: int, opts: EncodeOptions | None = None) -> dict:
    """What bpe_encode launches for these sizes and options (nothing is launched; no GPU needed)."""
    plan = _Plan()
    c_opts = ctypes.byref(opts._c()) if opts is not None else None
    _check(load_library().bpe_encode_plan(int(n_bytes), int(n_pieces), c_opts, ctypes.byref(plan)))
    return _plan_dict(plan)


def bpe_encode_raw_plan(n_bytes: int, max_pieces: int = 0, n_seqs: int = 1, has_seq_offsets: bool = False,
                        wants_piece_arrays: bool = False, opts: EncodeOptions | None = None) -> dict:
    """What bpe_encode_raw launches for these sizes and options."""
    plan = _Plan()
    c_opts = ctypes.byref(opts._c()) if opts is not None else None
    _check(load_library().bpe_encode_raw_plan(int(n_bytes), int(max_pieces), int(n_seqs), 1 if has_seq_offsets else 0,
                                              1 if wants_piece_arrays else 0, c_opts, ctypes.byref(plan)))
    return _plan_dict(plan)


def kernels_by_interval(plan: dict, n_intervals: int) -> list:
    """Names of the kernels each interval of a *_timed call holds ('' for an interval without a launch)."""
    names = [[] for _ in range(n_intervals)]
    for l in plan["launches"]:
        names[l["interval"]].append(l["kernel"])
    return ["+".join(n) for n in names]


def bpe_encode_timed(table: Table, data, piece_offsets, out_ids, out_offsets, workspace,
                     opts: EncodeOptions | None = None, stream=None):
    """bpe_encode with a HIP event between the kernels; synchronises and returns
    the N_TIMED_INTERVALS kernel durations in ms (bpe_encode_plan names the kernels of each)."""
    n_bytes = data.numel()
    n_pieces = piece_offsets.numel() - 1
    if out_offsets.numel() < n_pieces + 1 or out_ids.numel() < n_bytes:
        raise ValueError("output tensors are too small")
    c_opts = ctypes.byref(opts._c()) if opts is not None else None
    ms = (ctypes.c_float * N_TIMED_INTERVALS)()
    _check(load_library().bpe_encode_timed(
        table._h, _dev_ptr(data, "uint8"), _dev_ptr(piece_offsets, "int32"), n_bytes, n_pieces,
        _dev_ptr(out_ids, "int32"), _dev_ptr(out_offsets, "int32"),
        _dev_ptr(workspace, "uint8"), workspace.numel(), c_opts, _stream_ptr(stream),
        ctypes.cast(ms, ctypes.c_void_p)))
    return list(ms)


def bpe_encode_status(workspace, stream=None) -> int:
    """Synchronise and return the device-side verdict (0 or a negative code); workspace None:
    of the last bpe_encode_static on the current device."""
    return load_library().bpe_encode_status(_opt_ptr(workspace, "uint8"), _stream_ptr(stream))


def _opt_ptr(t, dtype_name: str):
    return None if t is None else _dev_ptr(t, dtype_name)


def bpe_pretokenize_workspace_bytes(n_bytes: int) -> int:
    return _check(load_library().bpe_pretokenize_workspace_bytes(int(n_bytes)))


def bpe_pretokenize(data, seq_offsets, piece_offsets, n_pieces, seq_first_piece, workspace,
                    opts: EncodeOptions | None = None, stream=None):
    """Enqueue the pre-tokenizer; all tensors live on the GPU.  ``seq_offsets``
    and ``seq_first_piece`` may be None.  Does not synchronise."""
    n_seqs = 0 if seq_offsets is None else seq_offsets.numel() - 1
    if seq_first_piece is not None and seq_first_piece.numel() < (2 if seq_offsets is None else n_seqs + 1):
        raise ValueError("seq_first_piece is too small")
    c_opts = ctypes.byref(opts._c()) if opts is not None else None
    _check(load_library().bpe_pretokenize(
        _dev_ptr(data, "uint8"), data.numel(), _opt_ptr(seq_offsets, "int32"), n_seqs,
        _dev_ptr(piece_offsets, "int32"), piece_offsets.numel() - 1, _dev_ptr(n_pieces, "int32"),
        _opt_ptr(seq_first_piece, "int32"), _dev_ptr(workspace, "uint8"), workspace.numel(), c_opts,
        _stream_ptr(stream)))


def bpe_encode_raw_workspace_bytes(n_bytes: int, max_pieces: int = 0, n_seqs: int = 1) -> int:
    return _check(load_library().bpe_encode_raw_workspace_bytes(int(n_bytes), int(max_pieces), int(n_seqs)))


def _raw_args(table, data, seq_offsets, max_pieces, out_ids, seq_token_offsets, piece_offsets, out_offsets,
              n_pieces, workspace, opts, stream):
    n_bytes = data.numel()
    n_seqs = 0 if seq_offsets is None else seq_offsets.numel() - 1
    cap = int(max_pieces) if max_pieces else n_bytes
    if out_ids.numel() < n_bytes or seq_token_offsets.numel() < (2 if seq_offsets is None else n_seqs + 1):
        raise ValueError("output tensors are too small")
    for t in (piece_offsets, out_offsets):
        if t is not None and t.numel() < cap + 1:
            raise ValueError("piece_offsets / out_offsets hold fewer than max_pieces + 1 entries")
    c_opts = ctypes.byref(opts._c()) if opts is not None else None
    return [table._h, _dev_ptr(data, "uint8"), n_bytes, _opt_ptr(seq_offsets, "int32"), n_seqs, cap,
            _dev_ptr(out_ids, "int32"), _dev_ptr(seq_token_offsets, "int32"), _opt_ptr(piece_offsets, "int32"),
            _opt_ptr(out_offsets, "int32"), _opt_ptr(n_pieces, "int32"), _dev_ptr(workspace, "uint8"),
            workspace.numel(), c_opts, _stream_ptr(stream)]


def bpe_encode_raw(table: Table, data, seq_offsets, out_ids, seq_token_offsets, workspace, max_pieces: int = 0,
                   piece_offsets=None, out_offsets=None, n_pieces=None, opts: EncodeOptions | None = None,
                   stream=None):
    """Enqueue pre-tokenizer + encode; all tensors live on the GPU.  Does not synchronise."""
    _check(load_library().bpe_encode_raw(*_raw_args(
        table, data, seq_offsets, max_pieces, out_ids, seq_token_offsets, piece_offsets, out_offsets, n_pieces,
        workspace, opts, stream)))


def bpe_encode_raw_timed(table: Table, data, seq_offsets, out_ids, seq_token_offsets, workspace,
                         max_pieces: int = 0, piece_offsets=None, out_offsets=None, n_pieces=None,
                         opts: EncodeOptions | None = None, stream=None):
    """bpe_encode_raw with a HIP event between the kernels; synchronises and
    returns the N_RAW_TIMED_INTERVALS kernel durations in ms (bpe_encode_raw_plan names the kernels of each)."""
    ms = (ctypes.c_float * N_RAW_TIMED_INTERVALS)()
    _check(load_library().bpe_encode_raw_timed(*_raw_args(
        table, data, seq_offsets, max_pieces, out_ids, seq_token_offsets, piece_offsets, out_offsets, n_pieces,
        workspace, opts, stream), ctypes.cast(ms, ctypes.c_void_p)))
    return list(ms)


class Vocab:
    """Device-resident byte expansions of all token ids, with an optional
    renumbering ``output_ids[id]`` (owns its device memory)."""

    def __init__(self, merges, ranks=None, merged_ids=None, output_ids=None):
        lib = load_library()
        m, mp = _host_i32(merges, (-1, 2))
        _, rp = _host_i32(ranks)
        _, ip = _host_i32(merged_ids)
        o, op = _host_i32(output_ids)
        h = ctypes.c_void_p()
        _check(lib.bpe_vocab_build(mp, rp, ip, m.shape[0], op, 0 if o is None else o.size, ctypes.byref(h)))
        self._h = h
        info = _VocabInfo()
        _check(lib.bpe_vocab_info(self._h, ctypes.byref(info)))
        self.info = {f: getattr(info, f) for f, _ in _VocabInfo._fields_}

    def free(self):
        if getattr(self, "_h", None):
            load_library().bpe_vocab_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def bpe_vocab_build(merges, ranks=None, merged_ids=None, output_ids=None) -> Vocab:
    return Vocab(merges, ranks, merged_ids, output_ids)


def bpe_map_ids(vocab: Vocab, ids_in, ids_out, to_output_ids: bool, n_device=None, stream=None):
    """Enqueue the renumbering of ``ids_in`` into ``ids_out`` (GPU int32 tensors, may be the same)."""
    if ids_out.numel() < ids_in.numel():
        raise ValueError("ids_out is too small")
    _check(load_library().bpe_map_ids(vocab._h, _dev_ptr(ids_in, "int32"), _dev_ptr(ids_out, "int32"),
                                      ids_in.numel(), _opt_ptr(n_device, "int32"), 1 if to_output_ids else 0,
                                      _stream_ptr(stream)))


def bpe_decode_workspace_bytes(n_tokens: int) -> int:
    return _check(load_library().bpe_decode_workspace_bytes(int(n_tokens)))


def bpe_decode(vocab: Vocab, ids, out_bytes, workspace, token_byte_offsets=None, n_bytes=None,
               n_tokens_device=None, ids_are_output_ids: bool = False, stream=None):
    """Enqueue the decoding of ``ids`` into ``out_bytes``; all tensors live on the GPU."""
    n = ids.numel()
    if token_byte_offsets is not None and token_byte_offsets.numel() < n + 1:
        raise ValueError("token_byte_offsets is too small")
    _check(load_library().bpe_decode(
        vocab._h, _dev_ptr(ids, "int32"), n, _opt_ptr(n_tokens_device, "int32"), 1 if ids_are_output_ids else 0,
        _dev_ptr(out_bytes, "uint8"), out_bytes.numel(), _opt_ptr(token_byte_offsets, "int32"),
        _opt_ptr(n_bytes, "int32"), _dev_ptr(workspace, "uint8"), workspace.numel(), _stream_ptr(stream)))


class Pool:
    """Preallocated workspace: one device allocation at creation, none per encode."""

    def __init__(self, max_bytes: int, max_pieces: int):
        lib = load_library()
        h = ctypes.c_void_p()
        _check(lib.bpe_pool_create(int(max_bytes), int(max_pieces), ctypes.byref(h)))
        self._h = h
        ws, nb = ctypes.c_void_p(), ctypes.c_int64()
        _check(lib.bpe_pool_workspace(self._h, ctypes.byref(ws), ctypes.byref(nb)))
        self.ptr, self.nbytes = ws.value, nb.value

    def destroy(self):
        if getattr(self, "_h", None):
            load_library().bpe_pool_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def encode(table: Table, data, piece_offsets, opts: EncodeOptions | None = None, check: bool = True):
    """Convenience wrapper for tests: allocates outputs and workspace with torch,
    runs bpe_encode, synchronises.  Returns (ids[total], out_offsets) as GPU tensors."""
    import torch
    dev = data.device
    n_bytes, n_pieces = data.numel(), piece_offsets.numel() - 1
    out_ids = torch.empty(max(n_bytes, 1), dtype=torch.int32, device=dev)
    out_off = torch.empty(n_pieces + 1, dtype=torch.int32, device=dev)
    need = bpe_dedup_workspace_bytes if opts is not None and opts.dedup else bpe_workspace_bytes
    ws = torch.empty(need(n_bytes, n_pieces), dtype=torch.uint8, device=dev)
    bpe_encode(table, data, piece_offsets, out_ids, out_off, ws, opts)
    st = bpe_encode_status(ws)
    if check and st != 0:
        raise BpeError(st, load_library().bpe_last_error().decode(errors="replace"))
    total = int(out_off[-1].item())
    return out_ids[:total], out_off
