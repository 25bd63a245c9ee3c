"""Registry of the five benchmark workloads and their merge tables.

The merge tables and the unit counts that size the token-targeted workloads
are *stored* values: ``oracle/make_tables.py`` (which calls only the CPU oracle
and this package) writes them to ``workloads/tables/`` and
``workloads/manifest.json``.  Nothing here depends on the HIP path.
"""
from __future__ import annotations

import hashlib
import json
import os

import numpy as np

from . import textgen

_HERE = os.path.dirname(os.path.abspath(__file__))
TABLE_DIR = os.path.join(_HERE, "tables")
MANIFEST_PATH = os.path.join(_HERE, "manifest.json")

# Merge tables: (word-list size, seeds, training-corpus bytes, requested merges, stress mix?)
TABLES = {
    "t1k":   dict(n_words=5_000,  vocab_seed=0x1001, train_seed=0x2001, train_bytes=1_000_000,  n_merges=1_000,   stress=False),
    "t50k":  dict(n_words=30_000, vocab_seed=0x1002, train_seed=0x2002, train_bytes=20_000_000, n_merges=50_000,  stress=False),
    "t100k": dict(n_words=30_000, vocab_seed=0x1002, train_seed=0x2003, train_bytes=20_000_000, n_merges=100_000, stress=True),
}

# Workloads, in the order the benchmark definition lists them.
CONFIGS = {
    "tiny":    dict(table="t1k",   eval_seed=0x3001, max_bytes=4096),
    "seq32k":  dict(table="t50k",  eval_seed=0x3002, target_tokens=32_768),
    "seq131k": dict(table="t50k",  eval_seed=0x3003, target_tokens=131_072),
    "batch":   dict(table="t50k",  eval_seed=0x3004, n_seqs=256, seq_tokens=(1_000, 16_000), len_seed=0x4004),
    "stress":  dict(table="t100k", eval_seed=0x3005, max_bytes=4_000_000),
}
CONFIG_ORDER = ["tiny", "seq32k", "seq131k", "batch", "stress"]


def manifest() -> dict:
    if not os.path.exists(MANIFEST_PATH):
        raise FileNotFoundError(
            f"{MANIFEST_PATH} is missing: run `python -m oracle.make_tables` to train the merge tables")
    with open(MANIFEST_PATH) as f:
        return json.load(f)


def table_path(table: str) -> str:
    return os.path.join(TABLE_DIR, f"{table}.merges.i32")


def load_merges(table: str) -> np.ndarray:
    """int32 [n_merges, 2]; row k is the pair merged at rank k (merged id 256+k)."""
    m = np.fromfile(table_path(table), dtype="<i4").reshape(-1, 2)
    want = manifest()["tables"][table]
    if m.shape[0] != want["n_merges"] or sha256(m) != want["sha256"]:
        raise RuntimeError(f"merge table {table} does not match workloads/manifest.json")
    return m


def sha256(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def make_train_corpus(table: str) -> np.ndarray:
    t = TABLES[table]
    gen = textgen.gen_stress_stream if t["stress"] else textgen.gen_text_stream
    return gen(t["n_words"], t["vocab_seed"], t["train_seed"], max_bytes=t["train_bytes"])


def batch_target_tokens(cfg: dict) -> np.ndarray:
    lo, hi = cfg["seq_tokens"]
    z = textgen.splitmix64(cfg["len_seed"], 0, cfg["n_seqs"])
    return (z % np.uint64(hi - lo + 1)).astype(np.int64) + lo


def eval_stream(name: str, n_units: int | None = None, max_bytes: int | None = None) -> np.ndarray:
    """The evaluation stream of workload ``name``, cut by units or by bytes."""
    cfg = CONFIGS[name]
    t = TABLES[cfg["table"]]
    gen = textgen.gen_stress_stream if t["stress"] else textgen.gen_text_stream
    return gen(t["n_words"], t["vocab_seed"], cfg["eval_seed"], n_units=n_units, max_bytes=max_bytes)


def make_eval(name: str) -> dict:
    """Bytes, piece offsets and sequence layout of workload ``name``.

    Returns dict(bytes u8[n_bytes], piece_offsets i32[n_pieces+1],
    seq_first_piece i64[n_seqs+1], table str)."""
    cfg = CONFIGS[name]
    if "max_bytes" in cfg:
        data = eval_stream(name, max_bytes=cfg["max_bytes"])
        seq_byte_starts = np.array([0], dtype=np.int64)
    else:
        ev = manifest()["evals"][name]
        seq_units = np.asarray(ev["seq_units"], dtype=np.int64)
        data = eval_stream(name, n_units=int(seq_units.sum()))
        # every unit starts with a space, so unit starts are exactly the 0x20 bytes
        unit_starts = np.nonzero(data == 0x20)[0]
        first_unit = np.concatenate([[0], np.cumsum(seq_units)[:-1]])
        seq_byte_starts = unit_starts[first_unit]
    off = textgen.pretokenize(data, seq_byte_starts)
    seq_first_piece = np.concatenate(
        [np.searchsorted(off, seq_byte_starts), [off.size - 1]]).astype(np.int64)
    return dict(bytes=data, piece_offsets=off, seq_first_piece=seq_first_piece, table=cfg["table"])
