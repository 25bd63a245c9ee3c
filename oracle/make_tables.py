"""Train the workloads' merge tables and size the token-targeted workloads.

Run as ``python -m oracle.make_tables`` from the repository root.  Calls only
the CPU oracle and the ``workloads`` input generators; writes
``workloads/tables/<table>.merges.i32`` (little-endian int32 [n, 2], row k =
pair of rank k, merged id 256 + k) and ``workloads/manifest.json`` (table
hashes; for the workloads defined by a token count, the number of generator
units per sequence such that the oracle's token count is the largest one not
above the target).
"""
from __future__ import annotations

import json
import os
import sys
import time

import numpy as np

import oracle
from workloads import configs as C
from workloads import textgen


def _tokens_per_piece(table: oracle.Table, data: np.ndarray) -> np.ndarray:
    off = textgen.pretokenize(data)
    _, out_off = oracle.encode(table, data, off, n_threads=os.cpu_count() or 1)
    return np.diff(out_off).astype(np.int64)


def main() -> int:
    os.makedirs(C.TABLE_DIR, exist_ok=True)
    man = {"tables": {}, "evals": {}}
    tables = {}
    for name, spec in C.TABLES.items():
        t0 = time.time()
        corpus = C.make_train_corpus(name)
        merges = oracle.train(corpus, textgen.pretokenize(corpus), spec["n_merges"])
        merges.astype("<i4").tofile(C.table_path(name))
        man["tables"][name] = {
            "n_merges": int(merges.shape[0]),
            "sha256": C.sha256(merges),
            "train_corpus_sha256": C.sha256(corpus),
            "train_corpus_bytes": int(corpus.size),
        }
        tables[name] = oracle.Table(merges)
        print(f"{name}: {merges.shape[0]} merges in {time.time() - t0:.1f}s", flush=True)

    for name in C.CONFIG_ORDER:
        cfg = C.CONFIGS[name]
        table = tables[cfg["table"]]
        if "target_tokens" in cfg:
            targets = np.array([cfg["target_tokens"]], dtype=np.int64)
        elif "n_seqs" in cfg:
            targets = C.batch_target_tokens(cfg)
        else:
            continue
        # text units are exactly pieces (one space each, at the front)
        surplus = int(targets.sum()) + 4096
        data = C.eval_stream(name, n_units=surplus)
        tpp = _tokens_per_piece(table, data)
        assert tpp.size == surplus
        cum = np.concatenate([[0], np.cumsum(tpp)])
        seq_units, seq_tokens, at = [], [], 0
        for t in targets:
            end = int(np.searchsorted(cum, cum[at] + t, side="right")) - 1
            seq_units.append(end - at)
            seq_tokens.append(int(cum[end] - cum[at]))
            at = end
        man["evals"][name] = {"seq_units": seq_units, "seq_tokens": seq_tokens,
                              "n_tokens": int(sum(seq_tokens))}
        print(f"{name}: {len(seq_units)} sequence(s), {sum(seq_units)} pieces, "
              f"{sum(seq_tokens)} tokens", flush=True)

    with open(C.MANIFEST_PATH, "w") as f:
        json.dump(man, f, indent=1)
        f.write("\n")
    # record the content of every workload so that runs are comparable
    for name in C.CONFIG_ORDER:
        ev = C.make_eval(name)
        man["evals"].setdefault(name, {})
        man["evals"][name]["n_bytes"] = int(ev["bytes"].size)
        man["evals"][name]["n_pieces"] = int(ev["piece_offsets"].size - 1)
        man["evals"][name]["bytes_sha256"] = C.sha256(ev["bytes"])
    with open(C.MANIFEST_PATH, "w") as f:
        json.dump(man, f, indent=1)
        f.write("\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
