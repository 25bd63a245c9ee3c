"""Pins for the CPU oracle's decoder, its token byte offsets and the id
renumbering: hand-worked fixtures, an independent Python expansion, closed
forms, and library routines (cumsum, permutation inverse)."""
import os

import numpy as np
import pytest

from helpers import expand_ids

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "decode_examples.txt")


def _examples():
    cases = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        rules, syms, text, offs = [x.strip() for x in line.split("|")]
        ids, merges = {}, []
        tr = lambda c: ids.get(c, ord(" ") if c == "_" else ord(c))
        for k, rule in enumerate(r.strip() for r in rules.split(",")):
            lhs, name = rule.split("=")
            l, r = lhs.split()
            merges.append((tr(l), tr(r)))
            ids[name] = 256 + k
        toks = [] if syms == "-" else [tr(c) for c in syms.split()]
        want = b"" if text == "-" else text.replace("_", " ").encode()
        cases.append((merges, toks, want, [int(x) for x in offs.split()]))
    return cases


@pytest.mark.parametrize("merges,toks,want,offs", _examples())
def test_worked_examples(oracle_mod, merges, toks, want, offs):
    table = oracle_mod.Table(merges)
    assert oracle_mod.decode(table, toks).tobytes() == want
    assert oracle_mod.token_byte_offsets(table, toks).tolist() == offs


def test_examples_file_is_not_trivial():
    assert len(_examples()) >= 10


def _random_table(rng, n_merges):
    merges = []
    for k in range(n_merges):
        pool = 256 + k
        merges.append((int(rng.integers(0, pool)), int(rng.integers(0, pool))))
    return merges


def test_against_python_expansion(oracle_mod):
    rng = np.random.default_rng(17)
    for trial in range(40):
        n_merges = int(rng.integers(1, 60))
        merges = _random_table(rng, n_merges)
        # ranks are row numbers here; pairs may repeat, which the decoder does not care about
        table = oracle_mod.Table(merges)
        ids = rng.integers(0, 256 + n_merges, size=int(rng.integers(0, 50)))
        want = expand_ids(ids, merges)
        assert oracle_mod.decode(table, ids).tobytes() == want
        lens = [len(expand_ids([t], merges)) for t in ids]
        assert oracle_mod.token_byte_offsets(table, ids).tolist() == np.concatenate([[0], np.cumsum(lens)]).tolist()


def test_doubling_rules_closed_form(oracle_mod):
    # (x,x)->X1, (X1,X1)->X2, ...: token Xk is 2^k copies of x
    merges = [(120, 120)] + [(256 + k, 256 + k) for k in range(11)]
    table = oracle_mod.Table(merges)
    for k in range(12):
        assert oracle_mod.decode(table, [256 + k]).tobytes() == b"x" * (2 ** (k + 1))
    ids = [256 + 11, 120, 256 + 3]
    assert oracle_mod.token_byte_offsets(table, ids).tolist() == [0, 4096, 4097, 4113]


def test_custom_ids_and_unknown_ids(oracle_mod):
    table = oracle_mod.Table([(97, 98), (1000, 99)], ranks=[5, 9], merged_ids=[1000, 70000])
    assert oracle_mod.decode(table, [70000, 1000, 97]).tobytes() == b"abcaba"
    for bad in (256, 999, 1001, 70001, -1):
        with pytest.raises(ValueError):
            oracle_mod.decode(table, [97, bad])
        with pytest.raises(ValueError):
            oracle_mod.token_byte_offsets(table, [bad])


def test_round_trip_on_a_workload(oracle_mod):
    from workloads import configs as C
    ev = C.make_eval("tiny")
    merges = C.load_merges(ev["table"])
    table = oracle_mod.Table(merges)
    ids, out_off = oracle_mod.encode(table, ev["bytes"], ev["piece_offsets"])
    assert oracle_mod.decode(table, ids).tobytes() == ev["bytes"].tobytes()
    # a piece's tokens decode to the piece: token byte offsets at piece starts are the piece offsets
    tbo = oracle_mod.token_byte_offsets(table, ids)
    assert np.array_equal(tbo[out_off], ev["piece_offsets"])


def test_map_ids(oracle_mod):
    # hand example: bytes renumbered like a vocabulary file that lists '!' first
    output_ids = np.arange(300, dtype=np.int32)
    output_ids[0x21], output_ids[0] = 0, 0x21
    assert oracle_mod.map_ids([0x21, 0x22, 0, 299], output_ids).tolist() == [0, 0x22, 0x21, 299]
    assert oracle_mod.map_ids([0, 0x21, 299, 300, -1], output_ids, to_output_ids=False).tolist() == [0x21, 0, 299, -1, -1]
    assert oracle_mod.map_ids([300, -1], output_ids).tolist() == [-1, -1]
    # a random permutation: numpy's fancy indexing and argsort are the independent routines
    rng = np.random.default_rng(3)
    perm = rng.permutation(5000).astype(np.int32)
    ids = rng.integers(0, 5000, size=2000)
    assert np.array_equal(oracle_mod.map_ids(ids, perm), perm[ids])
    assert np.array_equal(oracle_mod.map_ids(perm[ids], perm, to_output_ids=False), ids)
    assert np.array_equal(oracle_mod.map_ids(ids, perm, to_output_ids=False), np.argsort(perm)[ids])
