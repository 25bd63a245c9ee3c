"""Pins for the CPU oracle's encoder: everything here is independent of the
oracle's own code (hand-worked fixtures, Python brute force, closed forms,
library routines, invariants)."""
import os

import numpy as np
import pytest

from helpers import brute_min_everywhere, brute_rank_order, expand_ids

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_examples.txt")


def _parse_examples():
    cases = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        text, rules, want = [x.strip() for x in line.split("|")]
        ids, merges = {}, []
        for k, rule in enumerate(r.strip() for r in rules.split(",")):
            lhs, name = rule.split("=")
            l, r = lhs.split()
            merges.append((ids.get(l, ord(l)), ids.get(r, ord(r))))
            ids[name] = 256 + k
        data = b"" if text == "-" else text.encode()
        expect = [] if want == "-" else [ids.get(s, ord(s)) for s in want.split()]
        cases.append((data, merges, expect))
    return cases


def _enc(oracle, table, data, off=None):
    data = np.frombuffer(bytes(data), dtype=np.uint8)
    off = [0, data.size] if off is None else off
    ids, out_off = oracle.encode(table, data, off)
    return [int(x) for x in ids], [int(x) for x in out_off]


@pytest.mark.parametrize("data,merges,expect", _parse_examples())
def test_worked_examples(oracle_mod, data, merges, expect):
    table = oracle_mod.Table(merges if merges else np.zeros((0, 2)))
    ids, off = _enc(oracle_mod, table, data)
    assert ids == expect
    assert off == [0, len(expect)]


def test_examples_file_is_not_trivial():
    assert len(_parse_examples()) >= 15


def _random_p1_table(rng, n_alpha, n_merges):
    """Random table with property P1: parts of rule k are bytes or ids made by rules < k."""
    alpha = [ord("a") + i for i in range(n_alpha)]
    merges, seen = [], set()
    while len(merges) < n_merges:
        pool = alpha + [256 + j for j in range(len(merges))]
        p = (int(rng.choice(pool)), int(rng.choice(pool)))
        if p not in seen:
            seen.add(p)
            merges.append(p)
    return alpha, merges


def test_against_brute_force_random_tables(oracle_mod):
    rng = np.random.default_rng(1234)
    n_checked = 0
    for trial in range(300):
        alpha, merges = _random_p1_table(rng, int(rng.integers(2, 5)), int(rng.integers(1, 12)))
        table = oracle_mod.Table(merges)
        pieces = [bytes(rng.choice(alpha, size=int(rng.integers(0, 14))).astype(np.uint8).tolist())
                  for _ in range(20)]
        data = b"".join(pieces)
        off = np.concatenate([[0], np.cumsum([len(p) for p in pieces])])
        ids, out_off = _enc(oracle_mod, table, data, off)
        for p, piece in enumerate(pieces):
            got = ids[out_off[p]:out_off[p + 1]]
            assert got == brute_min_everywhere(piece, merges)
            assert got == brute_rank_order(piece, merges)
            n_checked += 1
    assert n_checked == 6000


def test_against_brute_force_trained_tables(oracle_mod):
    """Tables from the trainer on tiny corpora over a 3-4 letter alphabet."""
    rng = np.random.default_rng(99)
    for trial in range(40):
        alpha = [ord("a") + i for i in range(int(rng.integers(3, 5)))]
        words = [bytes(rng.choice(alpha, size=int(rng.integers(1, 9))).astype(np.uint8).tolist())
                 for _ in range(12)]
        corpus = [words[int(i)] for i in rng.integers(0, len(words), size=200)]
        data = np.frombuffer(b"".join(corpus), dtype=np.uint8)
        off = np.concatenate([[0], np.cumsum([len(w) for w in corpus])]).astype(np.int32)
        merges = [tuple(int(x) for x in m) for m in oracle_mod.train(data, off, 15)]
        table = oracle_mod.Table(merges)
        tests = [bytes(rng.choice(alpha, size=int(rng.integers(0, 16))).astype(np.uint8).tolist())
                 for _ in range(50)]
        tdata = b"".join(tests)
        toff = np.concatenate([[0], np.cumsum([len(t) for t in tests])])
        ids, out_off = _enc(oracle_mod, table, tdata, toff)
        for p, piece in enumerate(tests):
            assert ids[out_off[p]:out_off[p + 1]] == brute_min_everywhere(piece, merges)


def test_empty_table_is_identity(oracle_mod):
    table = oracle_mod.Table(np.zeros((0, 2), dtype=np.int32))
    data = bytes(range(256)) * 2
    ids, off = _enc(oracle_mod, table, data, [0, 100, 100, 512])
    assert ids == list(data) and off == [0, 100, 100, 512]


@pytest.mark.parametrize("levels", [1, 3, 13])
def test_run_is_binary_expansion(oracle_mod, levels):
    """Rules (x,x)->X1, (X1,X1)->X2, ...: a run of L copies of x becomes the binary
    expansion of L, largest power first; the top level repeats when 2**levels <= L."""
    x = ord("q")
    merges = [(x, x)] + [(256 + k, 256 + k) for k in range(levels - 1)]
    table = oracle_mod.Table(merges)
    for L in list(range(0, 70)) + [255, 256, 1000, 4096, 4097]:
        ids, _ = _enc(oracle_mod, table, bytes([x]) * L)
        want = [256 + levels - 1] * (L >> levels)
        for bit in range(levels - 1, -1, -1):
            if (L >> bit) & 1:
                want.append(x if bit == 0 else 256 + bit - 1)
        assert ids == want, L


def test_single_rule_equals_bytes_replace(oracle_mod):
    """With one rule the result is Python's non-overlapping left-to-right replace."""
    rng = np.random.default_rng(7)
    for a, b in [(ord("a"), ord("a")), (ord("a"), ord("b")), (ord("b"), ord("a"))]:
        table = oracle_mod.Table([(a, b)])
        for _ in range(200):
            data = bytes(rng.choice([ord("a"), ord("b")], size=int(rng.integers(0, 40))).astype(np.uint8).tolist())
            ids, _ = _enc(oracle_mod, table, data)
            want = list(data.replace(bytes([a, b]), b"\xff"))   # 0xff never occurs in data
            assert [255 if t == 256 else t for t in ids] == want


def test_pieces_are_independent_and_offsets_run(oracle_mod):
    merges = [(ord("a"), ord("b")), (ord("b"), ord("a"))]
    table = oracle_mod.Table(merges)
    # "abab" cut into "a", "", "ba", "b": nothing merges across a cut, so the
    # rank-0 pair (a,b) never forms and only (b,a) inside the third piece merges
    ids, off = _enc(oracle_mod, table, b"abab", [0, 1, 1, 3, 4])
    assert (ids, off) == ([ord("a"), 257, ord("b")], [0, 1, 1, 2, 3])
    # uncut, the rank-0 pair wins twice
    ids, off = _enc(oracle_mod, table, b"abab")
    assert (ids, off) == ([256, 256], [0, 2])


def test_threads_do_not_change_the_result(oracle_mod):
    from workloads import configs as C
    ev = C.make_eval("tiny")
    table = oracle_mod.Table(C.load_merges("t1k"))
    a = oracle_mod.encode(table, ev["bytes"], ev["piece_offsets"], n_threads=1)
    b = oracle_mod.encode(table, ev["bytes"], ev["piece_offsets"], n_threads=5)
    assert (a[0] == b[0]).all() and (a[1] == b[1]).all()


def test_custom_ranks_and_merged_ids(oracle_mod):
    # rules listed out of rank order with explicit ids
    merges = [(ord("a"), ord("b")), (ord("b"), ord("c"))]
    table = oracle_mod.Table(merges, ranks=[1, 0], merged_ids=[1000, 2000])
    ids, _ = _enc(oracle_mod, table, b"abc")
    assert ids == [ord("a"), 2000]
    assert table.lookup(ord("a"), ord("b")) == (1, 1000)
    assert table.lookup(ord("b"), ord("a")) is None


@pytest.mark.parametrize("name", ["tiny", "seq32k"])
def test_invariants_on_workloads(oracle_mod, name):
    from workloads import configs as C
    ev = C.make_eval(name)
    merges = C.load_merges(ev["table"])
    table = oracle_mod.Table(merges)
    data, off = ev["bytes"], ev["piece_offsets"]
    ids, out_off = oracle_mod.encode(table, data, off, n_threads=4)
    rank = {(int(a), int(b)): k for k, (a, b) in enumerate(merges)}
    assert out_off[0] == 0 and out_off[-1] == ids.size
    assert ids.min() >= 0 and ids.max() < 256 + len(merges)
    # round trip, independently of the oracle's own decoder
    assert expand_ids(ids, merges) == data.tobytes()
    assert oracle_mod.decode(table, ids).tobytes() == data.tobytes()
    seen = {}
    for p in range(off.size - 1):
        toks = ids[out_off[p]:out_off[p + 1]]
        piece = data[off[p]:off[p + 1]].tobytes()
        assert len(toks) <= len(piece)
        # tokens of a piece spell exactly that piece (no token spans a boundary)
        if p % 37 == 0:
            assert expand_ids(toks, merges) == piece
        # no mergeable pair is left inside a piece
        for i in range(len(toks) - 1):
            assert (int(toks[i]), int(toks[i + 1])) not in rank
        # identical pieces encode identically
        key = tuple(int(t) for t in toks)
        assert seen.setdefault(piece, key) == key
