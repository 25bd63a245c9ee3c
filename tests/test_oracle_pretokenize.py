"""Pins for the CPU oracle's pre-tokenizer (piece starts: byte 0, sequence
starts, spaces).  Independent of the oracle's code: hand-worked fixtures, the
regex engine's zero-width split, closed forms, invariants, and the numpy
implementation the workload generator uses."""
import os
import re

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "pretokenize_examples.txt")


def _examples():
    cases = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        text, seq, off, first = [x.strip() for x in line.split("|")]
        data = b"" if text == "-" else text.replace("_", " ").encode()
        cases.append((data, [int(x) for x in seq.split()], [int(x) for x in off.split()],
                      [int(x) for x in first.split()]))
    return cases


def _u8(b):
    return np.frombuffer(bytes(b), dtype=np.uint8)


@pytest.mark.parametrize("data,seq,off,first", _examples())
def test_worked_examples(oracle_mod, data, seq, off, first):
    got_off, got_first = oracle_mod.pretokenize(_u8(data), seq)
    assert got_off.tolist() == off
    assert got_first.tolist() == first


def test_examples_file_is_not_trivial():
    assert len(_examples()) >= 10


def _regex_pieces(chunk: bytes):
    """Split before every space with the regex engine (zero-width look-ahead)."""
    return [x for x in re.split(rb"(?= )", chunk) if x]


def _random_text(rng, n, p_space):
    data = rng.integers(0, 256, size=n, dtype=np.uint8)
    data[data == 0x20] = 0x21
    data[rng.random(n) < p_space] = 0x20
    return data


@pytest.mark.parametrize("p_space", [0.0, 0.02, 0.15, 0.6, 1.0])
def test_against_regex_split(oracle_mod, p_space):
    rng = np.random.default_rng(int(p_space * 100) + 5)
    for trial in range(30):
        n = int(rng.integers(0, 400))
        data = _random_text(rng, n, p_space)
        n_seqs = int(rng.integers(1, 6))
        cuts = np.sort(rng.integers(0, n + 1, size=n_seqs - 1))
        seq = np.concatenate([[0], cuts, [n]]).astype(np.int32)
        off, first = oracle_mod.pretokenize(data, seq)
        want_off, want_first, raw = [0], [], data.tobytes()
        for k in range(n_seqs):
            want_first.append(len(want_off) - 1)
            for piece in _regex_pieces(raw[seq[k]:seq[k + 1]]):
                want_off.append(want_off[-1] + len(piece))
        want_first.append(len(want_off) - 1)
        assert off.tolist() == want_off
        assert first.tolist() == want_first


def test_closed_forms(oracle_mod):
    # all spaces: every byte is a piece; no space: one piece per non-empty sequence
    off, first = oracle_mod.pretokenize(_u8(b" " * 37))
    assert off.tolist() == list(range(38)) and first.tolist() == [0, 37]
    off, first = oracle_mod.pretokenize(_u8(b"x" * 37), [0, 10, 10, 37])
    assert off.tolist() == [0, 10, 37] and first.tolist() == [0, 1, 1, 2]
    # other white space, NUL and 0xA0 do not split
    off, _ = oracle_mod.pretokenize(_u8(b"a\tb\nc\x00d\xa0e\rf"))
    assert off.tolist() == [0, 11]
    # every k-th byte a space, text starting with a space: pieces of exactly k bytes
    for k in (1, 2, 7, 16, 17):
        data = _u8((b" " + b"y" * (k - 1)) * 20)
        off, _ = oracle_mod.pretokenize(data)
        assert off.tolist() == list(range(0, 20 * k + 1, k))


def test_invariants_and_generator_agreement(oracle_mod):
    from workloads import textgen
    rng = np.random.default_rng(11)
    for trial in range(20):
        n = int(rng.integers(1, 3000))
        data = _random_text(rng, n, 0.17)
        n_seqs = int(rng.integers(1, 9))
        seq = np.concatenate([[0], np.sort(rng.integers(0, n + 1, size=n_seqs - 1)), [n]]).astype(np.int32)
        off, first = oracle_mod.pretokenize(data, seq)
        assert off[0] == 0 and off[-1] == n and (np.diff(off) > 0).all()
        starts = set(off[:-1].tolist())
        for i in range(n):       # a byte starts a piece exactly when the rule says so
            assert (i in starts) == (i == 0 or data[i] == 0x20 or i in set(seq.tolist()))
        # a space can only be the first byte of its piece
        for q in range(off.size - 1):
            assert not (data[off[q] + 1:off[q + 1]] == 0x20).any()
        # sequence k begins exactly at its first piece, when it has one
        assert first[-1] == off.size - 1 and (np.diff(first) >= 0).all()
        for k in range(n_seqs):
            if seq[k] < seq[k + 1]:
                assert off[first[k]] == seq[k]
            else:
                assert first[k] == first[k + 1]
        assert first.tolist() == np.searchsorted(off[:-1], seq, side="left").tolist()
        # the numpy routine of the workload generator (written separately) agrees
        assert off.tolist() == textgen.pretokenize(data, seq[:-1]).tolist()


def test_workload_offsets_are_the_pretokenizer_output(oracle_mod):
    from workloads import configs as C
    for name in ("tiny", "seq32k"):
        ev = C.make_eval(name)
        off, first = oracle_mod.pretokenize(ev["bytes"])
        assert np.array_equal(off, ev["piece_offsets"])


def test_encode_raw_is_the_composition(oracle_mod):
    table = oracle_mod.Table([(ord("a"), ord("b")), (ord(" "), 256)])   # ab -> 256, " "+256 -> 257
    data = _u8(b"ab ab abab")
    ids, seq_tok, off, out_off = oracle_mod.encode_raw(table, data, [0, 2, 2, 10])
    assert off.tolist() == [0, 2, 5, 10]
    assert ids.tolist() == [256, 257, 257, 256]
    assert out_off.tolist() == [0, 1, 2, 4]
    assert seq_tok.tolist() == [0, 1, 1, 4]
