"""The merge loop on a run-length form of a piece ("lane per run"), checked on the CPU
against the oracle before any kernel uses it.

A piece that is mostly runs x x x ... is kept as a list of runs (symbol, count) in which
neighbours hold different symbols.  Its pairs are the interior pair (s, s) of every run
of two or more and the boundary pair between neighbouring runs.  A step takes the
lowest-ranked of them, the left-most on ties (the interior pair of a run lies left of
the boundary behind it), and
  * interior pair of run (s, c), merged id m: the run becomes (m, c // 2), followed by
    (s, 1) if c is odd: these are the c // 2 merges that the sequential loop makes one
    after the other, left to right, because every pair they create contains m and so
    ranks above the pair being merged;
  * boundary pair between (a, ca) and (b, cb): one merge, (a, ca - 1) (m, 1) (b, cb - 1);
then runs of no symbols go and neighbours with equal symbols are joined.  Restated here
in Python, independently of the HIP code; the final tokens must equal the oracle's."""
import numpy as np

from test_oracle_encode import _random_p1_table


def encode_runs(piece, merges, max_runs=64):
    """Tokens of the piece, or None if it ever needs more than max_runs runs."""
    rank = {(int(a), int(b)): k for k, (a, b) in enumerate(merges)}
    runs = []
    for x in piece:
        if runs and runs[-1][0] == int(x):
            runs[-1][1] += 1
        else:
            runs.append([int(x), 1])
    if len(runs) > max_runs:
        return None
    steps = 0
    while True:
        best = None
        for j, (s, c) in enumerate(runs):
            if c >= 2 and (s, s) in rank:
                key = (rank[(s, s)], j, 0)
                best = key if best is None or key < best else best
            if j + 1 < len(runs) and (s, runs[j + 1][0]) in rank:
                key = (rank[(s, runs[j + 1][0])], j, 1)
                best = key if best is None or key < best else best
        if best is None:
            break
        r, j, kind = best
        m = 256 + r
        if kind == 0:
            s, c = runs[j]
            new = [[m, c // 2]] + ([[s, 1]] if c % 2 else [])
            runs[j:j + 1] = new
        else:
            (a, ca), (b, cb) = runs[j], runs[j + 1]
            runs[j:j + 2] = [[a, ca - 1], [m, 1], [b, cb - 1]]
        out = []
        for s, c in runs:                   # runs of nothing go, equal neighbours are joined
            if c == 0:
                continue
            if out and out[-1][0] == s:
                out[-1][1] += c
            else:
                out.append([s, c])
        runs = out
        if len(runs) > max_runs:
            return None
        steps += 1
    return [s for s, c in runs for _ in range(c)]


def _oracle_tokens(oracle, merges, piece):
    data = np.frombuffer(bytes(piece), dtype=np.uint8) if isinstance(piece, (bytes, bytearray)) else np.asarray(piece, dtype=np.uint8)
    ids, _ = oracle.encode(oracle.Table(np.asarray(merges, dtype=np.int32).reshape(-1, 2)), data, [0, len(data)])
    return ids.tolist()


def test_worked_examples(oracle_mod):
    from test_oracle_encode import _parse_examples
    for data, merges, expect in _parse_examples():
        if merges and data:
            assert encode_runs(data, merges) == expect, data


def test_runs_of_every_length_are_the_binary_expansion(oracle_mod):
    merges = [(120, 120)] + [(256 + k, 256 + k) for k in range(12)]
    for n in list(range(1, 70)) + [255, 256, 257, 1000, 4095, 4096, 4097]:
        got = encode_runs(b"x" * n, merges)
        assert got == _oracle_tokens(oracle_mod, merges, b"x" * n)
        assert len(got) == bin(n).count("1") or n >= 8192
        got = encode_runs(b" " + b"x" * n, merges)
        assert got == _oracle_tokens(oracle_mod, merges, b" " + b"x" * n)


def test_random_run_like_pieces(oracle_mod):
    """Random tables over 2-5 letters (dense ties: interior and boundary pairs of every rank),
    pieces made of runs of random lengths."""
    rng = np.random.default_rng(4242)
    checked = 0
    for trial in range(400):
        alpha, merges = _random_p1_table(rng, int(rng.integers(2, 6)), int(rng.integers(1, 50)))
        n_runs = int(rng.integers(1, 20))
        syms = rng.choice(alpha, size=n_runs)
        reps = rng.integers(1, [3, 9, 40, 300][trial % 4], size=n_runs)
        piece = np.repeat(syms, reps).astype(np.uint8)
        got = encode_runs(piece, merges)
        if got is None:
            continue
        assert got == _oracle_tokens(oracle_mod, merges, piece), (trial, piece.tolist(), merges)
        checked += 1
    assert checked > 350


def test_stress_runs(oracle_mod):
    """The run pieces of the stress workload with its trained table."""
    from workloads import configs as C
    ev = C.make_eval("stress")
    merges = C.load_merges("t100k")
    off = ev["piece_offsets"]
    lens = np.diff(off)
    big = np.nonzero(lens > 64)[0]
    mlist = [tuple(int(x) for x in m) for m in merges]
    ot = oracle_mod.Table(merges)
    n_run = 0
    for q in big[:60]:
        piece = ev["bytes"][off[q]:off[q + 1]]
        got = encode_runs(piece, mlist)
        if got is None:
            continue              # random bytes: more than 64 runs
        want, _ = oracle_mod.encode(ot, piece, [0, piece.size])
        assert got == want.tolist(), q
        n_run += 1
    assert n_run >= 10
