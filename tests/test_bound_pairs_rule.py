"""Selection level 3 ("every pair that greedy is bound to merge, per pass") as a
rule, checked on the CPU against the oracle before any kernel uses it.

The rule (restated here in Python, independently of the HIP code): the pair
(u, v) at positions (i, i+1) with rank r may merge now if
  * walking left from u over pairs of rank > r one reaches, within a few steps, the
    start of the piece or a symbol that is the right part of no rule of rank <= r, and
  * walking right from v over pairs of rank >= r one reaches, within a few steps, the
    end of the piece or a symbol that is the left part of no rule of rank < r;
the occurrences of the piece's best rank are taken by the "everywhere, left to
right without overlap" rule instead.  The paper's introduction promises merging
non-overlapping local minima per pass and section 3.5 withdraws it; this is the
form of that idea that keeps the greedy result, and these tests are its
randomized equivalence check: the final tokens must equal the oracle's, no two
selected pairs may overlap, and every pass must make progress.
"""
import numpy as np

from test_oracle_encode import _random_p1_table

INF = 1 << 40


def _tables(merges):
    rank = {(int(a), int(b)): k for k, (a, b) in enumerate(merges)}
    lmin, rmin = {}, {}
    for k, (a, b) in enumerate(merges):
        rmin.setdefault(int(a), k)      # a as the left part
        lmin.setdefault(int(b), k)      # b as the right part
    return rank, lmin, rmin


def _bound(s, r, i, lmin, rmin, steps):
    ri = r[i]
    j, ok = i, False
    for _ in range(steps + 1):
        if j == 0 or lmin.get(s[j], INF) > ri:
            ok = True
            break
        if not r[j - 1] > ri:
            break
        j -= 1
    if not ok:
        return False
    j = i + 1
    for _ in range(steps + 1):
        if j == len(s) - 1 or rmin.get(s[j], INF) >= ri:
            return True
        if not r[j] >= ri:
            return False
        j += 1
    return False


def encode_bound_pairs(piece, merges, steps, with_best_rank=True):
    """Returns (tokens, passes).  with_best_rank=False: bound pairs only, and a
    best-rank pass whenever a pass merged fewer than an eighth of the symbols
    (what the windowed passes over pieces beyond the LDS do)."""
    rank, lmin, rmin = _tables(merges)
    s = [int(x) for x in piece]
    passes = 0
    force_best = False
    while len(s) >= 2:
        n = len(s)
        r = [rank.get((s[i], s[i + 1]), INF) for i in range(n - 1)]
        rho = min(r)
        if rho >= INF:
            break
        passes += 1
        sel = [False] * (n - 1)
        if with_best_rank or force_best:
            i = 0
            while i < n - 1:
                if r[i] != rho:
                    i += 1
                    continue
                if s[i] != s[i + 1]:
                    sel[i] = True
                    i += 1
                    continue
                j = i                      # run x x x ...: offsets 0, 2, 4 ... from its start
                while j < n - 1 and r[j] == rho:
                    j += 1
                for k in range(i, j, 2):
                    sel[k] = True
                i = j
        if not force_best:
            for i in range(n - 1):
                if r[i] < INF and (r[i] != rho or not with_best_rank) and _bound(s, r, i, lmin, rmin, steps):
                    sel[i] = True
        for i in range(n - 2):
            assert not (sel[i] and sel[i + 1]), "two selected pairs overlap"
        if with_best_rank:
            assert any(sel), "a pass without progress"
        out, i = [], 0
        while i < n:
            if i < n - 1 and sel[i]:
                out.append(256 + r[i])
                i += 2
            else:
                out.append(s[i])
                i += 1
        force_best = not with_best_rank and not force_best and n - len(out) < n // 8
        if not with_best_rank and not any(sel) and not force_best:
            force_best = True
        s = out
    return s, passes


def encode_bound_pairs_carried_rank(piece, merges, steps):
    """What the windowed passes over pieces beyond the LDS do: a pass knows the best
    rank of the state *before* the previous pass's merges (it was found while that
    pass looked at every pair), not of the present state.  If a pair of that rank
    is still there it is the present best rank as well, because every pair is either
    an old one or contains a fresh id and ranks above the merge that made it; so
    its occurrences are taken by the best-rank rule, everything else by the walks.
    Returns (tokens, passes); at most one pass in a row may merge nothing."""
    rank, lmin, rmin = _tables(merges)
    s = [int(x) for x in piece]
    passes, carried, idle = 0, None, 0
    while len(s) >= 2:
        n = len(s)
        r = [rank.get((s[i], s[i + 1]), INF) for i in range(n - 1)]
        rho = min(r)
        if rho >= INF:
            break
        if carried is not None and carried in r:
            assert carried == rho, "a carried rank that is present must be the best rank"
        passes += 1
        sel = [False] * (n - 1)
        i = 0
        while carried is not None and i < n - 1:
            if r[i] != carried:
                i += 1
                continue
            if s[i] != s[i + 1]:
                sel[i] = True
                i += 1
                continue
            j = i
            while j < n - 1 and r[j] == carried:
                j += 1
            for k in range(i, j, 2):
                sel[k] = True
            i = j
        for i in range(n - 1):
            if r[i] < INF and r[i] != carried and _bound(s, r, i, lmin, rmin, steps):
                sel[i] = True
        for i in range(n - 2):
            assert not (sel[i] and sel[i + 1]), "two selected pairs overlap"
        idle = 0 if any(sel) else idle + 1
        assert idle <= 1, "two passes in a row without progress"
        out, i = [], 0
        while i < n:
            if i < n - 1 and sel[i]:
                out.append(256 + r[i])
                i += 2
            else:
                out.append(s[i])
                i += 1
        carried = rho
        s = out
    return s, passes


def _oracle_tokens(oracle_mod, merges, piece):
    t = oracle_mod.Table(np.asarray(merges, dtype=np.int32).reshape(-1, 2))
    data = np.frombuffer(bytes(piece), dtype=np.uint8)
    ids, _ = oracle_mod.encode(t, data, np.array([0, data.size], dtype=np.int32))
    return [int(x) for x in ids]


def test_counter_examples_of_naive_local_minima(oracle_mod):
    x, y, a, b = (ord(c) for c in "xyab")
    merges = [(x, y), (256, a), (a, b)]
    for steps in (0, 1, 8):
        assert encode_bound_pairs(b"xyab", merges, steps)[0] == [257, b] == _oracle_tokens(oracle_mod, merges, b"xyab")
    # runs of one symbol whose pair is a rule, and whose merged id pairs with the symbol again
    u = ord("u")
    merges = [(u, u), (256, u)]
    for n in range(1, 12):
        piece = bytes([u] * n)
        for steps in (0, 2, 8):
            assert encode_bound_pairs(piece, merges, steps)[0] == _oracle_tokens(oracle_mod, merges, piece)


def test_random_tables_equal_oracle(oracle_mod):
    rng = np.random.default_rng(424242)
    n = 0
    for trial in range(400):
        alpha, merges = _random_p1_table(rng, int(rng.integers(2, 5)), int(rng.integers(1, 30)))
        for _ in range(4):
            piece = bytes(rng.choice(alpha, size=int(rng.integers(0, 60))).astype(np.uint8).tolist())
            want = _oracle_tokens(oracle_mod, merges, piece)
            for steps in (0, 1, 3, 8, 100):
                got, _ = encode_bound_pairs(piece, merges, steps)
                assert got == want, (merges, piece, steps)
            got, _ = encode_bound_pairs(piece, merges, 8, with_best_rank=False)
            assert got == want, (merges, piece, "bound pairs only")
            for steps in (0, 2, 8):
                got, _ = encode_bound_pairs_carried_rank(piece, merges, steps)
                assert got == want, (merges, piece, steps, "carried best rank")
            n += 1
    assert n == 1600


def test_trained_table_on_text_chunks(oracle_mod):
    """Word-like text cut into chunks (pieces that span many words): same tokens, far fewer passes."""
    from workloads import configs as C
    ev = C.make_eval("tiny")
    merges = [tuple(int(v) for v in m) for m in C.load_merges(ev["table"])]
    data = ev["bytes"]
    rng = np.random.default_rng(5)
    for size in (40, 200, 700):
        for _ in range(3):
            o = int(rng.integers(0, data.size - size))
            piece = bytes(data[o:o + size].tolist())
            want = _oracle_tokens(oracle_mod, merges, piece)
            got2, passes_best = encode_bound_pairs(piece, merges, -1)     # no walk at all: the best rank only
            got3, passes_bound = encode_bound_pairs(piece, merges, 8)
            gotw, _ = encode_bound_pairs(piece, merges, 8, with_best_rank=False)
            gotc, passes_carried = encode_bound_pairs_carried_rank(piece, merges, 8)
            assert got2 == want and got3 == want and gotw == want and gotc == want
            assert passes_carried <= 2 * passes_bound + 2
            assert passes_bound <= passes_best
            if size >= 200:
                assert 3 * passes_bound <= passes_best
