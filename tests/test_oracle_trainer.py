"""Pins for the oracle's BPE trainer."""
import numpy as np

from helpers import naive_train


def _corpus(rng, alpha, n_words, n_pieces, max_len):
    words = [bytes(rng.choice(alpha, size=int(rng.integers(1, max_len + 1))).astype(np.uint8).tolist())
             for _ in range(n_words)]
    return [words[int(i)] for i in rng.integers(0, n_words, size=n_pieces)]


def _flat(pieces):
    data = np.frombuffer(b"".join(pieces), dtype=np.uint8)
    off = np.concatenate([[0], np.cumsum([len(p) for p in pieces])]).astype(np.int32)
    return data, off


def test_matches_naive_recount_trainer(oracle_mod):
    rng = np.random.default_rng(5)
    for trial in range(60):
        alpha = [ord("a") + i for i in range(int(rng.integers(2, 6)))]
        pieces = _corpus(rng, alpha, int(rng.integers(3, 30)), int(rng.integers(20, 300)), 12)
        if trial % 5 == 0:   # long single-letter runs exercise overlapping pair counts
            pieces += [bytes([alpha[0]]) * int(rng.integers(2, 40))] * 3
        n = int(rng.integers(1, 40))
        want, segm = naive_train(pieces, n)
        data, off = _flat(pieces)
        got = [tuple(int(x) for x in m) for m in oracle_mod.train(data, off, n)]
        assert got == want
        # encoding a training piece with the full table gives the trainer's own segmentation
        table = oracle_mod.Table(got if got else np.zeros((0, 2)))
        ids, out_off = oracle_mod.encode(table, data, off)
        for p, piece in enumerate(pieces):
            assert [int(t) for t in ids[out_off[p]:out_off[p + 1]]] == segm[piece]


def test_stops_when_no_pair_is_left(oracle_mod):
    data, off = _flat([b"ab", b"ab", b"c"])
    merges = oracle_mod.train(data, off, 10)
    assert merges.tolist() == [[ord("a"), ord("b")]]


def _check_p1(merges):
    made_at = {}
    for k, (a, b) in enumerate(merges):
        for part in (int(a), int(b)):
            assert part < 256 or made_at[part] < k
        made_at[256 + k] = k
    assert len({(int(a), int(b)) for a, b in merges}) == len(merges)


def test_stored_tables_have_property_p1_and_match_the_manifest():
    from workloads import configs as C
    for name, spec in C.TABLES.items():
        merges = C.load_merges(name)          # checks count and hash against the manifest
        assert merges.shape == (spec["n_merges"], 2)
        _check_p1(merges)


def test_first_merge_is_the_most_frequent_byte_pair_and_table_regenerates(oracle_mod):
    from workloads import configs as C, textgen
    corpus = C.make_train_corpus("t1k")
    assert C.sha256(corpus) == C.manifest()["tables"]["t1k"]["train_corpus_sha256"]
    off = textgen.pretokenize(corpus)
    # independent histogram of adjacent byte pairs that do not straddle a piece start
    a, b = corpus[:-1].astype(np.int64), corpus[1:].astype(np.int64)
    inside = np.ones(corpus.size - 1, dtype=bool)
    inside[off[1:-1] - 1] = False
    hist = np.bincount((a * 256 + b)[inside], minlength=65536)
    top = int(hist.argmax())          # argmax takes the smallest index among ties
    merges = oracle_mod.train(corpus, off, 1000)
    assert (int(merges[0, 0]), int(merges[0, 1])) == (top // 256, top % 256)
    assert (merges == C.load_merges("t1k")).all()


def test_workload_generator_is_deterministic_and_matches_manifest():
    from workloads import configs as C
    man = C.manifest()["evals"]
    for name in ["tiny", "seq32k", "seq131k"]:
        ev = C.make_eval(name)
        assert C.sha256(ev["bytes"]) == man[name]["bytes_sha256"]
        assert ev["piece_offsets"].size - 1 == man[name]["n_pieces"]
        off = ev["piece_offsets"]
        assert off[0] == 0 and off[-1] == ev["bytes"].size and (np.diff(off) > 0).all()


def test_token_targets_are_met(oracle_mod):
    from workloads import configs as C
    ev = C.make_eval("seq32k")
    table = oracle_mod.Table(C.load_merges("t50k"))
    ids, _ = oracle_mod.encode(table, ev["bytes"], ev["piece_offsets"], n_threads=4)
    assert 32768 - 16 <= ids.size <= 32768
    assert ids.size == C.manifest()["evals"]["seq32k"]["n_tokens"]
