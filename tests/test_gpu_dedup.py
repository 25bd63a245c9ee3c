"""Piece de-duplication (option dedup) against the CPU oracle: every distinct piece of
at most 16 bytes is merged once; ids and offsets must not change."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2603_02597_amd as B
    B.load_library()
    return torch, B


def _check(gpu, oracle_mod, merges, data, off, label, fill=None, **kw):
    torch, B = gpu
    if isinstance(data, (bytes, bytearray)):
        data = np.frombuffer(bytes(data), dtype=np.uint8)
    data = np.array(data, dtype=np.uint8)
    off = np.ascontiguousarray(np.asarray(off, dtype=np.int32))
    print(f"[case] dedup {label} n_bytes={data.size} n_pieces={off.size - 1} {kw}", flush=True)
    merges = np.asarray(merges, dtype=np.int32).reshape(-1, 2)
    want_ids, want_off = oracle_mod.encode(oracle_mod.Table(merges), data, off, n_threads=16)
    gt = B.Table(merges)
    d, o = torch.from_numpy(data).cuda(), torch.from_numpy(off).cuda()
    n, n_pieces = d.numel(), o.numel() - 1
    ids = torch.full((max(n, 1),), -5, dtype=torch.int32, device="cuda")
    out_off = torch.full((n_pieces + 1,), -5, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.bpe_dedup_workspace_bytes(n, n_pieces), dtype=torch.uint8, device="cuda")
    if fill is not None:
        ws.fill_(fill)
    B.bpe_encode(gt, d, o, ids, out_off, ws, B.EncodeOptions(dedup=1, **kw))
    assert B.bpe_encode_status(ws) == 0
    got_ids, got_off = ids.cpu().numpy(), out_off.cpu().numpy()
    assert np.array_equal(got_off, want_off), f"offsets differ first at {np.nonzero(got_off != want_off)[0][:5]}"
    assert np.array_equal(got_ids[:want_ids.size], want_ids), "ids differ"
    assert (got_ids[want_ids.size:] == -5).all()
    gt.free()
    return ws


def test_worked_examples_and_edges(gpu, oracle_mod):
    from test_oracle_encode import _parse_examples
    for data, merges, expect in _parse_examples():
        if merges:
            rep = data * 5                       # the same piece five times, and once more in one piece
            off = [len(data) * k for k in range(6)]
            _check(gpu, oracle_mod, merges, np.frombuffer(rep + rep, dtype=np.uint8), off + [2 * len(rep)], f"worked {data!r}")
    merges = [(97, 97), (256, 256), (257, 257), (97, 98), (98, 97)]
    _check(gpu, oracle_mod, merges, b"", [0], "no pieces")
    _check(gpu, oracle_mod, merges, b"", [0, 0, 0], "only empty pieces")
    _check(gpu, oracle_mod, merges, b"a", [0, 1], "one byte")
    _check(gpu, oracle_mod, merges, b"aaabaaab", [0, 0, 1, 1, 1, 4, 4, 5, 8], "empty pieces around")
    # pieces of exactly 16 and 17 bytes (looked up / not looked up), equal up to their last byte
    data = b"a" * 16 + b"a" * 17 + b"a" * 16 + b"a" * 15 + b"b" + b"a" * 17 + b"a" * 15 + b"b"
    _check(gpu, oracle_mod, merges, data, [0, 16, 33, 49, 65, 82, 98], "16 / 17 bytes")
    # equal prefixes, different lengths: the length is part of the key
    _check(gpu, oracle_mod, merges, b"a" * 40, [0, 1, 3, 6, 10, 15, 21, 28, 36, 40], "prefixes")


@pytest.mark.parametrize("name", ["tiny", "seq32k", "seq131k", "batch", "stress"])
def test_workloads_exact(gpu, oracle_mod, name):
    from workloads import configs as C
    ev = C.make_eval(name)
    _check(gpu, oracle_mod, C.load_merges(ev["table"]), ev["bytes"], ev["piece_offsets"], name)


def test_workspace_contents_do_not_matter_and_calls_repeat(gpu, oracle_mod):
    torch, B = gpu
    from workloads import configs as C
    ev = C.make_eval("seq32k")
    merges = C.load_merges("t50k")
    for fill in (0x00, 0xFF, 0x5A):
        _check(gpu, oracle_mod, merges, ev["bytes"], ev["piece_offsets"], f"fill {fill:#x}", fill=fill)
    # the same workspace for call after call on other contents: nothing of an earlier call is taken for this one's
    table, ot = B.Table(merges), oracle_mod.Table(merges)
    host = ev["bytes"].copy()
    d, o = torch.from_numpy(host.copy()).cuda(), torch.from_numpy(ev["piece_offsets"].copy()).cuda()
    n, n_pieces = d.numel(), o.numel() - 1
    ids = torch.empty(n, dtype=torch.int32, device="cuda")
    out_off = torch.empty(n_pieces + 1, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.bpe_dedup_workspace_bytes(n, n_pieces), dtype=torch.uint8, device="cuda")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.bpe_encode(table, d, o, ids, out_off, ws, B.EncodeOptions(dedup=1))
    for replay in range(4):
        print(f"[case] dedup graph replay {replay}", flush=True)
        cur = host.copy()
        cur[cur == 0x65] = 0x61 + replay              # other letters: other pieces are equal to each other now
        d.copy_(torch.from_numpy(cur).cuda())
        ids.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert B.bpe_encode_status(ws) == 0
        want_ids, want_off = oracle_mod.encode(ot, cur, ev["piece_offsets"], n_threads=16)
        assert np.array_equal(out_off.cpu().numpy(), want_off)
        assert np.array_equal(ids.cpu().numpy()[:want_ids.size], want_ids)
    table.free()


def test_random_tables_with_many_repeats(gpu, oracle_mod):
    from test_oracle_encode import _random_p1_table
    rng = np.random.default_rng(606)
    for trial in range(12):
        alpha, merges = _random_p1_table(rng, int(rng.integers(2, 5)), int(rng.integers(1, 40)))
        # few distinct words, drawn over and over, and some longer pieces of every other path in between
        words = [rng.choice(alpha, size=int(rng.integers(0, 17))).astype(np.uint8) for _ in range(int(rng.integers(1, 300)))]
        picks = rng.integers(0, len(words), size=int(rng.integers(1, 6000)))
        parts = [words[k] for k in picks]
        for k in rng.integers(0, len(parts), size=20):
            parts[k] = rng.choice(alpha, size=int(rng.integers(17, 300))).astype(np.uint8)
        if trial % 3 == 0:
            parts[int(rng.integers(0, len(parts)))] = rng.choice(alpha, size=int(rng.integers(1100, 5000))).astype(np.uint8)
        lens = np.array([p.size for p in parts])
        data = np.concatenate(parts) if lens.sum() else np.zeros(0, dtype=np.uint8)
        off = np.concatenate([[0], np.cumsum(lens)])
        _check(gpu, oracle_mod, merges, data, off, f"random repeats {trial}", selection_level=int(rng.integers(0, 4)))


def test_options_that_do_not_go_with_it(gpu):
    torch, B = gpu
    table = B.Table([(97, 97)])
    d = torch.full((100,), 97, dtype=torch.uint8, device="cuda")
    o = torch.tensor([0, 50, 100], dtype=torch.int32, device="cuda")
    for kw in (dict(fused=1), dict(fused=2), dict(paper_kernel=1), dict(pieces_per_wave=8), dict(pieces_per_wave=-1)):
        with pytest.raises(B.BpeError) as e:
            B.encode(table, d, o, B.EncodeOptions(dedup=1, **kw))
        assert e.value.code == -10
    ids = torch.empty(100, dtype=torch.int32, device="cuda")
    off = torch.empty(3, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.bpe_workspace_bytes(100, 2), dtype=torch.uint8, device="cuda")       # too small for dedup
    with pytest.raises(B.BpeError) as e:
        B.bpe_encode(table, d, o, ids, off, ws, B.EncodeOptions(dedup=1))
    assert e.value.code == -8
    table.free()
