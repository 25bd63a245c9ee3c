"""Parity of the device pre-tokenizer and of the raw encode path (bytes +
sequence offsets in, token ids per sequence out) against the CPU oracle,
through the C ABI.  Offsets, counts and ids must match bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

BPE_ERR_SIZE, BPE_ERR_INPUT = -2, -11


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2603_02597_amd as B
    B.load_library()
    return torch, B


def _say(msg):
    print(msg, flush=True)


def _text(rng, n, p_space):
    data = rng.integers(0, 256, size=n, dtype=np.uint8)
    data[data == 0x20] = 0x21
    data[rng.random(n) < p_space] = 0x20
    return data


def _cuts(rng, n, n_seqs, n_empty=0):
    cuts = np.sort(rng.integers(0, n + 1, size=max(n_seqs - 1, 0)))
    seq = np.concatenate([[0], cuts, [n]])
    if n_empty:                                   # repeat some boundaries: empty sequences
        seq = np.sort(np.concatenate([seq, rng.choice(seq, size=n_empty)]))
    return seq.astype(np.int32)


def _pretokenize(gpu, data, seq, tile_kib=0, max_pieces=None, misalign=0, fill=None, want_first=True):
    """Runs bpe_pretokenize; returns (piece_offsets, n_pieces, seq_first_piece, status)."""
    torch, B = gpu
    n = data.size
    buf = torch.zeros(n + misalign + 16, dtype=torch.uint8, device="cuda")
    buf[misalign:misalign + n] = torch.from_numpy(np.array(data, dtype=np.uint8)).cuda()
    d = buf[misalign:misalign + n]
    cap = n if max_pieces is None else max_pieces
    off = torch.full((cap + 1,), -7, dtype=torch.int32, device="cuda")
    cnt = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    s = None if seq is None else torch.from_numpy(np.asarray(seq, dtype=np.int32)).cuda()
    n_first = 2 if seq is None else len(seq)
    first = torch.full((n_first,), -7, dtype=torch.int32, device="cuda") if want_first else None
    ws = torch.empty(B.bpe_pretokenize_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    if fill is not None:
        ws.copy_(torch.from_numpy(fill(ws.numel())).cuda())
    B.bpe_pretokenize(d, s, off, cnt, first, ws, B.EncodeOptions(pretokenize_tile_kib=tile_kib))
    st = B.bpe_encode_status(ws)
    return off.cpu().numpy(), int(cnt.item()), None if first is None else first.cpu().numpy(), st


def _check_pretokenize(gpu, oracle_mod, data, seq, label, **kw):
    _say(f"[case] pretokenize {label} n_bytes={data.size} n_seqs={None if seq is None else len(seq) - 1} {kw}")
    want_off, want_first = oracle_mod.pretokenize(data, seq)
    off, n_pieces, first, st = _pretokenize(gpu, data, seq, **kw)
    assert st == 0
    assert n_pieces == want_off.size - 1
    assert np.array_equal(off[:n_pieces + 1], want_off), \
        f"offsets differ first at {np.nonzero(off[:n_pieces + 1] != want_off)[0][:5]}"
    assert (off[n_pieces + 1:] == -7).all(), "wrote behind the last offset"
    if first is not None:
        assert np.array_equal(first, want_first), f"first pieces differ at {np.nonzero(first != want_first)[0][:5]}"


SIZES = [0, 1, 2, 15, 16, 17, 31, 1023, 1024, 1025, 4080, 4095, 4096, 4097, 16383, 16384, 16385, 65535, 65536,
         65537, 70001, 262144, 300007]


def test_pretokenize_sizes_and_tiles(gpu, oracle_mod):
    rng = np.random.default_rng(3)
    for n in SIZES:
        data = _text(rng, n, 0.15)
        for tile in (0, 4, 16, 64, 128, -64, -128):
            _check_pretokenize(gpu, oracle_mod, data, None, f"size {n}", tile_kib=tile)
        seq = _cuts(rng, n, 5, n_empty=2)
        _check_pretokenize(gpu, oracle_mod, data, seq, f"size {n} with sequences", tile_kib=4 if n % 2 else 16)


def test_pretokenize_space_densities(gpu, oracle_mod):
    rng = np.random.default_rng(4)
    for p_space in (0.0, 0.001, 0.02, 0.5, 1.0):
        for n in (5000, 66000):
            data = _text(rng, n, p_space)
            for tile in (4, 16, 64, 128, -64, -128):
                _check_pretokenize(gpu, oracle_mod, data, _cuts(rng, n, 3), f"density {p_space}", tile_kib=tile)


def test_pretokenize_any_alignment(gpu, oracle_mod):
    rng = np.random.default_rng(5)
    for mis in range(16):
        for n in (1, 16 - mis if mis else 16, 4096 - mis, 4097, 20000):
            data = _text(rng, n, 0.2)
            data[0] = 0x20 if mis % 2 else 0x41
            _check_pretokenize(gpu, oracle_mod, data, _cuts(rng, n, 4, n_empty=1), f"misaligned by {mis}",
                               misalign=mis, tile_kib=(0, 4, 16, 64, -64, -128, 128, 4)[mis % 8])


def test_pretokenize_many_sequences(gpu, oracle_mod):
    rng = np.random.default_rng(6)
    n = 40000
    data = _text(rng, n, 0.1)
    # one sequence per byte, and more sequences than bytes (most of them empty)
    _check_pretokenize(gpu, oracle_mod, data[:3000], np.arange(3001, dtype=np.int32), "one sequence per byte",
                       tile_kib=4)
    for n_seqs, n_empty, tile in ((300, 0, 4), (2000, 500, 16), (5000, 9000, 64), (700, 10, 0), (900, 30, -64),
                                 (50, 3, -128), (4000, 100, 128)):
        _check_pretokenize(gpu, oracle_mod, data, _cuts(rng, n, n_seqs, n_empty), f"{n_seqs} sequences",
                           tile_kib=tile)
    # all sequences empty but one
    seq = np.array([0] * 40 + [n] * 40, dtype=np.int32)
    _check_pretokenize(gpu, oracle_mod, data, seq, "empty sequences at both ends", tile_kib=16)
    _check_pretokenize(gpu, oracle_mod, data[:0], np.zeros(5, dtype=np.int32), "empty input, empty sequences")


def test_pretokenize_without_first_piece_output(gpu, oracle_mod):
    rng = np.random.default_rng(7)
    data = _text(rng, 9000, 0.2)
    _check_pretokenize(gpu, oracle_mod, data, _cuts(rng, 9000, 6), "no seq_first_piece", want_first=False)
    _check_pretokenize(gpu, oracle_mod, data, None, "no sequences, no seq_first_piece", want_first=False)


def test_pretokenize_workloads(gpu, oracle_mod):
    from workloads import configs as C
    for name in ("tiny", "seq32k", "seq131k", "stress"):
        ev = C.make_eval(name)
        off, n_pieces, _, st = _pretokenize(gpu, ev["bytes"], None)
        _say(f"[case] pretokenize workload {name}: {n_pieces} pieces")
        assert st == 0 and n_pieces == ev["piece_offsets"].size - 1
        assert np.array_equal(off[:n_pieces + 1], ev["piece_offsets"])
    ev = C.make_eval("batch")
    seq = np.concatenate([ev["piece_offsets"][ev["seq_first_piece"][:-1]], [ev["bytes"].size]]).astype(np.int32)
    _check_pretokenize(gpu, oracle_mod, ev["bytes"], seq, "workload batch, 256 sequences")


def test_pretokenize_workspace_needs_no_clearing(gpu, oracle_mod):
    rng = np.random.default_rng(8)
    data = _text(rng, 150000, 0.15)
    seq = _cuts(rng, data.size, 9)
    fills = [lambda k: np.full(k, 0xFF, dtype=np.uint8), lambda k: np.zeros(k, dtype=np.uint8),
             lambda k: np.random.default_rng(1).integers(0, 256, size=k, dtype=np.uint8),
             lambda k: np.tile(np.array([2, 0, 0, 0], dtype=np.uint8), k // 4 + 1)[:k]]
    for i, fill in enumerate(fills):
        _check_pretokenize(gpu, oracle_mod, data, seq, f"workspace fill {i}", fill=fill, tile_kib=4)


def test_pretokenize_repeated_calls_share_a_workspace(gpu, oracle_mod):
    torch, B = gpu
    rng = np.random.default_rng(9)
    ws = torch.empty(B.bpe_pretokenize_workspace_bytes(100000), dtype=torch.uint8, device="cuda")
    for n in (100000, 5000, 70000, 1, 0, 99999):
        data = _text(rng, n, 0.3)
        want, _ = oracle_mod.pretokenize(data)
        d = torch.from_numpy(data).cuda() if n else torch.empty(0, dtype=torch.uint8, device="cuda")
        off = torch.empty(n + 1, dtype=torch.int32, device="cuda")
        cnt = torch.empty(1, dtype=torch.int32, device="cuda")
        B.bpe_pretokenize(d, None, off, cnt, None, ws)
        assert B.bpe_encode_status(ws) == 0
        assert int(cnt.item()) == want.size - 1 and np.array_equal(off.cpu().numpy()[:want.size], want)


def test_pretokenize_too_many_pieces_is_reported(gpu, oracle_mod):
    rng = np.random.default_rng(10)
    data = _text(rng, 30000, 0.3)
    want, _ = oracle_mod.pretokenize(data)
    n_true = want.size - 1
    for cap in (n_true, n_true - 1, 100, 1, 0):
        off, n_pieces, first, st = _pretokenize(gpu, data, None, max_pieces=cap)
        _say(f"[case] capacity {cap} of {n_true} pieces -> status {st}")
        if cap >= n_true:
            assert st == 0 and n_pieces == n_true and np.array_equal(off[:n_true + 1], want)
        else:
            assert st == BPE_ERR_SIZE and n_pieces == cap
            assert np.array_equal(off[:cap], want[:cap]) and off[cap] == data.size


def test_pretokenize_invalid_sequence_offsets_are_reported(gpu):
    rng = np.random.default_rng(12)
    n = 20000
    data = _text(rng, n, 0.2)
    bad_sets = [[0, 500, 400, n], [1, 500, n], [0, 500, n - 1], [0, -5, n], [0, n + 7, n], [0, 2 ** 31 - 1, n],
                [0, -2 ** 31, n], list(rng.integers(-50000, 50000, size=300))]
    for seq in bad_sets:
        for tile in (4, 64):
            off, n_pieces, first, st = _pretokenize(gpu, data, np.array(seq, dtype=np.int64).astype(np.int32),
                                                    tile_kib=tile)
            _say(f"[case] invalid seq_offsets {seq[:4]}... -> status {st}")
            assert st == BPE_ERR_INPUT
            assert 0 <= n_pieces <= n and (off[n_pieces + 1:] == -7).all()


def test_argument_errors(gpu):
    torch, B = gpu
    d = torch.zeros(100, dtype=torch.uint8, device="cuda")
    off = torch.zeros(101, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.bpe_pretokenize_workspace_bytes(100), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.BpeError) as e:
        B.bpe_pretokenize(d, None, off, cnt, None, ws[:128])
    assert e.value.code == -8
    with pytest.raises(B.BpeError) as e:
        B.bpe_pretokenize(d, None, off, cnt, None, ws, B.EncodeOptions(pretokenize_tile_kib=8))
    assert e.value.code == -10
    assert B.load_library().bpe_pretokenize_workspace_bytes(-1) == BPE_ERR_SIZE
    assert B.load_library().bpe_encode_raw_workspace_bytes(2 ** 31, 0, 1) == BPE_ERR_SIZE


# ---------------------------------------------------------------------------
# raw path: bytes + sequence offsets -> token ids per sequence

def _check_raw(gpu, oracle_mod, merges, data, seq, label, max_pieces=0, own_arrays=True, opts=None, misalign=0):
    torch, B = gpu
    n = data.size
    _say(f"[case] raw {label} n_bytes={n} n_seqs={None if seq is None else len(seq) - 1} "
         f"max_pieces={max_pieces} own_arrays={own_arrays} opts={opts}")
    ot = oracle_mod.Table(merges)
    want_ids, want_seq_tok, want_off, want_out_off = oracle_mod.encode_raw(ot, data, seq, n_threads=16)
    gt = B.Table(merges)
    buf = torch.zeros(n + misalign + 16, dtype=torch.uint8, device="cuda")
    buf[misalign:misalign + n] = torch.from_numpy(np.array(data, dtype=np.uint8)).cuda()
    d = buf[misalign:misalign + n]
    s = None if seq is None else torch.from_numpy(np.asarray(seq, dtype=np.int32)).cuda()
    n_seqs = 1 if seq is None else len(seq) - 1
    cap = max_pieces if max_pieces else n
    out_ids = torch.full((max(n, 1),), -7, dtype=torch.int32, device="cuda")
    seq_tok = torch.full((n_seqs + 1,), -7, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.bpe_encode_raw_workspace_bytes(n, max_pieces, n_seqs), dtype=torch.uint8, device="cuda")
    poff = ooff = cnt = None
    if own_arrays:
        poff = torch.full((cap + 1,), -7, dtype=torch.int32, device="cuda")
        ooff = torch.full((cap + 1,), -7, dtype=torch.int32, device="cuda")
        cnt = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    B.bpe_encode_raw(gt, d, s, out_ids, seq_tok, ws, max_pieces, poff, ooff, cnt, opts)
    assert B.bpe_encode_status(ws) == 0
    got_seq_tok = seq_tok.cpu().numpy()
    assert np.array_equal(got_seq_tok, want_seq_tok), \
        f"sequence token offsets differ at {np.nonzero(got_seq_tok != want_seq_tok)[0][:5]}"
    total = int(want_seq_tok[-1])
    got_ids = out_ids.cpu().numpy()
    assert np.array_equal(got_ids[:total], want_ids), f"ids differ first at {np.nonzero(got_ids[:total] != want_ids)[0][:5]}"
    assert (got_ids[total:] == -7).all(), "wrote behind the last token"
    if own_arrays:
        n_pieces = int(cnt.item())
        assert n_pieces == want_off.size - 1
        assert np.array_equal(poff.cpu().numpy()[:n_pieces + 1], want_off)
        assert np.array_equal(ooff.cpu().numpy()[:n_pieces + 1], want_out_off)
    gt.free()


def test_raw_small_cases(gpu, oracle_mod):
    _, B = gpu
    merges = [(97, 98), (32, 256), (256, 256), (97, 97), (259, 259), (32, 97)]
    u8 = lambda b: np.frombuffer(b, dtype=np.uint8)
    for own in (True, False):
        _check_raw(gpu, oracle_mod, merges, u8(b""), None, "empty", own_arrays=own)
        _check_raw(gpu, oracle_mod, merges, u8(b""), [0, 0, 0], "empty with sequences", own_arrays=own)
        _check_raw(gpu, oracle_mod, merges, u8(b"a"), None, "one byte", own_arrays=own)
        _check_raw(gpu, oracle_mod, merges, u8(b" "), [0, 1], "one space", own_arrays=own)
        _check_raw(gpu, oracle_mod, merges, u8(b"ab ab abab  aaaa"), [0, 2, 2, 9, 16], "words", own_arrays=own)
        _check_raw(gpu, oracle_mod, merges, u8(b"ab ab abab  aaaa"), None, "words, one sequence", own_arrays=own)
        _check_raw(gpu, oracle_mod, merges, u8(b"abababab" * 40), [0, 3, 160, 320], "long piece cut by sequences",
                   own_arrays=own)
    for opts in (B.EncodeOptions(pieces_per_wave=3), B.EncodeOptions(tiny_max_len=-1, selection_level=1),
                 B.EncodeOptions(tiny_max_len=2, wave_max_len=4, wave_lds_max_len=8, pretokenize_tile_kib=64)):
        _check_raw(gpu, oracle_mod, merges, u8(b" ab abab aaaa ababababab a" * 30), [0, 100, 100, 780], "options",
                   opts=opts)


def test_raw_random_text(gpu, oracle_mod):
    from workloads import configs as C
    merges = C.load_merges("t1k")
    rng = np.random.default_rng(21)
    ev = C.make_eval("tiny")["bytes"]
    for trial in range(12):
        n = int(rng.integers(1, 20000))
        # workload text repeated, with some random bytes and extra spaces
        data = np.resize(ev, n).copy()
        noise = rng.random(n) < 0.03
        data[noise] = rng.integers(0, 256, size=int(noise.sum()), dtype=np.uint8)
        seq = _cuts(rng, n, int(rng.integers(1, 40)), n_empty=int(rng.integers(0, 5)))
        n_true = oracle_mod.pretokenize(data, seq)[0].size - 1
        _check_raw(gpu, oracle_mod, merges, data, seq, f"random text {trial}",
                   max_pieces=(0, n_true, n_true + 1000)[trial % 3], own_arrays=bool(trial % 2),
                   misalign=trial % 16)


def test_raw_workloads(gpu, oracle_mod):
    from workloads import configs as C
    for name in ("tiny", "seq32k", "seq131k", "stress"):
        ev = C.make_eval(name)
        merges = C.load_merges(ev["table"])
        _check_raw(gpu, oracle_mod, merges, ev["bytes"], None, f"workload {name}")
        n_true = ev["piece_offsets"].size - 1
        _check_raw(gpu, oracle_mod, merges, ev["bytes"], None, f"workload {name}, tight capacity",
                   max_pieces=n_true, own_arrays=False)


def test_raw_batch_workload(gpu, oracle_mod):
    from workloads import configs as C
    ev = C.make_eval("batch")
    merges = C.load_merges(ev["table"])
    seq = np.concatenate([ev["piece_offsets"][ev["seq_first_piece"][:-1]], [ev["bytes"].size]]).astype(np.int32)
    _check_raw(gpu, oracle_mod, merges, ev["bytes"], seq, "workload batch", max_pieces=ev["bytes"].size // 4)


def test_raw_with_long_piece_workgroups(gpu, oracle_mod):
    """The caller fixes tiles of 256 pieces (pieces_per_wave 64): the long pieces go to workgroups of
    their own at the head of the merge kernel's grid, by default from 1025 tiles on, or when asked for."""
    _, B = gpu
    from workloads import configs as C
    E = B.EncodeOptions
    ev = C.make_eval("stress")
    merges = C.load_merges(ev["table"])
    n_true = ev["piece_offsets"].size - 1
    _check_raw(gpu, oracle_mod, merges, ev["bytes"], None, "stress, default groups", opts=E(pieces_per_wave=64))
    _check_raw(gpu, oracle_mod, merges, ev["bytes"], None, "stress, tight capacity, 16 tiles per group",
               max_pieces=n_true, own_arrays=False, opts=E(pieces_per_wave=64, long_groups=16))
    _check_raw(gpu, oracle_mod, merges, ev["bytes"], None, "stress, no groups", opts=E(pieces_per_wave=64, long_groups=-1))
    ev = C.make_eval("batch")
    seq = np.concatenate([ev["piece_offsets"][ev["seq_first_piece"][:-1]], [ev["bytes"].size]]).astype(np.int32)
    _check_raw(gpu, oracle_mod, C.load_merges(ev["table"]), ev["bytes"], seq, "batch with groups",
               max_pieces=ev["bytes"].size // 4, opts=E(pieces_per_wave=64))
    # few tiles, every path, every piece long, lists that fill up
    merges = [(97, 98), (32, 256), (256, 256), (97, 97), (259, 259), (32, 97)]
    text = np.frombuffer(b" ab abab aaaa ababababab a" * 300 + b" " + b"ab" * 700 + b" " + b"a" * 3000, dtype=np.uint8)
    for kw in (dict(long_groups=1), dict(long_groups=3, tiny_max_len=2), dict(long_groups=256, tiny_max_len=-1),
               dict(long_groups=2, selection_level=1, column_max_len=-1)):
        _check_raw(gpu, oracle_mod, merges, text, [0, 100, 100, 780, text.size], f"few tiles {kw}",
                   opts=E(pieces_per_wave=64, **kw))


def test_raw_deep_grids(gpu, oracle_mod):
    """Grids of 4096 tiles and more, where an emit workgroup takes four tiles at a time: tile
    counts that are no multiple of four, with and without the scan kernel."""
    _, B = gpu
    from workloads import configs as C
    ev = C.make_eval("seq131k")
    merges = C.load_merges(ev["table"])
    n_true = ev["piece_offsets"].size - 1
    for ppw in (4, 1):           # 16 and 4 pieces per tile: 7,899 and 31,595 tiles
        _check_raw(gpu, oracle_mod, merges, ev["bytes"], None, f"seq131k, pieces_per_wave {ppw}",
                   max_pieces=n_true + 5, opts=B.EncodeOptions(pieces_per_wave=ppw))
    cut = int(ev["piece_offsets"][16 * 4097 + 1])
    _check_raw(gpu, oracle_mod, merges, ev["bytes"][:cut], None, "seq131k cut to 4,098 tiles",
               opts=B.EncodeOptions(pieces_per_wave=4))


def test_raw_sequence_offsets_from_the_emit_kernel_and_from_their_own(gpu, oracle_mod):
    """Up to 1023 sequences the emit kernel writes the first token of every sequence, beyond
    that a kernel of its own does: both sides of the limit, empty sequences at both ends and in
    between, several tiles, and a grid deep enough for four tiles per emit workgroup."""
    _, B = gpu
    from workloads import configs as C
    merges = C.load_merges("t1k")
    rng = np.random.default_rng(9)
    text = C.make_eval("seq32k")["bytes"]
    for n_seqs, n_empty in ((1023, 0), (1023, 700), (1024, 0), (1024, 300), (8000, 5000), (2, 0)):
        n = int(rng.integers(30000, 60000))
        seq = _cuts(rng, n, n_seqs - n_empty, n_empty)
        if n_empty:                 # empty sequences at the very start and the very end as well
            seq[1], seq[-2] = 0, n
        assert len(seq) - 1 == n_seqs and (np.diff(seq) >= 0).all()
        _check_raw(gpu, oracle_mod, merges, text[:n], seq, f"{n_seqs} sequences, {n_empty} of them added as empty ones")
    ev = C.make_eval("seq131k")
    n = ev["bytes"].size
    seq = np.sort(np.concatenate([[0, 0, n, n, n], rng.integers(0, n + 1, size=300)])).astype(np.int32)
    _check_raw(gpu, oracle_mod, C.load_merges(ev["table"]), ev["bytes"], seq, "deep grid with sequences",
               opts=B.EncodeOptions(pieces_per_wave=4))


def test_raw_too_many_pieces_is_reported(gpu, oracle_mod):
    torch, B = gpu
    from workloads import configs as C
    ev = C.make_eval("tiny")
    gt = B.Table(C.load_merges(ev["table"]))
    n = ev["bytes"].size
    d = torch.from_numpy(ev["bytes"].copy()).cuda()
    out_ids = torch.empty(n, dtype=torch.int32, device="cuda")
    seq_tok = torch.empty(2, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.bpe_encode_raw_workspace_bytes(n, 100, 1), dtype=torch.uint8, device="cuda")
    B.bpe_encode_raw(gt, d, None, out_ids, seq_tok, ws, max_pieces=100)
    assert B.bpe_encode_status(ws) == BPE_ERR_SIZE
    gt.free()


def test_raw_byte_tiles(gpu, oracle_mod):
    """Token-only calls on at most 1,310,720 bytes: no pre-tokenizer launch, the merge workgroups find the pieces
    in their own 1280 bytes.  Tiles with more than 256 pieces, with none, pieces that span tiles, starts and
    sequence cuts at the tile edges, unaligned input, both sides of the size limit."""
    _, B = gpu
    from workloads import configs as C
    merges = C.load_merges("t1k")
    assert B.kernels_by_interval(B.bpe_encode_raw_plan(5000, 0, 1, False, False), B.N_RAW_TIMED_INTERVALS)[1] == "merge_bytes_kernel"
    u8 = lambda b: np.frombuffer(b, dtype=np.uint8)
    rng = np.random.default_rng(77)
    text = C.make_eval("tiny")["bytes"]
    cases = {
        "only spaces": u8(b" " * 4000),
        "a space every other byte": u8(b"a " * 2000),
        "a space every third byte": u8(b"ab " * 1500),
        "no space at all": np.resize(text[text != 0x20], 5000),
        "one space, late": np.concatenate([np.resize(text[text != 0x20], 3000), u8(b" "), np.resize(text[text != 0x20], 2000)]),
        "runs of one byte across tiles": u8(b" " + b"e" * 2600 + b" " + b"t" * 1279 + b" x"),
    }
    for edge in (1278, 1279, 1280, 1281, 2559, 2560, 2561):         # a start right at, before and behind a tile edge
        d = np.resize(text[text != 0x20], 4000).copy()
        d[edge] = 0x20
        cases[f"single space at {edge}"] = d
        d = np.resize(text, 4000).copy()
        d[edge - 3:edge + 3] = 0x20
        cases[f"six spaces around {edge}"] = d
    for label, data in cases.items():
        for misalign in (0, 3):
            _check_raw(gpu, oracle_mod, merges, data, None, label, own_arrays=False, misalign=misalign)
        n = data.size
        for seq in ([0, 1280, 2560, n], [0, 1279, 1279, 1281, n], [0, 1, 2, n - 1, n], list(range(0, n + 1, 97)) + [n]):
            _check_raw(gpu, oracle_mod, merges, data, seq, label + ", sequences", own_arrays=False)
    # one sequence per byte: every byte starts a piece
    _check_raw(gpu, oracle_mod, merges, np.resize(text, 3000), np.arange(3001, dtype=np.int32), "one sequence per byte",
               own_arrays=False)
    # random texts with random cuts
    for trial in range(10):
        n = int(rng.integers(1, 30000))
        data = np.resize(text, n).copy()
        noise = rng.random(n) < (0.03, 0.3)[trial % 2]
        data[noise] = rng.choice(np.array([0x20, 0x20, 0x61, 0x00, 0xFF], dtype=np.uint8), size=int(noise.sum()))
        seq = _cuts(rng, n, int(rng.integers(1, 60)), n_empty=int(rng.integers(0, 5)))
        _check_raw(gpu, oracle_mod, merges, data, seq, f"random text {trial}", own_arrays=False, misalign=trial % 7)
    # the workloads that fit, with and without sequence offsets; both sides of the size limit
    for name in ("tiny", "seq32k", "seq131k"):
        ev = C.make_eval(name)
        m = C.load_merges(ev["table"])
        _check_raw(gpu, oracle_mod, m, ev["bytes"], None, f"workload {name}", own_arrays=False)
        cuts = np.sort(rng.integers(0, ev["bytes"].size, size=30)).astype(np.int32)
        _check_raw(gpu, oracle_mod, m, ev["bytes"], np.concatenate([[0], cuts, [ev["bytes"].size]]).astype(np.int32),
                   f"workload {name}, 31 sequences", own_arrays=False)
    ev = C.make_eval("seq131k")
    m = C.load_merges(ev["table"])
    for n in (1024 * 1280, 1024 * 1280 + 1):
        _check_raw(gpu, oracle_mod, m, np.resize(ev["bytes"], n), None, f"{n} bytes", own_arrays=False)


def test_raw_byte_tiles_report_invalid_sequence_offsets(gpu):
    """Token-only calls (no pre-tokenizer launch): sequence offsets that do not start at 0, end at n_bytes or
    increase are reported, whatever the number of sequences, and nothing is written out of bounds."""
    torch, B = gpu
    from workloads import configs as C
    gt = B.Table(C.load_merges("t1k"))
    data = torch.from_numpy(np.resize(C.make_eval("tiny")["bytes"], 5000).copy()).cuda()
    n = data.numel()
    for seq in ([0, n - 1], [3, n], [0, n + 7], [0, 2000, 1000, n], [0, 100, n + 1, n], [-5, 100, n]):
        _say(f"[case] raw byte tiles, invalid sequence offsets {seq}")
        s = torch.tensor(seq, dtype=torch.int32, device="cuda")
        guard = 64
        out_ids = torch.full((n + guard,), -7, dtype=torch.int32, device="cuda")
        seq_tok = torch.full((len(seq) + guard,), -7, dtype=torch.int32, device="cuda")
        ws = torch.empty(B.bpe_encode_raw_workspace_bytes(n, 0, len(seq) - 1), dtype=torch.uint8, device="cuda")
        B.bpe_encode_raw(gt, data, s, out_ids[:n], seq_tok[:len(seq)], ws, 0, None, None, None, None)
        assert B.bpe_encode_status(ws) == BPE_ERR_INPUT
        assert (out_ids[n:] == -7).all() and (seq_tok[len(seq):] == -7).all()
    gt.free()
