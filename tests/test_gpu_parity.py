"""Parity of the HIP path against the CPU oracle, through the C ABI.
Token ids and offsets must match bit for bit."""
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


def _say(msg):
    print(msg, flush=True)


def _run(gpu, oracle_mod, merges, data, off, opts=None, ranks=None, merged_ids=None, label=""):
    torch, B = gpu
    if isinstance(data, (bytes, bytearray)):
        data = np.frombuffer(bytes(data), dtype=np.uint8)
    data = np.array(data, dtype=np.uint8)        # writable copy
    off = np.ascontiguousarray(np.asarray(off, dtype=np.int32))
    _say(f"[case] {label} n_bytes={data.size} n_pieces={off.size - 1} opts={opts}")
    merges = np.asarray(merges, dtype=np.int32).reshape(-1, 2)
    ot = oracle_mod.Table(merges, ranks, merged_ids)
    want_ids, want_off = oracle_mod.encode(ot, data, off, n_threads=16)
    gt = B.Table(merges, ranks, merged_ids)
    d = torch.from_numpy(data).cuda()
    o = torch.from_numpy(off).cuda()
    ids, out_off = B.encode(gt, d, o, opts)
    got_ids, got_off = ids.cpu().numpy(), out_off.cpu().numpy()
    assert got_off.shape == want_off.shape
    assert (got_off == want_off).all(), f"offsets differ first at {np.nonzero(got_off != want_off)[0][:5]}"
    assert got_ids.shape == want_ids.shape
    assert (got_ids == want_ids).all(), f"ids differ first at {np.nonzero(got_ids != want_ids)[0][:5]}"
    gt.free()
    return got_ids, got_off


def _opt_sets(B):
    E = B.EncodeOptions
    # without the 64-entry columns: the lane-per-symbol path takes the pieces of 17-64 bytes
    old = [dict(),
           dict(selection_level=1),
           dict(pieces_per_wave=1),
           dict(pieces_per_wave=7),
           dict(pieces_per_wave=-1),                                   # one piece per workgroup
           dict(tiny_max_len=-1),                                      # no lane-per-piece path
           dict(tiny_max_len=-1, selection_level=1),
           dict(tiny_max_len=3, wave_max_len=6, wave_lds_max_len=12),  # all four paths on small inputs
           dict(tiny_max_len=-1, wave_max_len=-1),                     # wavefront-LDS + workgroup paths
           dict(tiny_max_len=2, wave_max_len=-1, wave_lds_max_len=40, selection_level=1),
           dict(tiny_max_len=-1, wave_max_len=-1, wave_lds_max_len=-1),                  # workgroup path only (LDS)
           dict(tiny_max_len=-1, wave_max_len=-1, wave_lds_max_len=-1, lds_max_len=2),   # ... in the workspace
           dict(tiny_max_len=-1, wave_max_len=-1, wave_lds_max_len=-1, lds_max_len=2, selection_level=1,
                pieces_per_wave=3),
           dict(selection_level=3),                                    # every bound pair per pass on the long-piece paths
           dict(selection_level=3, tiny_max_len=-1, wave_max_len=-1),  # ... one wavefront up to 512 symbols, else the workgroup
           dict(selection_level=3, tiny_max_len=-1, wave_max_len=-1, wave_lds_max_len=-1, pieces_per_wave=-1),   # ... the workgroup only
           dict(selection_level=3, tiny_max_len=-1, wave_max_len=-1, wave_lds_max_len=-1, lds_max_len=2),  # ... in windows of 320
           dict(selection_level=3, tiny_max_len=4, wave_max_len=-1, wave_lds_max_len=100, lds_max_len=300, pieces_per_wave=5)]
    old = [dict(column_max_len=-1, **d) for d in old]
    # with them (the default: pieces of 17-64 bytes, 16 per wavefront and round)
    cols = [dict(),
            dict(tiny_max_len=-1),                                     # every piece of up to 64 bytes in a 64-entry column
            dict(tiny_max_len=-1, pieces_per_wave=1),
            dict(tiny_max_len=-1, pieces_per_wave=-1, selection_level=2),
            dict(tiny_max_len=5, column_max_len=33),                   # the lane-per-symbol path behind the columns
            dict(tiny_max_len=3, column_max_len=9, wave_max_len=20, wave_lds_max_len=50, lds_max_len=80),   # all five paths
            dict(tiny_max_len=-1, column_max_len=17, wave_max_len=-1, selection_level=1, pieces_per_wave=40)]
    # merge_kernel's long-piece workgroups (several kernels, 256 pieces per tile; by default only from 1025 tiles on)
    groups = [dict(long_groups=1),
              dict(long_groups=3, tiny_max_len=5),
              dict(long_groups=2, selection_level=2),
              dict(long_groups=256, tiny_max_len=-1),                  # every piece is a long piece: the lists fill up and are worked off in between
              dict(long_groups=256, column_max_len=-1, wave_lds_max_len=100),
              dict(long_groups=7, selection_level=1, wave_max_len=-1)]
    base = cols + old
    # every set with the single-kernel path and with the merge + emit path
    # (fused=2: the single kernel whatever the grid and the piece lengths; fused=1 is refused beyond 1024 tiles
    # and for pieces that average more than 64 bytes)
    return [None] + [E(fused=2, **d) for d in base[1:]] + [E(fused=-1, **d) for d in base + groups]


def test_table_lookup_matches_host_map(gpu):
    torch, B = gpu
    from workloads import configs as C
    merges = C.load_merges("t50k")
    table = B.Table(merges)
    rng = np.random.default_rng(11)
    miss = rng.integers(0, 50256, size=(200_000, 2)).astype(np.int32)
    # right id 0: the word such a query compares can equal what an empty slot holds
    zero_b = np.stack([np.arange(50256), np.zeros(50256)], axis=1).astype(np.int32)
    pairs = np.concatenate([merges, miss, zero_b, zero_b[:, ::-1], np.array([[-1, 5], [5, -1]], dtype=np.int32)])
    present = {(int(a), int(b)): k for k, (a, b) in enumerate(merges)}
    want = np.array([present.get((int(a), int(b)), -1) for a, b in pairs], dtype=np.int32)
    p = torch.from_numpy(pairs).cuda()
    r = torch.empty(len(pairs), dtype=torch.int32, device="cuda")
    m = torch.empty(len(pairs), dtype=torch.int32, device="cuda")
    B.bpe_table_lookup(table, p, r, m)
    torch.cuda.synchronize()
    r, m = r.cpu().numpy(), m.cpu().numpy()
    assert (r == want).all()
    assert (m == np.where(want >= 0, want + 256, -1)).all()
    # caller's rank values come back even when they are sparse and out of order
    t2 = B.Table([(97, 98), (98, 99)], ranks=[70, 30], merged_ids=[1000, 2000])
    p2 = torch.tensor([[97, 98], [98, 99], [99, 97]], dtype=torch.int32, device="cuda")
    r2 = torch.empty(3, dtype=torch.int32, device="cuda")
    m2 = torch.empty(3, dtype=torch.int32, device="cuda")
    B.bpe_table_lookup(t2, p2, r2, m2)
    torch.cuda.synchronize()
    assert r2.tolist() == [70, 30, -1] and m2.tolist() == [1000, 2000, -1]


def test_worked_examples(gpu, oracle_mod):
    from test_oracle_encode import _parse_examples
    _, B = gpu
    for data, merges, expect in _parse_examples():
        if not merges:
            continue
        for opts in _opt_sets(B):
            got, _ = _run(gpu, oracle_mod, merges, np.frombuffer(data, dtype=np.uint8), [0, len(data)],
                          opts, label=f"worked {data!r}")
            assert got.tolist() == expect


def test_edge_cases(gpu, oracle_mod):
    _, B = gpu
    merges = [(97, 97), (256, 256), (257, 257), (97, 98), (98, 97)]
    for opts in _opt_sets(B):
        _run(gpu, oracle_mod, merges, b"", [0], opts, label="no pieces")
        _run(gpu, oracle_mod, merges, b"", [0, 0, 0], opts, label="only empty pieces")
        _run(gpu, oracle_mod, merges, b"a", [0, 1], opts, label="one byte")
        _run(gpu, oracle_mod, merges, b"aaab", [0, 0, 1, 1, 1, 4, 4], opts, label="empty pieces around")
        for n in [63, 64, 65, 127, 128, 129]:
            _run(gpu, oracle_mod, merges, b"a" * n, [0, n], opts, label=f"run {n}")
            _run(gpu, oracle_mod, merges, b"ab" * n, [0, n, 2 * n], opts, label=f"two pieces of {n}")
    # empty table: output = bytes
    data = bytes(range(256)) * 3
    _run(gpu, oracle_mod, np.zeros((0, 2)), data, [0, 5, 5, 300, 768], label="empty table")


def test_runs_of_every_length(gpu, oracle_mod):
    merges = [(120, 120)] + [(256 + k, 256 + k) for k in range(12)]
    lens = list(range(1, 200)) + [255, 256, 257, 1000, 4095, 4096, 4097, 7168, 7169, 10_000]
    data = b"".join(b"x" * n for n in lens)
    off = np.concatenate([[0], np.cumsum(lens)])
    _, B = gpu
    for opts in [None, B.EncodeOptions(selection_level=1), B.EncodeOptions(lds_max_len=100, wave_lds_max_len=-1),
                 B.EncodeOptions(tiny_max_len=-1, wave_max_len=-1), B.EncodeOptions(wave_lds_max_len=-1),
                 B.EncodeOptions(fused=2), B.EncodeOptions(fused=2, selection_level=1)]:
        _run(gpu, oracle_mod, merges, data, off, opts, label="runs")


def test_custom_ranks_and_ids(gpu, oracle_mod):
    merges = [(97, 98), (98, 99), (1000, 99)]
    _run(gpu, oracle_mod, merges, b"abcabc abc", [0, 6, 10], ranks=[5, 9, 7], merged_ids=[1000, 2000, 3000],
         label="custom ranks/ids")
    # the largest ids there are, as left and as right parts
    top = (1 << 24) - 1
    _run(gpu, oracle_mod, [(97, 98), (top, 99), (100, top - 1), (top - 2, top - 2)], b"abcabc dabc dabcdabc ab",
         [0, 6, 11, 20, 23], merged_ids=[top, top - 1, top - 2, 256], label="ids up to 2^24 - 1")


def test_random_small_alphabet(gpu, oracle_mod):
    """Random tables over 2-4 letters and random ragged pieces, including long ones."""
    _, B = gpu
    from test_oracle_encode import _random_p1_table
    rng = np.random.default_rng(2024)
    for trial in range(70):
        alpha, merges = _random_p1_table(rng, int(rng.integers(2, 5)), int(rng.integers(1, 40)))
        lens = np.concatenate([rng.integers(0, 20, size=3000), rng.integers(50, 80, size=60),
                               rng.integers(100, 700, size=8)])
        if trial % 3 == 2:       # pieces for the workgroup path: in LDS, at its limit, in the workspace
            lens = np.concatenate([lens, rng.integers(1025, 4104, size=2), [4104, 4105], rng.integers(4106, 6000, size=1)])
        rng.shuffle(lens)
        data = rng.choice(alpha, size=int(lens.sum())).astype(np.uint8)
        off = np.concatenate([[0], np.cumsum(lens)])
        opts = _opt_sets(B)[trial % len(_opt_sets(B))]
        ranks = merged_ids = None
        if trial % 4 == 1:       # sparse merged ids anywhere below 2^24, sparse ranks, rows in random order
            new_ids = rng.choice(np.arange(256, 1 << 24), size=len(merges), replace=False)
            remap = lambda x: int(new_ids[x - 256]) if x >= 256 else x
            merges = [(remap(a), remap(b)) for a, b in merges]
            ranks = np.sort(rng.choice(np.arange(0, 1 << 30), size=len(merges), replace=False))
            order = rng.permutation(len(merges))
            merges, ranks, merged_ids = [merges[k] for k in order], ranks[order], new_ids[order]
        _run(gpu, oracle_mod, merges, data, off, opts, ranks=ranks, merged_ids=merged_ids,
             label=f"random alphabet {trial}")


@pytest.mark.parametrize("fused", [1, -1])
@pytest.mark.parametrize("name", ["tiny", "seq32k", "seq131k"])
def test_workloads_exact(gpu, oracle_mod, name, fused):
    from workloads import configs as C
    _, B = gpu
    ev = C.make_eval(name)
    _run(gpu, oracle_mod, C.load_merges(ev["table"]), ev["bytes"], ev["piece_offsets"],
         B.EncodeOptions(fused=fused), label=name)


def test_tiny_all_option_sets(gpu, oracle_mod):
    from workloads import configs as C
    _, B = gpu
    ev = C.make_eval("tiny")
    for opts in _opt_sets(B):
        _run(gpu, oracle_mod, C.load_merges("t1k"), ev["bytes"], ev["piece_offsets"], opts, label="tiny")


@pytest.mark.parametrize("fused", [2, -1])
def test_batch_exact(gpu, oracle_mod, fused):
    from workloads import configs as C
    _, B = gpu
    ev = C.make_eval("batch")
    ids, off = _run(gpu, oracle_mod, C.load_merges("t50k"), ev["bytes"], ev["piece_offsets"],
                    B.EncodeOptions(fused=fused), label="batch")
    # per-sequence slicing through seq_first_piece
    sfp = ev["seq_first_piece"]
    assert len(sfp) == 257 and off[sfp[-1]] == ids.size


def test_deep_grids_of_the_emit_kernels(gpu, oracle_mod):
    """Grids of 4096 tiles and more, where a workgroup of the emit kernel takes four tiles:
    with the tile totals added up by the workgroup (up to 8192 tiles) and taken from the
    scan kernel (beyond), tile counts that are no multiple of four, pieces of many tokens."""
    _, B = gpu
    from workloads import configs as C
    from test_oracle_encode import _random_p1_table
    ev = C.make_eval("seq131k")
    merges = C.load_merges(ev["table"])
    off = ev["piece_offsets"]
    for ppw, n_pieces in ((4, 126380), (4, 16 * 4096 - 15), (4, 16 * 4097 + 1), (1, 126380), (1, 4 * 8192 + 1),
                          (-1, 8193), (-1, 4099)):
        n = min(n_pieces, off.size - 1)
        _run(gpu, oracle_mod, merges, ev["bytes"][:off[n]], off[:n + 1],
             B.EncodeOptions(fused=-1, pieces_per_wave=ppw), label=f"deep grid, {n} pieces, pieces_per_wave {ppw}")
    # random bytes and runs: most pieces keep several tokens, some more than eight, some hundreds
    rng = np.random.default_rng(77)
    alpha, small = _random_p1_table(rng, 3, 12)
    lens = np.concatenate([rng.integers(0, 14, size=20000), rng.integers(20, 64, size=300), rng.integers(200, 900, size=12)])
    rng.shuffle(lens)
    data = rng.choice(alpha, size=int(lens.sum())).astype(np.uint8)
    offs = np.concatenate([[0], np.cumsum(lens)])
    for ppw in (1, -1):
        _run(gpu, oracle_mod, small, data, offs, B.EncodeOptions(fused=-1, pieces_per_wave=ppw),
             label=f"deep grid, many tokens per piece, pieces_per_wave {ppw}")


def test_deep_grids_of_word_sized_pieces(gpu, oracle_mod):
    """4096 tiles of 256 pieces and more (the grids on which the emit workgroups take four tiles
    each): empty pieces, pieces of every other path in between, tile counts that are no multiple
    of four, a last tile that is not full, and every selection level."""
    _, B = gpu
    from test_oracle_encode import _random_p1_table
    rng = np.random.default_rng(4096)
    for trial, n_pieces in enumerate((4096 * 256, 4097 * 256 + 3, 4099 * 256 - 100, 4100 * 256 + 1)):
        alpha, merges = _random_p1_table(rng, int(rng.integers(2, 6)), int(rng.integers(5, 60)))
        lens = rng.integers(0, 17, size=n_pieces)
        lens[rng.integers(0, n_pieces, size=400)] = rng.integers(17, 65, size=400)
        lens[rng.integers(0, n_pieces, size=40)] = rng.integers(65, 1200, size=40)
        lens[rng.integers(0, n_pieces, size=4)] = rng.integers(2100, 5000, size=4)
        data = rng.choice(alpha, size=int(lens.sum())).astype(np.uint8)
        off = np.concatenate([[0], np.cumsum(lens)])
        opts = [None, B.EncodeOptions(selection_level=1), B.EncodeOptions(selection_level=2, tiny_max_len=9),
                B.EncodeOptions(selection_level=3, pieces_per_wave=64, fused=-1)][trial]
        _run(gpu, oracle_mod, merges, data, off, opts, label=f"deep grid of word-sized pieces {trial}")


@pytest.mark.parametrize("fused", [0, 2, -1, "all in the tile", "16 tiles per long-piece workgroup"])
def test_stress_exact(gpu, oracle_mod, fused):
    """Full 4 MB stress input at the default options (what bench.py runs): every id and
    every offset against the oracle, and on top of that the structural properties of the
    long pieces (they spell their bytes, no mergeable pair is left)."""
    torch, B = gpu
    from workloads import configs as C
    from helpers import expand_ids
    ev = C.make_eval("stress")
    merges = C.load_merges("t100k")
    data, off = ev["bytes"], ev["piece_offsets"]
    opts = {0: None, "all in the tile": B.EncodeOptions(long_groups=-1),
            "16 tiles per long-piece workgroup": B.EncodeOptions(long_groups=16)}.get(fused) if not isinstance(fused, int) or fused == 0 \
        else B.EncodeOptions(fused=fused)
    ids, out_off = _run(gpu, oracle_mod, merges, data, off, opts, label=f"stress fused={fused}")
    lens = np.diff(off)
    big = np.nonzero(lens > 512)[0]
    assert big.size > 10 and lens.max() == 4097
    rank = {(int(a), int(b)) for a, b in merges}
    for q in big:
        toks = ids[out_off[q]:out_off[q + 1]]
        assert expand_ids(toks, merges) == data[off[q]:off[q + 1]].tobytes()
        assert all((int(toks[i]), int(toks[i + 1])) not in rank for i in range(len(toks) - 1))
    assert out_off[-1] == ids.size


def test_two_runs_are_identical_and_workspace_is_reusable(gpu):
    torch, B = gpu
    from workloads import configs as C
    ev = C.make_eval("seq32k")
    table = B.Table(C.load_merges("t50k"))
    d, o = torch.from_numpy(ev["bytes"]).cuda(), torch.from_numpy(ev["piece_offsets"]).cuda()
    n_bytes, n_pieces = d.numel(), o.numel() - 1
    ws = torch.empty(B.bpe_workspace_bytes(n_bytes, n_pieces), dtype=torch.uint8, device="cuda")
    outs = []
    for fill, fused in ((0x00, 1), (0xFF, 1), (0x5A, 1), (0xFF, -1), (0x00, -1), (None, 1), (None, 0)):
        if fill is not None:
            ws.fill_(fill)      # workspace contents must not matter
        ids = torch.full((n_bytes,), -7, dtype=torch.int32, device="cuda")
        off = torch.full((n_pieces + 1,), -7, dtype=torch.int32, device="cuda")
        B.bpe_encode(table, d, o, ids, off, ws, B.EncodeOptions(fused=fused))
        assert B.bpe_encode_status(ws) == 0
        outs.append((ids.cpu().numpy(), off.cpu().numpy()))
    for ids, off in outs[1:]:
        assert (ids == outs[0][0]).all() and (off == outs[0][1]).all()
    total = outs[0][1][-1]
    assert (outs[0][0][total:] == -7).all()     # nothing written past the tokens


def test_pool_workspace(gpu, oracle_mod):
    import ctypes
    torch, B = gpu
    from workloads import configs as C
    ev = C.make_eval("tiny")
    merges = C.load_merges("t1k")
    table = B.Table(merges)
    d, o = torch.from_numpy(ev["bytes"]).cuda(), torch.from_numpy(ev["piece_offsets"]).cuda()
    pool = B.Pool(1 << 20, 1 << 18)
    assert pool.nbytes >= B.bpe_workspace_bytes(d.numel(), o.numel() - 1) and pool.ptr % 256 == 0
    ids = torch.empty(d.numel(), dtype=torch.int32, device="cuda")
    off = torch.empty(o.numel(), dtype=torch.int32, device="cuda")
    lib = B.load_library()
    for _ in range(3):
        rc = lib.bpe_encode(table._h, ctypes.c_void_p(d.data_ptr()), ctypes.c_void_p(o.data_ptr()),
                            d.numel(), o.numel() - 1, ctypes.c_void_p(ids.data_ptr()),
                            ctypes.c_void_p(off.data_ptr()), ctypes.c_void_p(pool.ptr), pool.nbytes, None,
                            ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0
    assert lib.bpe_encode_status(ctypes.c_void_p(pool.ptr), None) == 0
    want_ids, want_off = oracle_mod.encode(oracle_mod.Table(merges), ev["bytes"], ev["piece_offsets"])
    assert (off.cpu().numpy() == want_off).all()
    assert (ids.cpu().numpy()[: want_ids.size] == want_ids).all()
    # too-small workspace is refused on the host
    rc = lib.bpe_encode(table._h, ctypes.c_void_p(d.data_ptr()), ctypes.c_void_p(o.data_ptr()),
                        d.numel(), o.numel() - 1, ctypes.c_void_p(ids.data_ptr()),
                        ctypes.c_void_p(off.data_ptr()), ctypes.c_void_p(pool.ptr), 1024, None, None)
    assert rc == -8
    # the same pool serves the pre-tokenizer, the raw path and the decoder (sizes within its limits)
    n = d.numel()
    vp = ctypes.c_void_p
    assert pool.nbytes >= B.bpe_encode_raw_workspace_bytes(n, 1 << 18, 1)
    assert pool.nbytes >= B.bpe_pretokenize_workspace_bytes(n) and pool.nbytes >= B.bpe_decode_workspace_bytes(n)
    vocab = B.Vocab(merges)
    seq_tok = torch.empty(2, dtype=torch.int32, device="cuda")
    text = torch.empty(n, dtype=torch.uint8, device="cuda")
    poff = torch.empty((1 << 18) + 1, dtype=torch.int32, device="cuda")
    cnt = torch.empty(1, dtype=torch.int32, device="cuda")
    stream = vp(torch.cuda.current_stream().cuda_stream)
    ids.fill_(-1)
    assert lib.bpe_pretokenize(vp(d.data_ptr()), n, None, 0, vp(poff.data_ptr()), 1 << 18, vp(cnt.data_ptr()), None,
                               vp(pool.ptr), pool.nbytes, None, stream) == 0
    assert lib.bpe_encode_status(vp(pool.ptr), None) == 0 and int(cnt.item()) == o.numel() - 1
    assert lib.bpe_encode_raw(table._h, vp(d.data_ptr()), n, None, 0, 1 << 18, vp(ids.data_ptr()),
                              vp(seq_tok.data_ptr()), None, None, None, vp(pool.ptr), pool.nbytes, None, stream) == 0
    assert lib.bpe_encode_status(vp(pool.ptr), None) == 0
    assert seq_tok.tolist() == [0, want_ids.size] and (ids.cpu().numpy()[: want_ids.size] == want_ids).all()
    assert lib.bpe_decode(vocab._h, vp(ids.data_ptr()), want_ids.size, None, 0, vp(text.data_ptr()), n, None, None,
                          vp(pool.ptr), pool.nbytes, stream) == 0
    assert lib.bpe_encode_status(vp(pool.ptr), None) == 0 and (text.cpu().numpy() == ev["bytes"]).all()
    vocab.free()
    pool.destroy()


def test_no_call_of_the_serving_path_allocates(gpu):
    """Free device memory as the driver reports it (hipMemGetInfo: it sees every allocation of the
    process, the library's own included, which torch's counters do not) stays the same over
    loops of bpe_encode, bpe_encode_raw, bpe_pretokenize, bpe_decode and bpe_map_ids, on every
    kernel path the five workload shapes take."""
    torch, B = gpu
    from workloads import configs as C
    for name in ("tiny", "seq131k", "stress"):
        ev = C.make_eval(name)
        merges = C.load_merges(ev["table"])
        table = B.Table(merges)
        vocab = B.Vocab(merges, output_ids=np.arange(256 + merges.shape[0], dtype=np.int32)[::-1].copy())
        d, o = torch.from_numpy(ev["bytes"].copy()).cuda(), torch.from_numpy(ev["piece_offsets"].copy()).cuda()
        n, n_pieces = d.numel(), o.numel() - 1
        pool = B.Pool(n, n_pieces)
        ws = torch.empty(pool.nbytes, dtype=torch.uint8, device="cuda")     # same size, torch-owned, for the binding
        ids = torch.empty(n, dtype=torch.int32, device="cuda")
        off = torch.empty(n_pieces + 1, dtype=torch.int32, device="cuda")
        seq_tok = torch.empty(2, dtype=torch.int32, device="cuda")
        cnt = torch.empty(1, dtype=torch.int32, device="cuda")
        text = torch.empty(n, dtype=torch.uint8, device="cuda")
        stream = torch.cuda.current_stream()

        def calls():
            B.bpe_encode(table, d, o, ids, off, ws, None, stream)
            B.bpe_encode(table, d, o, ids, off, ws, B.EncodeOptions(fused=-1, selection_level=2), stream)
            B.bpe_pretokenize(d, None, off, cnt, None, ws, None, stream)
            B.bpe_encode_raw(table, d, None, ids, seq_tok, ws, n_pieces, None, None, None, None, stream)
            B.bpe_map_ids(vocab, ids, ids, True, seq_tok[1:], stream)
            B.bpe_decode(vocab, ids, text, ws, None, cnt, seq_tok[1:], True, stream)
        calls()                       # code objects are loaded and torch's pool is warm after the first round
        assert B.bpe_encode_status(ws) == 0
        free_before = torch.cuda.mem_get_info()[0]
        for _ in range(5):
            calls()
        assert B.bpe_encode_status(ws) == 0
        assert torch.cuda.mem_get_info()[0] == free_before, name
        assert bytes(text.cpu().numpy()) == ev["bytes"].tobytes()
        pool.destroy()
        table.free()
        vocab.free()


def test_forced_single_kernel_beyond_the_resident_grid_is_refused(gpu):
    torch, B = gpu
    table = B.Table([(97, 97)])
    d = torch.full((4000,), 97, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.BpeError) as e:        # one piece of 4000 bytes
        B.encode(table, d, torch.tensor([0, 4000], dtype=torch.int32, device="cuda"), B.EncodeOptions(fused=1))
    assert e.value.code == -10
    ids, _ = B.encode(table, d, torch.tensor([0, 4000], dtype=torch.int32, device="cuda"), B.EncodeOptions(fused=2))
    assert ids.numel() == 2000
    table.free()


def test_bad_offsets_are_reported_not_followed(gpu):
    torch, B = gpu
    table = B.Table([(97, 97)])
    d = torch.from_numpy(np.frombuffer(b"a" * 1000, dtype=np.uint8).copy()).cuda()
    for bad in ([0, 500, 400, 1000], [0, 2000, 1000], [0, -5, 1000], [10, 1000], [0, 900],
                [0, 600, 100, 700, 200, 800, 300, 900, 400, 1000]):
        for fused in (2, -1):
            o = torch.tensor(bad, dtype=torch.int32, device="cuda")
            _say(f"[case] bad offsets {bad} fused={fused}")
            with pytest.raises(B.BpeError) as e:
                B.encode(table, d, o, B.EncodeOptions(fused=fused))
            assert e.value.code == -11
    # and the workspace verdict resets on the next good call
    ids, off = B.encode(table, d, torch.tensor([0, 1000], dtype=torch.int32, device="cuda"))
    assert ids.numel() == 500


def test_calls_can_be_captured_in_a_graph(gpu, oracle_mod):
    """bpe_encode, bpe_encode_raw and bpe_decode only enqueue kernels, so a caller may
    record them into a HIP graph and replay it on new contents of the same buffers.
    Every replay, with eager work and synchronisations in between, must give what the
    oracle gives for the bytes of that replay (nothing of an earlier replay may be
    taken for this one's: the call id of a recorded call never changes)."""
    torch, B = gpu
    from workloads import configs as C
    for name in ("tiny", "seq131k"):
        ev = C.make_eval(name)
        merges = C.load_merges(ev["table"])
        ot = oracle_mod.Table(merges)
        table, vocab = B.Table(merges), B.Vocab(merges)
        host = ev["bytes"].copy()
        data = torch.from_numpy(host.copy()).cuda()
        off = torch.from_numpy(ev["piece_offsets"].copy()).cuda()
        n, n_pieces = data.numel(), off.numel() - 1
        out_ids = torch.zeros(n, dtype=torch.int32, device="cuda")
        out_off = torch.zeros(n_pieces + 1, dtype=torch.int32, device="cuda")
        raw_ids = torch.zeros(n, dtype=torch.int32, device="cuda")
        seq_tok = torch.zeros(2, dtype=torch.int32, device="cuda")
        text = torch.zeros(n, dtype=torch.uint8, device="cuda")
        n_text = torch.zeros(1, dtype=torch.int32, device="cuda")
        ws = torch.empty(B.bpe_workspace_bytes(n, n_pieces), dtype=torch.uint8, device="cuda")
        ws_raw = torch.empty(B.bpe_encode_raw_workspace_bytes(n, 0, 1), dtype=torch.uint8, device="cuda")
        ws_dec = torch.empty(B.bpe_decode_workspace_bytes(n), dtype=torch.uint8, device="cuda")
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            B.bpe_encode(table, data, off, out_ids, out_off, ws)
            B.bpe_encode_raw(table, data, None, raw_ids, seq_tok, ws_raw)
            # the token count is taken from the device, as a caller without a host round trip would
            B.bpe_decode(vocab, raw_ids, text, ws_dec, n_bytes=n_text, n_tokens_device=seq_tok[1:])
        torch.cuda.synchronize()
        for replay in range(5):
            print(f"[case] graph replay {replay} of {name}", flush=True)
            # new contents: other letters, and from the third replay on other pieces too
            cur = host.copy()
            cur[cur == 0x65] = 0x61 + replay
            if replay >= 2:
                cur[cur == 0x61 + replay + 3] = 0x20
            data.copy_(torch.from_numpy(cur).cuda())
            out_ids.fill_(-1); out_off.fill_(-1); raw_ids.fill_(-1); text.fill_(0)     # eager work in between
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert B.bpe_encode_status(ws) == 0 and B.bpe_encode_status(ws_raw) == 0 and B.bpe_encode_status(ws_dec) == 0
            want_ids, want_off = oracle_mod.encode(ot, cur, ev["piece_offsets"], n_threads=16)
            assert np.array_equal(out_off.cpu().numpy(), want_off)
            assert np.array_equal(out_ids.cpu().numpy()[:want_ids.size], want_ids)
            want_raw, want_seq, _, _ = oracle_mod.encode_raw(ot, cur, None, n_threads=16)
            assert seq_tok.tolist() == want_seq.tolist()
            assert np.array_equal(raw_ids.cpu().numpy()[:want_raw.size], want_raw)
            assert int(n_text.item()) == n and np.array_equal(text.cpu().numpy(), cur)
        table.free()
        vocab.free()


def test_a_reported_condition_is_cleared(gpu):
    """bpe_encode_status reports bad offsets once; the next status of the same,
    untouched workspace is clean, so replays of a recorded call are judged afresh."""
    torch, B = gpu
    table = B.Table([(97, 98)])
    data = torch.full((100,), 97, dtype=torch.uint8, device="cuda")
    bad = torch.tensor([0, 60, 40, 100], dtype=torch.int32, device="cuda")
    out_ids = torch.empty(100, dtype=torch.int32, device="cuda")
    out_off = torch.empty(4, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.bpe_workspace_bytes(100, 3), dtype=torch.uint8, device="cuda")
    B.bpe_encode(table, data, bad, out_ids, out_off, ws)
    assert B.bpe_encode_status(ws) == -11
    assert B.bpe_encode_status(ws) == 0
    table.free()


def test_status_of_a_workspace_no_call_has_used(gpu):
    """Fresh, zero-filled or otherwise filled memory: no verdict to report, and nothing is written."""
    torch, B = gpu
    for fill in (0x00, 0xFF, 0x5A):
        ws = torch.full((4096,), fill, dtype=torch.uint8, device="cuda")
        assert B.bpe_encode_status(ws) == 0
        assert (ws == fill).all()
    g = torch.Generator(device="cuda").manual_seed(5)
    ws = torch.randint(0, 256, (4096,), dtype=torch.uint8, device="cuda", generator=g)
    keep = ws.clone()
    assert B.bpe_encode_status(ws) == 0 and torch.equal(ws, keep)
