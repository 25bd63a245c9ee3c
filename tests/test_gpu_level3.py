"""Selection level 3 (every pair that greedy is bound to merge, per pass) on the
long-piece paths, through the C ABI, bit for bit against the CPU oracle: pieces
that span many words (text cut into fixed chunks, the regime of the paper's own
pipeline, section 3.1), runs, the stress mix, and the sizes around the limits of
the LDS-resident and the windowed passes."""
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


def _check(gpu, oracle_mod, merges, data, off, label, **kw):
    torch, B = gpu
    data = np.array(data, dtype=np.uint8)
    off = np.ascontiguousarray(np.asarray(off, dtype=np.int32))
    print(f"[case] level 3 {label} n_bytes={data.size} n_pieces={off.size - 1} {kw}", flush=True)
    merges = np.asarray(merges, dtype=np.int32).reshape(-1, 2)
    want_ids, want_off = oracle_mod.encode(oracle_mod.Table(merges), data, off, n_threads=16)
    gt = B.Table(merges)
    opts = dict(selection_level=3)
    opts.update(kw)
    ids, out_off = B.encode(gt, torch.from_numpy(data).cuda(), torch.from_numpy(off).cuda(), B.EncodeOptions(**opts))
    got_ids, got_off = ids.cpu().numpy(), out_off.cpu().numpy()
    assert np.array_equal(got_off, want_off), f"offsets differ first at {np.nonzero(got_off != want_off)[0][:5]}"
    assert np.array_equal(got_ids, want_ids), f"ids differ first at {np.nonzero(got_ids != want_ids)[0][:5]}"
    gt.free()


LONG_ONLY = dict(tiny_max_len=-1, wave_max_len=-1)                          # one wavefront <= 512 symbols, else the workgroup
GROUP_ONLY = dict(tiny_max_len=-1, wave_max_len=-1, wave_lds_max_len=-1)    # the workgroup for everything
WINDOWS = dict(tiny_max_len=-1, wave_max_len=-1, wave_lds_max_len=-1, lds_max_len=2)   # windows of 320 symbols that decide 62


def test_worked_examples_and_edges(gpu, oracle_mod):
    from test_oracle_encode import _parse_examples
    for kw in (dict(), LONG_ONLY, GROUP_ONLY, WINDOWS):
        for data, merges, expect in _parse_examples():
            if merges:
                _check(gpu, oracle_mod, merges, np.frombuffer(data, dtype=np.uint8), [0, len(data)], f"worked {data!r}", **kw)
        merges = [(97, 97), (256, 256), (257, 257), (97, 98), (98, 97), (256, 97)]
        u8 = lambda b: np.frombuffer(b, dtype=np.uint8)
        _check(gpu, oracle_mod, merges, u8(b""), [0], "no piece", **kw)
        _check(gpu, oracle_mod, merges, u8(b""), [0, 0, 0], "empty pieces", **kw)
        _check(gpu, oracle_mod, merges, u8(b"aaab"), [0, 0, 1, 1, 1, 4, 4], "empty pieces around", **kw)
        for n in (1, 2, 3, 61, 62, 63, 64, 65, 123, 124, 125, 319, 320, 321, 381, 382, 383, 511, 512, 513, 639, 640, 641, 1000, 2051, 2052, 2053, 2054,
                  4063, 4064, 4065, 4104, 4105, 10000):
            _check(gpu, oracle_mod, merges, u8(b"a" * n), [0, n], f"run {n}", **kw)
            _check(gpu, oracle_mod, merges, u8(b"ab" * n), [0, n, 2 * n], f"two pieces of {n}", **kw)


@pytest.mark.parametrize("name", ["tiny", "seq32k"])
def test_chunked_text(gpu, oracle_mod, name):
    from workloads import configs as C, textgen
    ev = C.make_eval(name)
    merges = C.load_merges(ev["table"])
    data = ev["bytes"]
    sizes = (1, 2, 7, 17, 64, 65, 100, 512, 513, 640, 641, 1000, 2052, 2053, 4096, 9000, 70000) if name == "tiny" else \
            (300, 2052, 2053, 5000, 10000)
    for chunk in sizes:
        off = textgen.fixed_chunks(data.size, chunk)
        _check(gpu, oracle_mod, merges, data, off, f"{name} chunks of {chunk}")
        _check(gpu, oracle_mod, merges, data, off, f"{name} chunks of {chunk}", **GROUP_ONLY)
        if chunk <= 9000:
            _check(gpu, oracle_mod, merges, data, off, f"{name} chunks of {chunk}", **WINDOWS)


def test_few_long_pieces_at_every_level(gpu, oracle_mod):
    """A few pieces of several KiB each take the workgroup of 16 wavefronts: all
    selection levels, resident and in windows, text and runs."""
    from workloads import configs as C, textgen
    ev = C.make_eval("seq32k")
    merges = C.load_merges(ev["table"])
    data = ev["bytes"][:60000].copy()
    data[20000:26000] = ord("a")              # a run inside the text
    data[40000:40003] = ord("b")
    for chunk in (3000, 4032, 4033, 8064, 8065, 20000):
        off = textgen.fixed_chunks(data.size, chunk)
        for level in (0, 1, 2, 3):
            if level == 1 and chunk > 8064:
                continue                      # one merge per pass over 20,000 symbols: minutes of nothing new
            _check(gpu, oracle_mod, merges, data, off, f"chunks of {chunk}, level {level}", selection_level=level)
            _check(gpu, oracle_mod, merges, data, off, f"chunks of {chunk}, level {level}, small windows",
                   selection_level=level, lds_max_len=2)


def test_workloads_in_full(gpu, oracle_mod):
    from workloads import configs as C
    for name in ("tiny", "seq32k", "stress"):
        ev = C.make_eval(name)
        merges = C.load_merges(ev["table"])
        _check(gpu, oracle_mod, merges, ev["bytes"], ev["piece_offsets"], name)
        _check(gpu, oracle_mod, merges, ev["bytes"], ev["piece_offsets"], name, fused=-1, pieces_per_wave=16)
        # the default choice (level 3, runs by the best rank) and the best-rank passes for everything
        _check(gpu, oracle_mod, merges, ev["bytes"], ev["piece_offsets"], name, selection_level=0)
        _check(gpu, oracle_mod, merges, ev["bytes"], ev["piece_offsets"], name, selection_level=2)


def test_random_bytes_and_runs_in_long_pieces(gpu, oracle_mod):
    """Pieces of thousands of symbols over a few letters: ties, runs and dense rules."""
    from test_oracle_encode import _random_p1_table
    rng = np.random.default_rng(77)
    for trial in range(24):
        alpha, merges = _random_p1_table(rng, int(rng.integers(2, 6)), int(rng.integers(1, 60)))
        lens = np.concatenate([rng.integers(0, 100, size=40), rng.integers(400, 600, size=6),
                               rng.integers(1900, 2200, size=4), rng.integers(4000, 12000, size=2)])
        rng.shuffle(lens)
        parts = []
        for n in lens:
            if rng.random() < 0.3:       # runs of random lengths
                reps = rng.integers(1, 40, size=int(n) + 1)
                syms = rng.choice(alpha, size=int(n) + 1)
                parts.append(np.repeat(syms, reps)[:int(n)])
            else:
                parts.append(rng.choice(alpha, size=int(n)))
        data = np.concatenate(parts).astype(np.uint8)
        off = np.concatenate([[0], np.cumsum(lens)])
        kw = [dict(), LONG_ONLY, GROUP_ONLY, WINDOWS][trial % 4]
        _check(gpu, oracle_mod, merges, data, off, f"random long pieces {trial}", **kw)


def test_raw_path_chooses_its_tiles_for_long_pieces(gpu, oracle_mod):
    """bpe_encode_raw on text without spaces, cut into sequences: the pieces are the
    sequences, and the kernels choose the pieces per wavefront on the device."""
    torch, B = gpu
    from workloads import configs as C
    ev = C.make_eval("seq32k")
    merges = C.load_merges(ev["table"])
    data = ev["bytes"].copy()
    data[data == 0x20] = ord("e")
    ot, gt = oracle_mod.Table(merges), B.Table(merges)
    d = torch.from_numpy(data).cuda()
    for seq_len, cap in ((40, 0), (300, 0), (300, 4000), (3000, 100), (3000, 0), (100000, 0)):
        if seq_len == 100000:       # one piece of 20,000 bytes and plain text after it
            data2 = np.concatenate([data[:20000], ev["bytes"][20000:60000]])
            seq = np.array([0, data2.size], dtype=np.int32)
            d2 = torch.from_numpy(data2).cuda()
        else:
            data2, d2 = data, d
            seq = np.concatenate([np.arange(0, data.size, seq_len), [data.size]]).astype(np.int32)
        print(f"[case] raw path, sequences of {seq_len} bytes without spaces, max_pieces={cap}", flush=True)
        want_ids, want_seq, _, _ = oracle_mod.encode_raw(ot, data2, seq, n_threads=16)
        n_seqs = seq.size - 1
        ws = torch.empty(B.bpe_encode_raw_workspace_bytes(data2.size, cap, n_seqs), dtype=torch.uint8, device="cuda")
        ids = torch.empty(data2.size, dtype=torch.int32, device="cuda")
        seq_tok = torch.empty(n_seqs + 1, dtype=torch.int32, device="cuda")
        B.bpe_encode_raw(gt, d2, torch.from_numpy(seq).cuda(), ids, seq_tok, ws, max_pieces=cap)
        assert B.bpe_encode_status(ws) == 0
        got_seq = seq_tok.cpu().numpy()
        assert np.array_equal(got_seq, want_seq)
        assert np.array_equal(ids.cpu().numpy()[:want_ids.size], want_ids)
    gt.free()
