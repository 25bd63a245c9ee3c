"""Parity of the device decoder (bpe_decode) and of the id renumbering
(bpe_map_ids) against the CPU oracle, through the C ABI, byte for byte."""
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


def _decode(gpu, vocab, ids, capacity, misalign=0, want_offsets=True, n_device=None, output_ids=False):
    torch, B = gpu
    ids = np.ascontiguousarray(np.asarray(ids, dtype=np.int32))
    d_ids = torch.from_numpy(ids).cuda() if ids.size else torch.empty(0, dtype=torch.int32, device="cuda")
    buf = torch.full((capacity + misalign + 8,), 0xEE, dtype=torch.uint8, device="cuda")
    out = buf[misalign:misalign + capacity]
    tbo = torch.full((ids.size + 1,), -7, dtype=torch.int32, device="cuda") if want_offsets else None
    nb = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.bpe_decode_workspace_bytes(ids.size), dtype=torch.uint8, device="cuda")
    nd = None if n_device is None else torch.tensor([n_device], dtype=torch.int32, device="cuda")
    B.bpe_decode(vocab, d_ids, out, ws, tbo, nb, nd, output_ids)
    st = B.bpe_encode_status(ws)
    return buf.cpu().numpy(), None if tbo is None else tbo.cpu().numpy(), int(nb.item()), st


def _check(gpu, oracle_mod, merges, ids, label, ranks=None, merged_ids=None, slack=0, **kw):
    torch, B = gpu
    ids = np.asarray(ids, dtype=np.int32)
    print(f"[case] decode {label} n_tokens={ids.size} {kw}", flush=True)
    ot = oracle_mod.Table(merges, ranks, merged_ids)
    want = oracle_mod.decode(ot, ids)
    want_off = oracle_mod.token_byte_offsets(ot, ids)
    vocab = B.Vocab(merges, ranks, merged_ids)
    mis = kw.get("misalign", 0)
    buf, tbo, nb, st = _decode(gpu, vocab, ids, want.size + slack, **kw)
    assert st == 0
    assert nb == want.size
    assert np.array_equal(buf[mis:mis + want.size], want), \
        f"bytes differ first at {np.nonzero(buf[mis:mis + want.size] != want)[0][:5]}"
    assert (buf[:mis] == 0xEE).all() and (buf[mis + want.size:] == 0xEE).all(), "wrote outside the output"
    if tbo is not None:
        assert np.array_equal(tbo, want_off)
    vocab.free()


def test_worked_examples(gpu, oracle_mod):
    from test_oracle_decode import _examples
    for merges, toks, want, offs in _examples():
        _check(gpu, oracle_mod, merges, toks, f"worked {want!r}")
        _check(gpu, oracle_mod, merges, toks, f"worked {want!r}, misaligned", misalign=3, slack=5)


def test_sizes_and_alignments(gpu, oracle_mod):
    from workloads import configs as C
    merges = C.load_merges("t1k")
    rng = np.random.default_rng(31)
    for n in (0, 1, 2, 3, 4, 5, 255, 256, 257, 1023, 1024, 1025, 2048, 4097, 50000):
        ids = rng.integers(0, 256 + len(merges), size=n)
        for mis in (0, 1, 2, 3):
            _check(gpu, oracle_mod, merges, ids, f"{n} random tokens", misalign=mis, slack=mis)
    _check(gpu, oracle_mod, merges, rng.integers(0, 256, size=3000), "bytes only", want_offsets=False)


def test_round_trip_workloads(gpu, oracle_mod):
    from workloads import configs as C
    for name in ("tiny", "seq32k", "seq131k", "stress", "batch"):
        ev = C.make_eval(name)
        merges = C.load_merges(ev["table"])
        ids, _ = oracle_mod.encode(oracle_mod.Table(merges), ev["bytes"], ev["piece_offsets"], n_threads=16)
        torch, B = gpu
        vocab = B.Vocab(merges)
        buf, tbo, nb, st = _decode(gpu, vocab, ids, ev["bytes"].size)
        print(f"[case] round trip {name}: {ids.size} tokens -> {nb} bytes, longest token "
              f"{vocab.info['max_token_bytes']}", flush=True)
        assert st == 0 and nb == ev["bytes"].size
        assert np.array_equal(buf[:nb], ev["bytes"])
        vocab.free()


def test_long_tokens(gpu, oracle_mod):
    # doubling rules: token 256 + k is 2^(k+1) bytes; tiles of such tokens exceed the LDS stage
    merges = [(120, 120)] + [(256 + k, 256 + k) for k in range(13)]
    rng = np.random.default_rng(33)
    for n in (1, 7, 300, 1500, 3000):
        ids = rng.integers(256, 256 + 14, size=n)
        ids[rng.random(n) < 0.3] = 121
        _check(gpu, oracle_mod, merges, ids, f"{n} tokens of up to 16 KiB", misalign=n % 4)
    _check(gpu, oracle_mod, merges, [256 + 13] * 5 + [120] * 2000 + [256 + 6] * 70, "long and short tiles mixed")


def test_many_tokens_take_larger_tiles(gpu, oracle_mod):
    # above 512 Ki tokens a tile is 2 rounds of 1024 tokens, above 4 Mi tokens 4 rounds
    from workloads import configs as C
    merges = C.load_merges("t1k")
    ot = oracle_mod.Table(merges)
    rng = np.random.default_rng(41)
    torch, B = gpu
    vocab = B.Vocab(merges)
    for n in (512 * 1024 + 1, 700_001, 4096 * 1024 + 1, 4_400_003):
        ids = rng.integers(0, 256 + len(merges), size=n).astype(np.int32)
        ids[rng.integers(0, n, size=50)] = 256 + len(merges) - 1
        _check(gpu, oracle_mod, merges, ids, f"{n} random tokens", misalign=n % 4)
        # device-side count that ends inside a tile, inside a round, and at 0
        for n_dev in (n - 3000, 5, 0):
            want = oracle_mod.decode(ot, ids[:n_dev])
            buf, tbo, nb, st = _decode(gpu, vocab, ids, want.size + 100, n_device=n_dev)
            assert st == 0 and nb == want.size and np.array_equal(buf[:nb], want) and (buf[nb:] == 0xEE).all()
        # an output that is too small: nothing behind the capacity, the status says so
        want = oracle_mod.decode(ot, ids)
        buf, tbo, nb, st = _decode(gpu, vocab, ids, want.size - 70000)
        assert st == BPE_ERR_SIZE and nb == want.size - 70000 and (buf[want.size - 70000:] == 0xEE).all()
        assert np.array_equal(tbo, oracle_mod.token_byte_offsets(ot, ids))
    # long tokens in the larger tiles: rounds that do not fit the LDS stage
    merges2 = [(120, 120)] + [(256 + k, 256 + k) for k in range(9)]
    ids = rng.integers(256, 256 + 10, size=4_300_000)
    ids[rng.random(ids.size) < 0.97] = 120
    _check(gpu, oracle_mod, merges2, ids, "4.3 M tokens, some of 1 KiB", misalign=1)
    vocab.free()


def test_custom_ids(gpu, oracle_mod):
    merges = [(97, 98), (1000, 99), (70000, 70000)]
    _check(gpu, oracle_mod, merges, [70000, 1000, 97, 300, 300, 99], "sparse merged ids", ranks=[5, 9, 40],
           merged_ids=[1000, 70000, 300])


def test_device_side_token_count(gpu, oracle_mod):
    torch, B = gpu
    from workloads import configs as C
    merges = C.load_merges("t1k")
    ot = oracle_mod.Table(merges)
    rng = np.random.default_rng(35)
    ids = rng.integers(0, 256 + len(merges), size=5000)
    vocab = B.Vocab(merges)
    for n_dev in (0, 1, 1024, 1025, 4999, 5000, 9999, -3):
        n = min(max(n_dev, 0), 5000)
        want = oracle_mod.decode(ot, ids[:n])
        buf, tbo, nb, st = _decode(gpu, vocab, ids, 40000, n_device=n_dev)
        print(f"[case] device count {n_dev}", flush=True)
        assert st == 0 and nb == want.size and np.array_equal(buf[:nb], want) and (buf[nb:] == 0xEE).all()
        assert np.array_equal(tbo[:n + 1], oracle_mod.token_byte_offsets(ot, ids[:n])) and (tbo[n + 1:] == -7).all()
    vocab.free()


def test_output_too_small_is_reported(gpu, oracle_mod):
    torch, B = gpu
    merges = [(120, 120)] + [(256 + k, 256 + k) for k in range(8)]
    ot = oracle_mod.Table(merges)
    rng = np.random.default_rng(36)
    ids = rng.integers(255, 256 + 9, size=4000)
    ids[ids == 255] = 65
    want = oracle_mod.decode(ot, ids)
    vocab = B.Vocab(merges)
    for cap in (want.size, want.size - 1, want.size // 2, 5, 0):
        buf, tbo, nb, st = _decode(gpu, vocab, ids, cap)
        print(f"[case] capacity {cap} of {want.size} bytes -> status {st}", flush=True)
        if cap >= want.size:
            assert st == 0 and nb == want.size
        else:
            assert st == BPE_ERR_SIZE and nb == cap
        assert (buf[cap:] == 0xEE).all(), "wrote behind the capacity"
        # tiles that fit entirely are complete; offsets are always the true ones
        assert np.array_equal(tbo, oracle_mod.token_byte_offsets(ot, ids))
    vocab.free()


def test_unknown_ids_are_reported(gpu, oracle_mod):
    torch, B = gpu
    merges = [(97, 98), (300, 99)]
    vocab = B.Vocab(merges, merged_ids=[300, 500])
    for bad in (256, 299, 301, 501, -1, 2 ** 31 - 1, -2 ** 31):
        buf, tbo, nb, st = _decode(gpu, vocab, [97, 300, bad, 500, 98], 64)
        print(f"[case] unknown id {bad} -> status {st}", flush=True)
        assert st == BPE_ERR_INPUT
        assert buf[:nb].tobytes() == b"aab" + b"abc" + b"b"     # the unknown id contributes nothing
        assert tbo.tolist() == [0, 1, 3, 3, 6, 7]
    vocab.free()


def test_output_ids(gpu, oracle_mod):
    torch, B = gpu
    from workloads import configs as C
    ev = C.make_eval("tiny")
    merges = C.load_merges(ev["table"])
    n_ids = 256 + len(merges)
    rng = np.random.default_rng(37)
    output_ids = (rng.permutation(n_ids) + 1000).astype(np.int32)      # a renumbering with a gap below 1000
    vocab = B.Vocab(merges, output_ids=output_ids)
    assert vocab.info["has_output_ids"] == 1 and vocab.info["n_output_ids"] == int(output_ids.max()) + 1
    ids, _ = oracle_mod.encode(oracle_mod.Table(merges), ev["bytes"], ev["piece_offsets"])
    # internal -> output on the device, only the first n_device entries
    d_ids = torch.from_numpy(ids).cuda()
    d_out = torch.full((ids.size,), -7, dtype=torch.int32, device="cuda")
    n_dev = torch.tensor([ids.size - 10], dtype=torch.int32, device="cuda")
    B.bpe_map_ids(vocab, d_ids, d_out, True, n_dev)
    torch.cuda.synchronize()
    got = d_out.cpu().numpy()
    assert np.array_equal(got[:-10], oracle_mod.map_ids(ids[:-10], output_ids)) and (got[-10:] == -7).all()
    # decode straight from output ids
    ext = oracle_mod.map_ids(ids, output_ids)
    buf, tbo, nb, st = _decode(gpu, vocab, ext, ev["bytes"].size, output_ids=True)
    assert st == 0 and np.array_equal(buf[:nb], ev["bytes"])
    # and back, in place, with values the vocabulary does not know
    probe = np.concatenate([ext[:100], [0, 999, int(output_ids.max()) + 1, -5]]).astype(np.int32)
    d = torch.from_numpy(probe).cuda()
    B.bpe_map_ids(vocab, d, d, False)
    torch.cuda.synchronize()
    assert np.array_equal(d.cpu().numpy(), oracle_mod.map_ids(probe, output_ids, to_output_ids=False))
    assert d.cpu().numpy()[-4:].tolist() == [-1, -1, -1, -1]
    # unknown output ids are reported by the decoder
    buf, tbo, nb, st = _decode(gpu, vocab, [int(ext[0]), 5], 64, output_ids=True)
    assert st == BPE_ERR_INPUT
    vocab.free()
    plain = B.Vocab(merges)
    with pytest.raises(B.BpeError) as e:
        B.bpe_map_ids(plain, d, d, True)
    assert e.value.code == -10
    plain.free()


def test_vocab_build_errors(gpu):
    torch, B = gpu
    with pytest.raises(B.BpeError) as e:
        B.Vocab([(97, 98)], output_ids=np.arange(10))
    assert e.value.code == -2
    with pytest.raises(B.BpeError) as e:
        B.Vocab([(97, 98)], output_ids=np.zeros(257))
    assert e.value.code == -6
    with pytest.raises(B.BpeError) as e:      # a rule that uses an id made later
        B.Vocab([(256, 97), (97, 98)])
    assert e.value.code == -7
    # expansions that would not fit: 21 doublings = 2 MiB
    with pytest.raises(B.BpeError) as e:
        B.Vocab([(120, 120)] + [(256 + k, 256 + k) for k in range(21)])
    assert e.value.code == -2
