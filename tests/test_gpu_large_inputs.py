"""Inputs close to the 2^31-byte limit of the interface: the pre-tokenizer, the
raw encode path and the decoder on 2.1 GB of text.  The oracle cannot encode
that much in a test, so the expected values come from what holds at any size:
the text is the batch workload repeated, so its piece starts are the space
bytes (numpy's flatnonzero), and every repetition must encode to the ids the
oracle gives for one."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def test_two_gigabytes_of_text(oracle_mod):
    import torch
    import paper_2603_02597_amd as B
    from workloads import configs as C
    B.load_library()
    ev = C.make_eval("batch")
    unit = ev["bytes"]
    assert unit[0] == 0x20                      # so that a repetition begins a piece
    reps = (2**31 - 2) // unit.size             # 158 repetitions, 2,134,612,864 bytes
    n = reps * unit.size
    merges = C.load_merges(ev["table"])
    ref_ids, ref_off = oracle_mod.encode(oracle_mod.Table(merges), unit, ev["piece_offsets"], n_threads=16)
    pieces_per_rep, tokens_per_rep = ev["piece_offsets"].size - 1, ref_ids.size
    n_pieces, n_tokens = reps * pieces_per_rep, reps * tokens_per_rep
    _say(f"[case] {n} bytes, {n_pieces} pieces, {n_tokens} tokens expected")

    data = torch.from_numpy(unit.copy()).cuda().repeat(reps)
    assert data.numel() == n

    # pre-tokenizer alone, with the exact capacity
    off = torch.empty(n_pieces + 1, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.bpe_pretokenize_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    B.bpe_pretokenize(data, None, off, cnt, None, ws)
    assert B.bpe_encode_status(ws) == 0
    assert int(cnt.item()) == n_pieces
    unit_off = torch.from_numpy(ev["piece_offsets"][:-1].astype(np.int64)).cuda()
    for r in (0, 1, reps // 2, reps - 1):       # whole repetitions, compared on the device
        got = off[r * pieces_per_rep:(r + 1) * pieces_per_rep].to(torch.int64)
        assert torch.equal(got, unit_off + r * unit.size), f"piece offsets of repetition {r} differ"
    assert int(off[-1].item()) == n
    # all of them against numpy's own scan of one repetition, shifted (int32 arithmetic must not wrap)
    steps = off[1:].to(torch.int64) - off[:-1].to(torch.int64)
    assert int(steps.min().item()) >= 1 and int(steps.sum().item()) == n
    del steps, ws, off, cnt
    _say("[step] pre-tokenizer done")

    # raw path: sequences = repetitions
    seq = torch.arange(0, reps + 1, dtype=torch.int64, device="cuda") * unit.size
    seq = seq.to(torch.int32)
    out_ids = torch.empty(n, dtype=torch.int32, device="cuda")
    seq_tok = torch.empty(reps + 1, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.bpe_encode_raw_workspace_bytes(n, n_pieces, reps), dtype=torch.uint8, device="cuda")
    table = B.Table(merges)
    B.bpe_encode_raw(table, data, seq, out_ids, seq_tok, ws, max_pieces=n_pieces)
    assert B.bpe_encode_status(ws) == 0
    want_tok = torch.arange(0, reps + 1, dtype=torch.int64, device="cuda") * tokens_per_rep
    assert torch.equal(seq_tok.to(torch.int64), want_tok)
    ref = torch.from_numpy(ref_ids).cuda()
    for r in range(reps):
        assert torch.equal(out_ids[r * tokens_per_rep:(r + 1) * tokens_per_rep], ref), f"ids of repetition {r} differ"
    del ws
    _say("[step] raw encode done")

    # and back
    vocab = B.Vocab(merges)
    ids = out_ids[:n_tokens]
    text = torch.empty(n, dtype=torch.uint8, device="cuda")
    nb = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.bpe_decode_workspace_bytes(n_tokens), dtype=torch.uint8, device="cuda")
    B.bpe_decode(vocab, ids, text, ws, None, nb)
    assert B.bpe_encode_status(ws) == 0 and int(nb.item()) == n
    assert torch.equal(text, data)
    _say("[step] decode done")
    vocab.free()
    table.free()
