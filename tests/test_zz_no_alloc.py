"""bpe_encode_static, the entry point that allocates nothing (its workspace is an
array built into the library), against bpe_encode on the same inputs: two calls in a
row through the C ABI, the second on a smaller input, ids and offsets bit for bit, and
both against the oracle.  Collected last on purpose."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _free_device_bytes(torch):
    free, _ = torch.cuda.mem_get_info()
    return free


def test_static_entry_point_matches_bpe_encode(oracle_mod):
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    import paper_2603_02597_amd as B
    from workloads import configs as C
    lib = B.load_library()
    vp = ctypes.c_void_p
    merges = C.load_merges("t50k")
    table = B.Table(merges)
    ot = oracle_mod.Table(merges)
    big, small = C.make_eval("seq131k"), C.make_eval("seq32k")
    stream = vp(torch.cuda.current_stream().cuda_stream)

    # every buffer of both calls exists before the first one: the calls themselves must not allocate
    bufs = []
    for ev in (big, small):
        d = torch.from_numpy(ev["bytes"].copy()).cuda()
        o = torch.from_numpy(ev["piece_offsets"].copy()).cuda()
        n, n_pieces = d.numel(), o.numel() - 1
        assert B.bpe_workspace_bytes(n, n_pieces) <= B.STATIC_SCRATCH_BYTES
        ws = torch.empty(B.bpe_workspace_bytes(n, n_pieces), dtype=torch.uint8, device="cuda")
        outs = [torch.full((n,), -3, dtype=torch.int32, device="cuda") for _ in range(2)]
        offs = [torch.full((n_pieces + 1,), -3, dtype=torch.int32, device="cuda") for _ in range(2)]
        bufs.append((ev, d, o, n, n_pieces, ws, outs, offs))
    torch.cuda.synchronize()

    for call, (ev, d, o, n, n_pieces, ws, outs, offs) in enumerate(bufs):   # the larger input first, then the smaller one
        print(f"[case] bpe_encode_static n_bytes={n} n_pieces={n_pieces}", flush=True)
        free_before = _free_device_bytes(torch)
        rc = lib.bpe_encode_static(table._h, vp(d.data_ptr()), vp(o.data_ptr()), n, n_pieces, vp(outs[0].data_ptr()),
                                   vp(offs[0].data_ptr()), None, stream)
        assert rc == 0, lib.bpe_last_error()
        assert lib.bpe_encode_status(None, stream) == 0
        # (the first call on a device may make the runtime load the library's code object, array included)
        assert call == 0 or _free_device_bytes(torch) == free_before, "bpe_encode_static changed the free device memory"
        rc = lib.bpe_encode(table._h, vp(d.data_ptr()), vp(o.data_ptr()), n, n_pieces, vp(outs[1].data_ptr()),
                            vp(offs[1].data_ptr()), vp(ws.data_ptr()), ws.numel(), None, stream)
        assert rc == 0 and lib.bpe_encode_status(vp(ws.data_ptr()), stream) == 0
        got_ids, got_off = outs[0].cpu().numpy(), offs[0].cpu().numpy()
        ref_ids, ref_off = outs[1].cpu().numpy(), offs[1].cpu().numpy()
        assert np.array_equal(got_off, ref_off) and np.array_equal(got_ids, ref_ids)   # incl. the untouched tail
        want_ids, want_off = oracle_mod.encode(ot, ev["bytes"], ev["piece_offsets"], n_threads=16)
        assert np.array_equal(got_off, want_off) and np.array_equal(got_ids[:want_ids.size], want_ids)
        assert (got_ids[want_ids.size:] == -3).all()

    # bad offsets are reported through the built-in array's status block, once
    bad = torch.tensor([0, 60, 40, 100], dtype=torch.int32, device="cuda")
    ev, d, o, n, n_pieces, ws, outs, offs = bufs[1]
    rc = lib.bpe_encode_static(table._h, vp(d.data_ptr()), vp(bad.data_ptr()), 100, 3, vp(outs[0].data_ptr()),
                               vp(offs[0].data_ptr()), None, stream)
    assert rc == 0 and lib.bpe_encode_status(None, stream) == -11 and lib.bpe_encode_status(None, stream) == 0

    # beyond the array: refused on the host, nothing launched
    ev = C.make_eval("batch")
    n, n_pieces = ev["bytes"].size, ev["piece_offsets"].size - 1
    assert B.bpe_workspace_bytes(n, n_pieces) > B.STATIC_SCRATCH_BYTES
    rc = lib.bpe_encode_static(table._h, vp(d.data_ptr()), vp(o.data_ptr()), n, n_pieces, vp(outs[0].data_ptr()),
                               vp(offs[0].data_ptr()), None, stream)
    assert rc == -2 and b"16777216" in lib.bpe_last_error()
    table.free()
