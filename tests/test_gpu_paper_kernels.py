"""The paper's own kernels (option paper_kernel: section 3.4 baseline, section
3.5 optimized; one workgroup per chunk, one merge per pass) against the CPU
oracle on the same chunk offsets, through the C ABI, bit for bit."""
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


def _check(gpu, oracle_mod, merges, data, off, variant, label, **kw):
    torch, B = gpu
    data = np.array(data, dtype=np.uint8)
    off = np.ascontiguousarray(np.asarray(off, dtype=np.int32))
    print(f"[case] paper kernel {variant} {label} n_bytes={data.size} n_chunks={off.size - 1} {kw}", flush=True)
    merges = np.asarray(merges, dtype=np.int32).reshape(-1, 2)
    want_ids, want_off = oracle_mod.encode(oracle_mod.Table(merges), data, off, n_threads=16)
    gt = B.Table(merges)
    ids, out_off = B.encode(gt, torch.from_numpy(data).cuda(), torch.from_numpy(off).cuda(),
                            B.EncodeOptions(paper_kernel=variant, **kw))
    got_ids, got_off = ids.cpu().numpy(), out_off.cpu().numpy()
    assert np.array_equal(got_off, want_off), f"offsets differ first at {np.nonzero(got_off != want_off)[0][:5]}"
    assert np.array_equal(got_ids, want_ids), f"ids differ first at {np.nonzero(got_ids != want_ids)[0][:5]}"
    gt.free()


@pytest.mark.parametrize("variant", [1, 2])
def test_worked_examples_and_edges(gpu, oracle_mod, variant):
    from test_oracle_encode import _parse_examples
    for data, merges, expect in _parse_examples():
        if merges:
            _check(gpu, oracle_mod, merges, np.frombuffer(data, dtype=np.uint8), [0, len(data)], variant,
                   f"worked {data!r}")
    merges = [(97, 97), (256, 256), (257, 257), (97, 98), (98, 97)]
    u8 = lambda b: np.frombuffer(b, dtype=np.uint8)
    _check(gpu, oracle_mod, merges, u8(b""), [0], variant, "no chunk")
    _check(gpu, oracle_mod, merges, u8(b""), [0, 0, 0], variant, "empty chunks")
    _check(gpu, oracle_mod, merges, u8(b"aaab"), [0, 0, 1, 1, 1, 4, 4], variant, "empty chunks around")
    # around one symbol per thread (256), where the baseline kernel switches its compaction
    for n in (1, 2, 3, 255, 256, 257, 258, 511, 512, 513, 1000):
        _check(gpu, oracle_mod, merges, u8(b"a" * n), [0, n], variant, f"run {n}")
        _check(gpu, oracle_mod, merges, u8(b"ab" * n), [0, n, 2 * n], variant, f"two chunks of {n}")


@pytest.mark.parametrize("variant", [1, 2])
def test_chunked_text(gpu, oracle_mod, variant):
    from workloads import configs as C, textgen
    ev = C.make_eval("tiny")
    merges = C.load_merges(ev["table"])
    data = ev["bytes"]
    for chunk in (1, 2, 7, 100, 255, 256, 257, 1000, 4096):
        _check(gpu, oracle_mod, merges, data, textgen.fixed_chunks(data.size, chunk), variant, f"chunks of {chunk}")
    # the pieces of the pre-tokenizer as chunks
    _check(gpu, oracle_mod, merges, data, ev["piece_offsets"], variant, "pieces as chunks")
    ev = C.make_eval("seq32k")
    merges = C.load_merges(ev["table"])
    data = ev["bytes"][:60000]
    # around the LDS budget of 4,104 symbols, and in the workspace beyond it
    for chunk in (2048, 4104, 4105, 9000):
        _check(gpu, oracle_mod, merges, data, textgen.fixed_chunks(data.size, chunk), variant, f"chunks of {chunk}")
    _check(gpu, oracle_mod, merges, data[:5000], textgen.fixed_chunks(5000, 700), variant, "LDS budget of 300",
           lds_max_len=300)


def test_stress_pieces_as_chunks(gpu, oracle_mod):
    from workloads import configs as C
    ev = C.make_eval("stress")
    merges = C.load_merges(ev["table"])
    # a slice with random-byte pieces and long runs
    off = ev["piece_offsets"]
    hi = int(np.searchsorted(off, 150000))
    for variant in (1, 2):
        _check(gpu, oracle_mod, merges, ev["bytes"][:off[hi]], off[:hi + 1], variant, "stress slice")


def test_not_available_on_the_raw_path(gpu):
    torch, B = gpu
    gt = B.Table([(97, 98)])
    d = torch.zeros(10, dtype=torch.uint8, device="cuda")
    out = torch.empty(10, dtype=torch.int32, device="cuda")
    tok = torch.empty(2, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.bpe_encode_raw_workspace_bytes(10, 0, 1), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.BpeError) as e:
        B.bpe_encode_raw(gt, d, None, out, tok, ws, opts=B.EncodeOptions(paper_kernel=1))
    assert e.value.code == -10
    gt.free()
