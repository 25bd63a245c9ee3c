"""The list-of-texts call of the paper's binding (section 3.7) on top of
bpe_encode_raw / bpe_decode, against the CPU oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _texts(rng, data, n):
    cuts = np.sort(rng.integers(0, data.size + 1, size=n - 1))
    b = np.concatenate([[0], cuts, [data.size]])
    return [data[b[k]:b[k + 1]].tobytes() for k in range(n)]


def test_tokenize_and_decode_batches(oracle_mod):
    import torch
    assert torch.cuda.is_available()
    import paper_2603_02597_amd as B
    from workloads import configs as C
    ev = C.make_eval("seq32k")
    merges = C.load_merges(ev["table"])
    ot = oracle_mod.Table(merges)
    rng = np.random.default_rng(51)
    n_ids = 256 + len(merges)
    output_ids = (rng.permutation(n_ids) + 7).astype(np.int32)
    for renumber in (False, True):
        tok = B.Tokenizer(merges, output_ids=output_ids if renumber else None)
        # batches of different sizes through the same object: buffers grow and are reused
        for n_texts, lo, hi in ((1, 0, 100), (5, 0, 3000), (300, 0, 200000), (40, 50000, 60000), (3, 0, 10)):
            data = ev["bytes"][lo:hi]
            texts = _texts(rng, data, n_texts) + [b"", "café naïve 中文"]
            got, ms = tok.tokenize_batch(texts)
            print(f"[case] {len(texts)} texts, {sum(len(t) for t in texts if isinstance(t, bytes))} bytes, "
                  f"renumbered={renumber}, kernels {ms * 1e3:.1f} us", flush=True)
            assert len(got) == len(texts) and ms >= 0
            for t, ids in zip(texts, got):
                raw = t.encode("utf-8") if isinstance(t, str) else t
                want, _, _, _ = oracle_mod.encode_raw(ot, np.frombuffer(raw, dtype=np.uint8))
                if renumber:
                    want = oracle_mod.map_ids(want, output_ids)
                assert np.array_equal(ids, want)
            back = tok.decode_batch(got)
            assert back == [t.encode("utf-8") if isinstance(t, str) else t for t in texts]
        assert tok.tokenize_batch([]) == ([], 0.0) and tok.decode_batch([]) == []
        tok.close()
    # tokens far longer than the first guess of the output size
    merges2 = [(120, 120)] + [(256 + k, 256 + k) for k in range(11)]
    tok = B.Tokenizer(merges2)
    ids, _ = tok.tokenize_batch([b"x" * 100000, b" " + b"x" * 4096])
    assert [len(a) for a in ids] == [len(oracle_mod.encode_raw(oracle_mod.Table(merges2), np.full(100000, 120, dtype=np.uint8))[0]), 2]
    assert tok.decode_batch(ids) == [b"x" * 100000, b" " + b"x" * 4096]
    tok.close()
