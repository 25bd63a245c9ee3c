"""Host-side checks of the C-ABI library that need no GPU: exported symbols,
argument validation, the hash-table image."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2603_02597_amd as B
from paper_2603_02597_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "bpe_mi355x.h")).read()
    declared = set(re.findall(r"\b(bpe_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    lib = ctypes.CDLL(B.library_path()) if os.path.exists(B.library_path()) else B.load_library()
    for name in declared:
        assert hasattr(lib, name), name


def test_product_code_never_reaches_for_the_oracle():
    pkg = os.path.join(ROOT, "paper_2603_02597_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"(import\s+oracle|from\s+oracle|liboracle|oracle/)", text), f


def _seed(attempt):
    base = [0x9E3779, 0x85EBCB, 0xC2B2AF, 0x27D4EB]
    step = [0x1234, 0x0F1E, 0x2B5C, 0x3A96]
    return [(b + s * 2 * attempt) & 0xFFFFFF for b, s in zip(base, step)]


def _slot_lookup(slots, info, a, b):
    """Two-choice lookup as the header documents it; returns (rank order, merged) or None."""
    half = slots.shape[0] // 2
    shift = 24 - (half.bit_length() - 1)
    k1a, k1b, k2a, k2b = _seed(info["hash_attempt"])
    h1 = ((((a + b * k1b) & 0xFFFFFF) * k1a) & 0xFFFFFF) >> shift
    h2 = half + (((((a + b * k2b) & 0xFFFFFF) * k2a) & 0xFFFFFF) >> shift)
    key = (a << 32) | b
    for idx in (h1, h2):
        if int(slots[idx, 0]) == key:
            v = int(slots[idx, 1])
            return v & 0x3FFFFFF, v >> 32          # rank order (low 26 bits), merged id
    return None


def test_table_image_finds_every_key_and_no_other():
    from workloads import configs as C
    merges = C.load_merges("t1k")
    slots, info = B.bpe_table_image_build(merges)
    assert info["n_merges"] == 1000 and info["capacity"] == 131072 == B.bpe_table_capacity(1000)
    assert info["max_id"] == 1255
    assert int((slots[:, 0] != 0xFFFFFFFFFFFFFFFF).sum()) == 1000
    for k, (a, b) in enumerate(merges):
        assert _slot_lookup(slots, info, int(a), int(b)) == (k, 256 + k)
    present = {(int(a), int(b)) for a, b in merges}
    rng = np.random.default_rng(3)
    for a, b in rng.integers(0, 1256, size=(3000, 2)):
        if (int(a), int(b)) not in present:
            assert _slot_lookup(slots, info, int(a), int(b)) is None


def test_slot_index_and_key_rest_name_the_key():
    # A device slot keeps the low bits of the mix and the right id: with the slot index that must
    # determine the left id, i.e. the mix (mod 2^24) is a bijection of the left id for a fixed
    # right id, for every multiplier set.
    a = np.arange(1 << 24, dtype=np.uint64)
    for attempt, b in ((0, 0), (0, 0xFFFFFF), (3, 50255), (15, 77)):
        for ka, kb in (_seed(attempt)[:2], _seed(attempt)[2:]):
            assert ka % 2 == 1
            m = (((a + np.uint64(b * kb)) & np.uint64(0xFFFFFF)) * np.uint64(ka)) & np.uint64(0xFFFFFF)
            seen = np.zeros(1 << 24, dtype=bool)
            seen[m] = True
            assert seen.all()


def test_large_tables_place_every_key():
    from workloads import configs as C
    for name in ["t50k", "t100k"]:
        merges = C.load_merges(name)
        slots, info = B.bpe_table_image_build(merges)
        assert 5 * info["n_merges"] <= 2 * info["capacity"] <= 10 * info["n_merges"] and info["hash_attempt"] < 16
        keys = (merges[:, 0].astype(np.uint64) << np.uint64(32)) | merges[:, 1].astype(np.uint64)
        stored = slots[:, 0][slots[:, 0] != np.uint64(0xFFFFFFFFFFFFFFFF)]
        assert np.array_equal(np.sort(stored), np.sort(keys))
        for k in range(0, len(merges), 997):
            assert _slot_lookup(slots, info, int(merges[k, 0]), int(merges[k, 1])) == (k, 256 + k)


def test_small_and_dense_tables_place_every_key():
    # Few index bits were the hash's weak spot (pairs that share one id and have neighbouring
    # other ids fell into the same slot of both halves): small random tables and complete
    # blocks of pairs must all be placed, and with the first multiplier set.
    from test_oracle_encode import _random_p1_table
    rng = np.random.default_rng(11)
    for _ in range(400):
        _, merges = _random_p1_table(rng, int(rng.integers(2, 6)), int(rng.integers(1, 60)))
        _, info = B.bpe_table_image_build(merges)
        assert info["hash_attempt"] == 0 and info["capacity"] == 131072
    for n_ids in (2, 3, 4, 7, 10, 15, 40, 100):
        ids = range(256 - n_ids, 256)
        merges = np.array([(a, b) for a in ids for b in ids], dtype=np.int32)
        slots, info = B.bpe_table_image_build(merges)
        assert info["hash_attempt"] == 0
        for k in range(0, len(merges), max(1, len(merges) // 50)):
            assert _slot_lookup(slots, info, int(merges[k, 0]), int(merges[k, 1])) == (k, 256 + k)
    assert B.bpe_table_capacity(0) == B.bpe_table_capacity(52428) == 131072 and B.bpe_table_capacity(52429) == 262144


def test_rank_word_flags_say_where_a_merged_id_can_occur():
    # rules: (a,b)->256, (256,c)->257, (d,257)->258 : 256 is a left part, 257 a right part, 258 neither
    slots, info = B.bpe_table_image_build([[97, 98], [256, 99], [100, 257]])
    words = {int(s[1]) >> 32: (int(s[1]) >> 30) & 3 for s in slots if int(s[0]) != 0xFFFFFFFFFFFFFFFF}
    assert words == {256: 1, 257: 2, 258: 0}


def test_custom_ranks_and_ids_in_the_image():
    slots, info = B.bpe_table_image_build([[97, 98], [98, 99]], ranks=[7, 3], merged_ids=[1000, 2000])
    assert _slot_lookup(slots, info, 97, 98) == (1, 1000)      # rank 7 is second in rank order
    assert _slot_lookup(slots, info, 98, 99) == (0, 2000)
    assert info["max_id"] == 2000


@pytest.mark.parametrize("merges,ranks,ids,code", [
    ([[97, 98], [97, 98]], None, None, -4),            # duplicate pair
    ([[97, 98], [98, 99]], [0, 0], None, -5),          # duplicate rank
    ([[97, 98], [98, 99]], [0, -1], None, -5),         # negative rank
    ([[97, 98], [98, 99]], None, [300, 300], -6),      # duplicate merged id
    ([[97, 98], [98, 99]], None, [300, 255], -3),      # merged id collides with a byte
    ([[97, 98]], None, [1 << 24], -3),                 # merged id too large for the hash
    ([[97, 256]], None, None, -7),                     # uses the id it makes
    ([[257, 97], [97, 98]], None, None, -7),           # uses an id made later
    ([[97, 9999]], None, None, -3),                    # unknown id
    ([[-1, 97]], None, None, -3),                      # negative id
])
def test_table_validation_errors(merges, ranks, ids, code):
    with pytest.raises(B.BpeError) as e:
        B.bpe_table_image_build(merges, ranks, ids)
    assert e.value.code == code
    assert len(str(e.value)) > 20


def test_workspace_bytes_is_a_pure_function_of_the_sizes():
    lib = B.load_library()
    assert B.bpe_workspace_bytes(0, 0) > 0
    a, b = B.bpe_workspace_bytes(1000, 100), B.bpe_workspace_bytes(2000, 100)
    assert b > a and a % 256 == 0
    assert B.bpe_workspace_bytes(10**6, 10**5) <= 8 * 10**6 + 24 * 10**5 + 4096     # 8 B per byte, 24 B per piece
    assert lib.bpe_workspace_bytes(-1, 0) == -2
    assert lib.bpe_workspace_bytes(2**31, 0) == -2


def test_encode_rejects_bad_arguments_before_touching_the_gpu():
    lib = B.load_library()
    null = ctypes.c_void_p(0)
    rc = lib.bpe_encode(null, null, null, 0, 0, null, null, null, 0, None, null)
    assert rc == -1 and b"null" in lib.bpe_last_error()
    assert lib.bpe_table_build(null, null, null, 0, None) == -1
    assert lib.bpe_pool_create(-5, 0, ctypes.byref(ctypes.c_void_p())) == -2
    assert lib.bpe_table_info(null, None) == -1
    assert lib.bpe_table_free(null) == 0 and lib.bpe_pool_destroy(null) == 0


def test_workspace_sizes_of_the_other_entry_points():
    lib = B.load_library()
    # pre-tokenizer: one state word per 4 KiB of input, whatever tile size is taken
    a, b = B.bpe_pretokenize_workspace_bytes(0), B.bpe_pretokenize_workspace_bytes(10**9)
    assert a >= 512 and a % 256 == 0 and 8 * 10**9 / 4096 <= b <= 8 * 10**9 / 4096 + 4096
    assert lib.bpe_pretokenize_workspace_bytes(-1) == -2 and lib.bpe_pretokenize_workspace_bytes(2**31) == -2
    # raw path: the encode workspace for max_pieces pieces plus the piece arrays; 0 pieces means n_bytes
    n = 10**6
    assert B.bpe_encode_raw_workspace_bytes(n, 0, 1) == B.bpe_encode_raw_workspace_bytes(n, n, 1)
    small, big = B.bpe_encode_raw_workspace_bytes(n, n // 4, 1), B.bpe_encode_raw_workspace_bytes(n, n, 1)
    assert B.bpe_workspace_bytes(n, n // 4) < small < big
    assert B.bpe_encode_raw_workspace_bytes(n, n, 5000) > big
    assert lib.bpe_encode_raw_workspace_bytes(n, -1, 1) == -2 and lib.bpe_encode_raw_workspace_bytes(n, n, -1) == -2
    # decoder: one state word per 1024 tokens
    assert B.bpe_decode_workspace_bytes(0) >= 512
    assert 8 * 10**9 / 1024 <= B.bpe_decode_workspace_bytes(10**9) <= 8 * 10**9 / 1024 + 4096
    assert lib.bpe_decode_workspace_bytes(-1) == -2


def test_other_entry_points_reject_bad_arguments_before_touching_the_gpu():
    lib = B.load_library()
    null = ctypes.c_void_p(0)
    one = ctypes.c_void_p(256)     # never dereferenced: every call below fails its checks first
    assert lib.bpe_pretokenize(null, 10, null, 0, null, 10, null, null, null, 0, None, null) == -1
    assert lib.bpe_pretokenize(one, -1, null, 0, one, 10, one, null, one, 1 << 20, None, null) == -2
    assert lib.bpe_pretokenize(one, 10, null, 0, one, 10, one, null, null, 0, None, null) == -8
    assert lib.bpe_pretokenize(one, 10, null, 0, one, 10, one, null, ctypes.c_void_p(257), 1 << 20, None, null) == -8
    bad = B.EncodeOptions(pretokenize_tile_kib=5)._c()
    assert lib.bpe_pretokenize(one, 10, null, 0, one, 10, one, null, one, 1 << 20, ctypes.byref(bad), null) == -10
    assert lib.bpe_encode_raw(null, one, 10, null, 0, 0, one, one, null, null, null, one, 1 << 20, None, null) == -1
    assert lib.bpe_decode(null, one, 10, null, 0, one, 10, null, null, one, 1 << 20, null) == -1
    assert lib.bpe_map_ids(null, one, one, 10, null, 1, null) == -1
    assert lib.bpe_vocab_build(null, null, null, 0, null, 0, None) == -1
    assert lib.bpe_vocab_free(null) == 0 and lib.bpe_vocab_info(null, None) == -1


@pytest.mark.parametrize("merges,ranks,ids,out_ids,code", [
    ([[97, 98]], None, None, list(range(10)), -2),                        # output ids: wrong length
    ([[97, 98]], None, None, [0] * 257, -6),                              # one output id for two ids
    ([[97, 98]], None, None, list(range(256)) + [1 << 24], -3),           # output id too large
    ([[97, 98]], None, None, [-1] + list(range(1, 257)), -3),             # negative output id
    ([[256, 97], [97, 98]], None, None, None, -7),                        # uses an id made later
    ([[97, 98], [98, 99]], None, [300, 300], None, -6),                   # duplicate merged id
    ([[120, 120]] + [[256 + k, 256 + k] for k in range(21)], None, None, None, -2),   # 2 MiB token
])
def test_vocab_validation_errors_come_before_any_gpu_call(merges, ranks, ids, out_ids, code):
    with pytest.raises(B.BpeError) as e:
        B.Vocab(merges, ranks, ids, out_ids)
    assert e.value.code == code
    assert len(str(e.value)) > 20


def test_option_struct_matches_the_header():
    # the binding's field list is the header's, in order
    text = open(os.path.join(ROOT, "include", "bpe_mi355x.h")).read()
    body = text[text.index("typedef struct {", text.index("Encoding (paper")):text.index("} bpe_encode_options;")]
    fields = re.findall(r"int32_t\s+(\w+);", body)
    from paper_2603_02597_amd.binding import _Options
    assert fields == [f for f, _ in _Options._fields_]


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_plan_names_what_the_calls_launch():
    """bpe_encode_plan / bpe_encode_raw_plan: pure functions of sizes and options (no GPU)."""
    E = B.EncodeOptions
    # the five workloads at their default options
    shapes = {"tiny": (4096, 682), "seq32k": (209426, 31582), "seq131k": (840501, 126380),
              "batch": (13510208, 2033454), "stress": (3999992, 528564)}
    plans = {k: B.bpe_encode_plan(*v) for k, v in shapes.items()}
    assert [l["kernel"] for l in plans["tiny"]["launches"]] == ["encode_kernel"] and plans["tiny"]["single_kernel"] == 1
    assert plans["tiny"]["n_tiles"] == 3 and plans["tiny"]["launches"][0]["grid"] == 3
    assert [l["kernel"] for l in plans["seq32k"]["launches"]] == ["encode_kernel"]
    assert [l["kernel"] for l in plans["seq131k"]["launches"]] == ["merge_tiles_kernel", "emit_kernel"]
    assert plans["seq131k"]["n_tiles"] == 494 and plans["seq131k"]["pieces_per_wave"] == 64
    # deep grids: merge_kernel, whose first workgroups (one for every four tiles) take the long pieces
    assert [l["kernel"] for l in plans["batch"]["launches"]] == ["merge_kernel", "emit_deep_kernel"]
    assert plans["batch"]["launches"][0]["grid"] == 7944 + (7944 + 3) // 4
    assert plans["batch"]["launches"][1]["grid"] == (7944 + 3) // 4
    assert [l["kernel"] for l in plans["stress"]["launches"]] == ["merge_kernel", "emit_kernel"]
    assert plans["stress"]["launches"][0]["grid"] == 2065 + (2065 + 3) // 4
    assert B.bpe_encode_plan(3999992, 528564, E(long_groups=-1))["launches"][0] == \
        {"kernel": "merge_tiles_kernel", "grid": 2065, "block": 256, "interval": 0}
    assert B.bpe_encode_plan(3999992, 528564, E(long_groups=16))["launches"][0]["grid"] == 2065 + 130
    assert B.kernels_by_interval(plans["seq131k"], B.N_TIMED_INTERVALS) == ["merge_tiles_kernel", "", "emit_kernel"]
    # beyond 8192 tiles a scan kernel runs between the two
    deep = B.bpe_encode_plan(40_000_000, 6_000_000)
    assert B.kernels_by_interval(deep, 3) == ["merge_kernel", "scan_tiles_kernel", "emit_deep_kernel"]
    assert B.kernels_by_interval(B.bpe_encode_plan(40_000_000, 6_000_000, E(long_groups=-1)), 3)[0] == "merge_tiles_kernel"
    # few very long pieces: 16 wavefronts per piece; the paper's kernels: one workgroup per piece
    assert B.bpe_encode_plan(400_000, 100)["launches"][0]["kernel"] == "merge_wide_kernel"
    paper = B.bpe_encode_plan(840501, 3284, E(paper_kernel=2))
    assert paper["launches"][0]["grid"] == 3284 and paper["n_tiles"] == 3284 and paper["single_kernel"] == 0
    # forced choices
    assert B.bpe_encode_plan(840501, 126380, E(fused=1))["single_kernel"] == 1
    assert B.bpe_encode_plan(4096, 682, E(fused=-1))["single_kernel"] == 0
    assert B.bpe_encode_plan(840501, 126380, E(pieces_per_wave=-1))["n_tiles"] == 126380
    # the raw path
    raw = B.bpe_encode_raw_plan(840501, 0, 1, False, True)
    assert B.kernels_by_interval(raw, B.N_RAW_TIMED_INTERVALS)[0] == "pretokenize_kernel"
    assert all(l["grid"] >= 1 for l in raw["launches"])
    # tokens only, all tiles resident at once: no pre-tokenizer launch, the merge workgroups take 1280 bytes each
    raw = B.bpe_encode_raw_plan(840501, 0, 1, False, False)
    assert B.kernels_by_interval(raw, B.N_RAW_TIMED_INTERVALS) == ["", "merge_bytes_kernel", "", "emit_bytes_kernel", ""]
    assert raw["launches"][0]["grid"] == -(-840501 // 1280) and raw["n_tiles"] == raw["launches"][0]["grid"]
    assert B.kernels_by_interval(B.bpe_encode_raw_plan(1024 * 1280, 0, 7, True, False), 5)[1] == "merge_bytes_kernel"
    assert B.kernels_by_interval(B.bpe_encode_raw_plan(1024 * 1280 + 1, 0, 7, True, False), 5)[0] == "pretokenize_kernel"
    for kw in (dict(fused=-1), dict(pieces_per_wave=64)):      # ... unless asked otherwise
        assert B.kernels_by_interval(B.bpe_encode_raw_plan(840501, 0, 1, False, False, E(**kw)), 5)[0] == "pretokenize_kernel"
    assert B.kernels_by_interval(B.bpe_encode_raw_plan(840501, 200000, 1, False, False), 5)[0] == "pretokenize_kernel"
    # option errors come back as from the calls themselves
    with pytest.raises(B.BpeError) as e:
        B.bpe_encode_plan(100, 10, E(selection_level=7))
    assert e.value.code == -10
    with pytest.raises(B.BpeError) as e:
        B.bpe_encode_plan(-1, 10)
    assert e.value.code == -2


def test_forced_single_kernel_is_refused_beyond_the_resident_grid():
    """fused = 1 only where no wait between workgroups can last: at most 1024 tiles of pieces
    that average at most 64 bytes; fused = 2 forces it."""
    E = B.EncodeOptions
    assert B.bpe_encode_plan(1024 * 256 * 6, 1024 * 256, E(fused=1))["single_kernel"] == 1
    for n_bytes, n_pieces in ((1025 * 256 * 6, 1024 * 256 + 1), (13510208, 2033454), (100_000, 1000), (4097, 1)):
        with pytest.raises(B.BpeError) as e:
            B.bpe_encode_plan(n_bytes, n_pieces, E(fused=1))
        assert e.value.code == -10 and "fused = 2" in str(e.value)
        plan = B.bpe_encode_plan(n_bytes, n_pieces, E(fused=2))
        assert plan["single_kernel"] == 1 and [l["kernel"] for l in plan["launches"]] == ["encode_kernel"]
    with pytest.raises(B.BpeError):
        B.bpe_encode_plan(100, 10, E(fused=3))



def test_status_from_words():
    """The verdict a host copy of a workspace's status words spells (word 2: the call, word 7: its
    check word; words 0, 1, 3 name that call if bad input / too little room / a wait that ran out)."""
    lib = B.load_library()
    def verdict(words):
        a = np.array(words, dtype=np.int32)
        return lib.bpe_status_from_words(a.ctypes.data_as(ctypes.c_void_p))
    check = 0x5AC3A53C
    call = 0x1234567
    ok = [0, 0, call, 0, 9, 9, 9, call ^ check]
    assert verdict(ok) == 0
    assert verdict([0] * 8) == 0 and verdict([-1] * 8) == 0 and verdict([call] * 8) == 0    # no call recorded
    assert verdict([call] + ok[1:]) == -11
    assert verdict(ok[:1] + [call] + ok[2:]) == -2
    assert verdict(ok[:3] + [call] + ok[4:]) == -9
    assert verdict([call, call, call, call] + ok[4:]) == -9          # a run-out wait outranks the rest
    assert lib.bpe_status_from_words(None) == -1
