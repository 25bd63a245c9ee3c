#!/usr/bin/env python3
"""Benchmark of the BPE merge-loop path on one MI355X.

A *step* is one bpe_encode call (all kernels of the path) over one workload
that is already resident in HBM.  Prints ONE JSON line: input MB/s (10^6 bytes
of input per second) as `value`, tokens/s, the HBM roofline of the dominant
kernel and the CPU oracle timed on the host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload seq131k]

--stage pretokenize times the device pre-tokenizer alone and --stage raw the
path from raw bytes (pre-tokenizer + encode, no host pass); --repeat R tiles
the workload's bytes R times to reach sizes at which HBM bandwidth binds.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak

def measured_traffic(workload: str, stage: str, kernel: str):
    """Bytes per launch that crossed the L2 <-> fabric boundary for this kernel on this
    workload, as the committed rocprofv3 --pmc summaries under profiles/ state it (lines
    `traffic: workload=W stage=S kernel=K bytes_per_launch=N`, written next to the counter
    readings and the commands they come from), or None if no summary covers the case."""
    import glob
    import re
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "pmc_traffic_*.txt"))):
        for line in open(path):
            m = re.match(r"traffic: workload=(\S+) stage=(\S+) kernel=(\S+) bytes_per_launch=(\d+)", line.strip())
            if m and m.group(1) == workload and m.group(2) == stage and m.group(3) == kernel:
                return {"bytes_per_launch": int(m.group(4)), "source": os.path.relpath(path, ROOT)}
    return None


def traffic_bytes(t):
    return None if t is None else t["bytes_per_launch"]


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def algorithmic_bytes(n_bytes: int, n_pieces: int, n_tokens: int) -> int:
    """What the method must move through HBM once: the input bytes, the piece
    offsets in, the token offsets out and the token ids out."""
    return n_bytes + 4 * (n_pieces + 1) + 4 * (n_pieces + 1) + 4 * n_tokens


def cpu_baseline(ev, merges, got_ids, got_off):
    """The oracle, untuned, on the host cores: the whole workload over and over
    for about 8 s per thread count, best run.  Also the check of the benchmarked
    output: every id and offset of the HIP path against the oracle's."""
    import numpy as np
    import oracle
    table = oracle.Table(merges)
    cores = max(1, min(os.cpu_count() or 1, 16))
    best = {1: float("inf"), cores: float("inf")}
    runs = {}
    ids = off = None
    for threads in sorted(set(best)):
        t_start = time.perf_counter()
        runs[threads] = 0
        while runs[threads] < 3 or (time.perf_counter() - t_start < 8.0 and runs[threads] < 2000):
            t0 = time.perf_counter()
            ids, off = oracle.encode(table, ev["bytes"], ev["piece_offsets"], n_threads=threads)
            best[threads] = min(best[threads], time.perf_counter() - t0)
            runs[threads] += 1
    assert np.array_equal(off, got_off), "token offsets of the HIP path differ from the oracle's"
    assert np.array_equal(ids, got_ids), "token ids of the HIP path differ from the oracle's"
    nb = ev["bytes"].size
    return {
        "value": nb / best[cores] / 1e6, "unit": "MB/s", "cores": cores, "cpu": cpu_model(), "kind": "oracle",
        "sample": f"whole workload, best of {runs[cores]} runs (about 8 s), pieces split statically over the threads",
        "tokens_per_s": ids.size / best[cores],
        "single_thread_MBps": nb / best[1] / 1e6,
        "output_checked": "all ids and offsets of the benchmarked call equal the oracle's",
    }


def side_measurements(B, torch, np, table, data, off, out_ids, out_off, ws, opts, stream, n_tokens, merges_host):
    """Outside the timed region: per-step latency spread, the rate with the PCIe
    copies of input and output included, and what a plain device copy reaches."""
    n_bytes = data.numel()
    # (1) one event pair and one synchronisation per step
    lat = []
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(100):
        e0.record(stream)
        B.bpe_encode(table, data, off, out_ids, out_off, ws, opts, stream)
        e1.record(stream)
        e1.synchronize()
        lat.append(e0.elapsed_time(e1) * 1e3)
    lat = np.sort(np.array(lat))
    # (2) pinned host input -> device, encode, token offsets and ids -> pinned host
    h_data = data.cpu().pin_memory()
    h_off = off.cpu().pin_memory()
    h_out_off = torch.empty(out_off.shape, dtype=torch.int32).pin_memory()
    h_out_ids = torch.empty(out_ids.shape, dtype=torch.int32).pin_memory()
    d_data, d_off = torch.empty_like(data), torch.empty_like(off)
    best = float("inf")
    for _ in range(12):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        d_data.copy_(h_data, non_blocking=True)
        d_off.copy_(h_off, non_blocking=True)
        B.bpe_encode(table, d_data, d_off, out_ids, out_off, ws, opts, stream)
        h_out_off.copy_(out_off, non_blocking=True)
        torch.cuda.synchronize()
        total = int(h_out_off[-1])
        h_out_ids[:total].copy_(out_ids[:total], non_blocking=True)
        torch.cuda.synchronize()
        best = min(best, time.perf_counter() - t0)
    assert total == n_tokens
    # (3) plain device-to-device copy of 256 MiB: bytes read + bytes written per second
    src = torch.zeros(64 << 20, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    e0.record(stream)
    for _ in range(10):
        dst.copy_(src)
    e1.record(stream)
    e1.synchronize()
    copy_gbs = 2 * src.numel() * 4 * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst
    # (4) the paper's own measure: one text on the host in, its ids on the host out (pre-tokenizer,
    # merges, copies both ways), through the Tokenizer class
    tok = B.Tokenizer(merges_host)
    text = data.cpu().numpy().tobytes()
    best_e2e, n_e2e = float("inf"), 0
    for _ in range(8):
        t0 = time.perf_counter()
        ids_e2e, _ = tok.tokenize_batch([text])
        best_e2e = min(best_e2e, time.perf_counter() - t0)
        n_e2e = int(ids_e2e[0].size)
    tok.close()
    assert n_e2e == n_tokens
    return {
        "end_to_end_tokenize_batch": {
            "ms": best_e2e * 1e3, "MB/s": n_bytes / best_e2e / 1e6,
            "note": "Tokenizer.tokenize_batch([text]): host bytes in, host ids out, best of 8; the paper's "
                    "Table 1 reports 53.4 ms for its 131K-token input on an RTX 4070 (other hardware, other "
                    "text, other tokens: context only)"},
        "step_latency_us": {"median": float(np.median(lat)), "p10": float(lat[10]), "p90": float(lat[90]),
                            "note": "100 steps, each bracketed by its own event pair and synchronised"},
        "with_pcie_copies": {"value": n_bytes / best / 1e6, "unit": "MB/s", "ms_per_step": best * 1e3,
                             "note": "pinned host bytes+offsets in, token offsets and ids out, best of 12"},
        "device_copy_GBps": copy_gbs,
    }


def calibrate_copy(torch):
    """Three plain device copies of 256 MiB: known traffic to scale profiler byte counters by."""
    src = torch.zeros(64 << 20, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()


def decode_main(args, B, torch, np, C) -> int:
    """--stage decode: token ids (made by bpe_encode from the workload) back to bytes."""
    ev = C.make_eval(args.workload)
    merges = C.load_merges(ev["table"])
    table, vocab = B.Table(merges), B.Vocab(merges)
    d = torch.from_numpy(ev["bytes"].copy()).cuda()
    ids, _ = B.encode(table, d, torch.from_numpy(ev["piece_offsets"].copy()).cuda())
    ids = ids.repeat(args.repeat).contiguous()
    n_tokens, n_bytes = ids.numel(), ev["bytes"].size * args.repeat
    out = torch.empty(n_bytes, dtype=torch.uint8, device="cuda")
    nb = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = torch.empty(B.bpe_decode_workspace_bytes(n_tokens), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    step = lambda: B.bpe_decode(vocab, ids, out, ws, None, nb, None, False, stream)
    for _ in range(args.warmup):
        step()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    per_step = (time.perf_counter() - t0) / args.steps
    assert B.bpe_encode_status(ws) == 0 and int(nb.item()) == n_bytes
    assert bytes(out[:ev["bytes"].size].cpu().numpy()) == ev["bytes"].tobytes(), "round trip failed"
    kernel_ms = ev0.elapsed_time(ev1) / args.steps
    alg = 4 * n_tokens + n_bytes          # ids in, bytes out
    achieved = alg / (kernel_ms * 1e-3) / 1e9
    result = {
        "metric": "MB/s of text decoded from token ids on 1 MI355X + HBM roofline %",
        "value": n_bytes / per_step / 1e6, "unit": "MB/s", "tokens_per_s": n_tokens / per_step,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": per_step * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": args.workload, "stage": "decode", "repeat": args.repeat, "n_bytes": n_bytes,
                   "n_tokens": n_tokens, "n_merges": int(merges.shape[0]),
                   "max_token_bytes": vocab.info["max_token_bytes"]},
        "roofline": {"bound": "hbm", "kernel": "decode_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic_bytes(measured_traffic(f"{args.workload}*{args.repeat}", "decode", "decode_kernel")),
                     "algorithmic_bytes": alg, "kernel_us": kernel_ms * 1e3},
    }
    if not args.no_cpu_baseline:
        import oracle
        sample = ids[:min(n_tokens, 1_000_000)].cpu().numpy()
        ot = oracle.Table(merges)
        t0 = time.perf_counter()
        text = oracle.decode(ot, sample)
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": text.size / dt / 1e6, "unit": "MB/s", "cores": 1, "cpu": cpu_model(),
                                  "kind": "oracle",
                                  "sample": f"first {sample.size} tokens, one run"}
    print(json.dumps(result))
    return 0


def stage_main(args, B, torch, np, C) -> int:
    """--stage pretokenize | raw: same contract line, other entry points."""
    if args.calibrate_copy:
        calibrate_copy(torch)
    ev = C.make_eval(args.workload)
    merges = C.load_merges(ev["table"])
    host = np.tile(ev["bytes"], args.repeat) if args.repeat > 1 else ev["bytes"].copy()
    n_bytes = host.size
    first = ev["seq_first_piece"]
    seq = None
    if first.size > 2 and args.repeat == 1:
        seq = np.concatenate([ev["piece_offsets"][first[:-1]], [n_bytes]]).astype(np.int32)
    n_seqs = 1 if seq is None else seq.size - 1
    data = torch.from_numpy(host).cuda()
    d_seq = None if seq is None else torch.from_numpy(seq).cuda()
    cap = args.max_pieces if args.max_pieces else n_bytes
    stream = torch.cuda.current_stream()
    opts = B.EncodeOptions(selection_level=args.selection_level, pieces_per_wave=args.pieces_per_wave,
                           pretokenize_tile_kib=args.pretokenize_tile_kib, long_groups=args.long_groups, fused=args.fused)
    # stage raw asks for tokens only, as Tokenizer.tokenize_batch does, unless --piece-arrays
    arrays = args.stage == "pretokenize" or args.piece_arrays
    piece_off = torch.empty(cap + 1, dtype=torch.int32, device="cuda") if arrays else None
    n_pieces_dev = torch.zeros(1, dtype=torch.int32, device="cuda") if arrays else None
    if args.stage == "pretokenize":
        first_dev = torch.empty(n_seqs + 1, dtype=torch.int32, device="cuda")
        ws = torch.empty(B.bpe_pretokenize_workspace_bytes(n_bytes), dtype=torch.uint8, device="cuda")
        step = lambda: B.bpe_pretokenize(data, d_seq, piece_off, n_pieces_dev, first_dev, ws, opts, stream)
    else:
        table = B.Table(merges)
        out_ids = torch.empty(n_bytes, dtype=torch.int32, device="cuda")
        out_off = torch.empty(cap + 1, dtype=torch.int32, device="cuda") if arrays else None
        seq_tok = torch.empty(n_seqs + 1, dtype=torch.int32, device="cuda")
        ws = torch.empty(B.bpe_encode_raw_workspace_bytes(n_bytes, cap, n_seqs), dtype=torch.uint8, device="cuda")
        step = lambda: B.bpe_encode_raw(table, data, d_seq, out_ids, seq_tok, ws, cap, piece_off, out_off,
                                        n_pieces_dev, opts, stream)
    for _ in range(args.warmup):
        step()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert B.bpe_encode_status(ws) == 0
    n_pieces = int(n_pieces_dev.item()) if arrays else None
    per_step = elapsed / args.steps
    if args.stage == "pretokenize":
        names = ["pretokenize_kernel"]
        kernel_ms = np.array([ev0.elapsed_time(ev1) / args.steps])
        n_tokens = None
        # bytes in, piece offsets out, sequence offsets in, first pieces out
        alg = n_bytes + 4 * (n_pieces + 1) + (8 * (n_seqs + 1) if seq is not None else 0)
    else:
        plan = B.bpe_encode_raw_plan(n_bytes, cap, n_seqs, seq is not None, arrays, opts)
        names = B.kernels_by_interval(plan, B.N_RAW_TIMED_INTERVALS)
        n_tokens = int(seq_tok[-1].item())
        kernel_ms = np.zeros(len(names))
        reps = max(10, min(args.steps, 50))
        for _ in range(reps):
            kernel_ms += np.array(B.bpe_encode_raw_timed(table, data, d_seq, out_ids, seq_tok, ws, cap, piece_off,
                                                         out_off, n_pieces_dev, opts, stream))
        kernel_ms /= reps
        kernel_ms[[i for i, k in enumerate(names) if not k]] = 0.0   # an interval without a launch: two event records
        # bytes in, token ids out, sequence offsets in and out
        alg = n_bytes + 4 * n_tokens + 8 * (n_seqs + 1)
    dom = int(kernel_ms.argmax())
    achieved = alg / (kernel_ms[dom] * 1e-3) / 1e9
    result = {
        "metric": f"MB/s of input through the {args.stage} stage on 1 MI355X + HBM roofline %",
        "value": n_bytes / per_step / 1e6, "unit": "MB/s",
        "tokens_per_s": None if n_tokens is None else n_tokens / per_step,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": per_step * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": args.workload, "stage": args.stage, "repeat": args.repeat, "n_bytes": n_bytes,
                   "n_pieces": n_pieces, "n_seqs": n_seqs, "n_tokens": n_tokens, "max_pieces": cap,
                   "n_merges": int(merges.shape[0])},
        "roofline": {
            "bound": "hbm", "kernel": names[dom], "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic_bytes(measured_traffic(f"{args.workload}*{args.repeat}", args.stage, names[dom])),
            "algorithmic_bytes": alg,
            "kernel_us": float(kernel_ms[dom] * 1e3),
            "all_kernels_us": {k: float(v * 1e3) for k, v in zip(names, kernel_ms) if k},
            "path_achieved": alg / per_step / 1e9,
        },
    }
    if not args.no_cpu_baseline:
        import oracle
        sample = host[:min(n_bytes, 4_000_000)]
        cores = max(1, min(os.cpu_count() or 1, 16))
        t0 = time.perf_counter()
        if args.stage == "pretokenize":
            oracle.pretokenize(sample)
        else:
            oracle.encode_raw(oracle.Table(merges), sample, None, n_threads=cores)
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": sample.size / dt / 1e6, "unit": "MB/s",
                                  "cores": 1 if args.stage == "pretokenize" else cores, "cpu": cpu_model(),
                                  "kind": "oracle",
                                  "sample": f"first {sample.size} bytes as one sequence, one run"}
    print(json.dumps(result))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="seq131k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-side-measurements", action="store_true",
                    help="skip the latency spread, the PCIe-inclusive rate and the device-copy rate")
    ap.add_argument("--selection-level", type=int, default=0)
    ap.add_argument("--pieces-per-wave", type=int, default=0)
    ap.add_argument("--fused", type=int, default=0, help="1: single kernel, -1: merge + emit kernels, 0: by grid size")
    ap.add_argument("--stage", default="encode", choices=["encode", "pretokenize", "raw", "decode"],
                    help="encode: bpe_encode on given pieces (the headline); pretokenize: bpe_pretokenize "
                         "alone; raw: bpe_encode_raw; decode: bpe_decode of the workload's tokens")
    ap.add_argument("--repeat", type=int, default=1, help="stages pretokenize/raw: tile the bytes this often")
    ap.add_argument("--max-pieces", type=int, default=0, help="stages pretokenize/raw: piece capacity (0 = n_bytes)")
    ap.add_argument("--piece-arrays", action="store_true",
                    help="stage raw: also ask for piece_offsets, out_offsets and n_pieces (the path with a pre-tokenizer launch)")
    ap.add_argument("--pretokenize-tile-kib", type=int, default=0)
    ap.add_argument("--chunk-bytes", type=int, default=0,
                    help="stage encode: replace the pieces by fixed chunks of this many bytes (the paper's "
                         "host-side chunking)")
    ap.add_argument("--paper-kernel", type=int, default=0,
                    help="stage encode: 1 / 2 = run the paper's baseline / optimized kernel, one workgroup per piece")
    ap.add_argument("--tiny-max-len", type=int, default=0,
                    help="stage encode: longest piece of the lane-per-piece path (0 = the library's choice)")
    ap.add_argument("--column-max-len", type=int, default=0,
                    help="stage encode: longest piece of the 64-entry column path (0 = the library's choice, -1 = off)")
    ap.add_argument("--long-groups", type=int, default=0,
                    help="stage encode: tiles per long-piece workgroup of merge_kernel (0 = default, -1 = none)")
    ap.add_argument("--dedup", type=int, default=0,
                    help="stage encode: 1 = merge every distinct piece of at most 16 bytes once (option dedup)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (known traffic) so that profiler "
                         "byte counters can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (pieces shard trivially, but no "
              "multi-GPU path is built); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2603_02597_amd as B
    from workloads import configs as C

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    B.load_library()

    if args.stage == "decode":
        return decode_main(args, B, torch, np, C)
    if args.stage != "encode":
        return stage_main(args, B, torch, np, C)

    ev = C.make_eval(args.workload)
    if args.chunk_bytes:
        from workloads import textgen
        ev["piece_offsets"] = textgen.fixed_chunks(ev["bytes"].size, args.chunk_bytes)
    merges = C.load_merges(ev["table"])
    table = B.Table(merges)
    data = torch.from_numpy(ev["bytes"].copy()).cuda()
    off = torch.from_numpy(ev["piece_offsets"].copy()).cuda()
    n_bytes, n_pieces = data.numel(), off.numel() - 1
    out_ids = torch.empty(n_bytes, dtype=torch.int32, device="cuda")
    out_off = torch.empty(n_pieces + 1, dtype=torch.int32, device="cuda")
    ws_bytes = B.bpe_dedup_workspace_bytes if args.dedup else B.bpe_workspace_bytes
    ws = torch.empty(ws_bytes(n_bytes, n_pieces), dtype=torch.uint8, device="cuda")
    opts = B.EncodeOptions(selection_level=args.selection_level, pieces_per_wave=args.pieces_per_wave,
                           fused=args.fused, paper_kernel=args.paper_kernel, dedup=args.dedup, long_groups=args.long_groups,
                           tiny_max_len=args.tiny_max_len, column_max_len=args.column_max_len)
    stream = torch.cuda.current_stream()

    if args.calibrate_copy:
        calibrate_copy(torch)

    for _ in range(args.warmup):
        B.bpe_encode(table, data, off, out_ids, out_off, ws, opts, stream)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        B.bpe_encode(table, data, off, out_ids, out_off, ws, opts, stream)
    ev1.record(stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    event_ms_per_step = ev0.elapsed_time(ev1) / args.steps
    assert B.bpe_encode_status(ws) == 0
    n_tokens = int(out_off[-1].item())
    ms_per_step = elapsed / args.steps * 1e3

    # Launch duration of the dominant kernel from HIP events on the stream the
    # kernels run on.  Single-kernel path: the events around the timed region,
    # divided by the number of launches (one per step).  Otherwise: an
    # event between the kernels of each call (bpe_encode_timed), same inputs.
    # Which kernels the library launched for this call comes from the library itself.
    plan = B.bpe_encode_plan(n_bytes, n_pieces, opts)
    names = B.kernels_by_interval(plan, B.N_TIMED_INTERVALS)
    if plan["single_kernel"]:
        kernel_ms = np.array([event_ms_per_step, 0.0, 0.0])
    else:
        kernel_ms = np.zeros(len(names))
        reps = max(10, min(args.steps, 100))
        for _ in range(reps):
            kernel_ms += np.array(B.bpe_encode_timed(table, data, off, out_ids, out_off, ws, opts, stream))
        kernel_ms /= reps
        kernel_ms[[i for i, k in enumerate(names) if not k]] = 0.0   # an interval without a launch: two event records
    dom = int(kernel_ms.argmax())
    alg = algorithmic_bytes(n_bytes, n_pieces, n_tokens)
    achieved = alg / (kernel_ms[dom] * 1e-3) / 1e9
    traffic = measured_traffic(args.workload, "encode", names[dom]) if not (args.chunk_bytes or args.paper_kernel or args.dedup) else None
    got_ids, got_off = out_ids[:n_tokens].cpu().numpy(), out_off.cpu().numpy()

    result = {
        "metric": "MB/s and tokens/s tokenized on 1 MI355X (131k-token seq) + HBM roofline %",
        "value": n_bytes / (elapsed / args.steps) / 1e6,
        "unit": "MB/s",
        "tokens_per_s": n_tokens / (elapsed / args.steps),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": args.workload, "n_bytes": n_bytes, "n_pieces": n_pieces,
                   "n_tokens": n_tokens, "n_merges": int(merges.shape[0]),
                   "selection_level": 1 if args.paper_kernel else (args.selection_level or "auto"),
                   "chunk_bytes": args.chunk_bytes, "paper_kernel": args.paper_kernel, "dedup": args.dedup},
        "roofline": {
            "bound": "hbm", "kernel": names[dom], "achieved": achieved, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": None if traffic is None else traffic["bytes_per_launch"],
            "traffic_source": None if traffic is None else traffic["source"],
            "algorithmic_bytes": alg, "kernel_us": float(kernel_ms[dom] * 1e3),
            "all_kernels_us": {k: float(v * 1e3) for k, v in zip(names, kernel_ms) if k},
            "path_achieved": alg / (elapsed / args.steps) / 1e9,
            "path_frac": alg / (elapsed / args.steps) / 1e9 / HBM_PEAK_GBS,
            "launches": plan["launches"],
        },
    }
    if not args.no_side_measurements:
        result.update(side_measurements(B, torch, np, table, data, off, out_ids, out_off, ws, opts, stream,
                                        n_tokens, merges))
        result["roofline"]["frac_of_device_copy"] = achieved / result["device_copy_GBps"]
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(ev, merges, got_ids, got_off)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
