"""The paper's Python-facing call (section 3.7): a list of texts in, token ids
per text and the kernel time out.  Marshalling only: the texts are concatenated
behind their offsets into one pinned host buffer, copied to the GPU with one copy,
and bpe_encode_raw does the rest (piece starts, merges, ids per text) in its
kernels; one copy brings offsets and ids back; decode_batch goes the other way
through bpe_decode.  Buffers grow to the largest batch seen and are reused,
so a steady stream of batches allocates nothing."""
from __future__ import annotations

import ctypes

import numpy as np

from . import binding as B


def _hip_runtime():
    """The HIP runtime this process already has mapped (torch brought it), for plain
    asynchronous copies without a tensor operation's overhead; None if it cannot be found."""
    try:
        with open("/proc/self/maps") as f:
            paths = {line.split()[-1] for line in f if "libamdhip64" in line}
        if len(paths) != 1:
            return None
        lib = ctypes.CDLL(paths.pop())
        lib.hipMemcpyAsync.restype = ctypes.c_int
        lib.hipMemcpyAsync.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
        return lib
    except (OSError, AttributeError):
        return None


class Tokenizer:
    def __init__(self, merges, ranks=None, merged_ids=None, output_ids=None, device="cuda:0"):
        import torch
        self._torch = torch
        self.device = torch.device(device)
        with torch.cuda.device(self.device):
            self.table = B.Table(merges, ranks, merged_ids)
            self.vocab = B.Vocab(merges, ranks, merged_ids, output_ids)
        self._use_output_ids = output_ids is not None
        self._hip = _hip_runtime()
        self._cap_bytes = self._cap_seqs = 0
        self._ids_per_byte = None     # most ids per input byte of any batch so far (sizes the first copy out)

    def _reserve(self, n_bytes: int, n_seqs: int):
        torch = self._torch
        if n_bytes <= self._cap_bytes and n_seqs <= self._cap_seqs:
            return
        nb = max(n_bytes, 2 * self._cap_bytes, 1 << 16)
        ns = max(n_seqs, 2 * self._cap_seqs, 64)
        dev = self.device
        # One buffer each way, so that a batch is one copy in and one copy out:
        # in  = [sequence offsets int32 (n_seqs + 1) | bytes], packed per call;
        # out = [first token of every sequence int32 (n_seqs + 1) | token ids].
        self._h_in = torch.empty(4 * (ns + 1) + nb, dtype=torch.uint8).pin_memory()
        self._d_in = torch.empty(4 * (ns + 1) + nb, dtype=torch.uint8, device=dev)
        self._h_out = torch.empty(ns + 1 + nb, dtype=torch.int32).pin_memory()
        self._d_out = torch.empty(ns + 1 + nb, dtype=torch.int32, device=dev)
        self._h_status = torch.zeros(8, dtype=torch.int32).pin_memory()
        self._h_in_np, self._h_out_np = self._h_in.numpy(), self._h_out.numpy()
        self._ws = torch.empty(B.bpe_encode_raw_workspace_bytes(nb, 0, ns), dtype=torch.uint8, device=dev)
        self._ws_status = self._ws[:32].view(torch.int32)
        self._events = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
        self._cap_bytes, self._cap_seqs = nb, ns

    def _copy(self, dst, src, lo: int, hi: int, kind: int, stream):
        """Asynchronous copy of elements [lo, hi) between a pinned and a device tensor of one
        dtype on `stream` (kind 1: host to device, 2: device to host)."""
        if self._hip is None:
            dst[lo:hi].copy_(src[lo:hi], non_blocking=True)
            return
        size = dst.element_size()
        rc = self._hip.hipMemcpyAsync(dst.data_ptr() + lo * size, src.data_ptr() + lo * size, (hi - lo) * size, kind,
                                      stream.cuda_stream)
        if rc != 0:
            raise RuntimeError(f"hipMemcpyAsync failed with error {rc}")

    def tokenize_batch(self, texts):
        """texts: list of bytes (or str, encoded as UTF-8).  Returns (list of int32
        arrays, kernel_ms): the ids of every text and the GPU time of the kernels.
        One copy in, the kernels, one copy out (sequence token offsets and as many ids
        as batches so far needed per input byte, with a margin), the status words, one
        synchronisation; only a batch that needs more ids than that pays a second copy."""
        torch = self._torch
        raw = [t.encode("utf-8") if isinstance(t, str) else t for t in texts]
        n_seqs = len(raw)
        if n_seqs == 0:
            return [], 0.0
        if n_seqs == 1:
            joined = raw[0]
            ends = (len(joined),)
        else:
            joined = b"".join(raw)
            ends = np.cumsum(np.fromiter((len(r) for r in raw), dtype=np.int64, count=n_seqs))
        n_bytes = len(joined)
        if n_bytes >= 2**31 - 1:
            raise ValueError("a batch must stay below 2^31 bytes")
        with torch.cuda.device(self.device):
            self._reserve(n_bytes, n_seqs)
            lib = B.load_library()
            vp = ctypes.c_void_p
            n_in = 4 * (n_seqs + 1)
            seq_np = self._h_in_np[:n_in].view(np.int32)
            seq_np[0] = 0
            seq_np[1:] = ends
            if n_bytes:       # one copy, straight into the pinned buffer
                self._h_in_np[n_in:n_in + n_bytes] = np.frombuffer(joined, dtype=np.uint8)
            stream = torch.cuda.current_stream()
            self._copy(self._d_in, self._h_in, 0, n_in + n_bytes, 1, stream)
            e0, e1 = self._events
            e0.record(stream)
            d_in, d_out = self._d_in.data_ptr(), self._d_out.data_ptr()
            d_tok, d_ids = d_out, d_out + n_in
            rc = lib.bpe_encode_raw(self.table._h, vp(d_in + n_in), n_bytes, vp(d_in), n_seqs, 0, vp(d_ids), vp(d_tok),
                                    None, None, None, vp(self._ws.data_ptr()), self._ws.numel(), None,
                                    vp(stream.cuda_stream))
            if rc == 0 and self._use_output_ids:
                rc = lib.bpe_map_ids(self.vocab._h, vp(d_ids), vp(d_ids), n_bytes, vp(d_tok + 4 * n_seqs), 1,
                                     vp(stream.cuda_stream))
            if rc != 0:
                raise B.BpeError(rc, lib.bpe_last_error().decode(errors="replace"))
            e1.record(stream)
            n_guess = min(n_bytes, int(n_bytes * (self._ids_per_byte or 0.25) * 1.25) + 64)
            self._copy(self._h_out, self._d_out, 0, n_seqs + 1 + n_guess, 2, stream)
            self._copy(self._h_status, self._ws_status, 0, 8, 2, stream)
            stream.synchronize()
            st = lib.bpe_status_from_words(vp(self._h_status.data_ptr()))
            if st != 0:
                raise B.BpeError(st, lib.bpe_last_error().decode(errors="replace"))
            tok = self._h_out_np[:n_seqs + 1].copy()
            total = int(tok[-1])
            if total > n_guess:
                self._copy(self._h_out, self._d_out, n_seqs + 1 + n_guess, n_seqs + 1 + total, 2, stream)
                stream.synchronize()
            if n_bytes:
                self._ids_per_byte = max(self._ids_per_byte or 0.0, total / n_bytes)
            ids = self._h_out_np[n_seqs + 1:n_seqs + 1 + total]
            return [ids[tok[k]:tok[k + 1]].copy() for k in range(n_seqs)], e0.elapsed_time(e1)

    def decode_batch(self, ids_list):
        """ids_list: list of int arrays (output ids if the tokenizer has them).  Returns list of bytes."""
        torch = self._torch
        arrs = [np.ascontiguousarray(np.asarray(a, dtype=np.int32)) for a in ids_list]
        if not arrs:
            return []
        bounds = np.concatenate([[0], np.cumsum([a.size for a in arrs])]).astype(np.int64)
        n_tokens = int(bounds[-1])
        if n_tokens == 0:
            return [b"" for _ in arrs]
        with torch.cuda.device(self.device):
            dev = self.device
            ids = torch.from_numpy(np.concatenate(arrs)).to(dev)
            # a first guess of 16 bytes per token; the kernel reports the true size if that is too small
            cap = min(n_tokens * int(self.vocab.info["max_token_bytes"]), max(16 * n_tokens, 1 << 20), 2**31 - 2)
            tbo = torch.empty(n_tokens + 1, dtype=torch.int32, device=dev)
            ws = torch.empty(B.bpe_decode_workspace_bytes(n_tokens), dtype=torch.uint8, device=dev)
            for attempt in range(2):
                out = torch.empty(cap, dtype=torch.uint8, device=dev)
                B.bpe_decode(self.vocab, ids, out, ws, token_byte_offsets=tbo, ids_are_output_ids=self._use_output_ids)
                st = B.bpe_encode_status(ws)
                if st == -2 and attempt == 0:          # BPE_ERR_SIZE: the offsets are the true ones
                    cap = int(tbo[-1].item())
                    if cap < 0:
                        raise ValueError("the decoded text would exceed 2^31 bytes")
                    continue
                if st != 0:
                    raise B.BpeError(st, B.load_library().bpe_last_error().decode(errors="replace"))
                break
            starts = tbo[torch.from_numpy(bounds).to(dev)].cpu().numpy()
            text = out[:int(starts[-1])].cpu().numpy().tobytes()
            return [text[starts[k]:starts[k + 1]] for k in range(len(arrs))]

    def close(self):
        self.table.free()
        self.vocab.free()
