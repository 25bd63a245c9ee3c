"""The paper's Python-facing call (section 3.7): a list of texts in, token ids
per text and the kernel time out.  Marshalling only: the texts are concatenated
into one pinned host buffer, copied to the GPU, and bpe_encode_raw does the rest
(piece starts, merges, ids per text) in its kernels; decode_batch goes the other
way through bpe_decode.  Buffers grow to the largest batch seen and are reused,
so a steady stream of batches allocates nothing."""
from __future__ import annotations

import numpy as np

from . import binding as B


class Tokenizer:
    def __init__(self, merges, ranks=None, merged_ids=None, output_ids=None, device="cuda:0"):
        import torch
        self._torch = torch
        self.device = torch.device(device)
        with torch.cuda.device(self.device):
            self.table = B.Table(merges, ranks, merged_ids)
            self.vocab = B.Vocab(merges, ranks, merged_ids, output_ids)
        self._use_output_ids = output_ids is not None
        self._cap_bytes = self._cap_seqs = self._cap_tokens = 0

    def _reserve(self, n_bytes: int, n_seqs: int):
        torch = self._torch
        if n_bytes <= self._cap_bytes and n_seqs <= self._cap_seqs:
            return
        nb = max(n_bytes, 2 * self._cap_bytes, 1 << 16)
        ns = max(n_seqs, 2 * self._cap_seqs, 64)
        dev = self.device
        self._h_bytes = torch.empty(nb, dtype=torch.uint8).pin_memory()
        self._h_seq = torch.empty(ns + 1, dtype=torch.int32).pin_memory()
        self._h_ids = torch.empty(nb, dtype=torch.int32).pin_memory()
        self._h_tok = torch.empty(ns + 1, dtype=torch.int32).pin_memory()
        self._d_bytes = torch.empty(nb, dtype=torch.uint8, device=dev)
        self._d_seq = torch.empty(ns + 1, dtype=torch.int32, device=dev)
        self._d_ids = torch.empty(nb, dtype=torch.int32, device=dev)
        self._d_tok = torch.empty(ns + 1, dtype=torch.int32, device=dev)
        self._ws = torch.empty(B.bpe_encode_raw_workspace_bytes(nb, 0, ns), dtype=torch.uint8, device=dev)
        self._cap_bytes, self._cap_seqs = nb, ns

    def tokenize_batch(self, texts):
        """texts: list of bytes (or str, encoded as UTF-8).  Returns (list of int32
        arrays, kernel_ms): the ids of every text and the GPU time of the kernels."""
        torch = self._torch
        raw = [t.encode("utf-8") if isinstance(t, str) else bytes(t) for t in texts]
        lens = np.fromiter((len(r) for r in raw), dtype=np.int64, count=len(raw))
        n_bytes, n_seqs = int(lens.sum()), len(raw)
        if n_bytes >= 2**31 - 1:
            raise ValueError("a batch must stay below 2^31 bytes")
        if n_seqs == 0:
            return [], 0.0
        with torch.cuda.device(self.device):
            self._reserve(n_bytes, n_seqs)
            if n_bytes:       # one copy, straight into the pinned buffer
                joined = raw[0] if n_seqs == 1 else b"".join(raw)
                np.copyto(self._h_bytes.numpy()[:n_bytes], np.frombuffer(joined, dtype=np.uint8))
            self._h_seq[0] = 0
            self._h_seq[1:n_seqs + 1] = torch.from_numpy(np.cumsum(lens).astype(np.int32))
            stream = torch.cuda.current_stream()
            d_bytes, d_seq = self._d_bytes[:n_bytes], self._d_seq[:n_seqs + 1]
            d_bytes.copy_(self._h_bytes[:n_bytes], non_blocking=True)
            d_seq.copy_(self._h_seq[:n_seqs + 1], non_blocking=True)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            B.bpe_encode_raw(self.table, d_bytes, d_seq, self._d_ids, self._d_tok, self._ws, stream=stream)
            if self._use_output_ids:
                B.bpe_map_ids(self.vocab, self._d_ids[:n_bytes], self._d_ids[:n_bytes], True,
                              n_device=self._d_tok[n_seqs:n_seqs + 1], stream=stream)
            e1.record(stream)
            self._h_tok[:n_seqs + 1].copy_(self._d_tok[:n_seqs + 1], non_blocking=True)
            stream.synchronize()
            st = B.bpe_encode_status(self._ws, stream)
            if st != 0:
                raise B.BpeError(st, B.load_library().bpe_last_error().decode(errors="replace"))
            tok = self._h_tok[:n_seqs + 1].numpy().copy()
            total = int(tok[-1])
            self._h_ids[:total].copy_(self._d_ids[:total], non_blocking=True)
            stream.synchronize()
            ids = self._h_ids[:total].numpy()
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
