"""Seeded pseudo-text generator and the piece splitter.

Everything is drawn from one counter-based 64-bit generator (SplitMix64 used
as a function of the draw index), so any slice of a stream can be produced
independently and numpy can vectorise the whole thing.

Stream recipe (one *unit* per 8 consecutive draws):
  * with probability ``p_run``   : ``' '`` + one non-space byte repeated L times,
    L uniform in [64, 4096] (the first such unit of a stream uses L = 4096);
  * with probability ``p_rand``  : ``' '`` + L uniformly random bytes 0..255,
    L uniform in [1, 64];
  * otherwise a text unit: with probability 0.05 ``' '`` + 1..4 characters from
    ``PUNCT``; else ``' '`` + a pseudo-word whose rank k is drawn with
    P(k) proportional to k**-1.1; with probability 0.01 a ``'\\n'`` is appended.
Pieces are whatever ``pretokenize`` recovers: a piece starts at index 0, at
every sequence start and before every byte 0x20.
"""
from __future__ import annotations

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

# Approximate relative letter frequencies of English text, a..z, in 1/10000.
LETTER_FREQ = np.array(
    [817, 129, 278, 425, 1270, 223, 202, 609, 697, 15, 77, 403, 241,
     675, 751, 193, 10, 599, 633, 906, 276, 98, 236, 15, 197, 7],
    dtype=np.float64,
)
PUNCT = np.frombuffer(b"0123456789.,;:!?'\"()-/&%$#@*+=<>[]_", dtype=np.uint8)

ZIPF_S = 1.1
P_PUNCT = 0.05
P_NEWLINE = 0.01
DRAWS_PER_UNIT = 8


def splitmix64(seed: int, start: int, count: int) -> np.ndarray:
    """Outputs number ``start`` .. ``start+count-1`` of the SplitMix64 sequence
    whose state starts at ``seed`` (output i mixes ``seed + (i+1)*GAMMA``)."""
    with np.errstate(over="ignore"):
        i = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + i * _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _unit(z: np.ndarray) -> np.ndarray:
    """u64 -> float64 uniform in [0, 1)."""
    return (z >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def make_wordlist(n_words: int, seed: int):
    """``n_words`` pseudo-words: length uniform in 1..10, letters i.i.d. from
    ``LETTER_FREQ``.  Returns (flat uint8 letters, start[n_words], len[n_words])."""
    lens = (splitmix64(seed, 0, n_words) % np.uint64(10)).astype(np.int64) + 1
    starts = np.zeros(n_words, dtype=np.int64)
    np.cumsum(lens[:-1], out=starts[1:])
    total = int(lens.sum())
    cdf = np.cumsum(LETTER_FREQ) / LETTER_FREQ.sum()
    u = _unit(splitmix64(seed ^ 0x5DEECE66D, 0, total))
    letters = np.minimum(np.searchsorted(cdf, u, side="right"), 25).astype(np.uint8) + ord("a")
    return letters, starts, lens


def _ragged_arange(lens: np.ndarray) -> np.ndarray:
    """[0..lens[0]), [0..lens[1]), ... concatenated."""
    total = int(lens.sum())
    ends = np.cumsum(lens)
    return np.arange(total, dtype=np.int64) - np.repeat(ends - lens, lens)


def _gen_units(wordlist, zipf_cdf, seed: int, first_unit: int, n_units: int,
               p_rand: float, p_run: float, force_first_run: bool):
    """Bytes of units ``first_unit .. first_unit+n_units-1`` and their lengths."""
    letters, wstart, wlen = wordlist
    d = splitmix64(seed, first_unit * DRAWS_PER_UNIT, n_units * DRAWS_PER_UNIT)
    d = d.reshape(n_units, DRAWS_PER_UNIT)
    u_kind = _unit(d[:, 0])
    is_run = u_kind < p_run
    is_rand = (~is_run) & (u_kind < p_run + p_rand)
    is_text = ~(is_run | is_rand)
    is_punct = is_text & (_unit(d[:, 2]) < P_PUNCT)
    is_word = is_text & ~is_punct
    newline = is_text & (_unit(d[:, 3]) < P_NEWLINE)

    rank = np.minimum(np.searchsorted(zipf_cdf, _unit(d[:, 1]), side="right"),
                      len(wlen) - 1)
    body_len = np.zeros(n_units, dtype=np.int64)
    body_len[is_word] = wlen[rank[is_word]]
    body_len[is_punct] = (d[is_punct, 4] % np.uint64(4)).astype(np.int64) + 1
    body_len[is_rand] = (d[is_rand, 4] % np.uint64(64)).astype(np.int64) + 1
    run_len = (d[is_run, 4] % np.uint64(4096 - 64 + 1)).astype(np.int64) + 64
    if force_first_run and run_len.size:
        run_len[0] = 4096
    body_len[is_run] = run_len

    unit_len = 1 + body_len + newline.astype(np.int64)
    unit_off = np.zeros(n_units + 1, dtype=np.int64)
    np.cumsum(unit_len, out=unit_off[1:])
    out = np.full(int(unit_off[-1]), 0x20, dtype=np.uint8)
    body_at = unit_off[:-1] + 1

    # words: ragged gather from the flat letter array
    wl = body_len[is_word]
    if wl.size:
        k = _ragged_arange(wl)
        out[np.repeat(body_at[is_word], wl) + k] = letters[np.repeat(wstart[rank[is_word]], wl) + k]
    # punctuation / digits: up to 4 characters cut from one draw
    pl = body_len[is_punct]
    if pl.size:
        k = _ragged_arange(pl)
        src = np.repeat(d[is_punct, 5], pl) >> (np.uint64(8) * k.astype(np.uint64))
        out[np.repeat(body_at[is_punct], pl) + k] = PUNCT[(src & np.uint64(0xFF)) % np.uint64(len(PUNCT))]
    # uniformly random bytes: 64 per unit from a side stream indexed by the unit number
    rl = body_len[is_rand]
    if rl.size:
        k = _ragged_arange(rl)
        unit_no = np.nonzero(is_rand)[0].astype(np.int64) + first_unit
        side = seed ^ 0xA5A5A5A5DEADBEEF
        with np.errstate(over="ignore"):
            word_idx = np.repeat(unit_no * 8, rl) + (k >> 3)
        # one SplitMix64 output per 8 random bytes, evaluated only where needed
        z = _splitmix_at(side, word_idx)
        out[np.repeat(body_at[is_rand], rl) + k] = (
            (z >> (np.uint64(8) * (k & 7).astype(np.uint64))) & np.uint64(0xFF)).astype(np.uint8)
    # single-character runs (never a space)
    if run_len.size:
        c = (d[is_run, 5] % np.uint64(255)).astype(np.int64)
        c = np.where(c >= 0x20, c + 1, c).astype(np.uint8)
        k = _ragged_arange(run_len)
        out[np.repeat(body_at[is_run], run_len) + k] = np.repeat(c, run_len)
    nl_at = (unit_off[:-1] + 1 + body_len)[newline]
    out[nl_at] = 0x0A
    return out, unit_len


def _splitmix_at(seed: int, idx: np.ndarray) -> np.ndarray:
    """SplitMix64 output number ``idx[j]`` for every j (idx need not be sorted)."""
    with np.errstate(over="ignore"):
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + (idx.astype(np.uint64) + np.uint64(1)) * _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _zipf_cdf(n_words: int) -> np.ndarray:
    w = np.arange(1, n_words + 1, dtype=np.float64) ** (-ZIPF_S)
    return np.cumsum(w) / w.sum()


def gen_stream(n_words: int, vocab_seed: int, stream_seed: int, *,
               max_bytes: int | None = None, n_units: int | None = None,
               p_rand: float = 0.0, p_run: float = 0.0,
               chunk_units: int = 1 << 19) -> np.ndarray:
    """A stream of whole units: exactly ``n_units`` of them, or as many as fit in
    ``max_bytes`` (the cut falls on a unit boundary)."""
    assert (max_bytes is None) != (n_units is None)
    wordlist = make_wordlist(n_words, vocab_seed)
    cdf = _zipf_cdf(n_words)
    parts, have_bytes, have_units, seen_run = [], 0, 0, False
    while True:
        want = chunk_units if n_units is None else min(chunk_units, n_units - have_units)
        if want <= 0:
            break
        out, ulen = _gen_units(wordlist, cdf, stream_seed, have_units, want,
                               p_rand, p_run, force_first_run=(p_run > 0 and not seen_run))
        if p_run > 0 and not seen_run:
            seen_run = bool((ulen > 64).any())
        if max_bytes is not None and have_bytes + out.size > max_bytes:
            ends = np.cumsum(ulen)
            keep = int(np.searchsorted(ends, max_bytes - have_bytes, side="right"))
            parts.append(out[: int(ends[keep - 1])] if keep else out[:0])
            break
        parts.append(out)
        have_bytes += out.size
        have_units += want
    return np.concatenate(parts) if parts else np.zeros(0, dtype=np.uint8)


def gen_text_stream(n_words, vocab_seed, stream_seed, **kw) -> np.ndarray:
    """Zipfian pseudo-text only."""
    return gen_stream(n_words, vocab_seed, stream_seed, **kw)


# Unit probabilities that give, by *bytes*, 85 % text, 10 % random-byte units and
# 5 % single-character runs (mean unit lengths about 6.3, 33.5 and 2081 bytes).
STRESS_P_RAND = 0.0225
STRESS_P_RUN = 0.000195


def gen_stress_stream(n_words, vocab_seed, stream_seed, **kw) -> np.ndarray:
    return gen_stream(n_words, vocab_seed, stream_seed,
                      p_rand=STRESS_P_RAND, p_run=STRESS_P_RUN, **kw)


def pretokenize(data: np.ndarray, seq_starts=None) -> np.ndarray:
    """Piece boundaries of ``data``: int32 offsets [n_pieces+1], first 0, last
    ``len(data)``.  A piece starts at index 0, at every index in ``seq_starts``
    and before every byte 0x20; nothing else splits."""
    data = np.asarray(data, dtype=np.uint8)
    n = data.size
    if n == 0:
        return np.zeros(1, dtype=np.int32)
    start = data == 0x20
    start[0] = True
    if seq_starts is not None:
        s = np.asarray(seq_starts, dtype=np.int64)
        start[s[s < n]] = True
    off = np.nonzero(start)[0]
    return np.concatenate([off, [n]]).astype(np.int32)


def fixed_chunks(n_bytes: int, chunk_bytes: int) -> np.ndarray:
    """Offsets that cut ``n_bytes`` bytes into chunks of ``chunk_bytes`` (the last
    one shorter): int32 [n_chunks + 1], first 0, last ``n_bytes``.  This is the
    host-side chunking of the paper's pipeline (section 3.1, stage 2; section 3.6),
    used to run its kernels for comparison."""
    assert chunk_bytes >= 1
    off = np.arange(0, n_bytes, chunk_bytes, dtype=np.int64)
    return np.concatenate([off, [n_bytes]]).astype(np.int32)
