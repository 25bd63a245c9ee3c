"""Independent Python re-statements used to pin the oracle (no oracle code here)."""
from __future__ import annotations


def brute_min_everywhere(piece, merges):
    """Classic formulation: find the lowest rank among the pairs present, merge
    every occurrence of that pair left to right, repeat."""
    rank = {tuple(p): k for k, p in enumerate(merges)}
    s = list(piece)
    while True:
        present = [rank[(s[i], s[i + 1])] for i in range(len(s) - 1) if (s[i], s[i + 1]) in rank]
        if not present:
            return s
        k = min(present)
        a, b = merges[k]
        out, i = [], 0
        while i < len(s):
            if i + 1 < len(s) and s[i] == a and s[i + 1] == b:
                out.append(256 + k)
                i += 2
            else:
                out.append(s[i])
                i += 1
        s = out


def brute_rank_order(piece, merges):
    """Apply rule 0 everywhere, then rule 1 everywhere, ... (valid when every
    rule's parts are made by earlier rules)."""
    s = list(piece)
    for k, (a, b) in enumerate(merges):
        out, i = [], 0
        while i < len(s):
            if i + 1 < len(s) and s[i] == a and s[i + 1] == b:
                out.append(256 + k)
                i += 2
            else:
                out.append(s[i])
                i += 1
        s = out
    return s


def expand_ids(ids, merges):
    """Bytes of a token sequence by recursive expansion of merged ids."""
    out = []
    stack = list(reversed([int(x) for x in ids]))
    while stack:
        t = stack.pop()
        if t < 256:
            out.append(t)
        else:
            a, b = merges[t - 256]
            stack.append(int(b))
            stack.append(int(a))
    return bytes(out)


def naive_train(pieces, n_merges):
    """Recount-everything BPE trainer.  pieces: list of bytes.  Returns
    (merges, final segmentation per distinct piece)."""
    from collections import Counter
    freq = Counter(pieces)
    words = {w: list(w) for w in freq}
    merges = []
    for k in range(n_merges):
        cnt = Counter()
        for w, s in words.items():
            for i in range(len(s) - 1):
                cnt[(s[i], s[i + 1])] += freq[w]
        if not cnt:
            break
        best = max(cnt.values())
        a, b = min(p for p, c in cnt.items() if c == best)
        merges.append((a, b))
        for w, s in words.items():
            out, i = [], 0
            while i < len(s):
                if i + 1 < len(s) and s[i] == a and s[i + 1] == b:
                    out.append(256 + k)
                    i += 2
                else:
                    out.append(s[i])
                    i += 1
            words[w] = out
    return merges, words
