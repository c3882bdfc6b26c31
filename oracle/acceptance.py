"""Oracle: verification of the drafts (Sec. 2.1 Eq. 4; Sec. 3.4 Eq. 7 and Eq. 8).

TEST INFRASTRUCTURE ONLY -- never imported by the product package.

Row r carries draft x~_{r+1} and the logits of q_{r+1}.  Softmax at temperature 1; ties in
the ordering of probabilities are broken towards the smaller token id, so that k = 1 is
deterministic greedy decoding.

    rank(x) = #{ v : l_v > l_x  or  (l_v == l_x and v < x) }
    q(x)    = exp(l_x - m) / sum_v exp(l_v - m),   m = max_v l_v
    mode 0  (Eq. 8)          accept  <=>  rank(x) < k  and  q(x) > p
    mode 1                   accept  <=>  rank(x) == 0  or  mode-0 condition
    mode 2  (Eq. 7 alone)    accept  <=>  rank(x) < k
    mode 3  (threshold alone, as the ablation words it)  accept <=> rank(x) == 0 or q(x) > p
Greedy verification (Eq. 4) is mode 0 with k = 1 and p < 0.

Rows are examined from the first; the scan stops at the first rejected draft or after
draft_len drafts.  With a accepted drafts the step emits x~_1..x~_a followed by
argmax q_{a+1} (the correction when a draft failed, the bonus token when all passed).

Token trees (Sec. 3.4: "if a predecessor node in the token tree is rejected, all of its successor nodes will be
skipped ... ultimately accepting the verified branch with the maximum length"): node i with token x_i and parent
node parent[i] (-1: child of the root) is examined against the distribution of its parent's row (row parent[i] + 1;
row 0 belongs to the pending token).  It is verified iff its parent is (the root always is) and x_i passes the rule.
The accepted branch is the deepest verified node's path; among equally deep ones the first in the pseudo-sequence.
The step emits that path's tokens followed by the argmax of its last node's row.
"""
from __future__ import annotations

import numpy as np


def row_stats(logits: np.ndarray, x: int, k: int, p: float):
    """For one row: rank, q, argmax and the distances of the decision to its boundaries."""
    l = np.asarray(logits, dtype=np.float64)
    V = l.size
    idx = np.arange(V)
    ahead = (l > l[x]) | ((l == l[x]) & (idx < x))
    rank = int(ahead.sum())
    m = l.max()
    z = np.exp(l - m).sum()
    q = float(np.exp(l[x] - m) / z)
    top = int(np.argmax(l))                                   # first maximum = smallest id
    others = np.delete(l, x)
    if k - 1 < others.size:
        kth_other = np.partition(others, others.size - k)[others.size - k]   # k-th largest of the rest
        rank_margin = float(abs(l[x] - kth_other))
    else:
        rank_margin = float("inf")
    logq_margin = float(abs(np.log(q) - np.log(p))) if (p > 0 and q > 0) else float("inf")
    srt = np.partition(l, V - 2)[V - 2:] if V >= 2 else np.array([l[0], l[0]])
    argmax_gap = float(srt[1] - srt[0]) if V >= 2 else float("inf")
    return {"rank": rank, "q": q, "argmax": top, "rank_margin": rank_margin,
            "logq_margin": logq_margin, "argmax_gap": argmax_gap}


def accepts(rank: int, q: float, k: int, p: float, mode: int) -> bool:
    if mode == 0:
        return rank < k and q > p
    if mode == 1:
        return rank == 0 or (rank < k and q > p)
    if mode == 2:
        return rank < k
    if mode == 3:
        return rank == 0 or q > p
    raise ValueError("mode")


def verify_sequence(logits: np.ndarray, drafts, draft_len: int, k: int, p: float, mode: int = 0):
    """logits [R][V] for rows 0..R-1 (R >= draft_len + 1); drafts[0..draft_len-1].
    Returns (accept_len, emitted tokens list of length accept_len + 1, per-row stats examined)."""
    a = 0
    stats = []
    while a < draft_len:
        st = row_stats(logits[a], int(drafts[a]), k, p)
        st["accepted"] = accepts(st["rank"], st["q"], k, p, mode)
        stats.append(st)
        if not st["accepted"]:
            break
        a += 1
    l = np.asarray(logits[a], dtype=np.float64)
    nxt = int(np.argmax(l))
    srt = np.partition(l, l.size - 2)[l.size - 2:]
    out = [int(t) for t in drafts[:a]] + [nxt]
    return a, out, stats, float(srt[1] - srt[0])


def verify_batch(logits: np.ndarray, drafts: np.ndarray, draft_len, k: int, p: float, mode: int = 0):
    """logits [B][R][V], drafts [B][K] (-1 padded).  Returns accept_len int32[B],
    out_tokens int32[B][K+1] (-1 padded), list of per-sequence row stats, and the
    top-1/top-2 logit gap of each emitting row."""
    B, R = logits.shape[0], logits.shape[1]
    acc = np.zeros(B, dtype=np.int32)
    out = np.full((B, R), -1, dtype=np.int32)
    all_stats, gaps = [], np.zeros(B)
    for b in range(B):
        a, toks, st, gap = verify_sequence(logits[b], drafts[b], int(draft_len[b]), k, p, mode)
        acc[b] = a
        out[b, :len(toks)] = toks
        all_stats.append(st)
        gaps[b] = gap
    return acc, out, all_stats, gaps


def verify_tree(logits: np.ndarray, tokens, parent, n_nodes: int, k: int, p: float, mode: int = 0):
    """logits [R][V] (R >= n_nodes + 1); tokens[i], parent[i] for the nodes of the pseudo-sequence.
    Returns (path: accepted node indices root-side first, emitted tokens (path tokens + one more), per-node stats
    of the examined nodes {node: stats}, top-1/top-2 gap of the emitting row)."""
    verified, depth, stats = {}, {}, {}
    best, best_depth = -1, 0
    for i in range(int(n_nodes)):
        par = int(parent[i])
        assert -1 <= par < i
        if par >= 0 and not verified[par]:
            verified[i] = False                   # skipped: a predecessor was rejected
            continue
        st = row_stats(logits[par + 1], int(tokens[i]), k, p)
        st["accepted"] = accepts(st["rank"], st["q"], k, p, mode)
        stats[i] = st
        verified[i] = st["accepted"]
        if verified[i]:
            depth[i] = (depth[par] if par >= 0 else 0) + 1
            if depth[i] > best_depth:
                best, best_depth = i, depth[i]
    path = []
    i = best
    while i >= 0:
        path.append(i)
        i = int(parent[i])
    path.reverse()
    l = np.asarray(logits[best + 1], dtype=np.float64)
    srt = np.partition(l, l.size - 2)[l.size - 2:]
    out = [int(tokens[i]) for i in path] + [int(np.argmax(l))]
    return path, out, stats, float(srt[1] - srt[0])
