"""Oracle: draft retrieval from a per-key pool (Sec. 3.2 pool construction, Sec. 3.3 Eq. 5).

TEST INFRASTRUCTURE ONLY -- never imported by the product package.

The paper keeps each group's old texts in a trie whose nodes carry tokens, looks up the
last n context tokens, shrinks n when too little comes back and prefers high-frequency
tokens when too much does.  Here that is written on plain sets of pool positions, by a
naive scan of the key's sub-pool, so that the answer does not depend on any index
structure:

  * the sub-pool of a key is the concatenation, in the order supplied, of the sequences
    tagged with that key; sub-pools are laid out by ascending key ("regrouped pool");
  * an occurrence of an n-gram w is a position e with P[e-n+1..e] == w, all inside one
    sequence, whose successor e+1 lies in the same sequence;
  * for n = min(n_max, context length) down to n_min: take all occurrences; extend a chain
    one token at a time by the most frequent successor among the surviving occurrences
    (ties -> smallest token id), keeping only the occurrences that agree with it; stop
    after K tokens or when no survivor has a successor left;
  * the first n whose chain has >= min_tokens tokens wins; otherwise the longest chain seen
    (ties -> larger n); nothing found -> draft_len 0, match_n 0, pool_index -1;
  * pool_index is the smallest surviving position (flat index in the regrouped pool), so
    P[pool_index+1 .. pool_index+draft_len] equals the draft.

This equals greedy descent of the paper's trie from the node the suffix reaches, always
into the child with the highest frequency (frequency = number of occurrences of the path).

Temporary branch (Sec. 3.2: the current prompt and the text generated so far are added to the
group's trie for the duration of this generation only): `own`, the sequence's own text, counts
as ONE MORE SEQUENCE of the key's sub-pool, placed after all of the key's pool sequences. The
rules above are unchanged (its last position, which the context suffix itself ends at, has no
successor and is therefore never an occurrence). A result whose smallest surviving position
lies in the own text is reported as pool_index = -2 - (position in the own text).

Tree drafts (Sec. 3.3, "tree-based drafting"): instead of one chain, the sub-tree of the trie below the node
the suffix reaches is retrieved, cut to at most K nodes. A node is a path of successor tokens; its frequency is
the number of occurrences whose continuation starts with that path. The paper keeps the highest-frequency tokens
when a retrieval returns more than K of them; here that reads: nodes are taken one at a time, always the best node not
yet taken whose parent is taken (the root's children at the start), best = higher frequency, then smaller
depth, then the parent that was taken earlier, then the smaller token id. (A child never has a higher frequency
than its parent, so this yields the K best nodes of the whole sub-tree in that order, and the result is a tree.)
The pseudo-sequence lists the nodes depth-first, the children of a node in the order they were taken (higher
frequency first, smaller token id on ties); parent[i] is the pseudo-sequence index of node i's parent, -1 for
children of the root. n is chosen as for chains: the first n (from n_max down) whose tree has >= min_tokens
nodes, else the largest tree seen (ties -> larger n).
"""
from __future__ import annotations

import numpy as np


class RegroupedPool:
    """Flat tokens grouped by ascending key plus per-position sequence bounds."""

    def __init__(self, tokens, seq_off, seq_key):
        tokens = np.asarray(tokens, dtype=np.int32)
        seq_off = np.asarray(seq_off, dtype=np.int64)
        seq_key = np.asarray(seq_key, dtype=np.int64)
        n_seq = seq_key.size
        order = np.argsort(seq_key, kind="stable")          # ascending key, supply order within a key
        lens = (seq_off[1:] - seq_off[:-1])[order]
        new_off = np.zeros(n_seq + 1, dtype=np.int64)
        np.cumsum(lens, out=new_off[1:])
        P = np.empty(int(new_off[-1]), dtype=np.int32)
        for i, s in enumerate(order):
            P[new_off[i]:new_off[i + 1]] = tokens[seq_off[s]:seq_off[s + 1]]
        self.P = P
        self.seq_begin = np.repeat(new_off[:-1], lens)      # per position: first index of its sequence
        self.seq_end = np.repeat(new_off[1:], lens)         # per position: one past its sequence
        self.key_range = {}
        keys_sorted = seq_key[order]
        i = 0
        while i < n_seq:
            j = i
            while j < n_seq and keys_sorted[j] == keys_sorted[i]:
                j += 1
            self.key_range[int(keys_sorted[i])] = (int(new_off[i]), int(new_off[j]))
            i = j


def _occurrences(pool: RegroupedPool, lo: int, hi: int, w: np.ndarray) -> np.ndarray:
    """All positions e in [lo, hi) that end an in-sequence copy of w and have an in-sequence successor."""
    n = w.size
    e = np.arange(lo, hi, dtype=np.int64)
    ok = (e - n + 1 >= pool.seq_begin[lo:hi]) & (e + 1 < pool.seq_end[lo:hi])
    e = e[ok]
    for j in range(n):                       # compare the j-th token from the end
        e = e[pool.P[e - j] == w[n - 1 - j]]
    return e


def _greedy_chain(pool: RegroupedPool, M: np.ndarray, K: int):
    chain = []
    for j in range(1, K + 1):
        alive = M[M + j < pool.seq_end[M]]
        if alive.size == 0:
            break
        succ = pool.P[alive + j]
        vals, counts = np.unique(succ, return_counts=True)   # vals ascending -> first max = smallest id
        tok = vals[np.argmax(counts)]
        chain.append(int(tok))
        M = alive[succ == tok]
    return chain, M


def _best_first_tree(pool: RegroupedPool, M0: np.ndarray, K: int):
    """Nodes of the continuation trie below the occurrences M0, taken best first (see the module text).
    Returns the taken nodes in the order taken: (token, index of the parent among the taken nodes or -1, depth, frequency)."""
    taken, frontier = [], []          # frontier entries: (-frequency, depth, parent index, token, occurrences)

    def grow(parent_idx: int, occ: np.ndarray, depth: int):
        """children of a taken node (or of the root): successors at offset depth + 1 of its occurrences"""
        alive = occ[occ + depth + 1 < pool.seq_end[occ]]
        if alive.size == 0:
            return
        succ = pool.P[alive + depth + 1]
        for tok in np.unique(succ):
            sel = alive[succ == tok]
            frontier.append((-int(sel.size), depth + 1, parent_idx, int(tok), sel))

    grow(-1, M0, 0)
    while frontier and len(taken) < K:
        j = min(range(len(frontier)), key=lambda i: frontier[i][:4])
        negf, depth, parent_idx, tok, occ = frontier.pop(j)
        taken.append((tok, parent_idx, depth, -negf))
        grow(len(taken) - 1, occ, depth)
    return taken


def _depth_first(taken):
    """Pseudo-sequence of the taken nodes: depth-first, siblings in the order they were taken.
    Returns (tokens, parents as pseudo-sequence indices (-1 = root), frequencies)."""
    kids = {}
    for i, (_, parent_idx, _, _) in enumerate(taken):
        kids.setdefault(parent_idx, []).append(i)              # ascending i = order taken
    tokens, parents, freqs = [], [], []

    def visit(i: int, parent_pos: int):
        pos = len(tokens)
        tokens.append(taken[i][0]); parents.append(parent_pos); freqs.append(taken[i][3])
        for c in kids.get(i, []):
            visit(c, pos)

    for c in kids.get(-1, []):
        visit(c, -1)
    return tokens, parents, freqs


def retrieve_tree_one(pool: RegroupedPool, key: int, ctx_tail, n_min: int, n_max: int, K: int, min_tokens: int = 1):
    """Tree form of retrieve_one.  Returns (tokens list, parents list, frequencies list, match_n)."""
    ctx = np.asarray(ctx_tail, dtype=np.int64)
    valid = 0
    while valid < ctx.size and ctx[ctx.size - 1 - valid] >= 0:
        valid += 1
    min_tokens = max(1, min_tokens)
    rng_ = pool.key_range.get(int(key))
    if rng_ is None or K <= 0:
        return [], [], [], 0
    lo, hi = rng_
    best = ([], [], [], 0)
    for n in range(min(n_max, valid), max(n_min, 1) - 1, -1):
        M0 = _occurrences(pool, lo, hi, ctx[ctx.size - n:])
        if M0.size == 0:
            continue
        tokens, parents, freqs = _depth_first(_best_first_tree(pool, M0, K))
        cand = (tokens, parents, freqs, n)
        if len(tokens) >= min_tokens:
            return cand
        if len(tokens) > len(best[0]):
            best = cand
    return best


def retrieve_tree(pool: RegroupedPool, keys, ctx_tails, n_min: int, n_max: int, K: int, min_tokens: int = 1):
    """Batched form.  Returns tokens int32[B][K] (-1 padded), parents int32[B][K] (-1 padded and for children of
    the root), n_nodes int32[B], match_n int32[B]."""
    B = len(keys)
    tokens = np.full((B, K), -1, dtype=np.int32)
    parents = np.full((B, K), -1, dtype=np.int32)
    nn = np.zeros(B, dtype=np.int32)
    mn = np.zeros(B, dtype=np.int32)
    for b in range(B):
        t, par, _, n = retrieve_tree_one(pool, keys[b], ctx_tails[b], n_min, n_max, K, min_tokens)
        tokens[b, :len(t)] = t
        parents[b, :len(t)] = par
        nn[b], mn[b] = len(t), n
    return tokens, parents, nn, mn


class _SubPoolWithOwnText:
    """The key's sub-pool [lo, hi) followed by the sequence's own text, as one position space."""

    def __init__(self, pool: RegroupedPool, lo: int, hi: int, own):
        own = np.asarray(own, dtype=np.int32)
        n = hi - lo
        self.P = np.concatenate([pool.P[lo:hi], own])
        self.seq_begin = np.concatenate([pool.seq_begin[lo:hi] - lo, np.full(own.size, n, dtype=np.int64)])
        self.seq_end = np.concatenate([pool.seq_end[lo:hi] - lo, np.full(own.size, n + own.size, dtype=np.int64)])
        self.n_pool, self.lo = n, lo

    def report(self, idx: int) -> int:
        return self.lo + idx if idx < self.n_pool else -2 - (idx - self.n_pool)


def retrieve_one(pool: RegroupedPool, key: int, ctx_tail, n_min: int, n_max: int, K: int,
                 min_tokens: int = 1, own=None):
    """ctx_tail: the last tokens of the context, right-aligned; entries < 0 are left padding.
    own: the sequence's own text so far (temporary branch), or None.
    Returns (drafts list, match_n, pool_index)."""
    if own is not None and len(own) > 0:
        lo, hi = pool.key_range.get(int(key), (0, 0))
        q = _SubPoolWithOwnText(pool, lo, hi, own)
        q.key_range = {int(key): (0, q.P.size)}
        chain, n, idx = retrieve_one(q, key, ctx_tail, n_min, n_max, K, min_tokens)
        return chain, n, (q.report(idx) if idx >= 0 else -1)
    ctx = np.asarray(ctx_tail, dtype=np.int64)
    valid = 0
    while valid < ctx.size and ctx[ctx.size - 1 - valid] >= 0:
        valid += 1
    min_tokens = max(1, min_tokens)
    rng_ = pool.key_range.get(int(key))
    if rng_ is None or K <= 0:
        return [], 0, -1
    lo, hi = rng_
    best = ([], 0, -1)
    for n in range(min(n_max, valid), max(n_min, 1) - 1, -1):
        M0 = _occurrences(pool, lo, hi, ctx[ctx.size - n:])
        if M0.size == 0:
            continue
        chain, M = _greedy_chain(pool, M0, K)
        cand = (chain, n, int(M.min()))
        if len(chain) >= min_tokens:
            return cand
        if len(chain) > len(best[0]):
            best = cand
    return best


def retrieve(pool: RegroupedPool, keys, ctx_tails, n_min: int, n_max: int, K: int, min_tokens: int = 1, own=None):
    """Batched form; own: per sequence its own text (list of arrays) or None.  Returns drafts int32[B][K]
    (-1 padded), draft_len int32[B], match_n int32[B], pool_index int64[B]."""
    B = len(keys)
    drafts = np.full((B, K), -1, dtype=np.int32)
    dl = np.zeros(B, dtype=np.int32)
    mn = np.zeros(B, dtype=np.int32)
    pi = np.full(B, -1, dtype=np.int64)
    for b in range(B):
        c, n, idx = retrieve_one(pool, keys[b], ctx_tails[b], n_min, n_max, K, min_tokens,
                                 None if own is None else own[b])
        drafts[b, :len(c)] = c
        dl[b], mn[b], pi[b] = len(c), n, idx
    return drafts, dl, mn, pi
