"""Pins for oracle.retrieval (Sec. 3.2-3.3, Eq. 5): an explicit trie with node frequencies
(the paper's data structure, built and walked here independently), hand-worked pools,
special cases and invariants."""
import numpy as np
import pytest

from oracle.retrieval import RegroupedPool, retrieve, retrieve_one


# ------------------------------------------------------------------ independent brute force
class _Node:
    __slots__ = ("count", "min_start", "kids")

    def __init__(self):
        self.count, self.min_start, self.kids = 0, None, {}


def _build_trie(seqs, depth):
    """Insert every window seq[s:s+depth] of every sequence; node.count = how many windows
    pass through it, node.min_start = smallest flat start position among them."""
    root = _Node()
    flat = 0
    for seq in seqs:
        for s in range(len(seq)):
            node = root
            for t in seq[s:s + depth]:
                node = node.kids.setdefault(int(t), _Node())
                node.count += 1
                if node.min_start is None:
                    node.min_start = flat + s
        flat += len(seq)
    return root


def trie_retrieve(seqs_of_key, base, ctx, n_min, n_max, K, min_tokens=1):
    """Greedy max-frequency descent below the node reached by the longest usable suffix."""
    ctx = [t for t in ctx if t >= 0]
    root = _build_trie(seqs_of_key, n_max + K)
    best = ([], 0, -1)
    for n in range(min(n_max, len(ctx)), n_min - 1, -1):
        node = root
        for t in ctx[len(ctx) - n:]:
            node = node.kids.get(int(t))
            if node is None:
                break
        if node is None or not node.kids:
            continue
        chain = []
        for _ in range(K):
            if not node.kids:
                break
            tok = min(node.kids, key=lambda t: (-node.kids[t].count, t))
            chain.append(tok)
            node = node.kids[tok]
        cand = (chain, n, base + node.min_start + n - 1)
        if len(chain) >= min_tokens:
            return cand
        if len(chain) > len(best[0]):
            best = cand
    return best


def _flatten(seqs, keys):
    toks = np.array([t for s in seqs for t in s], dtype=np.int32)
    off = np.cumsum([0] + [len(s) for s in seqs]).astype(np.int64)
    return toks, off, np.array(keys, dtype=np.int64)


# ------------------------------------------------------------------ hand-worked examples
def test_worked_example_three_sequences():
    # positions: 0..3 = 1 2 3 4 | 4..7 = 1 2 3 5 | 8..11 = 9 2 3 5
    pool = RegroupedPool(*_flatten([[1, 2, 3, 4], [1, 2, 3, 5], [9, 2, 3, 5]], [7, 7, 7]))
    # suffix (2,3) ends at 2, 6, 10; successors 4,5,5 -> 5 wins; survivors {6,10}; both sequences end
    assert retrieve_one(pool, 7, [8, 2, 3], 1, 2, 2) == ([5], 2, 6)
    # suffix (1,2,3) with n_max 3 ends at 2 and 6; successors 4 and 5 tie -> smaller id 4; survivor {2}
    assert retrieve_one(pool, 7, [1, 2, 3], 1, 3, 2) == ([4], 3, 2)
    # suffix (.,9,2): n=2 occurs once (e=9) -> literal continuation 3,5
    assert retrieve_one(pool, 7, [0, 9, 2], 1, 3, 4) == ([3, 5], 2, 9)
    # unseen last token: nothing at any n
    assert retrieve_one(pool, 7, [1, 2, 6], 1, 3, 4) == ([], 0, -1)
    # a token that only ends sequences (4 at e=3, 5 at e=7, 11) has no successor -> no occurrence
    assert retrieve_one(pool, 7, [2, 3, 4], 1, 3, 4) == ([], 0, -1)
    assert retrieve_one(pool, 7, [2, 3, 5], 1, 1, 4) == ([], 0, -1)
    # unknown key
    assert retrieve_one(pool, 8, [1, 2, 3], 1, 3, 2) == ([], 0, -1)


def test_worked_example_shrinking_n_and_frequency():
    #            0  1  2  3  4  5 | 6  7  8  9 10 | 11 12 13 14
    seqs = [[5, 6, 7, 8, 9, 1], [4, 6, 7, 3, 3], [2, 7, 3, 3]]
    pool = RegroupedPool(*_flatten(seqs, [1, 1, 1]))
    # context ... 0 6 7: n=3 (0,6,7) absent; n=2 (6,7) at e=2 and e=8, successors 8 and 3 tie -> 3
    #   survivors {8}; next 3 (e+2=10, last of its sequence) -> chain [3,3]
    assert retrieve_one(pool, 1, [0, 6, 7], 1, 3, 5) == ([3, 3], 2, 8)
    # n_max = 1: suffix (7) at e=2,8,12: successors 8,3,3 -> 3; survivors {8,12}; then 3,3 -> [3,3]
    assert retrieve_one(pool, 1, [0, 6, 7], 1, 1, 5) == ([3, 3], 1, 8)
    # K caps the chain
    assert retrieve_one(pool, 1, [0, 6, 7], 1, 1, 1) == ([3], 1, 8)
    # matches never straddle a sequence boundary: (1,4) spans seq 0 -> seq 1
    assert retrieve_one(pool, 1, [9, 1, 4], 2, 2, 3) == ([], 0, -1)
    # n_min = 2 forbids falling back to the single token
    assert retrieve_one(pool, 1, [0, 0, 7], 2, 3, 3) == ([], 0, -1)
    # min_tokens: n=3 (5,6,7) gives a 3-token chain 8,9,1; asking for >= 4 falls through to the
    # shorter suffixes, none is longer, so the longest seen (ties -> larger n) is kept
    assert retrieve_one(pool, 1, [5, 6, 7], 1, 3, 8, min_tokens=4) == ([8, 9, 1], 3, 2)


def test_keys_regroup_by_ascending_key_in_supply_order():
    seqs = [[1, 2, 3], [1, 2, 4], [1, 2, 5], [1, 2, 6]]
    pool = RegroupedPool(*_flatten(seqs, [20, 10, 20, 10]))
    assert pool.P.tolist() == [1, 2, 4, 1, 2, 6, 1, 2, 3, 1, 2, 5]
    assert pool.key_range == {10: (0, 6), 20: (6, 12)}
    assert retrieve_one(pool, 10, [1, 2], 1, 2, 3) == ([4], 2, 1)
    assert retrieve_one(pool, 20, [1, 2], 1, 2, 3) == ([3], 2, 7)


def test_special_cases():
    # constant pool: the chain is constant, as long as the sequence allows
    pool = RegroupedPool(*_flatten([[7] * 10], [0]))
    d, n, idx = retrieve_one(pool, 0, [7, 7, 7], 1, 3, 4)
    assert d == [7, 7, 7, 7] and n == 3 and idx == 2
    d, n, idx = retrieve_one(pool, 0, [7, 7, 7], 1, 3, 20)
    assert d == [7] * 7 and idx == 2          # from e=2 seven successors remain
    # exact prefix of a unique sequence: the literal next K tokens
    seq = list(range(100, 140))
    pool = RegroupedPool(*_flatten([seq, list(range(200, 240))], [0, 0]))
    assert retrieve_one(pool, 0, seq[:10], 1, 4, 6) == (seq[10:16], 4, 9)
    # context shorter than n_max (left padding -1)
    assert retrieve_one(pool, 0, [-1, -1, -1, 105], 1, 4, 2) == ([106, 107], 1, 5)
    assert retrieve_one(pool, 0, [-1, -1, -1, -1], 1, 4, 2) == ([], 0, -1)
    assert retrieve_one(pool, 0, seq[:10], 1, 4, 0) == ([], 0, -1)


# ------------------------------------------------------------------ randomised brute force
@pytest.mark.parametrize("seed", range(6))
def test_against_explicit_trie(seed):
    r = np.random.default_rng(seed)
    for trial in range(120):
        vocab = int(r.integers(2, 7))
        n_keys = int(r.integers(1, 4))
        n_seq = int(r.integers(1, 9))
        seqs = [r.integers(0, vocab, size=int(r.integers(1, 25))).tolist() for _ in range(n_seq)]
        keys = r.integers(0, n_keys, size=n_seq).tolist()
        pool = RegroupedPool(*_flatten(seqs, keys))
        n_max = int(r.integers(1, 5))
        n_min = int(r.integers(1, n_max + 1))
        K = int(r.integers(1, 7))
        mt = int(r.integers(1, 4))
        for q in range(6):
            key = int(r.integers(0, n_keys + 1))
            clen = int(r.integers(0, n_max + 1))
            ctx = [-1] * (n_max - clen) + r.integers(0, vocab, size=clen).tolist()
            got = retrieve_one(pool, key, ctx, n_min, n_max, K, mt)
            grouped = [s for s, k in zip(seqs, keys) if k == key]
            base = pool.key_range.get(key, (0, 0))[0]
            want = trie_retrieve(grouped, base, ctx, n_min, n_max, K, mt) if grouped else ([], 0, -1)
            assert got == want, (seed, trial, q, seqs, keys, key, ctx, n_min, n_max, K, mt)
            # invariants
            d, n, idx = got
            assert len(d) <= K
            if d:
                assert pool.P[idx + 1: idx + 1 + len(d)].tolist() == d
                assert pool.P[idx - n + 1: idx + 1].tolist() == ctx[len(ctx) - n:]
                assert pool.seq_end[idx] >= idx + 1 + len(d) and pool.seq_begin[idx] <= idx - n + 1
                lo, hi = pool.key_range[key]
                assert lo <= idx < hi


def test_batched_form_and_padding():
    pool = RegroupedPool(*_flatten([[1, 2, 3, 4], [1, 2, 3, 5], [9, 2, 3, 5]], [7, 7, 7]))
    drafts, dl, mn, pi = retrieve(pool, [7, 8, 7], [[8, 2, 3], [8, 2, 3], [0, 9, 2]], 1, 3, 3)
    assert drafts.tolist() == [[5, -1, -1], [-1, -1, -1], [3, 5, -1]]
    assert dl.tolist() == [1, 0, 2] and mn.tolist() == [2, 0, 2] and pi.tolist() == [6, -1, 9]
    assert drafts.dtype == np.int32 and pi.dtype == np.int64


# ------------------------------------------------------------------ temporary branch (the sequence's own text)
def test_temporary_branch_hand_worked():
    """Sec. 3.2: prompt + generated text join the key's trie for the current generation only."""
    pool = RegroupedPool(*_flatten([[1, 2, 3, 4]], [7]))
    # pool occurrence of (2, 3) at position 2 -> 4; own text has (2, 3) at positions 2 (-> 9) and 6 (its end, no
    # successor: not an occurrence). Votes 4:1, 9:1 -> smaller id 4; the pool sequence ends there.
    own = [7, 2, 3, 9, 5, 2, 3]
    assert retrieve_one(pool, 7, [5, 2, 3], 1, 2, 3, own=own) == ([4], 2, 2)
    # two own occurrences outvote the pool: (2, 3) -> 9 twice
    own = [2, 3, 9, 8, 2, 3, 9, 6, 2, 3]
    assert retrieve_one(pool, 7, [6, 2, 3], 1, 2, 2, own=own) == ([9, 6], 2, -2 - 5)      # 9 then {8, 6} tie -> 6
    # nothing in the pool: the draft comes from the own text alone, index = -2 - position
    pool2 = RegroupedPool(*_flatten([[1, 1, 1]], [7]))
    assert retrieve_one(pool2, 7, [5, 6], 1, 2, 3, own=[5, 6, 7, 5, 6]) == ([7, 5, 6], 2, -3)
    # unknown key: only the own text is searched
    assert retrieve_one(pool2, 99, [5, 6], 1, 2, 3, own=[5, 6, 7, 5, 6]) == ([7, 5, 6], 2, -3)
    # an own text that repeats nothing changes nothing; None and [] are the plain lookup
    plain = retrieve_one(pool, 7, [5, 2, 3], 1, 2, 3)
    assert plain == ([4], 2, 2)
    assert retrieve_one(pool, 7, [5, 2, 3], 1, 2, 3, own=[]) == plain
    assert retrieve_one(pool, 7, [5, 2, 3], 1, 2, 3, own=[8, 8, 5, 2, 3]) == plain


@pytest.mark.parametrize("seed", range(4))
def test_temporary_branch_against_explicit_trie(seed):
    """The own text is one more sequence of the key's trie, inserted after the key's pool sequences."""
    r = np.random.default_rng(100 + seed)
    for trial in range(120):
        vocab = int(r.integers(2, 6))
        n_keys = int(r.integers(1, 3))
        n_seq = int(r.integers(1, 7))
        seqs = [r.integers(0, vocab, size=int(r.integers(1, 20))).tolist() for _ in range(n_seq)]
        keys = r.integers(0, n_keys, size=n_seq).tolist()
        pool = RegroupedPool(*_flatten(seqs, keys))
        n_max = int(r.integers(1, 5))
        n_min = int(r.integers(1, n_max + 1))
        K = int(r.integers(1, 7))
        mt = int(r.integers(1, 4))
        for q in range(6):
            key = int(r.integers(0, n_keys + 1))
            own = r.integers(0, vocab, size=int(r.integers(1, 30))).tolist()
            ctx = ([-1] * n_max + own)[-n_max:]                    # the context is the own text's tail
            got = retrieve_one(pool, key, ctx, n_min, n_max, K, mt, own=own)
            grouped = [s for s, k in zip(seqs, keys) if k == key]
            n_pool = sum(len(s) for s in grouped)
            base = pool.key_range.get(key, (0, 0))[0]
            chain, n, idx = trie_retrieve(grouped + [own], 0, ctx, n_min, n_max, K, mt)
            want = (chain, n, (base + idx if idx < n_pool else -2 - (idx - n_pool)) if idx >= 0 else -1)
            assert got == want, (seed, trial, q, seqs, keys, key, own, n_min, n_max, K, mt)
            d, n, idx = got
            if d and idx <= -2:                                    # the draft literally follows that own-text position
                pos = -2 - idx
                assert own[pos + 1: pos + 1 + len(d)] == d and own[pos - n + 1: pos + 1] == ctx[len(ctx) - n:]
