"""Pins for the oracle's token-tree path (Sec. 3.3 tree-based drafting and tree attention; Sec. 3.4: the longest
verified branch): retrieval against an explicitly built trie whose nodes are sorted by an independently written
comparator, tree attention against one chain forward per branch, tree acceptance against brute force over the
root-to-leaf paths, and the strict == greedy invariant for whole tree steps."""
import functools

import numpy as np
import pytest

import synth
from oracle import acceptance, step
from oracle.decoder import Decoder
from oracle.retrieval import RegroupedPool, retrieve_one, retrieve_tree, retrieve_tree_one
from tests.test_oracle_retrieval import _build_trie, _flatten


# ------------------------------------------------------------------ retrieval
def _trie_tree(seqs_of_key, ctx, n_min, n_max, K, min_tokens=1):
    """Independent route: build the trie of all windows, walk to the suffix node, list EVERY node below it (depth
    <= K) with its count, sort the whole list with a comparator written from the rule's wording (higher count, then
    smaller depth, then the earlier parent -- compared recursively --, then the smaller token), keep the first K."""
    ctx = [t for t in ctx if t >= 0]
    root = _build_trie(seqs_of_key, n_max + K)
    best = ([], [], 0)
    for n in range(min(n_max, len(ctx)), n_min - 1, -1):
        node = root
        for t in ctx[len(ctx) - n:]:
            node = node.kids.get(int(t))
            if node is None:
                break
        if node is None or not node.kids:
            continue
        nodes = []                                    # (path tuple, count)

        def walk(nd, path):
            if len(path) == K:
                return
            for t, ch in nd.kids.items():
                nodes.append((path + (t,), ch.count))
                walk(ch, path + (t,))
        walk(node, ())
        count = dict(nodes)

        def cmp(a, b):                                # a, b: paths
            if a == b:
                return 0
            if count[a] != count[b]:
                return -1 if count[a] > count[b] else 1
            if len(a) != len(b):
                return -1 if len(a) < len(b) else 1
            if a[:-1] != b[:-1]:
                return cmp(a[:-1], b[:-1])
            return -1 if a[-1] < b[-1] else 1
        chosen = sorted((p for p, _ in nodes), key=functools.cmp_to_key(cmp))[:K]
        chosen_set = set(chosen)
        assert all(p[:-1] in chosen_set for p in chosen if len(p) > 1)      # closed under parents
        order = {p: i for i, p in enumerate(chosen)}
        tokens, parents = [], []

        def dfs(path, parent_pos):
            pos = len(tokens)
            tokens.append(path[-1]); parents.append(parent_pos)
            for ch in sorted((p for p in chosen if len(p) == len(path) + 1 and p[:-1] == path), key=order.get):
                dfs(ch, pos)
        for top in sorted((p for p in chosen if len(p) == 1), key=order.get):
            dfs(top, -1)
        cand = (tokens, parents, n)
        if len(tokens) >= min_tokens:
            return cand
        if len(tokens) > len(best[0]):
            best = cand
    return best


def test_tree_hand_worked():
    # after the suffix (2, 3): continuations 4 5 | 4 6 | 7 | 4 5  ->  counts: 4:3, 7:1, 4-5:2, 4-6:1
    seqs = [[1, 2, 3, 4, 5], [2, 3, 4, 6], [9, 2, 3, 7], [2, 3, 4, 5, 8]]
    pool = RegroupedPool(*_flatten(seqs, [7, 7, 7, 7]))
    # K = 3: 4 (3), then 4-5 (2), then among the count-1 nodes the shallowest: 7 (depth 1) before 4-6 / 4-5-8
    t, par, f, n = retrieve_tree_one(pool, 7, [2, 3], 1, 2, 3)
    assert (t, par, f, n) == ([4, 5, 7], [-1, 0, -1], [3, 2, 1], 2)
    # K = 5: count-1 nodes by depth, then earlier parent: 7 (d1) | 4-6 (d2) | 4-5-8 (d3); pseudo-sequence is depth-first
    t, par, f, n = retrieve_tree_one(pool, 7, [2, 3], 1, 2, 5)
    assert (t, par, f) == ([4, 5, 8, 6, 7], [-1, 0, 1, 0, -1], [3, 2, 1, 1, 1])
    # K = 1 is the first token of the greedy chain; a single-branch pool gives the chain itself
    assert retrieve_tree_one(pool, 7, [2, 3], 1, 2, 1)[0] == retrieve_one(pool, 7, [2, 3], 1, 2, 1)[0] == [4]
    lone = RegroupedPool(*_flatten([[5, 6, 7, 8, 9]], [1]))
    assert retrieve_tree_one(lone, 1, [5, 6], 1, 2, 4)[:2] == ([7, 8, 9], [-1, 0, 1])
    # unknown key, no match, and shrinking n when the long suffix gives too few nodes
    assert retrieve_tree_one(pool, 8, [2, 3], 1, 2, 3) == ([], [], [], 0)
    assert retrieve_tree_one(pool, 7, [5, 5], 1, 2, 3) == ([8], [-1], [1], 1)      # (5, 5) never occurs; (5) once, before 8
    assert retrieve_tree_one(pool, 7, [6, 6], 1, 2, 3) == ([], [], [], 0)          # 6 ends its sequence: no successor
    t, par, f, n = retrieve_tree_one(pool, 7, [9, 2, 3], 1, 3, 3, min_tokens=2)     # (9,2,3) -> only "7": 1 node < 2
    assert n == 2 and t == [4, 5, 7]


@pytest.mark.parametrize("seed", range(60))
def test_tree_against_explicit_trie(seed):
    r = np.random.default_rng(seed)
    vocab = int(r.integers(2, 6))
    seqs = [r.integers(0, vocab, size=int(r.integers(1, 14))).tolist() for _ in range(int(r.integers(1, 9)))]
    keys = r.integers(0, 2, size=len(seqs)).tolist()
    pool = RegroupedPool(*_flatten(seqs, keys))
    for _ in range(12):
        key = int(r.integers(0, 2))
        n_max = int(r.integers(1, 4)); n_min = int(r.integers(1, n_max + 1))
        K = int(r.integers(1, 9)); mt = int(r.integers(1, 4))
        ctx = r.integers(0, vocab, size=int(r.integers(0, 5))).tolist()
        tail = ([-1] * n_max + ctx)[-n_max:]
        of_key = [s for s, k in zip(seqs, keys) if k == key]
        want = _trie_tree(of_key, tail, n_min, n_max, K, mt)
        got = retrieve_tree_one(pool, key, tail, n_min, n_max, K, mt)
        assert (got[0], got[1], got[3]) == want, (seqs, keys, key, tail, n_min, n_max, K, mt)
        # invariants: parents precede children; frequencies never grow along a branch; at most K nodes
        t, par, f, _ = got
        assert len(t) <= K and all(-1 <= q < i for i, q in enumerate(par))
        assert all(par[i] < 0 or f[i] <= f[par[i]] for i in range(len(t)))
    tk, pa, nn, mn = retrieve_tree(pool, [0, 1], [[-1, 1], [0, 1]], 1, 2, 4)
    for b in range(2):
        t, par, _, n = retrieve_tree_one(pool, b, [[-1, 1], [0, 1]][b], 1, 2, 4)
        assert tk[b, :nn[b]].tolist() == t and pa[b, :nn[b]].tolist() == par and mn[b] == n and (tk[b, nn[b]:] == -1).all()


# ------------------------------------------------------------------ tree attention and acceptance
@pytest.fixture(scope="module")
def tiny():
    sh = synth.SHAPES["tiny"].with_(lm_gain=4.0)
    w = synth.gen_all_weights(sh)
    return sh, Decoder(sh.n_layers, sh.d, sh.n_heads, sh.ffn, sh.vocab, w, sh.eps, sh.rope_base)


def _random_tree(r, K, vocab):
    parents = [-1] + [int(r.integers(-1, i)) for i in range(1, K)]
    # make it a valid pseudo-sequence order (parents before children) -- any parent < i is; tokens random
    return r.integers(0, vocab, size=K).tolist(), parents


def test_tree_attention_equals_one_chain_per_branch(tiny):
    """Tree attention lets every node see only its own branch: the logits of a node's row must equal the logits
    the (pinned) chain forward gives when that branch alone is verified."""
    sh, dec = tiny
    r = np.random.default_rng(5)
    prompt = synth.uniform_tokens(31, 1, 0, 13, sh.vocab).tolist()
    for K in (1, 4, 9):
        tokens, parents = _random_tree(r, K, sh.vocab)
        s = step.Sequence(dec, 0, prompt, 64)
        tree_logits = dec.verify_forward(s.cache, [s.pending] + tokens, [-1] + [q + 1 for q in parents])
        for i in range(K):
            path = [i]
            while parents[path[0]] >= 0:
                path.insert(0, parents[path[0]])
            s2 = step.Sequence(dec, 0, prompt, 64)
            chain_logits = dec.verify_forward(s2.cache, [s2.pending] + [tokens[j] for j in path])
            np.testing.assert_allclose(tree_logits[i + 1], chain_logits[len(path)], rtol=0, atol=1e-10)
        np.testing.assert_allclose(tree_logits[0], dec.verify_forward(step.Sequence(dec, 0, prompt, 64).cache, [prompt[-1]])[0], atol=1e-10)


@pytest.mark.parametrize("seed", range(40))
def test_tree_acceptance_against_paths_brute_force(seed):
    """Brute force: every root-to-node path is a chain; the tree's accepted branch is the path with the longest
    accepted prefix under the (pinned) chain rule, the first such path in pseudo-sequence order."""
    r = np.random.default_rng(seed)
    V, K = 12, int(r.integers(1, 9))
    n_nodes = int(r.integers(0, K + 1))
    tokens, parents = _random_tree(r, K, V)
    logits = r.standard_normal((K + 1, V)) * 2.0
    for i in range(n_nodes):                       # make a good share of the drafts likely
        if r.random() < 0.6:
            tokens[i] = int(np.argsort(-logits[parents[i] + 1], kind="stable")[int(r.integers(0, 3))])
    k, p, mode = int(r.integers(1, 4)), float(r.choice([-1.0, 0.05, 0.2])), int(r.integers(0, 4))
    path, out, stats, gap = acceptance.verify_tree(logits, tokens, parents, n_nodes, k, p, mode)
    best = ([], None)
    for i in range(n_nodes):
        chain = [i]
        while parents[chain[0]] >= 0:
            chain.insert(0, parents[chain[0]])
        rows = [0] + [j + 1 for j in chain]
        a, toks, _, _ = acceptance.verify_sequence(logits[rows], [tokens[j] for j in chain], len(chain), k, p, mode)
        if a == len(chain) and a > len(best[0]):
            best = (chain, toks)
    if best[1] is None:
        assert path == [] and out == [int(np.argmax(logits[0]))]
    else:
        assert path == best[0] and out == best[1]
    assert all(parents[path[j]] == (path[j - 1] if j else -1) for j in range(len(path)))


def test_strict_tree_steps_reproduce_greedy_decoding_and_one_branch_equals_the_chain_step(tiny):
    sh, dec = tiny
    prompt = synth.uniform_tokens(14, 1, 0, 9, sh.vocab).tolist()
    ref = step.autoregressive_greedy(dec, step.Sequence(dec, 5, prompt, 128), 30)
    text = np.array(prompt + ref, dtype=np.int32)
    noisy = text.copy(); noisy[12::5] = (noisy[12::5] + 1) % sh.vocab
    pool = RegroupedPool(np.concatenate([text, noisy]), np.array([0, text.size, 2 * text.size]), np.array([5, 5]))
    s = step.Sequence(dec, 5, prompt, 128)
    total = 0
    while total < 30:
        res = step.laser_tree_step(dec, pool, [s], 1, 3, 6, 1, -1.0)
        a = int(res["accept_len"][0])
        assert 0 <= a <= int(res["tree_len"][0]) <= 6
        assert s.cache.length == len(s.tokens) - 1
        total += a + 1
    assert s.tokens[len(prompt):len(prompt) + 30] == ref
    # a tree that is one branch gives exactly the chain step's result (same logits, same decision, same cache)
    r = np.random.default_rng(2)
    drafts = np.array([ref[:3] + r.integers(0, sh.vocab, size=2).tolist()])
    s1, s2 = step.Sequence(dec, 5, prompt, 64), step.Sequence(dec, 5, prompt, 64)
    c = step.verify_step(dec, [s1], drafts, [5], 2, 0.1, 0, return_logits=True)
    t = step.verify_tree_step(dec, [s2], drafts, np.array([[-1, 0, 1, 2, 3]]), [5], 2, 0.1, 0, return_logits=True)
    assert c["accept_len"].tolist() == t["accept_len"].tolist() and c["out_tokens"].tolist() == t["out_tokens"].tolist()
    np.testing.assert_array_equal(c["logits"], t["logits"])
    assert s1.tokens == s2.tokens and s1.cache.length == s2.cache.length
    np.testing.assert_array_equal(s1.cache.k[:, :s1.cache.length], s2.cache.k[:, :s2.cache.length])
    # and a two-branch tree whose SECOND branch is the right one: its keys/values are moved behind the pending token
    wrong = (ref[0] + 1) % sh.vocab
    s3 = step.Sequence(dec, 5, prompt, 64)
    t = step.verify_tree_step(dec, [s3], np.array([[wrong, ref[1], ref[0], ref[1], ref[2]]]), np.array([[-1, 0, -1, 2, 3]]), [5], 1, -1.0)
    assert t["accept_path"][0, :3].tolist() == [2, 3, 4] and t["out_tokens"][0, :4].tolist() == ref[:4]
    s4 = step.Sequence(dec, 5, prompt, 64)
    step.verify_step(dec, [s4], np.array([ref[:3]]), [3], 1, -1.0)
    assert s3.cache.length == s4.cache.length
    np.testing.assert_allclose(s3.cache.k[:, :s3.cache.length], s4.cache.k[:, :s4.cache.length], atol=1e-12)
    np.testing.assert_allclose(s3.cache.v[:, :s3.cache.length], s4.cache.v[:, :s4.cache.length], atol=1e-12)


def test_generate_stops_at_eos_and_max_new_and_matches_greedy_under_strict(tiny):
    """The generation loop (Sec. 3.1): under strict verification the emitted text is the greedy text, whatever the
    drafts (chain, tree, temporary branch, none), cut after the end-of-sequence token or at max_new_tokens."""
    sh, dec = tiny
    prompts = [synth.uniform_tokens(15 + i, 1, 0, 7 + i, sh.vocab).tolist() for i in range(2)]
    ref = [step.autoregressive_greedy(dec, step.Sequence(dec, i, pr, 128), 40) for i, pr in enumerate(prompts)]
    flat = np.concatenate([np.array(pr[-3:] + rf, dtype=np.int32) for pr, rf in zip(prompts, ref)])
    off = np.array([0, 43, 86]); pool = RegroupedPool(flat, off, np.array([0, 1]))
    eos = ref[0][17]
    stop0 = ref[0].index(eos) + 1
    for kw in (dict(), dict(tree=True), dict(temporary_branch=16)):
        seqs = [step.Sequence(dec, i, pr, 128) for i, pr in enumerate(prompts)]
        texts, cnt = step.generate(dec, pool, seqs, 1, 3, 6, 1, -1.0, max_new_tokens=29, eos_token=eos, **kw)
        want1 = ref[1][:29] if eos not in ref[1][:29] else ref[1][:ref[1].index(eos) + 1]
        assert texts[0] == ref[0][:min(stop0, 29)] and texts[1] == want1, kw
        for s, pr, t, c in zip(seqs, prompts, texts, cnt):
            assert s.tokens == pr + t and s.cache.length == len(s.tokens) - 1
            assert c[2] == len(t) - c[0] and c[2] <= c[3] <= c[1] and c[0] < len(t)       # several tokens per step
    seqs = [step.Sequence(dec, i, pr, 128) for i, pr in enumerate(prompts)]
    texts, cnt = step.generate(dec, None, seqs, 1, 3, 6, 1, -1.0, max_new_tokens=12)
    assert texts == [r[:12] for r in ref] and all(c == [12, 0, 0, 0] for c in cnt)
