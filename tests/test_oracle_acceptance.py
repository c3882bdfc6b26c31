"""Pins for oracle.acceptance and oracle.step (Eq. 4, 7, 8 and the correction rule of Sec. 2.1):
full-sort brute force on small vocabularies, closed forms, and the invariants the paper
states (strict verification reproduces greedy autoregressive decoding; at most K+1 tokens
per step; relaxing can only lengthen acceptance)."""
import math

import numpy as np
import pytest

import synth
from oracle import acceptance, step
from oracle.decoder import Decoder
from oracle.retrieval import RegroupedPool


# ------------------------------------------------------------------ brute force by literal definition
def brute_accept(logits_row, x, k, p):
    """TopK as a literally sorted list of (probability desc, id asc); membership and threshold."""
    l = [float(v) for v in logits_row]
    m = max(l)
    ex = [math.exp(v - m) for v in l]
    z = sum(ex)
    prob = [e / z for e in ex]
    order = sorted(range(len(l)), key=lambda v: (-l[v], v))
    return (x in order[:k]), prob[x] > p, order[0], order.index(x)


@pytest.mark.parametrize("seed", range(4))
def test_rows_against_full_sort(seed):
    r = np.random.default_rng(seed)
    for _ in range(300):
        V = int(r.integers(2, 40))
        l = np.round(r.standard_normal(V) * 2, 1)          # coarse grid -> plenty of exact ties
        x = int(r.integers(0, V))
        k = int(r.integers(1, 5))
        p = float(r.choice([-1.0, 0.0, 0.05, 0.1, 0.3]))
        st = acceptance.row_stats(l, x, k, p)
        in_topk, above, top, pos = brute_accept(l, x, k, p)
        assert st["rank"] == pos and st["argmax"] == top
        assert (st["rank"] < k) == in_topk and (st["q"] > p) == above
        assert acceptance.accepts(st["rank"], st["q"], k, p, 0) == (in_topk and above)
        assert acceptance.accepts(st["rank"], st["q"], k, p, 1) == (pos == 0 or (in_topk and above))
        assert acceptance.accepts(st["rank"], st["q"], k, p, 2) == in_topk
        assert acceptance.accepts(st["rank"], st["q"], k, p, 3) == (pos == 0 or above)


def test_closed_forms():
    NEG = -1e30
    # two live logits a, b: q(a) = sigmoid(a - b); q > 0.1 <=> a - b > ln(1/9)
    for gap, want in [(-2.19, True), (-2.20, False), (0.0, True)]:
        l = np.full(10, NEG); l[3] = gap; l[7] = 0.0
        st = acceptance.row_stats(l, 3, 2, 0.1)
        assert np.isclose(st["q"], 1 / (1 + math.exp(-gap)))
        assert acceptance.accepts(st["rank"], st["q"], 2, 0.1, 0) == want
        assert np.isclose(st["logq_margin"], abs(math.log(st["q"]) - math.log(0.1)))
    # uniform logits: q = 1/V and rank = token id (ties to the smaller id)
    l = np.zeros(16)
    for x in (0, 1, 5):
        st = acceptance.row_stats(l, x, 2, 0.05)
        assert st["rank"] == x and np.isclose(st["q"], 1 / 16) and st["argmax"] == 0
    # threshold is strict: q == p rejects
    l = np.zeros(4)
    st = acceptance.row_stats(l, 0, 1, 0.25)
    assert st["q"] == 0.25 and not acceptance.accepts(st["rank"], st["q"], 1, 0.25, 0)
    # rank margin: logits 5,4,3,1 ; x = id 2 (l=3), k=2 -> boundary is the 2nd largest other (4)
    st = acceptance.row_stats(np.array([5.0, 4.0, 3.0, 1.0]), 2, 2, 0.0)
    assert st["rank"] == 2 and np.isclose(st["rank_margin"], 1.0) and np.isclose(st["argmax_gap"], 1.0)
    st = acceptance.row_stats(np.array([5.0, 4.0, 3.0, 1.0]), 1, 2, 0.0)
    assert st["rank"] == 1 and np.isclose(st["rank_margin"], 1.0)   # other logits 5,3,1: 2nd largest is 3


def test_scan_stops_and_corrects():
    V = 6
    L = np.full((4, V), -5.0)
    L[0, 2] = 3.0                      # argmax 2
    L[1, 4] = 3.0; L[1, 1] = 2.5       # argmax 4, runner-up 1
    L[2, 0] = 3.0
    L[3, 5] = 3.0
    # strict: drafts 2,1,0 -> first accepted, second rejected -> corrected to 4
    a, out, st, _ = acceptance.verify_sequence(L, [2, 1, 0], 3, 1, -1.0)
    assert (a, out) == (1, [2, 4]) and len(st) == 2
    # relaxed k=2: runner-up passes (q = e^2.5 / (e^3 + e^2.5 + 4 e^-5) ~ 0.377 > 0.1) -> all three + bonus 5
    a, out, _, _ = acceptance.verify_sequence(L, [2, 1, 0], 3, 2, 0.1)
    assert (a, out) == (3, [2, 1, 0, 5])
    # threshold bites: p = 0.4 rejects the runner-up again
    a, out, _, _ = acceptance.verify_sequence(L, [2, 1, 0], 3, 2, 0.4)
    assert (a, out) == (1, [2, 4])
    # draft_len 0 -> plain greedy step
    assert acceptance.verify_sequence(L, [9, 9, 9], 0, 2, 0.1)[:2] == (0, [2])
    # batch form pads with -1
    acc, out, _, _ = acceptance.verify_batch(L[None], np.array([[2, 1, 0]]), [3], 1, -1.0)
    assert acc.tolist() == [1] and out.tolist() == [[2, 4, -1, -1]]


def test_monotone_in_k_and_p():
    r = np.random.default_rng(5)
    for _ in range(200):
        V, R = 12, 6
        L = r.standard_normal((R, V)) * 3
        d = r.integers(0, V, size=R - 1)
        prev = -1
        for k in (1, 2, 3, 5):
            a = acceptance.verify_sequence(L, d, R - 1, k, 0.05)[0]
            assert a >= prev; prev = a
        prev = 99
        for p in (-1.0, 0.01, 0.1, 0.3, 0.9):
            a = acceptance.verify_sequence(L, d, R - 1, 3, p)[0]
            assert a <= prev; prev = a
        # mode 1 is never shorter than strict; mode 0 can be only when the top-1 probability is <= p
        strict = acceptance.verify_sequence(L, d, R - 1, 1, -1.0)[0]
        assert acceptance.verify_sequence(L, d, R - 1, 2, 0.1, mode=1)[0] >= strict


# ------------------------------------------------------------------ whole-step invariants on the tiny model
@pytest.fixture(scope="module")
def tiny():
    sh = synth.SHAPES["tiny"].with_(lm_gain=4.0)
    w = synth.gen_all_weights(sh)
    return sh, Decoder(sh.n_layers, sh.d, sh.n_heads, sh.ffn, sh.vocab, w, sh.eps, sh.rope_base)


def test_strict_verification_reproduces_greedy_decoding(tiny):
    sh, dec = tiny
    prompt = synth.uniform_tokens(11, 1, 0, 12, sh.vocab).tolist()
    ref_seq = step.Sequence(dec, 0, prompt, 96)
    ref = step.autoregressive_greedy(dec, ref_seq, 24)
    r = np.random.default_rng(3)
    K = 4
    for kind in ("random", "perfect", "half", "empty"):
        s = step.Sequence(dec, 0, prompt, 96)
        produced = []
        while len(produced) < 24:
            done = len(produced)
            truth = ref[done:done + K]
            if kind == "random":
                d, dl = r.integers(0, sh.vocab, size=K).tolist(), K
            elif kind == "perfect":
                d, dl = truth + [0] * (K - len(truth)), len(truth)
            elif kind == "half":
                d = truth[:2] + r.integers(0, sh.vocab, size=K - len(truth[:2])).tolist(); dl = K
            else:
                d, dl = [-1] * K, 0
            res = step.verify_step(dec, [s], np.array([d]), [dl], 1, -1.0)
            a = int(res["accept_len"][0])
            assert 0 <= a <= dl <= K
            emitted = res["out_tokens"][0, :a + 1].tolist()
            assert len(emitted) <= K + 1
            if kind == "perfect":
                assert a == dl
            if kind == "empty":
                assert a == 0
            if kind == "half" and len(truth) >= 2:
                assert a >= 2
            produced += emitted
        assert produced[:24] == ref, kind
        assert s.tokens[len(prompt):len(prompt) + 24] == ref


def test_relaxed_step_emits_only_rule_abiding_tokens(tiny):
    sh, dec = tiny
    prompt = synth.uniform_tokens(12, 1, 0, 10, sh.vocab).tolist()
    s = step.Sequence(dec, 0, prompt, 64)
    r = np.random.default_rng(8)
    for _ in range(6):
        d = r.integers(0, sh.vocab, size=4)
        before = list(s.tokens)
        res = step.verify_step(dec, [s], d[None], [4], 2, 0.1, return_logits=True)
        a = int(res["accept_len"][0])
        # replay: each accepted draft must satisfy Eq. 8 under a fresh single-row forward
        chk = step.Sequence(dec, 0, before, 64)
        for j in range(a):
            l = dec.verify_forward(chk.cache, [chk.pending])[0]
            chk.cache.commit(1)
            pr = np.exp(l - l.max()); pr /= pr.sum()
            assert d[j] in np.argsort(-l, kind="stable")[:2] and pr[d[j]] > 0.1
            chk.tokens.append(int(d[j]))
        l = dec.verify_forward(chk.cache, [chk.pending])[0]
        assert res["out_tokens"][0, a] == int(np.argmax(l))
        assert s.cache.length == len(s.tokens) - 1


def test_laser_step_uses_pool_and_matches_greedy_under_strict(tiny):
    sh, dec = tiny
    prompt = synth.uniform_tokens(13, 1, 0, 8, sh.vocab).tolist()
    ref = step.autoregressive_greedy(dec, step.Sequence(dec, 5, prompt, 96), 30)
    # pool = the model's own earlier output (how the paper builds pools), under key 5
    text = np.array(prompt + ref, dtype=np.int32)
    pool = RegroupedPool(text, np.array([0, text.size]), np.array([5]))
    s = step.Sequence(dec, 5, prompt, 96)
    steps, total = 0, 0
    while total < 30:
        res = step.laser_step(dec, pool, [s], 1, 3, 5, 1, -1.0)
        total += int(res["accept_len"][0]) + 1
        steps += 1
    assert s.tokens[len(prompt):len(prompt) + 30] == ref
    assert steps <= 8                      # ~6 tokens per step when the pool holds the answer


def test_laser_step_temporary_branch_is_the_last_w_tokens_of_the_own_text(tiny):
    """Sec. 3.2: the current prompt and the text generated so far join the key's trie while the text is being
    generated. laser_step(temporary_branch=W) must hand retrieval exactly the last W tokens the sequence holds
    (prompt + everything emitted so far), per sequence. Pinned by (1) a hand-worked window, (2) an explicit trie
    built independently over pool + own text at every step of a generation, (3) strict == greedy."""
    from tests.test_oracle_retrieval import trie_retrieve
    sh, dec = tiny
    empty = RegroupedPool(np.zeros(0, dtype=np.int32), np.array([0]), np.zeros(0, dtype=np.int64))
    # (1) own text 5 6 7 8 9 1 2 3 5 6: the suffix (5, 6) occurred at its start, followed by 7 8 9 1.
    #     A window of 10 tokens sees that occurrence, a window of 4 tokens (2 3 5 6) does not.
    prompt = [5, 6, 7, 8, 9, 1, 2, 3, 5, 6]
    for W, want_drafts, want_idx in ((10, [7, 8, 9, 1], -2 - 1), (8, [], -1), (4, [], -1)):
        s = step.Sequence(dec, 3, prompt, 64)
        res = step.laser_step(dec, empty, [s], 1, 2, 4, 1, -1.0, temporary_branch=W)
        assert res["drafts"][0, :res["draft_len"][0]].tolist() == want_drafts, W
        assert int(res["pool_index"][0]) == want_idx and int(res["match_n"][0]) == (2 if want_drafts else 0)
    # without the branch nothing is found at all
    s = step.Sequence(dec, 3, prompt, 64)
    assert int(step.laser_step(dec, empty, [s], 1, 2, 4, 1, -1.0)["draft_len"][0]) == 0
    # (2) + (3): two sequences of different keys generate 20 tokens each; every step's drafts equal the greedy
    # descent of an explicit trie over [pool sequences of the key] + [last W tokens of that sequence]
    pool_seqs = [[9, 4, 4, 7, 1, 2], [4, 4, 8, 3], [1, 2, 3, 4, 4, 7]]
    pool_keys = [1, 2, 1]
    toks = np.array([t for q in pool_seqs for t in q], dtype=np.int32)
    off = np.cumsum([0] + [len(q) for q in pool_seqs]).astype(np.int64)
    pool = RegroupedPool(toks, off, np.array(pool_keys, dtype=np.int64))
    prompts = {1: synth.uniform_tokens(21, 1, 0, 9, sh.vocab).tolist() + [4, 4], 2: [4, 4, 8, 4, 4]}
    refs = {k: step.autoregressive_greedy(dec, step.Sequence(dec, k, pr, 96), 20) for k, pr in prompts.items()}
    W, n_max, K = 7, 2, 3
    seqs = [step.Sequence(dec, k, prompts[k], 96) for k in (1, 2)]
    base = {1: 0, 2: sum(len(q) for q, k in zip(pool_seqs, pool_keys) if k == 1)}
    n_pool = {k: sum(len(q) for q, kk in zip(pool_seqs, pool_keys) if kk == k) for k in (1, 2)}
    for _ in range(12):
        before = [list(s.tokens) for s in seqs]
        res = step.laser_step(dec, pool, seqs, 1, n_max, K, 1, -1.0, temporary_branch=W)
        for i, s in enumerate(seqs):
            own = before[i][-W:]
            of_key = [q for q, k in zip(pool_seqs, pool_keys) if k == s.key]
            chain, n, idx = trie_retrieve(of_key + [own], base[s.key], before[i][-n_max:], 1, n_max, K)
            assert res["drafts"][i, :res["draft_len"][i]].tolist() == chain
            if chain:
                # positions past the key's pool text lie in the own text and are reported as -2 - position
                want = idx if idx - base[s.key] < n_pool[s.key] else -2 - (idx - base[s.key] - n_pool[s.key])
                assert int(res["pool_index"][i]) == want and int(res["match_n"][i]) == n
    for s in seqs:
        n = min(20, len(s.tokens) - len(prompts[s.key]))
        assert n >= 12 and s.tokens[len(prompts[s.key]):len(prompts[s.key]) + n] == refs[s.key][:n]
