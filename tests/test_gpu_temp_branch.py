"""GPU parity for the temporary branch (Sec. 3.2: prompt + generated text join the key's trie while a text is
being generated): laser_retrieve_drafts_temp against oracle.retrieval with `own`, bit-exact (drafts, draft_len,
match_n, pool_index), and laser_own_text_append against its definition (append, sliding window)."""
import numpy as np
import pytest
import torch

import synth
from oracle.retrieval import RegroupedPool, retrieve

pytestmark = pytest.mark.gpu


def _laser():
    import paper_2408_05676_amd as laser
    return laser


def _flat(seqs, keys):
    toks = np.array([t for s in seqs for t in s], dtype=np.int32)
    off = np.cumsum([0] + [len(s) for s in seqs]).astype(np.int64)
    return toks, off, np.array(keys, dtype=np.int64)


def _compare(toks, off, keys, q_keys, owns, n_min, n_max, K, mt=1, cap=None, tails=None):
    """owns: one token list per query; the context tail is the own text's tail unless `tails` is given."""
    laser = _laser()
    pool = laser.Pool(toks, off, keys, n_max)
    ora = RegroupedPool(toks, off, keys)
    B = len(q_keys)
    cap = cap or max(1, max(len(o) for o in owns))
    own_t = np.full((B, cap), -7, dtype=np.int32)                  # garbage beyond own_len must never be read as text
    own_len = np.zeros(B, dtype=np.int32)
    for b, o in enumerate(owns):
        own_t[b, :len(o)] = o
        own_len[b] = len(o)
    if tails is None:
        tails = [([-1] * n_max + list(o))[-n_max:] for o in owns]
    tails = np.asarray(tails, dtype=np.int32).reshape(B, n_max)
    g = laser.retrieve_drafts_temp(pool, torch.tensor(np.asarray(q_keys, dtype=np.int64), device="cuda"),
                                   torch.tensor(tails, device="cuda"), torch.tensor(own_t, device="cuda"),
                                   torch.tensor(own_len, device="cuda"), n_min, n_max, K, mt)
    torch.cuda.synchronize()
    d, dl, mn, pi = (t.cpu().numpy() for t in g)
    od, odl, omn, opi = retrieve(ora, q_keys, tails, n_min, n_max, K, mt, own=[list(o) for o in owns])
    assert (dl == odl).all(), (dl, odl)
    assert (mn == omn).all(), (mn, omn)
    assert (pi == opi).all(), (pi, opi)
    assert (d == od).all()
    pool.close()
    return d, dl, mn, pi


def test_hand_worked_temporary_branches():
    toks, off, keys = _flat([[1, 2, 3, 4]], [7])
    owns = [[7, 2, 3, 9, 5, 2, 3], [2, 3, 9, 8, 2, 3, 9, 6, 2, 3], [8, 8, 5, 2, 3], [5, 6, 7, 5, 6], [4]]
    d, dl, mn, pi = _compare(toks, off, keys, [7, 7, 7, 99, 7], owns, 1, 2, 3)
    assert d.tolist() == [[4, -1, -1], [9, 6, 2], [4, -1, -1], [7, 5, 6], [-1, -1, -1]]
    assert pi.tolist() == [2, -7, 2, -3, -1] and mn.tolist() == [2, 2, 2, 2, 0]


@pytest.mark.parametrize("seed", range(3))
def test_random_small_pools_with_own_text(seed):
    r = np.random.default_rng(300 + seed)
    for trial in range(25):
        vocab = int(r.integers(2, 8))
        n_keys = int(r.integers(1, 4))
        n_seq = int(r.integers(1, 20))
        seqs = [r.integers(0, vocab, size=int(r.integers(1, 40))).tolist() for _ in range(n_seq)]
        keys = r.integers(0, n_keys, size=n_seq).tolist()
        n_max = int(r.integers(1, 5))
        n_min = int(r.integers(1, n_max + 1))
        K = int(r.integers(1, 12))
        B = 16
        q_keys = r.integers(0, n_keys + 1, size=B).tolist()          # includes an unknown key
        owns = [r.integers(0, vocab, size=int(r.integers(0, 120))).tolist() for _ in range(B)]
        _compare(*_flat(seqs, keys), q_keys, owns, n_min, n_max, K, mt=int(r.integers(1, 4)), cap=int(r.integers(120, 200)))


def test_long_own_text_many_occurrences_and_streamed_pool_run():
    r = np.random.default_rng(7)
    # (a) own text of the maximum length over a two-token alphabet: thousands of own occurrences per n-gram, K = 63
    own = r.integers(0, 2, size=4096).tolist()
    _compare(*_flat([[0, 1, 0, 1, 1]], [1]), [1, 5], [own, own[:4095]], 1, 4, 63, cap=4096)
    # (b) a pool run of 5000 occurrences (streamed, not kept in LDS) voting together with own occurrences that
    #     decide the winner: the pool says 3 -> 3 always; the own text adds 3 -> 4 more often than the pool's count
    own = ([3, 4] * 2048)[:4096]                                          # 2047 occurrences of 3 -> 4 with a successor
    _compare(*_flat([[3] * 1500, [3] * 40], [1, 1]), [1], [own + []], 1, 1, 8, cap=4096, tails=[[3]])
    _compare(*_flat([[3] * 5001, [3] * 40], [1, 1]), [1], [own], 1, 1, 8, cap=4096, tails=[[3]])
    # (c) the benchmark pool: own text = a 1024-token context whose continuation exists in the pool
    spec = synth.POOLS["7b_latency"]
    pool = synth.gen_pool(spec)
    ctx = synth.gen_contexts(spec, 32, 1024, 3, salt=3, min_remaining=8)
    d, dl, mn, pi = _compare(pool["tokens"], pool["seq_off"], pool["seq_key"], ctx["keys"],
                             [c.tolist() for c in ctx["ctx"]], 1, 3, 8, cap=1100)
    assert (dl > 0).mean() > 0.5


def test_own_text_append_and_sliding_window():
    laser = _laser()
    r = np.random.default_rng(11)
    B, K, cap = 6, 5, 40
    own = np.full((B, cap), -7, dtype=np.int32)
    lens = np.array([0, 3, 36, 38, 40, 40], dtype=np.int32)
    want = []
    for b in range(B):
        own[b, :lens[b]] = r.integers(0, 1000, size=lens[b])
        want.append(own[b, :lens[b]].tolist())
    own_d, len_d = torch.tensor(own, device="cuda"), torch.tensor(lens, device="cuda")
    for step in range(12):
        acc = r.integers(0, K + 1, size=B).astype(np.int32)
        out = r.integers(0, 1000, size=(B, K + 1)).astype(np.int32)
        for b in range(B):
            out[b, acc[b] + 1:] = -1
            want[b] = (want[b] + out[b, :acc[b] + 1].tolist())[-cap:]
        laser.own_text_append(own_d, len_d, torch.tensor(out, device="cuda"), torch.tensor(acc, device="cuda"))
        torch.cuda.synchronize()
        got_len, got = len_d.cpu().numpy(), own_d.cpu().numpy()
        for b in range(B):
            assert got_len[b] == len(want[b]) and got[b, :got_len[b]].tolist() == want[b], (step, b)
    # a cap smaller than one step's tokens keeps the newest; bad arguments are refused
    small, slen = torch.zeros((1, 3), dtype=torch.int32, device="cuda"), torch.zeros(1, dtype=torch.int32, device="cuda")
    laser.own_text_append(small, slen, torch.tensor([[1, 2, 3, 4, 5, 6]], dtype=torch.int32, device="cuda"),
                          torch.tensor([4], dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    assert slen.item() == 3 and small.cpu().numpy().tolist() == [[3, 4, 5]]
    with pytest.raises(laser.LaserError):
        laser.own_text_append(torch.zeros((1, 5000), dtype=torch.int32, device="cuda"), slen,
                              torch.zeros((1, 2), dtype=torch.int32, device="cuda"), slen)
