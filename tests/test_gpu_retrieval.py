"""GPU parity: laser_pool_build + laser_retrieve_drafts vs oracle.retrieval, bit-exact
(drafts, draft_len, match_n, pool_index), through the C ABI."""
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


def _compare(toks, off, keys, q_keys, tails, n_min, n_max, K, mt=1, build_n_max=None):
    laser = _laser()
    pool = laser.Pool(toks, off, keys, build_n_max or n_max)
    ora = RegroupedPool(toks, off, keys)
    info = pool.info()
    assert info["n_tokens"] == ora.P.size and info["n_keys"] == len(ora.key_range)
    if ora.P.size:
        assert (pool.read_tokens(0, ora.P.size) == ora.P).all()
    tails = np.asarray(tails, dtype=np.int32).reshape(len(q_keys), n_max)
    g = laser.retrieve_drafts(pool, torch.tensor(np.asarray(q_keys, dtype=np.int64), device="cuda"),
                              torch.tensor(tails, device="cuda"), n_min, n_max, K, mt)
    torch.cuda.synchronize()
    d, dl, mn, pi = (t.cpu().numpy() for t in g)
    od, odl, omn, opi = retrieve(ora, q_keys, tails, n_min, n_max, K, mt)
    assert (dl == odl).all(), (dl, odl)
    assert (mn == omn).all()
    assert (pi == opi).all()
    assert (d == od).all()
    pool.close()
    return d, dl, mn, pi


def test_hand_worked_pools():
    toks, off, keys = _flat([[1, 2, 3, 4], [1, 2, 3, 5], [9, 2, 3, 5]], [7, 7, 7])
    d, dl, mn, pi = _compare(toks, off, keys, [7, 7, 7, 8, 7], [[8, 2, 3], [1, 2, 3], [0, 9, 2], [1, 2, 3], [2, 3, 4]],
                             1, 3, 4)
    assert dl.tolist() == [1, 1, 2, 0, 0] and pi.tolist() == [6, 2, 9, -1, -1]


@pytest.mark.parametrize("seed", range(3))
def test_random_small_pools(seed):
    r = np.random.default_rng(100 + seed)
    for trial in range(25):
        vocab = int(r.integers(2, 9))
        n_keys = int(r.integers(1, 5))
        n_seq = int(r.integers(1, 30))
        seqs = [r.integers(0, vocab, size=int(r.integers(1, 40))).tolist() for _ in range(n_seq)]
        keys = (r.integers(0, n_keys, size=n_seq) * 1000003 - 17).tolist()
        n_max = int(r.integers(1, 5))
        n_min = int(r.integers(1, n_max + 1))
        K = int(r.integers(0, 9))
        mt = int(r.integers(1, 4))
        B = 33
        qk = (r.integers(0, n_keys + 1, size=B) * 1000003 - 17).tolist()
        tails = r.integers(0, vocab, size=(B, n_max))
        pad = r.integers(0, n_max + 1, size=B)
        for b in range(B):
            tails[b, :pad[b]] = -1 if r.random() < 0.3 else tails[b, :pad[b]]
        _compare(*_flat(seqs, keys), qk, tails, n_min, n_max, K, mt, build_n_max=min(8, n_max + int(r.integers(0, 3))))


def test_edge_cases():
    laser = _laser()
    # empty pool, empty batch, K = 0
    toks, off, keys = np.zeros(0, np.int32), np.zeros(1, np.int64), np.zeros(0, np.int64)
    _compare(toks, off, keys, [1, 2], [[1, 2], [3, 4]], 1, 2, 3)
    toks, off, keys = _flat([[1, 2, 3]], [0])
    _compare(toks, off, keys, [], np.zeros((0, 2), np.int32), 1, 2, 3)
    _compare(toks, off, keys, [0], [[1, 2]], 1, 2, 0)
    # sequences of length 1 have no successor anywhere
    _compare(*_flat([[4], [4], [4]], [0, 0, 0]), [0], [[4]], 1, 1, 2)
    # argument errors come back as codes, not crashes
    pool = laser.Pool(toks, off, keys, 2)
    k = torch.zeros(1, dtype=torch.int64, device="cuda")
    with pytest.raises(laser.LaserError):
        laser.retrieve_drafts(pool, k, torch.zeros((1, 3), dtype=torch.int32, device="cuda"), 1, 3, 2)   # n_max > pool's
    with pytest.raises(laser.LaserError):
        laser.retrieve_drafts(pool, k, torch.zeros((1, 2), dtype=torch.int32, device="cuda"), 0, 2, 2)   # n_min < 1
    with pytest.raises(laser.LaserError):
        laser.retrieve_drafts(pool, k, torch.zeros((1, 2), dtype=torch.int32, device="cuda"), 1, 2, 64)  # K too large
    with pytest.raises(laser.LaserError):
        laser.Pool(toks, off, keys, 9)
    with pytest.raises(laser.LaserError):
        laser.Pool(np.array([1, -2, 3], np.int32), off, keys, 2)


def test_many_occurrences_streamed_and_vote_table_overflow():
    # (a) constant pool: 5000 occurrences of every n-gram (> the 2048 a wave keeps in LDS), K = 63
    _compare(*_flat([[3] * 5001, [3] * 40], [1, 1]), [1], [[3, 3, 3]], 1, 3, 63)
    # (b) token 7 followed by 3000 distinct successors, one of them twice (must win), then a tie
    #     between several successors where the smallest id must win
    seqs = []
    for t in range(3000):
        seqs.append([7, 100 + t, 5, 6])
    seqs.append([7, 2999 + 100, 5, 9])
    seqs += [[8, 50 + t] for t in range(1500)]           # all successors of 8 tie at 1: smallest id wins
    toks, off, keys = _flat(seqs, [0] * len(seqs))
    d, dl, mn, pi = _compare(toks, off, keys, [0, 0], [[1, 7], [1, 8]], 1, 2, 3)
    assert d[0].tolist() == [3099, 5, 6] and d[1].tolist() == [50, -1, -1]
    # (c) more than 2048 survivors after the first vote, narrowing later
    seqs = [[1, 2, 3, 4, int(t % 7)] for t in range(4000)] + [[1, 2, 9, 9, 9]] * 100
    _compare(*_flat(seqs, [0] * len(seqs)), [0], [[0, 1]], 1, 2, 6)


@pytest.mark.parametrize("name,B,ctx_len,n_min,n_max,K", [
    ("tiny", 64, 64, 1, 3, 4),
    ("1b", 128, 512, 1, 3, 8),
    ("7b_latency", 64, 1024, 1, 3, 8),
    ("7b_throughput", 256, 512, 1, 3, 10),
])
def test_benchmark_pools(name, B, ctx_len, n_min, n_max, K):
    spec = synth.POOLS[name]
    pool = synth.gen_pool(spec)
    ctx = synth.gen_contexts(spec, B, ctx_len, n_max, salt=3, min_remaining=K)
    d, dl, mn, pi = _compare(pool["tokens"], pool["seq_off"], pool["seq_key"], ctx["keys"],
                             ctx["ctx"][:, -n_max:], n_min, n_max, K)
    assert (dl > 0).mean() > 0.5          # the recipe gives contexts whose continuation is in the pool


def test_stress_shape_sampled():
    # the stress recipe (lognormal sub-pools, one key per sequence, K = 16, n up to 4) at 1/50 scale
    spec = synth.POOLS["stress"].with_(n_seq=20000, n_keys=20000)
    pool = synth.gen_pool(spec)
    ctx = synth.gen_contexts(spec, 4096, 8, 4, salt=5)
    # contexts must use keys that exist in this scaled pool: draw ranks below n_seq
    _compare(pool["tokens"], pool["seq_off"], pool["seq_key"], ctx["keys"], ctx["ctx"][:, -4:], 1, 4, 16)
