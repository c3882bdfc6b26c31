"""GPU parity of the token-tree path (Sec. 3.3 tree-based drafting + tree attention, Sec. 3.4 longest verified
branch) through the C ABI: laser_retrieve_tree bit-exact against the oracle's best-first sub-tree, laser_verify_tree
logits / accepted branch against the oracle's tree attention and tree acceptance, laser_kv_commit_tree by the logits
of the steps that follow (they read the compacted keys/values)."""
import numpy as np
import pytest
import torch

import synth
from oracle import retrieval, step
from oracle.decoder import Decoder
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _laser():
    import paper_2408_05676_amd as laser
    return laser


def _check_trees(pool_np, ctxs, keys, n_min, n_max, K, min_tokens=1):
    laser = _laser()
    toks, off, skey = pool_np
    pool = laser.Pool(toks, off, skey, n_max)
    opool = retrieval.RegroupedPool(toks, off, skey)
    tails = np.full((len(ctxs), n_max), -1, dtype=np.int32)
    for b, c in enumerate(ctxs):
        c = list(c)[-n_max:]
        if c:
            tails[b, n_max - len(c):] = c
    tk, pa, fr, tl, mn = laser.retrieve_tree(pool, torch.tensor(np.asarray(keys, dtype=np.int64), device="cuda"),
                                             torch.tensor(tails, device="cuda"), n_min, n_max, K, min_tokens)
    torch.cuda.synchronize()
    tk, pa, fr, tl, mn = (t.cpu().numpy() for t in (tk, pa, fr, tl, mn))
    for b in range(len(ctxs)):
        t, par, f, n = retrieval.retrieve_tree_one(opool, keys[b], tails[b], n_min, n_max, K, min_tokens)
        assert tl[b] == len(t) and mn[b] == n, (b, tl[b], len(t), mn[b], n)
        assert tk[b, :tl[b]].tolist() == t and pa[b, :tl[b]].tolist() == par and fr[b, :tl[b]].tolist() == f, (b, ctxs[b])
        assert (tk[b, tl[b]:] == -1).all() and (pa[b, tl[b]:] == -1).all()
    pool.close()
    return tl


def test_retrieve_tree_hand_worked_and_random_pools():
    seqs = [[1, 2, 3, 4, 5], [2, 3, 4, 6], [9, 2, 3, 7], [2, 3, 4, 5, 8]]
    flat = np.array([t for s in seqs for t in s], dtype=np.int32)
    off = np.cumsum([0] + [len(s) for s in seqs]).astype(np.int64)
    pool = (flat, off, np.full(4, 7, dtype=np.int64))
    for K in (1, 3, 5, 8):
        _check_trees(pool, [[2, 3], [9, 2, 3], [5, 5], [6, 6], [3]], [7, 7, 7, 7, 8], 1, 3, K)
    _check_trees(pool, [[9, 2, 3]], [7], 1, 3, 3, min_tokens=2)
    r = np.random.default_rng(3)
    for trial in range(12):
        vocab = int(r.integers(2, 9))
        n_seq = int(r.integers(1, 40))
        seqs = [r.integers(0, vocab, size=int(r.integers(1, 30))) for _ in range(n_seq)]
        keys = r.integers(0, 3, size=n_seq).astype(np.int64)
        flat = np.concatenate(seqs).astype(np.int32)
        off = np.cumsum([0] + [len(s) for s in seqs]).astype(np.int64)
        n_max = int(r.integers(1, 5))
        ctxs = [r.integers(0, vocab, size=int(r.integers(0, 6))).tolist() for _ in range(24)]
        ck = r.integers(0, 4, size=24).tolist()
        _check_trees((flat, off, keys), ctxs, ck, int(r.integers(1, n_max + 1)), n_max, int(r.integers(1, 33)), int(r.integers(1, 4)))


def test_retrieve_tree_many_occurrences_and_benchmark_pool():
    # one key, a tiny vocabulary: thousands of occurrences of every suffix (beyond what a wave keeps in LDS), wide votes
    r = np.random.default_rng(4)
    seqs = [r.integers(0, 3, size=400) for _ in range(30)]
    flat = np.concatenate(seqs).astype(np.int32)
    off = np.cumsum([0] + [len(s) for s in seqs]).astype(np.int64)
    _check_trees((flat, off, np.zeros(30, dtype=np.int64)), [[0], [1, 2], [2, 2, 1], [0, 1, 2]], [0] * 4, 1, 3, 32)
    # many distinct successors of one token (the vote table overflows and is partitioned)
    big = np.concatenate([np.stack([np.full(3000, 5), np.arange(3000) % 2500 + 10, np.arange(3000) % 7 + 3000], axis=1).ravel(),
                          np.array([5, 11, 3001, 5, 11, 3001])]).astype(np.int32)
    n3 = 3000
    off = np.concatenate([np.arange(0, 3 * n3 + 1, 3), [3 * n3 + 6]]).astype(np.int64)
    _check_trees((big, off, np.zeros(n3 + 1, dtype=np.int64)), [[5], [5, 11]], [0, 0], 1, 2, 12)
    # the tiny benchmark pool with its own contexts
    spec = synth.POOLS["tiny"]
    pd = synth.gen_pool(spec)
    ctx = synth.gen_contexts(spec, 16, 64, 3, salt=3, min_remaining=4)
    tl = _check_trees((pd["tokens"], pd["seq_off"], pd["seq_key"]), [c for c in ctx["ctx"]], ctx["keys"].tolist(), 1, 3, 8)
    assert tl.max() == 8


_ORACLES = {}


def _oracle(sh):
    key = (sh.name, sh.n_layers, sh.lm_gain)
    if key not in _ORACLES:
        _ORACLES.clear()
        _ORACLES[key] = Decoder(sh.n_layers, sh.d, sh.n_heads, sh.ffn, sh.vocab, synth.gen_all_weights(sh), sh.eps, sh.rope_base)
    return _ORACLES[key]


def _random_tree(r, K, n_nodes):
    par = np.full(K, -1, dtype=np.int32)
    for i in range(1, n_nodes):
        par[i] = int(r.integers(-1, i))
    return par


def _run_tree_steps(sh, B, ctx_len, K, n_steps, k, p, mode=0, seed=1, chainlike=False, fused=None):
    """n_steps tree-verify + tree-commit steps on the GPU against the oracle; the trees are random shapes whose
    tokens mix the oracle's own greedy continuation (so that branches get accepted, also second branches) with
    random tokens; ragged node counts. Later steps read what laser_kv_commit_tree moved."""
    laser = _laser()
    dec = _oracle(sh)
    cap = ctx_len + (K + 1) * (n_steps + 1) + 16
    model = gu.make_model(sh, max_rows=B * max(K + 1, 16), max_batch=B, max_pos=cap + 16)
    if fused is not None:                # 1: the persistent few-row kernel where it applies (at most 16 rows), 0: never
        model.set_option("fused", fused)
    kv = gu.make_kv(sh, n_pages=B * (cap // 16 + 2), max_seqs=B + 1, max_pages_per_seq=cap // 16 + 2)
    seq_ids = [B - b for b in range(B)]
    prompts = synth.uniform_tokens(seed, 60, 0, B * ctx_len, sh.vocab).reshape(B, ctx_len)
    for s in seq_ids:
        kv.reserve(s, cap)
    pend = gu.prefill(model, kv, seq_ids, prompts)
    seqs = [step.Sequence(dec, 0, prompts[b], cap) for b in range(B)]
    r = np.random.default_rng(seed)
    worst, flips_total, acc_sum, second_branch = 0.0, 0, 0, 0
    for it in range(n_steps):
        tokens = r.integers(0, sh.vocab, size=(B, K)).astype(np.int32)
        parents = np.full((B, K), -1, dtype=np.int32)
        nn = np.zeros(B, dtype=np.int32)
        for b in range(B):
            nn[b] = K if (b + it) % 4 else int(r.integers(0, K + 1))
            parents[b] = np.arange(-1, K - 1) if chainlike else _random_tree(r, K, int(nn[b]))
            if nn[b] and (b + it) % 3 != 2:
                probe = step.Sequence.__new__(step.Sequence)
                probe.key, probe.tokens = 0, list(seqs[b].tokens)
                probe.cache = dec.new_cache(cap)
                probe.cache.k[:], probe.cache.v[:] = seqs[b].cache.k, seqs[b].cache.v
                probe.cache.length = seqs[b].cache.length
                good = step.autoregressive_greedy(dec, probe, K)
                # walk a random root-to-leaf path and put the model's own continuation on its first nodes
                depth = np.zeros(K, dtype=np.int64)
                for i in range(int(nn[b])):
                    depth[i] = 1 if parents[b, i] < 0 else depth[parents[b, i]] + 1
                leaf = int(r.integers(0, nn[b]))
                n_good = int(r.integers(0, depth[leaf] + 1))
                i = leaf
                while i >= 0:
                    if depth[i] <= n_good:
                        tokens[b, i] = good[depth[i] - 1]
                    i = int(parents[b, i])
            tokens[b, nn[b]:] = -1
            parents[b, nn[b]:] = -1
        tk, pa, tl = (torch.tensor(x, device="cuda") for x in (tokens, parents, nn))
        acc, out, path, logits = laser.verify_tree(model, kv, seq_ids, pend, tk, pa, tl, k, p, mode, want_logits=True)
        laser.kv_commit_tree(kv, seq_ids, acc, path)
        torch.cuda.synchronize()
        ora = step.verify_tree_step(dec, seqs, tokens, parents, nn, k, p, mode, return_logits=True)
        ok, max_err, ratio = gu.logits_close(logits.cpu().numpy().astype(np.float64), ora["logits"])
        worst = max(worst, ratio)
        assert ok, f"step {it}: logits off: max abs err {max_err}, {ratio:.2f}x the bound"
        acc_g, out_g, path_g = acc.cpu().numpy(), out.cpu().numpy(), path.cpu().numpy()
        diverged = False
        for b in range(B):
            a = int(acc_g[b])
            # well-formed: the path is a branch of the tree and the emitted tokens are its tokens
            assert 0 <= a <= nn[b] and (path_g[b, a:] == -1).all() and (out_g[b, a + 1:] == -1).all()
            assert all(parents[b, path_g[b, j]] == (path_g[b, j - 1] if j else -1) for j in range(a))
            assert out_g[b, :a].tolist() == [int(tokens[b, i]) for i in path_g[b, :a]] and 0 <= out_g[b, a] < sh.vocab
            same = (a == int(ora["accept_len"][b]) and path_g[b].tolist() == ora["accept_path"][b].tolist()
                    and out_g[b].tolist() == ora["out_tokens"][b].tolist())
            if not same:
                st = ora["stats"][b]
                margins = [min(s["rank_margin"], s["logq_margin"] / 2.0) for s in st.values()] + [float(ora["argmax_gap"][b])]
                tol = 3.0 * (gu.ATOL + gu.RTOL * float(np.abs(ora["logits"][b]).max()))
                assert min(margins) <= tol, f"step {it} sequence {b}: branch differs outside tolerance: {path_g[b].tolist()} vs {ora['accept_path'][b].tolist()}"
                flips_total += 1
                diverged = True
            acc_sum += a
            second_branch += int(a > 0 and path_g[b, a - 1] != a - 1)
        if diverged:
            break
        pend = torch.tensor([s.pending for s in seqs], dtype=torch.int32, device="cuda")
        assert kv.read_lens(seq_ids).tolist() == [s.cache.length for s in seqs]
    print(f"[tree {sh.name} B={B} ctx={ctx_len} K={K} k={k} p={p} mode={mode}] worst logit error {worst:.3f} of bound, "
          f"accepted nodes {acc_sum}, branches that needed compaction {second_branch}, in-tolerance flips {flips_total}")
    model.close(); kv.close()
    return acc_sum, second_branch


@pytest.mark.parametrize("shape_name", ["tiny", "tiny128"])
def test_verify_tree_against_the_oracle(shape_name):
    sh = synth.SHAPES[shape_name].with_(lm_gain=4.0)
    a, c = _run_tree_steps(sh, B=3, ctx_len=41, K=7, n_steps=5, k=1, p=-1.0, seed=3)           # 24 rows
    assert a > 0 and c > 0          # later steps did read compacted keys/values
    _run_tree_steps(sh, B=2, ctx_len=300, K=6, n_steps=3, k=2, p=0.005, seed=4, fused=0)         # few rows, split context
    _run_tree_steps(sh, B=14, ctx_len=21, K=9, n_steps=2, k=3, p=0.02, mode=1, seed=5)          # 140 rows: tiled GEMMs + tiled head
    _run_tree_steps(sh, B=2, ctx_len=20, K=31, n_steps=2, k=2, p=0.005, seed=6)                  # 32 rows per sequence: two query tiles


def test_verify_tree_persistent_kernel():
    """Token trees of at most 16 rows on the persistent few-row kernel (ancestor mask in its attention phase, depth
    positions, the nodes' logits picked from their parents' rows, tree walk in its acceptance phase)."""
    sh = synth.SHAPES["tiny128"].with_(lm_gain=4.0)
    a, c = _run_tree_steps(sh, B=1, ctx_len=41, K=8, n_steps=6, k=1, p=-1.0, seed=3, fused=1)
    assert a > 0
    a2, c2 = _run_tree_steps(sh, B=2, ctx_len=300, K=7, n_steps=4, k=2, p=0.005, seed=4, fused=1)    # 16 rows, split context
    assert a2 > 0 and c + c2 > 0    # a later step did read compacted keys/values
    a3, c3 = _run_tree_steps(sh, B=1, ctx_len=20, K=15, n_steps=3, k=3, p=0.02, mode=1, seed=7, fused=1)   # the largest tree it takes
    assert a3 > 0 and c3 > 0
    _run_tree_steps(sh, B=3, ctx_len=33, K=4, n_steps=3, k=2, p=0.005, mode=3, seed=6, fused=1)      # three sequences
    sh7 = synth.SHAPES["7b"].with_(n_layers=2)
    a7, c7 = _run_tree_steps(sh7, B=1, ctx_len=150, K=8, n_steps=3, k=2, p=0.0, seed=9, fused=1)
    assert a7 > 0 and c7 > 0


def test_verify_tree_7b_width():
    sh = synth.SHAPES["7b"].with_(n_layers=2)
    _run_tree_steps(sh, B=2, ctx_len=150, K=8, n_steps=2, k=2, p=0.0, seed=7)


@pytest.mark.parametrize("fused", [0, 1])
def test_a_chain_given_as_a_tree_is_bit_identical_to_the_chain_call(fused):
    laser = _laser()
    sh = synth.SHAPES["tiny128"].with_(lm_gain=4.0)
    B, K, ctx_len = (2, 6, 37) if fused else (3, 6, 37)        # 14 rows fit the persistent kernel
    prompts = synth.uniform_tokens(9, 60, 0, B * ctx_len, sh.vocab).reshape(B, ctx_len)
    drafts = torch.tensor(synth.uniform_tokens(9, 61, 0, B * K, sh.vocab).reshape(B, K).astype(np.int32), device="cuda")
    dl = torch.tensor([6, 3, 0][:B], dtype=torch.int32, device="cuda")
    res = []
    for tree in (False, True):
        model = gu.make_model(sh, max_rows=B * 16, max_batch=B, max_pos=128)
        model.set_option("fused", fused)
        kv = gu.make_kv(sh, n_pages=B * 8, max_seqs=B, max_pages_per_seq=8)
        ids = list(range(B))
        for s in ids:
            kv.reserve(s, 96)
        pend = gu.prefill(model, kv, ids, prompts)
        if tree:
            par = torch.tensor(np.tile(np.arange(-1, K - 1, dtype=np.int32), (B, 1)), device="cuda")
            acc, out, path, lg = laser.verify_tree(model, kv, ids, pend, drafts, par, dl, 2, 0.05, 0, want_logits=True)
            assert all(path.cpu().numpy()[b, :a].tolist() == list(range(a)) for b, a in enumerate(acc.cpu().tolist()))
        else:
            acc, out, lg = laser.verify_step(model, kv, ids, pend, drafts, dl, 2, 0.05, 0, want_logits=True)
        torch.cuda.synchronize()
        res.append((acc.cpu().numpy(), out.cpu().numpy(), lg.cpu().numpy()))
        model.close(); kv.close()
    assert (res[0][0] == res[1][0]).all() and (res[0][1] == res[1][1]).all()
    assert np.array_equal(res[0][2], res[1][2])                       # bit for bit


def test_tree_loop_against_the_oracle_and_accepted_length_gain():
    """Whole steps retrieve_tree -> verify_tree -> commit_tree -> ctx_advance on the tiny model with a pool that holds
    noisy copies of the model's own continuation, against the oracle's laser_tree_step; and the accepted length per
    step of trees (8 and 16 nodes) against chains of 8 tokens on the same workload."""
    laser = _laser()
    sh = synth.SHAPES["tiny"].with_(lm_gain=4.0)
    dec = _oracle(sh)
    B, n_max, ctx_len, n_steps = 4, 3, 24, 8
    prompts = synth.uniform_tokens(21, 60, 0, B * ctx_len, sh.vocab).reshape(B, ctx_len)
    conts = [step.autoregressive_greedy(dec, step.Sequence(dec, b, prompts[b], 256), 90) for b in range(B)]
    r = np.random.default_rng(1)
    seqs_tok, keys = [], []
    for b in range(B):
        text = np.array(list(prompts[b, -n_max:]) + conts[b], dtype=np.int32)
        for _ in range(4):                                     # four noisy copies: branches that differ where they were hit
            noisy = text.copy()
            hit = r.random(noisy.size) < 0.12
            hit[:n_max] = False
            noisy[hit] = r.integers(0, sh.vocab, size=int(hit.sum()))
            seqs_tok.append(noisy); keys.append(b)
    flat = np.concatenate(seqs_tok).astype(np.int32)
    off = np.cumsum([0] + [len(s) for s in seqs_tok]).astype(np.int64)
    skey = np.array(keys, dtype=np.int64)
    opool = retrieval.RegroupedPool(flat, off, skey)
    accepted = {}
    for mode_name, K in (("tree", 8), ("chain", 8), ("tree", 16)):
        pool = laser.Pool(flat, off, skey, n_max)
        cap = ctx_len + (K + 1) * (n_steps + 1) + 16
        model = gu.make_model(sh, max_rows=B * 32, max_batch=B, max_pos=cap + 16)
        model.set_option("fused", 0)
        kv = gu.make_kv(sh, n_pages=B * (cap // 16 + 2), max_seqs=B, max_pages_per_seq=cap // 16 + 2)
        ids = list(range(B))
        for s in ids:
            kv.reserve(s, cap)
        pend = gu.prefill(model, kv, ids, prompts)
        tail = torch.tensor(prompts[:, -n_max:].astype(np.int32), device="cuda")
        kd = torch.arange(B, dtype=torch.int64, device="cuda")
        seqs = [step.Sequence(dec, b, prompts[b], cap) for b in range(B)]
        total = 0
        for it in range(n_steps):
            if mode_name == "tree":
                tk, pa, fr, tl, mn = laser.retrieve_tree(pool, kd, tail, 1, n_max, K)
                acc, out, path, _ = laser.verify_tree(model, kv, ids, pend, tk, pa, tl, 1, -1.0, 0)
                laser.kv_commit_tree(kv, ids, acc, path)
                ora = step.laser_tree_step(dec, opool, seqs, 1, n_max, K, 1, -1.0, 0)
                assert (tk.cpu().numpy() == ora["tree_tokens"]).all() and (pa.cpu().numpy() == ora["tree_parent"]).all()
                assert (tl.cpu().numpy() == ora["tree_len"]).all()
            else:
                dr, dl, mn, pi = laser.retrieve_drafts(pool, kd, tail, 1, n_max, K)
                acc, out, _ = laser.verify_step(model, kv, ids, pend, dr, dl, 1, -1.0, 0)
                laser.kv_commit(kv, ids, acc)
                ora = step.laser_step(dec, opool, seqs, 1, n_max, K, 1, -1.0, 0)
                assert (dr.cpu().numpy() == ora["drafts"]).all()
            laser.ctx_advance(tail, pend, out, acc)
            torch.cuda.synchronize()
            if not ((acc.cpu().numpy() == ora["accept_len"]).all() and (out.cpu().numpy() == ora["out_tokens"]).all()):
                print(f"[{mode_name} loop] step {it}: a decision inside the tolerance differs; comparison stops here")
                break
            assert kv.read_lens(ids).tolist() == [s.cache.length for s in seqs]
            total += int(acc.sum())
        accepted[(mode_name, K)] = total / (B * (it + 1))
        model.close(); kv.close(); pool.close()
    print(f"[tree loop] accepted drafts per step and sequence: chain of 8 tokens {accepted[('chain', 8)]:.2f}, tree of 8 nodes "
          f"{accepted[('tree', 8)]:.2f}, tree of 16 nodes {accepted[('tree', 16)]:.2f}")
    assert accepted[("tree", 16)] >= accepted[("chain", 8)] > 0


def test_tree_and_generate_edge_cases():
    """Empty batches and trees, the largest tree, malformed parent entries, a one-token generation and an
    end-of-sequence token that comes first."""
    laser = _laser()
    sh = synth.SHAPES["tiny128"].with_(lm_gain=4.0)
    dec = _oracle(sh)
    B, K, ctx_len = 2, laser.binding.MAX_TREE, 19
    cap = ctx_len + 3 * (K + 1) + 16
    model = gu.make_model(sh, max_rows=B * (K + 1), max_batch=B, max_pos=cap + 16)
    kv = gu.make_kv(sh, n_pages=B * (cap // 16 + 2), max_seqs=B, max_pages_per_seq=cap // 16 + 2)
    ids = [0, 1]
    for s in ids:
        kv.reserve(s, cap)
    prompts = synth.uniform_tokens(33, 60, 0, B * ctx_len, sh.vocab).reshape(B, ctx_len)
    pend = gu.prefill(model, kv, ids, prompts)
    seqs = [step.Sequence(dec, 0, prompts[b], cap) for b in range(B)]
    # B = 0 and K = 0 calls are no-ops / plain one-token steps
    e = torch.empty((0, 4), dtype=torch.int32, device="cuda")
    e1 = torch.empty(0, dtype=torch.int32, device="cuda")
    laser.verify_tree(model, kv, [], e1, e, e, e1, 1, 0.0)
    laser.kv_commit_tree(kv, [], e1, e)
    # the largest tree (32 nodes): a wide root, a deep branch, and entries that do not name an earlier node (they hang off the root)
    r = np.random.default_rng(8)
    good = step.autoregressive_greedy(dec, _clone(dec, seqs[0], cap), 6)
    tokens = r.integers(0, sh.vocab, size=(B, K)).astype(np.int32)
    parents = np.full((B, K), -1, dtype=np.int32)
    parents[0, 16:] = np.arange(15, K - 1)                    # nodes 16..31: a chain below node 15 ...
    tokens[0, 15] = good[0]
    tokens[0, 16:21] = good[1:6]                              # ... that carries the model's own continuation
    parents[1, 1:] = [int(r.integers(-1, i)) for i in range(1, K)]
    bad = parents.copy()
    bad[1, 5], bad[1, 9] = 7, -4                              # not earlier nodes: read as -1
    parents[1, 5], parents[1, 9] = -1, -1
    nn = np.array([K, K], dtype=np.int32)
    acc, out, path, logits = laser.verify_tree(model, kv, ids, pend, torch.tensor(tokens, device="cuda"), torch.tensor(bad, device="cuda"),
                                               torch.tensor(nn, device="cuda"), 1, -1.0, 0, want_logits=True)
    laser.kv_commit_tree(kv, ids, acc, path)
    torch.cuda.synchronize()
    ora = step.verify_tree_step(dec, seqs, tokens, parents, nn, 1, -1.0, 0, return_logits=True)
    ok, max_err, ratio = gu.logits_close(logits.cpu().numpy().astype(np.float64), ora["logits"])
    assert ok, (max_err, ratio)
    assert acc.cpu().tolist() == ora["accept_len"].tolist() and acc.cpu().tolist()[0] == 6
    assert path.cpu().numpy().tolist() == ora["accept_path"].tolist() and out.cpu().numpy().tolist() == ora["out_tokens"].tolist()
    assert kv.read_lens(ids).tolist() == [s.cache.length for s in seqs]
    # an empty tree is a plain one-token step
    pend = torch.tensor([s.pending for s in seqs], dtype=torch.int32, device="cuda")
    zero = torch.zeros(B, dtype=torch.int32, device="cuda")
    acc, out, path, _ = laser.verify_tree(model, kv, ids, pend, torch.tensor(tokens, device="cuda"), torch.tensor(parents, device="cuda"), zero, 2, 0.1, 0)
    laser.kv_commit_tree(kv, ids, acc, path)
    ora = step.verify_tree_step(dec, seqs, tokens, parents, [0, 0], 2, 0.1, 0)
    assert acc.cpu().tolist() == [0, 0] and out.cpu().numpy()[:, 0].tolist() == ora["out_tokens"][:, 0].tolist() and (out.cpu().numpy()[:, 1:] == -1).all()
    # generation: one token; an end-of-sequence token that is the very first one; a look at the counter every step
    pend = torch.tensor([s.pending for s in seqs], dtype=torch.int32, device="cuda")
    tail = torch.tensor(np.stack([np.array(s.tokens[-3:], dtype=np.int32) for s in seqs]), device="cuda")
    first = [int(np.argmax(dec.verify_forward(_clone(dec, s, cap).cache, [s.pending])[0])) for s in seqs]
    gen, glen, cnt, steps, _ = laser.generate(model, kv, None, ids, None, tail, pend, 0, 1, 1, -1.0, 0, max_new_tokens=5, eos_token=first[0], check_every=1)
    assert glen.cpu().tolist()[0] == 1 and gen.cpu().numpy()[0].tolist() == [first[0], -1, -1, -1, -1]
    assert glen.cpu().tolist()[1] == (1 if first[1] == first[0] else 5) and steps == glen.max().item()
    with pytest.raises(laser.LaserError):
        laser.retrieve_tree(laser.Pool(np.zeros(4, dtype=np.int32), np.array([0, 4]), np.array([1]), 2), torch.zeros(1, dtype=torch.int64, device="cuda"),
                            torch.zeros((1, 2), dtype=torch.int32, device="cuda"), 1, 2, K + 1)      # more nodes than LASER_MAX_TREE
    model.close(); kv.close()


def _clone(dec, s, cap):
    c = step.Sequence.__new__(step.Sequence)
    c.key, c.tokens = s.key, list(s.tokens)
    c.cache = dec.new_cache(cap)
    c.cache.k[:], c.cache.v[:] = s.cache.k, s.cache.v
    c.cache.length = s.cache.length
    return c
