"""GPU tests at the benchmark's full sizes, in the launch configurations bench.py times.
The float64 oracle cannot run a 32-layer 7B forward inside a test, so the full-size checks are
(a) properties that hold at any size and (b) sampled outputs the oracle computes one by one."""
import numpy as np
import pytest
import torch

import synth
from synth.model import torch_gen_weight

pytestmark = pytest.mark.gpu


def _engine(shape, B, K, ctx_len, extra, fused):
    import paper_2408_05676_amd as laser
    from paper_2408_05676_amd.harness import Engine, stacked_weights
    weights = stacked_weights(lambda n, l: torch_gen_weight(shape, n, l, "cuda"), shape)
    eng = Engine(shape, weights, B, K, ctx_len + extra, 3)
    eng.model.set_option("fused", fused)
    return laser, eng


@pytest.mark.parametrize("fused", [1, 0])
def test_7b_latency_strict_speculation_reproduces_greedy_decoding(fused):
    """Sec. 2.1 / Sec. 4.2: with greedy verification the generated text is identical to
    autoregressive decoding. Checked token for token at the 7B latency shape (32 layers, B = 1,
    context 1024, K = 8) for perfect, partly wrong and useless drafts."""
    sh = synth.SHAPES["7b"]
    B, K, ctx_len, N = 1, 8, 1024, 72
    laser, eng = _engine(sh, B, K, ctx_len, 400, fused)
    ctx = synth.gen_contexts(synth.POOLS["7b_latency"], B, ctx_len, 3, salt=1, min_remaining=K)
    eng.prefill(ctx["ctx"])
    ref = eng.generate_greedy(N)[0]                       # one token per forward
    r = np.random.default_rng(0)
    for kind in ("perfect", "half", "random"):
        eng.kv.set_len(0, ctx_len - 1)
        pend = int(ctx["ctx"][0, -1])
        produced, steps = [], 0
        while len(produced) + K + 1 <= N:
            done = len(produced)
            d = ref[done:done + K].copy()
            if kind == "half":
                d[int(r.integers(1, K)):] = int(r.integers(0, sh.vocab))
            elif kind == "random":
                d = r.integers(0, sh.vocab, size=K).astype(np.int32)
            eng.pending.fill_(pend)
            eng.drafts.copy_(torch.as_tensor(d.astype(np.int32)).reshape(1, K))
            eng.draft_len.fill_(K)
            acc, out, _ = laser.verify_step(eng.model, eng.kv, eng.seq_ids, eng.pending, eng.drafts, eng.draft_len, 1, -1.0, 0)
            laser.kv_commit(eng.kv, eng.seq_ids, acc)
            a = int(acc[0])
            emitted = out[0, :a + 1].cpu().tolist()
            if kind == "perfect":
                assert a == K, (steps, a)
            produced += emitted
            pend = emitted[-1]
            steps += 1
            if steps % 8 == 0:
                eng.kv.read_lens([0])                     # tightens the host's length bound
        assert produced == ref[:len(produced)].tolist(), kind
        assert int(eng.kv.read_lens([0])[0]) == ctx_len - 1 + len(produced)
        print(f"[7b fused={fused}] {kind}: {len(produced)} tokens in {steps} steps, identical to greedy decoding")
    assert not eng.model.aborted()
    eng.close()


def test_7b_throughput_strict_speculation_reproduces_greedy_decoding():
    """The same property at the throughput shape (32 layers, B = 64, prompt 512, K = 10, paged cache):
    M = 704 rows per step on the tiled matrix-core GEMMs. The reference text is decoded with the same
    launch shape (K = 10 rows per sequence, no drafts), so every row goes through identical arithmetic;
    each sequence then gets its own mix of right and wrong drafts."""
    sh = synth.SHAPES["7b"]
    B, K, ctx_len, N = 64, 10, 512, 23
    laser, eng = _engine(sh, B, K, ctx_len, 160, 0)
    ctx = synth.gen_contexts(synth.POOLS["7b_throughput"], B, ctx_len, 3, salt=1, min_remaining=K)
    eng.prefill(ctx["ctx"])
    first = torch.as_tensor(np.ascontiguousarray(ctx["ctx"][:, -1]), dtype=torch.int32).cuda()

    # reference: one token per step and sequence
    eng.pending.copy_(first)
    eng.drafts.fill_(-1)
    eng.draft_len.fill_(0)
    ref = np.empty((B, N), dtype=np.int32)
    for i in range(N):
        acc, out, _ = laser.verify_step(eng.model, eng.kv, eng.seq_ids, eng.pending, eng.drafts, eng.draft_len, 1, -1.0, 0)
        assert int(acc.abs().sum()) == 0
        laser.kv_commit(eng.kv, eng.seq_ids, acc)
        eng.pending.copy_(out[:, 0])
        ref[:, i] = out[:, 0].cpu().numpy()
        eng.kv.read_lens(eng.seq_ids)                    # tightens the host's length bound (it assumes K+1 per step)
    assert eng.kv.read_lens(eng.seq_ids).tolist() == [ctx_len - 1 + N] * B

    # speculation: sequence b's drafts are right up to a cut of its own (K = all right), then wrong
    r = np.random.default_rng(3)
    for b in range(B):
        eng.kv.set_len(b, ctx_len - 1)
    done = np.zeros(B, dtype=np.int64)                      # tokens produced so far per sequence
    produced = [[] for _ in range(B)]
    pend = ctx["ctx"][:, -1].astype(np.int32).copy()
    steps = 0
    while (done + K + 1 <= N).all():
        d = np.stack([ref[b, done[b]:done[b] + K] for b in range(B)]).astype(np.int32)
        cut = r.integers(0, K + 1, size=B)
        cut[::7] = K
        for b in range(B):
            if cut[b] < K:
                d[b, cut[b]] = (d[b, cut[b]] + 1 + int(r.integers(0, sh.vocab - 1))) % sh.vocab    # certainly wrong
                d[b, cut[b] + 1:] = r.integers(0, sh.vocab, size=K - cut[b] - 1)
        eng.pending.copy_(torch.as_tensor(pend))
        eng.drafts.copy_(torch.as_tensor(d))
        eng.draft_len.fill_(K)
        acc, out, _ = laser.verify_step(eng.model, eng.kv, eng.seq_ids, eng.pending, eng.drafts, eng.draft_len, 1, -1.0, 0)
        laser.kv_commit(eng.kv, eng.seq_ids, acc)
        a, o = acc.cpu().numpy(), out.cpu().numpy()
        assert a.tolist() == cut.tolist(), steps           # exactly the right drafts are accepted
        for b in range(B):
            produced[b] += o[b, :a[b] + 1].tolist()
            pend[b] = o[b, a[b]]
        done += a + 1
        steps += 1
        eng.kv.read_lens(eng.seq_ids)
    for b in range(B):
        assert produced[b] == ref[b, :len(produced[b])].tolist(), b
    assert eng.kv.read_lens(eng.seq_ids).tolist() == (ctx_len - 1 + done).tolist()
    print(f"[7b throughput] {int(done.sum())} tokens in {steps} steps of 704 rows, identical to one-token decoding")
    eng.close()


def test_head_stress_shape_sampled_against_the_oracle():
    """Output head + acceptance at the stress shape (d 4096, vocabulary 128256, 256 sequences x 16 rows =
    4096 rows) through laser_verify_head; the oracle recomputes three whole sequences (48 rows) from the
    same weights and hidden states; every sequence's emitted row is checked for form."""
    import paper_2408_05676_amd as laser
    from oracle import acceptance
    from tests import gpu_util as gu
    sh = synth.SHAPES["head128k"]
    B, K = 256, 15
    R = K + 1
    w = torch_gen_weight(sh, "wlm", -1, "cuda").contiguous()
    model = laser.Model(0, sh.d, sh.n_heads, sh.ffn, sh.vocab, {"wlm": w}, B * R, B, 0)
    g = torch.Generator(device="cuda").manual_seed(7)
    # hidden states with a planted direction so that some drafts clear the threshold: h = a * w[t] + noise
    planted = torch.randint(0, sh.vocab, (B, R), generator=g, device="cuda")
    noise = torch.randn((B, R, sh.d), generator=g, device="cuda") * 0.5
    amp = 5.0 + torch.rand((B, R, 1), generator=g, device="cuda") * 9.0
    h = (amp * w[planted].float() + noise).to(torch.float16)    # planted logit ~ 1.64 amp against ~N(0, 0.64^2) others
    drafts = planted[:, :K].to(torch.int32).clone()
    wrong = torch.rand((B, K), generator=g, device="cuda") < 0.12
    drafts[wrong] = torch.randint(0, sh.vocab, (int(wrong.sum()),), generator=g, device="cuda", dtype=torch.int32)
    dl = torch.randint(0, K + 1, (B,), generator=g, device="cuda", dtype=torch.int32)
    dl[::5] = K
    k, p = 2, 0.1
    acc, out, lg = laser.verify_head(model, h, drafts, dl, k, p, 0, want_logits=True)
    torch.cuda.synchronize()
    a, o, d_np, dl_np = acc.cpu().numpy(), out.cpu().numpy(), drafts.cpu().numpy(), dl.cpu().numpy()
    assert (a >= 0).all() and (a <= dl_np).all()
    for b in range(B):
        assert o[b, :a[b]].tolist() == d_np[b, :a[b]].tolist() and 0 <= o[b, a[b]] < sh.vocab and (o[b, a[b] + 1:] == -1).all()
    S = [0, 117, 255]
    w64 = w.float().cpu().numpy().astype(np.float64)
    h64 = h[S].float().cpu().numpy().astype(np.float64)
    logits = h64 @ w64.T                                      # [3][16][V]
    ok, max_err, ratio = gu.logits_close(lg[S].cpu().numpy().astype(np.float64), logits)
    assert ok, (max_err, ratio)
    oa, oo, stats, gaps = acceptance.verify_batch(logits, d_np[S], dl_np[S], k, p, 0)
    ora = {"accept_len": oa, "out_tokens": oo, "stats": stats, "argmax_gap": gaps, "logits": logits}
    flips, bad = gu.classify_step(a[S], o[S], ora, d_np[S], dl_np[S], k, p)
    assert not bad, bad
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        laser.verify_head(model, h, drafts, dl, k, p, 0, out=(acc, out))
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 5
    print(f"[head 128k] {ms:.2f} ms per launch = {2.0 * B * R * sh.d * sh.vocab / ms / 1e9:.0f} TFLOP/s")
    print(f"[head 128k] 4096 rows; sampled sequences: worst logit error {ratio:.3f} of bound, flips {flips}, "
          f"accepted lengths {a[S].tolist()} (oracle {list(map(int, oa))}), mean accepted {a.mean():.2f}")
    model.close()


def test_retrieval_stress_shape_full_size():
    """Draft retrieval at the stress shape: 100 M pool tokens in 1 M keyed sub-pools (lognormal lengths),
    4096 concurrent contexts, suffix length 1..4, K = 16. The regrouped token array and all 4096 results
    are compared with the oracle bit for bit (its lookups only touch the contexts' own sub-pools)."""
    import paper_2408_05676_amd as laser
    from oracle.retrieval import RegroupedPool, retrieve
    spec = synth.POOLS["stress"]
    assert spec.n_seq == 1_000_000
    pool = synth.gen_pool(spec)
    B, n_max, K = 4096, 4, 16
    ctx = synth.gen_contexts(spec, B, 8, n_max, salt=5)
    tails = np.ascontiguousarray(ctx["ctx"][:, -n_max:]).astype(np.int32)
    P = laser.Pool(pool["tokens"], pool["seq_off"], pool["seq_key"], n_max)
    ora = RegroupedPool(pool["tokens"], pool["seq_off"], pool["seq_key"])
    info = P.info()
    assert info["n_tokens"] == ora.P.size == pool["tokens"].size and info["n_keys"] == len(ora.key_range)
    for start in (0, ora.P.size // 2, ora.P.size - 4096):              # sampled windows of the regrouped array
        assert (P.read_tokens(start, 4096) == ora.P[start:start + 4096]).all()
    g = laser.retrieve_drafts(P, torch.tensor(ctx["keys"].astype(np.int64), device="cuda"), torch.tensor(tails, device="cuda"),
                              1, n_max, K, 1)
    torch.cuda.synchronize()
    d, dl, mn, pi = (t.cpu().numpy() for t in g)
    od, odl, omn, opi = retrieve(ora, ctx["keys"], tails, 1, n_max, K, 1)
    assert (dl == odl).all() and (mn == omn).all() and (pi == opi).all() and (d == od).all()
    hit = dl > 0
    for b in np.nonzero(hit)[0][:512]:                                 # the chain literally occurs in the pool
        assert (ora.P[pi[b] + 1:pi[b] + 1 + dl[b]] == d[b, :dl[b]]).all()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    kd, td = torch.tensor(ctx["keys"].astype(np.int64), device="cuda"), torch.tensor(tails, device="cuda")
    e0.record()
    for _ in range(20):
        laser.retrieve_drafts(P, kd, td, 1, n_max, K, 1, out=g)
    e1.record()
    torch.cuda.synchronize()
    print(f"[retrieval stress] {ora.P.size} tokens, {len(ora.key_range)} keys, {int(hit.sum())} of {B} contexts matched, "
          f"mean draft length {dl[hit].mean():.2f}; {e0.elapsed_time(e1) * 1e3 / 20:.1f} us per batch of {B} lookups")
    P.close()
