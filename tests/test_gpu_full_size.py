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
