"""GPU parity of laser_generate (the whole generation loop, Sec. 3.1) through the C ABI against the oracle's loop:
emitted texts, lengths and counters for chain drafts, token trees, the temporary branch and no drafts at all; stops
at the end-of-sequence token and at max_new_tokens inside a step; finished sequences stay unchanged in the batch."""
import numpy as np
import pytest
import torch

import synth
from oracle import retrieval, step
from oracle.decoder import Decoder
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape_name,fused", [("tiny", 1), ("tiny128", 0), ("tiny128", 1)])
def test_generate_against_the_oracle(shape_name, fused):
    import paper_2408_05676_amd as laser
    sh = synth.SHAPES[shape_name].with_(lm_gain=4.0)
    dec = Decoder(sh.n_layers, sh.d, sh.n_heads, sh.ffn, sh.vocab, synth.gen_all_weights(sh), sh.eps, sh.rope_base)
    B, K, n_max, max_new = 3, 4, 3, 37                                  # 15 rows: the persistent kernel when fused = 1
    lens = [21, 33, 26]
    prompts = [synth.uniform_tokens(70 + b, 1, 0, lens[b], sh.vocab) for b in range(B)]
    ref = [step.autoregressive_greedy(dec, step.Sequence(dec, b, prompts[b], 128), 48) for b in range(B)]
    r = np.random.default_rng(2)
    texts, keys = [], []
    for b in range(B):
        full = np.array(list(prompts[b][-n_max:]) + ref[b], dtype=np.int32)
        for _ in range(3):
            noisy = full.copy()
            hit = r.random(noisy.size) < 0.1
            hit[:n_max] = False
            noisy[hit] = r.integers(0, sh.vocab, size=int(hit.sum()))
            texts.append(noisy); keys.append(b)
    flat = np.concatenate(texts).astype(np.int32)
    off = np.cumsum([0] + [len(t) for t in texts]).astype(np.int64)
    skey = np.array(keys, dtype=np.int64)
    opool = retrieval.RegroupedPool(flat, off, skey)
    pool = laser.Pool(flat, off, skey, n_max)
    eos = ref[1][22]                                                     # sequence 1 stops early
    cap = max(lens) + max_new + 2 * (K + 1) + 16
    for kind in ("chain", "tree", "temp", "none"):
        model = gu.make_model(sh, max_rows=B * 16, max_batch=B, max_pos=cap + 16)
        model.set_option("fused", fused)
        kv = gu.make_kv(sh, n_pages=B * (cap // 16 + 2), max_seqs=B, max_pages_per_seq=cap // 16 + 2)
        ids = list(range(B))
        for s in ids:
            kv.reserve(s, cap)
        pend = gu.prefill(model, kv, ids, prompts)
        tail = torch.tensor(np.stack([p[-n_max:] for p in prompts]).astype(np.int32), device="cuda")
        kd = torch.arange(B, dtype=torch.int64, device="cuda")
        own = own_len = None
        if kind == "temp":
            own = torch.zeros((B, 64), dtype=torch.int32, device="cuda")
            own_len = torch.tensor([min(l, 64) for l in lens], dtype=torch.int32, device="cuda")
            for b in range(B):
                own[b, :min(lens[b], 64)] = torch.tensor(prompts[b][-64:].astype(np.int32), device="cuda")
        gen, glen, cnt, steps, ms = laser.generate(model, kv, None if kind == "none" else pool, ids, kd, tail, pend, K, 1, 1, -1.0, 0,
                                                   max_new_tokens=max_new, eos_token=eos, tree=(kind == "tree"), check_every=3,
                                                   own_tokens=own, own_len=own_len, time_retrieval=True)
        seqs = [step.Sequence(dec, b, prompts[b], cap) for b in range(B)]
        want, wcnt = step.generate(dec, None if kind == "none" else opool, seqs, 1, n_max, K, 1, -1.0, 0, max_new_tokens=max_new,
                                   eos_token=eos, tree=(kind == "tree"), temporary_branch=64 if kind == "temp" else 0)
        gen, glen, cnt = gen.cpu().numpy(), glen.cpu().numpy(), cnt.cpu().numpy()
        for b in range(B):
            assert gen[b, :glen[b]].tolist() == want[b], (kind, b)
            assert (gen[b, glen[b]:] == -1).all()
            assert want[b] == (ref[b][:max_new] if eos not in ref[b][:max_new] else ref[b][:ref[b].index(eos) + 1])   # strict == greedy
            assert cnt[b].tolist() == wcnt[b], (kind, b, cnt[b].tolist(), wcnt[b])
        assert kv.read_lens(ids).tolist() == [s.cache.length for s in seqs]
        assert pend.cpu().tolist() == [s.pending for s in seqs]
        assert max(c[0] for c in wcnt) <= steps <= max(c[0] for c in wcnt) + 3        # stopped at the next look after the last one finished
        print(f"[generate {shape_name} fused={fused} {kind}] {steps} steps for {glen.tolist()} tokens, drafts kept per step "
              f"{cnt[:, 2].sum() / max(cnt[:, 0].sum(), 1):.2f}, retrieval {ms:.3f} ms")
        model.close(); kv.close()
    pool.close()
