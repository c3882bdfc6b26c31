#!/usr/bin/env python3
"""Writes tests/golden/full_depth_7b.npz: what the float64 oracle computes at the FULL 7B shape
(32 layers, d 4096, 32 heads, FFN 11008, vocabulary 32000; seeded weights of synth/model.py) for two
verify steps (Eq. 3 / Eq. 6 forward, Eq. 8 acceptance with k = 2, p = 0):

  c3    the latency configuration itself: one sequence, context 1024, K = 8
  many  12 sequences, context 24, K = 8 (108 rows: the many-row launch shape); the oracle follows
        sequences 0 and 7
  mid   6 sequences, context 24, K = 8 (54 rows: the 17..80-row launch shape); the oracle follows
        sequences 1 and 4

It calls only oracle/ and synth/ (never the HIP library). The oracle needs the 7B weights on the host
(26 GB as float32) and a quarter of an hour on 8 cores, more than a GPU test may take, so the GPU tests
compare against this file instead. Stored per followed sequence: the prompt, the drafts, every fourth
logit column plus the 64 largest logits of every row (float32), the accepted length, the emitted tokens
and the oracle's deciding margins.

    python tests/golden/make_full_depth.py            # all cases
    python tests/golden/make_full_depth.py mid        # only the named cases; the others are kept from the file
"""
from __future__ import annotations

import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth                                   # noqa: E402
from oracle import acceptance, step            # noqa: E402
from oracle.decoder import Decoder             # noqa: E402

K_TOP, P_THR, MODE = 2, 0.0, 0
COL_STRIDE, N_TOP = 4, 64
CASES = {
    #        B   ctx   K  followed  seed  right drafts
    "c3": (1, 1024, 8, [0], 41, 5),
    "many": (12, 24, 8, [0, 7], 13, 3),
    "mid": (6, 24, 8, [1, 4], 17, 3),
}


def main():
    t0 = time.time()
    sh = synth.SHAPES["7b"]
    dec = Decoder(sh.n_layers, sh.d, sh.n_heads, sh.ffn, sh.vocab, synth.gen_all_weights(sh), sh.eps, sh.rope_base)
    print(f"weights ready {time.time() - t0:.0f} s", flush=True)
    out = {}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "full_depth_7b.npz")
    only = sys.argv[1:]
    if only:                                       # keep what the file (written by this script) holds for the other cases
        with np.load(path) as old:
            out.update({k: old[k] for k in old.files if k != "params" and k.split("_")[0] not in only})
    for name, (B, ctx, K, follow, seed, n_right) in CASES.items():
        if only and name not in only:
            continue
        prompts = synth.uniform_tokens(seed, 50, 0, B * ctx, sh.vocab).reshape(B, ctx)
        drafts = synth.uniform_tokens(seed, 51, 0, B * K, sh.vocab).reshape(B, K).copy()
        dl = np.full(B, K, dtype=np.int32)
        cap = ctx + 2 * (K + 1)
        seqs = [step.Sequence(dec, 0, prompts[b], cap) for b in follow]
        print(f"{name}: prefill done {time.time() - t0:.0f} s", flush=True)
        # The first n_right drafts are made right one pass at a time: row j of a forward gives the model's
        # own next token after draft j, which becomes draft j + 1 of the next pass.
        for j in range(n_right):
            for i, b in enumerate(follow):
                row_tokens = [seqs[i].pending] + [int(t) for t in drafts[b]]
                logits = dec.verify_forward(seqs[i].cache, row_tokens)
                drafts[b, j] = int(np.argmax(logits[j]))
            print(f"{name}: pass {j} {time.time() - t0:.0f} s", flush=True)
        res = step.verify_step(dec, seqs, drafts[follow], dl[follow], K_TOP, P_THR, MODE, return_logits=True)
        lg = res["logits"]                                           # [followed][K+1][V]
        cols = np.arange(0, sh.vocab, COL_STRIDE, dtype=np.int32)
        top_idx = np.argsort(-lg, axis=-1, kind="stable")[..., :N_TOP].astype(np.int32)
        R = K + 1
        rank_margin = np.full((len(follow), R), np.inf)
        logq_margin = np.full((len(follow), R), np.inf)
        for i, st in enumerate(res["stats"]):
            for r, s in enumerate(st):
                rank_margin[i, r], logq_margin[i, r] = s["rank_margin"], s["logq_margin"]
        out.update({
            f"{name}_shape": np.array([B, ctx, K], dtype=np.int32), f"{name}_follow": np.array(follow, dtype=np.int32),
            f"{name}_prompts": prompts.astype(np.int32), f"{name}_drafts": drafts.astype(np.int32), f"{name}_draft_len": dl,
            f"{name}_cols": cols, f"{name}_logits_cols": lg[..., cols].astype(np.float32),
            f"{name}_top_idx": top_idx, f"{name}_top_val": np.take_along_axis(lg, top_idx, axis=-1).astype(np.float32),
            f"{name}_row_absmax": np.abs(lg).max(axis=-1), f"{name}_accept_len": res["accept_len"].astype(np.int32),
            f"{name}_out_tokens": res["out_tokens"].astype(np.int32), f"{name}_rank_margin": rank_margin,
            f"{name}_logq_margin": logq_margin, f"{name}_argmax_gap": np.asarray(res["argmax_gap"], dtype=np.float64),
        })
        print(f"{name}: accepted {res['accept_len'].tolist()}, emitted {res['out_tokens'].tolist()}, "
              f"logit std {lg.std():.3f}, {time.time() - t0:.0f} s", flush=True)
    out["params"] = np.array([K_TOP, P_THR, MODE], dtype=np.float64)
    np.savez(path, **out)
    print(f"wrote {path} ({os.path.getsize(path) / 1e6:.2f} MB) in {time.time() - t0:.0f} s")


if __name__ == "__main__":
    main()
