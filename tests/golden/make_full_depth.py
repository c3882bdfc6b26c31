#!/usr/bin/env python3
"""Writes tests/golden/full_depth_<shape>.npz: what the float64 oracle computes at the FULL depth of the
7B shape (32 layers, d 4096, 32 heads, FFN 11008, vocabulary 32000) and of the 1B shape (16 layers, d 2048,
16 heads, FFN 5632, vocabulary 32000), seeded weights of synth/model.py, for one verify step per case
(Eq. 3 / Eq. 6 forward, Eq. 8 acceptance):

  7b  c3    the latency configuration itself: one sequence, context 1024, K = 8
      many  12 sequences, context 24, K = 8 (108 rows: one tile of the many-row launch shape); the oracle
            follows sequences 0 and 7
      mid   6 sequences, context 24, K = 8 (54 rows: the 17..80-row launch shape); sequences 1 and 4
      thr   64 sequences, context 24, K = 10 (704 rows: the throughput configuration's launch shape, six row
            tiles with a ragged last one); sequences 0, 37 and 63
  1b  c2    the 1B configuration itself: 8 sequences, context 512, K = 8; sequences 2 and 5

Every case is stored in two variants that share prompts and the cached context:
  <case>    k = 2, p = 0, final-norm gain as generated (lm_gain 1): the logits comparison proper
  <case>p   k = 2, p = 0.1 (the paper's defaults, Sec. 4.1.4) with the final-norm gain scaled by lm_gain = 5,
            so that top-1 / top-2 probabilities lie on both sides of the threshold and Eq. 8's second clause
            decides rows; one of its right drafts is replaced by the row's second-ranked token.

It calls only oracle/ and synth/ (never the HIP library). The 7B oracle needs the weights on the host (26 GB as
float32) and about half an hour on 8 cores, more than a GPU test may take, so the GPU tests compare against
these files instead. Stored per followed sequence: the prompt, the drafts, every fourth logit column plus the
64 largest logits of every row (float32), the accepted length, the emitted tokens, the oracle's deciding
margins, and <case>_params = [k, p, mode, lm_gain].

    python tests/golden/make_full_depth.py            # all cases of both shapes
    python tests/golden/make_full_depth.py thr c2     # only the named cases; the others are kept from the files
"""
from __future__ import annotations

import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth                                   # noqa: E402
from oracle import step                        # noqa: E402
from oracle.decoder import Decoder             # noqa: E402

COL_STRIDE, N_TOP = 4, 64
SHARP_GAIN = 5.0
CASES = {
    #        shape  B   ctx   K  followed  seed  right drafts
    "c3": ("7b", 1, 1024, 8, [0], 41, 5),
    "many": ("7b", 12, 24, 8, [0, 7], 13, 3),
    "mid": ("7b", 6, 24, 8, [1, 4], 17, 3),
    "thr": ("7b", 64, 24, 10, [0, 37, 63], 23, 4),
    "c2": ("1b", 8, 512, 8, [2, 5], 29, 4),
}
#            suffix  k  p    mode  lm_gain
VARIANTS = (("", 2, 0.0, 0, 1.0), ("p", 2, 0.1, 0, SHARP_GAIN))
HERE = os.path.dirname(os.path.abspath(__file__))


def golden_path(shape_name: str) -> str:
    return os.path.join(HERE, f"full_depth_{shape_name}.npz")


def verify_without_commit(dec, seqs, drafts, dl, k, p, mode):
    """step.verify_step, then the sequences are put back where they were (the keys/values it wrote behind the
    committed context are the same for every variant: they do not depend on the final norm)."""
    saved = [(s.cache.length, list(s.tokens)) for s in seqs]
    res = step.verify_step(dec, seqs, drafts, dl, k, p, mode, return_logits=True)
    for s, (ln, tk) in zip(seqs, saved):
        s.cache.length, s.tokens = ln, tk
    return res


def pack(name, B, ctx, K, follow, prompts, drafts, dl, res, params, vocab):
    lg = res["logits"]                                           # [followed][K+1][V]
    cols = np.arange(0, vocab, COL_STRIDE, dtype=np.int32)
    top_idx = np.argsort(-lg, axis=-1, kind="stable")[..., :N_TOP].astype(np.int32)
    R = K + 1
    rank_margin = np.full((len(follow), R), np.inf)
    logq_margin = np.full((len(follow), R), np.inf)
    for i, st in enumerate(res["stats"]):
        for r, s in enumerate(st):
            rank_margin[i, r], logq_margin[i, r] = s["rank_margin"], s["logq_margin"]
    return {
        f"{name}_shape": np.array([B, ctx, K], dtype=np.int32), f"{name}_follow": np.array(follow, dtype=np.int32),
        f"{name}_prompts": prompts.astype(np.int32), f"{name}_drafts": drafts.astype(np.int32), f"{name}_draft_len": dl,
        f"{name}_cols": cols, f"{name}_logits_cols": lg[..., cols].astype(np.float32),
        f"{name}_top_idx": top_idx, f"{name}_top_val": np.take_along_axis(lg, top_idx, axis=-1).astype(np.float32),
        f"{name}_row_absmax": np.abs(lg).max(axis=-1), f"{name}_accept_len": res["accept_len"].astype(np.int32),
        f"{name}_out_tokens": res["out_tokens"].astype(np.int32), f"{name}_rank_margin": rank_margin,
        f"{name}_logq_margin": logq_margin, f"{name}_argmax_gap": np.asarray(res["argmax_gap"], dtype=np.float64),
        f"{name}_params": np.array(params, dtype=np.float64),
    }


def run_shape(shape_name: str, names, t0: float):
    sh = synth.SHAPES[shape_name]
    path = golden_path(shape_name)
    out = {}
    if os.path.exists(path):                       # keep what the file (written by this script) holds for the other cases
        with np.load(path) as old:
            drop = set(names) | {n + v[0] for n in names for v in VARIANTS}
            out.update({k: old[k] for k in old.files if k != "params" and k.split("_")[0] not in drop})
    weights = synth.gen_all_weights(sh)
    decs = {}
    for _, _, _, _, gain in VARIANTS:
        w = weights if gain == 1.0 else {**weights, ("gf", -1): synth.gen_weight(sh.with_(lm_gain=gain), "gf")}
        decs[gain] = Decoder(sh.n_layers, sh.d, sh.n_heads, sh.ffn, sh.vocab, w, sh.eps, sh.rope_base)
    dec = decs[1.0]
    print(f"{shape_name}: weights ready {time.time() - t0:.0f} s", flush=True)
    for name in names:
        _, B, ctx, K, follow, seed, n_right = CASES[name]
        prompts = synth.uniform_tokens(seed, 50, 0, B * ctx, sh.vocab).reshape(B, ctx)
        drafts = synth.uniform_tokens(seed, 51, 0, B * K, sh.vocab).reshape(B, K).copy()
        dl = np.full(B, K, dtype=np.int32)
        cap = ctx + 2 * (K + 1)
        seqs = [step.Sequence(dec, 0, prompts[b], cap) for b in follow]
        print(f"{name}: prefill done {time.time() - t0:.0f} s", flush=True)
        # The first n_right drafts are made right one pass at a time: row j of a forward gives the model's
        # own next token after draft j, which becomes draft j + 1 of the next pass.
        second = {}
        for j in range(n_right):
            for i, b in enumerate(follow):
                row_tokens = [seqs[i].pending] + [int(t) for t in drafts[b]]
                logits = dec.verify_forward(seqs[i].cache, row_tokens)
                order = np.argsort(-logits[j], kind="stable")
                drafts[b, j] = int(order[0])
                second[b] = int(order[1])          # of the last right row
            print(f"{name}: pass {j} {time.time() - t0:.0f} s", flush=True)
        for suffix, k, p, mode, gain in VARIANTS:
            dv = drafts.copy()
            if suffix:                             # a second-ranked draft where the last right one stood
                for b in follow:
                    dv[b, n_right - 1] = second[b]
            res = verify_without_commit(decs[gain], seqs, dv[follow], dl[follow], k, p, mode)
            out.update(pack(name + suffix, B, ctx, K, follow, prompts, dv, dl, res, [k, p, mode, gain], sh.vocab))
            qs = [[round(s["q"], 4) for s in st] for st in res["stats"]]
            print(f"{name}{suffix}: accepted {res['accept_len'].tolist()}, emitted {res['out_tokens'].tolist()}, "
                  f"q of the examined drafts {qs}, logit std {res['logits'].std():.3f}, {time.time() - t0:.0f} s", flush=True)
    np.savez(path, **out)
    print(f"wrote {path} ({os.path.getsize(path) / 1e6:.2f} MB) in {time.time() - t0:.0f} s", flush=True)


def main():
    t0 = time.time()
    only = sys.argv[1:] or list(CASES)
    for shape_name in ("1b", "7b"):
        names = [n for n in CASES if CASES[n][0] == shape_name and n in only]
        if names:
            run_shape(shape_name, names, t0)


if __name__ == "__main__":
    main()
