"""Helpers for the GPU parity tests: build the HIP-side model from the seeded weight recipe, run
prefill through the C ABI, and compare step results with the oracle under the stated tolerance."""
from __future__ import annotations

import numpy as np
import torch

import synth
from synth.model import torch_gen_weight

ATOL, RTOL = 2e-2, 1e-2          # logits: |gpu - oracle| <= ATOL + RTOL * |oracle|


def gpu_weights(sh: synth.ModelShape, device="cuda") -> dict:
    w = {}
    for name in ("wqkv", "wo", "wgu", "wdown", "g1", "g2"):
        if sh.n_layers:
            w[name] = torch.stack([torch_gen_weight(sh, name, l, device) for l in range(sh.n_layers)]).contiguous()
    for name in ("emb", "wlm", "gf"):
        if name == "emb" and sh.n_layers == 0:
            continue
        w[name] = torch_gen_weight(sh, name, -1, device).contiguous()
    return w


def make_model(sh: synth.ModelShape, max_rows: int, max_batch: int, max_pos: int):
    import paper_2408_05676_amd as laser
    w = gpu_weights(sh)
    return laser.Model(sh.n_layers, sh.d, sh.n_heads, sh.ffn, sh.vocab, w, max_rows, max_batch, max_pos,
                       eps=sh.eps, rope_base=sh.rope_base)


def make_kv(sh: synth.ModelShape, n_pages: int, max_seqs: int, max_pages_per_seq: int):
    import paper_2408_05676_amd as laser
    return laser.KVCache(sh.n_layers, sh.n_heads, sh.head_dim, n_pages, max_seqs, max_pages_per_seq)


def prefill(model, kv, seq_ids, prompts, chunk: int = 16):
    """Feed every prompt but its last token through laser_verify_step in chunks, forcing acceptance at commit.
    prompts: int[B][T], or a list of B arrays of different lengths (each chunk then runs the sequences that
    still have tokens left, with ragged draft lengths). Returns the pending tokens (last prompt token of each
    sequence) as a CUDA tensor."""
    import paper_2408_05676_amd as laser
    prompts = [np.asarray(p) for p in prompts]
    B = len(prompts)
    pos = 0
    while True:
        act = [b for b in range(B) if pos < len(prompts[b]) - 1]
        if not act:
            break
        n = [min(chunk, len(prompts[b]) - 1 - pos) for b in act]
        K = max(n) - 1
        dr = np.zeros((len(act), K), dtype=np.int32)
        for i, b in enumerate(act):
            dr[i, :n[i] - 1] = prompts[b][pos + 1:pos + n[i]]
        pend = torch.tensor([int(prompts[b][pos]) for b in act], dtype=torch.int32, device="cuda")
        dl = torch.tensor([v - 1 for v in n], dtype=torch.int32, device="cuda")
        ids = [seq_ids[b] for b in act]
        laser.verify_step(model, kv, ids, pend, torch.tensor(dr, device="cuda"), dl, 1, -1.0)
        laser.kv_commit(kv, ids, dl)              # accept_len := rows - 1 -> all fed rows become permanent
        pos += chunk
    return torch.tensor([int(p[-1]) for p in prompts], dtype=torch.int32, device="cuda")


def logits_close(g: np.ndarray, o: np.ndarray):
    err = np.abs(g - o)
    bound = ATOL + RTOL * np.abs(o)
    return bool((err <= bound).all()), float(err.max()), float((err / bound).max())


def classify_step(acc_g, out_g, ora, drafts, draft_len, k, p, slack=3.0):
    """Compare accepted lengths / emitted tokens with the oracle result `ora` (from
    oracle.step.verify_step with return_logits). A disagreement counts as an in-tolerance flip
    when, at the first row whose decision differs, the oracle's deciding margin is below the
    logit tolerance (times `slack`); anything else is a real mismatch."""
    flips, bad = 0, []
    B = len(acc_g)
    for b in range(B):
        a_o = int(ora["accept_len"][b])
        a_g = int(acc_g[b])
        same = a_o == a_g and list(out_g[b]) == list(ora["out_tokens"][b])
        if same:
            continue
        row = min(a_o, a_g)
        lrow = ora["logits"][b, row]
        tol = slack * (ATOL + RTOL * float(np.abs(lrow).max()))
        margins = []
        if a_o != a_g:
            st = ora["stats"][b][row] if row < len(ora["stats"][b]) else None
            if st is None:                      # oracle stopped at draft_len; GPU cannot go further
                bad.append((b, a_o, a_g, "beyond draft_len"))
                continue
            margins = [st["rank_margin"], st["logq_margin"] / 2.0]
        else:                                   # same length, different correction token
            margins = [float(ora["argmax_gap"][b])]
        if min(margins) <= tol:
            flips += 1
        else:
            bad.append((b, a_o, a_g, margins, tol))
    return flips, bad
