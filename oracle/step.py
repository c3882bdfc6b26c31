"""Oracle: one whole Draft-then-Verify decoding step and the loops built from it
(Sec. 2.1 Eq. 1-4; Sec. 3.3-3.4).

TEST INFRASTRUCTURE ONLY -- never imported by the product package.
"""
from __future__ import annotations

import numpy as np

from . import acceptance, retrieval
from .decoder import Decoder


class Sequence:
    """One generation stream: its pool key, every token so far, and its KV cache.
    The last token (`pending`) is not in the cache yet; it is row 0 of the next forward."""

    def __init__(self, dec: Decoder, key: int, prompt, capacity: int):
        prompt = [int(t) for t in prompt]
        assert len(prompt) >= 1
        self.key = int(key)
        self.tokens = prompt[:]
        self.cache = dec.new_cache(capacity)
        if len(prompt) > 1:                     # prefill everything but the last token
            dec.hidden(self.cache, prompt[:-1])
            self.cache.commit(len(prompt) - 1)

    @property
    def pending(self) -> int:
        return self.tokens[-1]


def autoregressive_greedy(dec: Decoder, seq: Sequence, n_new: int):
    """Eq. 1 with argmax: one forward per token.  Returns the n_new generated tokens."""
    out = []
    for _ in range(n_new):
        logits = dec.verify_forward(seq.cache, [seq.pending])
        seq.cache.commit(1)
        t = int(np.argmax(logits[0]))
        seq.tokens.append(t)
        out.append(t)
    return out


def verify_step(dec: Decoder, seqs, drafts, draft_len, k: int, p: float, mode: int = 0,
                return_logits: bool = False):
    """Verify given drafts for every sequence (R = K+1 rows each), apply the acceptance rule,
    commit accepted tokens.  drafts int[B][K] (-1 padded; padded rows are fed token 0 and
    their outputs ignored)."""
    drafts = np.asarray(drafts)
    B, K = drafts.shape
    logits = np.empty((B, K + 1, dec.V), dtype=np.float64)
    for b, s in enumerate(seqs):
        row_tokens = [s.pending] + [int(t) if j < draft_len[b] else 0 for j, t in enumerate(drafts[b])]
        logits[b] = dec.verify_forward(s.cache, row_tokens)
    acc, out, stats, gaps = acceptance.verify_batch(logits, drafts, draft_len, k, p, mode)
    for b, s in enumerate(seqs):
        s.cache.commit(int(acc[b]) + 1)          # pending + accepted drafts become permanent
        s.tokens.extend(int(t) for t in out[b, :acc[b] + 1])
    res = {"accept_len": acc, "out_tokens": out, "stats": stats, "argmax_gap": gaps}
    if return_logits:
        res["logits"] = logits
    return res


def laser_step(dec: Decoder, pool: retrieval.RegroupedPool, seqs, n_min: int, n_max: int, K: int,
               k: int, p: float, mode: int = 0, min_tokens: int = 1, return_logits: bool = False,
               temporary_branch: int = 0):
    """retrieve -> verify -> accept -> commit for a batch of sequences.
    temporary_branch = W > 0: each sequence's own text (its last W tokens: prompt and everything emitted so far)
    is searched as one more sequence of its key's sub-pool (Sec. 3.2)."""
    tails = []
    for s in seqs:
        t = s.tokens[-n_max:]
        tails.append([-1] * (n_max - len(t)) + t)
    own = [s.tokens[-temporary_branch:] for s in seqs] if temporary_branch > 0 else None
    drafts, dl, mn, pi = retrieval.retrieve(pool, [s.key for s in seqs], tails, n_min, n_max, K, min_tokens, own=own)
    res = verify_step(dec, seqs, drafts, dl, k, p, mode, return_logits)
    res.update({"drafts": drafts, "draft_len": dl, "match_n": mn, "pool_index": pi})
    return res


def verify_tree_step(dec: Decoder, seqs, tokens, parents, n_nodes, k: int, p: float, mode: int = 0,
                     return_logits: bool = False):
    """Verify a token tree per sequence in one forward (tree attention), accept the longest verified branch, move
    its keys/values behind the pending token and commit them.  tokens, parents int[B][K] (pseudo-sequence order,
    parents = node index or -1; entries past n_nodes[b] are padding: fed as token 0 hanging off the previous row)."""
    tokens, parents = np.asarray(tokens), np.asarray(parents)
    B, K = tokens.shape
    logits = np.empty((B, K + 1, dec.V), dtype=np.float64)
    acc = np.zeros(B, dtype=np.int32)
    out = np.full((B, K + 1), -1, dtype=np.int32)
    paths = np.full((B, K), -1, dtype=np.int32)
    all_stats, gaps = [], np.zeros(B)
    for b, s in enumerate(seqs):
        nn = int(n_nodes[b])
        row_tokens = [s.pending] + [int(tokens[b, j]) if j < nn else 0 for j in range(K)]
        parent_row = [-1] + [int(parents[b, j]) + 1 if j < nn else j for j in range(K)]
        logits[b] = dec.verify_forward(s.cache, row_tokens, parent_row)
        path, toks, st, gap = acceptance.verify_tree(logits[b], tokens[b], parents[b], nn, k, p, mode)
        s.cache.compact([i + 1 for i in path])
        s.cache.commit(len(path) + 1)
        s.tokens.extend(toks)
        acc[b] = len(path)
        out[b, :len(toks)] = toks
        paths[b, :len(path)] = path
        all_stats.append(st)
        gaps[b] = gap
    res = {"accept_len": acc, "out_tokens": out, "accept_path": paths, "stats": all_stats, "argmax_gap": gaps}
    if return_logits:
        res["logits"] = logits
    return res


def laser_tree_step(dec: Decoder, pool: retrieval.RegroupedPool, seqs, n_min: int, n_max: int, K: int,
                    k: int, p: float, mode: int = 0, min_tokens: int = 1, return_logits: bool = False):
    """retrieve a token tree -> verify with tree attention -> accept the longest verified branch -> commit."""
    tails = []
    for s in seqs:
        t = s.tokens[-n_max:]
        tails.append([-1] * (n_max - len(t)) + t)
    tokens, parents, nn, mn = retrieval.retrieve_tree(pool, [s.key for s in seqs], tails, n_min, n_max, K, min_tokens)
    res = verify_tree_step(dec, seqs, tokens, parents, nn, k, p, mode, return_logits)
    res.update({"tree_tokens": tokens, "tree_parent": parents, "tree_len": nn, "match_n": mn})
    return res


def generate(dec: Decoder, pool, seqs, n_min: int, n_max: int, K: int, k: int, p: float, mode: int = 0,
             min_tokens: int = 1, max_new_tokens: int = 64, eos_token: int = -1, tree: bool = False,
             temporary_branch: int = 0):
    """The whole generation (Sec. 3.1): Draft-then-Verify steps until every sequence has emitted max_new_tokens
    tokens or eos_token (which is kept).  What a step emits beyond either limit is dropped, and only the kept
    tokens are committed.  pool None: one token per step (Eq. 1).  Sequences are independent; each runs its own
    steps.  Returns (list of emitted-token lists, per-sequence counters [steps, drafts offered, drafts kept,
    drafts accepted by the rule])."""
    texts, counters = [], []
    for s in seqs:
        emitted, cnt = [], [0, 0, 0, 0]
        while len(emitted) < max_new_tokens and (not emitted or emitted[-1] != eos_token):
            before_len, before_tokens = s.cache.length, list(s.tokens)
            if pool is None:
                res = verify_step(dec, [s], np.zeros((1, 0), dtype=np.int32), [0], k, p, mode)
                offered = 0
            elif tree:
                res = laser_tree_step(dec, pool, [s], n_min, n_max, K, k, p, mode, min_tokens)
                offered = int(res["tree_len"][0])
            else:
                res = laser_step(dec, pool, [s], n_min, n_max, K, k, p, mode, min_tokens, temporary_branch=temporary_branch)
                offered = int(res["draft_len"][0])
            a = int(res["accept_len"][0])
            out = [int(t) for t in res["out_tokens"][0, :a + 1]]
            n_emit = min(a + 1, max_new_tokens - len(emitted))
            if eos_token in out[:n_emit]:
                n_emit = out.index(eos_token) + 1
            # keep only n_emit tokens: the step committed a + 1
            s.cache.length = before_len + n_emit
            s.tokens = before_tokens + out[:n_emit]
            emitted += out[:n_emit]
            cnt[0] += 1; cnt[1] += offered; cnt[2] += n_emit - 1; cnt[3] += a
        texts.append(emitted)
        counters.append(cnt)
    return texts, counters
