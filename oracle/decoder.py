"""Oracle: the verify forward of the target model (Sec. 2.1 Eq. 1 and 3, Sec. 3.4 Eq. 6).

TEST INFRASTRUCTURE ONLY -- never imported by the product package.

The paper treats the LLM as a black box that maps context + K drafts to K+1 next-token
distributions in one pass.  The architecture comes from the benchmark shapes: pre-norm
decoder blocks, RMSNorm (eps 1e-6), rotary positions (base 10000, element i paired with
i + head_dim/2), multi-head causal attention with scale 1/sqrt(head_dim), SwiGLU FFN,
no biases, untied embedding and output head.  Everything is evaluated in float64 (or the
dtype asked for) on the weight values handed in; activations and the KV cache are never
rounded.

Rows r = 0..R-1 of one sequence hold the tokens [pending, draft_1 .. draft_{R-1}] at
positions len+r; row r's output is the distribution of the token after it (q_{r+1}).  Keys
and values of all R rows are written behind the cache speculatively; `commit` keeps the
pending token plus the accepted drafts.

Token trees (Sec. 3.3, tree attention): the rows after the first may form a tree instead of a chain. parent_row[r]
(r >= 1) names the row whose token precedes row r's token (0 = the pending token); the pseudo-sequence lists parents
before children.  Row r then sits at position len + depth(r) and sees the committed cache, its ancestors and itself --
never a row of another branch.  Keys and values still go to slots len + r in row order; `compact` moves the
rows of an accepted branch to the slots right behind the pending token before they are committed.
"""
from __future__ import annotations

import numpy as np


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(v: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """v: [T][H][dh]; pos: [T].  Rotates the pair (v[i], v[i+dh/2]) by angle pos * base^(-2i/dh)."""
    dh = v.shape[-1]
    half = dh // 2
    inv_freq = base ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    ang = pos.astype(np.float64)[:, None] * inv_freq[None, :]          # [T][half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1).astype(v.dtype)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


class KVCache:
    """Per-sequence keys/values, [layer][slot][H][dh]; `length` = committed slots."""

    def __init__(self, n_layers: int, n_heads: int, head_dim: int, capacity: int, dtype=np.float64):
        self.k = np.zeros((n_layers, capacity, n_heads, head_dim), dtype=dtype)
        self.v = np.zeros_like(self.k)
        self.length = 0

    def commit(self, n_tokens: int) -> None:
        self.length += n_tokens

    def compact(self, rows) -> None:
        """rows: the row numbers (1-based behind the pending token's row 0, ascending) of an accepted branch.
        Their keys/values move from slots length + row to slots length + 1, length + 2, ..."""
        t0 = self.length
        for j, r in enumerate(rows):
            assert r >= j + 1
            self.k[:, t0 + 1 + j] = self.k[:, t0 + r]
            self.v[:, t0 + 1 + j] = self.v[:, t0 + r]


class Decoder:
    def __init__(self, n_layers, d, n_heads, ffn, vocab, weights, eps=1e-6, rope_base=10000.0,
                 dtype=np.float64):
        """weights[(name, layer)] -> array in the layouts of the data spec:
        wqkv [3d][d], wo [d][d], wgu [2F][d], wdown [d][F], g1, g2 [d]; ('emb',-1) [V][d],
        ('wlm',-1) [V][d], ('gf',-1) [d]."""
        self.L, self.d, self.H, self.F, self.V = n_layers, d, n_heads, ffn, vocab
        self.dh = d // n_heads
        self.w, self.eps, self.base, self.dt = weights, eps, rope_base, dtype

    def _w(self, name, layer=-1):
        return np.asarray(self.w[(name, layer)], dtype=self.dt)

    def new_cache(self, capacity: int) -> KVCache:
        return KVCache(self.L, self.H, self.dh, capacity, self.dt)

    def hidden(self, cache: KVCache, tokens, parent_row=None) -> np.ndarray:
        """Final-normed hidden states [R][d] for rows `tokens` placed after the committed cache.
        parent_row: None for a chain (row r follows row r - 1), else parent_row[r] < r for r >= 1 (entry 0 unused)."""
        tokens = np.asarray(tokens, dtype=np.int64)
        R, H, dh, d = tokens.size, self.H, self.dh, self.d
        t0 = cache.length
        if parent_row is None:
            parent_row = [-1] + list(range(R - 1))
        depth = np.zeros(R, dtype=np.int64)
        sees = [[0]] * R                        # rows of this pass a row attends to: its ancestors and itself
        for r in range(1, R):
            pr = int(parent_row[r])
            assert 0 <= pr < r
            depth[r] = depth[pr] + 1
            sees[r] = sees[pr] + [r]
        pos = t0 + depth
        x = self._w("emb")[tokens].copy()                                   # [R][d]
        for l in range(self.L):
            n1 = rmsnorm(x, self._w("g1", l), self.eps)
            qkv = n1 @ self._w("wqkv", l).T                                  # [R][3d]
            q = rope(qkv[:, :d].reshape(R, H, dh), pos, self.base)
            k = rope(qkv[:, d:2 * d].reshape(R, H, dh), pos, self.base)
            v = qkv[:, 2 * d:].reshape(R, H, dh)
            cache.k[l, t0:t0 + R] = k
            cache.v[l, t0:t0 + R] = v
            att = np.empty((R, H, dh), dtype=self.dt)
            for r in range(R):                                               # row r sees slots 0 .. t0-1 and its branch
                mine = [t0 + j for j in sees[r]]
                kk = np.concatenate([cache.k[l, :t0], cache.k[l, mine]])     # [T][H][dh]
                vv = np.concatenate([cache.v[l, :t0], cache.v[l, mine]])
                s = np.einsum("hd,thd->ht", q[r], kk) / np.sqrt(dh)          # [H][T]
                s = s - s.max(axis=1, keepdims=True)
                p = np.exp(s)
                p = p / p.sum(axis=1, keepdims=True)
                att[r] = np.einsum("ht,thd->hd", p, vv)
            x = x + att.reshape(R, d) @ self._w("wo", l).T
            n2 = rmsnorm(x, self._w("g2", l), self.eps)
            gu = n2 @ self._w("wgu", l).T                                    # [R][2F]
            x = x + (silu(gu[:, :self.F]) * gu[:, self.F:]) @ self._w("wdown", l).T
        return rmsnorm(x, self._w("gf"), self.eps)

    def head(self, h: np.ndarray) -> np.ndarray:
        return h @ self._w("wlm").T

    def verify_forward(self, cache: KVCache, tokens, parent_row=None) -> np.ndarray:
        """logits [R][V]; row r is the unnormalised log-distribution of the token that follows row r's token
        (q_{r+1} of Eq. 3 / Eq. 6 for a chain)."""
        return self.head(self.hidden(cache, tokens, parent_row))
