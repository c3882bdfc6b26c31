"""Host-side orchestration of the decoding loop over the C ABI (no arithmetic of the method here:
every step is a library call).  Used by bench.py, __graft_entry__.smoke() and the GPU tests."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as L


def stacked_weights(gen_one, shape, device="cuda") -> dict:
    """Build the stacked [L][...] weight tensors the model descriptor wants from a per-tensor
    generator gen_one(name, layer) -> CUDA tensor."""
    w = {}
    if shape.n_layers:
        for name in ("wqkv", "wo", "wgu", "wdown", "g1", "g2"):
            first = gen_one(name, 0)
            full = torch.empty((shape.n_layers,) + tuple(first.shape), dtype=first.dtype, device=device)
            full[0] = first
            del first
            for l in range(1, shape.n_layers):
                full[l] = gen_one(name, l)
            w[name] = full
        w["emb"] = gen_one("emb", -1)
    w["wlm"] = gen_one("wlm", -1)
    w["gf"] = gen_one("gf", -1)
    return w


class Engine:
    """One model + one KV cache + (optionally) one pool, and a batch of B running sequences whose
    state (pending token, context tail) lives on the device."""

    def __init__(self, shape, weights: dict, batch: int, K: int, max_len: int, n_max: int = 3,
                 prefill_chunk: int = 16, own_text_cap: int = 0):
        """own_text_cap > 0: keep each sequence's own text (prompt + emitted tokens, the most recent own_text_cap of
        them) on the device and search it as a temporary branch at every retrieval (Sec. 3.2)."""
        self.shape, self.B, self.K, self.n_max = shape, batch, K, n_max
        R = max(K + 1, prefill_chunk)
        pages_per_seq = (max_len + 15) // 16 + 1
        self.model = L.Model(shape.n_layers, shape.d, shape.n_heads, shape.ffn, shape.vocab, weights,
                             max_rows=batch * R, max_batch=batch, max_pos=pages_per_seq * 16,
                             eps=shape.eps, rope_base=shape.rope_base)
        self.kv = L.KVCache(shape.n_layers, shape.n_heads, shape.head_dim, n_pages=batch * pages_per_seq,
                            max_seqs=batch, max_pages_per_seq=pages_per_seq)
        self.seq_ids = np.arange(batch, dtype=np.int32)
        for s in range(batch):
            self.kv.reserve(s, pages_per_seq * 16)
        self.prefill_chunk = prefill_chunk
        dev = "cuda"
        self.pending = torch.zeros(batch, dtype=torch.int32, device=dev)
        self.ctx_tail = torch.full((batch, n_max), -1, dtype=torch.int32, device=dev)
        self.keys = torch.zeros(batch, dtype=torch.int64, device=dev)
        self.drafts = torch.full((batch, K), -1, dtype=torch.int32, device=dev)
        self.draft_len = torch.zeros(batch, dtype=torch.int32, device=dev)
        self.match_n = torch.zeros(batch, dtype=torch.int32, device=dev)
        self.pool_index = torch.zeros(batch, dtype=torch.int64, device=dev)
        self.accept_len = torch.zeros(batch, dtype=torch.int32, device=dev)
        self.out_tokens = torch.full((batch, K + 1), -1, dtype=torch.int32, device=dev)
        self.pool = None
        self.own_text = self.own_len = None
        if own_text_cap > 0:
            self.own_text = torch.zeros((batch, own_text_cap), dtype=torch.int32, device=dev)
            self.own_len = torch.zeros(batch, dtype=torch.int32, device=dev)

    def set_pool(self, pool: L.Pool, keys):
        self.pool = pool
        self.keys.copy_(torch.as_tensor(np.asarray(keys, dtype=np.int64)))

    def prefill(self, prompts: np.ndarray):
        """prompts int[B][T]: tokens 0..T-2 go into the cache, token T-1 becomes the pending one."""
        B, T = prompts.shape
        assert B == self.B
        body = prompts[:, :-1]
        pos = 0
        while pos < T - 1:
            n = min(self.prefill_chunk, T - 1 - pos)
            pend = torch.as_tensor(np.ascontiguousarray(body[:, pos]), dtype=torch.int32).cuda()
            dr = torch.as_tensor(np.ascontiguousarray(body[:, pos + 1:pos + n]).reshape(B, n - 1), dtype=torch.int32).cuda()
            dl = torch.full((B,), n - 1, dtype=torch.int32, device="cuda")
            L.verify_step(self.model, self.kv, self.seq_ids, pend, dr, dl, 1, -1.0)
            L.kv_commit(self.kv, self.seq_ids, dl)
            pos += n
        self.pending.copy_(torch.as_tensor(np.ascontiguousarray(prompts[:, -1]), dtype=torch.int32))
        tail = np.full((B, self.n_max), -1, dtype=np.int32)
        t = min(T, self.n_max)
        tail[:, self.n_max - t:] = prompts[:, T - t:]
        self.ctx_tail.copy_(torch.as_tensor(tail))
        if self.own_text is not None:
            cap = self.own_text.shape[1]
            t = min(T, cap)
            self.own_text[:, :t] = torch.as_tensor(np.ascontiguousarray(prompts[:, T - t:]), dtype=torch.int32).cuda()
            self.own_len.fill_(t)

    def step(self, topk: int, p: float, mode: int = L.MODE_RV, n_min: int = 1, retrieve: bool = True):
        """retrieve -> verify -> commit -> context update; all asynchronous."""
        if retrieve and self.pool is not None and self.K > 0:
            out = (self.drafts, self.draft_len, self.match_n, self.pool_index)
            if self.own_text is not None:
                L.retrieve_drafts_temp(self.pool, self.keys, self.ctx_tail, self.own_text, self.own_len, n_min, self.n_max,
                                       self.K, 1, out=out)
            else:
                L.retrieve_drafts(self.pool, self.keys, self.ctx_tail, n_min, self.n_max, self.K, 1, out=out)
        L.verify_step(self.model, self.kv, self.seq_ids, self.pending, self.drafts, self.draft_len, topk, p, mode,
                      out=(self.accept_len, self.out_tokens))
        L.kv_commit(self.kv, self.seq_ids, self.accept_len)
        L.ctx_advance(self.ctx_tail, self.pending, self.out_tokens, self.accept_len)
        if self.own_text is not None:
            L.own_text_append(self.own_text, self.own_len, self.out_tokens, self.accept_len)

    def generate_greedy(self, n_tokens: int) -> np.ndarray:
        """Plain autoregressive greedy decoding (K = 0: one row per sequence): int32[B][n_tokens]."""
        out = torch.empty((self.B, n_tokens), dtype=torch.int32, device="cuda")
        no_drafts = torch.empty((self.B, 0), dtype=torch.int32, device="cuda")
        zero = torch.zeros(self.B, dtype=torch.int32, device="cuda")
        tok = torch.empty((self.B, 1), dtype=torch.int32, device="cuda")
        for i in range(n_tokens):
            L.verify_step(self.model, self.kv, self.seq_ids, self.pending, no_drafts, zero, 1, -1.0, out=(self.accept_len, tok))
            L.kv_commit(self.kv, self.seq_ids, self.accept_len)
            L.ctx_advance(self.ctx_tail, self.pending, tok, self.accept_len)
            if self.own_text is not None:
                L.own_text_append(self.own_text, self.own_len, tok, self.accept_len)
            out[:, i] = tok[:, 0]
        return out.cpu().numpy()

    def close(self):
        self.model.close()
        self.kv.close()
