"""Seeded template-plus-substitution token streams: retrieval pools and query contexts.

Recipe (stands in for the knowledge texts the paper's pools are built from): T random token
templates; a pool sequence is a copy of one template in which each position is replaced,
independently with probability `sub_rate`, by a uniform random token; a context is a fresh
substituted copy of a template of the same key, cut at a random point and left-padded with
random tokens to the requested length.  Every key owns a small set of templates
(`templates_per_key`), which is what makes a per-key pool more relevant than a global one.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

from . import rng

_S_TEMPL, _S_SUBMASK, _S_SUBTOK, _S_KEY, _S_TSEL, _S_LEN, _S_CUT, _S_PAD, _S_OFF = range(100, 109)


@dataclass(frozen=True)
class PoolSpec:
    name: str
    vocab: int
    n_seq: int
    seq_len: int              # fixed length, or the mean when lognormal_len is set
    n_templates: int
    sub_rate: float
    n_keys: int = 1
    key_dist: str = "round_robin"   # "round_robin" | "zipf"
    zipf_a: float = 1.1
    templates_per_key: int = 2
    lognormal_len: bool = False     # lengths ~ lognormal(sigma=1), mean seq_len, clipped to [8, 8192]
    seed: int = 0x504F4F4C

    def with_(self, **kw) -> "PoolSpec":
        return replace(self, **kw)


POOLS = {
    "tiny": PoolSpec("tiny", 2048, 500, 64, 20, 0.10),
    "1b": PoolSpec("1b", 32000, 10_000, 256, 200, 0.15, n_keys=1000),
    "7b_latency": PoolSpec("7b_latency", 32000, 2000, 256, 50, 0.10),
    "7b_throughput": PoolSpec("7b_throughput", 32000, 3906, 256, 500, 0.10, n_keys=10_000,
                              key_dist="zipf"),
    "stress": PoolSpec("stress", 128256, 1_000_000, 100, 4096, 0.10, n_keys=1_000_000,
                       templates_per_key=1, lognormal_len=True),
}


def gen_templates(spec: PoolSpec) -> np.ndarray:
    """int32[n_templates][template_len]; template_len = seq_len (256 for lognormal pools)."""
    tl = 256 if spec.lognormal_len else spec.seq_len
    t = rng.uniform_tokens(spec.seed, _S_TEMPL, 0, spec.n_templates * tl, spec.vocab)
    return t.reshape(spec.n_templates, tl)


def _zipf_ranks(seed, stream, count, n, a):
    w = np.arange(1, n + 1, dtype=np.float64) ** (-a)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    u = rng.uniform_unit(seed, stream, 0, count)
    return np.minimum(np.searchsorted(cdf, u, side="right"), n - 1).astype(np.int64)


def _key_ids(spec: PoolSpec, ranks: np.ndarray) -> np.ndarray:
    """Map a key's rank (0 = most popular) to an opaque, non-contiguous int64 key id."""
    return (ranks.astype(np.int64) * 2654435761 + 12345) % (1 << 40)


def _template_of(spec: PoolSpec, ranks: np.ndarray, choice: np.ndarray) -> np.ndarray:
    return ((ranks * 7 + choice) % spec.n_templates).astype(np.int64)


def _substitute(spec: PoolSpec, toks: np.ndarray, stream_salt: int, start: int) -> np.ndarray:
    n = toks.size
    u = rng.uniform_unit(spec.seed, _S_SUBMASK + 1000 * stream_salt, start, n)
    r = rng.uniform_tokens(spec.seed, _S_SUBTOK + 1000 * stream_salt, start, n, spec.vocab)
    return np.where(u < spec.sub_rate, r, toks.reshape(-1)).astype(np.int32)


def noisy_copy(spec: PoolSpec, toks: np.ndarray, salt: int) -> np.ndarray:
    """A copy of `toks` with the pool's substitution noise (seeded by `salt`)."""
    toks = np.asarray(toks, dtype=np.int32)
    return _substitute(spec, toks.copy(), 50 + salt, 0).reshape(toks.shape)


def gen_pool(spec: PoolSpec):
    """Returns dict(tokens int32[N], seq_off int64[n_seq+1], seq_key int64[n_seq],
    seq_rank int64[n_seq], seq_template int64[n_seq])."""
    templ = gen_templates(spec)
    tl = templ.shape[1]
    ns = spec.n_seq
    if spec.key_dist == "zipf":
        ranks = _zipf_ranks(spec.seed, _S_KEY, ns, spec.n_keys, spec.zipf_a)
    else:
        ranks = np.arange(ns, dtype=np.int64) % spec.n_keys
    choice = (rng.hash_u64(spec.seed, _S_TSEL, 0, ns) % np.uint64(spec.templates_per_key)).astype(np.int64)
    tid = _template_of(spec, ranks, choice)
    if spec.lognormal_len:
        # lognormal with sigma 1 and the requested mean, from a 12-uniform bell variate
        z = sum(rng.uniform_unit(spec.seed, _S_LEN + 10 * j, 0, ns) for j in range(12)) - 6.0
        ln = np.exp(np.log(spec.seq_len) - 0.5 + z)
        lens = np.clip(np.rint(ln), 8, 8192).astype(np.int64)
        offs = (rng.hash_u64(spec.seed, _S_OFF, 0, ns) % np.uint64(tl)).astype(np.int64)
    else:
        lens = np.full(ns, spec.seq_len, dtype=np.int64)
        offs = np.zeros(ns, dtype=np.int64)
    seq_off = np.zeros(ns + 1, dtype=np.int64)
    np.cumsum(lens, out=seq_off[1:])
    n_tok = int(seq_off[-1])
    tokens = np.empty(n_tok, dtype=np.int32)
    step = 1 << 22
    s0 = 0
    while s0 < ns:  # chunk over sequences so the expanded index arrays stay bounded
        s1 = s0
        acc = 0
        while s1 < ns and acc < step:
            s1 = min(ns, s1 + 4096)
            acc = int(seq_off[s1] - seq_off[s0])
        lo, hi = int(seq_off[s0]), int(seq_off[s1])
        rep = np.repeat(np.arange(s0, s1), lens[s0:s1])
        within = np.arange(lo, hi) - seq_off[rep]
        base = templ[tid[rep], (offs[rep] + within) % tl]
        tokens[lo:hi] = _substitute(spec, base, 0, lo)
        s0 = s1
    return {"tokens": tokens, "seq_off": seq_off, "seq_key": _key_ids(spec, ranks),
            "seq_rank": ranks, "seq_template": tid}


def gen_contexts(spec: PoolSpec, batch: int, ctx_len: int, n_max: int, salt: int = 1,
                 min_remaining: int = 0):
    """Returns dict(keys int64[B], ctx int32[B][ctx_len], template int64[B], cut int64[B]).

    ctx[b, -cut:] is a freshly substituted copy of template[b][:cut] (or its last ctx_len
    tokens); the part before it is uniform random padding.  `cut` is uniform over
    [n_max, template_len - min_remaining].  Keys follow the pool's key distribution.
    """
    templ = gen_templates(spec)
    tl = templ.shape[1]
    st = 7000 + 50 * salt
    if spec.key_dist == "zipf":
        ranks = _zipf_ranks(spec.seed, st + 0, batch, spec.n_keys, spec.zipf_a)
    else:
        ranks = (rng.hash_u64(spec.seed, st + 0, 0, batch) % np.uint64(spec.n_keys)).astype(np.int64)
    choice = (rng.hash_u64(spec.seed, st + 1, 0, batch) % np.uint64(spec.templates_per_key)).astype(np.int64)
    tid = _template_of(spec, ranks, choice)
    hi = max(n_max, tl - min_remaining)
    cut = n_max + (rng.hash_u64(spec.seed, st + 2, 0, batch) % np.uint64(hi - n_max + 1)).astype(np.int64)
    ctx = rng.uniform_tokens(spec.seed, st + 3, 0, batch * ctx_len, spec.vocab).reshape(batch, ctx_len)
    for b in range(batch):
        c = int(cut[b])
        body = _substitute(spec, templ[tid[b], :c].copy(), 2 + salt, b * tl)
        take = min(c, ctx_len)
        ctx[b, ctx_len - take:] = body[c - take:]
    return {"keys": _key_ids(spec, ranks), "ctx": ctx, "template": tid, "cut": cut, "rank": ranks}
