"""Pins for oracle.decoder (Eq. 1, 3, 6): an independent torch-CPU evaluation of the same
architecture without any cache (library attention with an explicit mask, rotary
positions as complex multiplication), cached-vs-uncached-vs-sequential consistency, and
closed forms."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth
from oracle.decoder import Decoder, rmsnorm, rope, silu


def _make(shape_name="tiny", **kw):
    sh = synth.SHAPES[shape_name].with_(**kw)
    w = synth.gen_all_weights(sh)
    return sh, w, Decoder(sh.n_layers, sh.d, sh.n_heads, sh.ffn, sh.vocab, w, sh.eps, sh.rope_base)


def torch_full_forward(sh, w, tokens):
    """No cache: all T tokens at once, float64, library ops."""
    T, H, dh, d = len(tokens), sh.n_heads, sh.head_dim, sh.d
    tw = lambda n, l=-1: torch.from_numpy(np.asarray(w[(n, l)], dtype=np.float64))
    x = tw("emb")[torch.tensor(tokens)]
    half = dh // 2
    freqs = sh.rope_base ** (-torch.arange(half, dtype=torch.float64) * 2 / dh)
    rot = torch.polar(torch.ones(T, half, dtype=torch.float64),
                      torch.arange(T, dtype=torch.float64)[:, None] * freqs[None, :])   # e^{i pos f}

    def rotary(v):                                   # v [T][H][dh]; (v_i + i v_{i+half}) * e^{i theta}
        z = torch.complex(v[..., :half], v[..., half:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    mask = torch.tril(torch.ones(T, T, dtype=torch.bool))
    for l in range(sh.n_layers):
        n1 = F.rms_norm(x, (d,), tw("g1", l), sh.eps)
        qkv = F.linear(n1, tw("wqkv", l))
        q, k, v = (qkv[:, i * d:(i + 1) * d].reshape(T, H, dh) for i in range(3))
        q, k = rotary(q), rotary(k)
        a = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1),
                                           attn_mask=mask)          # [H][T][dh], default scale 1/sqrt(dh)
        x = x + F.linear(a.transpose(0, 1).reshape(T, d), tw("wo", l))
        n2 = F.rms_norm(x, (d,), tw("g2", l), sh.eps)
        gu = F.linear(n2, tw("wgu", l))
        x = x + F.linear(F.silu(gu[:, :sh.ffn]) * gu[:, sh.ffn:], tw("wdown", l))
    h = F.rms_norm(x, (d,), tw("gf"), sh.eps)
    return F.linear(h, tw("wlm")).numpy()


@pytest.mark.parametrize("shape_name", ["tiny", "tiny128"])
def test_cached_rows_equal_uncached_library_forward(shape_name):
    sh, w, dec = _make(shape_name)
    toks = synth.uniform_tokens(1, 1, 0, 23, sh.vocab).tolist()
    ref = torch_full_forward(sh, w, toks)                       # [23][V]
    cache = dec.new_cache(64)
    dec.hidden(cache, toks[:14])
    cache.commit(14)
    got = dec.verify_forward(cache, toks[14:])                  # rows at positions 14..22
    assert np.abs(got - ref[14:]).max() < 1e-9
    # the prefill rows themselves
    cache2 = dec.new_cache(64)
    got2 = dec.verify_forward(cache2, toks)
    assert np.abs(got2 - ref).max() < 1e-9


def test_multi_row_equals_sequential_single_rows_and_rollback():
    sh, w, dec = _make("tiny")
    toks = synth.uniform_tokens(2, 1, 0, 30, sh.vocab).tolist()
    c1 = dec.new_cache(64)
    dec.hidden(c1, toks[:20]); c1.commit(20)
    block = dec.verify_forward(c1, toks[20:26])                 # 6 rows in one pass
    c2 = dec.new_cache(64)
    dec.hidden(c2, toks[:20]); c2.commit(20)
    for r in range(6):
        one = dec.verify_forward(c2, [toks[20 + r]])
        c2.commit(1)
        assert np.abs(one[0] - block[r]).max() < 1e-9
    # accept only 2 of the 6 rows, then continue with different tokens: dead slots must not leak
    c1.commit(2)
    other = toks[26:30]
    after = dec.verify_forward(c1, other)
    ref = torch_full_forward(sh, w, toks[:22] + other)
    assert np.abs(after - ref[22:]).max() < 1e-9


def test_closed_forms():
    sh, w, dec = _make("tiny")
    # zero output head -> uniform distribution
    wz = dict(w); wz[("wlm", -1)] = np.zeros_like(w[("wlm", -1)])
    dz = Decoder(sh.n_layers, sh.d, sh.n_heads, sh.ffn, sh.vocab, wz)
    assert np.all(dz.verify_forward(dz.new_cache(8), [1, 2, 3]) == 0.0)
    # all block weights zero: hidden = rmsnorm(embedding) * gf, logits = that times wlm^T
    wz = {k: (np.zeros_like(v) if k[0] in ("wqkv", "wo", "wgu", "wdown") else v) for k, v in w.items()}
    dz = Decoder(sh.n_layers, sh.d, sh.n_heads, sh.ffn, sh.vocab, wz)
    e = w[("emb", -1)][[5, 9]].astype(np.float64)
    h = e / np.sqrt((e ** 2).mean(-1, keepdims=True) + 1e-6) * w[("gf", -1)]
    assert np.allclose(dz.verify_forward(dz.new_cache(8), [5, 9]), h @ w[("wlm", -1)].T.astype(np.float64),
                       atol=1e-12)
    # rmsnorm of a constant vector c with unit gain is sign(c) (up to eps)
    assert np.allclose(rmsnorm(np.full((1, 8), -3.0), np.ones(8), 0.0), -1.0)
    # silu(0) = 0, silu(x) - silu(-x) = x
    xs = np.linspace(-4, 4, 9)
    assert silu(np.zeros(1))[0] == 0 and np.allclose(silu(xs) - silu(-xs), xs)


def test_rope_properties():
    r = np.random.default_rng(0)
    v = r.standard_normal((5, 3, 16))
    # position 0 is the identity; norms are preserved
    assert np.array_equal(rope(v, np.zeros(5, dtype=np.int64), 10000.0), v)
    out = rope(v, np.arange(5) + 100, 10000.0)
    assert np.allclose(np.linalg.norm(out, axis=-1), np.linalg.norm(v, axis=-1))
    # scores depend on the position difference only
    q, k = r.standard_normal((1, 1, 16)), r.standard_normal((1, 1, 16))
    s1 = (rope(q, np.array([7]), 10000.0) * rope(k, np.array([3]), 10000.0)).sum()
    s2 = (rope(q, np.array([1007]), 10000.0) * rope(k, np.array([1003]), 10000.0)).sum()
    assert abs(s1 - s2) < 1e-9
    # first pair (elements 0 and dh/2) turns by exactly pos radians; last pair by pos * base^(-(dh-2)/dh)
    e0 = np.zeros((1, 1, 16)); e0[0, 0, 0] = 1.0
    o = rope(e0, np.array([2]), 10000.0)[0, 0]
    assert np.isclose(o[0], np.cos(2.0)) and np.isclose(o[8], np.sin(2.0))
    e7 = np.zeros((1, 1, 16)); e7[0, 0, 7] = 1.0
    o = rope(e7, np.array([2]), 10000.0)[0, 0]
    ang = 2.0 * 10000.0 ** (-14 / 16)
    assert np.isclose(o[7], np.cos(ang)) and np.isclose(o[15], np.sin(ang))


def test_float32_mode_close_to_float64():
    sh, w, dec64 = _make("tiny")
    dec32 = Decoder(sh.n_layers, sh.d, sh.n_heads, sh.ffn, sh.vocab, w, dtype=np.float32)
    toks = synth.uniform_tokens(4, 1, 0, 12, sh.vocab).tolist()
    a = dec64.verify_forward(dec64.new_cache(16), toks)
    b = dec32.verify_forward(dec32.new_cache(16), toks)
    assert b.dtype == np.float32 and np.abs(a - b).max() < 1e-4
