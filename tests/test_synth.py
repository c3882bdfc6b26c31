"""The shared input generators: determinism, numpy/torch twins, distribution shape."""
import numpy as np
import torch

import synth
from synth import rng
from synth.model import torch_gen_weight


def test_hash_is_counter_based():
    a = rng.hash_u64(7, 3, 0, 1000)
    b = rng.hash_u64(7, 3, 500, 100)
    assert (a[500:600] == b).all()
    assert (rng.hash_u64(7, 4, 0, 1000) != a).mean() > 0.99
    assert len(set(a.tolist())) == 1000


def test_splitmix_reference_values():
    # splitmix64 finaliser applied to x = 1, computed with python integers
    x = 1
    x ^= x >> 30; x = (x * 0xBF58476D1CE4E5B9) % 2**64
    x ^= x >> 27; x = (x * 0x94D049BB133111EB) % 2**64
    x ^= x >> 31
    assert rng._mix_int(1) == x
    base = rng.stream_base(5, 9)
    assert int(rng.hash_u64(5, 9, 11, 1)[0]) == rng._mix_int(base + 11)


def test_torch_twin_bitwise_equal():
    h = rng.hash_u64(123, 45, 1000, 4096)
    t = rng.torch_hash_i64(123, 45, 1000, 4096, "cpu").numpy().view(np.uint64)
    assert (h == t).all()
    a = rng.approx_normal_f32(9, 2, 77, 5000, 0.02)
    b = rng.torch_approx_normal(9, 2, 77, 5000, 0.02).numpy()
    assert (a.view(np.uint32) == b.view(np.uint32)).all()
    g = rng.approx_normal_f32(9, 2, 0, 500, 0.1, 1.0)
    gt = rng.torch_approx_normal(9, 2, 0, 500, 0.1, 1.0).numpy()
    assert (g.view(np.uint32) == gt.view(np.uint32)).all()


def test_bf16_rounding_matches_torch_and_ties_to_even():
    x = rng.approx_normal_f32(1, 1, 0, 20000, 1.0)
    ours = rng.bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (ours == ref).all()
    # 1 + 2^-8 is exactly halfway between bf16 neighbours 1.0 and 1 + 2^-7: goes to even (1.0)
    assert rng.round_to_bf16_f32(np.array([1.0 + 2.0 ** -8], np.float32))[0] == 1.0
    assert rng.round_to_bf16_f32(np.array([1.0 + 3 * 2.0 ** -8], np.float32))[0] == np.float32(1.0 + 2.0 ** -6)


def test_normal_moments():
    x = rng.approx_normal_f32(3, 3, 0, 400000, 0.02).astype(np.float64)
    assert abs(x.mean()) < 2e-4
    assert abs(x.std() - 0.02) < 2e-4
    assert np.abs(x).max() < 0.02 * 3.47


def test_weights_slices_and_torch_twin():
    sh = synth.SHAPES["tiny"]
    full = synth.gen_weight(sh, "wgu", 1)
    part = synth.gen_weight(sh, "wgu", 1, row0=100, rows=7)
    assert full.shape == (2 * sh.ffn, sh.d)
    assert (full[100:107] == part).all()
    t = torch_gen_weight(sh, "wgu", 1).to(torch.float32).numpy()
    assert (t == full).all()
    assert (synth.round_to_bf16_f32(full) == full).all()
    g = synth.gen_weight(sh, "g1", 0)
    assert abs(g.mean() - 1) < 0.03 and g.std() > 0.05
    assert (torch_gen_weight(sh, "g1", 0).numpy() == g).all()
    sh2 = sh.with_(lm_gain=3.0)
    assert np.allclose(synth.gen_weight(sh2, "gf"), 3.0 * synth.gen_weight(sh, "gf"))


def test_pool_recipe_shape():
    spec = synth.POOLS["tiny"]
    pool = synth.gen_pool(spec)
    assert pool["tokens"].size == 500 * 64 and pool["seq_off"][-1] == 500 * 64
    templ = synth.gen_templates(spec)
    same = np.mean([np.mean(pool["tokens"][i * 64:(i + 1) * 64] == templ[pool["seq_template"][i]])
                    for i in range(500)])
    assert 0.87 < same < 0.93                      # 10 % substitution
    c = synth.gen_contexts(spec, 16, 64, 3)
    assert c["ctx"].shape == (16, 64) and (c["cut"] >= 3).all()
    b = 0
    cut = int(c["cut"][b])
    tail = c["ctx"][b, 64 - cut:]
    assert np.mean(tail == templ[c["template"][b], :cut]) > 0.6


def test_pool_zipf_and_lognormal():
    spec = synth.POOLS["stress"].with_(n_seq=20000, n_keys=20000)
    pool = synth.gen_pool(spec)
    lens = np.diff(pool["seq_off"])
    assert lens.min() >= 8 and lens.max() <= 8192 and 80 < lens.mean() < 120
    z = synth.POOLS["7b_throughput"]
    pz = synth.gen_pool(z)
    top = np.bincount(pz["seq_rank"]).max() / z.n_seq
    assert 0.05 < top < 0.3                        # Zipf(1.1) over 10k keys: head key ~ 13 %
