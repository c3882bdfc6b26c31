#!/usr/bin/env python3
"""Benchmark of the retrieve -> verify -> accept -> commit step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3|c4|7b_b8|1b|tiny|stress]
    python bench.py --study [--study-shape 1b|7b|tiny]     # generation loop: pooling schemes, pool sizes, acceptance rules

A "step" is one pass of the whole hot path over the batch: laser_retrieve_drafts,
laser_verify_step (embedding .. fused head + acceptance), laser_kv_commit, laser_ctx_advance.
All inputs are resident in HBM before the timed region. Prints ONE JSON line.

Workload (seeded, synthetic): random-init weights of the named shape; contexts and pools from the
template + substitution recipe; the pool additionally holds a noisy copy of the model's own greedy
continuation of each benchmark context (the paper builds its pools from the same model's earlier
outputs), so that drafts are accepted in multi-token chunks that break where the copy was
substituted. `value` counts the tokens the step really emitted (accepted drafts + 1 per step).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

WORKLOADS = {
    #        shape  B   ctx   K  pool             n_max  default steps
    "c3": dict(shape="7b", B=1, ctx=1024, K=8, pool="7b_latency", n_max=3, steps=50, warmup=5,
               label="7B shape latency: B=1, context 1024, K=8, pool 2k x 256 tokens (benchmark configuration 2)"),
    "c4": dict(shape="7b", B=64, ctx=512, K=10, pool="7b_throughput", n_max=3, steps=32, warmup=3,
               label="7B shape throughput: B=64, prompt 512 + generated, K=10, paged KV (benchmark configuration 3)"),
    "7b_b8": dict(shape="7b", B=8, ctx=1024, K=8, pool="7b_latency", n_max=3, steps=50, warmup=4,
                  label="7B shape, small batch: B=8, context 1024, K=8 (72 rows: between the latency and the throughput workload)"),
    "1b": dict(shape="1b", B=8, ctx=512, K=8, pool="1b", n_max=3, steps=50, warmup=5,
               label="1B shape: B=8, context 512, K=8 (benchmark configuration 1)"),
    "tiny": dict(shape="tiny", B=2, ctx=64, K=4, pool="tiny", n_max=3, steps=20, warmup=3,
                 label="Tiny: B=2, context 64, K=4 (benchmark configuration 0)"),
}

# Substitution rate of the replayed continuation (the pool texts themselves keep the configs' 10-15 %). The paper
# reports 5.1-8.3 accepted draft tokens per step (its Tab. 3; 6.8-7.5 for the full method) on texts that closely
# repeat the pool; 2 % puts this workload's mean at about 6.5 with K = 8. Measured on the c3 workload: 2 % -> 6.5,
# 3 % -> 5.0, 5 % -> 4.3, 10 % (the pool's own rate) -> 2.9 accepted drafts per step; --regime floor -> 0.
REPLAY_NOISE = 0.02
HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0


def algorithmic_bytes(sh, B, K, ctx_len):
    """Bytes one step must move: every streamed weight once, the cached K/V of every sequence once,
    the new K/V written once."""
    R = K + 1
    w = sh.n_params() * 2
    kv_read = sh.n_layers * B * (ctx_len + R) * sh.d * 2 * 2
    kv_write = sh.n_layers * B * R * sh.d * 2 * 2
    return w + kv_read + kv_write


def host_threads() -> int:
    n = len(os.sched_getaffinity(0))
    env = os.environ.get("OMP_NUM_THREADS")
    return min(n, int(env)) if env and env.isdigit() else n


def cpu_baseline(sh, wl, tokens_per_step, n_sample_layers=4):
    """Time the oracle (as it stands) on a bounded sample of the same step: retrieval on the real
    pool for the batch, `n_sample_layers` decoder layers + final norm + head + acceptance on
    R rows per sequence against a cache of the configured length holding seeded random K/V."""
    import synth
    from oracle import acceptance, retrieval
    from oracle.decoder import Decoder

    B, K, ctx_len = min(wl["B"], 2), wl["K"], wl["ctx"]
    R = K + 1
    Ls = min(n_sample_layers, sh.n_layers)
    weights = {}
    for l in range(Ls):
        for n in ("wqkv", "wo", "wgu", "wdown", "g1", "g2"):
            weights[(n, l)] = synth.gen_weight(sh, n, l)
    for n in ("emb", "wlm", "gf"):
        weights[(n, -1)] = synth.gen_weight(sh, n)
    dec = Decoder(Ls, sh.d, sh.n_heads, sh.ffn, sh.vocab, weights, sh.eps, sh.rope_base)
    caches = []
    for b in range(B):
        c = dec.new_cache(ctx_len + R)
        n = Ls * (ctx_len - 1) * sh.d
        c.k[:, :ctx_len - 1] = synth.approx_normal_f32(7, 900 + b, 0, n, 1.3).reshape(Ls, ctx_len - 1, sh.n_heads, sh.head_dim)
        c.v[:, :ctx_len - 1] = synth.approx_normal_f32(7, 950 + b, 0, n, 1.3).reshape(Ls, ctx_len - 1, sh.n_heads, sh.head_dim)
        c.length = ctx_len - 1
        caches.append(c)
    spec = synth.POOLS[wl["pool"]]
    pool = synth.gen_pool(spec)
    opool = retrieval.RegroupedPool(pool["tokens"], pool["seq_off"], pool["seq_key"])
    ctx = synth.gen_contexts(spec, B, ctx_len, wl["n_max"], salt=1, min_remaining=K)
    rows = synth.uniform_tokens(11, 1, 0, B * R, sh.vocab).reshape(B, R)

    # repeat the sample until about 12 s of oracle time have been spent (at least once, at most 8 times)
    t_retr = t_layers = t_head = 0.0
    reps = 0
    while reps < 8 and (reps == 0 or t_retr + t_layers + t_head < 12.0):
        t0 = time.perf_counter()
        drafts, dl, _, _ = retrieval.retrieve(opool, ctx["keys"], ctx["ctx"][:, -wl["n_max"]:], 1, wl["n_max"], K)
        t_retr += time.perf_counter() - t0
        t0 = time.perf_counter()
        hs = [dec.hidden(caches[b], rows[b]) for b in range(B)]
        t_layers += time.perf_counter() - t0
        t0 = time.perf_counter()
        logits = np.stack([dec.head(h) for h in hs])
        acceptance.verify_batch(logits, drafts, dl, 2, 0.1, 0)
        t_head += time.perf_counter() - t0
        for c in caches:
            c.length = ctx_len - 1
        reps += 1
    total_measured = t_retr + t_layers + t_head
    t_retr, t_layers, t_head = t_retr / reps, t_layers / reps, t_head / reps
    scale_b = wl["B"] / B
    est = (t_retr + t_layers * (sh.n_layers / max(Ls, 1)) + t_head) * scale_b
    return {
        "value": wl["B"] * tokens_per_step / est, "unit": "accepted tokens/s", "cores": host_threads(), "kind": "oracle",
        "sample": (f"{B} of {wl['B']} sequences, {Ls} of {sh.n_layers} layers + head + retrieval + acceptance, "
                   f"float64 numpy, mean of {reps} repetitions ({total_measured:.1f} s of oracle time); "
                   f"layer time scaled x{sh.n_layers / max(Ls, 1):g}, batch x{scale_b:g} (extrapolated); "
                   f"tokens/step taken equal to the GPU run's"),
        "est_step_s": est, "measured_s": t_retr + t_layers + t_head,
    }


def run_workload(args, name, steps, warmup, weights_cache):
    """Builds the engine for workload `name`, times `steps` steps and returns (result dict, shape, workload, tokens/step)."""
    import torch
    import synth
    from synth.model import torch_gen_weight
    import paper_2408_05676_amd as laser
    from paper_2408_05676_amd.harness import Engine, stacked_weights

    wl = WORKLOADS[name]
    steps = steps if steps is not None else wl["steps"]
    warmup = warmup if warmup is not None else wl["warmup"]
    B, K, ctx_len, n_max = wl["B"], wl["K"], wl["ctx"], wl["n_max"]
    R = K + 1
    topk, p, mode = (1, -1.0, 0) if args.regime == "strict" else (2, 0.1, 0)
    gain = args.lm_gain if args.lm_gain is not None else (5.0 if args.regime == "rv" else 1.0)
    sh = synth.SHAPES[wl["shape"]].with_(lm_gain=gain)
    dev = "cuda"
    torch.cuda.set_device(0)

    t_setup = time.perf_counter()
    wkey = (wl["shape"], gain)
    if wkey not in weights_cache:
        weights_cache.clear()
        weights_cache[wkey] = stacked_weights(lambda n, l: torch_gen_weight(sh, n, l, dev), sh, dev)
    weights = weights_cache[wkey]
    n_gen = (steps + warmup) * R + 16                       # tokens the replayed continuation must cover
    max_len = ctx_len + 2 * n_gen + R + 32
    own_cap = min(4096, max_len) if args.temp_branch else 0   # temporary branch: the sequence's own text is searched too
    eng = Engine(sh, weights, B, K, max_len, n_max, own_text_cap=own_cap)
    path = "generic" if args.no_fused else args.path
    fused_possible = B * R <= 16 and sh.n_layers > 0
    if not fused_possible:
        path = "generic"
    spec = synth.POOLS[wl["pool"]]
    ctx = synth.gen_contexts(spec, B, ctx_len, n_max, salt=1, min_remaining=K)
    eng.prefill(ctx["ctx"])

    def rollback():
        for b in range(B):
            eng.kv.set_len(b, ctx_len - 1)
        eng.pending.copy_(torch.as_tensor(np.ascontiguousarray(ctx["ctx"][:, -1]), dtype=torch.int32))
        eng.ctx_tail.copy_(torch.as_tensor(np.ascontiguousarray(ctx["ctx"][:, -n_max:]), dtype=torch.int32))
        if eng.own_text is not None:
            t = min(ctx_len, own_cap)
            eng.own_text[:, :t] = torch.as_tensor(np.ascontiguousarray(ctx["ctx"][:, ctx_len - t:]), dtype=torch.int32).cuda()
            eng.own_len.fill_(t)

    # Few-row workloads have two verify paths; time a few steps of each (no pool yet: rows without drafts
    # cost the same) and keep the faster for everything that follows, the replayed continuation included.
    path_ms = {}
    if path == "auto":
        rollback()
        for pname, flag in (("fused", 1), ("generic", 0)):
            eng.model.set_option("fused", flag)
            eng.step(topk, p, mode)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(4):
                eng.step(topk, p, mode)
            torch.cuda.synchronize()
            path_ms[pname] = (time.perf_counter() - t0) * 1e3 / 4
            rollback()
        path = min(path_ms, key=path_ms.get)
    eng.model.set_option("fused", 1 if path == "fused" else 0)
    for kv_ in args.model_option:
        eng.model.set_option(kv_.split("=")[0], int(kv_.split("=")[1]))

    pool_data = synth.gen_pool(spec)
    toks, off, keys = pool_data["tokens"], pool_data["seq_off"], pool_data["seq_key"]
    replay_noise = args.replay_noise if args.replay_noise is not None else REPLAY_NOISE
    ar_tok_s = None
    if args.regime != "floor":
        torch.cuda.synchronize()
        t_ar = time.perf_counter()
        cont = eng.generate_greedy(n_gen)                   # the model's own continuation (HIP path), one token per step
        ar_tok_s = B * n_gen / (time.perf_counter() - t_ar)
        extra = []
        for b in range(B):
            text = np.concatenate([ctx["ctx"][b, -n_max:], cont[b]]).astype(np.int32)
            noisy = synth.noisy_copy(spec.with_(sub_rate=replay_noise), text, salt=b)
            noisy[:n_max] = text[:n_max]
            extra.append(noisy)
        toks = np.concatenate([toks] + extra)
        off = np.concatenate([off, off[-1] + np.cumsum([len(e) for e in extra])]).astype(np.int64)
        keys = np.concatenate([keys, ctx["keys"]]).astype(np.int64)
        rollback()                                          # back to the state after prefill
    pool = laser.Pool(toks, off, keys, n_max)
    eng.set_pool(pool, ctx["keys"])
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t_setup

    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(warmup):
        eng.step(topk, p, mode)
    torch.cuda.synchronize()
    len0 = eng.kv.read_lens(eng.seq_ids).astype(np.int64)
    eng.model.profile_begin(steps * max(sh.n_layers, 1))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        eng.step(topk, p, mode)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gpu_ms = e0.elapsed_time(e1)
    dom_ms, dom_n = eng.model.profile_end()
    len1 = eng.kv.read_lens(eng.seq_ids).astype(np.int64)
    if eng.model.aborted():
        print("bench.py: the persistent kernel reported an aborted wait; results are invalid", file=sys.stderr)
        sys.exit(3)
    emitted = int((len1 - len0).sum())
    elapsed = max(wall, gpu_ms / 1e3)
    tokens_per_step = emitted / (steps * B)
    value = emitted / elapsed

    step_bytes = algorithmic_bytes(sh, B, K, ctx_len + int((len0 - (ctx_len - 1)).mean()))
    M = B * R
    dom_avg_s = dom_ms / 1e3 / max(dom_n, 1)
    if path == "fused":
        # few-row regime: the whole verify step (embedding .. head + acceptance) is ONE persistent kernel
        dom_name, dom_work, bound = "verify_fused_kernel (whole verify step)", step_bytes, "hbm"
    elif M <= 80:
        # dominant kernel: the gate/up projection (largest weight stream of every layer), weight-streaming form
        dom_name, bound = ("gemm_mid_kernel" if M > 16 else "gemm_skinny_kernel") + "<gate/up SwiGLU>", "hbm"
        dom_work = 2 * sh.ffn * sh.d * 2 + M * sh.d * 2 + M * sh.ffn * 2
    else:
        # many rows: the same projection runs as the LDS-tiled matrix-core GEMM and is compute-bound
        dom_name, bound = "gemm_mfma_kernel<gate/up SwiGLU>", "mfma"
        dom_work = 2.0 * M * 2 * sh.ffn * sh.d
    if bound == "hbm":
        peak, unit, achieved = HBM_PEAK_GBS, "GB/s", (dom_work / dom_avg_s / 1e9 if dom_n else 0.0)
        work_key = "bytes_per_launch"
    else:
        peak, unit, achieved = MFMA_F16_PEAK_TFLOPS, "TFLOP/s", (dom_work / dom_avg_s / 1e12 if dom_n else 0.0)
        work_key = "flops_per_launch"
    # measured peaks of this chip in this process (a streaming read / copy over 1 GiB, a register-resident fp16
    # matrix-instruction loop), beside the datasheet peak the fraction is quoted against
    scratch = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    read_gbs, copy_gbs = laser.probe_hbm(scratch, reps=10)
    mfma_tflops = laser.probe_mfma_f16(scratch, reps=5)
    exchange_us = exchange_errs = None
    if path == "fused":                  # what one phase boundary of the persistent kernel costs
        exchange_us, exchange_errs = laser.probe_exchange(scratch, 200)
    del scratch
    measured_peak = max(read_gbs, copy_gbs) if bound == "hbm" else mfma_tflops
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{name}_{path}.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get("bytes_per_launch")
    out = {
        "metric": "accepted tokens/s per verify step (7B shape, bs 1 & 64); % HBM / MFMA peak",
        "value": value, "unit": "accepted tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": elapsed * 1e3 / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights x fp16 activations (two-plane split where single fp16 is too coarse), fp32 accumulate", "data": "synthetic",
        "config": {"workload": wl["label"], "batch": B, "context": ctx_len, "K": K, "regime": args.regime,
                   "topk": topk, "p": p, "lm_gain": gain, "temporary_branch": bool(args.temp_branch), "replay_noise": replay_noise if args.regime != "floor" else None,
                   "tokens_per_step": tokens_per_step, "accepted_drafts_per_step": tokens_per_step - 1.0,
                   # context: the same library decoding one token per step (K = 0), and the floor of this step shape
                   # (no draft ever accepted); the paper reports 3-5x over its own autoregressive decoding on an RTX 4090
                   "autoregressive_tokens_per_s": ar_tok_s,
                   "speedup_vs_autoregressive": (value / ar_tok_s) if ar_tok_s else None,
                   "floor_tokens_per_s": B * steps / elapsed,
                   "gpu_ms_per_step": gpu_ms / steps, "setup_s": setup_s, "path": path, "path_probe_ms": path_ms,
                   "step_algorithmic_GB": step_bytes / 1e9,
                   "step_hbm_frac": step_bytes / (gpu_ms / 1e3 / steps) / 1e9 / HBM_PEAK_GBS},
        "roofline": {"bound": bound, "kernel": dom_name, "achieved": achieved,
                     "peak": peak, "unit": unit, "frac": achieved / peak, "traffic": traffic,
                     work_key: dom_work, "avg_launch_us": dom_avg_s * 1e6, "launches": dom_n,
                     "measured_peak": measured_peak, "frac_of_measured_peak": achieved / measured_peak if measured_peak else None,
                     "measured": {"hbm_read_GBs": read_gbs, "hbm_copy_GBs": copy_gbs, "mfma_f16_TFLOPs": mfma_tflops,
                                  "grid_exchange_us": exchange_us, "grid_exchange_errors": exchange_errs}},
    }
    eng.close()
    pool.close()
    return out, sh, wl, tokens_per_step


def run_stress(args):
    """The stress configuration (benchmark configuration 4): the fused output head + relaxed acceptance at d 4096, vocabulary
    128256, 256 sequences x 16 rows, and the draft lookup over a pool of 100 M tokens in 1 M keyed sub-pools for 4096
    concurrent contexts (suffix length 1..4, K = 16); beside them the floor of an empty kernel of as many wavefronts
    and a lookup batch of 2^20 contexts. One "step" = one lookup batch + one head launch."""
    import torch
    import synth
    from synth.model import torch_gen_weight
    import paper_2408_05676_amd as laser

    dev = "cuda"
    torch.cuda.set_device(0)
    steps = args.steps if args.steps is not None else 10
    warmup = args.warmup if args.warmup is not None else 2
    sh = synth.SHAPES["head128k"]
    B, K = 256, 15
    R = K + 1
    w = torch_gen_weight(sh, "wlm", -1, dev).contiguous()
    model = laser.Model(0, sh.d, sh.n_heads, sh.ffn, sh.vocab, {"wlm": w}, B * R, B, 0)
    g = torch.Generator(device=dev).manual_seed(7)
    # hidden states with a planted direction so that drafts land on both sides of the threshold: h = a * w[t] + noise
    planted = torch.randint(0, sh.vocab, (B, R), generator=g, device=dev)
    noise = torch.randn((B, R, sh.d), generator=g, device=dev) * 0.5
    amp = 5.0 + torch.rand((B, R, 1), generator=g, device=dev) * 9.0
    h = (amp * w[planted].float() + noise).to(torch.float16)
    drafts = planted[:, :K].to(torch.int32).clone()
    wrong = torch.rand((B, K), generator=g, device=dev) < 0.12
    drafts[wrong] = torch.randint(0, sh.vocab, (int(wrong.sum()),), generator=g, device=dev, dtype=torch.int32)
    dl = torch.full((B,), K, dtype=torch.int32, device=dev)
    acc = torch.empty(B, dtype=torch.int32, device=dev)
    out = torch.empty((B, R), dtype=torch.int32, device=dev)

    t0 = time.perf_counter()
    spec = synth.POOLS["stress"]
    pool_data = synth.gen_pool(spec)
    t_gen = time.perf_counter() - t0
    n_max, Kr, Br = 4, 16, 4096
    t0 = time.perf_counter()
    pool = laser.Pool(pool_data["tokens"], pool_data["seq_off"], pool_data["seq_key"], n_max)
    t_build = time.perf_counter() - t0
    ctx = synth.gen_contexts(spec, Br, 8, n_max, salt=5)
    kd = torch.tensor(ctx["keys"].astype(np.int64), device=dev)
    td = torch.tensor(np.ascontiguousarray(ctx["ctx"][:, -n_max:]).astype(np.int32), device=dev)
    rout = laser.retrieve_drafts(pool, kd, td, 1, n_max, Kr, 1)

    def step():
        laser.retrieve_drafts(pool, kd, td, 1, n_max, Kr, 1, out=rout)
        laser.verify_head(model, h, drafts, dl, 2, 0.1, 0, out=(acc, out))

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    t0 = time.perf_counter()
    ev[0].record()
    for _ in range(steps):
        step()
    ev[1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    step_ms = max(wall * 1e3, ev[0].elapsed_time(ev[1])) / steps
    emitted = int((acc + 1).sum())
    ev[2].record()
    for _ in range(steps):
        laser.verify_head(model, h, drafts, dl, 2, 0.1, 0, out=(acc, out))
    ev[3].record()
    torch.cuda.synchronize()
    head_ms = ev[2].elapsed_time(ev[3]) / steps
    ev[0].record()
    for _ in range(50):
        laser.retrieve_drafts(pool, kd, td, 1, n_max, Kr, 1, out=rout)
    ev[1].record()
    torch.cuda.synchronize()
    retr_us = ev[0].elapsed_time(ev[1]) * 1e3 / 50
    floor_us = laser.probe_launch(Br, 200)
    # 2^20 contexts: tails of random pool positions under their sub-pool's key (half of them with a replaced last token,
    # so that shorter suffixes are tried too); positions come from the regrouped token array the library reports
    n_big = 1 << 20
    info = pool.info()
    order = np.argsort(pool_data["seq_key"], kind="stable")
    lens = (pool_data["seq_off"][1:] - pool_data["seq_off"][:-1])[order]
    starts = np.concatenate([[0], np.cumsum(lens)])[:-1]
    r = np.random.default_rng(11)
    seq = r.integers(0, lens.size, size=n_big)
    posn = starts[seq] + np.minimum(r.integers(0, 1 << 30, size=n_big) % np.maximum(lens[seq] - 1, 1), lens[seq] - 1)
    regrouped = np.empty(info["n_tokens"], dtype=np.int32)
    for s0 in range(0, info["n_tokens"], 1 << 24):
        c = min(1 << 24, info["n_tokens"] - s0)
        regrouped[s0:s0 + c] = pool.read_tokens(s0, c)
    idx = posn[:, None] + np.arange(-n_max + 1, 1)[None, :]
    tails = np.where(idx >= starts[seq][:, None], regrouped[np.clip(idx, 0, regrouped.size - 1)], -1).astype(np.int32)
    swap = r.random(n_big) < 0.5
    tails[swap, -1] = r.integers(0, spec.vocab, size=int(swap.sum()))
    kbig = torch.tensor(pool_data["seq_key"][order][seq].astype(np.int64), device=dev)
    tbig = torch.tensor(tails, device=dev)
    big_out = laser.retrieve_drafts(pool, kbig, tbig, 1, n_max, Kr, 1)
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(5):
        laser.retrieve_drafts(pool, kbig, tbig, 1, n_max, Kr, 1, out=big_out)
    ev[1].record()
    torch.cuda.synchronize()
    big_ms = ev[0].elapsed_time(ev[1]) / 5
    hit_big = float((big_out[1] > 0).float().mean())
    flops = 2.0 * B * R * sh.d * sh.vocab
    scratch = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    read_gbs, copy_gbs = laser.probe_hbm(scratch, reps=10)
    mfma_tflops = laser.probe_mfma_f16(scratch, reps=5)
    del scratch
    achieved = flops / (head_ms * 1e-3) / 1e12
    out_json = {
        "metric": "accepted tokens/s per verify step (7B shape, bs 1 & 64); % HBM / MFMA peak",
        "value": emitted / (step_ms * 1e-3), "unit": "accepted tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": step_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights x fp16 hidden states, fp32 accumulate; int32 tokens", "data": "synthetic",
        "config": {"workload": "Retrieval + verify-head stress: pool of 100M tokens over 1M sub-pools, 4096 contexts, suffix 1-4, K=16; "
                               "head d 4096, vocab 128256, 256 sequences x 16 rows (benchmark configuration 4)",
                   "head_rows": B * R, "vocab": sh.vocab, "topk": 2, "p": 0.1, "accepted_drafts_per_sequence": emitted / B - 1.0,
                   "head_ms": head_ms, "retrieval_us_per_4096_lookups": retr_us, "lookups_per_s": Br / (retr_us * 1e-6),
                   "empty_kernel_us_4096_wavefronts": floor_us, "retrieval_over_floor": retr_us / floor_us,
                   "contexts_matched": float((rout[1] > 0).float().mean()),
                   "retrieval_ms_per_2^20_lookups": big_ms, "lookups_per_s_2^20": n_big / (big_ms * 1e-3),
                   "contexts_matched_2^20": hit_big,
                   "pool_tokens": int(info["n_tokens"]), "pool_keys": int(info["n_keys"]), "pool_device_GB": info["device_bytes"] / 1e9,
                   "pool_generate_s": t_gen, "pool_build_s": t_build},
        "roofline": {"bound": "mfma", "kernel": "gemm_mfma_kernel<head epilogue>", "achieved": achieved, "peak": MFMA_F16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / MFMA_F16_PEAK_TFLOPS, "traffic": None, "flops_per_launch": flops,
                     "avg_launch_us": head_ms * 1e3, "launches": steps, "measured_peak": mfma_tflops,
                     "frac_of_measured_peak": achieved / mfma_tflops,
                     "measured": {"hbm_read_GBs": read_gbs, "hbm_copy_GBs": copy_gbs, "mfma_f16_TFLOPs": mfma_tflops}},
    }
    model.close()
    pool.close()
    return out_json


def run_study(args):
    """Generation-loop study on synthetic data, shaped like the paper's pool study (Sec. 2.2), its ablation of pooling
    schemes with and without relaxed verification (Sec. 4.3.1) and of the acceptance rules (Sec. 4.3.2). U users in G
    groups; the text to generate for a user is the model's own greedy continuation of the user's prompt (decoded first,
    one token per step, through laser_generate without a pool); the earlier texts of similar users are m noisy copies
    of it (substitution rate s). Pooling schemes: CRP -- a pool per group holding the copies for its members; GRP --
    one pool for everything; RRP -- same number of pools, every copy in a random one and every user looking in a random
    one. Every run regenerates all texts with laser_generate (retrieve -> verify -> commit on the device)."""
    import torch
    import synth
    from synth.model import torch_gen_weight
    import paper_2408_05676_amd as laser
    from paper_2408_05676_amd.harness import Engine, stacked_weights

    dev = "cuda"
    torch.cuda.set_device(0)
    sh = synth.SHAPES[args.study_shape].with_(lm_gain=5.0 if args.study_shape != "tiny" else 4.0)
    U, G, B, ctx_len, T, K, n_max, m_copies, sub = 32, 8, 8, 96, 96, 8, 3, 4, 0.10
    eos_class = max(1, sh.vocab // 64)                 # tokens below this id end a text (a 1.6 % class: ~64 tokens expected)
    weights = stacked_weights(lambda n, l: torch_gen_weight(sh, n, l, dev), sh, dev)
    eng = Engine(sh, weights, B, 16, ctx_len + T + 64, n_max)          # buffers for up to 16 drafts (the tree run)
    prompts = synth.uniform_tokens(77, 1, 0, U * ctx_len, sh.vocab).reshape(U, ctx_len)
    group = np.arange(U) % G
    r = np.random.default_rng(5)

    def run_all(pool, keys_of_user, topk, p, mode, tree=False, Kd=K, eng=eng, B=B, U=U):
        """regenerate every user's text (the first U users, B at a time on engine eng); returns texts, counters, wall
        seconds, retrieval ms"""
        texts, cnts, secs, rms, bsteps = [], [], 0.0, 0.0, 0
        for u0 in range(0, U, B):
            us = list(range(u0, u0 + B))
            for b in range(B):
                eng.kv.set_len(b, 0)
            eng.prefill(prompts[us])
            kd = torch.tensor(np.asarray([keys_of_user[u] for u in us], dtype=np.int64), device=dev)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            gen, glen, cnt, steps, ms = laser.generate(eng.model, eng.kv, pool, eng.seq_ids, kd, eng.ctx_tail, eng.pending, Kd, 1, topk, p,
                                                       mode, max_new_tokens=T, tree=tree, check_every=4, time_retrieval=pool is not None)
            secs += time.perf_counter() - t0
            rms += ms or 0.0
            bsteps += steps
            texts += [row.tolist() for row in gen.cpu().numpy()]
            cnts += cnt.cpu().numpy().tolist()
        return texts, np.asarray(cnts), secs, rms, bsteps

    ar_texts, _, ar_secs, _, ar_steps = run_all(None, np.zeros(U), 1, -1.0, 0)
    # The reference text is decoded through the SAME launch shape as the runs it is compared with (B x (K + 1) rows, a pool
    # whose only key nobody looks up): one-token-per-step decoding takes other kernels (fewer rows), whose logits differ in
    # the last bits, and a random-init model's text forks at every near-tie.
    nobody = laser.Pool(np.zeros(4, dtype=np.int32), np.array([0, 4], dtype=np.int64), np.array([1 << 40], dtype=np.int64), n_max)
    greedy, _, _, _, _ = run_all(nobody, np.zeros(U), 1, -1.0, 0)
    nobody.close()
    copies = []                                        # (user, noisy text incl. the prompt's last n_max tokens)
    for u in range(U):
        full = np.array(list(prompts[u, -n_max:]) + greedy[u], dtype=np.int32)
        for c in range(m_copies):
            noisy = full.copy()
            hit = r.random(noisy.size) < sub
            hit[:n_max] = False
            noisy[hit] = r.integers(0, sh.vocab, size=int(hit.sum()))
            copies.append((u, noisy))
    distract = [synth.uniform_tokens(78, 2 + i, 0, T, sh.vocab) for i in range(U * m_copies)]     # unrelated texts of the same volume

    def build(scheme, frac=1.0):
        seqs, keys = [], []
        rr = np.random.default_rng(9)
        lookup = {u: int(group[u]) for u in range(U)}
        if scheme == "RRP":
            lookup = {u: int(rr.integers(0, G)) for u in range(U)}
        keep = rr.random(len(copies)) < frac
        for i, (u, t) in enumerate(copies):
            if not keep[i]:
                continue
            seqs.append(t)
            keys.append(0 if scheme == "GRP" else (int(group[u]) if scheme == "CRP" else int(rr.integers(0, G))))
        for i, t in enumerate(distract):
            if rr.random() < frac:
                seqs.append(t)
                keys.append(0 if scheme == "GRP" else i % G)
        if scheme == "GRP":
            lookup = {u: 0 for u in range(U)}
        flat = np.concatenate(seqs).astype(np.int32)
        off = np.cumsum([0] + [len(t) for t in seqs]).astype(np.int64)
        return laser.Pool(flat, off, np.asarray(keys, dtype=np.int64), n_max), lookup, int(flat.size)

    def summarise(name, texts, cnt, secs, rms, bsteps, extra=None):
        n_tok = sum(len([t for t in x if t >= 0]) for x in texts)
        to_eos = [next((i + 1 for i, t in enumerate(x) if 0 <= t < eos_class), len(x)) for x in texts]
        differs = sum(1 for u in range(len(texts)) if texts[u] != greedy[u])
        row = {"run": name, "tokens_per_s": n_tok / secs, "accepted_drafts_per_step": float(cnt[:, 2].sum() / max(cnt[:, 0].sum(), 1)),
               "sequence_steps": int(cnt[:, 0].sum()), "batch_steps": int(bsteps), "ms_per_batch_step": secs * 1e3 / max(bsteps, 1),
               "retrieval_us_per_batch_step": rms * 1e3 / max(bsteps, 1),
               "mean_length_to_eos_class": float(np.mean(to_eos)), "texts_differing_from_greedy": differs}
        row.update(extra or {})
        return row

    rows = [summarise("autoregressive (no pool, one row per sequence)", ar_texts, np.asarray([[T, 0, 0, 0]] * U), ar_secs, 0.0, ar_steps)]
    for scheme in ("GRP", "RRP", "CRP"):
        pool, lookup, n_tok = build(scheme)
        for rule, (topk, p) in (("strict", (1, -1.0)), ("RV", (2, 0.1))):
            res = run_all(pool, lookup, topk, p, 0)
            rows.append(summarise(f"{scheme} {rule}", *res, {"pool_tokens": n_tok}))
        pool.close()
    for frac in (0.125, 0.25, 0.5, 1.0):
        pool, lookup, n_tok = build("CRP", frac)
        res = run_all(pool, lookup, 2, 0.1, 0)
        rows.append(summarise(f"CRP RV pool size x{frac}", *res, {"pool_tokens": n_tok}))
        pool.close()
    pool, lookup, n_tok = build("CRP")
    for name, (topk, p, mode) in (("top-1 (strict)", (1, -1.0, 0)), ("top-k only (k=2)", (2, 0.0, 2)), ("top-p only (p=0.1)", (1, 0.1, 3)),
                                  ("RV (k=2, p=0.1)", (2, 0.1, 0)), ("top-1 or RV", (2, 0.1, 1)), ("top-k only (k=8)", (8, 0.0, 2))):
        rows.append(summarise(f"rule: {name}", *run_all(pool, lookup, topk, p, mode)))
    rows.append(summarise("CRP RV, token trees of 16 nodes", *run_all(pool, lookup, 2, 0.1, 0, tree=True, Kd=16)))
    # One sequence at a time (the latency regime: K + 1 = 9 rows, the persistent few-row kernel for chains and trees
    # alike), the first 8 users: a tree of 8 nodes costs the same rows as a chain of 8 drafts. The reference text was
    # decoded at another launch shape, so "differing" counts near-tie forks of the random-init model here, not errors.
    eng1 = Engine(sh, weights, 1, 16, ctx_len + T + 64, n_max)
    for name, tree in (("B=1, CRP RV, chains of 8 drafts", False), ("B=1, CRP RV, token trees of 8 nodes", True)):
        rows.append(summarise(name, *run_all(pool, lookup, 2, 0.1, 0, tree=tree, Kd=8, eng=eng1, B=1, U=8), {"users": 8}))
    eng1.close()
    pool.close()
    eng.close()
    return {"study": "generation loop on synthetic users (laser_generate)", "shape": sh.name, "users": U, "groups": G, "batch": B,
            "prompt": ctx_len, "new_tokens": T, "K": K, "copies_per_user": m_copies, "copy_substitution_rate": sub,
            "lm_gain": sh.lm_gain, "eos_class_size": eos_class, "rows": rows}


def run_phase_trace(args):
    """Phase table of the persistent few-row kernel (option fused_trace: thread 0 of every workgroup stamps the wall
    clock at phase edges): the latency workload's launch shape (7B width, B = 1, context 1024, K = 8) on a model of
    --trace-layers layers, microseconds per layer averaged over the layers and workgroups."""
    import torch
    import synth
    from paper_2408_05676_amd.harness import Engine, stacked_weights
    from synth.model import torch_gen_weight

    L = args.trace_layers
    sh = synth.SHAPES["7b"].with_(n_layers=L)
    B, K, ctx_len, n_max = 1, 8, 1024, 3
    weights = stacked_weights(lambda n, l: torch_gen_weight(sh, n, l, "cuda"), sh)
    eng = Engine(sh, weights, B, K, ctx_len + 256, n_max)
    ctx = synth.gen_contexts(synth.POOLS["7b_latency"], B, ctx_len, n_max, salt=1, min_remaining=K)
    eng.prefill(ctx["ctx"])
    eng.draft_len.fill_(K)
    eng.drafts.fill_(5)
    for _ in range(3):
        eng.step(2, 0.1, retrieve=False)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        eng.step(2, 0.1, retrieve=False)
    e1.record()
    torch.cuda.synchronize()
    untraced_ms = e0.elapsed_time(e1) / 10
    eng.model.set_option("fused_trace", 1)
    eng.step(2, 0.1, retrieve=False)
    eng.step(2, 0.1, retrieve=False)
    torch.cuda.synchronize()
    tr = eng.model.read_trace().astype(np.float64) / 100.0          # the counter runs at 100 MHz: microseconds
    names = ["qkv", "attention", "o_proj", "gate_up", "down"]
    r1 = lambda x: round(float(x), 1)
    phases = {}
    i = 2
    for n in names:
        body, wait = [], []
        for l in range(L):
            j = i + 10 * l
            body.append(tr[:, j] - tr[:, j - 1])
            wait.append(tr[:, j + 1] - tr[:, j])
        body, wait = np.array(body), np.array(wait)
        phases[n] = {"body_mean": r1(body.mean()), "body_slowest_wg": r1(body.max(axis=1).mean()),
                     "barrier_wait_mean": r1(wait.mean()), "barrier_wait_last_arriver": r1(wait.min(axis=1).mean())}
        i += 2
    fb = 2 * (5 * L + 2) + 4
    for pi, n in enumerate(["qkv", "o_proj", "gate_up", "down"]):
        pre, st, sm, ep = [], [], [], []
        for l in range(L):
            base = 2 + 10 * l + {0: 0, 1: 4, 2: 6, 3: 8}[pi]          # this phase's stamp in front of its barrier
            f = tr[:, fb + 16 * l + 3 * pi: fb + 16 * l + 3 * pi + 3]   # staged, streamed, staging begins
            pre.append(f[:, 2] - tr[:, base - 1])
            st.append(f[:, 0] - f[:, 2])
            sm.append(f[:, 1] - f[:, 0])
            ep.append(tr[:, base] - f[:, 1])
        phases[n].update({"before_staging": r1(np.mean(pre)), "staging_and_ring_fill": r1(np.mean(st)),
                          "streaming": r1(np.mean(sm)), "epilogue": r1(np.mean(ep))})
    i_end = 2 + 10 * L
    out = {"phase_trace": {"layers": L, "launch_shape": "7B width, B=1, context 1024, K=8 (9 rows)", "unit": "us",
                           "untraced_ms_per_step": round(untraced_ms, 4),
                           "per_layer": r1((tr[:, 1 + 10 * L] - tr[:, 1]).mean() / L), "phases": phases,
                           "embedding": r1((tr[:, 0] - tr[:, 0].min()).max() + np.mean(tr[:, 1] - tr[:, 0])),
                           "head_body_slowest_wg": r1((tr[:, i_end] - tr[:, i_end - 1]).max()),
                           "acceptance_slowest_wg": r1((tr[:, i_end + 2] - tr[:, i_end + 1]).max())}}
    eng.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c3", choices=sorted(WORKLOADS) + ["stress"])
    ap.add_argument("--study", action="store_true", help="run the generation-loop study instead of a timed workload (prints one JSON object)")
    ap.add_argument("--study-shape", default="1b", choices=["tiny", "1b", "7b"])
    ap.add_argument("--phase-trace", action="store_true",
                    help="print the persistent few-row kernel's per-phase timing table (one JSON object) instead of a timed workload")
    ap.add_argument("--trace-layers", type=int, default=8, help="layers of the model --phase-trace runs (7B width)")
    ap.add_argument("--regime", default="rv", choices=["rv", "strict", "floor"],
                    help="rv: k=2 p=0.1 (Eq. 8) on a sharpened head; strict: greedy (Eq. 4); floor: no pool replay")
    ap.add_argument("--lm-gain", type=float, default=None)
    ap.add_argument("--replay-noise", type=float, default=None,
                    help="substitution rate of the replayed copy of the model's own continuation that is added to the "
                         "pool (default: the rate that puts the accepted length per step into the band the paper reports)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--model-option", action="append", default=[], metavar="NAME=VALUE",
                    help="laser_model_set_option before the run (tuning knobs such as attn_whole_mult=1)")
    ap.add_argument("--temp-branch", action="store_true",
                    help="search each sequence's own text (prompt + emitted tokens, last 4096) as a temporary branch "
                         "of its pool at every retrieval (laser_retrieve_drafts_temp)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch one plain 1 GiB device copy before the timed region (a kernel of known "
                         "traffic against which hardware byte counters are scaled)")
    ap.add_argument("--path", default="auto", choices=["auto", "fused", "generic"],
                    help="few-row workloads can run the verify step as one persistent kernel (fused) or as the "
                         "general multi-kernel path; auto times a few steps of each and keeps the faster")
    ap.add_argument("--no-fused", action="store_true", help="same as --path generic")
    ap.add_argument("--no-throughput", action="store_true",
                    help="with the default (batch 1) workload, skip the batch-64 workload that is otherwise measured as well")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (sequences are independent, so more GPUs would each run this same "
              "path on their share of the batch, without collectives). "
              "--gpus N with N > 1 is not supported.", file=sys.stderr)
        sys.exit(2)

    if args.study:
        print(json.dumps(run_study(args)))
        return
    if args.phase_trace:
        print(json.dumps(run_phase_trace(args)))
        return
    if args.workload == "stress":
        print(json.dumps(run_stress(args)))
        return
    weights_cache = {}
    out, sh, wl, tokens_per_step = run_workload(args, args.workload, args.steps, args.warmup, weights_cache)
    if args.workload == "c3" and not args.no_throughput:
        # the metric names batch 1 AND batch 64 of the 7B shape: the batch-64 workload runs right after, on the same
        # weights, and is reported inside the same line (`value` stays the batch-1 workload's)
        o4, _, _, _ = run_workload(args, "c4", None, None, weights_cache)
        out["throughput_workload"] = {k: o4[k] for k in ("value", "unit", "steps", "warmup", "ms_per_step", "config", "roofline")}
    weights_cache.clear()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(sh, wl, tokens_per_step)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
