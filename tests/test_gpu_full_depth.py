"""GPU parity at the FULL depth of the 7B shape (32 layers): logits of laser_verify_step against the float64
oracle's, accepted lengths and emitted tokens against its decisions.

The oracle cannot run a 32-layer 7B forward inside a GPU test (26 GB of host weights, a quarter of an hour),
so its results were written once by tests/golden/make_full_depth.py, which calls only oracle/ and synth/,
into tests/golden/full_depth_7b.npz: every fourth logit column and the 64 largest logits of every row, the
accepted length, the emitted tokens and the deciding margins. Two cases: the latency configuration itself
(one sequence, context 1024, K = 8; both the persistent kernel and the general path), a 108-row batch on
the tiled many-row path (the oracle follows two of its twelve sequences) and a 54-row batch on the 17..80-row
path (two of six sequences)."""
import os

import numpy as np
import pytest
import torch

import synth
from synth.model import torch_gen_weight
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "full_depth_7b.npz")


@pytest.fixture(scope="module")
def weights_7b():
    from paper_2408_05676_amd.harness import stacked_weights
    sh = synth.SHAPES["7b"]
    w = stacked_weights(lambda n, l: torch_gen_weight(sh, n, l, "cuda"), sh)
    yield w
    del w
    torch.cuda.empty_cache()


def _case(name):
    g = np.load(GOLDEN)
    return {k[len(name) + 1:]: g[k] for k in g.files if k.startswith(name + "_")}, g["params"]


def _check(name, weights, fused, options=()):
    import paper_2408_05676_amd as laser
    from paper_2408_05676_amd.harness import Engine
    c, params = _case(name)
    k, p, mode = int(params[0]), float(params[1]), int(params[2])
    sh = synth.SHAPES["7b"]
    B, ctx, K = (int(v) for v in c["shape"])
    follow = c["follow"].tolist()
    eng = Engine(sh, weights, B, K, ctx + 4 * (K + 1), 3)
    eng.model.set_option("fused", fused)
    for o, v in options:
        eng.model.set_option(o, v)
    eng.prefill(c["prompts"])
    eng.drafts.copy_(torch.as_tensor(c["drafts"]))
    eng.draft_len.copy_(torch.as_tensor(c["draft_len"]))
    acc, out, logits = laser.verify_step(eng.model, eng.kv, eng.seq_ids, eng.pending, eng.drafts, eng.draft_len,
                                         k, p, mode, want_logits=True)
    torch.cuda.synchronize()
    lg = logits[follow].cpu().numpy().astype(np.float64)             # [followed][R][V]
    worst, rms = 0.0, []
    for got, want in ((lg[..., c["cols"]], c["logits_cols"].astype(np.float64)),
                      (np.take_along_axis(lg, c["top_idx"].astype(np.int64), axis=-1), c["top_val"].astype(np.float64))):
        err = np.abs(got - want)
        # the stored values are float32 roundings of the oracle's: half a unit in the last place of slack
        bound = gu.ATOL + gu.RTOL * np.abs(want) + np.abs(want) * 2.0 ** -24
        worst = max(worst, float((err / bound).max()))
        rms.append(float(np.sqrt((err ** 2).mean())))
    assert worst <= 1.0, f"{name} fused={fused}: logits {worst:.2f}x the bound"
    acc_g, out_g = acc.cpu().numpy()[follow], out.cpu().numpy()[follow]
    flips = 0
    for i in range(len(follow)):
        a_o, a_g = int(c["accept_len"][i]), int(acc_g[i])
        if a_o == a_g and out_g[i].tolist() == c["out_tokens"][i].tolist():
            continue
        row = min(a_o, a_g)
        tol = 3.0 * (gu.ATOL + gu.RTOL * float(c["row_absmax"][i, row]))
        margin = min(c["rank_margin"][i, row], c["logq_margin"][i, row] / 2.0) if a_o != a_g else c["argmax_gap"][i]
        assert margin <= tol, f"{name} fused={fused} sequence {follow[i]}: decision differs outside tolerance ({a_o} vs {a_g}, margin {margin})"
        flips += 1
    print(f"[7b 32 layers, {name}: B={B} ctx={ctx} K={K} fused={fused} {dict(options)}] worst logit error {worst:.3f} of bound "
          f"(rms {rms[0]:.5f}), accepted {acc_g.tolist()} (oracle {c['accept_len'].tolist()}), in-tolerance flips {flips}")
    assert not eng.model.aborted()
    eng.model.close()
    eng.kv.close()


@pytest.mark.parametrize("fused", [1, 0])
def test_latency_configuration_full_depth(weights_7b, fused):
    _check("c3", weights_7b, fused)


@pytest.mark.parametrize("split_ffn", [0, 1])
def test_many_row_path_full_depth(weights_7b, split_ffn):
    """108 rows: tiled matrix-core GEMMs. By default the gate/up product takes single fp16 rows there
    (option split_ffn = 0); both settings must stay inside the tolerance."""
    _check("many", weights_7b, 0, options=(("split_ffn", split_ffn),))


def test_mid_row_path_full_depth(weights_7b):
    """54 rows: the weight-streaming kernels that stage the activation chunk in LDS (four row tiles, reduction
    parts added by the rotary kernel and the norms), the head through the same kernel plus row statistics."""
    _check("mid", weights_7b, 0)
