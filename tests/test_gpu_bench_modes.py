"""The measurement tooling itself: bench.py's study and phase-trace modes run (on small shapes) and report figures
that make sense, so that the evidence they produce at full size can be reproduced."""
import importlib
import os
import sys
import types

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    if ROOT not in sys.path:
        sys.path.insert(0, ROOT)
    return importlib.import_module("bench")


def test_study_on_the_tiny_shape_reproduces_greedy_texts_under_strict_verification():
    bench = _bench()
    out = bench.run_study(types.SimpleNamespace(study_shape="tiny"))
    rows = {r["run"]: r for r in out["rows"]}
    assert out["shape"] == "tiny" and len(rows) >= 10
    # strict verification (Eq. 4) regenerates the reference texts exactly, whatever the pool
    for name in ("GRP strict", "CRP strict", "RRP strict"):
        assert rows[name]["texts_differing_from_greedy"] == 0, name
    # a keyed pool that holds the users' texts accepts more than a randomly grouped one (Sec. 4.3.1)
    assert rows["CRP strict"]["accepted_drafts_per_step"] > rows["RRP strict"]["accepted_drafts_per_step"]
    # the pool-size sweep does not lose acceptance as the pool grows (Sec. 2.2)
    sweep = [r["accepted_drafts_per_step"] for n, r in rows.items() if n.startswith("CRP RV pool size")]
    assert len(sweep) == 4 and sweep[-1] >= sweep[0]
    for r in out["rows"]:
        assert r["tokens_per_s"] > 0 and r["batch_steps"] > 0


def test_phase_trace_of_a_one_layer_model_adds_up():
    bench = _bench()
    out = bench.run_phase_trace(types.SimpleNamespace(trace_layers=1))["phase_trace"]
    assert out["layers"] == 1 and set(out["phases"]) == {"qkv", "attention", "o_proj", "gate_up", "down"}
    total = sum(p["body_mean"] + p["barrier_wait_mean"] for p in out["phases"].values())
    print(f"[trace] one layer: {out['per_layer']:.1f} us, phases sum {total:.1f} us, untraced step {out['untraced_ms_per_step']:.3f} ms")
    assert 20.0 < out["per_layer"] < 1000.0
    assert abs(total - out["per_layer"]) < 0.25 * out["per_layer"] + 5.0
    for name in ("qkv", "o_proj", "gate_up", "down"):
        p = out["phases"][name]
        assert p["streaming"] > 0 and p["staging_and_ring_fill"] > 0
