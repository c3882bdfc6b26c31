"""Decoder shapes of the benchmark configurations and their seeded random-init weights.

Weight recipe: every matrix entry is an approximately normal variate (see rng.py) of mean 0
and standard deviation 0.02; RMSNorm gains are 1 + 0.1 * variate so that a missing gain is
visible in tests; the final-norm gain is scaled by `lm_gain` (a sharpness knob: with
gain 1 a random-init model never puts more than ~0.3 % probability on any token, so a
probability threshold of 0.1 could not be exercised).  For `wdtype == "bf16"` the values
are rounded to bfloat16 (nearest-even) and that rounded value is what both the oracle and
the GPU path consume.

Layouts are row-major [out_features][in_features]:
    wqkv  [3d][d]   rows 0..d-1 = query, d..2d-1 = key, 2d..3d-1 = value projection
    wo    [d][d]
    wgu   [2F][d]   rows 0..F-1 = gate, F..2F-1 = up projection
    wdown [d][F]
    g1,g2 [d]       pre-attention / pre-FFN RMSNorm gains (float32)
    emb   [V][d]    input embedding;  wlm [V][d] output head (untied);  gf [d] final norm gain
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

from . import rng

SEED_BASE = 0x4C41534552  # "LASER"


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d: int
    n_heads: int
    ffn: int
    vocab: int
    wdtype: str = "bf16"      # "bf16" or "fp32": precision the stored weights are rounded to
    seed: int = SEED_BASE
    lm_gain: float = 1.0
    rope_base: float = 10000.0
    eps: float = 1e-6

    @property
    def head_dim(self) -> int:
        return self.d // self.n_heads

    def with_(self, **kw) -> "ModelShape":
        return replace(self, **kw)

    def n_params(self) -> int:
        per_layer = 4 * self.d * self.d + 3 * self.d * self.ffn
        return self.n_layers * per_layer + self.vocab * self.d  # streamed per step (no emb)


SHAPES = {
    # name            layers   d  heads   ffn   vocab
    "tiny": ModelShape("tiny", 2, 256, 4, 1024, 2048, "bf16", SEED_BASE + 0),
    "tiny128": ModelShape("tiny128", 2, 256, 2, 1024, 2048, "bf16", SEED_BASE + 5),
    "1b": ModelShape("1b", 16, 2048, 16, 5632, 32000, "bf16", SEED_BASE + 1),
    "7b": ModelShape("7b", 32, 4096, 32, 11008, 32000, "bf16", SEED_BASE + 2),
    "head128k": ModelShape("head128k", 0, 4096, 32, 11008, 128256, "bf16", SEED_BASE + 4),
}

_PER_LAYER = ("wqkv", "wo", "wgu", "wdown", "g1", "g2")
_GLOBAL = ("emb", "wlm", "gf")


def weight_names(shape: ModelShape):
    for layer in range(shape.n_layers):
        for n in _PER_LAYER:
            yield n, layer
    for n in _GLOBAL:
        yield n, -1


def weight_dims(shape: ModelShape, name: str):
    d, f, v = shape.d, shape.ffn, shape.vocab
    return {
        "wqkv": (3 * d, d), "wo": (d, d), "wgu": (2 * f, d), "wdown": (d, f),
        "g1": (d,), "g2": (d,), "emb": (v, d), "wlm": (v, d), "gf": (d,),
    }[name]


def _stream(name: str, layer: int) -> int:
    if layer >= 0:
        return 16 * layer + _PER_LAYER.index(name)
    return (1 << 20) + _GLOBAL.index(name)


def _is_gain(name: str) -> bool:
    return name in ("g1", "g2", "gf")


def gen_weight(shape: ModelShape, name: str, layer: int = -1, row0: int = 0, rows: int | None = None
               ) -> np.ndarray:
    """float32 numpy array with the (already rounded) values of one tensor, or of the row
    range [row0, row0+rows) of a matrix -- any slice can be regenerated on its own."""
    dims = weight_dims(shape, name)
    st = _stream(name, layer)
    if _is_gain(name):
        g = rng.approx_normal_f32(shape.seed, st, 0, dims[0], 0.1, 1.0)
        if name == "gf":
            g = g * np.float32(shape.lm_gain)
        return g
    rows = dims[0] - row0 if rows is None else rows
    w = rng.approx_normal_f32(shape.seed, st, row0 * dims[1], rows * dims[1], 0.02)
    if shape.wdtype == "bf16":
        w = rng.round_to_bf16_f32(w)
    return w.reshape(rows, dims[1])


def gen_all_weights(shape: ModelShape) -> dict:
    """{(name, layer): float32 array} for the whole model (small shapes only)."""
    return {(n, l): gen_weight(shape, n, l) for n, l in weight_names(shape)}


def torch_gen_weight(shape: ModelShape, name: str, layer: int = -1, device="cpu", chunk: int = 1 << 26):
    """Same values as gen_weight, as a torch tensor on `device`: bfloat16 for matrices when
    wdtype == "bf16" (float32 otherwise), float32 for gains."""
    import torch

    dims = weight_dims(shape, name)
    st = _stream(name, layer)
    if _is_gain(name):
        g = rng.torch_approx_normal(shape.seed, st, 0, dims[0], 0.1, 1.0, device)
        if name == "gf":
            g = g * float(np.float32(shape.lm_gain))
        return g
    n = dims[0] * dims[1]
    dt = torch.bfloat16 if shape.wdtype == "bf16" else torch.float32
    out = torch.empty(n, dtype=dt, device=device)
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        out[s:s + c] = rng.torch_approx_normal(shape.seed, st, s, c, 0.02, 0.0, device).to(dt)
    return out.reshape(dims)
