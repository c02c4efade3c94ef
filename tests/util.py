"""Shared test plumbing: turn synthetic torch inputs into the oracle's containers."""
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import esp_oracle as O  # noqa: E402
from paper_2603_17942_amd import synth  # noqa: E402


def to_np(t):
    return t.detach().to("cpu", torch.float32).numpy().astype(np.float64) if t.is_floating_point() \
        else t.detach().cpu().numpy()


def oracle_model(shape: synth.ModelShape, weights: dict, layers=None) -> O.Model:
    """Oracle Model over the same weight values (held as float64 arrays)."""
    n_layers = shape.n_layers if layers is None else layers
    w = {"embed": to_np(weights["embed"]), "lm_head": to_np(weights["lm_head"]),
         "final_norm": to_np(weights["final_norm"]),
         "layers": [{k: to_np(v) for k, v in weights["layers"][l].items()} for l in range(n_layers)]}
    return O.Model(n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                   shape.d_ff, shape.vocab, shape.rope_theta, shape.rms_eps, shape.qk_norm, w)


def small_shape(**kw) -> synth.ModelShape:
    base = dict(name="unit", n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16,
                d_ff=96, vocab=211, rope_theta=1.0e4, rms_eps=1.0e-5, qk_norm=False, dtype="f32")
    base.update(kw)
    return synth.ModelShape(**base)


def read_golden(path):
    """Golden text fixture: '#' lines are comments/citations; other lines are
    whitespace-separated fields."""
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            rows.append(line.split())
    return rows
