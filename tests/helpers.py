"""Test-side input shaping shared by the oracle pins and the GPU parity tests.

Nothing here is the method's arithmetic: these helpers only rescale the drawn
weights so that a random-init model behaves less degenerately (draft and target
sometimes agree, confidences spread over (0,1)), and define a few small shapes.
"""
from __future__ import annotations

import dataclasses
from typing import Dict

import torch

import synthetic_inputs as si

# small shapes: GQA (4 query heads on 2 KV heads), non-square everywhere
SMALL_GQA = si.ModelShape("small-gqa", 3, 96, 4, 2, 16, 136, 200, "fp32", 1e-6)
SMALL_GQA_BF16 = dataclasses.replace(SMALL_GQA, name="small-gqa-bf16", dtype="bf16", rms_eps=1e-5)
ONE_LAYER = si.ModelShape("one-layer", 1, 48, 4, 2, 12, 80, 64, "fp32", 1e-6)


def shaped_weights(shape: si.ModelShape, seed: int = 0, branch_scale: float = 0.15, head_scale: float = 40.0,
                   gain_jitter: float = 0.1, device="cpu") -> Dict[str, torch.Tensor]:
    """Drawn weights with the sublayer output projections (wo, wd) shrunk and the
    LM head enlarged.  Small branches make a layer-skipping draft agree with the
    target often but not always; a large head spreads the top-1 probability over
    (0,1) so that the confidence threshold actually decides something."""
    w = si.make_weights(shape, seed, device, gain_jitter=gain_jitter)
    for name in list(w):
        if name.endswith(".wo") or name.endswith(".wd"):
            w[name] = (w[name].float() * branch_scale).to(w[name].dtype)
        elif name == "lm_head":
            w[name] = (w[name].float() * head_scale).to(w[name].dtype)
    return w


def rel_err_rowmax(a, b):
    """max_i |a_i - b_i| / max_i |b_i| per row (b is the reference)."""
    import numpy as np
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    if a.ndim == 1:
        a, b = a[None], b[None]
    return np.max(np.abs(a - b), axis=-1) / np.max(np.abs(b), axis=-1)
