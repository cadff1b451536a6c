"""Seeded synthetic inputs: model shapes, weights, prompts and skip masks.

This module is shared by the CPU oracle's tests and by the HIP library's
tests and benchmark.  It holds none of the decoding method's arithmetic: it
only draws numbers.  Both sides receive the *same bytes* from here.

The paper evaluates trained LLaMA-2 / CodeLLaMA checkpoints on public text
datasets (Section 5.1, Appendix B.1).  Neither is available offline, so the
workloads here are random-init stand-ins of the same architecture and sizes:
matrices ~ N(0, 0.02^2), RMSNorm gains = 1, token ids uniform over the vocab.

Generator: counter-based.  Element i of tensor number t under seed s is a
pure function of (s, t, i), so tensors can be drawn in any order, in chunks
and on any device:
    key  = mix64(mix64(s) + t)
    h    = mix64(key + i)                      (mix64 = splitmix64 finaliser
                                                applied to x + golden-gamma)
    u1   = (top 32 bits of h + 0.5) / 2^32 ,  u2 = (low 32 bits + 0.5) / 2^32
    z    = sqrt(-2 ln u1) * cos(2 pi u2)       (Box-Muller, float64)
    w    = float32(0.02 * z)  [-> bf16 by round-to-nearest-even if asked]
The integer part is bit-exact on every device; the float64 transcendental
part may differ in the last ulp between a CPU and a GPU build of torch, which
is why every test feeds one drawn buffer to both sides instead of drawing
twice.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Iterator, List, Tuple

import numpy as np
import torch

_M64 = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _s64(v: int) -> int:
    """Python int -> the signed 64-bit value with the same bit pattern."""
    v &= _M64
    return v - (1 << 64) if v >= (1 << 63) else v


def mix64(x: int) -> int:
    """splitmix64 output function of (x + gamma), on Python ints."""
    z = (x + _GAMMA) & _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def _mix64_t(x: torch.Tensor) -> torch.Tensor:
    """mix64 on an int64 tensor (two's-complement wrap-around arithmetic)."""
    z = x + _s64(_GAMMA)
    z = (z ^ ((z >> 30) & ((1 << 34) - 1))) * _s64(_C1)
    z = (z ^ ((z >> 27) & ((1 << 37) - 1))) * _s64(_C2)
    return z ^ ((z >> 31) & ((1 << 33) - 1))


def tensor_key(seed: int, tensor_id: int) -> int:
    return mix64((mix64(seed) + tensor_id) & _M64)


def normal_tensor(seed: int, tensor_id: int, n: int, std: float = 0.02,
                  dtype: torch.dtype = torch.float32,
                  device: str | torch.device = "cpu",
                  chunk: int = 1 << 24) -> torch.Tensor:
    """n values ~ N(0, std^2) as float32 or bfloat16 (RNE from float32)."""
    out = torch.empty(n, dtype=dtype, device=device)
    key = _s64(tensor_key(seed, tensor_id))
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        idx = torch.arange(lo, hi, dtype=torch.int64, device=device)
        h = _mix64_t(idx + key)
        a = ((h >> 32) & 0xFFFFFFFF).to(torch.float64)
        b = (h & 0xFFFFFFFF).to(torch.float64)
        u1 = (a + 0.5) * (1.0 / 4294967296.0)
        u2 = (b + 0.5) * (1.0 / 4294967296.0)
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(2.0 * np.pi * u2)
        out[lo:hi] = (std * z).to(torch.float32).to(dtype)
    return out


def uniform_ids(seed: int, n: int, vocab: int) -> np.ndarray:
    """n token ids, uniform over [0, vocab) (bias < vocab / 2^31)."""
    key = tensor_key(seed, 0x1D5)
    return np.array([(mix64((key + i) & _M64) >> 33) % vocab for i in range(n)],
                    dtype=np.int32)


# --------------------------------------------------------------------------
# Model shapes
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    dtype: str            # "fp32" or "bf16": storage type of weights and KV
    rms_eps: float
    rope_theta: float = 1.0e4

    def with_layers(self, n_layers: int, name: str | None = None) -> "ModelShape":
        return dataclasses.replace(self, n_layers=n_layers,
                                   name=name or f"{self.name}-L{n_layers}")

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def attn_sublayer_elems(self) -> int:
        return self.hidden * (2 * self.q_dim + 2 * self.kv_dim)

    def mlp_sublayer_elems(self) -> int:
        return 3 * self.hidden * self.ffn

    def elem_bytes(self) -> int:
        return 4 if self.dtype == "fp32" else 2


TINY = ModelShape("tiny", 4, 256, 4, 4, 64, 688, 1024, "fp32", 1e-6)
LLAMA2_7B = ModelShape("llama2-7b", 32, 4096, 32, 32, 128, 11008, 32000, "bf16", 1e-5)
LLAMA2_13B = ModelShape("llama2-13b", 40, 5120, 40, 40, 128, 13824, 32000, "bf16", 1e-5)
LLAMA2_70B = ModelShape("llama2-70b", 80, 8192, 64, 8, 128, 28672, 32000, "bf16", 1e-5)
SHAPES: Dict[str, ModelShape] = {s.name: s for s in (TINY, LLAMA2_7B, LLAMA2_13B, LLAMA2_70B)}


@dataclasses.dataclass(frozen=True)
class Workload:
    """One of the run configurations (shape + prompt + speculation settings)."""
    name: str
    shape: ModelShape
    n_prompt: int
    n_new: int
    n_skip: int           # number of skipped sublayers (ignored for tiny: literal mask)
    max_k: int
    conf_threshold: float
    weight_seed: int = 0
    prompt_seed: int = 1
    mask_seed: int = 2


WORKLOADS: Dict[str, Workload] = {w.name: w for w in (
    Workload("tiny", TINY, 32, 64, 2, 4, 0.8),
    Workload("7b", LLAMA2_7B, 512, 256, 32, 8, 0.8),
    Workload("13b", LLAMA2_13B, 1024, 256, 36, 12, 0.8),
    Workload("7b-long", LLAMA2_7B, 8192, 128, 32, 8, 0.8),
    Workload("70b", LLAMA2_70B, 2048, 128, 80, 8, 0.8),
)}


# --------------------------------------------------------------------------
# Weights
# --------------------------------------------------------------------------
def tensor_specs(shape: ModelShape) -> List[Tuple[str, Tuple[int, ...], str]]:
    """(name, shape, kind) for every tensor, in the fixed drawing order.

    kind is "matrix" (row-major [out][in], N(0, 0.02^2)) or "gain" (ones).
    The position in this list is the tensor number used by the generator.
    """
    H, Q, KV, F, V = shape.hidden, shape.q_dim, shape.kv_dim, shape.ffn, shape.vocab
    specs: List[Tuple[str, Tuple[int, ...], str]] = [("embed", (V, H), "matrix")]
    for l in range(shape.n_layers):
        specs += [
            (f"l{l}.attn_norm", (H,), "gain"),
            (f"l{l}.wq", (Q, H), "matrix"),
            (f"l{l}.wk", (KV, H), "matrix"),
            (f"l{l}.wv", (KV, H), "matrix"),
            (f"l{l}.wo", (H, Q), "matrix"),
            (f"l{l}.mlp_norm", (H,), "gain"),
            (f"l{l}.wg", (F, H), "matrix"),
            (f"l{l}.wu", (F, H), "matrix"),
            (f"l{l}.wd", (H, F), "matrix"),
        ]
    specs += [("final_norm", (H,), "gain"), ("lm_head", (V, H), "matrix")]
    return specs


def iter_weights(shape: ModelShape, seed: int = 0,
                 device: str | torch.device = "cpu",
                 gain_jitter: float = 0.0) -> Iterator[Tuple[str, torch.Tensor]]:
    """Yield (name, tensor) one at a time so that a large model never has to
    sit in memory twice.  Matrices come in the shape's storage dtype; gains are
    always float32.  gain_jitter > 0 draws gains as 1 + N(0, jitter^2) instead
    of exactly one (used by tests so that a dropped gain is visible)."""
    tdt = torch.float32 if shape.dtype == "fp32" else torch.bfloat16
    for tid, (name, shp, kind) in enumerate(tensor_specs(shape)):
        n = int(np.prod(shp))
        if kind == "gain":
            if gain_jitter > 0.0:
                t = 1.0 + normal_tensor(seed, tid, n, gain_jitter, torch.float32, device)
            else:
                t = torch.ones(n, dtype=torch.float32, device=device)
        else:
            t = normal_tensor(seed, tid, n, 0.02, tdt, device)
        yield name, t.reshape(shp)


def make_weights(shape: ModelShape, seed: int = 0, device: str | torch.device = "cpu",
                 gain_jitter: float = 0.0) -> Dict[str, torch.Tensor]:
    return dict(iter_weights(shape, seed, device, gain_jitter))


# --------------------------------------------------------------------------
# Skip masks  (index 2l = attention sublayer of layer l, 2l+1 = its MLP)
# --------------------------------------------------------------------------
def tiny_mask() -> np.ndarray:
    """The literal mask of the tiny workload: attention of layer 1, MLP of layer 2."""
    m = np.zeros(2 * TINY.n_layers, dtype=np.uint8)
    m[2 * 1] = 1
    m[2 * 2 + 1] = 1
    return m


def random_mask(n_layers: int, n_skip: int, seed: int,
                first_layer: int = 2, last_layer: int | None = None) -> np.ndarray:
    """n_skip sublayers chosen uniformly (partial Fisher-Yates) among the
    sublayers of layers first_layer..last_layer inclusive (default: all but the
    first two and last two layers)."""
    if last_layer is None:
        last_layer = n_layers - 3
    cand = [2 * l + s for l in range(first_layer, last_layer + 1) for s in (0, 1)]
    if not 0 <= n_skip <= len(cand):
        raise ValueError("n_skip out of range")
    key = tensor_key(seed, 0x3A5C)
    for i in range(n_skip):
        j = i + mix64((key + i) & _M64) % (len(cand) - i)
        cand[i], cand[j] = cand[j], cand[i]
    m = np.zeros(2 * n_layers, dtype=np.uint8)
    m[cand[:n_skip]] = 1
    return m


def workload_mask(w: Workload) -> np.ndarray:
    if w.shape.name == "tiny":
        return tiny_mask()
    return random_mask(w.shape.n_layers, w.n_skip, w.mask_seed)


def workload_prompt(w: Workload) -> np.ndarray:
    return uniform_ids(w.prompt_seed, w.n_prompt, w.shape.vocab)
