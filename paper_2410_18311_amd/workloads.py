"""Seeded synthetic inputs shaped like the paper's OPT / Llama FFN workloads.

This module holds NO arithmetic of the method: it only draws tensors.  Both the
HIP path and the CPU oracle are fed from here (the tests hand the same tensors
to each side), so that neither side ever produces the other's inputs.

The paper measures on trained OPT / Llama checkpoints and text datasets
(Sec. 5, "Models", "Tasks"); neither is available offline, so i.i.d. Gaussian
tensors with the real layer shapes, dtypes, prompt lengths and keep fractions
stand in for them.  Bytes moved per decode token are identical to the real
models'; which neurons win the selection is not.
"""

from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, Optional, Tuple

import numpy as np
import torch

TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
WEIGHT_STD = 0.02


@dataclass(frozen=True)
class Workload:
    name: str
    act: str                 # "relu" (OPT) or "swiglu" (Llama)
    dtype: str               # "f32" | "f16" | "bf16"
    d: int                   # d_model
    N: int                   # d_ff, the number of neurons per FFN layer
    L: int                   # FFN layers in the stack
    M: int                   # prefill tokens per sentence
    alpha: float             # token-wise keep fraction
    betas: Tuple[float, ...]  # sentence-wise keep fraction(s)
    decode_tokens: int
    sentences: int = 1       # independent sentences decoded together
    b_up: Optional[float] = None   # constant up-projection bias (None: no biases)
    down_layout: str = "out_major"  # "out_major" [d, N] (nn.Linear) | "neuron_major" [N, d]
    x_unit_rms: bool = False  # prefill / decode rows rescaled to RMS 1
    index: int = 0           # enters the seeds

    @property
    def torch_dtype(self):
        return TORCH_DTYPE[self.dtype]

    @property
    def n_mat(self) -> int:
        return 3 if self.act == "swiglu" else 2

    def scaled(self, **kw) -> "Workload":
        """Same recipe at other sizes (used by the parity tests)."""
        return dataclasses.replace(self, **kw)


WORKLOADS: Dict[str, Workload] = {
    w.name: w
    for w in (
        Workload("tiny_relu_f32", "relu", "f32", 256, 1024, 1, 32, 0.2, (0.4,), 16,
                 b_up=-0.02, index=1),
        Workload("opt6.7b_relu_f16", "relu", "f16", 4096, 16384, 32, 256, 0.2, (0.4,), 256,
                 b_up=-0.02, index=2),
        Workload("llama2_7b_swiglu_bf16", "swiglu", "bf16", 4096, 11008, 32, 512, 0.2, (0.4,), 256,
                 x_unit_rms=True, index=3),
        Workload("llama2_13b_swiglu_bf16", "swiglu", "bf16", 5120, 13824, 40, 1024, 0.2,
                 (0.2, 0.3, 0.4, 0.6), 512, x_unit_rms=True, index=4),
        Workload("opt66b_relu_f16_8sent", "relu", "f16", 9216, 36864, 64, 512, 0.2, (0.4,), 128,
                 sentences=8, b_up=-0.02, down_layout="neuron_major", index=5),
    )
}

_TENSOR_ID = {"w_up": 1, "w_gate": 2, "w_down": 3, "x_prefill": 4, "x_decode": 5}


def _seed(w: Workload, layer: int, tensor: str, sentence: int = 0) -> int:
    return ((w.index * 1009 + layer) * 131 + sentence) * 17 + _TENSOR_ID[tensor]


def _randn(shape, seed: int, device, dtype, scale: float = 1.0, unit_rms: bool = False):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    t = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if unit_rms:
        t = t / t.pow(2).mean(dim=-1, keepdim=True).sqrt()
    if scale != 1.0:
        t = t * scale
    return t.to(dtype).contiguous()


def layer_weights(w: Workload, layer: int, device="cpu") -> Dict[str, Optional[torch.Tensor]]:
    """Weights of one FFN layer: N(0, 0.02^2) matrices, constant biases.
    w_up, w_gate: [N, d].  w_down: [d, N] (out_major) or [N, d] (neuron_major)."""
    dt = w.torch_dtype
    out: Dict[str, Optional[torch.Tensor]] = {}
    out["w_up"] = _randn((w.N, w.d), _seed(w, layer, "w_up"), device, dt, WEIGHT_STD)
    out["w_gate"] = (_randn((w.N, w.d), _seed(w, layer, "w_gate"), device, dt, WEIGHT_STD)
                     if w.act == "swiglu" else None)
    down_shape = (w.d, w.N) if w.down_layout == "out_major" else (w.N, w.d)
    out["w_down"] = _randn(down_shape, _seed(w, layer, "w_down"), device, dt, WEIGHT_STD)
    if w.b_up is not None:
        out["b_up"] = torch.full((w.N,), w.b_up, device=device, dtype=torch.float32).to(dt)
        out["b_down"] = torch.zeros((w.d,), device=device, dtype=dt)
    else:
        out["b_up"] = None
        out["b_down"] = None
    return out


def prefill_hidden(w: Workload, layer: int, device="cpu", sentence: int = 0) -> torch.Tensor:
    """[M, d] prefill hidden states fed to this layer (each layer gets its own
    draw: the paper treats layers independently, "for i = 1..L", Sec. 4.1)."""
    return _randn((w.M, w.d), _seed(w, layer, "x_prefill", sentence), device, w.torch_dtype,
                  unit_rms=w.x_unit_rms)


def decode_hidden(w: Workload, layer: int, device="cpu", sentence: int = 0,
                  tokens: Optional[int] = None) -> torch.Tensor:
    """[decode_tokens, d] fresh hidden states for the decode steps."""
    t = w.decode_tokens if tokens is None else tokens
    return _randn((t, w.d), _seed(w, layer, "x_decode", sentence), device, w.torch_dtype,
                  unit_rms=w.x_unit_rms)


def tiny_relu_f32_numpy():
    """The small fp32 configuration exactly as specified: numpy
    default_rng(0), draw order W1, W2, X, decode inputs."""
    w = WORKLOADS["tiny_relu_f32"]
    rng = np.random.default_rng(0)
    w_up = (rng.standard_normal((w.N, w.d)) * WEIGHT_STD).astype(np.float32)
    w_down = (rng.standard_normal((w.d, w.N)) * WEIGHT_STD).astype(np.float32)
    x_prefill = rng.standard_normal((w.M, w.d)).astype(np.float32)
    x_decode = rng.standard_normal((w.decode_tokens, w.d)).astype(np.float32)
    return {
        "w_up": w_up, "w_gate": None, "w_down": w_down,
        "b_up": np.full((w.N,), w.b_up, dtype=np.float32),
        "b_down": np.zeros((w.d,), dtype=np.float32),
        "x_prefill": x_prefill, "x_decode": x_decode,
    }


def activation_like(M: int, N: int, seed: int, kind: str = "relu", levels: int = 0) -> np.ndarray:
    """A synthetic fp32 activation matrix for selection tests: ``relu`` has
    about half exact zeros, ``abs`` is all positive; ``levels`` > 0 quantises
    values to that many distinct levels to force heavy ties."""
    rng = np.random.default_rng(seed)
    z = rng.standard_normal((M, N)).astype(np.float32)
    if levels > 0:
        z = np.round(z * levels / 4.0).astype(np.float32) * np.float32(4.0 / levels)
    if kind == "relu":
        return np.maximum(z, np.float32(0.0))
    if kind == "abs":
        return np.abs(z)
    if kind == "raw":          # negatives left in: they must never be selected
        return z
    raise ValueError(kind)
