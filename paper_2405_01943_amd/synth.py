"""Seeded synthetic inputs shaped like the paper's calibration workload.

The paper calibrates on 128 sequences of 2048 C4 tokens run through public
checkpoints (Sec. 4.1); neither is available here, so these generators stand in
for them with the MLP shapes of the model-configuration table (Appendix A.1)
and activation statistics that mimic LLM hidden states (a few outlier channels,
optionally a heavy tail).

This module only draws random numbers and casts them: it holds none of the
method's arithmetic, and is the one piece shared by the GPU tests, the
benchmark and the CPU oracle's callers.  All draws come from torch generators
seeded from (seed, tensor tag, chunk index), so any token chunk can be
regenerated on its own.  CPU and GPU generators give different streams; a
caller that needs identical bits on both sides generates once and copies.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import torch


@dataclass(frozen=True)
class MlpConfig:
    name: str
    d: int                 # d_hidden
    d_int: int             # intermediate width
    tokens: int            # calibration tokens (128 x 2048 for the real shapes)
    dtype: str             # "f32" or "bf16"
    act: str               # "silu" | "gelu_tanh" | "gelu_erf" | "relu"
    chunk: int             # tokens handed to one calibration call
    t_tail: float          # probability that an entry is a Student-t(3) draw
    outlier_frac: float = 0.01
    outlier_scale: float = 20.0
    w_std: float = 0.02
    nm: Tuple[Tuple[int, int], ...] = ((2, 4),)   # (n_keep, m) patterns exercised
    unstructured: Optional[float] = None          # sparsity of the unstructured variant
    alpha_gate_up: float = 0.5                    # Eq. 4 exponent
    alpha_down: float = 1.0                       # Eq. 5 exponent
    dead_frac: float = 0.0                        # share of neurons whose Gate-Proj row is all zero

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def n_outlier(self) -> int:
        return max(1, round(self.outlier_frac * self.d))


CONFIGS = {
    c.name: c
    for c in [
        MlpConfig("tiny", 256, 688, 512, "f32", "silu", 512, 0.0),
        MlpConfig("llama2_7b", 4096, 11008, 262144, "bf16", "silu", 262144, 1e-3,
                  nm=((2, 4), (4, 8))),
        MlpConfig("mistral_7b", 4096, 14336, 262144, "bf16", "silu", 262144, 1e-3,
                  nm=((2, 4),), unstructured=0.5),
        MlpConfig("gemma_7b", 3072, 24576, 262144, "bf16", "gelu_tanh", 262144, 0.0,
                  nm=((4, 8),)),
        MlpConfig("llama2_70b", 8192, 28672, 262144, "bf16", "silu", 32768, 1e-3,
                  nm=((2, 4),)),
        # a sixth shape beside the five benchmark ones: LLaMA2-13B (the appendix table of model configurations)
        MlpConfig("llama2_13b", 5120, 13824, 262144, "bf16", "silu", 262144, 1e-3,
                  nm=((2, 4), (4, 8))),
        # the other GLU variants of Sec. 2.2 at the LLaMA2-7B shape: ReGLU (the ReluLLaMA model of
        # Sec. 4.1; 3 % of its neurons never fire) and GeGLU with the erf form of GELU
        MlpConfig("llama2_7b_reglu", 4096, 11008, 262144, "bf16", "relu", 262144, 1e-3,
                  nm=((2, 4),), unstructured=0.5, dead_frac=0.03),
        MlpConfig("llama2_7b_geglu_erf", 4096, 11008, 262144, "bf16", "gelu_erf", 262144, 1e-3,
                  nm=((4, 8),)),
    ]
}

_TAGS = {"x": 1, "wg": 2, "wu": 3, "wd": 4, "perm": 5, "tail": 6, "norms": 7, "dead": 8}


def _gen(device, seed: int, tag: str, idx: int = 0) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1_000_003 + _TAGS[tag]) * 1_000_003 + int(idx))
    return g


def outlier_channels(cfg: MlpConfig, seed: int = 0) -> torch.Tensor:
    """Indices of the input channels that carry x20 outliers (same on any device)."""
    perm = torch.randperm(cfg.d, generator=_gen("cpu", seed, "perm"))
    return perm[: cfg.n_outlier].sort().values


def dead_neurons(cfg: MlpConfig, seed: int = 0) -> torch.Tensor:
    """Indices of the neurons whose Gate-Proj row is all zero (same on any device); may be empty.

    With such a row the gate is 0 on every token, so the neuron's activation and its norm are
    exactly 0 whatever the activation function: the stand-in for a neuron that never fires.
    """
    n = int(round(cfg.dead_frac * cfg.d_int))
    perm = torch.randperm(cfg.d_int, generator=_gen("cpu", seed, "dead"))
    return perm[:n].sort().values


def make_weight(cfg: MlpConfig, which: str, device, seed: int = 0) -> torch.Tensor:
    """One of 'wg', 'wu' ([d_int, d]) or 'wd' ([d, d_int]), entries N(0, w_std); the Gate-Proj
    rows of the config's dead neurons are zero."""
    shape = (cfg.d_int, cfg.d) if which in ("wg", "wu") else (cfg.d, cfg.d_int)
    w = torch.randn(shape, generator=_gen(device, seed, which), device=device,
                    dtype=torch.float32)
    if which == "wg" and cfg.dead_frac > 0.0:
        w[dead_neurons(cfg, seed).to(device)] = 0.0
    return (w * cfg.w_std).to(cfg.torch_dtype)


def make_x(cfg: MlpConfig, chunk_idx: int, n_tokens: int, device, seed: int = 0) -> torch.Tensor:
    """Token chunk ``chunk_idx`` of the calibration activations, [n_tokens, d].

    N(0,1) entries; with probability ``t_tail`` an entry is replaced by a
    Student-t draw with 3 degrees of freedom; then the outlier channels are
    multiplied by ``outlier_scale``; then the cast to the config's dtype.
    """
    x = torch.randn((n_tokens, cfg.d), generator=_gen(device, seed, "x", chunk_idx),
                    device=device, dtype=torch.float32)
    if cfg.t_tail > 0.0:
        gt = _gen(device, seed, "tail", chunk_idx)
        sel = torch.rand((n_tokens, cfg.d), generator=gt, device=device) < cfg.t_tail
        k = int(sel.sum().item())
        z = torch.randn((k,), generator=gt, device=device)
        chi2 = torch.randn((k, 3), generator=gt, device=device).square().sum(dim=1)
        x[sel] = z / torch.sqrt(chi2 / 3.0)
        del sel
    ch = outlier_channels(cfg, seed).to(device)
    x[:, ch] *= cfg.outlier_scale
    return x.to(cfg.torch_dtype)


def make_norms(n: int, device, seed: int = 0, idx: int = 0) -> torch.Tensor:
    """A positive float32 vector with the spread of activation norms (log-normal)."""
    z = torch.randn((n,), generator=_gen(device, seed, "norms", idx), device=device)
    return torch.exp(0.7 * z + 3.0).to(torch.float32)
