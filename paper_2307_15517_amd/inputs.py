"""Seeded synthetic inputs shaped like the linear layers of the LLMs the paper evaluates.

This module holds no MXInt arithmetic: it only draws float32 tensors with
``numpy.random.default_rng(seed)``.  The tensors take the shapes of OPT-125M /
LLaMA-7B / LLaMA-13B linear layers and the heavy-tailed, outlier-channel
structure the paper reports for LLM activations (Section 2, Fig. 1a); they
stand in for the paper's models and datasets, which are not used here.

Each generator returns ``(x, wt)``: activations ``x`` [M, K] and weights ``wt``
[N, K] (one row per output feature, K contiguous, like ``torch.nn.Linear``).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np


@dataclass(frozen=True)
class LinearCase:
    """One linear layer of a workload: shapes plus the MXInt formats of both operands."""
    name: str
    M: int
    K: int
    N: int
    block: int
    wx: int          # stored bits per activation element, sign included
    ww: int          # stored bits per weight element, sign included
    act: str         # activation recipe, see activations()
    seed: int = 0


def weights(rng: np.random.Generator, N: int, K: int, std: float = 0.02) -> np.ndarray:
    """Gaussian weights, standard deviation ``std``."""
    return (rng.standard_normal((N, K)) * std).astype(np.float32)


def activations(rng: np.random.Generator, M: int, K: int, recipe: str) -> np.ndarray:
    """Activation recipes:

    "normal"            N(0,1)
    "normal_out6x50"    N(0,1), six feature channels (columns) scaled by 50
    "t3_out1pct_x100"   Student-t with 3 degrees of freedom, 1 % of the channels scaled by 100
    "normal_out1pct_x50" N(0,1), 1 % of the channels (at least one) scaled by 50
    """
    if recipe == "normal":
        x = rng.standard_normal((M, K))
    elif recipe == "normal_out6x50":
        x = rng.standard_normal((M, K))
        ch = rng.choice(K, 6, replace=False)
        x[:, ch] *= 50.0
    elif recipe == "t3_out1pct_x100":
        x = rng.standard_t(3, size=(M, K))
        ch = rng.choice(K, max(1, round(0.01 * K)), replace=False)
        x[:, ch] *= 100.0
    elif recipe == "normal_out1pct_x50":
        x = rng.standard_normal((M, K))
        ch = rng.choice(K, max(1, round(0.01 * K)), replace=False)
        x[:, ch] *= 50.0
    else:
        raise ValueError(recipe)
    return x.astype(np.float32)


def make(case: LinearCase, M: int | None = None) -> Tuple[np.ndarray, np.ndarray]:
    """Draw (x [M,K], wt [N,K]) for a case; ``M`` overrides the case's row count."""
    rng = np.random.default_rng(case.seed)
    m = case.M if M is None else M
    x = activations(rng, m, case.K, case.act)
    wt = weights(rng, case.N, case.K)
    return x, wt


def single_linear() -> List[LinearCase]:
    """One 768x768 linear on 16 tokens: block 16, activations 8 bits, weights 4 bits."""
    return [LinearCase("single_768x768", 16, 768, 768, 16, 8, 4, "normal", 0)]


def opt125m_layer(M: int = 128) -> List[LinearCase]:
    """The four linears of an OPT-125M decoder layer at sequence length 128."""
    f = dict(block=16, wx=6, ww=4, act="normal_out6x50")
    return [LinearCase("opt125m_qkv", M, 768, 2304, seed=1, **f),
            LinearCase("opt125m_out", M, 768, 768, seed=2, **f),
            LinearCase("opt125m_fc1", M, 768, 3072, seed=3, **f),
            LinearCase("opt125m_fc2", M, 3072, 768, seed=4, **f)]


def llama7b_prefill(M: int = 2048) -> List[LinearCase]:
    """LLaMA-7B linears on a 2048-token prefill: q/k/v/o, gate/up, down."""
    f = dict(block=32, wx=8, ww=4, act="t3_out1pct_x100")
    return [LinearCase("llama7b_qkvo", M, 4096, 4096, seed=10, **f),
            LinearCase("llama7b_gate_up", M, 4096, 11008, seed=11, **f),
            LinearCase("llama7b_down", M, 11008, 4096, seed=12, **f)]


def llama13b_decode(M: int = 1) -> List[LinearCase]:
    """LLaMA-13B linears on M decode tokens (M in 1, 4, 8): 4-bit weights, block 16."""
    f = dict(block=16, wx=8, ww=4, act="normal")
    return [LinearCase("llama13b_qkvo", M, 5120, 5120, seed=20, **f),
            LinearCase("llama13b_gate_up", M, 5120, 13824, seed=21, **f),
            LinearCase("llama13b_down", M, 13824, 5120, seed=22, **f)]


def attention_widths(seed: int) -> Tuple[int, int, int, int]:
    """Per-tensor stored widths (Q, K, P, V) drawn uniformly from 2..8 (Fig. 1b motivates the spread)."""
    rng = np.random.default_rng(seed)
    w = rng.integers(2, 9, size=4)
    return int(w[0]), int(w[1]), int(w[2]), int(w[3])


def attention_qkv(seed: int, heads: int = 32, seq: int = 2048, dim: int = 128):
    """Q, K, V float32 [heads, seq, dim], N(0,1) with 1 % of the dim channels (at least one) x50."""
    rng = np.random.default_rng(1000 + seed)
    out = []
    for _ in range(3):
        t = rng.standard_normal((heads, seq, dim))
        ch = rng.choice(dim, max(1, round(0.01 * dim)), replace=False)
        t[:, :, ch] *= 50.0
        out.append(t.astype(np.float32))
    return tuple(out)
