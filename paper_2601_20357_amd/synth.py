"""Seeded synthetic inputs for the TABED hot path (numpy only).

This module holds no step of the method: it only draws the tensors the method
consumes -- the shared LM-head matrix W, the n drafts' last hidden states H for
every in-block position, the target model's logits, and temperatures.  Both the
CPU oracle's tests and the GPU tests/benchmark draw their inputs here, so that
the two sides see the same bytes.

The shapes stand in for the paper's LVLM workloads (LLaMA-vocabulary 68M-class
draft head, larger-vocabulary model families); their datasets and checkpoints
are not used.  Target logits are made *correlated* with one draft's logits by
adding noise to a plain fp32 matrix product of the stored H and W values; that
product is part of the input recipe, not of the method under test.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int
    V: int
    d: int
    n: int
    B: int
    gamma: int
    h: int
    w_dtype: int          # 0 fp32, 1 bf16
    target: str           # recipe for target logits, see make_round()
    rounds: int
    sigma: float = 0.0
    temperature: str = "one"   # "one" | "greedy" | "mixed07"
    switch_every: int = 64     # "switching" recipe: rounds after which the target follows the next draft

    @property
    def M(self) -> int:
        return self.n * self.B


WORKLOADS = {
    "tiny": Workload("tiny", 1, V=1000, d=64, n=2, B=1, gamma=3, h=4, w_dtype=0,
                     target="independent", sigma=2.0, rounds=64),
    "llava": Workload("llava", 2, V=32000, d=768, n=4, B=1, gamma=5, h=8, w_dtype=1,
                      target="draft0", sigma=0.5, rounds=512),
    "serving": Workload("serving", 3, V=32000, d=768, n=4, B=16, gamma=5, h=8, w_dtype=1,
                        target="per_seq_sigma", rounds=256),
    "lvlm": Workload("lvlm", 4, V=152064, d=896, n=4, B=8, gamma=7, h=16, w_dtype=1,
                     target="switching", sigma=0.8, rounds=256),
    "stress": Workload("stress", 5, V=128256, d=2048, n=8, B=64, gamma=5, h=16, w_dtype=1,
                       target="student_t", sigma=0.5, rounds=256, temperature="mixed07"),
}


def scaled(wl: Workload, **kw) -> Workload:
    """Same recipe at other sizes (parity tests shrink V, B, ... to what the oracle finishes in seconds)."""
    return replace(wl, **kw)


# ------------------------------------------------------------------ bf16 storage helpers
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(x: np.ndarray, w_dtype: int) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float32) if w_dtype == 0 else bf16_bits(x)


def as_f32(x: np.ndarray, w_dtype: int) -> np.ndarray:
    """The exact fp32 value of every stored element."""
    return np.ascontiguousarray(x, dtype=np.float32) if w_dtype == 0 else bf16_to_f32(x)


# ------------------------------------------------------------------ generators
def _rng(wl: Workload, k: int) -> np.random.Generator:
    return np.random.default_rng(1000 * wl.cfg_id + k)


def make_lm_head(wl: Workload) -> np.ndarray:
    """W [V,d] ~ N(0, 0.02) in the storage dtype (fp32 array or bf16 bit patterns)."""
    w = _rng(wl, 0).standard_normal((wl.V, wl.d), dtype=np.float32) * np.float32(0.02)
    return _store(w, wl.w_dtype)


def make_temperature(wl: Workload, mode: str | None = None) -> np.ndarray:
    """Per-sequence temperature [B]; 0 marks a greedy row."""
    mode = mode or wl.temperature
    if mode == "one":
        return np.ones(wl.B, dtype=np.float32)
    if mode == "greedy":
        return np.zeros(wl.B, dtype=np.float32)
    if mode == "mixed07":
        t = np.zeros(wl.B, dtype=np.float32)
        t[1::2] = 0.7
        return t
    raise ValueError(mode)


def make_seq_sigma(wl: Workload) -> np.ndarray:
    """Per-sequence target-noise level, fixed for the run ("per_seq_sigma" recipe)."""
    return _rng(wl, 1).uniform(0.2, 1.5, size=wl.B).astype(np.float32)


def matching_draft(wl: Workload, rnd: int) -> int:
    """The draft whose logits the target's are built from in round `rnd`."""
    return (rnd // wl.switch_every) % wl.n if wl.target == "switching" else 0


def make_round(wl: Workload, W: np.ndarray, rnd: int):
    """Inputs of SD round `rnd`.

    Returns (H, target_logits):
      H [gamma+1, B, n, d] storage dtype -- hidden states ~ N(0,1) of the n drafts at every in-block
        position; slot gamma only feeds the recipe of the bonus row's target logits.
      target_logits [B, gamma+1, V] fp32.
    """
    g = _rng(wl, 10 + rnd)
    Hf = g.standard_normal((wl.gamma + 1, wl.B, wl.n, wl.d), dtype=np.float32)
    H = _store(Hf, wl.w_dtype)
    shape = (wl.B, wl.gamma + 1, wl.V)
    if wl.target == "independent":
        return H, (g.standard_normal(shape, dtype=np.float32) * np.float32(wl.sigma))
    jstar = matching_draft(wl, rnd)
    Wf = as_f32(W, wl.w_dtype)
    Hj = as_f32(H, wl.w_dtype)[:, :, jstar, :]                        # [gamma+1, B, d]
    base = np.einsum("ibk,vk->biv", Hj, Wf, optimize=True).astype(np.float32)
    if wl.target == "student_t":
        noise = g.standard_t(3.0, size=shape).astype(np.float32) * np.float32(wl.sigma)
    else:
        noise = g.standard_normal(shape, dtype=np.float32)
        if wl.target == "per_seq_sigma":
            noise *= make_seq_sigma(wl)[:, None, None]
        else:
            noise *= np.float32(wl.sigma)
    return H, np.ascontiguousarray(base + noise, dtype=np.float32)


def make_tree_leaves(wl: Workload, W: np.ndarray, H: np.ndarray, rnd: int, width: int) -> np.ndarray:
    """Target logits after the leaves of a width-`width` token tree: [B, gamma, width-1, V] fp32.

    No model exists to condition on a leaf token, so the row after sibling s of position i follows the recipe of
    the next position's target row (the matching draft's logits at hidden state H[i+1]) with a noise draw of its own.
    """
    S = width - 1
    g = _rng(wl, 500000 + rnd)
    shape = (wl.B, wl.gamma, S, wl.V)
    if wl.target == "independent":
        return g.standard_normal(shape, dtype=np.float32) * np.float32(wl.sigma)
    jstar = matching_draft(wl, rnd)
    Wf = as_f32(W, wl.w_dtype)
    Hj = as_f32(H, wl.w_dtype)[1:, :, jstar, :]                       # [gamma, B, d]: positions 1..gamma
    base = np.einsum("ibk,vk->biv", Hj, Wf, optimize=True).astype(np.float32)     # [B, gamma, V]
    if wl.target == "student_t":
        noise = g.standard_t(3.0, size=shape).astype(np.float32) * np.float32(wl.sigma)
    else:
        noise = g.standard_normal(shape, dtype=np.float32)
        noise *= make_seq_sigma(wl)[:, None, None, None] if wl.target == "per_seq_sigma" else np.float32(wl.sigma)
    return np.ascontiguousarray(base[:, :, None, :] + noise, dtype=np.float32)


# ------------------------------------------------------------------ draft-model body (random weights: latency study)
@dataclass(frozen=True)
class BodyConfig:
    """Shape of the LLaMA-style draft model in front of the LM head (the paper's drafts are 68M / 160M LLaMA models;
    their trained weights are not used here)."""
    layers: int = 2
    d: int = 768
    heads: int = 12
    d_ff: int = 3072
    V: int = 32000
    max_ctx: int = 1024
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5


BODY_68M = BodyConfig()                  # the 68M-class draft: 2 layers of width 768 (Sec. 4.1, Target and Draft Models)
BODY_160M = BodyConfig(layers=12)        # the 160M-class draft: 12 layers of the same width
BODIES = {"68m": BODY_68M, "160m": BODY_160M}


def scaled_body(bc: BodyConfig, d: int, V: int) -> BodyConfig:
    """The same depth at another hidden size and vocabulary: heads of 64, an MLP four times as wide."""
    return replace(bc, d=d, heads=d // 64, d_ff=4 * d, V=V)


def make_body_weights(bc: BodyConfig, seed: int = 0) -> dict:
    """Random weights of the body: matrices ~ N(0, 0.02) as bf16 bit patterns, norm gains 1 + N(0, 0.1) in fp32."""
    g = np.random.default_rng(7000 + seed)
    mat = lambda *shape: bf16_bits(g.standard_normal(shape, dtype=np.float32) * np.float32(0.02))
    gain = lambda: (1.0 + 0.1 * g.standard_normal(bc.d)).astype(np.float32)
    return dict(
        embed=bf16_bits(g.standard_normal((bc.V, bc.d), dtype=np.float32)),
        g_attn=[gain() for _ in range(bc.layers)], wqkv=[mat(3 * bc.d, bc.d) for _ in range(bc.layers)],
        wo=[mat(bc.d, bc.d) for _ in range(bc.layers)], g_mlp=[gain() for _ in range(bc.layers)],
        wgu=[mat(2 * bc.d_ff, bc.d) for _ in range(bc.layers)], wdown=[mat(bc.d, bc.d_ff) for _ in range(bc.layers)],
        g_final=gain())
