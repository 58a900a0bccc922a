"""Seeded synthetic workloads for the capacity-aware MoE layer.

This module only draws random inputs and rounds them to their storage type.  It
holds none of the method's arithmetic (no softmax, no top-k, no capacity rule, no
FFN), so both the CPU oracle's tests and the HIP path may take their inputs from
it without sharing any computation.

The paper evaluates trained MoE models on public evaluation suites; neither the
weights nor the datasets are available here.  These generators stand in for them:
shapes follow the model families the paper names (OLMoE-, Mixtral-, fine-grained-
and decode-shaped layers) and the router bias is skewed so that the peak expert
load reaches several times the mean, as the paper's test-time load analysis
reports (Sec. 3.1, Fig. "expert_capacity"; App. "Layer-wise Expert Load").
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

MODE_NONE, MODE_TOKEN_DROP, MODE_EXPANDED_DROP = 0, 1, 2
SCOPE_LOCAL, SCOPE_GLOBAL, SCOPE_LOCAL_DEVICE, SCOPE_GLOBAL_DEVICE = 0, 1, 2, 3
DTYPE_F32, DTYPE_BF16 = 0, 1

BASE_SEED = 20250305


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape and skew recipe of one layer configuration."""

    name: str
    index: int            # position in the list of configurations (seed offset)
    n_tokens: int
    d_model: int
    n_experts: int
    top_k: int
    d_hidden: int
    device_groups: int    # G simulated expert-parallel devices
    dtype: int            # DTYPE_F32 or DTYPE_BF16 for x, expert weights and y
    skew: str             # "normal", "zipf" or "one_hot"
    skew_param: float     # sigma, Zipf exponent, or the logit offset of the hot expert

    def seed(self, trial: int = 0) -> int:
        return BASE_SEED + 100 * self.index + trial


WORKLOADS = {
    "tiny": Workload("tiny", 1, 128, 64, 8, 2, 128, 1, DTYPE_F32, "normal", 1.0),
    "olmoe": Workload("olmoe", 2, 4096, 2048, 64, 8, 1024, 1, DTYPE_BF16, "zipf", 1.1),
    "mixtral": Workload("mixtral", 3, 8192, 4096, 8, 2, 14336, 4, DTYPE_BF16, "normal", 1.5),
    "finegrained": Workload("finegrained", 4, 16384, 2048, 128, 8, 768, 8, DTYPE_BF16, "zipf", 1.2),
    "decode": Workload("decode", 5, 256, 4096, 64, 6, 1408, 8, DTYPE_BF16, "one_hot", 3.0),
}


def scaled(w: Workload, **changes) -> Workload:
    """A copy of a workload with some sizes replaced (used for reduced parity cases)."""
    return dataclasses.replace(w, **changes)


# ---------------------------------------------------------------------------
# storage-type rounding
# ---------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to the fp32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


class Stored:
    """A tensor in its storage type: `.f32` are the exact values, `.bits` the bf16 patterns (or None)."""

    __slots__ = ("f32", "bits")

    def __init__(self, values_f32: np.ndarray, dtype: int, keep_f32: bool = True):
        if dtype == DTYPE_BF16:
            self.bits = f32_to_bf16_bits(values_f32)
            self.f32 = bf16_bits_to_f32(self.bits) if keep_f32 else None
        else:
            self.bits = None
            self.f32 = np.ascontiguousarray(values_f32, dtype=np.float32)

    def values(self) -> np.ndarray:
        return self.f32 if self.f32 is not None else bf16_bits_to_f32(self.bits)


# ---------------------------------------------------------------------------
# generators
# ---------------------------------------------------------------------------
def _streams(w: Workload, trial: int):
    root = np.random.SeedSequence(w.seed(trial))
    s_x, s_router, s_bias, s_experts = root.spawn(4)
    return s_x, s_router, s_bias, s_experts


def router_bias(w: Workload, trial: int = 0) -> np.ndarray:
    """Per-expert logit bias that produces the load skew of the workload."""
    _, _, s_bias, _ = _streams(w, trial)
    rng = np.random.default_rng(s_bias)
    e = w.n_experts
    if w.skew == "normal":
        b = rng.standard_normal(e) * w.skew_param
    elif w.skew == "zipf":
        ranks = np.arange(1, e + 1, dtype=np.float64)
        p = ranks ** (-w.skew_param)
        p /= p.sum()
        b = np.log(p)[rng.permutation(e)]
    elif w.skew == "one_hot":
        b = np.zeros(e)
        b[int(rng.integers(e))] = w.skew_param
    else:
        raise ValueError(w.skew)
    return b.astype(np.float32)


def tokens(w: Workload, trial: int = 0) -> Stored:
    """x ~ N(0,1), shape [N, d]."""
    s_x, _, _, _ = _streams(w, trial)
    rng = np.random.default_rng(s_x)
    return Stored(rng.standard_normal((w.n_tokens, w.d_model), dtype=np.float32), w.dtype)


def router_weight(w: Workload, trial: int = 0) -> np.ndarray:
    """W_r ~ N(0, 1/d), shape [E, d], always fp32 (router arithmetic is fp32)."""
    _, s_router, _, _ = _streams(w, trial)
    rng = np.random.default_rng(s_router)
    scale = np.float32(1.0 / math.sqrt(w.d_model))
    return rng.standard_normal((w.n_experts, w.d_model), dtype=np.float32) * scale


def expert_weights(w: Workload, expert: int, trial: int = 0, keep_f32: bool = True):
    """(W_gate [h,d], W_up [h,d], W_down [d,h]) of one expert; gate/up ~ N(0,1/d), down ~ N(0,1/h).

    Each expert has its own stream, so a test can draw a few experts of a large layer.
    """
    _, _, _, s_experts = _streams(w, trial)
    rng = np.random.default_rng(s_experts.spawn(w.n_experts)[expert])
    h, d = w.d_hidden, w.d_model
    sg = np.float32(1.0 / math.sqrt(d))
    sd = np.float32(1.0 / math.sqrt(h))
    gate = Stored(rng.standard_normal((h, d), dtype=np.float32) * sg, w.dtype, keep_f32)
    up = Stored(rng.standard_normal((h, d), dtype=np.float32) * sg, w.dtype, keep_f32)
    down = Stored(rng.standard_normal((d, h), dtype=np.float32) * sd, w.dtype, keep_f32)
    return gate, up, down


def logits_with_ties(w: Workload, trial: int = 0, levels: int = 5, pool_fraction: float = 0.125) -> np.ndarray:
    """Router logits built to tie: few distinct rows, each quantised to a few levels.

    Tokens are drawn from a small pool of rows, so many tokens carry bit-identical
    scores for an expert (ties at the capacity threshold), and each row holds repeated
    values (ties inside the top-k).  Shape [N, E], fp32.
    """
    rng = np.random.default_rng(np.random.SeedSequence([w.seed(trial), 77]))
    pool = max(2, int(w.n_tokens * pool_fraction))
    rows = rng.integers(0, levels, size=(pool, w.n_experts)).astype(np.float32) * np.float32(0.5)
    rows += router_bias(w, trial).round()[None, :]
    return np.ascontiguousarray(rows[rng.integers(0, pool, size=w.n_tokens)])
