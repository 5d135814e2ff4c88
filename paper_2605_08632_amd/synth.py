"""Seeded synthetic inputs for the CAT-loss hot path of PARD-2.

This module only *draws inputs*: hidden states, an LM-head weight, target ids,
block valid-lengths and external confidences, with the shapes and structure of
the draft-training workload (draft blocks of K slots per anchor, Eq.4; large
vocabularies; acceptance that decays with slot position and confidences that
correlate with acceptance, Fig.2).  It contains none of the method's arithmetic
(no logits, softmax, weights or gradients): where a recipe needs the head's
argmax, the caller passes it in.  Both the CPU oracle's tests and the HIP
path's tests/benchmark draw from here so that they see identical bits.

Storage rounding (bf16, round-to-nearest-even) is done once, here, on the host;
every consumer works from the rounded values.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

IGNORE_INDEX = -100
BASE_SEED = 20260508


# --------------------------------------------------------------------------
# bf16 storage helpers (bit manipulation only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (RNE) and return the 16-bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    # round-to-nearest-even on the 16 discarded bits; NaN never occurs here
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# workload table
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    """One synthetic workload: a draft head of width d over V ids, B anchors x K slots."""
    name: str
    index: int
    dtype: str            # "bf16" | "fp32": storage type of H and W
    B: int
    K: int
    d: int
    V: int
    p_agree: object       # float, or ("linear", hi, lo) across slot position
    fallback: str         # "uniform" | "zipf"
    ragged_frac: float = 0.0   # fraction of blocks that get a short valid length
    beta: float = 0.1     # CE coefficient used in training (Eq.12, Table 6)

    @property
    def T(self) -> int:
        return self.B * self.K

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


WORKLOADS = {
    "c0_tiny_fp32": Workload("c0_tiny_fp32", 0, "fp32", 8, 8, 256, 4096, 0.6, "uniform"),
    "c1_small_bf16": Workload("c1_small_bf16", 1, "bf16", 256, 8, 2048, 32000, 0.6, "uniform"),
    "c2_llama1b_bf16": Workload("c2_llama1b_bf16", 2, "bf16", 1024, 8, 2048, 128256, 0.5, "zipf"),
    "c3_qwen06b_bf16": Workload("c3_qwen06b_bf16", 3, "bf16", 1024, 16, 1024, 151936,
                                ("linear", 0.9, 0.3), "uniform"),
    "c4_8bwidth_bf16": Workload("c4_8bwidth_bf16", 4, "bf16", 2048, 8, 4096, 128256, 0.5, "zipf",
                                ragged_frac=0.10),
}


@dataclass
class Head:
    """Hidden states and head weight in storage precision.

    `H`, `W` are float32 arrays holding exactly the stored values (for bf16 the
    float32 widening of the rounded bits); `H_bits`, `W_bits` are the uint16
    bf16 patterns (None for fp32 storage).
    """
    H: np.ndarray
    W: np.ndarray
    H_bits: Optional[np.ndarray] = None
    W_bits: Optional[np.ndarray] = None
    dtype: str = "fp32"


def _unit_rms_rows(H: np.ndarray) -> np.ndarray:
    rms = np.sqrt(np.mean(H.astype(np.float64) ** 2, axis=1, keepdims=True))
    return (H / rms).astype(np.float32)


def make_head(seed: int, T: int, d: int, V: int, dtype: str, w_scale: float = 4.0,
              row_attempts: Optional[np.ndarray] = None) -> Head:
    """H ~ N(0,1) with every row scaled to RMS 1; W ~ N(0, 1/d) * w_scale.

    With unit-RMS rows the logits have standard deviation ~ w_scale: a peaked
    but non-degenerate softmax.  `row_attempts[t] = a > 0` replaces row t of H by
    the a-th re-draw of that row (its own seeded stream): callers use it to move a
    row whose two largest logits nearly tie, where "the" argmax is not well-posed
    under reordered fp32 accumulation.
    """
    rng = np.random.default_rng([seed, 0])
    H = rng.standard_normal((T, d), dtype=np.float32)
    if row_attempts is not None:
        for t in np.nonzero(row_attempts)[0]:
            r = np.random.default_rng([seed, 7, int(t), int(row_attempts[t])])
            H[t] = r.standard_normal(d, dtype=np.float32)
    H = _unit_rms_rows(H)
    W = rng.standard_normal((V, d), dtype=np.float32)
    W *= np.float32(w_scale / np.sqrt(d))
    if dtype == "bf16":
        hb = f32_to_bf16_bits(H)
        wb = f32_to_bf16_bits(W)
        return Head(bf16_bits_to_f32(hb), bf16_bits_to_f32(wb), hb, wb, "bf16")
    if dtype == "fp32":
        return Head(H, W, None, None, "fp32")
    raise ValueError(f"unknown dtype {dtype!r}")


def make_teacher(seed: int, head: Head, dt: int, noise: float = 2.0) -> Head:
    """Teacher hidden states Ht[T, dt] and head Wt[V, dt] (storage type of `head`) for the distillation term.

    A target model is wider than its drafter and its distribution resembles the drafter's
    without equalling it.  For dt > d the teacher extends the draft head's operands,
        Ht = [H | noise * E],   Wt = [W | F],   E ~ N(0,1) with unit-RMS rows, F ~ N(0, 1/(dt-d)),
    so that its logits are the draft's plus independent noise of standard deviation ~`noise`.
    For dt <= d an unrelated head of width dt is drawn instead.
    """
    T, d = head.H.shape
    V = head.W.shape[0]
    if dt <= d:
        return make_head(int(np.random.default_rng([seed, 11]).integers(1 << 30)), T, dt, V, head.dtype)
    rng = np.random.default_rng([seed, 12])
    E = _unit_rms_rows(rng.standard_normal((T, dt - d), dtype=np.float32)) * np.float32(noise)
    F = rng.standard_normal((V, dt - d), dtype=np.float32) * np.float32(1.0 / np.sqrt(dt - d))
    if head.dtype == "fp32":
        return Head(np.concatenate([head.H, E], axis=1), np.concatenate([head.W, F], axis=1), None, None, "fp32")
    hb = np.concatenate([head.H_bits, f32_to_bf16_bits(E)], axis=1)
    wb = np.concatenate([head.W_bits, f32_to_bf16_bits(F)], axis=1)
    return Head(bf16_bits_to_f32(hb), bf16_bits_to_f32(wb), hb, wb, "bf16")


def _fallback_ids(rng: np.random.Generator, n: int, V: int, kind: str) -> np.ndarray:
    if kind == "uniform":
        return rng.integers(0, V, size=n, dtype=np.int64)
    if kind == "zipf":
        # bounded Zipf: P(rank r) ~ r^-1.1 for r = 1..V, id = r - 1
        r = np.arange(1, V + 1, dtype=np.float64)
        cdf = np.cumsum(r ** -1.1)
        cdf /= cdf[-1]
        ids = np.searchsorted(cdf, rng.random(n), side="left")
        return np.minimum(ids, V - 1).astype(np.int64)
    raise ValueError(f"unknown fallback {kind!r}")


def agree_probability(p_agree, B: int, K: int) -> np.ndarray:
    """Per-row probability [T] that the target equals the head's argmax."""
    if isinstance(p_agree, tuple):
        kind, hi, lo = p_agree
        assert kind == "linear"
        per_slot = hi - (hi - lo) * (np.arange(K) / max(K - 1, 1))
    else:
        per_slot = np.full(K, float(p_agree))
    return np.tile(per_slot, B)


def make_targets(seed: int, argmax: np.ndarray, B: int, K: int, V: int, p_agree,
                 fallback: str):
    """Targets y[T] (int32): the supplied argmax with probability p_agree, else a fallback id.

    Returns (y, agree_mask).  `argmax` is an input: this module never computes it.
    """
    T = B * K
    argmax = np.asarray(argmax).reshape(T)
    rng = np.random.default_rng([seed, 1])
    agree = rng.random(T) < agree_probability(p_agree, B, K)
    fb = _fallback_ids(rng, T, V, fallback)
    y = np.where(agree, argmax.astype(np.int64), fb).astype(np.int32)
    return y, agree


def make_valid_len(seed: int, B: int, K: int, ragged_frac: float) -> np.ndarray:
    """valid_len[B] int32: K for most blocks; a Bernoulli(ragged_frac) subset gets U{1..K-1}."""
    rng = np.random.default_rng([seed, 2])
    vl = np.full(B, K, dtype=np.int32)
    if ragged_frac > 0 and K > 1:
        short = rng.random(B) < ragged_frac
        vl[short] = rng.integers(1, K, size=int(short.sum()), dtype=np.int32)
    return vl


def apply_tail_padding(y: np.ndarray, valid_len: np.ndarray, K: int) -> np.ndarray:
    """Set y = IGNORE_INDEX on the slots k >= valid_len[b] of every block."""
    y = y.copy().reshape(-1, K)
    slot = np.arange(K)[None, :]
    y[slot >= valid_len[:, None]] = IGNORE_INDEX
    return y.reshape(-1)


def make_external_conf(seed: int, agree: np.ndarray) -> np.ndarray:
    """Teacher confidences conf_in[T] in [0.05, 0.95]: higher on rows where the target
    agrees with the head's argmax (Beta(4,2)) than elsewhere (Beta(2,4))."""
    rng = np.random.default_rng([seed, 3])
    n = agree.shape[0]
    u = np.where(agree, rng.beta(4.0, 2.0, n), rng.beta(2.0, 4.0, n))
    return np.clip(0.05 + 0.9 * u, 0.0, 1.0).astype(np.float32)
