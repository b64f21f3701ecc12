"""Seeded synthetic inputs shaped like the paper's workloads.

The paper trains and evaluates its predictors on pre-attention activations
collected from three real MoE models (section 4.4) and on their routers'
selections (eq. 1-2).  Neither the activations nor the models are available
here, so every tensor is drawn from a counter-based generator (NumPy's Philox,
keyed by workload, layer and tensor) with the gross statistics of those inputs:

* ``x``   post-norm hidden states: N(0,1) with a few fixed outlier channels
          scaled by 8, each row divided by its RMS (section 4.2 takes X right
          after the pre-attention normalisation), stored as bf16 or fp32;
* ``W1``  [r, d] ~ N(0, 1/d) and ``W2`` [E, r] ~ N(0, 1/r), one independent
          pair per layer (section 4.2: a separate predictor per layer);
* ``b2``  optional output bias carrying a Zipf(s = 1.2) expert-popularity skew;
* ``ref`` labels from a stand-in for the true router of eq. 1-2: the top-k of
          (W2 W1 + 0.1 G) x (+ b2) with G ~ N(0, 1/d), so that a predictor
          built from (W1, W2) agrees with it on most but not all tokens.

This module is the one piece shared by the CPU oracle's tests and the GPU
path's tests: it only *produces inputs*.  The label router and the near-tie
construction below use NumPy's matmul/argsort as data-generation tools; they
are neither called by nor shared with the predictor implementations.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

from .configs import Workload

BASE_KEY = 0x251110676
SIGMA_ROUTER = 0.1
ZIPF_S = 1.2
ZIPF_BETA = 0.6

# tensor ids for the generator key
_T_X, _T_W1, _T_W2, _T_G, _T_OUTLIER, _T_ZIPF, _T_TIE, _T_DUP = range(8)


def rng(config_id: int, layer: int, tensor_id: int, bank: int = 0) -> np.random.Generator:
    """Counter-based generator for one tensor: Philox keyed by its coordinates."""
    key0 = (BASE_KEY ^ (config_id << 40) ^ (bank << 32)) & 0xFFFFFFFFFFFFFFFF
    key1 = ((layer << 8) | tensor_id) & 0xFFFFFFFFFFFFFFFF
    return np.random.Generator(np.random.Philox(key=[key0, key1]))


# ----------------------------------------------------------------------------
# bf16 storage helpers (input formatting only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 array holding exactly the values the storage dtype can represent."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    if dtype == "f32":
        return a
    raise ValueError(dtype)


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------
def make_x(w: Workload, layer: int, T: int) -> np.ndarray:
    g = rng(w.config_id, layer, _T_X)
    x = g.standard_normal((T, w.d), dtype=np.float32)
    ch = rng(w.config_id, layer, _T_OUTLIER).choice(w.d, size=w.outliers, replace=False)
    x[:, ch] *= np.float32(8.0)
    if w.rms_scale:
        rms = np.sqrt(np.mean(x.astype(np.float64) ** 2, axis=1, keepdims=True))
        x = (x / rms).astype(np.float32)
    return round_to_storage(x, w.dtype)


def make_w1(w: Workload, layer: int, bank: int = 0) -> np.ndarray:
    g = rng(w.config_id, layer, _T_W1, bank)
    a = g.standard_normal((w.r, w.d), dtype=np.float32) * np.float32(1.0 / np.sqrt(w.d))
    return round_to_storage(a, w.dtype)


def make_w2(w: Workload, layer: int, bank: int = 0, dup_pairs: int = 0) -> np.ndarray:
    g = rng(w.config_id, layer, _T_W2, bank)
    a = g.standard_normal((w.E, w.r), dtype=np.float32) * np.float32(1.0 / np.sqrt(w.r))
    if dup_pairs:
        # duplicated rows give logits that tie bit-for-bit on every token
        pick = rng(w.config_id, layer, _T_DUP, bank).choice(w.E, size=2 * dup_pairs, replace=False)
        for a_id, b_id in pick.reshape(dup_pairs, 2):
            a[b_id] = a[a_id]
    return round_to_storage(a, w.dtype)


def make_b2(w: Workload, layer: int) -> Optional[np.ndarray]:
    if not w.zipf_bias:
        return None
    perm = rng(w.config_id, layer, _T_ZIPF).permutation(w.E)
    logp = -ZIPF_S * np.log(np.arange(1, w.E + 1, dtype=np.float64))
    b = np.empty(w.E, dtype=np.float64)
    b[perm] = ZIPF_BETA * (logp - logp.mean())
    return round_to_storage(b.astype(np.float32), w.dtype)


def make_router(w: Workload, layer: int, W1: np.ndarray, W2: np.ndarray) -> np.ndarray:
    """Stand-in for the true gate W_g of eq. 1: W2 W1 + sigma G, in float64."""
    G = rng(w.config_id, layer, _T_G).standard_normal((w.E, w.d)) / np.sqrt(w.d)
    return W2.astype(np.float64) @ W1.astype(np.float64) + SIGMA_ROUTER * G


def router_labels(Wg: np.ndarray, x: np.ndarray, b2: Optional[np.ndarray], k: int) -> np.ndarray:
    """Labels of eq. 2: the k highest router scores, ties to the lower expert id."""
    z = x.astype(np.float64) @ Wg.T
    if b2 is not None:
        z = z + b2.astype(np.float64)[None, :]
    return np.argsort(-z, axis=1, kind="stable")[:, :k].astype(np.int32)


def _bf16_ulp(a: np.ndarray) -> np.ndarray:
    """Spacing of bf16 numbers at |a| (a holds bf16-representable fp32)."""
    e = np.floor(np.log2(np.maximum(np.abs(a.astype(np.float64)), 2.0 ** -126)))
    return 2.0 ** (e - 7)


def plant_near_ties(w: Workload, layer: int, x: np.ndarray, W1: np.ndarray, W2: np.ndarray,
                    k: int, frac: float, gap_hi: float = 1e-3, rounds: int = 12) -> np.ndarray:
    """Move a seeded `frac` of the rows of x so that the predictor's k-th and
    (k+1)-th logits (in exact arithmetic) are less than `gap_hi` apart.

    The row is shifted along the difference of the two experts' collapsed
    weight rows, re-rounded to storage, then single coordinates are nudged by
    one storage ulp towards the middle of the target interval.  Returns the
    indices of the rows that were modified; x is changed in place.
    """
    T = x.shape[0]
    n = int(round(frac * T))
    if n == 0:
        return np.zeros(0, dtype=np.int64)
    g = rng(w.config_id, layer, _T_TIE)
    rows = np.sort(g.choice(T, size=n, replace=False))
    M = W2.astype(np.float64) @ W1.astype(np.float64)            # [E, d]
    xs = x[rows].astype(np.float64)
    z = xs @ M.T
    order = np.argsort(-z, axis=1, kind="stable")
    a, b = order[:, k - 1], order[:, k]
    v = M[a] - M[b]                                              # [n, d]
    ar = np.arange(n)
    gap = z[ar, a] - z[ar, b]
    delta = g.uniform(0.0, gap_hi, size=n)
    vv = np.sum(v * v, axis=1)
    movable = vv > 0                     # duplicated W2 rows give v = 0: that row already ties exactly
    step = np.where(movable, (gap - delta) / np.where(movable, vv, 1.0), 0.0)
    xs = xs - step[:, None] * v
    xs = round_to_storage(xs.astype(np.float32), w.dtype).astype(np.float64)
    if w.dtype == "bf16":
        target = 0.5 * gap_hi
        for _ in range(rounds):
            gap = np.sum(xs * v, axis=1)
            need = target - gap
            done = (gap > 0.1 * gap_hi) & (gap < 0.9 * gap_hi)
            if done.all():
                break
            ulp = _bf16_ulp(xs)
            step = v * ulp                                      # gap change for +1 ulp
            err = np.abs(need[:, None] - np.sign(need)[:, None] * np.abs(step))
            i = np.argmin(err, axis=1)
            s = np.sign(need) * np.sign(step[ar, i])
            upd = ~done
            xs[ar[upd], i[upd]] += (s * ulp[ar, i])[upd]
            xs = round_to_storage(xs.astype(np.float32), w.dtype).astype(np.float64)
    x[rows] = xs.astype(np.float32)
    return rows


@dataclass
class LayerInputs:
    x: np.ndarray                 # [T, d] fp32 values representable in the storage dtype
    W1: np.ndarray                # [r, d]
    W2: np.ndarray                # [E, r]
    b2: Optional[np.ndarray]      # [E] or None
    ref: np.ndarray               # [T, k] int32 router labels
    tie_rows: np.ndarray          # rows with a planted near-tie


def make_layer(w: Workload, layer: int, T: int, *, adversarial: bool = True) -> LayerInputs:
    """All inputs of one layer of a workload at T tokens."""
    dup = 1 if (adversarial and w.exact_tie_rows) else 0
    W1 = make_w1(w, layer)
    W2 = make_w2(w, layer, dup_pairs=dup)
    b2 = make_b2(w, layer)
    x = make_x(w, layer, T)
    tie_rows = np.zeros(0, dtype=np.int64)
    if adversarial and w.near_tie_frac > 0:
        tie_rows = plant_near_ties(w, layer, x, W1, W2, w.k, w.near_tie_frac)
    Wg = make_router(w, layer, W1, W2)
    ref = router_labels(Wg, x, b2, w.k)
    return LayerInputs(x=x, W1=W1, W2=W2, b2=b2, ref=ref, tie_rows=tie_rows)
