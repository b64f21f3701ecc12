"""CPU oracle for the pre-attention expert predictor.  TEST INFRASTRUCTURE ONLY.

Thin ctypes/NumPy wrapper over ``paep_oracle.c`` (plain C, double-precision
accumulation, full sort).  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the product path never does, and this
package imports nothing from the product.

``build()`` compiles the C file with gcc (OpenMP over tokens) into
``oracle/libpaep_oracle.so``; ``lib()`` loads it, building it first if absent.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "paep_oracle.c")
_SO = os.path.join(_HERE, "libpaep_oracle.so")
_lib = None

ACT_NONE, ACT_SILU, ACT_GELU = 0, 1, 2


def build(force: bool = True) -> str:
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-fno-fast-math", _SRC, "-o", _SO, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_SO)
        c_i, c_p = ctypes.c_int, ctypes.c_void_p
        L.paep_oracle_predict.argtypes = [c_i] * 7 + [c_p] * 8
        L.paep_oracle_predict.restype = c_i
        L.paep_oracle_group.argtypes = [c_p, c_i, c_i] + [c_p] * 6
        L.paep_oracle_group.restype = c_i
        L.paep_oracle_score.argtypes = [c_p, c_i, c_p, c_i, c_i, c_i, c_p, c_p]
        L.paep_oracle_score.restype = c_i
        L.paep_oracle_num_threads.restype = c_i
        L.paep_oracle_round_bf16.argtypes = [ctypes.c_double]
        L.paep_oracle_round_bf16.restype = ctypes.c_double
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().paep_oracle_num_threads())


def round_bf16(v: float) -> float:
    return float(lib().paep_oracle_round_bf16(float(v)))


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def predict(x, W1, W2, k: int, *, b1=None, b2=None, act: int = ACT_NONE,
            round_h: bool = False, want_logits: bool = True
            ) -> Tuple[np.ndarray, np.ndarray, Optional[np.ndarray]]:
    """One layer: x[T,d], W1[r,d], W2[E,r] -> idx[T,k] int32, probs[T,k] f32, logits[T,E] f64."""
    x, W1, W2 = _f32(x), _f32(W1), _f32(W2)
    T, d = x.shape
    r, d1 = W1.shape
    E, r1 = W2.shape
    if d1 != d or r1 != r:
        raise ValueError("shape mismatch between x, W1, W2")
    b1 = None if b1 is None else _f32(b1)
    b2 = None if b2 is None else _f32(b2)
    if b1 is not None and b1.shape != (r,):
        raise ValueError("b1 must be [r]")
    if b2 is not None and b2.shape != (E,):
        raise ValueError("b2 must be [E]")
    idx = np.empty((T, k), dtype=np.int32)
    probs = np.empty((T, k), dtype=np.float32)
    logits = np.empty((T, E), dtype=np.float64) if want_logits else None
    rc = lib().paep_oracle_predict(T, d, r, E, k, int(act), int(bool(round_h)),
                                   _ptr(x), _ptr(W1), _ptr(W2), _ptr(b1), _ptr(b2),
                                   _ptr(idx), _ptr(probs), _ptr(logits))
    if rc != 0:
        raise ValueError("paep_oracle_predict rejected its arguments")
    return idx, probs, logits


def group_by_expert(idx, E: int):
    """idx[...] int32 (flattened) -> counts[E], offsets[E+1], token_pos[n], active[E], n_active, n_invalid."""
    flat = np.ascontiguousarray(idx, dtype=np.int32).reshape(-1)
    n = flat.size
    counts = np.empty(E, dtype=np.int32)
    offsets = np.empty(E + 1, dtype=np.int32)
    token_pos = np.empty(n, dtype=np.int32)
    active = np.empty(E, dtype=np.int32)
    n_active = np.zeros(1, dtype=np.int32)
    n_invalid = np.zeros(1, dtype=np.int32)
    rc = lib().paep_oracle_group(_ptr(flat), n, E, _ptr(counts), _ptr(offsets), _ptr(token_pos),
                                 _ptr(active), _ptr(n_active), _ptr(n_invalid))
    if rc != 0:
        raise ValueError("paep_oracle_group rejected its arguments")
    return counts, offsets, token_pos, active, int(n_active[0]), int(n_invalid[0])


def score(idx, ref, E: int, k_row=None) -> np.ndarray:
    """idx[T,k_pred], ref[T,k_ref] -> int64[4] = (n_exact, n_hit, n_cover, n_top1).
    k_row[T] (optional): row t uses only its first clamp(k_row[t], 1, k_pred) predicted ids."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    ref = np.ascontiguousarray(ref, dtype=np.int32)
    if idx.ndim != 2 or ref.ndim != 2 or idx.shape[0] != ref.shape[0]:
        raise ValueError("idx and ref must be [T,k_pred] and [T,k_ref]")
    out = np.zeros(4, dtype=np.int64)
    if k_row is not None:
        k_row = np.ascontiguousarray(k_row, dtype=np.int32).reshape(-1)
        if k_row.size != idx.shape[0]:
            raise ValueError("k_row must have one entry per row")
    rc = lib().paep_oracle_score(_ptr(idx), idx.shape[1], _ptr(ref), ref.shape[1],
                                 idx.shape[0], E, _ptr(k_row), _ptr(out))
    if rc != 0:
        raise ValueError("paep_oracle_score rejected its arguments")
    return out


def activation_profile(counts) -> Tuple[np.ndarray, int, float]:
    """Expert popularity of one layer from its activation counts (paper section 2.1: the distribution
    of expert activation frequencies and its Shannon entropy, 0.976 for DeepSeek-V2-Lite's near-uniform
    routing; popularity is what popularity-based prefetchers, section 2.2.2, order experts by).

    counts[E] (non-negative integers) ->
        order[E]   the experts with counts > 0 by descending count, equal counts by ascending id,
                   then -1 for the rest
        n_active   how many experts that is
        entropy    -sum_e p_e ln p_e / ln E with p_e = counts[e] / sum(counts), in double;
                   0 when E = 1 or nothing was counted (the convention 0 ln 0 = 0 applies)
    Written out as the definition: a full sort and a plain sum.
    """
    c = np.asarray(counts, dtype=np.int64).reshape(-1)
    if (c < 0).any():
        raise ValueError("counts must be non-negative")
    E = c.size
    ids = sorted((e for e in range(E) if c[e] > 0), key=lambda e: (-int(c[e]), e))
    order = np.full(E, -1, dtype=np.int32)
    order[:len(ids)] = ids
    total = int(c.sum())
    entropy = 0.0
    if E > 1 and total > 0:
        import math
        h = 0.0
        for e in range(E):
            if c[e] > 0:
                p = int(c[e]) / total
                h -= p * math.log(p)
        entropy = h / math.log(E)
    return order, len(ids), entropy


def confidence_select(idx, probs, k_base: int, ratio: float):
    """Confidence-driven over-provisioning of one layer (paper section 6, future work: rows predicted with high
    confidence stay in exact-match mode, the others are over-provisioned).  The paper names no confidence
    score; the one used here is the separation between the last expert of the exact-match set and the first
    one outside it: row t is confident when probs[t, k_base-1] >= ratio * probs[t, k_base] (ratio = exp(tau)
    for a margin tau between the two scores, since softmax shares one normaliser per row).  The comparison is
    made in float32 -- one rounded product, one compare -- so that every implementation takes the same decision.

    idx[T,kp] int32, probs[T,kp] float32 (descending), 1 <= k_base < kp ->
        k_row[T]      k_base for confident rows, kp for the others
        idx_out[T,kp] idx with the entries past k_row set to -1
        n_wide        number of rows that were widened
    """
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    probs = np.ascontiguousarray(probs, dtype=np.float32)
    T, kp = idx.shape
    if probs.shape != (T, kp) or not (1 <= k_base < kp):
        raise ValueError("need idx, probs of one shape [T,kp] and 1 <= k_base < kp")
    r32 = np.float32(ratio)
    k_row = np.empty(T, dtype=np.int32)
    idx_out = idx.copy()
    n_wide = 0
    for t in range(T):
        confident = probs[t, k_base - 1] >= np.float32(r32 * probs[t, k_base])
        k_row[t] = k_base if confident else kp
        if confident:
            idx_out[t, k_base:] = -1
        else:
            n_wide += 1
    return k_row, idx_out, n_wide


def confidence_outputs(logits, idx):
    """Confidence scores of one layer's selection (paper section 6 asks for prediction confidence scores to
    drive dynamic over-provisioning; section 4.4 trains the predictor through a sigmoid per expert, eq. 1
    normalises the router with a softmax).  From the scores s = logits[T,E] (float64, as returned by
    `predict`) and the selection idx[T,k] (descending score):

        softmax_topk[t,j] = exp(s[t,idx[t,j]]) / sum_{i<k} exp(s[t,idx[t,i]])     softmax over the k selected only
        sigmoid[t,j]      = 1 / (1 + exp(-s[t,idx[t,j]]))
        margin[t]         = (k-th largest score) - ((k+1)-th largest score), +inf when k = E

    all in float64, written out as the definitions (the maximum is subtracted inside the exponentials, which
    does not change the quotient).
    """
    z = np.asarray(logits, dtype=np.float64)
    idx = np.asarray(idx, dtype=np.int64)
    T, E = z.shape
    k = idx.shape[1]
    soft = np.empty((T, k), dtype=np.float64)
    sig = np.empty((T, k), dtype=np.float64)
    margin = np.empty(T, dtype=np.float64)
    for t in range(T):
        s = z[t, idx[t]]
        w = np.exp(s - s.max())
        soft[t] = w / w.sum()
        sig[t] = 1.0 / (1.0 + np.exp(-s))
        if k < E:
            desc = np.sort(z[t])[::-1]
            margin[t] = desc[k - 1] - desc[k]
        else:
            margin[t] = np.inf
    return soft, sig, margin


def fold_batchnorm(W1, b1, gamma, beta, mean, var, eps: float = 1e-5):
    """BatchNorm at inference folded into the first linear layer (paper section 4.3, Architecture 1:
    Linear -> BatchNorm -> GELU -> Dropout -> Linear; dropout is the identity at inference).  BatchNorm maps
    u_j to gamma_j (u_j - mean_j) / sqrt(var_j + eps) + beta_j, so with g_j = gamma_j / sqrt(var_j + eps)
        W1'[j,:] = g_j W1[j,:]        b1'[j] = g_j (b1[j] - mean_j) + beta_j
    One layer: W1[r,d], b1[r] or None, the four statistics [r]; float64 throughout."""
    W1 = np.asarray(W1, dtype=np.float64)
    r = W1.shape[0]
    b = np.zeros(r) if b1 is None else np.asarray(b1, dtype=np.float64)
    g = np.asarray(gamma, dtype=np.float64) / np.sqrt(np.asarray(var, dtype=np.float64) + float(eps))
    return g[:, None] * W1, g * (b - np.asarray(mean, dtype=np.float64)) + np.asarray(beta, dtype=np.float64)
