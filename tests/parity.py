"""Comparison of the GPU predictor with the CPU oracle (shared by the GPU tests
and the smoke check).

Tolerances
  * spec bar, against the oracle in exact (fp64) mode:
      |z_gpu - z_ref| <= TOL * s_t,  s_t = max_e |z_ref[t, e]|,
      TOL = 2e-2 for bf16 storage, 1e-5 for fp32 storage.
    A row is *strict* when every gap between consecutive oracle scores at sorted
    positions 0..k is >= TOL * s_t: its idx must match bit for bit.  Otherwise it
    is *exempt*: the reported experts must be distinct, each within
    TOL * s_t of the oracle's k-th score, and every expert whose oracle score
    is more than TOL * s_t ABOVE the k-th score must be among them (so a
    clearly better expert can never be dropped on a row that happens to have a
    near-tie elsewhere).
  * the selection machinery itself, with no tolerance at all: on EVERY row the
    reported idx must equal the top-k of the kernel's own exported scores under
    the ordering rule (score descending, equal scores by ascending expert id).
  * model bar (bf16 only), against the oracle with the hidden vector rounded to
    bf16 as the kernels do: the same two rules with TOL_MODEL = 2e-3.  What is
    left is fp32-vs-fp64 accumulation: ~sqrt(d) * 2^-24 relative per dot
    product, plus the rare hidden unit whose fp32 sum lands on the other side
    of a bf16 rounding boundary (about r * 1e-3 units per token, each moving a
    score by |W2| * ulp ~ 1e-4): a few 1e-4 of s_t at the paper's shapes.
  * probs: softmax is Lipschitz in the scores; with every score within
    delta = TOL * s_t, each probability is within (exp(2 delta) - 1) of its
    oracle value, relatively.  That bound is wide at bf16 tolerances, so the
    softmax arithmetic is pinned separately: against a float64 softmax of the
    kernel's own exported scores each probability must agree within
    PROB_TOL_OWN relative (fp32 exp and an fp32 sum over at most 1024 terms).
    The largest relative error against the oracle is reported as well.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

import oracle

TOL = {"bf16": 2e-2, "f32": 1e-5}
TOL_MODEL = 2e-3
PROB_TOL_OWN = 2e-5


@dataclass
class RowReport:
    rows: int = 0
    strict: int = 0
    exempt: int = 0
    exempt_differ: int = 0
    max_logit_err: float = 0.0       # in units of s_t
    idx_equal_rows: int = 0
    max_prob_rel_err: float = 0.0    # against the oracle's softmax, relative
    max_prob_rel_err_own: float = 0.0   # against a float64 softmax of the kernel's own scores
    own_topk_rows: int = 0           # rows on which idx was checked against the kernel's own scores

    def add(self, other: "RowReport"):
        self.rows += other.rows
        self.strict += other.strict
        self.exempt += other.exempt
        self.exempt_differ += other.exempt_differ
        self.idx_equal_rows += other.idx_equal_rows
        self.max_logit_err = max(self.max_logit_err, other.max_logit_err)
        self.max_prob_rel_err = max(self.max_prob_rel_err, other.max_prob_rel_err)
        self.max_prob_rel_err_own = max(self.max_prob_rel_err_own, other.max_prob_rel_err_own)
        self.own_topk_rows += other.own_topk_rows


def compare_rows(z_ref, idx_ref, probs_ref_all, idx_gpu, probs_gpu, z_gpu, k, tol, what="") -> RowReport:
    """One layer's rows.  z_ref [n,E] f64, idx_ref [n,k], probs_ref_all [n,E] f64;
    idx_gpu [n,k], probs_gpu [n,k], z_gpu [n,E] or None."""
    n, E = z_ref.shape
    rep = RowReport(rows=n)
    if n == 0:
        return rep
    s_t = np.abs(z_ref).max(axis=1)
    s_t = np.where(s_t > 0, s_t, 1.0)
    delta = tol * s_t
    if z_gpu is not None:
        err = np.abs(z_gpu.astype(np.float64) - z_ref)
        rep.max_logit_err = float((err.max(axis=1) / s_t).max())
        bad = err > delta[:, None] + 1e-30
        assert not bad.any(), (f"{what}: {bad.sum()} scores off by more than {tol} * s_t; "
                               f"worst {rep.max_logit_err:.3e}")
    zs = -np.sort(-z_ref, axis=1)
    kk = min(k + 1, E)
    gaps = zs[:, :kk - 1] - zs[:, 1:kk]
    strict = (gaps >= delta[:, None]).all(axis=1) if gaps.shape[1] else np.ones(n, bool)
    same = (idx_gpu == idx_ref).all(axis=1)
    rep.strict = int(strict.sum())
    rep.exempt = int(n - rep.strict)
    rep.idx_equal_rows = int(same.sum())
    rep.exempt_differ = int((~strict & ~same).sum())
    wrong = strict & ~same
    assert not wrong.any(), (f"{what}: idx differs on {wrong.sum()} strict rows, first t={np.flatnonzero(wrong)[0]}: "
                             f"gpu {idx_gpu[np.flatnonzero(wrong)[0]]} ref {idx_ref[np.flatnonzero(wrong)[0]]}")
    # exempt rows: valid ids, distinct, each close enough to the k-th score
    assert ((idx_gpu >= 0) & (idx_gpu < E)).all(), f"{what}: expert id out of range"
    srt = np.sort(idx_gpu, axis=1)
    assert (np.diff(srt, axis=1) > 0).all() if k > 1 else True, f"{what}: duplicate expert in a row"
    picked = np.take_along_axis(z_ref, idx_gpu.astype(np.int64), axis=1)
    kth = zs[:, k - 1]
    assert (picked >= (kth - delta)[:, None] - 1e-30).all(), f"{what}: a selected expert is below the k-th score by more than the tolerance"
    # nothing clearly better than the k-th score may be missing
    member = np.zeros((n, E), dtype=bool)
    np.put_along_axis(member, idx_gpu.astype(np.int64), True, axis=1)
    must = z_ref > (kth + delta)[:, None] + 1e-30
    dropped = must & ~member
    assert not dropped.any(), (f"{what}: row {np.flatnonzero(dropped.any(axis=1))[0]} drops an expert whose oracle "
                               f"score is above the k-th by more than the tolerance")
    # descending order up to the tolerance
    assert (np.diff(picked, axis=1) <= 2 * delta[:, None] + 1e-30).all(), f"{what}: selection is not in descending score order"
    # probabilities
    p_ref = np.take_along_axis(probs_ref_all, idx_gpu.astype(np.int64), axis=1)
    rel = np.expm1(2 * delta)[:, None] + 2e-5
    perr = np.abs(probs_gpu.astype(np.float64) - p_ref) / np.maximum(p_ref, 1e-300)
    rep.max_prob_rel_err = float(perr.max())
    assert (np.abs(probs_gpu.astype(np.float64) - p_ref) <= rel * p_ref + 1e-30).all(), f"{what}: probs outside the derived bound"
    if z_gpu is not None:
        check_own_scores(z_gpu, idx_gpu, probs_gpu, k, rep, what)
    return rep


def topk_rule(z, k):
    """The ordering rule applied to a score matrix: score descending, equal scores by ascending
    expert id (a stable sort of the negated scores; -0 and +0 compare equal)."""
    return np.argsort(-(z + 0.0), axis=1, kind="stable")[:, :k].astype(np.int32)


def check_own_scores(z_gpu, idx_gpu, probs_gpu, k, rep, what=""):
    """Tolerance-free check of the selection, and a sharp check of the softmax, against the
    scores the kernel itself exported (they are the values its epilogue selected from)."""
    assert np.isfinite(z_gpu).all(), f"{what}: non-finite exported score"
    own = topk_rule(z_gpu, k)
    bad = (own != idx_gpu).any(axis=1)
    assert not bad.any(), (f"{what}: idx is not the top-k of the kernel's own scores on {bad.sum()} rows, first "
                           f"t={np.flatnonzero(bad)[0]}: gpu {idx_gpu[np.flatnonzero(bad)[0]]} rule {own[np.flatnonzero(bad)[0]]}")
    rep.own_topk_rows = int(z_gpu.shape[0])
    p_own = np.take_along_axis(softmax64(z_gpu.astype(np.float64)), idx_gpu.astype(np.int64), axis=1)
    e_own = np.abs(probs_gpu.astype(np.float64) - p_own) / np.maximum(p_own, 1e-300)
    rep.max_prob_rel_err_own = float(e_own.max())
    assert rep.max_prob_rel_err_own <= PROB_TOL_OWN, (f"{what}: probs differ from the softmax of the kernel's own "
                                                      f"scores by {rep.max_prob_rel_err_own:.2e} relative")


def softmax64(z):
    m = z.max(axis=1, keepdims=True)
    e = np.exp(z - m)
    return e / e.sum(axis=1, keepdims=True)


def check_layer(lay_x, W1, W2, b1, b2, act, k, dtype, idx_gpu, probs_gpu, z_gpu, rows=None, what=""):
    """Runs the oracle on `rows` (default all) of one layer and checks the GPU
    outputs for those rows.  Returns (report_vs_exact, report_vs_model or None)."""
    if rows is None:
        rows = np.arange(lay_x.shape[0])
    xs = lay_x[rows]
    ig, pg = idx_gpu[rows], probs_gpu[rows]
    zg = None if z_gpu is None else z_gpu[rows]
    idx_ref, _, z_ref = oracle.predict(xs, W1, W2, k, b1=b1, b2=b2, act=act, round_h=False)
    rep = compare_rows(z_ref, idx_ref, softmax64(z_ref), ig, pg, zg, k, TOL[dtype], what + " [exact oracle]")
    rep_m = None
    if dtype == "bf16":
        idx_m, _, z_m = oracle.predict(xs, W1, W2, k, b1=b1, b2=b2, act=act, round_h=True)
        rep_m = compare_rows(z_m, idx_m, softmax64(z_m), ig, pg, zg, k, TOL_MODEL, what + " [bf16-hidden oracle]")
    return rep, rep_m
