"""The GPU-vs-oracle comparison itself, on the CPU: mistakes are planted in otherwise correct
selections and the checker must refuse each of them (and accept the correct ones)."""
import numpy as np
import pytest

import oracle
import parity


def _case(seed=0, n=64, E=24, k=4):
    g = np.random.default_rng(seed)
    z = g.standard_normal((n, E))
    idx = parity.topk_rule(z, k)
    P = parity.softmax64(z)
    probs = np.take_along_axis(P, idx.astype(np.int64), axis=1).astype(np.float32)
    return z, idx, P, probs


def test_correct_selection_passes_and_counts_rows():
    z, idx, P, probs = _case()
    rep = parity.compare_rows(z, idx, P, idx, probs, z.astype(np.float32).astype(np.float64), 4, 1e-5, "ok")
    assert rep.rows == 64 and rep.exempt_differ == 0 and rep.idx_equal_rows == 64


def test_topk_rule_agrees_with_the_oracle_ordering_on_ties():
    g = np.random.default_rng(3)
    z = g.integers(-2, 3, size=(50, 12)).astype(np.float64)        # many exact ties
    z[0, :4] = [0.0, -0.0, 0.0, -0.0]                               # the two zeros tie
    x = np.eye(12, dtype=np.float32)
    for t in range(z.shape[0]):                                     # oracle: identity maps, b2 carries the scores
        idx_o, _, z_o = oracle.predict(np.zeros((1, 12), np.float32), x, x, 5, b2=z[t].astype(np.float32))
        assert np.array_equal(parity.topk_rule(z[t:t + 1], 5)[0], idx_o[0])


def test_dropped_clear_winner_on_an_exempt_row_is_refused():
    # k = 2, scores (10, 5, 4.99): the row is exempt (5 vs 4.99), but expert 0 may not be dropped
    z = np.array([[10.0, 5.0, 4.99, 0.0]])
    P = parity.softmax64(z)
    ref = np.array([[0, 1]], dtype=np.int32)
    bad = np.array([[1, 2]], dtype=np.int32)
    pb = np.take_along_axis(P, bad.astype(np.int64), axis=1).astype(np.float32)
    with pytest.raises(AssertionError, match="drops an expert"):
        parity.compare_rows(z, ref, P, bad, pb, None, 2, 2e-2, "planted")
    ok = np.array([[0, 2]], dtype=np.int32)                          # swapping inside the band is allowed
    po = np.take_along_axis(P, ok.astype(np.int64), axis=1).astype(np.float32)
    rep = parity.compare_rows(z, ref, P, ok, po, None, 2, 2e-2, "allowed")
    assert rep.exempt == 1 and rep.exempt_differ == 1


def test_selection_that_contradicts_the_kernels_own_scores_is_refused():
    z, idx, P, probs = _case(1)
    wrong = idx.copy()
    wrong[7, [0, 1]] = wrong[7, [1, 0]]                              # order swapped on one row
    rep = parity.RowReport()
    with pytest.raises(AssertionError, match="own scores"):
        parity.check_own_scores(z.astype(np.float32), wrong, probs, 4, rep, "planted")


def test_tie_resolved_to_the_higher_id_is_refused():
    z = np.array([[1.0, 3.0, 3.0, 0.5]], dtype=np.float32)
    rep = parity.RowReport()
    P = parity.softmax64(z.astype(np.float64))
    good, bad = np.array([[1, 2]], np.int32), np.array([[2, 1]], np.int32)
    parity.check_own_scores(z, good, np.take_along_axis(P, good.astype(np.int64), 1).astype(np.float32), 2, rep)
    with pytest.raises(AssertionError, match="own scores"):
        parity.check_own_scores(z, bad, np.take_along_axis(P, bad.astype(np.int64), 1).astype(np.float32), 2, rep)


def test_sloppy_softmax_is_refused_by_the_own_score_check():
    z, idx, P, probs = _case(2)
    sloppy = (probs * np.float32(1.0 + 1e-3)).astype(np.float32)    # inside the wide oracle bound at bf16 tolerance
    parity.compare_rows(z, idx, P, idx, sloppy, None, 4, 2e-2, "wide bound passes")
    with pytest.raises(AssertionError, match="softmax of the kernel's own"):
        parity.compare_rows(z, idx, P, idx, sloppy, z.astype(np.float32).astype(np.float64), 4, 2e-2, "planted")


def test_strict_row_mismatch_duplicate_and_out_of_range_are_refused():
    z, idx, P, probs = _case(4)
    for plant in ("strict", "dup", "range"):
        bad = idx.copy()
        if plant == "strict":
            zs = -np.sort(-z, axis=1)
            t = int(np.flatnonzero((zs[:, :4] - zs[:, 1:5] >= 0.05).all(axis=1))[0])     # a row with clear gaps
            others = [e for e in range(z.shape[1]) if e not in idx[t]]
            bad[t, -1] = others[0]
        elif plant == "dup":
            bad[3, 1] = bad[3, 0]
        else:
            bad[5, 2] = z.shape[1]
        with pytest.raises(AssertionError):
            parity.compare_rows(z, idx, P, bad, probs, None, 4, 1e-5, plant)
