"""Pins for the CPU oracle: everything here checks `oracle/` against something
other than itself -- NumPy / SciPy / PyTorch library routines in float64,
closed forms, invariants the paper states, brute force on tiny inputs, and
hand-built cases.  Shapes are non-square on purpose so that a transposed
operand or a swapped index cannot pass.
"""
import math

import numpy as np
import pytest
import scipy.special
import torch

import oracle


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def _as_f32_exact(a):
    return a.astype(np.float32)


# ---------------------------------------------------------------- two linear maps
@pytest.mark.parametrize("T,d,r,E", [(5, 24, 7, 11), (3, 8, 40, 6), (1, 130, 3, 2)])
def test_logits_match_numpy_float64_matmul(T, d, r, E):
    x, W1, W2 = (_as_f32_exact(_rand(s, *sh)) for s, sh in ((1, (T, d)), (2, (r, d)), (3, (E, r))))
    _, _, z = oracle.predict(x, W1, W2, k=1)
    want = (W2.astype(np.float64) @ (W1.astype(np.float64) @ x.astype(np.float64).T)).T
    np.testing.assert_allclose(z, want, rtol=0, atol=1e-12 * np.abs(want).max())


def test_collapsed_form_W2W1_x():
    """Two linear maps with nothing in between equal one map by W2 W1."""
    T, d, r, E = 6, 33, 17, 9
    x, W1, W2 = _as_f32_exact(_rand(4, T, d)), _as_f32_exact(_rand(5, r, d)), _as_f32_exact(_rand(6, E, r))
    _, _, z = oracle.predict(x, W1, W2, k=2)
    M = W2.astype(np.float64) @ W1.astype(np.float64)
    want = x.astype(np.float64) @ M.T
    assert np.abs(z - want).max() <= 1e-12 * np.abs(want).max()


def test_bias_terms_are_added_once_each():
    T, d, r, E = 4, 10, 6, 5
    x, W1, W2 = _as_f32_exact(_rand(7, T, d)), _as_f32_exact(_rand(8, r, d)), _as_f32_exact(_rand(9, E, r))
    b1, b2 = _as_f32_exact(_rand(10, r)), _as_f32_exact(_rand(11, E))
    _, _, z = oracle.predict(x, W1, W2, k=1, b1=b1, b2=b2)
    h = x.astype(np.float64) @ W1.astype(np.float64).T + b1.astype(np.float64)
    want = h @ W2.astype(np.float64).T + b2.astype(np.float64)
    np.testing.assert_allclose(z, want, rtol=0, atol=1e-12 * np.abs(want).max())


def test_zero_input_gives_bias_and_uniform_probs():
    d, r, E, k = 12, 5, 8, 3
    W1, W2 = _as_f32_exact(_rand(12, r, d)), _as_f32_exact(_rand(13, E, r))
    x = np.zeros((2, d), dtype=np.float32)
    idx, probs, z = oracle.predict(x, W1, W2, k=k)
    assert np.all(z == 0.0)
    assert idx.tolist() == [[0, 1, 2]] * 2          # all tied: lowest ids, ascending
    np.testing.assert_allclose(probs, 1.0 / E, rtol=1e-7)
    b2 = np.array([0, 3, 1, 2, 9, -1, 8, 0.5], dtype=np.float32)
    idx, _, z = oracle.predict(x, W1, W2, k=k, b2=b2)
    assert np.all(z == b2.astype(np.float64)[None, :])
    assert idx.tolist() == [[4, 6, 1]] * 2


def test_identity_weights_select_topk_of_x():
    d = 9
    I = np.eye(d, dtype=np.float32)
    x = _as_f32_exact(_rand(14, 7, d))
    idx, _, z = oracle.predict(x, I, I, k=4)
    assert np.array_equal(z, x.astype(np.float64))
    want = np.argsort(-x.astype(np.float64), axis=1, kind="stable")[:, :4]
    assert np.array_equal(idx, want)


# ---------------------------------------------------------------- top-k
def _repeated_max(z, k):
    """Independent selection: k passes, each taking the first maximum left."""
    z = list(z)
    taken, out = set(), []
    for _ in range(k):
        best = None
        for e, v in enumerate(z):
            if e in taken:
                continue
            if best is None or v > z[best]:
                best = e
        taken.add(best)
        out.append(best)
    return out


@pytest.mark.parametrize("seed", range(6))
def test_topk_bruteforce_tiny(seed):
    g = np.random.default_rng(100 + seed)
    T, d, r, E = 8, 6, 5, int(g.integers(2, 17))
    k = int(g.integers(1, E + 1))
    # coarse integer-valued inputs make many exact ties
    x = g.integers(-2, 3, size=(T, d)).astype(np.float32)
    W1 = g.integers(-1, 2, size=(r, d)).astype(np.float32)
    W2 = g.integers(-1, 2, size=(E, r)).astype(np.float32)
    idx, _, z = oracle.predict(x, W1, W2, k=k)
    for t in range(T):
        assert idx[t].tolist() == _repeated_max(z[t], k)
        assert idx[t].tolist() == np.argsort(-z[t], kind="stable")[:k].tolist()


def test_topk_matches_torch_topk_on_tie_free_rows():
    T, d, r, E, k = 64, 20, 12, 50, 7
    x, W1, W2 = _as_f32_exact(_rand(20, T, d)), _as_f32_exact(_rand(21, r, d)), _as_f32_exact(_rand(22, E, r))
    idx, _, z = oracle.predict(x, W1, W2, k=k)
    vals, want = torch.topk(torch.from_numpy(z), k, dim=1, largest=True, sorted=True)
    assert np.array_equal(idx, want.numpy().astype(np.int32))


def test_duplicate_w2_rows_tie_to_lower_id():
    T, d, r, E, k = 40, 16, 10, 6, 3
    x, W1, W2 = _as_f32_exact(_rand(23, T, d)), _as_f32_exact(_rand(24, r, d)), _as_f32_exact(_rand(25, E, r))
    W2[4] = W2[1]
    idx, probs, z = oracle.predict(x, W1, W2, k=k)
    assert np.array_equal(z[:, 1], z[:, 4])
    seen_both = 0
    for t in range(T):
        row = idx[t].tolist()
        assert not (4 in row and 1 not in row)      # 4 can never be picked ahead of 1
        if 1 in row and 4 in row:
            seen_both += 1
            assert row.index(4) == row.index(1) + 1
            assert probs[t, row.index(1)] == probs[t, row.index(4)]
    assert seen_both > 0


def test_k_equals_E_is_a_permutation_and_probs_sum_to_one():
    T, d, r, E = 9, 14, 6, 13
    x, W1, W2 = _as_f32_exact(_rand(26, T, d)), _as_f32_exact(_rand(27, r, d)), _as_f32_exact(_rand(28, E, r))
    idx, probs, _ = oracle.predict(x, W1, W2, k=E)
    assert np.array_equal(np.sort(idx, axis=1), np.tile(np.arange(E), (T, 1)))
    np.testing.assert_allclose(probs.astype(np.float64).sum(axis=1), 1.0, atol=1e-6)
    assert np.all(np.diff(probs, axis=1) <= 0)


def test_nan_score_orders_last():
    d = 4
    I = np.eye(d, dtype=np.float32)
    x = np.array([[1.0, np.nan, 3.0, 2.0]], dtype=np.float32)
    # NaN * 0 = NaN poisons every sum through the identity maps, so feed the
    # NaN through the bias instead
    x0 = np.array([[1.0, 0.0, 3.0, 2.0]], dtype=np.float32)
    b2 = np.array([0.0, np.nan, 0.0, 0.0], dtype=np.float32)
    idx, _, _ = oracle.predict(x0, I, I, k=4, b2=b2)
    assert idx.tolist() == [[2, 3, 0, 1]]


# ---------------------------------------------------------------- softmax
def test_ranking_preservation_softmax_vs_logits():
    """Softmax is monotone: ranking the probabilities ranks the scores."""
    T, d, r, E, k = 50, 18, 9, 24, 6
    x, W1, W2 = _as_f32_exact(_rand(30, T, d)), _as_f32_exact(_rand(31, r, d)), _as_f32_exact(_rand(32, E, r))
    idx, probs, z = oracle.predict(x, W1, W2, k=k)
    p_all = scipy.special.softmax(z, axis=1)
    want = np.argsort(-p_all, axis=1, kind="stable")[:, :k]
    assert np.array_equal(idx, want)
    np.testing.assert_allclose(probs, np.take_along_axis(p_all, idx.astype(np.int64), axis=1),
                               rtol=2e-7)


def test_probs_match_torch_softmax_float64_and_shift_invariance():
    T, d, r, E, k = 10, 8, 5, 7, 7
    x, W1, W2 = _as_f32_exact(_rand(33, T, d)), _as_f32_exact(_rand(34, r, d)), _as_f32_exact(_rand(35, E, r))
    idx, probs, z = oracle.predict(x, W1, W2, k=k)
    p = torch.softmax(torch.from_numpy(z), dim=1).numpy()
    np.testing.assert_allclose(probs, np.take_along_axis(p, idx.astype(np.int64), axis=1), rtol=2e-7)
    shift = np.full(E, 3.0, dtype=np.float32)
    idx2, probs2, z2 = oracle.predict(x, W1, W2, k=k, b2=shift)
    assert np.array_equal(idx, idx2)
    np.testing.assert_allclose(probs2, probs, rtol=1e-6)
    np.testing.assert_allclose(z2, z + 3.0, atol=1e-12)


def test_large_scores_do_not_overflow():
    d = 3
    I = np.eye(d, dtype=np.float32)
    x = np.array([[1000.0, 999.0, -1000.0]], dtype=np.float32)
    idx, probs, _ = oracle.predict(x, I, I, k=3)
    e = math.exp(-1.0)
    np.testing.assert_allclose(probs[0], [1 / (1 + e), e / (1 + e), 0.0], rtol=1e-6, atol=1e-30)
    assert idx.tolist() == [[0, 1, 2]]


# ---------------------------------------------------------------- bf16 hidden rounding, activations
def test_round_bf16_matches_torch_and_ties_to_even():
    g = np.random.default_rng(40)
    vals = (g.standard_normal(2000) * np.exp(g.uniform(-20, 20, 2000))).astype(np.float32)
    want = torch.from_numpy(vals).to(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([oracle.round_bf16(float(v)) for v in vals])
    assert np.array_equal(got, want)
    assert oracle.round_bf16(1.0 + 2.0 ** -8) == 1.0                 # midpoint -> even
    assert oracle.round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6  # midpoint -> even (up)
    assert oracle.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 1.0 + 2.0 ** -7   # just above midpoint
    assert oracle.round_bf16(-0.3) == -0.30078125
    assert oracle.round_bf16(0.0) == 0.0


def test_round_h_mode_rounds_hidden_once():
    T, d, r, E = 7, 32, 12, 5
    x, W1, W2 = (torch.from_numpy(_as_f32_exact(_rand(s, *sh))).to(torch.bfloat16)
                 for s, sh in ((41, (T, d)), (42, (r, d)), (43, (E, r))))
    xf, W1f, W2f = (a.to(torch.float32).numpy() for a in (x, W1, W2))
    _, _, z = oracle.predict(xf, W1f, W2f, k=1, round_h=True)
    h = torch.from_numpy(xf.astype(np.float64) @ W1f.astype(np.float64).T)
    # torch rounds double -> bf16 via float; use float-exact check where that is safe
    h_b = h.to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    want = h_b @ W2f.astype(np.float64).T
    np.testing.assert_allclose(z, want, rtol=0, atol=1e-12 * np.abs(want).max())
    _, _, z_exact = oracle.predict(xf, W1f, W2f, k=1, round_h=False)
    assert np.abs(z - z_exact).max() > 0            # the rounding really happened
    assert np.abs(z - z_exact).max() < 2.0 ** -8 * np.abs(h.numpy()).max() * np.abs(W2f).sum(axis=1).max()


@pytest.mark.parametrize("act,fn", [
    (oracle.ACT_SILU, lambda t: torch.nn.functional.silu(t)),
    (oracle.ACT_GELU, lambda t: torch.nn.functional.gelu(t, approximate="none")),
])
def test_activation_between_the_maps(act, fn):
    T, d, r, E = 6, 15, 11, 4
    x, W1, W2 = _as_f32_exact(_rand(44, T, d)), _as_f32_exact(_rand(45, r, d)), _as_f32_exact(_rand(46, E, r))
    b1 = _as_f32_exact(_rand(47, r))
    _, _, z = oracle.predict(x, W1, W2, k=1, b1=b1, act=act)
    h = torch.from_numpy(x.astype(np.float64) @ W1.astype(np.float64).T + b1.astype(np.float64))
    want = fn(h).numpy() @ W2.astype(np.float64).T
    np.testing.assert_allclose(z, want, rtol=0, atol=1e-12 * np.abs(want).max())


# ---------------------------------------------------------------- grouping
@pytest.mark.parametrize("T,k,E,seed", [(1, 1, 1, 0), (37, 6, 64, 1), (300, 2, 16, 2), (5, 8, 256, 3)])
def test_group_matches_numpy_counting_sort(T, k, E, seed):
    g = np.random.default_rng(seed)
    idx = g.integers(0, E, size=(T, k)).astype(np.int32)
    counts, offsets, pos, active, n_active, n_invalid = oracle.group_by_expert(idx, E)
    flat = idx.reshape(-1)
    assert np.array_equal(counts, np.bincount(flat, minlength=E))
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(counts)]))
    assert np.array_equal(pos, np.argsort(flat, kind="stable"))
    assert n_invalid == 0
    want_active = np.flatnonzero(counts)
    assert n_active == want_active.size
    assert np.array_equal(active[:n_active], want_active)
    assert np.all(active[n_active:] == -1)
    # invariants
    assert counts.sum() == T * k
    assert np.array_equal(np.sort(pos), np.arange(T * k))
    assert np.all(np.diff(flat[pos]) >= 0)
    for e in range(E):
        seg = pos[offsets[e]:offsets[e + 1]]
        assert np.all(flat[seg] == e) and np.all(np.diff(seg) > 0)


def test_group_on_topk_output_gives_k_distinct_groups_per_token():
    T, d, r, E, k = 30, 12, 8, 10, 4
    x, W1, W2 = _as_f32_exact(_rand(50, T, d)), _as_f32_exact(_rand(51, r, d)), _as_f32_exact(_rand(52, E, r))
    idx, _, _ = oracle.predict(x, W1, W2, k=k)
    counts, offsets, pos, *_ = oracle.group_by_expert(idx, E)
    tokens = pos // k
    owner = np.repeat(np.arange(E), counts)
    for t in range(T):
        assert len(set(owner[tokens == t])) == k


def test_group_skips_and_counts_invalid_ids():
    idx = np.array([[3, -1], [7, 0], [3, 8], [0, 3]], dtype=np.int32)
    counts, offsets, pos, active, n_active, n_invalid = oracle.group_by_expert(idx, 8)
    assert n_invalid == 2
    assert counts.tolist() == [2, 0, 0, 3, 0, 0, 0, 1]
    assert offsets.tolist() == [0, 2, 2, 2, 5, 5, 5, 5, 6]
    assert pos.tolist() == [3, 6, 0, 4, 7, 2, -1, -1]
    assert active[:n_active].tolist() == [0, 3, 7]


def test_group_empty():
    counts, offsets, pos, active, n_active, n_invalid = oracle.group_by_expert(
        np.zeros((0, 4), dtype=np.int32), 5)
    assert counts.tolist() == [0] * 5 and offsets.tolist() == [0] * 6
    assert pos.size == 0 and n_active == 0 and n_invalid == 0


# ---------------------------------------------------------------- accuracy counters
def test_score_hand_built_cases():
    E, T, k = 12, 5, 3
    ref = np.array([[0, 1, 2], [3, 4, 5], [6, 7, 8], [9, 10, 11], [0, 5, 10]], dtype=np.int32)
    assert oracle.score(ref, ref, E).tolist() == [T, T * k, T, T]
    perm = ref[:, [2, 0, 1]]
    assert oracle.score(perm, ref, E).tolist() == [T, T * k, T, T]
    disjoint = (ref + 3) % E
    disjoint[4] = [1, 2, 3]
    assert oracle.score(disjoint, ref, E).tolist() == [0, 0, 0, 0]
    one_swapped = ref.copy()
    one_swapped[:, 2] = [11, 11, 11, 0, 11]
    assert oracle.score(one_swapped, ref, E).tolist() == [0, T * (k - 1), 0, T]
    first_only = np.array([[0, 9, 10], [3, 9, 10], [6, 9, 10], [9, 0, 1], [0, 1, 2]], dtype=np.int32)
    assert oracle.score(first_only, ref, E).tolist() == [0, T, 0, T]
    last_only = first_only[:, [1, 2, 0]]
    assert oracle.score(last_only, ref, E).tolist() == [0, T, 0, 0]


def test_score_over_provisioned_superset():
    E = 20
    ref = np.array([[0, 1], [5, 6], [9, 3]], dtype=np.int32)
    wide = np.array([[7, 0, 1, 8], [5, 11, 12, 13], [3, 9, 14, 15]], dtype=np.int32)
    # rows 0 and 2 cover their labels, row 1 misses expert 6
    assert oracle.score(wide, ref, E).tolist() == [0, 5, 2, 2]


def test_score_duplicates_count_once_and_invalid_rows_add_nothing():
    E = 6
    ref = np.array([[1, 1, 2], [0, 1, 2], [0, 1, 2]], dtype=np.int32)
    idx = np.array([[2, 1, 2], [0, 1, 6], [0, -1, 2]], dtype=np.int32)
    # row 0: sets {1,2} == {1,2}; rows 1 and 2 hold an id outside [0, E)
    assert oracle.score(idx, ref, E).tolist() == [1, 2, 1, 1]


def test_score_against_python_sets():
    g = np.random.default_rng(60)
    E, T = 16, 400
    idx = np.stack([g.permutation(E)[:5] for _ in range(T)]).astype(np.int32)
    ref = np.stack([g.permutation(E)[:3] for _ in range(T)]).astype(np.int32)
    want = [0, 0, 0, 0]
    for p, q in zip(idx.tolist(), ref.tolist()):
        P, R = set(p), set(q)
        want[0] += P == R
        want[1] += len(P & R)
        want[2] += R <= P
        want[3] += p[0] in R
    assert oracle.score(idx, ref, E).tolist() == want


def test_paper_accuracy_definitions_on_a_worked_case():
    """Section 5.1: exact match needs all k experts; top-1 needs the best
    prediction among the k true experts; over-provisioning hits when the
    wider prediction covers them."""
    E = 64
    true6 = np.array([[4, 9, 17, 30, 41, 63]], dtype=np.int32)
    pred6 = np.array([[9, 4, 17, 30, 41, 62]], dtype=np.int32)      # five of six right
    pred10 = np.array([[9, 4, 17, 30, 41, 62, 63, 1, 2, 3]], dtype=np.int32)
    assert oracle.score(pred6, true6, E).tolist() == [0, 5, 0, 1]
    assert oracle.score(pred10, true6, E).tolist() == [0, 6, 1, 1]


# ---------------------------------------------------------------- activation profile (section 2.1)
def test_activation_profile_entropy_closed_forms():
    # uniform counts: entropy 1; a single active expert: 0; nothing counted or one expert: 0
    for E in (2, 7, 64, 1000):
        order, n, h = oracle.activation_profile(np.full(E, 5))
        assert n == E and order.tolist() == list(range(E)) and abs(h - 1.0) < 1e-13          # a sum of E terms: rounding ~ E * 2^-53
        one = np.zeros(E, dtype=np.int64); one[E // 2] = 9
        order, n, h = oracle.activation_profile(one)
        assert n == 1 and order[0] == E // 2 and (order[1:] == -1).all() and h == 0.0
        assert oracle.activation_profile(np.zeros(E, dtype=np.int64))[1:] == (0, 0.0)
    assert oracle.activation_profile(np.array([3]))[2] == 0.0
    # m equally used experts out of E: ln m / ln E
    c = np.zeros(16, dtype=np.int64); c[[1, 4, 9, 15]] = 7
    assert abs(oracle.activation_profile(c)[2] - math.log(4) / math.log(16)) < 1e-14
    # two experts with shares a and 1-a: the binary entropy function over ln 2
    a = 3 / 8
    want = -(a * math.log(a) + (1 - a) * math.log(1 - a)) / math.log(2)
    assert abs(oracle.activation_profile(np.array([3, 5]))[2] - want) < 1e-14
    # the skew the Phi-shaped workload plants (Zipf, s = 1.2) is well below the near-uniform 0.976 of the paper
    z = np.round(1e6 / np.arange(1, 17) ** 1.2).astype(np.int64)
    assert 0.5 < oracle.activation_profile(z)[2] < 0.9


def test_activation_profile_order_by_brute_force_and_invariances():
    g = np.random.default_rng(11)
    for E in (1, 2, 5, 33, 257):
        c = g.integers(0, 4, size=E) * g.integers(0, 3, size=E)          # many ties, many zeros
        order, n, h = oracle.activation_profile(c)
        # brute force: repeatedly take the largest remaining count, lowest id first
        rest = {e: int(c[e]) for e in range(E) if c[e] > 0}
        want = []
        while rest:
            best = max(rest.values())
            e = min(k for k, v in rest.items() if v == best)
            want.append(e); del rest[e]
        assert order[:n].tolist() == want and (order[n:] == -1).all() and n == len(want)
        # entropy ignores which expert holds which count, and the scale of the counts
        perm = g.permutation(E)
        assert abs(oracle.activation_profile(c[perm])[2] - h) < 1e-12
        assert abs(oracle.activation_profile(c * 7)[2] - h) < 1e-12
        # against the library routine for the same definition
        if E > 1 and c.sum() > 0:
            from scipy.stats import entropy as sp_entropy
            assert abs(float(sp_entropy(c[c > 0] / c.sum())) / math.log(E) - h) < 1e-12


# ---------------------------------------------------------------- confidence-driven over-provisioning (section 6)
def test_score_with_row_widths_against_sets_and_special_cases():
    g = np.random.default_rng(21)
    E, T, kp, kr = 24, 400, 7, 3
    ref = np.stack([g.choice(E, kr, replace=False) for _ in range(T)]).astype(np.int32)
    idx = np.stack([g.choice(E, kp, replace=False) for _ in range(T)]).astype(np.int32)
    idx[::3, :kr] = ref[::3]                                   # a third of the rows predict the labels first
    k_row = g.integers(-2, kp + 3, size=T).astype(np.int32)    # also out-of-range widths: clamped to [1, kp]
    want = np.zeros(4, dtype=np.int64)
    for t in range(T):
        w = min(max(int(k_row[t]), 1), kp)
        P, R = set(idx[t, :w].tolist()), set(ref[t].tolist())
        want += [P == R, len(P & R), R <= P, idx[t, 0] in R]
    assert oracle.score(idx, ref, E, k_row=k_row).tolist() == want.tolist()
    # the full width is the plain score; a constant width is the score of the truncated prediction
    assert oracle.score(idx, ref, E, k_row=np.full(T, kp)).tolist() == oracle.score(idx, ref, E).tolist()
    assert oracle.score(idx, ref, E, k_row=np.full(T, kr)).tolist() == oracle.score(idx[:, :kr], ref, E).tolist()
    # ids past a row's width are not looked at, even invalid ones
    bad = idx.copy(); bad[:, kr:] = -1
    assert oracle.score(bad, ref, E, k_row=np.full(T, kr)).tolist() == oracle.score(idx[:, :kr], ref, E).tolist()


def test_confidence_select_hand_cases_and_monotonicity():
    probs = np.array([[0.50, 0.30, 0.10, 0.05],     # p1/p2 = 3
                      [0.40, 0.35, 0.15, 0.05],     # 2.333
                      [0.30, 0.30, 0.30, 0.05],     # 1
                      [0.60, 0.20, 0.19, 0.01]],    # 1.0526
                     dtype=np.float32)
    idx = np.arange(16, dtype=np.int32).reshape(4, 4)
    k_row, out, n_wide = oracle.confidence_select(idx, probs, 2, 2.5)
    assert k_row.tolist() == [2, 4, 4, 4] and n_wide == 3
    assert out.tolist() == [[0, 1, -1, -1], [4, 5, 6, 7], [8, 9, 10, 11], [12, 13, 14, 15]]
    # ratio 1: sorted probabilities always pass, nobody is widened; a huge ratio widens everybody
    assert oracle.confidence_select(idx, probs, 2, 1.0)[0].tolist() == [2, 2, 2, 2]
    assert oracle.confidence_select(idx, probs, 2, 1e30)[2] == 4
    assert oracle.confidence_select(idx, probs, 1, 1.0)[0].tolist() == [1, 1, 1, 1]
    # the number of widened rows never falls as the required separation grows; the decision equals the
    # logit-margin rule z_a - z_b >= tau up to rounding (checked away from the boundary)
    g = np.random.default_rng(22)
    z = g.standard_normal((500, 16))
    order = np.argsort(-z, axis=1)[:, :6]
    zs = np.take_along_axis(z, order, axis=1)
    p = (np.exp(zs) / np.exp(z).sum(axis=1, keepdims=True)).astype(np.float32)
    last = -1
    for tau in (0.0, 0.05, 0.2, 0.5, 1.0, 2.0):
        k_row, _, n_wide = oracle.confidence_select(order.astype(np.int32), p, 3, math.exp(tau))
        assert n_wide >= last
        last = n_wide
        gap = zs[:, 2] - zs[:, 3]
        clear = np.abs(gap - tau) > 1e-4
        assert np.array_equal((k_row == 3)[clear], (gap >= tau)[clear])


# ---------------------------------------------------------------- confidence outputs (sections 6 and 4.4)
def _conf_case(seed=0, T=40, d=24, r=16, E=12, k=4):
    g = np.random.default_rng(seed)
    x = g.standard_normal((T, d)).astype(np.float32)
    W1 = (g.standard_normal((r, d)) / np.sqrt(d)).astype(np.float32)
    W2 = (g.standard_normal((E, r)) * 2 / np.sqrt(r)).astype(np.float32)
    idx, probs, z = oracle.predict(x, W1, W2, k)
    return x, W1, W2, idx, probs, z


def test_confidence_softmax_over_the_selection_sums_to_one_and_is_the_library_softmax_of_those_scores():
    import scipy.special
    _, _, _, idx, probs, z = _conf_case()
    soft, _, _ = oracle.confidence_outputs(z, idx)
    assert np.allclose(soft.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    sel = np.take_along_axis(z, idx.astype(np.int64), axis=1)
    assert np.allclose(soft, scipy.special.softmax(sel, axis=1), rtol=1e-13, atol=0)
    # and it is the all-expert softmax (eq. 1) renormalised over the selection
    p_all = scipy.special.softmax(z, axis=1)
    p_sel = np.take_along_axis(p_all, idx.astype(np.int64), axis=1)
    assert np.allclose(soft, p_sel / p_sel.sum(axis=1, keepdims=True), rtol=1e-12, atol=0)
    assert (np.diff(soft, axis=1) <= 0).all()                      # descending like the scores


def test_confidence_sigmoid_is_the_library_sigmoid():
    import scipy.special
    import torch
    _, _, _, idx, _, z = _conf_case(1)
    _, sig, _ = oracle.confidence_outputs(z, idx)
    sel = np.take_along_axis(z, idx.astype(np.int64), axis=1)
    assert np.allclose(sig, scipy.special.expit(sel), rtol=1e-14, atol=0)
    assert np.allclose(sig, torch.sigmoid(torch.from_numpy(sel)).numpy(), rtol=1e-14, atol=0)
    assert np.allclose(oracle.confidence_outputs(np.zeros((1, 3)), np.array([[0, 1]]))[1], 0.5)


def test_confidence_margin_is_the_gap_after_the_selection():
    x, W1, W2, idx, probs, z = _conf_case(2, k=4)
    _, _, margin = oracle.confidence_outputs(z, idx)
    # independent route: predict one expert more; the margin is the gap between its last two scores,
    # and (one softmax normaliser per row) the log of the ratio of their probabilities
    idx5, probs5, _ = oracle.predict(x, W1, W2, 5)
    gap = z[np.arange(z.shape[0]), idx5[:, 3]] - z[np.arange(z.shape[0]), idx5[:, 4]]
    assert np.array_equal(margin, gap)
    assert np.allclose(margin, np.log(probs5[:, 3].astype(np.float64) / probs5[:, 4]), rtol=0, atol=1e-5)
    assert (margin >= 0).all()
    # brute force on the full ordering
    for t in range(z.shape[0]):
        order = sorted(range(z.shape[1]), key=lambda e: (-z[t, e], e))
        assert margin[t] == z[t, order[3]] - z[t, order[4]]
    # hand case, an exact tie at the boundary, and k = E
    zz = np.array([[3.0, 1.0, 2.0, 0.5], [1.0, 1.0, 1.0, 0.0]])
    assert oracle.confidence_outputs(zz, np.array([[0, 2], [0, 1]]))[2].tolist() == [1.0, 0.0]
    assert np.isinf(oracle.confidence_outputs(zz, np.array([[0, 2, 1, 3], [0, 1, 2, 3]]))[2]).all()


# ---------------------------------------------------------------- BatchNorm folding (section 4.3, Architecture 1)
def test_batchnorm_folds_into_the_first_layer():
    import torch
    import torch.nn.functional as F
    g = np.random.default_rng(5)
    T, d, r, E, k = 30, 20, 14, 9, 3
    x = g.standard_normal((T, d)).astype(np.float32)
    W1 = (g.standard_normal((r, d)) / np.sqrt(d)).astype(np.float32)
    b1 = (0.2 * g.standard_normal(r)).astype(np.float32)
    W2 = (g.standard_normal((E, r)) / np.sqrt(r)).astype(np.float32)
    gamma, beta = 1 + 0.3 * g.standard_normal(r), 0.2 * g.standard_normal(r)
    mean, var, eps = 0.5 * g.standard_normal(r), 0.5 + g.random(r), 1e-5
    W1f, b1f = oracle.fold_batchnorm(W1, b1, gamma, beta, mean, var, eps)
    # the library's BatchNorm (inference form) on u = W1 x + b1, in float64
    t64 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    u = t64(x) @ t64(W1).T + t64(b1)
    bn = F.batch_norm(u, t64(mean), t64(var), weight=t64(gamma), bias=t64(beta), training=False, eps=eps)
    assert np.allclose(x.astype(np.float64) @ W1f.T + b1f, bn.numpy(), rtol=1e-12, atol=1e-12)
    # the whole Architecture-1 block through the oracle with folded weights = Linear, BN, exact GELU, Linear.
    # (the oracle takes float32 storage, so fold first, then round once, and feed both sides the same weights)
    W1s, b1s = W1f.astype(np.float32), b1f.astype(np.float32)
    _, _, z = oracle.predict(x, W1s, W2, k, b1=b1s, act=oracle.ACT_GELU)
    want = F.gelu(t64(x) @ t64(W1s).T + t64(b1s), approximate="none") @ t64(W2).T
    assert np.allclose(z, want.numpy(), rtol=1e-12, atol=1e-12)
    # no bias given = zero bias; unit statistics = identity
    W1n, b1n = oracle.fold_batchnorm(W1, None, np.ones(r), np.zeros(r), np.zeros(r), np.ones(r), 0.0)
    assert np.array_equal(W1n, W1.astype(np.float64)) and not b1n.any()
