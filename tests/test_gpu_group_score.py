"""GPU parity of paep_group_by_expert and paep_score with the CPU oracle:
integer work, compared bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_10676_amd import binding as B
from paper_2511_10676_amd import configs, datagen

pytestmark = pytest.mark.gpu


def _skewed_idx(g, L, T, k, E, zipf=1.2):
    """Per-token k distinct experts, popularity ~ Zipf (the Gumbel top-k trick)."""
    logp = -zipf * np.log(np.arange(1, E + 1))
    out = np.empty((L, T, k), dtype=np.int32)
    for l in range(L):
        perm = g.permutation(E)
        keys = logp[None, :] + g.gumbel(size=(T, E))
        out[l] = perm[np.argsort(-keys, axis=1)[:, :k]]
    return out


def _check_group(idx, E):
    L, T, k = idx.shape
    got = B.group_by_expert(torch.from_numpy(idx).cuda(), E)
    torch.cuda.synchronize()
    for l in range(L):
        counts, offsets, pos, active, n_active, n_invalid = oracle.group_by_expert(idx[l], E)
        assert np.array_equal(got.counts[l].cpu().numpy(), counts), f"counts layer {l}"
        assert np.array_equal(got.offsets[l].cpu().numpy(), offsets), f"offsets layer {l}"
        assert np.array_equal(got.token_pos[l].cpu().numpy(), pos), f"token_pos layer {l}"
        assert np.array_equal(got.active[l].cpu().numpy(), active), f"active layer {l}"
        assert int(got.n_active[l]) == n_active and int(got.n_invalid[l]) == n_invalid
    return got


@pytest.mark.parametrize("T,k,E,L", [
    (1, 1, 1, 1), (0, 6, 64, 2), (1, 6, 64, 3), (9, 7, 64, 1), (64, 1, 16, 2), (65, 1, 16, 2),
    (171, 6, 64, 2), (1024, 1, 2, 1), (1025, 1, 300, 1), (4096, 6, 64, 3), (8192, 8, 128, 2),
    (8192, 2, 16, 2), (32768, 8, 256, 1), (700, 3, 1000, 2),
    # either side of the single-launch limit of 32768 selections per layer
    (4096, 8, 128, 2), (4097, 8, 128, 2), (32768, 1, 64, 1), (32769, 1, 64, 2), (2000, 16, 1024, 2), (65537, 1, 64, 2),
    # the single-launch kernel cuts a layer into 2, 4 or 8 independent parts: either side of each switch, ragged
    # lengths, and a layer too short for its last part to hold anything
    (4096, 1, 64, 2), (4097, 1, 64, 2), (8192, 1, 64, 2), (8193, 1, 64, 1), (16384, 1, 200, 1), (16385, 1, 256, 2),
    (2731, 6, 64, 3), (5461, 6, 16, 2), (4099, 7, 100, 2), (2048, 1, 256, 2), (2049, 1, 256, 2), (2049, 1, 257, 1),
])
def test_group_matches_oracle(T, k, E, L):
    g = np.random.default_rng(T * 31 + k * 7 + E)
    idx = _skewed_idx(g, L, T, min(k, E), E) if T > 0 else np.zeros((L, 0, k), dtype=np.int32)
    _check_group(idx, E)


@pytest.mark.parametrize("T,k,E,L,lo", [
    # layers beyond 32768 selections: parts of 8192 positions counted by a launch of their own
    (8192, 8, 128, 3, 0), (8193, 8, 128, 2, 0), (32768, 8, 256, 2, 0), (4097, 8, 1024, 2, -2), (40000, 4, 1000, 1, 0),
    (32769, 1, 7, 2, -1), (9000, 10, 64, 2, 0),
    # more than 64 parts of 8192: longer parts (35 of 16384; 63 and 64 of 32768)
    (70000, 8, 64, 1, 0), (258000, 8, 256, 1, 0), (262144, 8, 128, 1, -1),
    # more than 64 parts of the longest kind LDS allows: the columns get a launch of their own
    (262200, 8, 64, 2, -1), (66000, 16, 1024, 1, 0), (300000, 9, 300, 1, -3),
])
def test_group_long_layers(T, k, E, L, lo):
    g = np.random.default_rng(T + k + E)
    hi = E + (3 if lo < 0 else 0)                                  # lo < 0: ids outside [0, E) among them
    idx = g.integers(lo, hi, size=(L, T, k)).astype(np.int32)
    idx[:, : T // 3][idx[:, : T // 3] % 5 == 1] = E - 1            # uneven groups, more so early in the layer
    need = B.group_workspace_bytes(L, T, k, E)
    assert need > 0
    got = _check_group(idx, E)
    assert (int(got.n_invalid.sum()) > 0) == (lo < 0)


def test_group_with_invalid_ids_and_repeats():
    g = np.random.default_rng(5)
    idx = g.integers(-3, 70, size=(2, 3000, 6)).astype(np.int32)     # ids outside [0, 64) on purpose
    got = _check_group(idx, 64)
    assert int(got.n_invalid.sum()) > 0
    one = np.full((1, 5000, 8), 7, dtype=np.int32)                  # everything lands in one group
    _check_group(one, 128)
    # the same in the sizes where a layer is cut into parts: -2 and other negative ids among the invalid ones,
    # valid ids only in the first part (so the later parts own nothing but a stretch of the -1 tail)
    idx = g.integers(-3, 70, size=(2, 4000, 6)).astype(np.int32)
    idx[:, 700:] = np.where(idx[:, 700:] % 2 == 0, -2, 64 + idx[:, 700:] % 5)
    got = _check_group(idx, 64)
    assert int(got.n_invalid[0]) > 3300 * 6
    _check_group(np.full((2, 3000, 8), 5, dtype=np.int32), 6)


def test_group_is_reproducible():
    g = np.random.default_rng(6)
    idx = torch.from_numpy(_skewed_idx(g, 2, 5000, 8, 128)).cuda()
    a = B.group_by_expert(idx, 128)
    b = B.group_by_expert(idx, 128)
    torch.cuda.synchronize()
    for u, v in zip(a, b):
        assert torch.equal(u, v)


@pytest.mark.parametrize("T,kp,kr,E,L", [
    (0, 6, 6, 64, 2), (1, 2, 2, 16, 1), (255, 6, 6, 64, 2), (257, 10, 6, 64, 3), (4096, 6, 6, 64, 2),
    (5000, 12, 8, 128, 2), (3000, 8, 8, 256, 1), (999, 3, 2, 16, 4), (500, 32, 5, 1000, 1),
    # either side of the single-launch limit of 4096 tokens per layer; more than 8 ids per row
    (4097, 6, 6, 64, 2), (20000, 8, 8, 256, 1), (6000, 20, 9, 700, 1), (300, 9, 32, 64, 2),
    # nine to sixteen ids per row: one workgroup per layer up to 2048 rows, several beyond; over sixteen: 1024
    (2048, 16, 16, 64, 2), (2049, 12, 8, 128, 2), (4096, 10, 6, 64, 3), (1024, 20, 9, 64, 2), (1025, 20, 9, 300, 1),
    (1023, 6, 6, 64, 1), (8191, 2, 2, 16, 2),
])
def test_score_matches_oracle(T, kp, kr, E, L):
    g = np.random.default_rng(T + kp * 3 + E)
    ref = _skewed_idx(g, L, T, kr, E) if T else np.zeros((L, 0, kr), np.int32)
    idx = np.empty((L, T, kp), dtype=np.int32)
    for l in range(L):
        for t in range(T):
            # mostly the label set (shuffled, padded with other experts), sometimes perturbed
            keep = ref[l, t].copy()
            if g.random() < 0.4:
                keep[g.integers(kr)] = g.integers(E)
            pool = np.setdiff1d(np.arange(E), keep)
            row = np.concatenate([np.unique(keep), g.permutation(pool)])[:kp]
            idx[l, t] = g.permutation(row)
    got = B.score(torch.from_numpy(idx).cuda(), torch.from_numpy(ref).cuda(), E)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    for l in range(L):
        want = oracle.score(idx[l], ref[l], E)
        assert got[l].tolist() == want.tolist(), f"layer {l}"


def test_score_hand_cases_and_invalid_rows():
    E = 12
    ref = np.array([[[0, 1, 2], [3, 4, 5], [6, 7, 8], [9, 10, 11], [0, 5, 10]]], dtype=np.int32)
    idx = np.array([[[2, 1, 0], [3, 4, 11], [6, 6, 6], [12, 10, 9], [1, 2, 3]]], dtype=np.int32)
    got = B.score(torch.from_numpy(idx).cuda(), torch.from_numpy(ref).cuda(), E).cpu().numpy()[0]
    assert got.tolist() == oracle.score(idx[0], ref[0], E).tolist() == [1, 6, 1, 3]


def test_toy_end_to_end_matches_oracle_and_golden():
    import json, os
    w = configs.get("toy")
    lay = datagen.make_layer(w, 0, w.prefill_T[0])
    dev = lambda a: torch.from_numpy(a).cuda()
    out = B.predict(dev(lay.x), dev(lay.W1), dev(lay.W2), w.k)
    grp = B.group_by_expert(out.idx, w.E)
    sc = B.score(out.idx, dev(lay.ref)[None], w.E)
    torch.cuda.synchronize()
    idx_ref, probs_ref, _ = oracle.predict(lay.x, lay.W1, lay.W2, w.k)
    # fp32 storage: the GPU selection equals the oracle's wherever the oracle's gap exceeds the tolerance;
    # on this seed that is every row
    assert np.array_equal(out.idx[0].cpu().numpy(), idx_ref)
    counts, offsets, pos, active, n_active, _ = oracle.group_by_expert(idx_ref, w.E)
    assert np.array_equal(grp.counts[0].cpu().numpy(), counts)
    assert np.array_equal(grp.token_pos[0].cpu().numpy(), pos)
    with open(os.path.join(os.path.dirname(__file__), "golden", "toy_oracle.json")) as f:
        gold = json.load(f)
    assert sc[0].cpu().numpy().tolist() == gold["score_k2_vs_ref"] == oracle.score(idx_ref, lay.ref, w.E).tolist()


# ---------------------------------------------------------------- activation profile
@pytest.mark.parametrize("E,L,T,k", [(1, 2, 50, 1), (2, 1, 100, 1), (16, 3, 4000, 2), (64, 4, 4096, 6), (257, 2, 900, 8),
                                     (1024, 2, 3000, 16), (64, 2, 0, 6)])
def test_activation_profile_matches_oracle(E, L, T, k):
    g = np.random.default_rng(E * 5 + T)
    idx = _skewed_idx(g, L, T, min(k, E), E) if T > 0 else np.zeros((L, 0, k), dtype=np.int32)
    grp = B.group_by_expert(torch.from_numpy(idx).cuda(), E)
    prof = B.activation_profile(grp.counts)
    torch.cuda.synchronize()
    for l in range(L):
        counts = oracle.group_by_expert(idx[l], E)[0]
        order, n_active, entropy = oracle.activation_profile(counts)
        assert np.array_equal(prof.order[l].cpu().numpy(), order), f"order layer {l}"
        assert int(prof.n_active[l]) == n_active
        # both sides sum at most 1024 terms of magnitude < 1 in double, in different orders
        assert abs(float(prof.entropy[l]) - entropy) <= 1e-12, f"entropy layer {l}"


def test_activation_profile_ties_and_uniform():
    c = torch.tensor([[5, 0, 5, 9, 0, 5, 9, 1], [3] * 8], dtype=torch.int32, device="cuda")
    prof = B.activation_profile(c)
    torch.cuda.synchronize()
    assert prof.order[0].tolist() == [3, 6, 0, 2, 5, 7, -1, -1] and prof.n_active.tolist() == [6, 8]
    assert prof.order[1].tolist() == list(range(8)) and abs(float(prof.entropy[1]) - 1.0) < 1e-13
    want = oracle.activation_profile(c[0].cpu().numpy())
    assert abs(float(prof.entropy[0]) - want[2]) <= 1e-12


# ---------------------------------------------------------------- confidence-driven over-provisioning
def _sorted_softmax(g, L, T, kp, E, temp):
    """Synthetic predictor output: the kp largest softmax values of random scores, and their experts."""
    z = g.standard_normal((L, T, E)) * temp
    order = np.argsort(-z, axis=2, kind="stable")[:, :, :kp]
    zs = np.take_along_axis(z, order, axis=2)
    p = np.exp(zs - z.max(axis=2, keepdims=True)) / np.exp(z - z.max(axis=2, keepdims=True)).sum(axis=2, keepdims=True)
    return order.astype(np.int32), p.astype(np.float32)


@pytest.mark.parametrize("L,T,E,kp,kb,kr,ratio", [
    (2, 1, 16, 3, 2, 2, 1.5), (3, 50, 64, 10, 6, 6, 1.2), (2, 4097, 64, 10, 6, 6, 1.05), (1, 700, 128, 12, 8, 8, 1.0),
    (4, 63, 16, 3, 2, 2, 3.0), (2, 300, 300, 32, 1, 5, 1.3), (2, 0, 64, 10, 6, 6, 1.2),
])
def test_confidence_select_group_and_score_match_oracle(L, T, E, kp, kb, kr, ratio):
    g = np.random.default_rng(L * 1000 + T + kp)
    idx, probs = _sorted_softmax(g, L, T, kp, E, temp=1.5) if T else (np.zeros((L, 0, kp), np.int32), np.zeros((L, 0, kp), np.float32))
    ref = np.ascontiguousarray(idx[:, :, :kr]).copy()
    if T:
        flip = g.random((L, T)) < 0.3                        # some labels differ from the prediction's head
        ref[flip, kr - 1] = idx[flip, kp - 1]
    got = B.confidence_select(torch.from_numpy(idx).cuda(), torch.from_numpy(probs).cuda(), kb, ratio)
    grp = B.group_by_expert(got.idx, E)
    sc = B.score(got.idx, torch.from_numpy(ref).cuda(), E, k_row=got.k_row)
    torch.cuda.synchronize()
    for l in range(L):
        k_row, idx_out, n_wide = oracle.confidence_select(idx[l], probs[l], kb, ratio)
        assert np.array_equal(got.k_row[l].cpu().numpy(), k_row), f"k_row layer {l}"
        assert np.array_equal(got.idx[l].cpu().numpy(), idx_out), f"idx_out layer {l}"
        assert int(got.n_wide[l]) == n_wide
        counts, offsets, pos, active, n_active, n_invalid = oracle.group_by_expert(idx_out, E)
        assert np.array_equal(grp.counts[l].cpu().numpy(), counts) and np.array_equal(grp.token_pos[l].cpu().numpy(), pos)
        assert int(grp.n_invalid[l]) == n_invalid == int((kp - k_row).sum())
        assert sc[l].cpu().numpy().tolist() == oracle.score(idx_out, ref[l], E, k_row=k_row).tolist()


def test_score_rows_with_arbitrary_widths():
    g = np.random.default_rng(77)
    L, T, E, kp, kr = 2, 5000, 64, 9, 4
    idx = np.stack([[g.choice(E, kp, replace=False) for _ in range(T)] for _ in range(L)]).astype(np.int32)
    ref = np.stack([[g.choice(E, kr, replace=False) for _ in range(T)] for _ in range(L)]).astype(np.int32)
    ref[:, ::2] = idx[:, ::2, :kr]
    k_row = g.integers(-1, kp + 2, size=(L, T)).astype(np.int32)
    sc = B.score(torch.from_numpy(idx).cuda(), torch.from_numpy(ref).cuda(), E, k_row=torch.from_numpy(k_row).cuda())
    torch.cuda.synchronize()
    for l in range(L):
        assert sc[l].cpu().numpy().tolist() == oracle.score(idx[l], ref[l], E, k_row=k_row[l]).tolist()
