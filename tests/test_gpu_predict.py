"""GPU parity of paep_predict with the CPU oracle, through the C ABI.
Small cases span several tiles and ragged tails on every kernel family and are
checked on every row.  The paper-shaped cases run at full token count with as
many layers as it takes for the launcher to choose the tile configuration and
r split it chooses for the whole model (the choice is asserted through
paep_predict_plan), and are checked on seeded row samples -- on every row for
the DeepSeek-V2-Lite shape."""
import numpy as np
import pytest
import torch

from paper_2511_10676_amd import binding as B
from paper_2511_10676_amd import configs, datagen

import oracle
import parity

pytestmark = pytest.mark.gpu
ACT_ID = {"none": 0, "silu": 1, "gelu": 2}


def _dev(a, dtype):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.cuda()


def _rand_layers(seed, L, T, d, r, E, dtype, bias=False, outliers=True):
    g = np.random.default_rng(seed)
    x = g.standard_normal((L, T, d)).astype(np.float32)
    if outliers and d >= 8:
        x[:, :, g.choice(d, 4, replace=False)] *= 8
    W1 = (g.standard_normal((L, r, d)) / np.sqrt(d)).astype(np.float32)
    W2 = (g.standard_normal((L, E, r)) / np.sqrt(r)).astype(np.float32)
    b1 = (0.3 * g.standard_normal((L, r))).astype(np.float32) if bias else None
    b2 = (0.5 * g.standard_normal((L, E))).astype(np.float32) if bias else None
    rs = lambda a: None if a is None else datagen.round_to_storage(a, dtype)
    return rs(x), rs(W1), rs(W2), rs(b1), rs(b2)


def _run_and_check(x, W1, W2, b1, b2, k, dtype, act="none", path="auto", rows=None, what=""):
    L = W1.shape[0]
    out = B.predict(_dev(x, dtype), _dev(W1, dtype), _dev(W2, dtype), k,
                    b1=None if b1 is None else _dev(b1, dtype), b2=None if b2 is None else _dev(b2, dtype),
                    act=act, path=path, want_logits=True)
    torch.cuda.synchronize()
    idx, probs, z = out.idx.cpu().numpy(), out.probs.cpu().numpy(), out.logits.cpu().numpy()
    tot, tot_m = parity.RowReport(), parity.RowReport()
    for l in range(L):
        xl = x[l] if x.shape[0] == L else x[0]
        rep, rep_m = parity.check_layer(xl, W1[l], W2[l], None if b1 is None else b1[l],
                                        None if b2 is None else b2[l], ACT_ID[act], k, dtype,
                                        idx[l], probs[l], z[l], rows=rows, what=f"{what} layer {l}")
        tot.add(rep)
        if rep_m:
            tot_m.add(rep_m)
    print(f"{what}: path={out.path} rows={tot.rows} strict={tot.strict} exempt={tot.exempt} "
          f"exempt_differ={tot.exempt_differ} max_err={tot.max_logit_err:.2e}*s_t prob_rel_err={tot.max_prob_rel_err:.2e} "
          f"(vs own scores {tot.max_prob_rel_err_own:.2e}, idx = rule(own scores) on {tot.own_topk_rows} rows) | "
          f"vs bf16-hidden oracle: strict={tot_m.strict} differ={tot_m.exempt_differ} "
          f"max_err={tot_m.max_logit_err:.2e}*s_t prob_rel_err={tot_m.max_prob_rel_err:.2e}", flush=True)
    assert tot.own_topk_rows == tot.rows
    return out, tot, tot_m


def _plan(T, d, r, E, k, L):
    return B.predict_plan(B.make_desc(T, d, r, E, k, L, B.BF16))


# ------------------------------------------------------------------ toy / simple path
def test_toy_fp32_all_rows():
    w = configs.get("toy")
    lay = datagen.make_layer(w, 0, w.prefill_T[0])
    out, tot, _ = _run_and_check(lay.x[None], lay.W1[None], lay.W2[None], None, None, w.k, "f32", what="toy")
    assert out.path == "simple"
    assert tot.exempt_differ == 0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("act", ["none", "silu", "gelu"])
def test_simple_path_odd_shapes(dtype, act):
    x, W1, W2, b1, b2 = _rand_layers(1, L=2, T=37, d=72, r=40, E=13, dtype=dtype, bias=True)
    out, *_ = _run_and_check(x, W1, W2, b1, b2, 5, dtype, act=act, path="simple", what=f"simple {dtype} {act}")
    assert out.path == "simple"


def test_simple_path_large_k_and_E():
    x, W1, W2, b1, b2 = _rand_layers(2, L=1, T=9, d=64, r=128, E=1000, dtype="f32")
    _run_and_check(x, W1, W2, None, None, 32, "f32", path="simple", what="simple E=1000 k=32")
    _run_and_check(x[:, :, :], W1, W2[:, :7], None, None, 7, "f32", path="simple", what="simple k=E=7")


# ------------------------------------------------------------------ decode path
@pytest.mark.parametrize("T", [1, 5, 16, 17, 33, 64])
def test_decode_path_small(T):
    x, W1, W2, b1, b2 = _rand_layers(10 + T, L=3, T=T, d=512, r=192, E=48, dtype="bf16", bias=True)
    out, *_ = _run_and_check(x, W1, W2, b1, b2, 6, "bf16", path="decode", what=f"decode T={T}")
    assert out.path == "decode"


@pytest.mark.parametrize("E,k,act", [(40, 8, "none"), (16, 2, "silu"), (250, 12, "gelu"), (8, 8, "none")])
def test_decode_path_ragged_experts(E, k, act):
    x, W1, W2, b1, b2 = _rand_layers(30 + E, L=2, T=7, d=256, r=128, E=E, dtype="bf16", bias=True)
    _run_and_check(x, W1, W2, b1, b2, k, "bf16", act=act, path="decode", what=f"decode E={E} k={k} {act}")


@pytest.mark.parametrize("T,d,r,E,k,act,L", [
    # r in whole slices of 128: a workgroup takes 128 hidden units, its waves split the rows and share the tokens
    # through a ring of LDS stages of 128 columns (otherwise: slices of 64, waves split d, covered by the cases
    # above).  The ring has three stages in calls of fewer than 384 slices (the cases with 3 layers) and two
    # beyond (the first two cases); d = 128 is a single stage, d = 384 and 640 a ragged last round, 250 experts
    # give a wave two expert blocks; up to 32 tokens a stage holds 32 token rows, beyond that 64
    (1, 256, 1024, 48, 6, "none", 48), (16, 384, 512, 48, 6, "gelu", 96), (17, 384, 256, 48, 6, "none", 3),
    (32, 640, 128, 48, 6, "silu", 3), (33, 384, 256, 250, 12, "gelu", 3), (48, 1024, 384, 64, 6, "none", 3),
    (64, 640, 256, 48, 8, "none", 3), (64, 128, 128, 16, 2, "silu", 3),
])
def test_decode_row_split_kernel(T, d, r, E, k, act, L):
    x, W1, W2, b1, b2 = _rand_layers(70 + T + d, L=L, T=T, d=d, r=r, E=E, dtype="bf16", bias=True)
    out, *_ = _run_and_check(x, W1, W2, b1, b2, k, "bf16", act=act, path="decode", what=f"decode rows T={T} d={d} r={r} E={E}")
    assert out.path == "decode"


def test_decode_shared_tokens_across_layers():
    x, W1, W2, _, _ = _rand_layers(50, L=4, T=3, d=256, r=64, E=32, dtype="bf16")
    _run_and_check(x[:1], W1, W2, None, None, 4, "bf16", path="decode", what="decode shared x")
    # the same through the row-split kernel (r = 256), no biases, both token-block sizes
    for T in (20, 50):
        x, W1, W2, _, _ = _rand_layers(52 + T, L=4, T=T, d=256, r=256, E=32, dtype="bf16")
        _run_and_check(x[:1], W1, W2, None, None, 4, "bf16", path="decode", what=f"decode rows shared x T={T}")


def test_decode_row_split_many_experts_and_wide_k():
    # 512 experts (eight per lane in the finalize kernel, four expert blocks per wave in the slices kernel) and k = 32
    x, W1, W2, b1, b2 = _rand_layers(57, L=2, T=40, d=256, r=256, E=512, dtype="bf16", bias=True)
    _run_and_check(x, W1, W2, b1, b2, 32, "bf16", act="silu", path="decode", what="decode rows E=512 k=32")
    x, W1, W2, b1, b2 = _rand_layers(58, L=2, T=9, d=128, r=128, E=130, dtype="bf16", bias=True)
    _run_and_check(x, W1, W2, b1, b2, 16, "bf16", path="decode", what="decode rows E=130 k=16")


# ------------------------------------------------------------------ prefill path
def test_prefill_shared_tokens_across_layers():
    x, W1, W2, _, _ = _rand_layers(51, L=5, T=333, d=256, r=256, E=48, dtype="bf16")
    _run_and_check(x[:1], W1, W2, None, None, 6, "bf16", path="prefill", what="prefill shared x")


@pytest.mark.parametrize("T", [1, 127, 128, 300])
def test_prefill_path_small(T):
    x, W1, W2, b1, b2 = _rand_layers(60 + T, L=2, T=T, d=256, r=256, E=64, dtype="bf16", bias=True)
    out, *_ = _run_and_check(x, W1, W2, b1, b2, 6, "bf16", path="prefill", what=f"prefill T={T}")
    assert out.path == "prefill"


@pytest.mark.parametrize("E,k,act", [(16, 2, "none"), (40, 8, "silu"), (128, 8, "none"), (256, 12, "gelu"), (200, 16, "none")])
def test_prefill_path_expert_counts(E, k, act):
    x, W1, W2, b1, b2 = _rand_layers(80 + E, L=2, T=150, d=128, r=384, E=E, dtype="bf16", bias=(act != "none"))
    _run_and_check(x, W1, W2, b1, b2, k, "bf16", act=act, path="prefill", what=f"prefill E={E} k={k} {act}")


def test_duplicate_w2_rows_tie_to_lower_id_on_every_path():
    for path, T in (("simple", 40), ("decode", 40), ("prefill", 200)):
        x, W1, W2, _, _ = _rand_layers(90, L=1, T=T, d=256, r=128, E=32, dtype="bf16")
        W2[0, 20] = W2[0, 3]
        out, tot, tot_m = _run_and_check(x, W1, W2, None, None, 6, "bf16", path=path, what=f"ties {path}")
        idx = out.idx.cpu().numpy()[0]
        z = out.logits.cpu().numpy()[0]
        assert np.array_equal(z[:, 3], z[:, 20])
        both = 0
        for row in idx.tolist():
            assert not (20 in row and 3 not in row)
            if 3 in row and 20 in row:
                both += 1
                assert row.index(20) == row.index(3) + 1
        assert both > 0


def test_results_are_reproducible_bit_for_bit():
    for path, T in (("decode", 33), ("prefill", 260), ("simple", 20)):
        x, W1, W2, _, _ = _rand_layers(95, L=2, T=T, d=256, r=128, E=64, dtype="bf16")
        xs, a, b = _dev(x, "bf16"), _dev(W1, "bf16"), _dev(W2, "bf16")
        outs = []
        for _ in range(3):
            o = B.predict(xs, a, b, 6, path=path, want_logits=True)
            torch.cuda.synchronize()
            outs.append((o.idx.cpu().numpy().tobytes(), o.probs.cpu().numpy().tobytes(), o.logits.cpu().numpy().tobytes()))
        assert outs[0] == outs[1] == outs[2], path


def test_empty_call():
    x, W1, W2, _, _ = _rand_layers(96, L=2, T=0, d=256, r=128, E=64, dtype="bf16")
    o = B.predict(_dev(x, "bf16"), _dev(W1, "bf16"), _dev(W2, "bf16"), 6)
    assert o.idx.shape == (2, 0, 6)


@pytest.mark.parametrize("E,k,r,d,L,T", [
    (64, 6, 256, 64, 4, 8229), (128, 8, 128, 64, 4, 8229), (256, 8, 384, 64, 4, 8229), (24, 2, 512, 64, 4, 8229),
    # d = 4096: the token tile is large enough that r is split over two workgroups per tile
    # (score tiles through the workspace, ticketed last-arriver reduction); so it is, further, in
    # every case here with fewer than 256 tiles
    (64, 6, 512, 4096, 4, 8300), (200, 8, 256, 4096, 4, 8300),
    # several chunks of r per tile, many layers, a single layer with many tiles
    (64, 6, 768, 64, 4, 8229), (64, 6, 1024, 64, 16, 8229), (128, 8, 640, 64, 9, 8229), (16, 2, 1280, 32, 1, 33000),
    # 64 < E <= 128 with r a multiple of 256: the 256 x 256 tile with the waves side by side
    (128, 8, 512, 64, 4, 8229), (100, 8, 256, 128, 4, 8229),
    # more than 64 experts with d = 96 and d = 32: three tiles and one tile per chunk of r, so the W2 slice in
    # LDS has to be waited for explicitly before each second product
    (128, 8, 256, 96, 4, 8229), (200, 8, 256, 32, 4, 8229),
])
def test_prefill_large_tile_configs_with_ragged_tail(E, k, r, d, L, T):
    """Enough tokens that the large-tile kernels are chosen, a token count that
    is not a multiple of any tile, every row checked."""
    x, W1, W2, b1, b2 = _rand_layers(70 + E, L=L, T=T, d=d, r=r, E=E, dtype="bf16", bias=True)
    out, *_ = _run_and_check(x, W1, W2, b1, b2, k, "bf16", path="prefill", what=f"prefill large tiles E={E} r={r} d={d}")
    assert out.path == "prefill"


@pytest.mark.parametrize("E,k,r,d,L,T,tile,groups,cpg", [
    # at least 256 token tiles: every workgroup walks all of r by itself, several chunks of it --
    # the configuration a whole model's worth of layers runs in
    (64, 6, 1024, 64, 8, 8229, "256x256", 1, 4),
    (128, 8, 1024, 64, 8, 8229, "256x256 wide", 1, 4),
    (256, 8, 512, 64, 8, 8229, "256x128", 1, 4),
    (200, 12, 640, 128, 8, 8229, "256x128", 1, 5),
    # 9 layers x 33 tiles = 256 + 41: the 41 tiles beyond the full round are cut along r into four pieces each
    # that meet in the workspace, the other 256 are not (same kernel, two parts of one grid)
    (64, 6, 1024, 64, 9, 8229, "256x256", 1, 4),
    (128, 8, 1024, 64, 9, 8229, "256x256 wide", 1, 4),
    (256, 8, 512, 64, 9, 8229, "256x128", 1, 4),
    # ... and with long rows (d = 4096) r split over two workgroups per tile, again at >= 256 tiles:
    # score tiles through the workspace, last arriver adds them (release/acquire through one thread's fences)
    (64, 6, 512, 4096, 8, 8300, "256x256", 2, 1),
])
def test_prefill_many_tiles_every_row(E, k, r, d, L, T, tile, groups, cpg):
    plan = _plan(T, d, r, E, k, L)
    assert (plan.path, plan.tile, plan.groups, plan.chunks_per_group) == ("prefill", tile, groups, cpg), plan
    x, W1, W2, b1, b2 = _rand_layers(170 + E + d, L=L, T=T, d=d, r=r, E=E, dtype="bf16", bias=True)
    out, *_ = _run_and_check(x, W1, W2, b1, b2, k, "bf16", what=f"prefill many tiles E={E} r={r} d={d} {plan}")
    assert out.path == "prefill"


# ------------------------------------------------------------------ paper-shaped, full size, sampled rows
def _paper_shaped(name, T, layers, n_rows, path):
    w = configs.get(name)
    L = len(layers)
    lays = [datagen.make_layer(w, l, T) for l in layers]
    x = np.stack([a.x for a in lays]); W1 = np.stack([a.W1 for a in lays]); W2 = np.stack([a.W2 for a in lays])
    b2 = np.stack([a.b2 for a in lays]) if lays[0].b2 is not None else None
    rows = None
    if n_rows < T:
        g = np.random.default_rng(1234 + T)
        rows = np.sort(np.concatenate([g.choice(T, n_rows - 2, replace=False), [0, T - 1]]))
        for a in lays:
            if a.tie_rows.size:
                rows = np.union1d(rows, a.tie_rows[:32])
    out, tot, tot_m = _run_and_check(x, W1, W2, None, b2, w.k, w.dtype, rows=rows, what=f"{name} T={T} L={L}")
    assert out.path == path
    return out, tot, tot_m, lays


@pytest.mark.parametrize("T", [1, 8, 64])
def test_deepseek_shaped_decode_all_layers(T):
    _paper_shaped("deepseek_v2_lite", T, range(26), T, "decode")


def test_deepseek_shaped_prefill_all_layers_every_row():
    w = configs.get("deepseek_v2_lite")
    plan = _plan(4096, w.d, w.r, w.E, w.k, w.L)
    assert (plan.tile, plan.groups, plan.chunks_per_group) == ("256x256", 1, 8), plan
    out, tot, tot_m, _ = _paper_shaped("deepseek_v2_lite", 4096, range(26), 4096, "prefill")
    assert tot.rows == 26 * 4096


@pytest.mark.parametrize("T", [1, 16, 64])
def test_qwen3_shaped_decode(T):
    _paper_shaped("qwen3_30b_a3b", T, range(0, 48, 6), T, "decode")


def test_qwen3_shaped_prefill_sampled():
    """Eight layers: 256 token tiles, which makes the launcher choose what it chooses for all 48."""
    w = configs.get("qwen3_30b_a3b")
    layers = [0, 6, 13, 17, 24, 30, 41, 47]
    full, part = _plan(8192, w.d, w.r, w.E, w.k, w.L), _plan(8192, w.d, w.r, w.E, w.k, len(layers))
    assert full == part and (part.tile, part.groups, part.chunks_per_group) == ("256x256 wide", 1, 8), (full, part)
    _paper_shaped("qwen3_30b_a3b", 8192, layers, 48, "prefill")


@pytest.mark.parametrize("T", [1, 32])
def test_phi_shaped_decode(T):
    _paper_shaped("phi_mini_moe", T, range(0, 32, 4), T, "decode")


def test_phi_shaped_prefill_sampled():
    w = configs.get("phi_mini_moe")
    layers = [0, 4, 9, 13, 20, 24, 27, 31]
    full, part = _plan(8192, w.d, w.r, w.E, w.k, w.L), _plan(8192, w.d, w.r, w.E, w.k, len(layers))
    assert full == part and part.groups == 2, (full, part)
    _paper_shaped("phi_mini_moe", 8192, layers, 32, "prefill")


def test_stress_shaped_prefill_sampled_with_near_ties():
    """Two layers of 32768 tokens: 256 token tiles, the launcher's choice for all 48 layers."""
    w = configs.get("stress")
    full, part = _plan(32768, w.d, w.r, w.E, w.k, w.L), _plan(32768, w.d, w.r, w.E, w.k, 2)
    assert full == part and (part.tile, part.groups, part.chunks_per_group) == ("256x128", 1, 32), (full, part)
    out, tot, tot_m, lays = _paper_shaped("stress", 32768, [0, 47], 64, "prefill")
    assert lays[0].tie_rows.size == 328
    # the planted rows sit inside the tolerance band; they must still be valid selections
    assert tot.exempt > 0


# ------------------------------------------------------------------ properties of the whole output at full size
def _check_output_properties(out, E, k):
    """What must hold for every row at any size: ids in range and distinct, probabilities positive,
    descending, and no more than the whole softmax mass."""
    idx, probs = out.idx, out.probs
    assert bool(((idx >= 0) & (idx < E)).all())
    srt = torch.sort(idx, dim=-1).values
    assert bool((srt[..., 1:] != srt[..., :-1]).all()), "an expert selected twice in one row"
    assert bool((probs > 0).all()) and bool(torch.isfinite(probs).all())
    assert bool((probs[..., :-1] >= probs[..., 1:]).all()), "probabilities not in descending order"
    assert float(probs.sum(dim=-1).max()) <= 1.0 + 1e-5


@pytest.mark.parametrize("name,T", [("deepseek_v2_lite", 4096), ("deepseek_v2_lite", 64), ("qwen3_30b_a3b", 8192),
                                    ("phi_mini_moe", 8192), ("stress", 32768)])
def test_full_size_outputs_have_the_required_properties_and_feed_grouping(name, T):
    """All layers, the benchmark's launch configuration, random weights generated on the device; every row of the
    output is checked for the properties above, and grouping/scoring of it for their conservation laws."""
    w = configs.get(name)
    g = torch.Generator(device="cuda"); g.manual_seed(7)
    x = torch.randn((w.L, T, w.d), device="cuda", generator=g).to(torch.bfloat16)
    W1 = (torch.randn((w.L, w.r, w.d), device="cuda", generator=g) / w.d ** 0.5).to(torch.bfloat16)
    W2 = (torch.randn((w.L, w.E, w.r), device="cuda", generator=g) / w.r ** 0.5).to(torch.bfloat16)
    out = B.predict(x, W1, W2, w.k)
    torch.cuda.synchronize()
    _check_output_properties(out, w.E, w.k)
    grp = B.group_by_expert(out.idx, w.E)
    sc = B.score(out.idx, out.idx, w.E)
    torch.cuda.synchronize()
    assert bool((grp.counts.sum(dim=1) == T * w.k).all()) and bool((grp.offsets[:, -1] == T * w.k).all())
    assert bool((grp.n_invalid == 0).all())
    # every position appears exactly once in a layer's token lists
    pos = torch.sort(grp.token_pos, dim=1).values
    assert bool((pos == torch.arange(T * w.k, device="cuda", dtype=torch.int32)[None, :]).all())
    # a prediction scored against itself: every row exact, every expert a hit
    assert sc.cpu().tolist() == [[T, T * w.k, T, T]] * w.L


# ------------------------------------------------------------------ the smallest shapes each kernel family accepts
@pytest.mark.parametrize("path,T,d,r,E,k,L", [
    ("prefill", 1, 32, 128, 1, 1, 1), ("prefill", 3, 32, 128, 2, 2, 3), ("prefill", 129, 64, 256, 5, 5, 1),
    ("prefill", 257, 32, 128, 33, 16, 2), ("decode", 1, 128, 64, 1, 1, 1), ("decode", 64, 128, 64, 3, 2, 2),
    ("decode", 2, 128, 128, 512, 32, 1), ("simple", 1, 8, 8, 1, 1, 1), ("simple", 2, 16, 8, 3, 3, 2),
])
def test_smallest_shapes(path, T, d, r, E, k, L):
    x, W1, W2, b1, b2 = _rand_layers(500 + T + E, L=L, T=T, d=d, r=r, E=E, dtype="bf16", bias=True, outliers=False)
    out, *_ = _run_and_check(x, W1, W2, b1, b2, k, "bf16", path=path, what=f"smallest {path} T={T} d={d} r={r} E={E}")
    assert out.path == path


# ------------------------------------------------------------------ activation counts from the predictor's epilogue
@pytest.mark.parametrize("path,T,d,r,E,k,L,dtype", [
    ("simple", 37, 72, 40, 13, 5, 2, "f32"), ("decode", 7, 256, 128, 40, 8, 3, "bf16"),
    ("decode", 64, 256, 128, 250, 12, 2, "bf16"), ("prefill", 300, 128, 384, 64, 6, 2, "bf16"),
    ("prefill", 700, 128, 256, 200, 16, 3, "bf16"), ("prefill", 8300, 64, 512, 64, 6, 4, "bf16"),
])
def test_counted_predict_adds_the_histogram_of_its_selections(path, T, d, r, E, k, L, dtype):
    x, W1, W2, _, _ = _rand_layers(900 + T, L=L, T=T, d=d, r=r, E=E, dtype=dtype)
    xs, a, b = _dev(x, dtype), _dev(W1, dtype), _dev(W2, dtype)
    plain = B.predict(xs, a, b, k, path=path)
    counts = torch.full((L, E), 3, dtype=torch.int32, device="cuda")          # not zero: the call adds
    out = B.predict(xs, a, b, k, path=path, counts=counts)
    out2 = B.predict(xs, a, b, k, path=path, counts=counts)                   # accumulates over calls
    torch.cuda.synchronize()
    assert out.path == path
    assert torch.equal(out.idx, plain.idx) and torch.equal(out.probs, plain.probs) and torch.equal(out2.idx, plain.idx)
    for l in range(L):
        hist = torch.bincount(out.idx[l].flatten().to(torch.int64), minlength=E).to(torch.int32)
        assert torch.equal(counts[l], 3 + 2 * hist), f"layer {l}"
    # against the oracle: its own selection on the rows where the selection is unambiguous (strict rows:
    # every gap among its top k+1 scores above the tolerance; in fp32 that is every row), the kernel's
    # selection on the others (those rows are checked for validity by the parity tests)
    tol = parity.TOL_MODEL if dtype == "bf16" else parity.TOL["f32"]
    n_strict = 0
    for l in range(L):
        idx_o, _, z_o = oracle.predict(x[l], W1[l], W2[l], k, round_h=(dtype == "bf16"))
        zs = -np.sort(-z_o, axis=1)
        s_t = np.abs(z_o).max(axis=1)
        strict = (zs[:, :min(k, E - 1)] - zs[:, 1:min(k, E - 1) + 1] >= tol * s_t[:, None]).all(axis=1)
        n_strict += int(strict.sum())
        mixed = np.where(strict[:, None], idx_o, out.idx[l].cpu().numpy())
        want = oracle.group_by_expert(mixed, E)[0]
        assert np.array_equal((counts[l].cpu().numpy() - 3) // 2, want), f"layer {l}"
    assert n_strict > 0.1 * L * T                 # the oracle's own selection decides a good share of the rows


# ------------------------------------------------------------------ confidence outputs (sections 6 and 4.4)
@pytest.mark.parametrize("path,T,d,r,E,k,L,dtype", [
    ("simple", 37, 72, 40, 13, 5, 2, "f32"), ("simple", 9, 64, 128, 40, 32, 1, "f32"),
    ("decode", 7, 256, 128, 40, 8, 3, "bf16"), ("decode", 64, 256, 128, 250, 12, 2, "bf16"),
    ("prefill", 300, 128, 384, 64, 6, 2, "bf16"), ("prefill", 700, 128, 256, 200, 15, 3, "bf16"),
    ("prefill", 8300, 64, 512, 128, 8, 4, "bf16"), ("prefill", 150, 128, 128, 8, 8, 1, "bf16"),
])
def test_confidence_outputs_match_the_oracle(path, T, d, r, E, k, L, dtype):
    x, W1, W2, _, _ = _rand_layers(1300 + T + k, L=L, T=T, d=d, r=r, E=E, dtype=dtype)
    xs, a, b = _dev(x, dtype), _dev(W1, dtype), _dev(W2, dtype)
    base = B.predict(xs, a, b, k, path=path, want_logits=True)
    outs = {m: B.predict(xs, a, b, k, path=path, prob=m, want_margin=True) for m in ("softmax", "softmax_topk", "sigmoid")}
    torch.cuda.synchronize()
    tol = parity.TOL["bf16" if dtype == "bf16" else "f32"]
    for m, o in outs.items():
        assert o.path == path, (m, o.path)
        assert torch.equal(o.idx, base.idx), m                    # all three scores are monotone: same selection
        assert torch.equal(o.margin, outs["softmax"].margin)
    assert torch.equal(outs["softmax"].probs, base.probs)
    zg = base.logits.cpu().numpy()
    idx = base.idx.cpu().numpy()
    for l in range(L):
        # (a) sharp, against the kernel's own scores: definitions evaluated in float64 on what it selected from
        soft_o, sig_o, margin_o = oracle.confidence_outputs(zg[l].astype(np.float64), idx[l])
        for name, want in (("softmax_topk", soft_o), ("sigmoid", sig_o)):
            got = outs[name].probs[l].cpu().numpy().astype(np.float64)
            assert np.abs(got - want).max() <= parity.PROB_TOL_OWN * np.abs(want).max() + 1e-30, (name, l)
            assert (np.abs(got - want) <= parity.PROB_TOL_OWN * want + 1e-12).all(), (name, l)
        mg = outs["softmax"].margin[l].cpu().numpy()
        if k < E:
            own = -np.sort(-zg[l], axis=1)
            assert np.array_equal(mg, own[:, k - 1] - own[:, k]), f"margin layer {l}"      # one fp32 subtraction
        else:
            assert np.isinf(mg).all() and (mg > 0).all()
        # (b) against the oracle's own scores, within what the score tolerance allows
        idx_r, _, z_r = oracle.predict(x[l], W1[l], W2[l], k)
        _, _, margin_r = oracle.confidence_outputs(z_r, idx_r)
        delta = tol * np.abs(z_r).max(axis=1)
        if k < E:
            assert (np.abs(mg - margin_r) <= 2 * delta + 1e-6).all(), f"margin vs oracle, layer {l}"
        soft_r, sig_r, _ = oracle.confidence_outputs(z_r, idx[l])          # the oracle's scores at the kernel's selection
        got = outs["softmax_topk"].probs[l].cpu().numpy()
        assert (np.abs(got - soft_r) <= (np.expm1(2 * delta)[:, None] + 2e-5) * soft_r + 1e-30).all()
        got = outs["sigmoid"].probs[l].cpu().numpy()
        assert (np.abs(got - sig_r) <= (np.expm1(delta)[:, None] + 2e-5) * sig_r + 1e-30).all()
    assert np.allclose(outs["softmax_topk"].probs.sum(dim=-1).cpu().numpy(), 1.0, atol=1e-5)


def test_margin_on_the_prefill_path_needs_room_for_one_more_candidate():
    x, W1, W2, _, _ = _rand_layers(1400, L=1, T=200, d=128, r=128, E=64, dtype="bf16")
    xs, a, b = _dev(x, "bf16"), _dev(W1, "bf16"), _dev(W2, "bf16")
    with pytest.raises(B.PaepError) as e:
        B.predict(xs, a, b, 16, path="prefill", want_margin=True)
    assert e.value.status == 8                                          # PAEP_ERR_UNSUPPORTED
    o = B.predict(xs, a, b, 16, want_margin=True, want_logits=True)      # AUTO falls back to a family that can
    torch.cuda.synchronize()
    assert o.path == "simple"
    own = -np.sort(-o.logits[0].cpu().numpy(), axis=1)
    assert np.array_equal(o.margin[0].cpu().numpy(), own[:, 15] - own[:, 16])


# ------------------------------------------------------------------ BatchNorm folded into the first layer (section 4.3)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fold_batchnorm_matches_the_oracle_and_feeds_predict(dtype):
    g = np.random.default_rng(77)
    L, T, d, r, E, k = 2, 50, 72, 40, 13, 5
    x, W1, W2, b1, _ = _rand_layers(78, L=L, T=T, d=d, r=r, E=E, dtype=dtype, bias=True)
    gamma = (1 + 0.3 * g.standard_normal((L, r))).astype(np.float32)
    beta = (0.2 * g.standard_normal((L, r))).astype(np.float32)
    mean = (0.5 * g.standard_normal((L, r))).astype(np.float32)
    var = (0.5 + g.random((L, r))).astype(np.float32)
    f32 = lambda v: torch.from_numpy(v).cuda()
    W1f, b1f = B.fold_batchnorm(_dev(W1, dtype), _dev(b1, dtype), f32(gamma), f32(beta), f32(mean), f32(var), 1e-5)
    W1n, _ = B.fold_batchnorm(_dev(W1, dtype), None, f32(gamma), f32(beta), f32(mean), f32(var), 1e-5)
    torch.cuda.synchronize()
    assert torch.equal(W1n, W1f)
    ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -22                   # one rounding to storage + fp32 arithmetic
    for l in range(L):
        Wo, bo = oracle.fold_batchnorm(W1[l], b1[l], gamma[l], beta[l], mean[l], var[l], 1e-5)
        assert (np.abs(W1f[l].float().cpu().numpy() - Wo) <= ulp * np.abs(Wo) + 1e-30).all()
        assert (np.abs(b1f[l].float().cpu().numpy() - bo) <= ulp * np.abs(bo) + 1e-6).all()
    # Architecture 1 end to end: folded weights + exact GELU through the predictor, against the oracle on the same weights
    Wh, bh = W1f.float().cpu().numpy(), b1f.float().cpu().numpy()
    _run_and_check(x, Wh, W2, bh, None, k, dtype, act="gelu", path="simple", what=f"arch-1 folded {dtype}")
