"""The synthetic-input generator: storage rounding, determinism and the
statistics the workload recipe promises."""
import numpy as np
import torch

from paper_2511_10676_amd import configs, datagen


def test_bf16_rounding_matches_torch():
    g = np.random.default_rng(0)
    a = (g.standard_normal(5000) * np.exp(g.uniform(-10, 10, 5000))).astype(np.float32)
    bits = datagen.f32_to_bf16_bits(a)
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, want)
    back = datagen.bf16_bits_to_f32(bits)
    assert np.array_equal(back, torch.from_numpy(a).to(torch.bfloat16).float().numpy())


def test_generator_is_keyed_and_reproducible():
    w = configs.get("toy")
    a, b = datagen.make_w1(w, 0), datagen.make_w1(w, 0)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, datagen.make_w1(w, 1))
    assert not np.array_equal(a, datagen.make_w1(w, 0, bank=1))


def test_toy_recipe():
    w = configs.get("toy")
    lay = datagen.make_layer(w, 0, 512)
    assert lay.x.shape == (512, 256) and lay.W1.shape == (64, 256) and lay.W2.shape == (16, 64)
    assert lay.b2 is None and lay.ref.shape == (512, 2)
    # exactly four outlier channels carry 8x the scale
    ch_std = lay.x.std(axis=0)
    assert np.sum(ch_std > 4.0) == 4 and np.sum(ch_std < 1.5) == 252
    assert abs(lay.W1.std() * np.sqrt(256) - 1) < 0.05
    assert abs(lay.W2.std() * np.sqrt(64) - 1) < 0.1
    assert np.all((lay.ref >= 0) & (lay.ref < 16))
    assert np.all(lay.ref[:, 0] != lay.ref[:, 1])


def test_bf16_workload_values_are_representable_and_rms_scaled():
    w = configs.get("deepseek_v2_lite")
    x = datagen.make_x(w, 3, 16)
    assert np.array_equal(x, datagen.round_to_storage(x, "bf16"))
    rms = np.sqrt(np.mean(x.astype(np.float64) ** 2, axis=1))
    assert np.all(np.abs(rms - 1) < 5e-3)
    assert w.outliers == 4


def test_zipf_bias_skews_selection():
    w = configs.get("phi_mini_moe")
    b2 = datagen.make_b2(w, 0)
    assert b2.shape == (16,) and abs(float(b2.astype(np.float64).mean())) < 0.01
    srt = np.sort(b2)[::-1]
    # log-probabilities fall like -1.2 * beta * log(rank)
    np.testing.assert_allclose(srt[0] - srt[1], datagen.ZIPF_S * datagen.ZIPF_BETA * np.log(2), atol=0.01)


def test_near_tie_planting_small():
    w = configs.Workload("mini_stress", 9, L=1, d=128, r=64, E=32, k=4, dtype="bf16",
                         near_tie_frac=0.25, exact_tie_rows=1)
    lay = datagen.make_layer(w, 0, 64)
    assert lay.tie_rows.size == 16
    M = lay.W2.astype(np.float64) @ lay.W1.astype(np.float64)
    z = lay.x.astype(np.float64) @ M.T
    s = -np.sort(-z, axis=1)
    gap = s[:, w.k - 1] - s[:, w.k]
    assert np.mean(np.abs(gap[lay.tie_rows]) < 1e-3) >= 0.75
    others = np.setdiff1d(np.arange(64), lay.tie_rows)
    assert np.median(gap[others]) > 10 * np.median(np.abs(gap[lay.tie_rows]))
    # one duplicated W2 row pair
    dup = [(a, b) for a in range(w.E) for b in range(a + 1, w.E) if np.array_equal(lay.W2[a], lay.W2[b])]
    assert len(dup) == 1
