"""Seeded input generators: determinism, storage-type exactness, index structure."""
import numpy as np

from paper_2604_18103_amd import inputs as I


def test_bf16_rounding_ties_to_even_and_is_idempotent():
    a = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7, -3.14159, 1e-20, 65504.0], np.float32)
    r = I.round_to_bf16(a)
    assert r[0] == 1.0
    assert r[1] == 1.0                       # halfway between 1 and 1+2^-7: even mantissa wins
    assert r[2] == np.float32(1.0 + 2 ** -6)  # halfway between 1+2^-7 and 1+2^-6: even wins
    assert r[3] == np.float32(1.0 + 2 ** -7)
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    assert np.array_equal(I.round_to_bf16(r), r)
    assert np.all(np.abs(r - a) <= np.abs(a) * 2 ** -8)


def test_layer_inputs_are_deterministic_and_exact_in_storage_type():
    cfg = I.scaled(I.CONFIGS["qwen_8k"], 96)
    a, b = I.make_layer_inputs(cfg), I.make_layer_inputs(cfg)
    for key in a:
        assert np.array_equal(a[key], b[key])
    for key in ("x", "q", "k", "v", "w_o"):
        assert a[key].dtype == np.float32
        assert np.all((a[key].view(np.uint32) & 0xFFFF) == 0)
    assert a["x"].shape == (96, 3584) and a["q"].shape == (96, 28, 128)
    assert a["k"].shape == (96, 4, 128) and a["w_o"].shape == (3584, 3584)
    assert abs(float(a["w_o"].std()) * np.sqrt(3584) - 1.0) < 0.01


def test_active_idx_sorted_unique_subset():
    idx = I.make_active_idx(1000, 400, seed=2)
    assert idx.dtype == np.int32 and idx.shape == (400,)
    assert np.all(np.diff(idx) > 0) and idx[0] >= 0 and idx[-1] < 1000
    assert np.array_equal(I.make_active_idx(64, 64, 0), np.arange(64))


def test_row_scale_is_heavy_tailed():
    cfg = I.scaled(I.CONFIGS["tiny_f32"], 4000)
    x = I.make_hidden(cfg)
    norms = np.sqrt((x.astype(np.float64) ** 2).sum(1)) / np.sqrt(cfg.d)
    logn = np.log(norms)
    assert abs(logn.mean()) < 0.1 and abs(logn.std() - 1.5) < 0.1
    mix = I.scaled(I.CONFIGS["llama_128k_40"], 3000, d=64, n_q_heads=1, n_kv_heads=1)
    lm = np.log(np.sqrt((I.make_hidden(mix).astype(np.float64) ** 2).sum(1)) / 8.0)
    assert 0.6 < lm.mean() < 1.0             # 0.8 * 1 + 0.2 * 0


def test_percentile_tau_splits_at_h():
    rng = np.random.default_rng(0)
    s = rng.random(1001).astype(np.float32).astype(np.float64)
    tau, h = I.percentile_tau(s, 0.3)
    assert h == 300 and int((s < tau).sum()) == 300
    assert I.percentile_tau(s, 0.0) == (0.0, 0)


def test_sample_rows_cover_edges():
    r = I.sample_rows(1000, 64, seed=1)
    assert r[0] == 0 and r[-1] == 999 and np.all(np.diff(r) > 0)
    assert {127, 128, 129}.issubset(set(r.tolist()))
    assert I.sample_rows(5, 64, seed=1).tolist() == [0, 1, 2, 3, 4]
