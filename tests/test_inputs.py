"""Host-side checks of the seeded input generators (CPU only)."""
import numpy as np

from paper_2508_02317_amd import inputs as I


def test_bf16_rounding_is_nearest_even():
    a = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -3.14159, 0.0, 1e-30], dtype=np.float32)
    r = I.round_to_bf16(a)
    assert r[0] == 1.0
    assert r[1] == 1.0                       # tie -> even mantissa
    assert r[2] == np.float32(1.0 + 2 ** -7)
    assert r[3] == np.float32(1.0 + 2 ** -6)  # tie -> even mantissa (up)
    assert abs(r[4] - a[4]) <= abs(a[4]) * 2 ** -8
    assert np.array_equal(I.round_to_bf16(r), r)
    assert np.array_equal(I.from_bf16_bits(I.bf16_bits(r)), r)


def test_generators_are_seeded_and_shape_independent():
    cfg = I.CONFIGS["tiny"]
    a = I.make_inputs(cfg); b = I.make_inputs(cfg)
    for key in a:
        assert np.array_equal(a[key], b[key])
    # changing f must not change X, the router or the logits
    c = I.make_inputs(I.scaled(cfg, f=64))
    assert np.array_equal(a["X"], c["X"]) and np.array_equal(a["logits"], c["logits"])
    assert a["logits"].dtype == np.float32 and a["logits"].shape == (cfg.T, cfg.E)
    assert abs(a["Wg"].std() - 0.02) < 2e-3 and abs(a["X"].std() - 1.0) < 2e-2
    ref = (a["X"].astype(np.float64) @ a["Wr"].astype(np.float64)).astype(np.float32)
    assert np.array_equal(ref, a["logits"])


def test_bf16_config_values_are_representable():
    cfg = I.scaled(I.CONFIGS["small"], T=64, d=64, f=32, E=4)
    a = I.make_inputs(cfg)
    for key in ("X", "Wr", "Wg", "Wu", "Wd", "dY"):
        assert np.array_equal(I.round_to_bf16(a[key]), a[key]), key


def test_mixed_modal_rows_have_two_scales():
    cfg = I.scaled(I.CONFIGS["a3b_long"], d=64, f=32, E=8, k=2)
    s = I.modality_row_scale(cfg)
    assert set(np.unique(s).tolist()) == {1.0, 4.0}
    frac = float(np.mean(s == 4.0))
    assert 0.3 < frac < 0.7
    runs = np.diff(np.flatnonzero(np.diff(s) != 0))
    assert runs.min() >= 64 and runs.max() <= 2048
    X = I.make_inputs(cfg)["X"]
    assert abs(X[s == 1.0].std() - 1.0) < 0.05 and abs(X[s == 4.0].std() - 4.0) < 0.2


def test_zipf_rank_spreads_hot_experts_over_gpus():
    r = I.zipf_rank(np.arange(128))
    assert sorted(r.tolist()) == list(range(1, 129))
    assert r[0] == 1 and r[16] == 2 and r[1] == 9


def test_select_local_share_is_pure_selection():
    idx = np.array([[3, 20, 1], [40, 41, 42], [0, 17, 2]], dtype=np.int32)
    w = np.arange(9, dtype=np.float64).reshape(3, 3)
    tok, li, lw = I.select_local_share(idx, w, 16, 4)
    assert tok.tolist() == [0, 0, 2, 2]
    assert li[:, 0].tolist() == [3, 1, 0, 2]
    assert lw[:, 0].tolist() == [0.0, 2.0, 6.0, 8.0]
