"""The seeded input generators: determinism, shapes, dtypes, value ranges."""
import numpy as np

import workloads as W


def test_bf16_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0], dtype=np.float32)
    back = W.f32_from_bf16_bits(W.bf16_bits_from_f32(x))
    assert back.tolist() == [1.0, 1.0, 1.015625, -2.5, 0.0]


def test_weights_are_reproducible_and_name_keyed():
    wl = W.get_workload("C1")
    a = W.make_weights(wl.shape, wl.seed)
    b = W.make_weights(wl.shape, wl.seed, names=["layers.1.w_up"])
    assert np.array_equal(a["layers.1.w_up"], b["layers.1.w_up"])
    assert a["layers.1.w_up"].shape == (704, 256) and a["layers.1.w_up"].dtype == np.float32
    assert abs(float(a["layers.0.wq"].std()) - 0.02) < 1e-3
    assert abs(float(a["final_norm"].mean()) - 1.0) < 5e-3
    assert not np.array_equal(a["layers.0.wq"], a["layers.0.wk"])
    assert set(a) == set(W.weight_names(wl.shape))


def test_observations_shapes_and_ranges():
    for name in ("C1", "C2"):
        wl = W.get_workload(name)
        o = W.make_observations(wl)
        assert o["patch_emb"].shape == (wl.batch * wl.n_patches, wl.shape.d_model)
        assert o["cu_patch"][-1] == wl.batch * wl.n_patches
        assert o["instr_ids"].min() >= 0 and o["instr_ids"].max() < wl.shape.action_id0
        assert o["cu_instr"][-1] == len(o["instr_ids"])
    wl = W.get_workload("C4").scaled(batch=16)
    wl = wl.scaled(shape=W.get_workload("C1").shape)
    o = W.make_observations(wl)
    lens = np.diff(o["cu_instr"])
    assert lens.min() >= 20 and lens.max() <= 60 and len(set(lens.tolist())) > 1


def test_gumbel_noise_is_finite_and_standard():
    wl = W.get_workload("C4").scaled(batch=64)
    g = W.make_gumbel(wl)
    assert g.shape == (64, 7, 256) and g.dtype == np.float32 and np.isfinite(g).all()
    assert abs(float(g.mean()) - 0.5772) < 0.02       # Euler-Mascheroni
    assert abs(float(g.var()) - np.pi ** 2 / 6) < 0.05
