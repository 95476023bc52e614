"""Host-side checks of the seeded generator and of the tie-band validator."""
import numpy as np

from inputs import CONFIGS, make_unit, round_to_bf16, unit_ids
from oracle import tie_band


def test_generator_is_deterministic_and_per_unit_independent():
    cfg = CONFIGS[0]
    a = make_unit(cfg, 0, 0, 2)
    b = make_unit(cfg, 0, 0, 2)
    c = make_unit(cfg, 0, 0, 3)
    assert np.array_equal(a.Q, b.Q) and np.array_equal(a.K, b.K) and np.array_equal(a.V, b.V)
    assert not np.array_equal(a.Q, c.Q)
    assert a.Q.shape == (cfg.prompt_len + cfg.steps, cfg.head_dim)
    assert len(a.heavy_positions) == round(0.02 * cfg.total_len)
    assert len(set(a.heavy_positions.tolist())) == len(a.heavy_positions)


def test_config_table_matches_the_benchmark_shapes():
    units = [c.units for c in CONFIGS]
    assert units == [4, 32, 512, 8192, 40]
    assert [(c.prompt_len, c.budget, c.steps) for c in CONFIGS] == [
        (256, 128, 64), (4096, 2048, 0), (3072, 2048, 512), (8192, 1024, 256), (32768, 4096, 1024)]
    assert len(unit_ids(CONFIGS[2])) == 512
    c4 = CONFIGS[3]
    assert abs(c4.heavy_fraction(0) - 0.005) < 1e-12 and abs(c4.heavy_fraction(31) - 0.05) < 1e-12


def test_bf16_rounding_is_nearest_even_and_idempotent():
    x = np.array([1.0, 1.00390625, 1.01171875, -3.14159, 1e-20, 65504.0], dtype=np.float32)
    r = round_to_bf16(x)
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    assert np.array_equal(round_to_bf16(r), r)
    assert r[0] == 1.0
    assert r[1] == 1.0  # 1 + 2^-8 is a tie between 1.0 and 1.0078125 -> even mantissa
    assert r[2] == np.float32(1.015625)  # 1 + 3*2^-8 is a tie -> rounds up to even
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)
    cfg = CONFIGS[1]
    u = make_unit(cfg, 0, 0, 0, total_len=64)
    assert np.all((u.K.view(np.uint32) & 0xFFFF) == 0)


def _case():
    mas = np.array([0.30, 0.10, 0.20, 0.05, 0.40])
    var = np.array([0.010, 0.020, 0.030, 0.040, 0.050])
    eps_m = 1e-3 * mas
    eps_v = np.full(5, 1e-5)
    return mas, var, eps_m, eps_v


def test_tie_band_accepts_the_exact_answer_and_rejects_wrong_ones():
    mas, var, eps_m, eps_v = _case()
    # scope 3 -> {0,1,2}; victim = 1
    assert tie_band.admissible_eviction(mas, var, eps_m, eps_v, 3, 1, [1])[0]
    assert not tie_band.admissible_eviction(mas, var, eps_m, eps_v, 3, 1, [3])[0]  # outside the scope
    assert not tie_band.admissible_eviction(mas, var, eps_m, eps_v, 3, 1, [2])[0]  # not the lowest MAS
    assert not tie_band.admissible_eviction(mas, var, eps_m, eps_v, 3, 1, [1, 2])[0]  # wrong count
    # E = 2 -> eligible 4 lowest var {0,1,2,3}; two lowest MAS {3,1}
    assert tie_band.admissible_eviction(mas, var, eps_m, eps_v, 3, 2, [1, 3])[0]
    assert not tie_band.admissible_eviction(mas, var, eps_m, eps_v, 3, 2, [1, 2])[0]


def test_tie_band_accepts_a_swap_at_the_variance_threshold_only_inside_the_band():
    mas, var, eps_m, eps_v = _case()
    var = var.copy()
    var[3] = var[2] + 1e-6  # tokens 2 and 3 are indistinguishable at the scope boundary
    # scope 3: oracle scope {0,1,2} -> victim 1; but with 3 in place of 2 the victim is 3 (MAS .05)
    assert tie_band.admissible_eviction(mas, var, eps_m, eps_v, 3, 1, [1])[0]
    assert tie_band.admissible_eviction(mas, var, eps_m, eps_v, 3, 1, [3])[0]
    var[3] = var[2] + 1e-3  # clearly apart
    assert not tie_band.admissible_eviction(mas, var, eps_m, eps_v, 3, 1, [3])[0]


def test_tie_band_accepts_near_equal_mas_only_inside_the_band():
    mas, var, eps_m, eps_v = _case()
    mas = mas.copy()
    mas[2] = mas[1] * (1 + 5e-4)
    eps_m = 1e-3 * mas
    assert tie_band.admissible_eviction(mas, var, eps_m, eps_v, 3, 1, [2])[0]
    mas[2] = mas[1] * 1.01
    eps_m = 1e-3 * mas
    assert not tie_band.admissible_eviction(mas, var, eps_m, eps_v, 3, 1, [2])[0]


def test_bands_follow_the_cancelling_terms():
    eps_m, eps_v = tie_band.bands([2.0], [1.5], [4.0], rel=1e-3)
    assert np.isclose(eps_m[0], 1e-3 * 0.5)
    assert np.isclose(eps_v[0], 1e-3 * (1.5 / 4 + 0.25))
