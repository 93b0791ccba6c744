"""The synthetic input recipe: shapes, determinism, dtype rounding, structure."""
import numpy as np

from paper_2604_18348_amd import workloads as wl


def test_token_counts_match_the_configurations():
    want = {"c1": 4096, "c2": 17776, "c3": 32760, "c4": 75600, "c5": 180000}
    for k, n in want.items():
        assert wl.n_tokens(wl.CONFIGS[k]) == n


def test_c1_is_deterministic_fp32_mixture():
    Q, K, V = wl.make_qkv("c1")
    Q2, K2, V2 = wl.make_qkv("c1")
    assert Q.shape == (1, 4096, 64) and Q.dtype == np.float32
    assert np.array_equal(Q, Q2) and np.array_equal(K, K2) and np.array_equal(V, V2)
    assert abs(float(V.std()) - 1.0) < 0.02
    # within-component spread 0.3 around N(0,1) means: total variance ~ 1 + 0.09
    assert 0.8 < float(K.var()) < 1.4


def test_bf16_configs_are_bf16_representable_and_heads_independent():
    cfg = wl.CONFIGS["c2"]
    Q, K, V = wl.make_head(cfg, 3)
    for a in (Q, K, V):
        assert np.all((a.view(np.uint32) & 0xFFFF) == 0)
    Qb, _, _ = wl.make_head(cfg, 4)
    assert not np.array_equal(Q, Qb)
    Qd, Kd, _ = wl.make_head(cfg, 25)                  # diffuse head: isotropic
    assert abs(float(Kd.var()) - 1.0) < 0.02


def test_round_bf16_ties_to_even():
    a = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -1.0 - 2.0 ** -8], dtype=np.float32)
    assert wl.round_bf16_f32(a).tolist() == [1.0, 1.0 + 2.0 ** -6, -1.0]


def test_make_small_shapes():
    Q, K, V = wl.make_small(5, 1000, 64, 12, H=2, dtype="bf16")
    assert Q.shape == (2, 1000, 64)
    assert np.all((K.view(np.uint32) & 0xFFFF) == 0)
