"""Pins for cluster scores (Eq. 1, Eq. 2 / Alg. 2), arg-top-k (Alg. 3 l.8) and the top-p budget."""
import math

import numpy as np
import pytest

from oracle import adacluster_oracle as orc


def test_box_score_equals_eq1_loops_and_bounds_every_member():
    rng = np.random.default_rng(0)
    Qc = orc.normalize_rows(rng.standard_normal((5, 7)))
    pages = [rng.standard_normal((n, 7)) for n in (1, 3, 9, 4)]
    bmin = np.stack([p.min(axis=0) for p in pages])
    bmax = np.stack([p.max(axis=0) for p in pages])
    S = orc.score_box(Qc, bmin, bmax)
    for i in range(5):
        for j, p in enumerate(pages):
            assert math.isclose(S[i, j], orc.quest_upper_bound_loops(Qc[i], p), rel_tol=1e-13, abs_tol=1e-14)
            assert S[i, j] >= (p @ Qc[i]).max() - 1e-13          # upper bound of every q.k in the page


def test_eq2_on_one_vector_is_quest_over_the_page_with_the_origin():
    """Reading of Eq. 2: with k+ = max(k,0), k- = min(k,0) of a single vector c it equals
    Eq. 1 on the two-point page {c, 0}, i.e. sum_d max(q_d c_d, 0)."""
    rng = np.random.default_rng(1)
    Qc = rng.standard_normal((4, 9))
    Kc = rng.standard_normal((6, 9))
    S = orc.score_tensorquest(Qc, Kc)
    for i in range(4):
        for j in range(6):
            page = np.stack([Kc[j], np.zeros(9)])
            assert math.isclose(S[i, j], orc.quest_upper_bound_loops(Qc[i], page), rel_tol=1e-13, abs_tol=1e-14)
            assert math.isclose(S[i, j], sum(max(float(a) * float(b), 0.0) for a, b in zip(Qc[i], Kc[j])),
                                rel_tol=1e-13, abs_tol=1e-14)
    assert np.all(S >= orc.score_dot(Qc, Kc) - 1e-13)


def test_all_modes_agree_for_nonnegative_singletons():
    rng = np.random.default_rng(2)
    Qc = np.abs(rng.standard_normal((3, 5)))
    Kc = np.abs(rng.standard_normal((4, 5)))
    a = orc.score_tensorquest(Qc, Kc)
    b = orc.score_box(Qc, Kc, Kc)
    c = orc.score_dot(Qc, Kc)
    assert np.allclose(a, c, atol=1e-14) and np.allclose(b, c, atol=1e-14)
    assert np.allclose(c, Qc @ Kc.T, atol=1e-13)


def test_empty_clusters_score_minus_infinity():
    rng = np.random.default_rng(3)
    Qc, Kc = rng.standard_normal((3, 4)), rng.standard_normal((5, 4))
    S = orc.cluster_scores(orc.SCORE_TQ, Qc, Kc, None, None, np.array([3, 0, 2, 0, 1]))
    assert np.all(np.isneginf(S[:, [1, 3]])) and np.all(np.isfinite(S[:, [0, 2, 4]]))


def test_topk_against_full_sort_and_ties():
    rng = np.random.default_rng(4)
    S = rng.standard_normal((6, 20))
    S[:, 3] = -np.inf
    sel = orc.select_topk(S, 5)
    for i in range(6):
        ref = np.sort(np.argsort(-S[i], kind="stable")[:5])
        assert np.array_equal(sel[i], ref)
        assert 3 not in sel[i]
    # ties: equal scores -> lowest indices win
    T = np.zeros((1, 8))
    assert orc.select_topk(T, 3)[0].tolist() == [0, 1, 2]
    T[0, 6] = 1.0
    assert orc.select_topk(T, 3)[0].tolist() == [0, 1, 6]
    # budget larger than the number of non-empty clusters -> all of them
    T[0, 2] = -np.inf
    assert orc.select_topk(T, 100)[0].tolist() == [0, 1, 3, 4, 5, 6, 7]


def test_topk_sets_invariant_under_query_scaling():
    """App. A.2: scaling a query row by a positive factor keeps the score order."""
    rng = np.random.default_rng(5)
    Qc, Kc = rng.standard_normal((5, 16)), rng.standard_normal((30, 16))
    f = 2.0 ** rng.integers(-3, 4, size=(5, 1))         # exact scalings
    a = orc.select_topk(orc.score_tensorquest(Qc, Kc), 7)
    b = orc.select_topk(orc.score_tensorquest(Qc * f, Kc), 7)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_exp_det_matches_libm():
    x = -np.concatenate([np.linspace(0, 50, 2001), np.array([0.0, 1e-300, 699.9, 700.5, 1e4])])
    got = orc.exp_det(x)
    ref = np.array([math.exp(v) if v >= -700 else 0.0 for v in x])
    ok = ref > 0
    assert np.max(np.abs(got[ok] / ref[ok] - 1)) < 4e-16
    assert np.all(got[~ok] == 0)
    assert orc.exp_det(np.array([0.0]))[0] == 1.0


def test_topp_mass_property_and_minimality():
    rng = np.random.default_rng(6)
    S = 3 * rng.standard_normal((8, 25))
    sizes = rng.integers(0, 40, 25)
    sizes[4] = 0
    S[:, sizes == 0] = -np.inf
    alpha = rng.uniform(0.2, 2.0, 8)
    for p in (0.3, 0.9, 0.999):
        sel = orc.select_topp(S, sizes, alpha, p)
        for i in range(8):
            w = np.where(sizes > 0, sizes * np.exp(alpha[i] * (np.where(sizes > 0, S[i], 0) - S[i][sizes > 0].max())), 0.0)
            tot = w.sum()
            chosen = sel[i]
            assert len(chosen) >= 1 and np.all(sizes[chosen] > 0)
            assert w[chosen].sum() >= p * tot * (1 - 1e-12)
            # chosen = the heaviest clusters; dropping the lightest chosen one falls below p
            rest = np.setdiff1d(np.flatnonzero(sizes > 0), chosen)
            if rest.size:
                assert w[chosen].min() >= w[rest].max() - 1e-15
            assert w[chosen].sum() - w[chosen].min() < p * tot * (1 + 1e-12)


def test_topp_one_selects_every_nonempty_cluster_and_zero_selects_one():
    rng = np.random.default_rng(7)
    S = rng.standard_normal((3, 10))
    sizes = np.array([1, 0, 3, 4, 0, 2, 2, 9, 1, 1])
    S[:, sizes == 0] = -np.inf
    alpha = np.ones(3)
    for row in orc.select_topp(S, sizes, alpha, 1.0):
        assert row.tolist() == [0, 2, 3, 5, 6, 7, 8, 9]
    for i, row in enumerate(orc.select_topp(S, sizes, alpha, 1e-9)):
        w = np.where(sizes > 0, sizes * np.exp(np.where(sizes > 0, S[i], -1e9)), 0)
        assert row.tolist() == [int(np.argmax(w))]


def test_end_to_end_select_all_equals_dense_and_flag_equals_dense():
    """Alg. 3: topk >= #clusters, top_p = 1 and F = True all reduce to dense attention."""
    rng = np.random.default_rng(8)
    mu_q, mu_k = rng.standard_normal((6, 8)), rng.standard_normal((6, 8))
    comp = rng.integers(0, 6, 160)
    Q = (mu_q[comp] + 0.3 * rng.standard_normal((160, 8)))[None]
    K = (mu_k[comp] + 0.3 * rng.standard_normal((160, 8)))[None]
    V = rng.standard_normal((1, 160, 8))
    dense = orc.dense_attention(Q[0], K[0], V[0])
    base = dict(q_clusters=5, q_iters=3, k_iters=3, k_m0=6, k_m_min=2, k_max_clusters=40, tau_factor=1.5)
    for use_gather in (False, True):
        O, info, tau = orc.adacluster_attention(Q, K, V, topk=10 ** 6, use_gather=use_gather, **base)
        assert not info[0]["k"]["full_flag"]
        assert np.max(np.abs(O[0] - dense)) < 1e-12
    O, info, _ = orc.adacluster_attention(Q, K, V, select_mode=1, top_p=1.0, **base)
    assert np.max(np.abs(O[0] - dense)) < 1e-12
    O, info, _ = orc.adacluster_attention(Q, K, V, topk=1, **{**base, "k_max_clusters": 6})
    assert info[0]["k"]["full_flag"] and np.max(np.abs(O[0] - dense)) < 1e-12
    # and a real sparse call differs from dense but is a convex combination of V rows
    O, info, _ = orc.adacluster_attention(Q, K, V, topk=2, **base)
    assert np.max(np.abs(O[0] - dense)) > 1e-6
    assert O.min() >= V.min() - 1e-12 and O.max() <= V.max() + 1e-12
    O2, _, _ = orc.adacluster_attention(Q, K, V, topk=2, use_gather=True, **base)
    assert np.max(np.abs(O - O2)) < 1e-12


def test_concentrated_attention_is_kept_by_a_small_selection():
    """The purpose of the method, on the oracle: queries whose soft-max mass sits on the keys of their own
    component (query means = scaled key means) are served by 4 selected clusters of 16 to within 1e-3 of
    dense attention, at under a third of the work."""
    rng = np.random.default_rng(5)
    N, d, M, Cq = 600, 32, 12, 16
    comp = rng.integers(0, M, N)
    mu = rng.standard_normal((M, d))
    K = mu[comp] + 0.15 * rng.standard_normal((N, d))
    Q = 3.0 * mu[comp] + 0.15 * rng.standard_normal((N, d))
    V = rng.standard_normal((N, d))
    O, info, _ = orc.adacluster_attention(Q[None], K[None], V[None], q_clusters=Cq, q_iters=3, k_iters=3, k_m0=12,
                                          k_m_min=3, k_max_clusters=60, tau_factor=1.5, topk=4, use_gather=True)
    k, q, sel = info[0]["k"], info[0]["q"], info[0]["sel"]
    assert not k["full_flag"]
    pairs = sum(int(q["sizes"][i]) * int(k["sizes"][sel[i]].sum()) for i in range(Cq))
    dense = orc.dense_attention(Q, K, V)
    rel = np.linalg.norm(O[0] - dense) / np.linalg.norm(dense)
    print("density", pairs / N ** 2, "rel-L2", rel, "clusters", k["sizes"].shape[0])
    assert pairs / N ** 2 < 0.33 and rel < 1e-3
