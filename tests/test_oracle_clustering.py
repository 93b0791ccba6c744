"""Pins for the oracle's clustering: query k-means on the sphere (Sec. 3.1, Alg. 3 l.1)
and multi-stage key k-means (Alg. 1).  Evidence: explicit-loop recomputation of
arg-min / member means, textbook behaviour on well-separated mixtures, and the
structural invariants the algorithm's text fixes."""
import math

import numpy as np
import pytest

from oracle import adacluster_oracle as orc


def separated_mixture(seed, n_per=30, m=6, d=8, spread=0.05, scale=6.0):
    rng = np.random.default_rng(seed)
    mu = scale * rng.standard_normal((m, d))
    comp = np.repeat(np.arange(m), n_per)
    X = mu[comp] + spread * rng.standard_normal((m * n_per, d))
    return X, comp, mu


def loops_argmin(X, C):
    lab = []
    for x in X:
        best, bj = None, -1
        for j, c in enumerate(C):
            dist = sum((float(a) - float(b)) ** 2 for a, b in zip(x, c))
            if best is None or dist < best:
                best, bj = dist, j
        lab.append(bj)
    return np.asarray(lab)


def test_strided_indices_are_midpoints():
    assert orc.strided_indices(10, 5).tolist() == [1, 3, 5, 7, 9]
    assert orc.strided_indices(7, 3).tolist() == [1, 3, 5]
    idx = orc.strided_indices(4096, 32)
    assert idx[0] == 64 and idx[-1] == 4096 - 64 and np.all(np.diff(idx) == 128)
    assert orc.strided_indices(5, 5).tolist() == [0, 1, 2, 3, 4]


def test_round_to_bf16_known_values():
    # 1 + 2^-8 is a tie between 1 and 1+2^-7 -> even (1.0); 1 + 3*2^-8 ties up to 1+2^-6
    assert orc.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert orc.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert orc.round_to_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20]))[0] == 1.0 + 2.0 ** -7
    assert orc.round_to_bf16(np.array([-3.140625]))[0] == -3.140625
    x = np.random.default_rng(0).standard_normal(1000)
    r = orc.round_to_bf16(x)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)


def test_euclid_kmeans_recovers_separated_components():
    X, comp, mu = separated_mixture(0)
    # one seed per component: the first member of each
    init = X[[np.flatnonzero(comp == j)[0] for j in range(6)]]
    labels, C, d2 = orc.euclid_kmeans(X, 6, 3, init_centroids=init)
    assert np.array_equal(labels, comp)
    for j in range(6):
        assert np.allclose(C[j], X[comp == j].mean(axis=0), atol=1e-12)
    assert np.allclose(d2, np.sum((X - C[labels]) ** 2, axis=1))


def test_euclid_assign_is_bruteforce_argmin_and_ties_go_low():
    rng = np.random.default_rng(1)
    X, C = rng.standard_normal((40, 5)), rng.standard_normal((7, 5))
    assert np.array_equal(orc.euclid_assign(X, C), loops_argmin(X, C))
    C2 = np.concatenate([C, C[2:3]], axis=0)            # duplicate centre 2 as centre 7
    lab = orc.euclid_assign(X, C2)
    assert not np.any(lab == 7)


def test_euclid_kmeans_labels_are_argmin_to_returned_centres():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((200, 6))
    for iters in (1, 2, 4):
        labels, C, d2 = orc.euclid_kmeans(X, 9, iters)
        assert np.array_equal(labels, loops_argmin(X, C))
    # one pass = assignment to the strided sample itself
    labels, C, _ = orc.euclid_kmeans(X, 9, 1)
    assert np.array_equal(C, X[orc.strided_indices(200, 9)])


def test_euclid_kmeans_second_pass_uses_member_means():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((120, 4))
    l1, C1, _ = orc.euclid_kmeans(X, 5, 1)
    _, C2, _ = orc.euclid_kmeans(X, 5, 2)
    for j in range(5):
        mem = [X[i] for i in range(120) if l1[i] == j]
        if mem:
            mean = [sum(float(v[k]) for v in mem) / len(mem) for k in range(4)]
            assert np.allclose(C2[j], mean, atol=1e-13)
        else:
            assert np.array_equal(C2[j], C1[j])


def test_empty_cluster_keeps_its_centre():
    X = np.array([[0.0, 0.0], [0.1, 0.0], [0.0, 0.1], [5.0, 5.0]])
    init = np.array([[0.0, 0.0], [5.0, 5.0], [100.0, 100.0]])
    labels, C, _ = orc.euclid_kmeans(X, 3, 3, init_centroids=init)
    assert np.array_equal(C[2], [100.0, 100.0])
    assert labels.tolist() == [0, 0, 0, 1]


def test_query_kmeans_angle_clusters_ignore_norms():
    rng = np.random.default_rng(4)
    dirs = np.linalg.qr(rng.standard_normal((8, 8)))[0][:4]        # 4 orthonormal directions
    comp = np.repeat(np.arange(4), 25)
    Q = dirs[comp] + 0.02 * rng.standard_normal((100, 8))
    Q = Q * rng.uniform(0.1, 20.0, size=(100, 1))                  # wild norms
    init = orc.normalize_rows(Q)[[0, 25, 50, 75]]
    out = orc.query_kmeans(Q, 4, 3, init_centroids=init)
    assert np.array_equal(out["labels"], comp)
    assert np.allclose(np.linalg.norm(out["centroids"], axis=1), 1.0, atol=1e-14)
    for j in range(4):
        s = orc.normalize_rows(Q)[comp == j].sum(axis=0)
        assert np.allclose(out["centroids"][j], s / np.linalg.norm(s), atol=1e-13)
        assert math.isclose(out["mean_norm"][j], np.linalg.norm(Q[comp == j], axis=1).mean(), rel_tol=1e-13)
    # labels are the arg-max cosine to the returned assignment centres
    cos = orc.normalize_rows(Q) @ out["assign_centroids"].T
    assert np.array_equal(out["labels"], np.argmax(cos, axis=1))


def test_query_labels_invariant_under_positive_row_scaling():
    """App. A.2: normalisation removes the query length, so rescaling rows changes nothing."""
    rng = np.random.default_rng(5)
    Q = rng.standard_normal((300, 16))
    a = orc.query_kmeans(Q, 7, 3)
    b = orc.query_kmeans(Q * rng.uniform(0.5, 4.0, (300, 1)), 7, 3)
    assert np.array_equal(a["labels"], b["labels"])
    assert np.allclose(a["centroids"], b["centroids"], atol=1e-12)


def test_query_kmeans_without_normalisation_is_plain_kmeans_and_feels_the_norms():
    """Component ablation "w/o Norm": on well-separated blobs with one seed per blob it returns the blob
    ids and the sample means (textbook k-means); on the wild-norm data above it no longer finds the four
    directions, which is what normalisation is for."""
    rng = np.random.default_rng(14)
    means = 10.0 * rng.standard_normal((5, 6))
    comp = np.repeat(np.arange(5), 40)
    Q = means[comp] + 0.1 * rng.standard_normal((200, 6))
    out = orc.query_kmeans(Q, 5, 3, init_centroids=Q[[0, 40, 80, 120, 160]], normalize=False)
    assert np.array_equal(out["labels"], comp)
    for j in range(5):
        assert np.allclose(out["centroids"][j], Q[comp == j].mean(axis=0), atol=1e-13)
    assert np.array_equal(out["mean_norm"], np.ones(5))
    d2 = ((Q[:, None, :] - out["assign_centroids"][None]) ** 2).sum(-1)
    assert np.array_equal(out["labels"], np.argmin(d2, axis=1))
    # the same routine as the stage k-means of Algorithm 1
    lab2, ca2, _ = orc.euclid_kmeans(Q, 5, 3, init_centroids=Q[[0, 40, 80, 120, 160]])
    assert np.array_equal(out["labels"], lab2) and np.array_equal(out["assign_centroids"], ca2)
    # wild norms: directions are lost without normalisation
    rng = np.random.default_rng(4)
    dirs = np.linalg.qr(rng.standard_normal((8, 8)))[0][:4]
    comp = np.repeat(np.arange(4), 25)
    Qw = (dirs[comp] + 0.02 * rng.standard_normal((100, 8))) * rng.uniform(0.1, 20.0, size=(100, 1))
    raw = orc.query_kmeans(Qw, 4, 3, init_centroids=Qw[[0, 25, 50, 75]], normalize=False)
    assert not np.array_equal(raw["labels"], comp)


def test_zero_query_goes_to_cluster_zero():
    rng = np.random.default_rng(6)
    Q = rng.standard_normal((50, 4))
    Q[10] = 0.0
    out = orc.query_kmeans(Q, 5, 2)
    assert out["labels"][10] == 0


def test_stage_cluster_count_rule():
    assert orc.stage_cluster_count(1000, 1000, 100, 8) == 100
    assert orc.stage_cluster_count(250, 1000, 100, 8) == 25
    assert orc.stage_cluster_count(251, 1000, 100, 8) == 26        # ceil
    assert orc.stage_cluster_count(10, 1000, 100, 8) == 8          # floor m_min
    assert orc.stage_cluster_count(5, 1000, 100, 8) == 5           # never more centres than points
    # The fraction is a float32 parameter of the call: float32(0.03) = 0.0299999993..., so 3 % of 1000
    # tokens is floor(29.9999993) = 29, not 30; float32(0.1) = 0.100000001... gives 100; 0.25 is exact.
    assert orc.min_unassigned_count(0.03, 1000) == 29
    assert orc.min_unassigned_count(0.1, 1000) == 100
    assert orc.min_unassigned_count(0.25, 1000) == 250
    assert orc.min_unassigned_count(0.0, 1000) == 0


def _check_alg1_invariants(K, out, tau, n_max, m0, m_min, iters, max_stages, frac):
    N = K.shape[0]
    offs = out["stage_offs"]
    C = out["assign_centroids"]
    n_stage = len(offs) - 1
    assert C.shape[0] == offs[-1]
    # |C| = sum of the stage counts, each following the rule on the |U| entering the stage
    in_U = np.ones(N, dtype=bool)
    for t in range(n_stage):
        m_t = offs[t + 1] - offs[t]
        assert m_t == orc.stage_cluster_count(in_U.sum(), N, m0, m_min)
        assert out["n_unassigned"][t] == in_U.sum()
        Ct = C[offs[t]:offs[t + 1]]
        idx = np.flatnonzero(in_U)
        d = np.sqrt(((K[idx][:, None, :] - Ct[None]) ** 2).sum(-1)).min(axis=1)
        removed = d < tau
        # every token removed at stage t was within tau of a stage-t centre; the rest were not
        assert np.array_equal(out["stage_of"][idx] == t, removed)
        in_U[idx[removed]] = False
    assert out["n_unassigned"][n_stage] == in_U.sum()
    assert np.all(out["stage_of"][in_U] == -1)
    # final labels: nearest centre among all of C
    assert np.array_equal(out["labels"], loops_argmin(K, C))
    # final centroids: member means; sizes; boxes
    for j in range(C.shape[0]):
        mem = K[out["labels"] == j]
        assert out["sizes"][j] == mem.shape[0]
        if mem.shape[0]:
            assert np.allclose(out["centroids"][j], mem.mean(axis=0), atol=1e-12)
            assert np.array_equal(out["box_min"][j], mem.min(axis=0))
            assert np.array_equal(out["box_max"][j], mem.max(axis=0))
    # why did it stop?
    u_left = int(in_U.sum())
    if out["full_flag"]:
        assert u_left > 0 and offs[-1] >= n_max
    else:
        assert (u_left == 0 or n_stage >= max_stages
                or u_left <= orc.min_unassigned_count(frac, N))
        if u_left > 0:
            assert offs[-1] < n_max
    # the cap test comes before a stage is added: |C| may pass n_max by less than one stage
    if n_stage > 1:
        assert offs[-2] < n_max


@pytest.mark.parametrize("seed,tau,n_max", [(0, 1.2, 64), (1, 0.9, 40), (2, 2.5, 64), (3, 0.7, 24)])
def test_multistage_invariants(seed, tau, n_max):
    rng = np.random.default_rng(seed)
    mu = 3.0 * rng.standard_normal((10, 6))
    comp = rng.integers(0, 10, 400)
    K = mu[comp] + 0.25 * rng.standard_normal((400, 6))
    out_mask = rng.random(400) < 0.05
    K[out_mask] = 3.0 * rng.standard_normal((int(out_mask.sum()), 6))
    out = orc.multistage_kmeans(K, tau, n_max, m0=12, m_min=3, n_iters=3, max_stages=10)
    _check_alg1_invariants(K, out, tau, n_max, 12, 3, 3, 10, 0.0)


def test_multistage_infinite_tau_is_plain_kmeans():
    rng = np.random.default_rng(7)
    K = rng.standard_normal((150, 5))
    out = orc.multistage_kmeans(K, float("inf"), 100, m0=10, m_min=2, n_iters=3)
    labels, C, _ = orc.euclid_kmeans(K, 10, 3)
    assert len(out["stage_offs"]) == 2 and out["stage_offs"][-1] == 10
    assert np.array_equal(out["assign_centroids"], C)
    assert np.array_equal(out["labels"], labels)
    assert not out["full_flag"]
    assert np.all(out["stage_of"] == 0)


def test_multistage_small_cap_sets_flag_after_first_stage():
    rng = np.random.default_rng(8)
    K = rng.standard_normal((150, 5))
    out = orc.multistage_kmeans(K, 0.5, 10, m0=10, m_min=2, n_iters=2)       # n_max <= m0
    assert out["full_flag"] and len(out["stage_offs"]) == 2


def test_multistage_zero_tau_never_removes_and_ends_full():
    rng = np.random.default_rng(9)
    K = rng.standard_normal((120, 4))
    out = orc.multistage_kmeans(K, 0.0, 35, m0=10, m_min=2, n_iters=2, max_stages=50)
    assert out["full_flag"]
    assert np.all(out["stage_of"] == -1)
    assert out["stage_offs"].tolist() == [0, 10, 20, 30, 40]               # overshoot < one stage
    assert np.array_equal(out["labels"], loops_argmin(K, out["assign_centroids"]))


def test_multistage_stage_limit_and_fraction_stop_do_not_set_flag():
    rng = np.random.default_rng(10)
    K = rng.standard_normal((300, 6))
    out = orc.multistage_kmeans(K, 0.0, 10 ** 6, m0=10, m_min=2, n_iters=1, max_stages=3)
    assert not out["full_flag"] and len(out["stage_offs"]) == 4
    mu = 4.0 * rng.standard_normal((5, 6))
    K2 = mu[rng.integers(0, 5, 300)] + 0.05 * rng.standard_normal((300, 6))
    K2[:6] = 10 + rng.standard_normal((6, 6))                                # 2 % stragglers
    out2 = orc.multistage_kmeans(K2, 0.6, 10 ** 6, m0=8, m_min=2, n_iters=3, min_unassigned_frac=0.03)
    assert not out2["full_flag"]
    assert 0 < out2["n_unassigned"][-1] <= 9
    _check_alg1_invariants(K2, out2, 0.6, 10 ** 6, 8, 2, 3, 10, 0.03)


def test_diffuse_keys_need_more_clusters_than_compact_keys():
    """Sec. 3.2.1-3.2.2: scattered keys get larger cluster counts under one threshold."""
    rng = np.random.default_rng(11)
    mu = 4.0 * rng.standard_normal((8, 8))
    compact = mu[rng.integers(0, 8, 600)] + 0.1 * rng.standard_normal((600, 8))
    diffuse = 2.0 * rng.standard_normal((600, 8))
    a = orc.multistage_kmeans(compact, 1.0, 10 ** 6, m0=16, m_min=4, n_iters=3)
    b = orc.multistage_kmeans(diffuse, 1.0, 10 ** 6, m0=16, m_min=4, n_iters=3)
    assert b["stage_offs"][-1] > a["stage_offs"][-1]


def test_tau_from_factor_is_scaled_mean_distance():
    rng = np.random.default_rng(12)
    Ks = [rng.standard_normal((90, 4)), 2 * rng.standard_normal((90, 4))]
    tau = orc.tau_from_factor(Ks, 1.5, 6, 2)
    ds = []
    for K in Ks:
        labels, C, _ = orc.euclid_kmeans(K, 6, 2)
        ds += [math.sqrt(sum((float(a) - float(b)) ** 2 for a, b in zip(K[i], C[labels[i]]))) for i in range(90)]
    assert math.isclose(tau, 1.5 * sum(ds) / len(ds), rel_tol=1e-12)


def test_cauchy_schwarz_bound_of_key_clustering():
    """Sec. 3.2.1: q.c(k) - q.k <= ||q|| ||k - c(k)|| for every pair."""
    rng = np.random.default_rng(13)
    K = rng.standard_normal((80, 6))
    Q = rng.standard_normal((20, 6))
    labels, C, d2 = orc.euclid_kmeans(K, 7, 3)
    lhs = Q @ C[labels].T - Q @ K.T
    rhs = np.linalg.norm(Q, axis=1)[:, None] * np.sqrt(d2)[None, :]
    assert np.all(lhs <= rhs + 1e-12)


def test_round_fn_is_applied_to_assignment_centres():
    rng = np.random.default_rng(14)
    X = rng.standard_normal((100, 8))
    labels, C, _ = orc.euclid_kmeans(X, 5, 3, round_fn=orc.round_to_bf16)
    assert np.array_equal(C, orc.round_to_bf16(C))
    assert np.array_equal(labels, loops_argmin(X, C))


def test_warm_start_keeps_count_and_follows_lloyd_from_given_centres():
    """Sec. 3.2.2 "Efficient initialization": fixed cluster count, previous centres as the start."""
    X, comp, mu = separated_mixture(20, n_per=25, m=5, d=6)
    true_means = np.stack([X[comp == j].mean(axis=0) for j in range(5)])
    out = orc.warm_key_clustering(X, true_means + 0.01, 2)
    assert np.array_equal(out["labels"], comp)                       # a fixed point of Lloyd
    assert np.allclose(out["centroids"], true_means, atol=1e-12)
    assert out["assign_centroids"].shape == (5, 6)
    # one pass = plain nearest-centre assignment to the centres given
    rng = np.random.default_rng(21)
    prev = rng.standard_normal((7, 6))
    out1 = orc.warm_key_clustering(X, prev, 1)
    assert np.array_equal(out1["assign_centroids"], prev)
    assert np.array_equal(out1["labels"], loops_argmin(X, prev))
    # an empty cluster keeps the centre it was given
    far = np.concatenate([true_means, np.full((1, 6), 100.0)])
    out2 = orc.warm_key_clustering(X, far, 3)
    assert out2["sizes"][5] == 0 and np.array_equal(out2["assign_centroids"][5], far[5])


def test_compactness_mse_pins():
    """Sec. 3.2.1 MSE: explicit loops; zero when every token is its own centre; for member means the
    textbook identity sum ||k - c||^2 = sum ||k||^2 - sum_j n_j ||c_j||^2; a shifted centre adds
    exactly n_j ||shift||^2 (parallel-axis)."""
    rng = np.random.default_rng(17)
    N, d, m = 57, 6, 5
    K = rng.standard_normal((N, d))
    lab = rng.integers(0, m, N)
    lab[:m] = np.arange(m)
    C = rng.standard_normal((m, d))
    tot = 0.0
    for n in range(N):
        for j in range(d):
            tot += (K[n, j] - C[lab[n], j]) ** 2
    assert math.isclose(orc.compactness_mse(K, lab, C), tot / N, rel_tol=1e-12)
    assert orc.compactness_mse(K, np.arange(N), K) == 0.0
    means = np.stack([K[lab == j].mean(0) for j in range(m)])
    sizes = np.bincount(lab, minlength=m)
    ident = (np.sum(K * K) - np.sum(sizes * np.sum(means * means, axis=1))) / N
    assert math.isclose(orc.compactness_mse(K, lab, means), ident, rel_tol=1e-10)
    shift = rng.standard_normal(d)
    moved = means.copy(); moved[2] += shift
    extra = sizes[2] * float(shift @ shift) / N
    assert math.isclose(orc.compactness_mse(K, lab, moved), orc.compactness_mse(K, lab, means) + extra, rel_tol=1e-10)
    assert math.isclose(orc.compactness_score([0.5, 1.5]), 1.0)
