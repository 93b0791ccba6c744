"""Pins for the oracle's attention functions (Alg. 3 lines 9-10 and the dense branch).

Independent evidence: explicit Python loops with math.exp, closed forms, and the
textbook special cases the clustered call must reduce to.
"""
import math

import numpy as np
import pytest

from oracle import adacluster_oracle as orc


def brute_force_attention(Q, K, V, scale, allow=None):
    Nq, d = Q.shape
    out = np.zeros((Nq, V.shape[1]))
    for n in range(Nq):
        logits = []
        for m in range(K.shape[0]):
            if allow is not None and not allow(n, m):
                logits.append(None)
                continue
            s = 0.0
            for j in range(d):
                s += float(Q[n, j]) * float(K[m, j])
            logits.append(s * scale)
        mx = max(x for x in logits if x is not None)
        den = 0.0
        acc = [0.0] * V.shape[1]
        for m, x in enumerate(logits):
            if x is None:
                continue
            p = math.exp(x - mx)
            den += p
            for j in range(V.shape[1]):
                acc[j] += p * float(V[m, j])
        out[n] = [a / den for a in acc]
    return out


def test_dense_matches_brute_force_loops():
    rng = np.random.default_rng(1)
    Q, K, V = rng.standard_normal((7, 5)), rng.standard_normal((11, 5)), rng.standard_normal((11, 3))
    got = orc.dense_attention(Q, K, V, 0.37)
    ref = brute_force_attention(Q, K, V, 0.37)
    assert np.max(np.abs(got - ref)) < 1e-13


def test_dense_default_scale_is_inverse_sqrt_d():
    rng = np.random.default_rng(2)
    Q, K, V = rng.standard_normal((4, 16)), rng.standard_normal((9, 16)), rng.standard_normal((9, 16))
    assert np.allclose(orc.dense_attention(Q, K, V), brute_force_attention(Q, K, V, 0.25), atol=1e-13)


def test_dense_closed_forms():
    rng = np.random.default_rng(3)
    Q = rng.standard_normal((6, 8))
    K = rng.standard_normal((10, 8))
    V = rng.standard_normal((10, 8))
    # constant V -> that constant
    assert np.allclose(orc.dense_attention(Q, K, np.ones_like(V)), 1.0, atol=1e-14)
    # identical keys -> uniform weights -> mean of V
    Ksame = np.tile(K[:1], (10, 1))
    assert np.allclose(orc.dense_attention(Q, Ksame, V), V.mean(axis=0)[None, :], atol=1e-13)
    # one key -> its value
    assert np.allclose(orc.dense_attention(Q, K[:1], V[:1]), np.tile(V[:1], (6, 1)), atol=1e-14)
    # two keys, zero query: weights 1/2, 1/2
    assert np.allclose(orc.dense_attention(np.zeros((1, 8)), K[:2], V[:2]), V[:2].mean(axis=0)[None], atol=1e-14)
    # two keys: logistic weight
    q = Q[:1]
    s0, s1 = float(q[0] @ K[0]) / math.sqrt(8), float(q[0] @ K[1]) / math.sqrt(8)
    w0 = 1.0 / (1.0 + math.exp(s1 - s0))
    assert np.allclose(orc.dense_attention(q, K[:2], V[:2]), w0 * V[0] + (1 - w0) * V[1], atol=1e-13)


def test_dense_is_shift_invariant_and_large_logits_are_safe():
    rng = np.random.default_rng(4)
    Q, K, V = 40 * rng.standard_normal((5, 8)), 40 * rng.standard_normal((9, 8)), rng.standard_normal((9, 8))
    out = orc.dense_attention(Q, K, V)
    assert np.all(np.isfinite(out))
    assert np.allclose(out, brute_force_attention(Q, K, V, 1 / math.sqrt(8)), atol=1e-12)


def _random_clustered_problem(seed, N=48, d=8, cq=4, ck=6):
    rng = np.random.default_rng(seed)
    Q, K, V = rng.standard_normal((N, d)), rng.standard_normal((N, d)), rng.standard_normal((N, d))
    ql = rng.integers(0, cq, N)
    kl = rng.integers(0, ck, N)
    sel = []
    for i in range(cq):
        k = rng.integers(1, ck + 1)
        sel.append(np.sort(rng.choice(ck, size=k, replace=False)))
    return Q, K, V, ql, kl, sel


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_sparse_mask_matches_brute_force_and_gather_form(seed):
    Q, K, V, ql, kl, sel = _random_clustered_problem(seed)
    # make sure no query row is left without keys
    for i, s in enumerate(sel):
        assert np.isin(kl, s).any()
    sets = [set(s.tolist()) for s in sel]
    ref = brute_force_attention(Q, K, V, 1 / math.sqrt(8), allow=lambda n, m: kl[m] in sets[ql[n]])
    a = orc.sparse_attention_mask(Q, K, V, ql, kl, sel)
    b = orc.sparse_attention_gather(Q, K, V, ql, kl, sel)
    assert np.max(np.abs(a - ref)) < 1e-13
    assert np.max(np.abs(b - ref)) < 1e-13


def test_select_all_reproduces_dense():
    Q, K, V, ql, kl, _ = _random_clustered_problem(7)
    sel = [np.arange(6) for _ in range(4)]
    dense = orc.dense_attention(Q, K, V)
    assert np.max(np.abs(orc.sparse_attention_mask(Q, K, V, ql, kl, sel) - dense)) < 1e-12
    assert np.max(np.abs(orc.sparse_attention_gather(Q, K, V, ql, kl, sel) - dense)) < 1e-12


def test_one_selected_cluster_with_constant_value():
    Q, K, V, ql, kl, _ = _random_clustered_problem(8)
    V = V.copy()
    V[kl == 2] = 3.25
    sel = [np.array([2]) for _ in range(4)]
    out = orc.sparse_attention_mask(Q, K, V, ql, kl, sel)
    assert np.allclose(out, 3.25, atol=1e-13)


def test_gather_rows_subset():
    Q, K, V, ql, kl, sel = _random_clustered_problem(9)
    full = orc.sparse_attention_gather(Q, K, V, ql, kl, sel)
    rows = np.array([0, 5, 17, 40])
    part = orc.sparse_attention_gather(Q, K, V, ql, kl, sel, rows=rows)
    assert np.allclose(part[rows], full[rows], atol=1e-14)
    others = np.setdiff1d(np.arange(48), rows)
    assert np.all(part[others] == 0)


def test_empty_selection_and_empty_cluster_rows_are_zero():
    Q, K, V, ql, kl, sel = _random_clustered_problem(10)
    sel = list(sel)
    sel[1] = np.zeros(0, dtype=np.int64)
    a = orc.sparse_attention_mask(Q, K, V, ql, kl, sel, n_kclusters=6)
    b = orc.sparse_attention_gather(Q, K, V, ql, kl, sel)
    assert np.all(a[ql == 1] == 0) and np.all(b[ql == 1] == 0)
    assert np.allclose(a, b, atol=1e-13)


def test_planted_mistakes_are_caught():
    """A wrong scale, a dropped max-subtraction sign or transposed operands must fail the pins."""
    rng = np.random.default_rng(11)
    Q, K, V = rng.standard_normal((5, 8)), rng.standard_normal((9, 8)), rng.standard_normal((9, 8))
    ref = brute_force_attention(Q, K, V, 1 / math.sqrt(8))
    wrong_scale = orc.dense_attention(Q, K, V, 1.0 / 8)
    assert np.max(np.abs(wrong_scale - ref)) > 1e-3
    neg = orc.dense_attention(-Q, K, V)
    assert np.max(np.abs(neg - ref)) > 1e-3
