"""Seeded random configurations of the fused call (Algorithm 3), small enough for the oracle: shapes,
cluster counts, budgets, dtypes and switches drawn at random; every case is checked the chained way
(the GPU's own centroids drive the oracle's selection, its labels and selection the oracle's attention),
plus the invariants of the clusterings."""
import numpy as np
import pytest
import torch

from oracle import adacluster_oracle as orc
from paper_2604_18348_amd import binding as B
from paper_2604_18348_amd import workloads as wl
from tests.helpers import attn_errors, sel_from_dev, to_dev, to_np
from tests.test_gpu_e2e import oracle_from_gpu_intermediates, oracle_selection_from_gpu_centroids

pytestmark = pytest.mark.gpu


def draw(seed):
    r = np.random.default_rng(1000 + seed)
    bf16 = bool(r.integers(0, 4) > 0)
    d = int(r.choice([64, 128]))
    N = int(r.choice([1, 33, 257, 700, 1500, 2900, 5000]))
    H = int(r.integers(1, 4))
    Cq = int(min(N, r.choice([1, 3, 9, 33, 65])))
    m0 = int(min(N, r.choice([1, 4, 16, 40, 130])))
    m_min = int(min(m0, r.choice([1, 2, 8])))
    nmax = int(max(m0, r.choice([m0, 2 * m0, 8 * m0 + 3])))
    params = dict(q_clusters=Cq, q_iters=int(r.integers(1, 4)), k_iters=int(r.integers(1, 4)), k_m0=m0, k_m_min=m_min,
                  k_max_clusters=nmax, k_max_stages=int(r.integers(1, 8)),
                  min_unassigned_frac=float(r.choice([0.0, 0.03, 0.3])), tau_factor=float(r.choice([0.8, 1.5, 3.0])),
                  score_mode=int(r.choice([0, 2])),           # Alg. 2 on centroids or the plain dot
                  select_mode=int(r.integers(0, 2)), topk=int(r.choice([1, 3, 16, 10 ** 6])),
                  top_p=float(r.choice([0.3, 0.9, 1.0])), q_no_norm=int(r.integers(0, 4) == 0))
    return bf16, d, N, H, params


@pytest.mark.parametrize("seed", range(24))
def test_random_configuration(seed):
    bf16, d, N, H, params = draw(seed)
    dtype = B.BF16 if bf16 else B.F32
    M = max(1, min(12, N))
    Q, K, V = wl.make_small(500 + seed, N, d, M, dtype="bf16" if bf16 else "f32", H=H)
    p = B.Params(H=H, N=N, d=d, dtype=dtype, **params)
    print("case", seed, "bf16" if bf16 else "f32", "H", H, "N", N, "d", d, params, flush=True)
    outs = B.alloc_outputs(p, "cuda")
    O = to_np(B.adacluster_attn(p, to_dev(Q, dtype), to_dev(K, dtype), to_dev(V, dtype), outs=outs))
    torch.cuda.synchronize()
    ql, kl = outs["q_labels"].cpu().numpy(), outs["k_labels"].cpu().numpy()
    kcnt = outs["k_count"].cpu().numpy()
    qs, ks = outs["q_sizes"].cpu().numpy(), outs["k_sizes"].cpu().numpy()
    sel_gpu = sel_from_dev(outs["sel_idx"], outs["sel_cnt"])
    chained = oracle_from_gpu_intermediates(Q, K, V, outs, p)
    for h in range(H):
        assert 1 <= kcnt[h] <= p.cap
        assert ql[h].min() >= 0 and ql[h].max() < p.q_clusters
        assert kl[h].min() >= 0 and kl[h].max() < kcnt[h]
        assert np.array_equal(qs[h], np.bincount(ql[h], minlength=p.q_clusters))
        assert np.array_equal(ks[h, :kcnt[h]], np.bincount(kl[h], minlength=kcnt[h]))
        sel_ref = oracle_selection_from_gpu_centroids(outs, p, h)
        for i in range(p.q_clusters):
            assert np.array_equal(sel_gpu[h][i], sel_ref[i]), (h, i)
        rel, mx = attn_errors(O[h], chained[h])
        if bf16:
            assert rel < 1e-2 and mx < 2e-2, (rel, mx)
        else:
            assert mx < 1e-4, (rel, mx)


@pytest.mark.parametrize("seed", range(16))
def test_random_key_clustering_keeps_the_structure_of_algorithm_1(seed):
    """Seeded random sizes, centre counts, pass counts, stage limits and thresholds of the key clustering
    alone (bf16), with a noisier first head half of the time: stage counts follow the rule, removals agree
    with the reported centres and the threshold, labels are the arg-min, member statistics match."""
    from tests.test_gpu_cluster import check_kcluster
    r = np.random.default_rng(7000 + seed)
    d = int(r.choice([64, 128]))
    N = int(r.choice([900, 2500, 6000, 9000, 14000]))
    H = int(r.integers(1, 4))
    m0 = int(r.choice([8, 24, 32, 60, 100, 128, 200]))
    m_min = int(min(m0, r.choice([1, 4, 16, 30])))
    p = B.Params(H=H, N=N, d=d, dtype=B.BF16, q_clusters=4, k_iters=int(r.integers(1, 4)), k_m0=m0, k_m_min=m_min,
                 k_max_clusters=int(r.choice([m0, 3 * m0, 10 * m0])), k_max_stages=int(r.integers(1, 9)),
                 tau_factor=float(r.choice([0.7, 0.9, 1.2, 1.5])),
                 min_unassigned_frac=float(r.choice([0.0, 0.02, 0.2])))
    _, K, _ = wl.make_small(9000 + seed, N, d, int(r.choice([6, 20, 60])), dtype="bf16", H=H)
    if r.integers(0, 2):
        K[0] = wl.round_bf16_f32(K[0] + float(r.choice([0.3, 1.0])) * r.standard_normal((N, d)).astype(np.float32))
    print("case", seed, "H", H, "N", N, "d", d, p, flush=True)
    out = B.adacluster_kcluster(p, to_dev(K, B.BF16))
    torch.cuda.synchronize()
    check_kcluster(K, p, out, B.BF16)
