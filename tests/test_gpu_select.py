"""GPU selection vs oracle: given identical centroids the selected index sets are bit-exact."""
import numpy as np
import pytest
import torch

from oracle import adacluster_oracle as orc
from paper_2604_18348_amd import binding as B
from tests.helpers import sel_from_dev

pytestmark = pytest.mark.gpu


def make_inputs(seed, H, Cq, cap, kc_list, d):
    rng = np.random.default_rng(seed)
    qc = rng.standard_normal((H, Cq, d)).astype(np.float32)
    qc /= np.linalg.norm(qc, axis=2, keepdims=True)
    kcent = rng.standard_normal((H, cap, d)).astype(np.float32)
    spread = np.abs(rng.standard_normal((H, cap, d))).astype(np.float32)
    bmin, bmax = kcent - spread, kcent + spread
    sizes = rng.integers(0, 50, (H, cap)).astype(np.int32)
    sizes[:, 1] = 0
    mean_norm = rng.uniform(4, 12, (H, Cq)).astype(np.float32)
    kcount = np.asarray(kc_list, dtype=np.int32)
    for h in range(H):
        sizes[h, kcount[h]:] = 0
    return qc, mean_norm, kcent, bmin, bmax, sizes, kcount


@pytest.mark.parametrize("score_mode", [B.SCORE_TQ, B.SCORE_BOX, B.SCORE_DOT])
@pytest.mark.parametrize("select_mode,topk,top_p", [(0, 8, 0.9), (0, 1, 0.9), (0, 500, 0.9), (1, 8, 0.9),
                                                   (1, 8, 0.3), (1, 8, 1.0)])
@pytest.mark.parametrize("d", [64, 128])
def test_selection_is_bit_exact(score_mode, select_mode, topk, top_p, d):
    H, Cq, m0, nmax = 3, 7, 40, 260
    cap = m0 + nmax
    qc, mean_norm, kcent, bmin, bmax, sizes, kcount = make_inputs(7, H, Cq, cap, [300, 33, 1], d)
    full = np.array([0, 0, 0], dtype=np.int32)
    p = B.Params(H=H, N=10000, d=d, q_clusters=Cq, k_m0=m0, k_m_min=4, k_max_clusters=nmax,
                 score_mode=score_mode, select_mode=select_mode, topk=topk, top_p=top_p)
    c = lambda a: torch.from_numpy(a).cuda()
    si, sc = B.adacluster_select(p, c(qc), c(mean_norm), c(kcent), c(bmin), c(bmax), c(sizes), c(kcount), c(full))
    got = sel_from_dev(si, sc)
    scale = float(np.float32(1.0 / np.sqrt(np.float32(d))))
    for h in range(H):
        kc = kcount[h]
        S = orc.cluster_scores(score_mode, qc[h].astype(np.float64), kcent[h, :kc].astype(np.float64),
                               bmin[h, :kc].astype(np.float64), bmax[h, :kc].astype(np.float64), sizes[h, :kc])
        if select_mode == 0:
            ref = orc.select_topk(S, topk)
        else:
            ref = orc.select_topp(S, sizes[h, :kc], mean_norm[h].astype(np.float64) * scale, top_p)
        for i in range(Cq):
            assert np.array_equal(got[h][i], ref[i]), (h, i, got[h][i], ref[i])


def test_full_flag_selects_all_nonempty_and_ties_go_low():
    H, Cq, d = 2, 3, 64
    m0, nmax = 8, 24
    cap = m0 + nmax
    qc, mean_norm, kcent, bmin, bmax, sizes, kcount = make_inputs(9, H, Cq, cap, [20, 20], d)
    kcent[1, :20] = kcent[1, 0]                      # all scores equal in head 1 -> lowest ids win
    sizes[1, :20] = 5
    full = np.array([1, 0], dtype=np.int32)
    p = B.Params(H=H, N=10000, d=d, q_clusters=Cq, k_m0=m0, k_m_min=4, k_max_clusters=nmax, topk=4)
    c = lambda a: torch.from_numpy(a).cuda()
    si, sc = B.adacluster_select(p, c(qc), c(mean_norm), c(kcent), None, None, c(sizes), c(kcount), c(full))
    got = sel_from_dev(si, sc)
    for i in range(Cq):
        assert np.array_equal(got[0][i], np.flatnonzero(sizes[0, :20] > 0))
        assert got[1][i].tolist() == [0, 1, 2, 3]


@pytest.mark.parametrize("topk", [5, 64, 300])
def test_equal_scores_at_the_topk_boundary_over_several_chunks(topk):
    """Duplicate key centroids give exactly equal scores; the ones that tie at the k-th place must be
    taken in ascending index order, wherever in the list they sit (the kernel walks the list 256 at a
    time)."""
    H, Cq, d = 2, 5, 64
    m0, nmax = 100, 700
    cap = m0 + nmax
    kc = 700
    qc, mean_norm, kcent, bmin, bmax, sizes, kcount = make_inputs(11, H, Cq, cap, [kc, kc], d)
    rng = np.random.default_rng(12)
    sizes[:, :kc] = 3
    sizes[:, 17] = 0
    for h in range(H):
        # 40 groups of 12 duplicates each, members spread over the whole list
        ids = rng.permutation(kc)[:480].reshape(40, 12)
        for g in ids:
            kcent[h, g] = kcent[h, g[0]]
    full = np.zeros(H, dtype=np.int32)
    p = B.Params(H=H, N=100000, d=d, q_clusters=Cq, k_m0=m0, k_m_min=4, k_max_clusters=nmax, topk=topk)
    c = lambda a: torch.from_numpy(a).cuda()
    si, sc = B.adacluster_select(p, c(qc), c(mean_norm), c(kcent), None, None, c(sizes), c(kcount), c(full))
    got = sel_from_dev(si, sc)
    for h in range(H):
        S = orc.cluster_scores(B.SCORE_TQ, qc[h].astype(np.float64), kcent[h, :kc].astype(np.float64), None, None,
                               sizes[h, :kc])
        ref = orc.select_topk(S, topk)
        for i in range(Cq):
            assert np.array_equal(got[h][i], ref[i]), (h, i)
