"""adacluster_stats_fetch against counts made on the oracle's side: stages, |U| per stage, |C|, F and the
executed (query, key) pairs, exactly; the issued (tile-padded) pairs against a recount from the sizes."""
import numpy as np
import pytest
import torch

from oracle import adacluster_oracle as orc
from paper_2604_18348_amd import binding as B
from paper_2604_18348_amd import workloads as wl
from tests.helpers import sel_from_dev, to_dev

pytestmark = pytest.mark.gpu


def pairs_from_sizes(q_sizes, k_sizes, sel, bm):
    """executed and issued pairs of one head, recounted: query clusters in tiles of bm rows, a tile's rows
    rounded up to whole 32-query waves and its keys to whole 64-key tiles (no key list cut)."""
    ex = iss = tiles = 0
    for i, s in enumerate(sel):
        keys = int(k_sizes[np.asarray(s, dtype=np.int64)].sum()) if len(s) else 0
        nq = int(q_sizes[i])
        ex += nq * keys
        for r0 in range(0, nq, bm):
            rows = min(bm, nq - r0)
            iss += (rows + 31) // 32 * 32 * ((keys + 63) // 64 * 64)
            tiles += 1
    return ex, iss, tiles


def test_stats_match_the_oracle_run_config1():
    """Config 1 runs the same trajectory on both sides, so the oracle's own stage loop gives the counts."""
    cfg = wl.CONFIGS["c1"]
    Q, K, V = wl.make_qkv("c1")
    p = B.Params(H=1, N=4096, d=64, dtype=B.F32, **cfg["params"])
    ws = B.workspace(p)
    outs = B.alloc_outputs(p, "cuda")
    B.adacluster_attn(p, to_dev(Q, B.F32), to_dev(K, B.F32), to_dev(V, B.F32), outs=outs, ws=ws)
    st = B.adacluster_stats_fetch(p, ws)[0]
    _, info, _ = orc.adacluster_attention(Q, K, V, use_gather=True, **cfg["params"])
    k = info[0]["k"]
    n_un = k["n_unassigned"]
    assert st["stages"] == len(n_un) - 1 and st["stages"] >= 2
    assert st["unassigned"][:len(n_un)] == [int(x) for x in n_un]
    assert st["k_count"] == k["assign_centroids"].shape[0] and st["full_flag"] == int(k["full_flag"])
    qs = np.bincount(info[0]["q"]["labels"], minlength=p.q_clusters)
    ex, iss, tiles = pairs_from_sizes(qs, k["sizes"], info[0]["sel"], 64)
    assert st["executed_pairs"] == ex
    assert st["issued_pairs"] == iss and st["q_tiles"] == tiles


@pytest.mark.parametrize("d,N,extra", [(64, 3100, dict(topk=6)), (128, 2300, dict(topk=4, tau_abs=3.0))])
def test_stats_match_counts_from_the_call_outputs(d, N, extra):
    """bf16, three heads, one diffuse (it ends with F set): the figures against the labels, stage marks and
    selections the same call returned."""
    H = 3
    Q, K, V = wl.make_small(41, N, d, 12, dtype="bf16", H=H)
    K[2] = wl.round_bf16_f32(np.random.default_rng(2).standard_normal((N, d)).astype(np.float32))
    p = B.Params(H=H, N=N, d=d, dtype=B.BF16, q_clusters=13, k_iters=2, k_m0=20, k_m_min=4, k_max_clusters=80,
                 min_unassigned_frac=0.03, **extra)
    ws = B.workspace(p)
    outs = B.alloc_outputs(p, "cuda")
    B.adacluster_attn(p, to_dev(Q, B.BF16), to_dev(K, B.BF16), to_dev(V, B.BF16), outs=outs, ws=ws)
    stats = B.adacluster_stats_fetch(p, ws)
    torch.cuda.synchronize()
    sof = outs["k_stage_of"].cpu().numpy()
    offs = outs["k_stage_offs"].cpu().numpy()
    kc, ff = outs["k_count"].cpu().numpy(), outs["full_flag"].cpu().numpy()
    qs, ks = outs["q_sizes"].cpu().numpy(), outs["k_sizes"].cpu().numpy()
    sel = sel_from_dev(outs["sel_idx"], outs["sel_cnt"])
    bm = 128
    assert ff[2] == 1
    for h in range(H):
        st = stats[h]
        assert st["k_count"] == kc[h] and st["full_flag"] == ff[h]
        stages = int(np.flatnonzero(offs[h] == kc[h])[0])          # first stage boundary that reaches |C|
        assert st["stages"] == stages
        # |U| at the head of stage t: tokens no earlier stage removed
        un = [int(((sof[h] < 0) | (sof[h] >= t)).sum()) for t in range(stages + 1)]
        assert st["unassigned"][:stages + 1] == un
        ex, iss, tiles = pairs_from_sizes(qs[h], ks[h], sel[h], bm)
        assert st["executed_pairs"] == ex
        if st["q_tiles"] == tiles:                                   # no key list was cut
            assert st["issued_pairs"] == iss
        assert st["issued_pairs"] >= st["executed_pairs"]
