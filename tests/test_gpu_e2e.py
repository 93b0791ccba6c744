"""End-to-end GPU parity of the fused call (Algorithm 3)."""
import numpy as np
import pytest
import torch

from oracle import adacluster_oracle as orc
from paper_2604_18348_amd import binding as B
from paper_2604_18348_amd import workloads as wl
from tests.helpers import attn_errors, sel_from_dev, to_dev, to_np

pytestmark = pytest.mark.gpu


def oracle_from_gpu_intermediates(Q, K, V, outs, p):
    """Chained oracle: the GPU's labels and selection drive the oracle's attention."""
    H = Q.shape[0]
    ql = outs["q_labels"].cpu().numpy()
    kl = outs["k_labels"].cpu().numpy()
    sel = sel_from_dev(outs["sel_idx"], outs["sel_cnt"])
    return np.stack([orc.sparse_attention_gather(Q[h], K[h], V[h], ql[h], kl[h], sel[h]) for h in range(H)])


def oracle_selection_from_gpu_centroids(outs, p, h):
    kc = int(outs["k_count"][h])
    sizes = outs["k_sizes"].cpu().numpy()[h, :kc]
    S = orc.cluster_scores(p.score_mode, to_np(outs["q_centroids"])[h], to_np(outs["k_centroids"])[h, :kc],
                           None, None, sizes)
    if bool(outs["full_flag"][h]):
        return [np.flatnonzero(sizes > 0) for _ in range(p.q_clusters)]
    if p.select_mode == 0:
        return orc.select_topk(S, p.topk)
    scale = float(np.float32(1.0 / np.sqrt(np.float32(p.d))))
    return orc.select_topp(S, sizes, to_np(outs["q_mean_norm"])[h] * scale, p.top_p)


def test_config1_fp32_free_running_matches_oracle():
    cfg = wl.CONFIGS["c1"]
    Q, K, V = wl.make_qkv("c1")
    p = B.Params(H=1, N=4096, d=64, dtype=B.F32, **cfg["params"])
    outs = B.alloc_outputs(p, "cuda")
    O = to_np(B.adacluster_attn(p, to_dev(Q, B.F32), to_dev(K, B.F32), to_dev(V, B.F32), outs=outs))
    torch.cuda.synchronize()
    ref, info, tau = orc.adacluster_attention(Q, K, V, use_gather=True, **cfg["params"])
    print("tau", float(outs["tau_used"][0]), tau, "k_count", int(outs["k_count"][0]),
          info[0]["k"]["assign_centroids"].shape[0], "stages", info[0]["k"]["stage_offs"])
    ql_agree = float((outs["q_labels"].cpu().numpy()[0] == info[0]["q"]["labels"]).mean())
    same_count = int(outs["k_count"][0]) == info[0]["k"]["assign_centroids"].shape[0]
    kl_agree = float((outs["k_labels"].cpu().numpy()[0] == info[0]["k"]["labels"]).mean()) if same_count else 0.0
    print("q label agreement", ql_agree, "k label agreement", kl_agree)
    # chained check always holds
    chained = oracle_from_gpu_intermediates(Q, K, V, outs, p)
    rel, mx = attn_errors(O[0], chained[0])
    print("chained", rel, mx)
    assert mx < 1e-4
    # selection from the GPU's centroids is bit-exact
    sel_gpu = sel_from_dev(outs["sel_idx"], outs["sel_cnt"])[0]
    sel_ref = oracle_selection_from_gpu_centroids(outs, p, 0)
    for i in range(p.q_clusters):
        assert np.array_equal(sel_gpu[i], sel_ref[i])
    # free-running: same trajectory on this well-separated input
    assert ql_agree == 1.0 and kl_agree == 1.0
    rel, mx = attn_errors(O[0], ref[0])
    print("free-running", rel, mx)
    assert mx < 1e-4


@pytest.mark.parametrize("name,d,N,extra", [
    ("bf16-topk", 64, 3100, dict(select_mode=0, topk=6)),
    ("bf16-topp", 128, 2200, dict(select_mode=1, top_p=0.9)),
    ("bf16-selectall", 64, 1500, dict(select_mode=0, topk=10 ** 6)),
])
def test_fused_bf16_chained(name, d, N, extra):
    H = 3
    Q, K, V = wl.make_small(31, N, d, 12, dtype="bf16", H=H)
    rng = np.random.default_rng(1)
    K[2] = wl.round_bf16_f32(rng.standard_normal((N, d)).astype(np.float32))      # diffuse head -> F
    p = B.Params(H=H, N=N, d=d, dtype=B.BF16, q_clusters=13, q_iters=3, k_iters=3, k_m0=20, k_m_min=4,
                 k_max_clusters=80, min_unassigned_frac=0.03, **extra)
    outs = B.alloc_outputs(p, "cuda")
    O = to_np(B.adacluster_attn(p, to_dev(Q, B.BF16), to_dev(K, B.BF16), to_dev(V, B.BF16), outs=outs))
    torch.cuda.synchronize()
    assert outs["full_flag"].cpu().tolist() == [0, 0, 1]
    chained = oracle_from_gpu_intermediates(Q, K, V, outs, p)
    sel_gpu = sel_from_dev(outs["sel_idx"], outs["sel_cnt"])
    for h in range(H):
        rel, mx = attn_errors(O[h], chained[h])
        print(name, h, "rel", rel, "max", mx, "k_count", int(outs["k_count"][h]))
        assert rel < 1e-2 and mx < 2e-2
        sel_ref = oracle_selection_from_gpu_centroids(outs, p, h)
        for i in range(p.q_clusters):
            assert np.array_equal(sel_gpu[h][i], sel_ref[i]), (h, i)
    # the flagged head is dense attention
    rel, mx = attn_errors(O[2], orc.dense_attention(Q[2], K[2], V[2]))
    assert rel < 1e-2 and mx < 2e-2
    if name == "bf16-selectall":
        for h in range(H):
            rel, mx = attn_errors(O[h], orc.dense_attention(Q[h], K[h], V[h]))
            assert rel < 1e-2 and mx < 2e-2
    # the fused call without output pointers gives the same result, and the call is deterministic
    O2 = to_np(B.adacluster_attn(p, to_dev(Q, B.BF16), to_dev(K, B.BF16), to_dev(V, B.BF16)))
    assert np.array_equal(O, O2)


def test_stagewise_calls_equal_the_fused_call():
    H, N, d = 2, 2000, 64
    Q, K, V = wl.make_small(32, N, d, 20, dtype="bf16", H=H)
    p = B.Params(H=H, N=N, d=d, dtype=B.BF16, q_clusters=9, k_m0=16, k_m_min=4, k_max_clusters=64, topk=5,
                 min_unassigned_frac=0.03)
    Qd, Kd, Vd = to_dev(Q, B.BF16), to_dev(K, B.BF16), to_dev(V, B.BF16)
    O_fused = B.adacluster_attn(p, Qd, Kd, Vd)
    q = B.adacluster_qcluster(p, Qd)
    k = B.adacluster_kcluster(p, Kd, want_box=False)
    si, sc = B.adacluster_select(p, q["q_centroids"], q["q_mean_norm"], k["k_centroids"], None, None, k["k_sizes"],
                                 k["k_count"], k["full_flag"])
    O_steps = B.adacluster_sparse_attn(p, Qd, Kd, Vd, q["q_labels"], k["k_labels"], k["k_count"], si, sc)
    torch.cuda.synchronize()
    assert torch.equal(O_fused, O_steps)


def test_fused_warm_start_call_chained():
    """A second call with q_init_mode = k_init_mode = 1 reuses the first call's centres."""
    H, N, d = 2, 2400, 64
    Q, K, V = wl.make_small(33, N, d, 16, dtype="bf16", H=H)
    p = B.Params(H=H, N=N, d=d, dtype=B.BF16, q_clusters=11, k_m0=20, k_m_min=4, k_max_clusters=80, topk=5,
                 min_unassigned_frac=0.03)
    outs = B.alloc_outputs(p, "cuda")
    B.adacluster_attn(p, to_dev(Q, B.BF16), to_dev(K, B.BF16), to_dev(V, B.BF16), outs=outs)
    kc0 = outs["k_count"].cpu().numpy().copy()
    rng = np.random.default_rng(2)
    Q2 = wl.round_bf16_f32(Q + 0.05 * rng.standard_normal(Q.shape).astype(np.float32))
    K2 = wl.round_bf16_f32(K + 0.05 * rng.standard_normal(K.shape).astype(np.float32))
    pw = B.Params(**{**p.__dict__, "q_init_mode": 1, "k_init_mode": 1, "q_iters": 2, "k_iters": 2})
    O = to_np(B.adacluster_attn(pw, to_dev(Q2, B.BF16), to_dev(K2, B.BF16), to_dev(V, B.BF16), outs=outs))
    torch.cuda.synchronize()
    assert np.array_equal(outs["k_count"].cpu().numpy(), kc0)
    chained = oracle_from_gpu_intermediates(Q2, K2, V, outs, pw)
    sel_gpu = sel_from_dev(outs["sel_idx"], outs["sel_cnt"])
    for h in range(H):
        rel, mx = attn_errors(O[h], chained[h])
        assert rel < 1e-2 and mx < 2e-2
        sel_ref = oracle_selection_from_gpu_centroids(outs, pw, h)
        for i in range(p.q_clusters):
            assert np.array_equal(sel_gpu[h][i], sel_ref[i])


def test_two_host_threads_on_one_device():
    """Two host threads run the fused call at the same time, each on a stream and a workspace of its own;
    the library's second stream, its events and the stage read-back slots are per thread, so both must
    reproduce what the same calls give one after the other (the call is deterministic)."""
    import threading
    H, N, d = 2, 2600, 64
    cases = []
    for seed in (41, 42):
        Q, K, V = wl.make_small(seed, N, d, 10, dtype="bf16", H=H)
        cases.append((to_dev(Q, B.BF16), to_dev(K, B.BF16), to_dev(V, B.BF16)))
    p = B.Params(H=H, N=N, d=d, dtype=B.BF16, q_clusters=9, q_iters=3, k_iters=3, k_m0=16, k_m_min=4,
                 k_max_clusters=64, min_unassigned_frac=0.03, topk=5)
    ref = [B.adacluster_attn(p, *c).clone() for c in cases]
    torch.cuda.synchronize()
    got = [None, None]
    errs = []

    def work(i):
        try:
            s = torch.cuda.Stream()
            with torch.cuda.stream(s):
                ws = B.workspace(p)
                for _ in range(5):
                    out = B.adacluster_attn(p, *cases[i], ws=ws)
                s.synchronize()
            got[i] = out
        except Exception as e:      # surfaced in the main thread
            errs.append(e)

    ts = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    assert not errs, errs
    for i in range(2):
        assert torch.equal(got[i], ref[i])


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
def test_hand_worked_call_on_the_device(dtype):
    """The eight-token call worked out by hand in tests/test_oracle_hand_worked.py, its two dimensions
    zero-padded to 64: the device must land on the hand-derived stages, centres, selections and rows."""
    from tests import test_oracle_hand_worked as hw
    d = 64
    pad = lambda X: np.concatenate([X, np.zeros((8, d - 2))], axis=1)[None].astype(np.float32)
    Q, K, V = pad(hw.Q), pad(hw.K), pad(hw.V)
    p = B.Params(H=1, N=8, d=d, dtype=dtype, score_mode=0, select_mode=0, **hw.PARAMS)
    outs = B.alloc_outputs(p, "cuda")
    O = to_np(B.adacluster_attn(p, to_dev(Q, dtype), to_dev(K, dtype), to_dev(V, dtype), outs=outs))[0]
    torch.cuda.synchronize()
    assert int(outs["k_count"][0]) == 3 and not bool(outs["full_flag"][0])
    assert outs["k_labels"].cpu().numpy()[0].tolist() == [0, 0, 0, 0, 1, 1, 1, 2]
    assert outs["q_labels"].cpu().numpy()[0].tolist() == [0, 0, 0, 0, 1, 1, 1, 1]
    assert outs["k_sizes"].cpu().numpy()[0, :3].tolist() == [4, 3, 1]
    kc = to_np(outs["k_centroids"])[0, :3]
    assert np.array_equal(kc[:, :2], np.array([[4.5, 1], [-4, 1], [-12, 5]])) and np.all(kc[:, 2:] == 0)
    qc = to_np(outs["q_centroids"])[0]
    assert np.allclose(qc[:, :2], [[hw.S2, hw.S2], [-hw.S2, hw.S2]], atol=1e-6) and np.all(qc[:, 2:] == 0)
    assert np.allclose(to_np(outs["q_mean_norm"])[0], 7.5, atol=1e-5)
    sel = sel_from_dev(outs["sel_idx"], outs["sel_cnt"])[0]
    assert [s.tolist() for s in sel] == [[0, 2], [1, 2]]
    tol = 1e-5 if dtype == B.F32 else 1e-2
    den0 = 3392 + 2.0 ** -8
    assert abs(O[0, 0] - 3392 / den0) < tol and abs(O[0, 1] - 2.0 ** -8 / den0) < tol
    den4 = 1344 + 2.0 ** 28
    assert abs(O[4, 0] - 100 * 1344 / den4) < tol and abs(O[4, 1] - (100 * 1344 + 2.0 ** 28) / den4) < tol
    assert np.all(O[:, 2:] == 0)
    assert np.allclose(O[:4, :2].sum(axis=1), 1.0, atol=tol)


@pytest.mark.parametrize("d", [64, 128])
def test_concentrated_attention_is_kept_by_a_small_selection(d):
    """What the method is for: when a query's soft-max mass sits on the keys of a few clusters (here the
    query means are the key means of the same component, scaled up), the centroid scores must find them:
    a selection of 4 clusters out of about 30 keeps nearly all of the dense soft-max mass, and the output is
    close to dense attention although three quarters of the keys are skipped."""
    from paper_2604_18348_amd.ablate import attention_mass_kept
    H, N, M = 2, 3000, 24
    rng = np.random.default_rng(77)
    comp = rng.integers(0, M, (H, N))
    mu = rng.standard_normal((H, M, d)).astype(np.float32)
    K = wl.round_bf16_f32(np.take_along_axis(mu, comp[..., None], 1) + 0.2 * rng.standard_normal((H, N, d)).astype(np.float32))
    Q = wl.round_bf16_f32(2.0 * np.take_along_axis(mu, comp[..., None], 1) + 0.2 * rng.standard_normal((H, N, d)).astype(np.float32))
    V = wl.round_bf16_f32(rng.standard_normal((H, N, d)).astype(np.float32))
    p = B.Params(H=H, N=N, d=d, dtype=B.BF16, q_clusters=24, q_iters=3, k_iters=3, k_m0=24, k_m_min=4,
                 k_max_clusters=96, tau_factor=1.5, min_unassigned_frac=0.03, topk=4)
    outs = B.alloc_outputs(p, "cuda")
    Qd, Kd, Vd = to_dev(Q, B.BF16), to_dev(K, B.BF16), to_dev(V, B.BF16)
    O = B.adacluster_attn(p, Qd, Kd, Vd, outs=outs)
    dense = B.adacluster_dense_attn(p, Qd, Kd, Vd)
    torch.cuda.synchronize()
    assert int(outs["full_flag"].sum()) == 0
    qs, ks = outs["q_sizes"].cpu().numpy().astype(np.int64), outs["k_sizes"].cpu().numpy().astype(np.int64)
    sel = sel_from_dev(outs["sel_idx"], outs["sel_cnt"])
    pairs = sum(int(qs[h, i]) * int(ks[h, sel[h][i]].sum()) for h in range(H) for i in range(p.q_clusters))
    density = pairs / (H * float(N) * float(N))
    mass = attention_mass_kept(torch, Qd, Kd, outs, p, 1.0 / np.sqrt(d), per_head=256)
    rel = float(torch.linalg.vector_norm(O.float() - dense.float()) / torch.linalg.vector_norm(dense.float()))
    print("density", density, "mass kept", mass, "rel-L2 vs dense", rel, "k_count", outs["k_count"].cpu().tolist())
    assert density < 0.3 and mass > 0.97 and rel < 0.1


def test_many_heads():
    """More heads than any benchmark configuration has (the per-head kernels take one workgroup per head,
    the attention grid deals heads to XCDs eight at a time with a remainder): a few heads checked the
    chained way, every head's selection checked against the oracle's."""
    H, N, d = 70, 640, 64
    Q, K, V = wl.make_small(91, N, d, 8, dtype="bf16", H=H)
    p = B.Params(H=H, N=N, d=d, dtype=B.BF16, q_clusters=5, q_iters=2, k_iters=2, k_m0=8, k_m_min=2,
                 k_max_clusters=40, min_unassigned_frac=0.02, topk=3)
    outs = B.alloc_outputs(p, "cuda")
    O = to_np(B.adacluster_attn(p, to_dev(Q, B.BF16), to_dev(K, B.BF16), to_dev(V, B.BF16), outs=outs))
    torch.cuda.synchronize()
    sel_gpu = sel_from_dev(outs["sel_idx"], outs["sel_cnt"])
    ql, kl = outs["q_labels"].cpu().numpy(), outs["k_labels"].cpu().numpy()
    for h in range(H):
        sel_ref = oracle_selection_from_gpu_centroids(outs, p, h)
        for i in range(p.q_clusters):
            assert np.array_equal(sel_gpu[h][i], sel_ref[i]), (h, i)
    for h in (0, 7, 8, 33, 63, 64, 69):
        ref = orc.sparse_attention_gather(Q[h], K[h], V[h], ql[h], kl[h], sel_gpu[h])
        rel, mx = attn_errors(O[h], ref)
        assert rel < 1e-2 and mx < 2e-2, (h, rel, mx)


def test_warm_start_call_replays_from_a_hip_graph():
    """The warm-start call (Sec. 3.2.2) has no host read-back and allocates nothing: captured into a HIP graph on
    the caller's stream (its second stream joins the capture through the fork and join events), every replay
    must give what the same sequence of eager calls gives, bit for bit.  The centres of a call are the start of
    the next, so replay r is compared with the r-th eager call from the same state; eager work and
    synchronisations sit between the replays."""
    import dataclasses
    H, N, d = 2, 3000, 64
    Q, K, V = wl.make_small(5, N, d, 12, dtype="bf16", H=H)
    Qd, Kd, Vd = to_dev(Q, B.BF16), to_dev(K, B.BF16), to_dev(V, B.BF16)
    p = B.Params(H=H, N=N, d=d, dtype=B.BF16, q_clusters=9, q_iters=3, k_iters=3, k_m0=20, k_m_min=4,
                 k_max_clusters=80, min_unassigned_frac=0.03, topk=5)
    ws = B.workspace(p)
    outs = B.alloc_outputs(p, "cuda")
    O = torch.empty_like(Qd)
    B.adacluster_attn(p, Qd, Kd, Vd, outs=outs, out=O, ws=ws)                  # the cold call of step 0
    torch.cuda.synchronize()
    pw = dataclasses.replace(p, q_init_mode=1, k_init_mode=1, q_iters=2, k_iters=2)
    state0 = {k: v.clone() for k, v in outs.items() if v is not None}

    def restore():
        for k, v in state0.items():
            outs[k].copy_(v)

    eager = []
    for _ in range(3):
        B.adacluster_attn(pw, Qd, Kd, Vd, outs=outs, out=O, ws=ws)
        torch.cuda.synchronize()
        eager.append(O.clone())
    restore()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.adacluster_attn(pw, Qd, Kd, Vd, outs=outs, out=O, ws=ws)
    restore()
    torch.cuda.synchronize()
    for r in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert float(torch.rand(4096, device="cuda").sum()) > 0                 # eager work between the replays
        assert torch.equal(O, eager[r]), r
