"""GPU parity of the attention kernels against the fp64 oracle (Alg. 3 lines 9-10, dense branch).

Tolerances (from the benchmark spec): fp32 I/O 1e-4 max-abs; bf16 I/O 1e-2 relative L2 and 2e-2
max-abs against the fp64 oracle fed the same bf16-rounded inputs."""
import numpy as np
import pytest
import torch

from oracle import adacluster_oracle as orc
from paper_2604_18348_amd import binding as B
from paper_2604_18348_amd import workloads as wl
from tests.helpers import attn_errors, sel_to_dev, to_dev, to_np

pytestmark = pytest.mark.gpu


def check(got, ref, dtype):
    rel, mx = attn_errors(got, ref)
    if dtype == B.F32:
        assert mx < 1e-4, (rel, mx)
    else:
        assert rel < 1e-2 and mx < 2e-2, (rel, mx)
    return rel, mx


def make_case(seed, N, d, dtype, H=2, Cq=5, Ck=23, M=12):
    Q, K, V = wl.make_small(seed, N, d, M, dtype="bf16" if dtype == B.BF16 else "f32", H=H)
    rng = np.random.default_rng(seed + 100)
    ql = rng.integers(0, Cq, (H, N)).astype(np.int32)
    kl = rng.integers(0, Ck, (H, N)).astype(np.int32)
    # ragged clusters: squeeze most keys into a few clusters, leave one empty
    kl[kl == 3] = 4
    sel = []
    for h in range(H):
        rows = []
        for i in range(Cq):
            k = int(rng.integers(1, Ck))
            rows.append(np.sort(rng.choice(Ck, size=k, replace=False)).astype(np.int64))
        sel.append(rows)
    return Q, K, V, ql, kl, sel


def run_sparse(Q, K, V, ql, kl, sel, dtype, Cq, Ck):
    H, N, d = Q.shape
    p = B.Params(H=H, N=N, d=d, dtype=dtype, q_clusters=Cq, k_m0=min(4, N), k_m_min=1,
                 k_max_clusters=max(Ck, 4))
    assert p.cap >= Ck
    si, sc = sel_to_dev(sel, Cq, p.cap)
    O = B.adacluster_sparse_attn(p, to_dev(Q, dtype), to_dev(K, dtype), to_dev(V, dtype),
                                 torch.from_numpy(ql).cuda(), torch.from_numpy(kl).cuda(),
                                 torch.full((H,), Ck, dtype=torch.int32, device="cuda"), si, sc)
    torch.cuda.synchronize()
    return to_np(O)


@pytest.mark.parametrize("dtype,d,N", [(B.BF16, 64, 1000), (B.BF16, 128, 1537), (B.BF16, 64, 37),
                                       (B.F32, 64, 700), (B.F32, 128, 333)])
def test_sparse_attention_matches_oracle(dtype, d, N):
    Cq, Ck = 5, 23
    Q, K, V, ql, kl, sel = make_case(1, N, d, dtype)
    got = run_sparse(Q, K, V, ql, kl, sel, dtype, Cq, Ck)
    for h in range(Q.shape[0]):
        ref = orc.sparse_attention_gather(Q[h], K[h], V[h], ql[h], kl[h], sel[h])
        print("sparse", dtype, d, N, h, check(got[h], ref, dtype))


@pytest.mark.parametrize("dtype,d,N", [(B.BF16, 64, 1000), (B.BF16, 128, 777), (B.F32, 64, 515), (B.BF16, 128, 1),
                                       (B.BF16, 64, 64), (B.BF16, 64, 2048 + 63)])
def test_dense_attention_matches_oracle(dtype, d, N):
    H = 2
    Q, K, V = wl.make_small(2, N, d, max(1, min(12, N)), dtype="bf16" if dtype == B.BF16 else "f32", H=H)
    p = B.Params(H=H, N=N, d=d, dtype=dtype, q_clusters=1, k_m0=1, k_m_min=1, k_max_clusters=1)
    O = to_np(B.adacluster_dense_attn(p, to_dev(Q, dtype), to_dev(K, dtype), to_dev(V, dtype)))
    for h in range(H):
        print("dense", dtype, d, N, h, check(O[h], orc.dense_attention(Q[h], K[h], V[h]), dtype))


@pytest.mark.parametrize("dtype", [B.BF16, B.F32])
def test_selecting_every_cluster_reproduces_dense(dtype):
    Cq, Ck = 5, 23
    Q, K, V, ql, kl, _ = make_case(3, 900, 64, dtype)
    sel = [[np.arange(Ck, dtype=np.int64) for _ in range(Cq)] for _ in range(Q.shape[0])]
    got = run_sparse(Q, K, V, ql, kl, sel, dtype, Cq, Ck)
    for h in range(Q.shape[0]):
        check(got[h], orc.dense_attention(Q[h], K[h], V[h]), dtype)


def test_more_ranges_than_the_lds_table_holds():
    """A query cluster whose selection is > 256 separate row ranges walks its range table from HBM
    instead of the LDS copy; every other of 700 tiny key clusters gives 350 ranges."""
    H, N, d, Cq, Ck = 2, 2800, 64, 3, 700
    Q, K, V = wl.make_small(7, N, d, 10, dtype="bf16", H=H)
    rng = np.random.default_rng(8)
    ql = rng.integers(0, Cq, (H, N)).astype(np.int32)
    kl = (np.arange(N) % Ck).astype(np.int32)[None].repeat(H, 0)
    kl = np.ascontiguousarray(rng.permuted(kl, axis=1))
    sel = [[np.arange(i % 2, Ck, 2, dtype=np.int64) if i < 2 else np.arange(0, Ck, 7, dtype=np.int64)
            for i in range(Cq)] for _ in range(H)]
    got = run_sparse(Q, K, V, ql, kl, sel, B.BF16, Cq, Ck)
    for h in range(H):
        ref = orc.sparse_attention_gather(Q[h], K[h], V[h], ql[h], kl[h], sel[h])
        print("many ranges", h, check(got[h], ref, B.BF16))


@pytest.mark.parametrize("H", [8, 11])
def test_heads_dealt_to_xcds_whole_and_leftover_heads(H):
    """Small heads take the mapping that gives every XCD whole heads, eight at a time, and splits the
    H mod 8 leftover heads by tile: H = 8 has no leftover, H = 11 has both kinds."""
    N, d, Cq, Ck = 300, 64, 5, 23
    Q, K, V, ql, kl, sel = make_case(9, N, d, B.BF16, H=H)
    got = run_sparse(Q, K, V, ql, kl, sel, B.BF16, Cq, Ck)
    for h in range(H):
        ref = orc.sparse_attention_gather(Q[h], K[h], V[h], ql[h], kl[h], sel[h])
        check(got[h], ref, B.BF16)
    p = B.Params(H=H, N=N, d=d, dtype=B.BF16, q_clusters=1, k_m0=1, k_m_min=1, k_max_clusters=1)
    O = to_np(B.adacluster_dense_attn(p, to_dev(Q, B.BF16), to_dev(K, B.BF16), to_dev(V, B.BF16)))
    for h in range(H):
        check(O[h], orc.dense_attention(Q[h], K[h], V[h]), B.BF16)


@pytest.mark.parametrize("d", [64, 128])
def test_skewed_selection_cuts_the_long_key_list(d):
    """One query cluster selects every key cluster (a list of 94 key tiles) while the others select one
    small cluster each: the long list is cut into chunks handled by separate workgroups and merged."""
    H, N, Cq, Ck = 2, 6000, 6, 40
    Q, K, V = wl.make_small(12, N, d, 10, dtype="bf16", H=H)
    rng = np.random.default_rng(13)
    ql = rng.integers(0, Cq, (H, N)).astype(np.int32)
    kl = rng.integers(0, Ck, (H, N)).astype(np.int32)
    sel = [[np.arange(Ck, dtype=np.int64) if i == 2 else np.array([i], dtype=np.int64) for i in range(Cq)]
           for _ in range(H)]
    got = run_sparse(Q, K, V, ql, kl, sel, B.BF16, Cq, Ck)
    for h in range(H):
        ref = orc.sparse_attention_gather(Q[h], K[h], V[h], ql[h], kl[h], sel[h])
        print("skewed", d, h, check(got[h], ref, B.BF16))


def test_more_cut_lists_than_partial_slots():
    """Ten query clusters of three query tiles select every key; the rest select one small cluster.  The
    chunks wanted (10 x 3 x 5) exceed the partial slots of a head, so the last lists are cut into fewer
    chunks or stay whole; every row must still match."""
    H, N, d, Cq, Ck = 1, 36000, 64, 60, 300
    Q, K, V = wl.make_small(14, N, d, 16, dtype="bf16", H=H)
    rng = np.random.default_rng(15)
    sizes = np.array([380] * 10 + [644] * 50)
    assert sizes.sum() == N
    ql = np.repeat(np.arange(Cq), sizes).astype(np.int32)
    ql = ql[rng.permutation(N)][None, :]
    kl = rng.integers(0, Ck, (H, N)).astype(np.int32)
    sel = [[np.arange(Ck, dtype=np.int64) if i < 10 else np.array([i], dtype=np.int64) for i in range(Cq)]]
    got = run_sparse(Q, K, V, ql, kl, sel, B.BF16, Cq, Ck)
    ref = orc.sparse_attention_gather(Q[0], K[0], V[0], ql[0], kl[0], sel[0])
    print("slot shortage", check(got[0], ref, B.BF16))


def test_empty_selection_gives_zero_rows_and_custom_scale():
    Cq, Ck = 5, 23
    Q, K, V, ql, kl, sel = make_case(4, 600, 64, B.BF16)
    for h in range(Q.shape[0]):
        sel[h][2] = np.zeros(0, dtype=np.int64)
        sel[h][3] = np.array([3], dtype=np.int64)        # cluster 3 is empty by construction
    got = run_sparse(Q, K, V, ql, kl, sel, B.BF16, Cq, Ck)
    for h in range(Q.shape[0]):
        assert np.all(got[h][ql[h] == 2] == 0) and np.all(got[h][ql[h] == 3] == 0)
        ref = orc.sparse_attention_gather(Q[h], K[h], V[h], ql[h], kl[h], sel[h])
        check(got[h], ref, B.BF16)
    # explicit softmax scale
    H, N, d = Q.shape
    p = B.Params(H=H, N=N, d=d, dtype=B.BF16, q_clusters=1, k_m0=1, k_m_min=1, k_max_clusters=1, softmax_scale=0.05)
    O = to_np(B.adacluster_dense_attn(p, to_dev(Q, B.BF16), to_dev(K, B.BF16), to_dev(V, B.BF16)))
    check(O[0], orc.dense_attention(Q[0], K[0], V[0], 0.05), B.BF16)


def test_large_logits_do_not_overflow():
    H, N, d = 1, 300, 64
    rng = np.random.default_rng(5)
    Q = wl.round_bf16_f32((6 * rng.standard_normal((H, N, d))).astype(np.float32))
    K = wl.round_bf16_f32((6 * rng.standard_normal((H, N, d))).astype(np.float32))
    V = wl.round_bf16_f32(rng.standard_normal((H, N, d)).astype(np.float32))
    p = B.Params(H=H, N=N, d=d, dtype=B.BF16, q_clusters=1, k_m0=1, k_m_min=1, k_max_clusters=1)
    O = to_np(B.adacluster_dense_attn(p, to_dev(Q, B.BF16), to_dev(K, B.BF16), to_dev(V, B.BF16)))
    assert np.all(np.isfinite(O))
    check(O[0], orc.dense_attention(Q[0], K[0], V[0]), B.BF16)
