"""Every entry point writes only inside the buffers it is given: the workspace and every output tensor sit
between guard bytes that the host checks after the call (ragged sizes, both dtypes, both head dims)."""
import numpy as np
import pytest
import torch

from paper_2604_18348_amd import binding as B
from paper_2604_18348_amd import workloads as wl
from tests.helpers import to_dev

pytestmark = pytest.mark.gpu

GUARD = 1024          # bytes on either side; a multiple of the 256-byte alignment the library asks for
FILL = 0xA5


class Guards:
    """Hands out device tensors that are the middle of a larger byte buffer whose ends hold FILL."""

    def __init__(self):
        self.bufs = []

    def tensor(self, shape, dtype, zero=False, name=""):
        shape = tuple(shape) if not isinstance(shape, int) else (shape,)
        nbytes = int(np.prod(shape, dtype=np.int64)) * torch.empty((), dtype=dtype).element_size()
        pad = (-nbytes) % 256
        buf = torch.full((GUARD + nbytes + pad + GUARD,), FILL, dtype=torch.uint8, device="cuda")
        assert buf.data_ptr() % 256 == 0
        mid = buf[GUARD:GUARD + nbytes]
        if zero:
            mid.zero_()
        self.bufs.append((name or str(shape), buf, nbytes))
        return mid.view(dtype).view(shape)

    def check(self):
        torch.cuda.synchronize()
        for name, buf, nbytes in self.bufs:
            front, back = buf[:GUARD], buf[GUARD + nbytes:]
            assert bool((front == FILL).all()), "bytes before %s were written" % name
            assert bool((back == FILL).all()), "bytes after %s were written" % name
        n = len(self.bufs)
        self.bufs = []
        return n


class TorchProxy:
    """torch, except that new tensors come from a Guards object (the binding allocates its outputs itself)."""

    def __init__(self, guards):
        self._g = guards

    def __getattr__(self, name):
        return getattr(torch, name)

    def empty(self, *shape, dtype=torch.float32, device=None, **kw):
        shape = shape[0] if len(shape) == 1 and not isinstance(shape[0], int) else shape
        return self._g.tensor(shape, dtype)

    def zeros(self, *shape, dtype=torch.float32, device=None, **kw):
        shape = shape[0] if len(shape) == 1 and not isinstance(shape[0], int) else shape
        return self._g.tensor(shape, dtype, zero=True)

    def empty_like(self, t, **kw):
        return self._g.tensor(t.shape, t.dtype)


@pytest.fixture
def guarded(monkeypatch):
    g = Guards()
    monkeypatch.setattr(B, "torch", TorchProxy(g))
    return g


def guarded_ws(g, p):
    return g.tensor((B.adacluster_workspace_bytes(p),), torch.uint8, name="workspace")


CASES = [(B.BF16, 64, 1237, 7, 3), (B.BF16, 128, 2051, 65, 2), (B.F32, 64, 701, 5, 2), (B.F32, 128, 333, 3, 1),
         (B.BF16, 64, 67, 65, 1), (B.BF16, 128, 16500, 9, 1)]


@pytest.mark.parametrize("dtype,d,N,Cq,H", CASES)
def test_guard_bytes_around_every_buffer(guarded, dtype, d, N, Cq, H):
    g = guarded
    name = "bf16" if dtype == B.BF16 else "f32"
    Q, K, V = wl.make_small(71, N, d, 10, dtype=name, H=H)
    Qd, Kd, Vd = to_dev(Q, dtype), to_dev(K, dtype), to_dev(V, dtype)
    p = B.Params(H=H, N=N, d=d, dtype=dtype, q_clusters=Cq, q_iters=3, k_iters=3, k_m0=24, k_m_min=4,
                 k_max_clusters=96, tau_factor=1.5, min_unassigned_frac=0.03, topk=6)
    checked = 0
    # the parts, each with its own workspace between guards
    qc = B.adacluster_qcluster(p, Qd, ws=guarded_ws(g, p))
    checked += g.check()
    kc = B.adacluster_kcluster(p, Kd, want_box=True, ws=guarded_ws(g, p))
    checked += g.check()
    sel_idx, sel_cnt = B.adacluster_select(p, qc["q_centroids"], qc["q_mean_norm"], kc["k_centroids"], kc["k_box_min"],
                                           kc["k_box_max"], kc["k_sizes"], kc["k_count"], kc["full_flag"],
                                           ws=guarded_ws(g, p))
    checked += g.check()
    O1 = B.adacluster_sparse_attn(p, Qd, Kd, Vd, qc["q_labels"], kc["k_labels"], kc["k_count"], sel_idx, sel_cnt,
                                  ws=guarded_ws(g, p))
    checked += g.check()
    B.adacluster_compactness(p, Kd, kc["k_labels"], kc["k_centroids"], ws=guarded_ws(g, p))
    checked += g.check()
    B.adacluster_compactness_noalloc(p, Kd, kc["k_labels"], kc["k_centroids"])
    checked += g.check()
    # warm start (previous centres and counts as the start)
    pw = B.Params(**{**p.__dict__, "k_init_mode": 1, "k_iters": 2, "q_init_mode": 1, "q_iters": 2})
    B.adacluster_kcluster(pw, Kd, want_box=False, ws=guarded_ws(g, pw), prev=kc)
    checked += g.check()
    B.adacluster_qcluster(pw, Qd, q_centroids_init=qc["q_centroids"], ws=guarded_ws(g, pw))
    checked += g.check()
    # the fused call with every intermediate exported, without, and the dense call
    ws = guarded_ws(g, p)
    outs = B.alloc_outputs(p, "cuda", want_box=True, want_stage=True)
    O2 = B.adacluster_attn(p, Qd, Kd, Vd, outs=outs, ws=ws)
    stats = B.adacluster_stats_fetch(p, ws)
    assert len(stats) == H
    checked += g.check()
    B.adacluster_attn(p, Qd, Kd, Vd, outs=None, ws=guarded_ws(g, p))
    checked += g.check()
    for mode in (1, 2):                                            # top-p; box scores
        pm = B.Params(**{**p.__dict__, "select_mode": 1, "top_p": 0.8} if mode == 1 else {**p.__dict__, "score_mode": 1})
        B.adacluster_attn(pm, Qd, Kd, Vd, outs=B.alloc_outputs(pm, "cuda", want_box=True), ws=guarded_ws(g, pm))
        checked += g.check()
    B.adacluster_dense_attn(p, Qd, Kd, Vd, ws=guarded_ws(g, p))
    checked += g.check()
    assert torch.equal(O1, O2)                                     # the parts and the fused call agree bit for bit
    print("guarded buffers checked:", checked)
    assert checked > 40


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_guard_bytes_quest_scores_and_probe(guarded, dtype):
    g = guarded
    gen = torch.Generator(device="cuda").manual_seed(3)
    H, Lq, Lk, d = 2, 77, 45, 64
    Q = torch.randn((H, Lq, d), device="cuda", generator=gen).to(dtype)
    A = torch.randn((H, Lk, d), device="cuda", generator=gen).to(dtype)
    Bm = torch.randn((H, Lk, d), device="cuda", generator=gen).to(dtype)
    Rp, Rn = torch.maximum(A, Bm).contiguous(), torch.minimum(A, Bm).contiguous()
    for form in (B.QUEST_ALU, B.QUEST_MFMA):
        if form == B.QUEST_MFMA and dtype != torch.bfloat16:
            continue                                   # the matrix-core form takes bf16 inputs
        B.adacluster_quest_scores(Q, Rp, Rn, form, clamp=(form == B.QUEST_MFMA))
        assert g.check() == 1
    sink = g.tensor((1024,), torch.float32, name="probe sink")
    B.adacluster_mfma_probe(10, sink)
    assert g.check() == 1
