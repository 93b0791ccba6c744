"""adacluster_compactness_noalloc (the entry point for callers that cannot allocate: its partial sums live in
an array inside the library's device image) against adacluster_compactness, which takes them from the
caller's workspace: the same kernels in the same order, so the results must be equal bit for bit, and within
1e-5 of the fp64 oracle.  Two calls in a row, the second on a smaller input, share the array."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import adacluster_oracle as orc
from paper_2604_18348_amd import binding as B
from paper_2604_18348_amd import workloads as wl
from tests.helpers import to_dev, to_np

pytestmark = pytest.mark.gpu


def _case(seed, H, N, d, dtype):
    name = "bf16" if dtype == B.BF16 else "f32"
    _, K, _ = wl.make_small(seed, N, d, 14, dtype=name, H=H)
    p = B.Params(H=H, N=N, d=d, dtype=dtype, q_clusters=8, k_iters=2, k_m0=20, k_m_min=4, k_max_clusters=80,
                 tau_factor=1.5, min_unassigned_frac=0.03)
    Kd = to_dev(K, dtype)
    out = B.adacluster_kcluster(p, Kd)
    torch.cuda.synchronize()
    return p, K, Kd, out


@pytest.mark.parametrize("dtype,d", [(B.BF16, 64), (B.BF16, 128), (B.F32, 64)])
def test_no_alloc_compactness_two_calls_in_a_row(dtype, d):
    big = _case(71, 3, 5300, d, dtype)        # six 1024-row blocks per head, the last one ragged
    small = _case(72, 2, 900, d, dtype)       # one block per head: most of the array keeps the first call's sums
    res = []
    for p, K, Kd, out in (big, small):
        want = B.adacluster_compactness(p, Kd, out["k_labels"], out["k_centroids"])
        got = torch.full((p.H,), -1.0, dtype=torch.float32, device="cuda")
        before = torch.cuda.memory_allocated()
        B.adacluster_compactness_noalloc(p, Kd, out["k_labels"], out["k_centroids"], out=got)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        res.append((p, K, out, want.cpu().numpy(), got.cpu().numpy()))
    for p, K, out, want, got in res:
        assert np.array_equal(want, got), (want, got)
        lab, cen = out["k_labels"].cpu().numpy(), to_np(out["k_centroids"])
        ref = np.array([orc.compactness_mse(K[h], lab[h], cen[h]) for h in range(p.H)])
        assert np.allclose(got, ref, rtol=1e-5, atol=1e-7), (got, ref)


def test_no_alloc_compactness_rejects_sizes_beyond_its_array():
    lib = B.load_library()
    p = B.Params(H=4096, N=20000, d=64, dtype=B.BF16, q_clusters=8, k_m0=20, k_m_min=4, k_max_clusters=80)
    one = torch.zeros(64, dtype=torch.float32, device="cuda")        # never touched: the call must fail first
    cp = p.c()
    rc = lib.adacluster_compactness_noalloc(ctypes.byref(cp), one.data_ptr(), one.data_ptr(), one.data_ptr(),
                                            one.data_ptr(), None)
    assert rc == -5
    buf = ctypes.create_string_buffer(256)
    lib.adacluster_last_error(buf, 256)
    assert b"exceeds" in buf.value
    rc = lib.adacluster_compactness_noalloc(ctypes.byref(cp), None, one.data_ptr(), one.data_ptr(), one.data_ptr(), None)
    assert rc == -1
