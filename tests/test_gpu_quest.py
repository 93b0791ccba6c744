"""GPU Quest scores (Eq. 1 with vector arithmetic, Eq. 2 / Algorithm 2 on the matrix cores) against the
fp64 oracle.  The inputs are bf16 (or fp32) values both sides read exactly; every product of two bf16
values is exact in fp32, so the only error is the fp32 accumulation over d terms: 1e-5 relative to the
sum of the absolute terms."""
import numpy as np
import pytest
import torch

from oracle import adacluster_oracle as orc
from paper_2604_18348_amd import binding as B
from paper_2604_18348_amd import workloads as wl

pytestmark = pytest.mark.gpu


def inputs(seed, H, Lq, Lk, d, bf16):
    rng = np.random.default_rng(seed)
    Q = rng.standard_normal((H, Lq, d)).astype(np.float32)
    C = rng.standard_normal((H, Lk, d)).astype(np.float32)
    spread = np.abs(rng.standard_normal((H, Lk, d))).astype(np.float32)
    lo, hi = C - spread, C + spread
    if bf16:
        Q, C, lo, hi = (wl.round_bf16_f32(a) for a in (Q, C, lo, hi))
    return Q, C, lo, hi


def dev(a, bf16):
    t = torch.from_numpy(a).cuda()
    return t.to(torch.bfloat16) if bf16 else t


@pytest.mark.parametrize("form,bf16", [(B.QUEST_ALU, True), (B.QUEST_MFMA, True), (B.QUEST_ALU, False)])
@pytest.mark.parametrize("Lq,Lk,d", [(65, 173, 64), (300, 70, 128), (1, 1, 64), (129, 257, 128)])
def test_box_scores_match_eq1(form, bf16, Lq, Lk, d):
    H = 2
    Q, _, lo, hi = inputs(3, H, Lq, Lk, d, bf16)
    S = B.adacluster_quest_scores(dev(Q, bf16), dev(hi, bf16), dev(lo, bf16), form).cpu().numpy()
    for h in range(H):
        ref = orc.score_box(Q[h].astype(np.float64), lo[h].astype(np.float64), hi[h].astype(np.float64))
        mag = np.abs(Q[h].astype(np.float64)) @ np.maximum(np.abs(lo[h]), np.abs(hi[h])).astype(np.float64).T
        assert np.all(np.abs(S[h] - ref) <= 1e-5 * mag + 1e-6), float(np.abs(S[h] - ref).max())


@pytest.mark.parametrize("form", [B.QUEST_ALU, B.QUEST_MFMA])
def test_clamped_centroids_are_algorithm_2(form):
    """One vector per page: R+ = max(c, 0), R- = min(c, 0), taken on the fly from the centroid tensor."""
    H, Lq, Lk, d = 3, 97, 200, 64
    Q, C, _, _ = inputs(5, H, Lq, Lk, d, True)
    Cd = dev(C, True)
    S = B.adacluster_quest_scores(dev(Q, True), Cd, Cd, form, clamp=True).cpu().numpy()
    for h in range(H):
        ref = orc.score_tensorquest(Q[h].astype(np.float64), C[h].astype(np.float64))
        mag = np.abs(Q[h].astype(np.float64)) @ np.abs(C[h]).astype(np.float64).T
        assert np.all(np.abs(S[h] - ref) <= 1e-5 * mag + 1e-6)


def test_the_two_forms_agree_and_bound_every_member():
    """Eq. 1 and Eq. 2 are the same number, and that number bounds q.k for every key inside the box."""
    H, Lq, Lk, d = 1, 64, 40, 128
    Q, C, lo, hi = inputs(7, H, Lq, Lk, d, True)
    a = B.adacluster_quest_scores(dev(Q, True), dev(hi, True), dev(lo, True), B.QUEST_ALU).cpu().numpy()
    b = B.adacluster_quest_scores(dev(Q, True), dev(hi, True), dev(lo, True), B.QUEST_MFMA).cpu().numpy()
    assert np.allclose(a, b, rtol=0, atol=2e-4)
    inner = (Q[0].astype(np.float64) @ C[0].astype(np.float64).T)       # the centre lies inside its box
    assert np.all(b[0] >= inner - 1e-4)
