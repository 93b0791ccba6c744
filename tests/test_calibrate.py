"""N_max from a calibration run (Sec. 4.1: the cap is set so that a given share of the units falls back to
full attention).  The prediction of the flag from one uncapped run of Algorithm 1 is exact: checked here
against the oracle run again with the chosen cap."""
import numpy as np
import pytest

from oracle import adacluster_oracle as orc
from paper_2604_18348_amd import calibrate as cal
from paper_2604_18348_amd import workloads as wl

KW = dict(m0=12, m_min=3, n_iters=3, max_stages=6)


def units(seed, n_units=6, N=600, d=16):
    """Units of growing diffuseness: the same mixture with more and more isotropic noise."""
    rng = np.random.default_rng(seed)
    mu = 4.0 * rng.standard_normal((8, d))
    comp = rng.integers(0, 8, N)
    return [mu[comp] + (0.2 + 0.35 * u) * rng.standard_normal((N, d)) for u in range(n_units)]


def exported_offs(ref, width=11):
    offs = np.full(width, ref["assign_centroids"].shape[0], dtype=np.int64)
    offs[:len(ref["stage_offs"])] = ref["stage_offs"]
    return offs


@pytest.mark.parametrize("frac_left", [0.0, 0.05])
@pytest.mark.parametrize("dense_fraction", [1 / 3, 0.5, 0.0])
def test_flag_prediction_is_exact_against_the_oracle(dense_fraction, frac_left):
    Ks = units(3)
    tau = 3.2
    free = [orc.multistage_kmeans(K, tau, 10 ** 6, min_unassigned_frac=frac_left, **KW) for K in Ks]
    assert not any(r["full_flag"] for r in free)
    theta = cal.flag_thresholds(np.stack([exported_offs(r) for r in free]),
                                [r["assign_centroids"].shape[0] for r in free],
                                [r["n_unassigned"][-1] > 0 for r in free])
    assert len(set(theta.tolist())) > 2                  # the units really differ
    n_max, predicted = cal.choose_n_max(theta, dense_fraction, n_min=KW["m0"])
    want = int(round(dense_fraction * len(Ks)))
    assert predicted.sum() >= min(want, int((theta >= KW["m0"]).sum()))
    if want == 0:
        assert predicted.sum() == 0
    capped = [orc.multistage_kmeans(K, tau, n_max, min_unassigned_frac=frac_left, **KW) for K in Ks]
    assert [bool(r["full_flag"]) for r in capped] == predicted.tolist()
    for r0, r1, f in zip(free, capped, predicted):
        if not f:                                        # an unflagged unit is untouched by the cap
            assert np.array_equal(r0["labels"], r1["labels"])
    # one below the threshold of a unit flags it, one above does not
    for u in range(len(Ks)):
        if theta[u] >= 1:
            assert orc.multistage_kmeans(Ks[u], tau, int(theta[u]), min_unassigned_frac=frac_left, **KW)["full_flag"]
        assert not orc.multistage_kmeans(Ks[u], tau, int(theta[u]) + 1, min_unassigned_frac=frac_left, **KW)["full_flag"]


def test_choose_n_max_on_plain_numbers():
    theta = np.array([0, 40, 10, 90, 25, 60, 0, 33, 12, 70])
    n_max, flags = cal.choose_n_max(theta, 0.2)           # the two largest: 90, 70
    assert n_max == 70 and flags.tolist() == [False, False, False, True, False, False, False, False, False, True]
    n_max, flags = cal.choose_n_max(theta, 0.0)
    assert n_max == 91 and not flags.any()
    n_max, flags = cal.choose_n_max(theta, 1.0, n_min=20)  # units below the smallest usable cap stay clustered
    assert n_max == 20 and flags.sum() == 6
    n_max, flags = cal.choose_n_max(np.array([5, 5, 5, 1]), 0.25)   # ties flag together
    assert n_max == 5 and flags.sum() == 3


@pytest.mark.gpu
@pytest.mark.parametrize("d", [64, 128])
def test_flag_prediction_is_exact_on_the_device(d):
    import dataclasses
    import torch
    from paper_2604_18348_amd import binding as B
    from tests.helpers import to_dev
    H, N = 6, 3000
    _, K, _ = wl.make_small(61, N, d, 12, dtype="bf16", H=H)
    rng = np.random.default_rng(62)
    for h in range(H):                                   # more and more isotropic noise
        K[h] = wl.round_bf16_f32(K[h] + (0.25 * h) * rng.standard_normal((N, d)).astype(np.float32))
    base = B.Params(H=H, N=N, d=d, dtype=B.BF16, q_clusters=4, k_iters=3, k_m0=16, k_m_min=4, k_max_clusters=200,
                    k_max_stages=6, tau_factor=1.2, min_unassigned_frac=0.02)
    Kd = to_dev(K, B.BF16)
    free = B.adacluster_kcluster(base, Kd, want_box=False)
    torch.cuda.synchronize()
    assert int(free["full_flag"].sum()) == 0
    left = (free["k_stage_of"] == -1).any(dim=1).cpu().numpy()
    theta = cal.flag_thresholds(free["k_stage_offs"].cpu().numpy(), free["k_count"].cpu().numpy(), left)
    print("theta", theta, "k_count", free["k_count"].cpu().numpy(), "left over", left)
    assert len(set(theta.tolist())) > 2
    n_max, predicted = cal.choose_n_max(theta, 1 / 3, n_min=base.k_m0)
    capped = B.adacluster_kcluster(dataclasses.replace(base, k_max_clusters=n_max), Kd, want_box=False)
    torch.cuda.synchronize()
    assert capped["full_flag"].cpu().numpy().astype(bool).tolist() == predicted.tolist()
    assert predicted.sum() >= 2
    keep = ~predicted
    assert torch.equal(capped["k_labels"][torch.from_numpy(keep).cuda()], free["k_labels"][torch.from_numpy(keep).cuda()])
